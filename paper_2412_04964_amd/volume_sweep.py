"""Latency of the quantized all-reduce arithmetic against the communication volume (the x-axis of the paper's
latency-versus-volume comparison, Section 5.3, and of its SM-count study), on one MI355X.

    python -m paper_2412_04964_amd.volume_sweep [--n-src 4] [--hidden 8192] [--group 128]

For every volume (tokens x hidden binary16 elements per partial, doubling from a few rows to 2^27 elements) and the
three settings the paper plots (INT8, INT6 = 4-bit reduce / 8-bit gather, INT4) it prints the time of the three
kernels called one by one (N quantizations, the fused dequantize-sum-requantize, the final dequantization) and of
fc_allreduce_sim, which runs them as a single launch.  The paper's curves include the exchanges between its GPUs; this
is the arithmetic alone, so the figure to read off is where launching stops and memory bandwidth starts to bound it.
(bench.py, with its long warm-up and five buffer sets, is the reference for absolute figures at the named workloads.)

Every stage is captured into a HIP graph over enough independent buffer sets that a large volume is read from HBM and
not from the 256 MB memory-side cache, and the graph is replayed; times are per all-reduce.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

PRECISIONS = {"INT8": (8, 8), "INT6": (4, 8), "INT4": (4, 4)}


def time_graph(torch, fn, sets, reps):
    """fn(k) enqueues one call on buffer set k; returns seconds per call under graph replay."""
    for k in range(sets):
        fn(k)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=torch.cuda.Stream()):
        for k in range(sets):
            fn(k)
    t_end = time.time() + 0.15                       # let the clocks settle on this load before timing
    while time.time() < t_end:
        g.replay()
        torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e-3 / (reps * sets)


def sweep(n_src: int, hidden: int, group: int, max_elems: int, seed: int = 0):
    import torch

    from . import binding as fc

    rows = []
    tokens = max(1, 65536 // hidden)
    while tokens * hidden <= max_elems:
        m = tokens * hidden
        per_set = (n_src + 1) * 2 * m
        sets = int(min(32, max(2, -(-(3 << 29) // per_set))))          # >= 1.5 GiB touched per round, 2..32 sets
        reps = int(max(3, min(200, (1 << 31) // (per_set * sets))))
        gen = torch.Generator(device="cuda")
        gen.manual_seed(seed)
        X = [torch.randn((n_src, tokens, hidden), generator=gen, device="cuda", dtype=torch.float16)
             for _ in range(sets)]
        Y = [torch.empty((tokens, hidden), device="cuda", dtype=torch.float16) for _ in range(sets)]
        for label, (b_rs, b_ag) in PRECISIONS.items():
            ws = torch.empty(max(16, fc.allreduce_sim_workspace_bytes(n_src, tokens, hidden, group, b_rs, b_ag)),
                             dtype=torch.uint8, device="cuda")
            C1 = [fc.quantize(X[k].view(n_src * tokens, hidden), group, b_rs) for k in range(sets)]
            F = [fc.dequant_reduce_requant(C1[k][0].view(n_src, tokens, -1), C1[k][1].view(n_src, tokens, -1),
                                           C1[k][2].view(n_src, tokens, -1), hidden, group, b_rs, b_ag)
                 for k in range(sets)]
            t_q = time_graph(torch, lambda k: fc.quantize(X[k].view(n_src * tokens, hidden), group, b_rs, out=C1[k]),
                             sets, reps)
            t_f = time_graph(torch, lambda k: fc.dequant_reduce_requant(
                C1[k][0].view(n_src, tokens, -1), C1[k][1].view(n_src, tokens, -1), C1[k][2].view(n_src, tokens, -1),
                hidden, group, b_rs, b_ag, out=F[k]), sets, reps)
            t_d = time_graph(torch, lambda k: fc.dequantize(*F[k], hidden, group, b_ag, out=Y[k]), sets, reps)
            t_one = time_graph(torch, lambda k: fc.allreduce_sim(X[k], group, b_rs, b_ag, out=Y[k], workspace=ws),
                               sets, reps)
            rows.append({"precision": label, "tokens": tokens, "elems_per_partial": m,
                         "fp16_MB_per_partial": round(2 * m / 1e6, 3),
                         "quantize_all_us": round(t_q * 1e6, 2), "fused_us": round(t_f * 1e6, 2),
                         "dequantize_us": round(t_d * 1e6, 2),
                         "three_kernels_us": round((t_q + t_f + t_d) * 1e6, 2),
                         "one_launch_us": round(t_one * 1e6, 2),
                         "one_launch_GBps": round(per_set / t_one / 1e9, 1)})
            del ws, C1, F
        del X, Y
        torch.cuda.empty_cache()
        tokens *= 2
    return rows


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--n-src", type=int, default=4)
    ap.add_argument("--hidden", type=int, default=8192)
    ap.add_argument("--group", type=int, default=128)
    ap.add_argument("--max-elems", type=int, default=1 << 27, help="largest volume: elements per partial")
    ap.add_argument("--json", action="store_true", help="print one JSON list instead of the table")
    a = ap.parse_args()
    import torch

    if not torch.cuda.is_available():
        sys.exit("volume_sweep needs a GPU: the HIP path has no CPU fallback")
    rows = sweep(a.n_src, a.hidden, a.group, a.max_elems)
    if a.json:
        print(json.dumps(rows))
        return
    print("N = %d partials, hidden %d, group %d; microseconds per all-reduce" % (a.n_src, a.hidden, a.group))
    print("%-5s %8s %12s %10s %8s %8s %10s %10s %9s" % ("prec", "tokens", "MB/partial", "quant xN", "fused", "dequant",
                                                       "3 kernels", "1 launch", "GB/s"))
    for r in rows:
        print("%-5s %8d %12.3f %10.2f %8.2f %8.2f %10.2f %10.2f %9.1f" % (
            r["precision"], r["tokens"], r["fp16_MB_per_partial"], r["quantize_all_us"], r["fused_us"],
            r["dequantize_us"], r["three_kernels_us"], r["one_launch_us"], r["one_launch_GBps"]))


if __name__ == "__main__":
    main()
