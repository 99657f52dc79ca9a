#!/usr/bin/env python3
"""Benchmark of the Flash Communication quantization path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

A step is one pass of the whole hot path over one batch of `--batch` independent
all-reduce volumes, stage by stage: N x fc_quantize for every volume of the
batch, then fc_dequant_reduce_requant for every volume, then fc_dequantize for
every volume.  Running a batch stage-major means that no kernel reads data its
producer has just left in the 256 MB memory-side cache (several gigabytes of
other traffic lie in between), so every timed byte comes from HBM, and the
launches of one kernel are back to back, so an event pair around a stage
measures sustained launch-to-launch time.  `--dependent` runs the stages of one
volume back to back instead (cache-warm hand-over, reported for comparison).

Prints ONE JSON line.  `value` is the headline metric of this build: achieved
GB/s of the fused dequant-reduce-requant kernel (algorithmic bytes per launch /
mean launch duration, HIP events on the launch stream inside the timed region).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import synth_inputs  # noqa: E402

HBM_PEAK_GBPS = 8000.0       # MI355X published HBM3E bandwidth
SETTLE_STEPS = 100           # untimed steps (warm-up included) every run does before the timed region


def fused_bytes(w) -> int:
    """Algorithmic bytes of one fused launch: N x (codes + meta) in, codes + meta out; meta is an
    fp32 scale and zero-point per group (8 bytes), the scale alone (4) for the symmetric quantizers, or
    a binary16 scale and zero-point in one word (4) for the compact-metadata variant."""
    m = w.elements
    mb = w.meta_bytes_per_group
    return w.n_src * (m * w.bits_in // 8 + mb * m // w.group) + m * w.bits_out // 8 + mb * m // w.group


def quantize_bytes(w) -> int:
    m = w.elements
    return 2 * m + m * w.bits_in // 8 + w.meta_bytes_per_group * m // w.group


def dequantize_bytes(w) -> int:
    m = w.elements
    return m * w.bits_out // 8 + w.meta_bytes_per_group * m // w.group + 2 * m


def load_profile_constant(name, key):
    """A per-launch figure of the fused kernel from the committed, calibrated rocprofv3 counter summary under
    profiles/ (hardware counters cannot be read from inside this process): `fused_hbm_bytes_per_launch` from
    --pmc FETCH_SIZE / WRITE_SIZE, `fused_valu_wave_instructions_per_launch` from --pmc SQ_INSTS_VALU.  None
    when no measurement exists.  These are stored constants, not measurements of the run that prints them."""
    p = os.path.join(ROOT, "profiles", "traffic_%s.txt" % name)
    if not os.path.exists(p):
        return None
    for line in open(p):
        if line.startswith(key):
            try:
                return int(line.split("=")[1])
            except ValueError:
                return None
    return None


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


# VALU issue peak of the part: 256 compute units x 4 SIMDs, one wave64 instruction per SIMD every 4 cycles at 2.4 GHz
VALU_PEAK_WAVE_INSTR_PER_S = 256 * 4 * 2.4e9 / 4


def cpu_baseline(w, x_host, budget_s=20.0):
    """The oracle's fused step on the host, single thread, full volume if it fits
    the time budget (else the leading rows)."""
    import oracle
    rows = w.tokens
    est = 16e-9 * w.elements * (1 + w.n_src / 4.0) * 1.5
    if est * 3 > budget_s:
        rows = max(16, int(w.tokens * budget_s / (est * 3)))
    xs = x_host[:, :rows]
    sym, fp8, cm = w.quantizer == "sym", w.quantizer == "fp8", w.quantizer == "cmeta"
    t_q = time.perf_counter()
    if fp8:
        parts = [oracle.quantize_fp8(xs[j], w.group) for j in range(w.n_src)]
    elif cm:
        parts = [oracle.quantize_cmeta(xs[j], w.group, w.bits_in) for j in range(w.n_src)]
    else:
        parts = [(oracle.quantize_sym if sym else oracle.quantize)(xs[j], w.group, w.bits_in)
                 for j in range(w.n_src)]
    t_q = time.perf_counter() - t_q                       # the first stage: n_src quantizations, timed once
    c = np.stack([p[0] for p in parts]); s = np.stack([p[1] for p in parts])
    z = None if (sym or fp8 or cm) else np.stack([p[2] for p in parts])
    best = None
    for _ in range(2):
        t0 = time.perf_counter()
        if fp8:
            fused = oracle.dequant_reduce_requant_fp8(c, s, w.hidden, w.group)
        elif sym:
            fused = oracle.dequant_reduce_requant_sym(c, s, w.hidden, w.group, w.bits_in, w.bits_out)
        elif cm:
            fused = oracle.dequant_reduce_requant_cmeta(c, s, w.hidden, w.group, w.bits_in, w.bits_out)
        else:
            fused = oracle.dequant_reduce_requant(c, s, z, w.hidden, w.group, w.bits_in, w.bits_out)
        dt = time.perf_counter() - t0
        best = dt if best is None else min(best, dt)
    t_d = time.perf_counter()                             # the last stage, timed once
    if fp8:
        oracle.dequantize_fp8(*fused, w.hidden, w.group)
    elif sym:
        oracle.dequantize_sym(*fused, w.hidden, w.group, w.bits_out)
    elif cm:
        oracle.dequantize_cmeta(*fused, w.hidden, w.group, w.bits_out)
    else:
        oracle.dequantize(*fused, w.hidden, w.group, w.bits_out)
    t_d = time.perf_counter() - t_d
    frac = rows / w.tokens
    return {
        "value": round(fused_bytes(w) * frac / best / 1e9, 4),
        "unit": "GB/s",
        "cores": 1,
        "cpu_model": cpu_model(),
        "kind": "oracle",
        "sample": "fused step of the plain-C oracle on rows [0,%d) of %d of volume 0, best of 2, "
                  "%.2f s per run" % (rows, w.tokens, best),
        "host_cpus": os.cpu_count(),
        "other_stages_GBps": {"quantize_xN": round(w.n_src * quantize_bytes(w) * frac / t_q / 1e9, 4),
                              "dequantize": round(dequantize_bytes(w) * frac / t_d / 1e9, 4)},
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # the part takes a few hundred launches after an idle period to settle its clocks, hence the long warm-up
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--workload", default="llama3_70b_prefill", choices=sorted(synth_inputs.WORKLOADS))
    ap.add_argument("--batch", type=int, default=0,
                    help="independent volumes per step (0 = enough for >= 4 GiB of traffic per step)")
    ap.add_argument("--dependent", action="store_true", help="run the stages of one volume back to back")
    ap.add_argument("--graph", choices=["auto", "on", "off"], default="auto",
                    help="replay each stage's launches from a captured HIP graph (auto: for volumes so "
                         "small that launching, not HBM, bounds them)")
    ap.add_argument("--group", type=int, default=0,
                    help="override the workload's group size (granularity sweep; 0 = as defined)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    a = ap.parse_args()

    if a.gpus != 1:
        sys.exit("bench.py: this build measures one GPU's share of the path only; "
                 "--gpus %d is not supported (run with --gpus 1)" % a.gpus)

    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    import paper_2412_04964_amd as fc
    fc.lib()

    w = synth_inputs.WORKLOADS[a.workload]
    if a.group:
        import dataclasses
        w = dataclasses.replace(w, name="%s_g%d" % (w.name, a.group), group=a.group)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    T, H, N, g = w.tokens, w.hidden, w.n_src, w.group
    vol_bytes = N * quantize_bytes(w) + fused_bytes(w) + dequantize_bytes(w)
    B = a.batch or max(4, min(256, -(-(4 << 30) // vol_bytes)))

    # volumes and per-volume intermediates, all resident in HBM before timing
    X = [synth_inputs.make_partials_device(N, T, H, w.seed + k, dev, w.outlier_frac, w.outlier_gain)
         for k in range(B)]
    C1 = [torch.empty((N, T, H * w.bits_in // 8), dtype=torch.uint8, device=dev) for _ in range(B)]
    S1 = [torch.empty((N, T, H // g), dtype=torch.float32, device=dev) for _ in range(B)]
    Z1 = [torch.empty_like(S1[0]) for _ in range(B)]
    C2 = [torch.empty((T, H * w.bits_out // 8), dtype=torch.uint8, device=dev) for _ in range(B)]
    S2 = [torch.empty((T, H // g), dtype=torch.float32, device=dev) for _ in range(B)]
    Z2 = [torch.empty_like(S2[0]) for _ in range(B)]
    Y = [torch.empty((T, H), dtype=torch.float16, device=dev) for _ in range(B)]

    sym, fp8, cm = w.quantizer == "sym", w.quantizer == "fp8", w.quantizer == "cmeta"
    qz = {"asym": fc.QUANTIZER_ASYM, "sym": fc.QUANTIZER_SYM, "fp8": fc.QUANTIZER_FP8}.get(w.quantizer)
    assert not (w.rotate and qz is None), "the rotation entry points take the fp32-metadata quantizers only"
    M1 = [t.view(torch.int32) for t in S1]          # the compact-metadata words live in the scale buffers
    M2 = [t.view(torch.int32) for t in S2]

    def stage_quantize(k):
        for j in range(N):
            if w.rotate:
                fc.quantize_rot(X[k][j], g, w.bits_in, qz, out=(C1[k][j], S1[k][j], Z1[k][j]))
            elif fp8:
                fc.quantize_fp8(X[k][j], g, out=(C1[k][j], S1[k][j]))
            elif sym:
                fc.quantize_sym(X[k][j], g, w.bits_in, out=(C1[k][j], S1[k][j]))
            elif cm:
                fc.quantize_cmeta(X[k][j], g, w.bits_in, out=(C1[k][j], M1[k][j]))
            else:
                fc.quantize(X[k][j], g, w.bits_in, out=(C1[k][j], S1[k][j], Z1[k][j]))

    def stage_fused(k):
        if fp8:
            fc.dequant_reduce_requant_fp8(C1[k], S1[k], H, g, out=(C2[k], S2[k]))
        elif sym:
            fc.dequant_reduce_requant_sym(C1[k], S1[k], H, g, w.bits_in, w.bits_out, out=(C2[k], S2[k]))
        elif cm:
            fc.dequant_reduce_requant_cmeta(C1[k], M1[k], H, g, w.bits_in, w.bits_out, out=(C2[k], M2[k]))
        else:
            fc.dequant_reduce_requant(C1[k], S1[k], Z1[k], H, g, w.bits_in, w.bits_out,
                                      out=(C2[k], S2[k], Z2[k]))

    def stage_dequantize(k):
        if w.rotate:
            fc.dequantize_rot(C2[k], S2[k], Z2[k], H, g, w.bits_out, qz, out=Y[k])
        elif fp8:
            fc.dequantize_fp8(C2[k], S2[k], H, g, out=Y[k])
        elif sym:
            fc.dequantize_sym(C2[k], S2[k], H, g, w.bits_out, out=Y[k])
        elif cm:
            fc.dequantize_cmeta(C2[k], M2[k], H, g, w.bits_out, out=Y[k])
        else:
            fc.dequantize(C2[k], S2[k], Z2[k], H, g, w.bits_out, out=Y[k])

    ev = {name: [] for name in ("q", "f", "d")}

    # Launch-bound volumes (decode: 0.6 MB per fused launch): the stage's B launches are captured once
    # into a HIP graph and replayed, so the figure is the GPU's launch-to-launch time and not the
    # interpreter's.  The library's entry points only enqueue kernels, so they capture as they are.
    use_graph = a.graph == "on" or (a.graph == "auto" and fused_bytes(w) < (8 << 20))
    graphs = {}
    if use_graph and not a.dependent:
        for _ in range(2):                               # load every kernel before capturing
            for k in range(B):
                stage_quantize(k); stage_fused(k); stage_dequantize(k)
        torch.cuda.synchronize()
        cap = torch.cuda.Stream()
        for name, fn in (("q", stage_quantize), ("f", stage_fused), ("d", stage_dequantize)):
            gr = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gr, stream=cap):
                for k in range(B):
                    fn(k)
            graphs[name] = gr

    def step(timed):
        if graphs:
            m = [torch.cuda.Event(enable_timing=True) for _ in range(4)] if timed else None
            for i, name in enumerate(("q", "f", "d")):
                if timed: m[i].record()
                graphs[name].replay()
            if timed:
                m[3].record()
                ev["q"].append((m[0], m[1], B)); ev["f"].append((m[1], m[2], B)); ev["d"].append((m[2], m[3], B))
            return
        if a.dependent:
            for k in range(B):
                m = [torch.cuda.Event(enable_timing=True) for _ in range(4)] if timed else None
                if timed: m[0].record()
                stage_quantize(k)
                if timed: m[1].record()
                stage_fused(k)
                if timed: m[2].record()
                stage_dequantize(k)
                if timed:
                    m[3].record()
                    ev["q"].append((m[0], m[1], 1)); ev["f"].append((m[1], m[2], 1))
                    ev["d"].append((m[2], m[3], 1))
            return
        m = [torch.cuda.Event(enable_timing=True) for _ in range(4)] if timed else None
        if timed: m[0].record()
        for k in range(B):
            stage_quantize(k)
        if timed: m[1].record()
        for k in range(B):
            stage_fused(k)
        if timed: m[2].record()
        for k in range(B):
            stage_dequantize(k)
        if timed:
            m[3].record()
            ev["q"].append((m[0], m[1], B)); ev["f"].append((m[1], m[2], B)); ev["d"].append((m[2], m[3], B))

    # After an idle period the part needs a few hundred launches (about 0.1 s of this work) before its clocks
    # settle; a run asked for with a short warm-up gets that much untimed work first, so that `--warmup`
    # only has to cover the usual first-launch effects.  Reported as config.settle_steps.
    settle_steps = max(0, SETTLE_STEPS - a.warmup)
    for _ in range(settle_steps):
        step(False)
    for _ in range(max(1, a.warmup)):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(a.steps):
        step(True)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    # the same access pattern without arithmetic (N code slabs in, one slab out), timed the same way
    slab = T * H * w.bits_in // 8
    R = [torch.empty(slab, dtype=torch.uint8, device=dev) for _ in range(B)]
    src = [C1[k].view(N, slab) for k in range(B)]
    for _ in range(3):
        for k in range(B):
            fc.stream_reference(src[k], R[k])
    sr0, sr1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    sr_reps = max(1, min(a.steps, 100))
    torch.cuda.synchronize()
    sr0.record()
    for _ in range(sr_reps):
        for k in range(B):
            fc.stream_reference(src[k], R[k])
    sr1.record()
    torch.cuda.synchronize()
    sr_s = sr0.elapsed_time(sr1) * 1e-3 / (sr_reps * B)
    sr_bytes = (N + 1) * slab

    # the opposite cut: the fused kernel's whole instruction stream with its traffic confined to the L2
    # (fc_fused_compute_probe of the bench library; instantiated for the three asymmetric benchmark configurations)
    probe_s = None
    if (w.quantizer == "asym" and not w.rotate and
            (N, w.bits_in, w.bits_out, g) in ((4, 4, 4, 128), (4, 8, 8, 128), (8, 4, 4, 64)) and T * H >= 64 * 128 * 32):
        PC = torch.empty_like(C2[0]); PS = torch.empty_like(S2[0]); PZ = torch.empty_like(Z2[0])
        for _ in range(20):
            fc.fused_compute_probe(C1[0], S1[0], Z1[0], H, g, w.bits_in, w.bits_out, out=(PC, PS, PZ))
        p0, p1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        p_reps = max(10, min(a.steps * B, 500))
        torch.cuda.synchronize()
        p0.record()
        for _ in range(p_reps):
            fc.fused_compute_probe(C1[0], S1[0], Z1[0], H, g, w.bits_in, w.bits_out, out=(PC, PS, PZ))
        p1.record()
        torch.cuda.synchronize()
        probe_s = p0.elapsed_time(p1) * 1e-3 / p_reps
        del PC, PS, PZ

    # The whole all-reduce as the library runs it (fc_allreduce_sim and its counterparts): with groups of at
    # most 1024 elements that is ONE launch which reads the N partials and writes the result, nothing else.  Timed
    # over the same rotating buffer sets; launch-bound volumes replay a HIP graph of B calls like the stages above.
    sim_s = None
    if not w.rotate and g <= 1024:
        WS = torch.empty(max(16, fc.allreduce_sim_workspace_bytes(N, T, H, g, w.bits_in, w.bits_out)),
                         dtype=torch.uint8, device=dev)

        def sim_round():
            for k in range(B):
                if fp8:
                    fc.allreduce_sim_fp8(X[k], g, out=Y[k], workspace=WS)
                elif sym:
                    fc.allreduce_sim_sym(X[k], g, w.bits_in, w.bits_out, out=Y[k], workspace=WS)
                elif cm:
                    fc.allreduce_sim_cmeta(X[k], g, w.bits_in, w.bits_out, out=Y[k], workspace=WS)
                else:
                    fc.allreduce_sim(X[k], g, w.bits_in, w.bits_out, out=Y[k], workspace=WS)

        sim_round()
        torch.cuda.synchronize()
        run_round = sim_round
        if graphs:
            gs = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gs, stream=torch.cuda.Stream()):
                sim_round()
            run_round = gs.replay
        for _ in range(20):
            run_round()
        s0, s1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s_reps = max(10, min(a.steps, 300))
        torch.cuda.synchronize()
        s0.record()
        for _ in range(s_reps):
            run_round()
        s1.record()
        torch.cuda.synchronize()
        sim_s = s0.elapsed_time(s1) * 1e-3 / (s_reps * B)
        del WS

    # one volume kept hot: the fused launch repeated on a single buffer set, whose working set (inputs and
    # outputs of one launch) fits the 256 MB memory-side cache for every workload but the 8-way fan-in
    cw0, cw1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    cw_reps = max(10, min(a.steps * B, 500))
    for _ in range(20):
        stage_fused(0)
    torch.cuda.synchronize()
    cw0.record()
    for _ in range(cw_reps):
        stage_fused(0)
    cw1.record()
    torch.cuda.synchronize()
    cw_s = cw0.elapsed_time(cw1) * 1e-3 / cw_reps

    # milliseconds per volume of each stage: mean over everything timed, and per timed step
    ms = {k: float(sum(s.elapsed_time(e) for s, e, _ in v) / sum(n for _, _, n in v)) for k, v in ev.items()}
    per_step_us = sorted(s.elapsed_time(e) / n * 1e3 for s, e, n in ev["f"])
    fused_median_us = per_step_us[len(per_step_us) // 2]
    fused_min_us = per_step_us[0]
    fused_s = ms["f"] * 1e-3
    fb = fused_bytes(w)
    achieved = fb / fused_s / 1e9

    out = {
        # `value` is the GB/s; the percentage of HBM peak that the metric also names is `pct_hbm_peak`
        "metric": "fused dequant-reduce-requant GB/s and %% HBM peak on 1 MI355X (%s)"
                  % ("70B prefill" if w.name == "llama3_70b_prefill" else w.name),
        "value": round(achieved, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": a.steps,
        "warmup": settle_steps + max(1, a.warmup),          # untimed steps actually run (config.warmup_requested as passed)
        "ms_per_step": round(wall / a.steps * 1e3, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": "%s: N=%d partial fp16 tensors of %d tokens x %d hidden, N(0,1) with %g%% outlier "
                        "channels x%g, %s, group %d"
                        % (w.name, N, T, H, 100 * w.outlier_frac, w.outlier_gain,
                           "FP8 E4M3 -> FP8 E4M3 symmetric" if fp8 else
                           "INT%d->INT%d %s" % (w.bits_in, w.bits_out, "symmetric" if sym else
                                                 "asymmetric, binary16 scale and zero-point" if cm else "asymmetric"), g)
                        + (", Hadamard rotation fused into quantize / dequantize" if w.rotate else ""),
            "n_src": N, "tokens": T, "hidden": H, "group": g, "bits_in": w.bits_in, "bits_out": w.bits_out,
            "volumes_per_step": B,
            "warmup_requested": a.warmup,
            "settle_steps": settle_steps,
            "stage_order": "volume-major (dependent)" if a.dependent else "stage-major over the batch",
            "launch": "HIP graph replay per stage" if graphs else "eager",
        },
        "pct_hbm_peak": round(100 * achieved / HBM_PEAK_GBPS, 2),
        "stages": {
            "quantize_xN": {"us": round(ms["q"] * 1e3, 2),
                            "GBps": round(N * quantize_bytes(w) / (ms["q"] * 1e-3) / 1e9, 1)},
            "dequant_reduce_requant": {"us": round(ms["f"] * 1e3, 2), "GBps": round(achieved, 1)},
            "dequantize": {"us": round(ms["d"] * 1e3, 2),
                           "GBps": round(dequantize_bytes(w) / (ms["d"] * 1e-3) / 1e9, 1)},
            "whole_path_GBps": round(B * vol_bytes / (wall / a.steps) / 1e9, 1),
        },
        "roofline": {
            "kernel": "k_dequant_reduce_requant%s<%d,%d,%d>%s" % ("_sym" if (sym or fp8) else "", w.bits_in, w.bits_out,
                                                                 N, " (E4M3)" if fp8 else " (binary16 metadata)" if cm else ""),
            "bound": "hbm",                                  # the metric's own roofline: bytes against the HBM peak
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBPS, 4),
            "algorithmic_bytes_per_launch": fb,
            "us_per_launch": round(ms["f"] * 1e3, 2),
            "us_per_launch_median_over_steps": round(fused_median_us, 2),
            "us_per_launch_min_over_steps": round(fused_min_us, 2),
            "launches_timed": a.steps * B,
            "cache_warm_single_set": {
                "what": "the same launch repeated on one buffer set (working set %.0f MB, memory-side cache "
                        "256 MB): not an HBM figure" % (fused_bytes(w) / 1e6),
                "us_per_launch": round(cw_s * 1e6, 2),
                "GBps": round(fused_bytes(w) / cw_s / 1e9, 1),
            },
            "traffic": load_profile_constant(w.name, "fused_hbm_bytes_per_launch"),
            "traffic_source": "stored constant: profiles/traffic_%s.txt (rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE, calibrated "
                              "against a copy of known size); not measured by this run" % w.name,
            "stream_reference": {
                "what": "fc_stream_reference: %d code slabs in, 1 out, the fused kernel's tiling and staging, "
                        "no arithmetic, no scales / zero-points" % N,
                "bytes_per_launch": sr_bytes,
                "us_per_launch": round(sr_s * 1e6, 2),
                "GBps": round(sr_bytes / sr_s / 1e9, 1),
                "fused_over_reference": round(achieved / (sr_bytes / sr_s / 1e9), 4),
            },
        },
    }
    if sim_s is not None:
        three = (ms["q"] + ms["f"] + ms["d"]) * 1e3
        sim_bytes = (N + 1) * 2 * T * H
        out["stages"]["allreduce_sim"] = {
            "what": "fc_allreduce_sim end to end, one launch: N binary16 partials in, binary16 result out, both "
                    "quantizations in registers (bit-identical to the three stages)",
            "us": round(sim_s * 1e6, 2),
            "bytes": sim_bytes,
            "GBps": round(sim_bytes / sim_s / 1e9, 1),
            "stages_as_benchmarked_us": round(three, 2),      # N quantize launches + fused + dequantize, as timed above
        }
    if probe_s is not None:
        valu = load_profile_constant(w.name, "fused_valu_wave_instructions_per_launch")
        out["roofline"]["compute_only"] = {
            "what": "fc_fused_compute_probe: the same launch (grid, instructions per wavefront) with every workgroup "
                    "working in the first 64 tiles, which stay in the L2: what the arithmetic alone costs",
            "us_per_launch": round(probe_s * 1e6, 2),
            "fused_over_compute_only": round(fused_s / probe_s, 4),
        }
        if valu:
            rate = valu / fused_s
            out["roofline"]["alu"] = {
                "bound": "alu", "unit": "wave64 VALU instructions/s",
                "instructions_per_launch": valu,
                "instructions_source": "stored constant: profiles/traffic_%s.txt (rocprofv3 --pmc SQ_INSTS_VALU)" % w.name,
                "achieved": round(rate, 1), "peak": VALU_PEAK_WAVE_INSTR_PER_S,
                "frac": round(rate / VALU_PEAK_WAVE_INSTR_PER_S, 4),
                "what": "peak = 256 CUs x 4 SIMDs x 2.4 GHz / 4 cycles per wave64 instruction",
            }
    # the paper's own figures: other hardware (L40, A100) and other quantities (end-to-end all-reduce latency
    # against NCCL, time to first token), quoted as context only, never as a baseline for `value`
    out["paper_context"] = ("Flash Communication reports up to 3.18x lower all-reduce latency than NCCL's ring "
                            "(Section 5.3) and 2.06x (LLaMA-3-8B, 4 x L40) / 1.19x (LLaMA-3-70B, 8 x A100) faster "
                            "time to first token (Section 4.3); none of these measures this kernel")
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, X[0].cpu().numpy())
        out["cpu_baseline"]["gpu_over_cpu"] = round(out["value"] / out["cpu_baseline"]["value"], 1)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
