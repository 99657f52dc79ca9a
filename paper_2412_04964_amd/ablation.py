"""Quantization-error sweep over the axes of the paper's ablations (precision and
symmetric/asymmetric quantizer: Table 4 and Table 6; group size: the block-size
figure of Section 3.2.1; naive versus Hadamard-rotated quantization: the rotation table of Section 4), on
synthetic activations.

    python -m paper_2412_04964_amd.ablation [--tokens 1024] [--hidden 8192] [--n-src 4]

The paper reports perplexity of real LLaMA models, which needs weights and
datasets; what can be measured without them is the error the quantized
all-reduce itself introduces: the mean squared error of fc_allreduce_sim's output
against the exact (fp32) sum of the same partial tensors, printed per setting
together with the signal-to-noise ratio.  All quantization work runs in the HIP
library; torch is used only to draw the inputs and to form the reference sum and
the mean.
"""
from __future__ import annotations

import argparse
import json
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

# label -> (bits before the reduce, bits before the gather); INT6 is the paper's mixed setting
PRECISIONS = {"INT8": (8, 8), "INT6": (4, 8), "INT4": (4, 4)}


def sweep(x, groups, precisions=PRECISIONS, rotation=False):
    """x: float16 CUDA tensor [N, tokens, hidden].  Returns a list of dict rows; rotation=True adds
    the same settings with the Hadamard rotation around the all-reduce (quantizer label + "+ht")."""
    import torch

    from . import binding as fc

    exact = x.float().sum(0)
    power = float((exact * exact).mean())
    rows = []
    for label, (b_rs, b_ag) in precisions.items():
        # "cmeta": the asymmetric quantizer with the scale and zero-point stored as binary16
        for quantizer, fn in (("asym", fc.allreduce_sim), ("sym", fc.allreduce_sim_sym),
                              ("cmeta", fc.allreduce_sim_cmeta)):
            for g in groups:
                if x.shape[2] % g:
                    continue
                y = fn(x, g, b_rs, b_ag)
                err = y.float() - exact
                mse = float((err * err).mean())
                rows.append({"precision": label, "quantizer": quantizer, "group": g, "mse": mse,
                             "snr_db": float(10.0 * torch.log10(torch.tensor(power / mse))) if mse > 0
                             else float("inf")})
    for g in groups:                                   # the paper's FP8_Sym rows
        if x.shape[2] % g:
            continue
        err = fc.allreduce_sim_fp8(x, g).float() - exact
        mse = float((err * err).mean())
        rows.append({"precision": "FP8", "quantizer": "sym", "group": g, "mse": mse,
                     "snr_db": float(10.0 * torch.log10(torch.tensor(power / mse))) if mse > 0 else float("inf")})
    block = x.shape[2] & -x.shape[2]                   # the rotation runs over blocks of this many elements
    if rotation and block in (1024, 2048, 4096, 8192):  # the "w/ HT" columns of the rotation table
        for label, b_rs, b_ag, qz in [(l, p[0], p[1], q) for l, p in precisions.items()
                                      for q in (fc.QUANTIZER_ASYM, fc.QUANTIZER_SYM)] + \
                                     [("FP8", 8, 8, fc.QUANTIZER_FP8)]:
            for g in groups:
                if x.shape[2] % g:
                    continue
                err = fc.allreduce_sim_rot(x, g, b_rs, b_ag, qz).float() - exact
                mse = float((err * err).mean())
                rows.append({"precision": label, "quantizer": ("asym", "sym", "sym")[qz] + "+ht", "group": g,
                             "mse": mse,
                             "snr_db": float(10.0 * torch.log10(torch.tensor(power / mse))) if mse > 0
                             else float("inf")})
    return rows


def main():
    import torch

    import synth_inputs

    ap = argparse.ArgumentParser()
    ap.add_argument("--tokens", type=int, default=1024)
    ap.add_argument("--hidden", type=int, default=8192)
    ap.add_argument("--n-src", type=int, default=4)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--json", action="store_true", help="print the rows as one JSON line")
    a = ap.parse_args()
    if not torch.cuda.is_available():
        sys.exit("ablation: no GPU visible; the HIP path has no CPU fallback")
    x = synth_inputs.make_partials_device(a.n_src, a.tokens, a.hidden, a.seed, "cuda")
    groups = [g for g in (32, 64, 128, 256, 512, 1024, 2048, 4096, 8192, 16384) if g <= a.hidden]
    rows = sweep(x, groups, rotation=True)
    if a.json:
        print(json.dumps(rows))
        return
    print("all-reduce quantization error, N=%d partials of %d x %d (N(0,1), 1%% outlier channels x20)"
          % (a.n_src, a.tokens, a.hidden))
    print("%-6s %-8s" % ("prec", "quant") + " ".join("%10s" % ("g=%d" % g) for g in groups))
    for label in ("FP8",) + tuple(PRECISIONS):
        for q in ("asym", "cmeta", "sym", "asym+ht", "sym+ht"):
            r = {row["group"]: row for row in rows if row["precision"] == label and row["quantizer"] == q}
            if r:
                print("%-6s %-8s" % (label, q) + " ".join("%10.3e" % r[g]["mse"] for g in groups))


if __name__ == "__main__":
    main()
