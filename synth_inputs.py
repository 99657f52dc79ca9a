"""Seeded synthetic activations shared by the oracle tests, the GPU parity tests
and the benchmark.  This module only draws random numbers and shapes them; it
contains none of the quantization arithmetic and imports neither the oracle nor
the GPU package.

The paper measures on real LLaMA-3 activations (outputs of the attention output
projection and the MLP down projection at batch 8 x 1024 tokens, Section 4.1 and
Figure 1) and notes that the down projection is hard to quantize because of
outlier channels (Section 3.2.1).  Those models are not available here, so the
stand-in is: N partial tensors of i.i.d. N(0,1) values, with 1 % of the hidden
channels (the same channels in every partial) multiplied by 20, rounded to
float16.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    n_src: int
    tokens: int
    hidden: int
    bits_in: int      # bit-width before the reduce (first FinegrainedQuantize)
    bits_out: int     # bit-width before the gather (second FinegrainedQuantize)
    group: int
    outlier_frac: float = 0.01
    outlier_gain: float = 20.0
    seed: int = 0
    quantizer: str = "asym"   # "asym": Eq. 1-2 (scale + zero-point), "sym": Eq. 3-4 (scale only),
                              # "fp8": E4M3 bytes with a per-group scale (the paper's FP8_Sym rows),
                              # "cmeta": Eq. 1-2 with the scale and zero-point stored as binary16 (4 bytes)

    rotate: bool = False      # Hadamard rotation around the all-reduce (Section 4 of the paper)

    @property
    def elements(self) -> int:
        return self.tokens * self.hidden

    @property
    def meta_bytes_per_group(self) -> int:
        return 8 if self.quantizer == "asym" else 4


# The five configurations the benchmark contract names, plus the paper's mixed-precision
# "INT6" setting (4 bit before the reduce, 8 bit before the gather; Section 3.2.3) at the headline shape,
# the symmetric quantizer of the paper's ablation (Table 6) at the two prefill shapes, and the
# coarsest granularity of the block-size study (one group per token) at the headline shape.
WORKLOADS = {
    "tiny": Workload("tiny", 2, 16, 4096, 8, 8, 128, outlier_frac=0.0),
    "llama3_8b_prefill": Workload("llama3_8b_prefill", 4, 8192, 4096, 8, 8, 128),
    "llama3_70b_prefill": Workload("llama3_70b_prefill", 4, 8192, 8192, 4, 4, 128),
    "wide_fanin": Workload("wide_fanin", 8, 8192, 8192, 4, 4, 64),
    "decode": Workload("decode", 8, 8, 8192, 8, 8, 128),
    "llama3_70b_prefill_int6": Workload("llama3_70b_prefill_int6", 4, 8192, 8192, 4, 8, 128),
    "llama3_70b_prefill_sym": Workload("llama3_70b_prefill_sym", 4, 8192, 8192, 4, 4, 128, quantizer="sym"),
    "llama3_70b_prefill_per_token": Workload("llama3_70b_prefill_per_token", 4, 8192, 8192, 4, 4, 8192),
    "llama3_70b_prefill_fp8": Workload("llama3_70b_prefill_fp8", 4, 8192, 8192, 8, 8, 128, quantizer="fp8"),
    "llama3_8b_prefill_fp8": Workload("llama3_8b_prefill_fp8", 4, 8192, 4096, 8, 8, 128, quantizer="fp8"),
    "llama3_70b_prefill_per_token_rot": Workload("llama3_70b_prefill_per_token_rot", 4, 8192, 8192, 4, 4, 8192,
                                                 rotate=True),
    "llama3_70b_prefill_rot": Workload("llama3_70b_prefill_rot", 4, 8192, 8192, 4, 4, 128, rotate=True),
    "llama3_8b_prefill_sym": Workload("llama3_8b_prefill_sym", 4, 8192, 4096, 8, 8, 128, quantizer="sym"),
    "llama3_70b_prefill_cmeta": Workload("llama3_70b_prefill_cmeta", 4, 8192, 8192, 4, 4, 128, quantizer="cmeta"),
    "llama3_8b_prefill_cmeta": Workload("llama3_8b_prefill_cmeta", 4, 8192, 4096, 8, 8, 128, quantizer="cmeta"),
    # the rotation table's LLaMA-2-13B row at its group size 1024: hidden 5120 is rotated as five blocks of 1024
    "llama2_13b_prefill_rot": Workload("llama2_13b_prefill_rot", 4, 8192, 5120, 4, 4, 1024, rotate=True),
}


def outlier_channels(hidden: int, frac: float, rng: np.random.Generator) -> np.ndarray:
    k = int(round(frac * hidden))
    if k == 0:
        return np.zeros(0, np.int64)
    return np.sort(rng.choice(hidden, k, replace=False))


def make_partials(n_src: int, tokens: int, hidden: int, seed: int = 0,
                  outlier_frac: float = 0.01, outlier_gain: float = 20.0) -> np.ndarray:
    """float16 [n_src, tokens, hidden], host memory."""
    rng = np.random.default_rng(seed)
    ch = outlier_channels(hidden, outlier_frac, rng)
    out = np.empty((n_src, tokens, hidden), np.float16)
    for j in range(n_src):
        x = rng.standard_normal((tokens, hidden), dtype=np.float32)
        if ch.size:
            x[:, ch] *= np.float32(outlier_gain)
        out[j] = x.astype(np.float16)
    return out


def make_workload(w: Workload, seed: int | None = None, tokens: int | None = None) -> np.ndarray:
    """Partials of a named workload; `tokens` overrides the row count (the
    row-sampled variants used where the full tensor is too big for the host)."""
    return make_partials(w.n_src, w.tokens if tokens is None else tokens, w.hidden,
                         w.seed if seed is None else seed, w.outlier_frac, w.outlier_gain)


def make_partials_device(n_src: int, tokens: int, hidden: int, seed: int, device,
                         outlier_frac: float = 0.01, outlier_gain: float = 20.0):
    """Same distribution drawn on the GPU with torch's seeded generator (used
    for the multi-gigabyte benchmark sets, which would take minutes to draw on
    the host).  Returns a float16 torch tensor [n_src, tokens, hidden]."""
    import torch

    rng = np.random.default_rng(seed)
    ch = outlier_channels(hidden, outlier_frac, rng)
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    out = torch.empty((n_src, tokens, hidden), dtype=torch.float16, device=device)
    gain = torch.ones(hidden, dtype=torch.float32, device=device)
    if ch.size:
        gain[torch.from_numpy(ch).to(device)] = outlier_gain
    for j in range(n_src):
        x = torch.randn((tokens, hidden), generator=g, dtype=torch.float32, device=device)
        out[j] = (x * gain).to(torch.float16)
        del x
    return out


def adversarial_groups(group: int, seed: int = 0) -> np.ndarray:
    """float16 [rows, 8*group]: rows of hand-picked hard groups (constant, all
    positive, all negative, zeros, tiny range on a large offset, float16
    extremes, subnormals, exact .5 ties) padded with N(0,1) groups."""
    rng = np.random.default_rng(seed)
    g = group
    rows = []

    def row(*groups):
        gs = [np.asarray(a, np.float32) for a in groups]
        while len(gs) < 8:
            gs.append(rng.standard_normal(g, dtype=np.float32))
        rows.append(np.concatenate(gs[:8]))

    ramp = np.arange(g, dtype=np.float32)
    row(np.full(g, 3.3), np.full(g, -0.7), np.zeros(g), np.full(g, 65504.0), np.full(g, -65504.0))
    row(1.0 + ramp / 1024.0, -1.0 - ramp / 1024.0, 1000.0 + (ramp % 2), 6.1e-5 * (ramp % 3),
        5.96e-8 * (ramp % 7))
    row(ramp - g / 2, (ramp - g / 2) * 0.5, (ramp % 16) * 0.25 - 2.0, (ramp % 256) * 0.125 - 1.0)
    row(np.where(ramp == 5, 65504.0, 0.0), np.where(ramp == 7, -65504.0, 65504.0),
        np.where(ramp % 2 == 0, 2048.0, 2049.0 - 1.0 + 2.0), rng.uniform(100, 101, g))
    row(rng.uniform(-1e-3, 1e-3, g), rng.uniform(0, 6e-5, g), rng.standard_normal(g) * 1000,
        np.abs(rng.standard_normal(g)) + 30.0, -np.abs(rng.standard_normal(g)) - 500.0)
    return np.stack(rows).astype(np.float16)


STRESS_KINDS = 6


def make_partials_stress(n_src: int, tokens: int, hidden: int, kind: int, seed: int = 0) -> np.ndarray:
    """float16 [n_src, tokens, hidden] from one of STRESS_KINDS value distributions chosen to reach the
    corners of the quantizers: 0 plain N(0,1); 1 per-row scales over 22 octaves; 2 a narrow band on a
    large offset (huge zero-points); 3 half-integers (rounding ties everywhere); 4 sparse large spikes
    (mostly-zero groups); 5 micro-noise on a constant (near-degenerate groups, float16 extremes)."""
    rng = np.random.default_rng(seed)
    shape = (n_src, tokens, hidden)
    if kind == 0:
        x = rng.standard_normal(shape)
    elif kind == 1:
        x = rng.standard_normal(shape) * np.exp(rng.uniform(-12, 10, (n_src, tokens, 1)))
    elif kind == 2:
        x = rng.uniform(100, 101, shape) * rng.choice([-1, 1])
    elif kind == 3:
        x = np.round(rng.standard_normal(shape) * 4) / 2
    elif kind == 4:
        x = rng.standard_normal(shape) * (rng.random(shape) < 0.02) * 1000
    else:
        x = rng.standard_normal(shape) * 1e-6 + rng.choice([0, 3, -500, 60000])
    return np.clip(x, -65504, 65504).astype(np.float16)
