"""The oracle reproduces, on the synthetic stand-in activations, the qualitative
findings of the paper's ablations (these are sanity checks of the whole Algorithm 1
chain, not bit-level pins): error grows as bits shrink (Tables 2-4: INT8 < INT6 <
INT4), asymmetric beats symmetric at low precision (Table 4), and finer groups
beat coarse ones, per-token being worst (block-size figure of Section 3.2.1)."""
import numpy as np

import oracle
import synth_inputs


def _mse(x, group, b_rs, b_ag, sym=False):
    fn = oracle.allreduce_sim_sym if sym else oracle.allreduce_sim
    y = fn(x, group, b_rs, b_ag).astype(np.float64)
    exact = x.astype(np.float64).sum(0)
    return float(np.mean((y - exact) ** 2))


def test_error_grows_as_precision_shrinks():
    x = synth_inputs.make_partials(4, 8, 4096, seed=1)
    for sym in (False, True):
        e8, e6, e4 = (_mse(x, 128, *b, sym=sym) for b in ((8, 8), (4, 8), (4, 4)))
        assert e8 < e6 < e4
        assert e4 > 50 * e8            # 4 bits fewer: step 17x coarser, error energy ~289x


def test_asymmetric_beats_symmetric():
    # at INT4 only while the step still resolves the bulk of the values: with 1 % outlier channels
    # x20 and groups of 1024 or more, 16 levels flatten every ordinary value to zero either way and
    # both errors saturate at the signal power
    x = synth_inputs.make_partials(4, 8, 4096, seed=2)
    for g in (32, 128, 512):
        assert _mse(x, g, 4, 4) < _mse(x, g, 4, 4, sym=True)
    for g in (32, 128, 1024, 4096):
        assert _mse(x, g, 8, 8) < _mse(x, g, 8, 8, sym=True)


def test_finer_groups_are_better_and_per_token_is_worst():
    x = synth_inputs.make_partials(4, 8, 4096, seed=3)
    for sym in (False, True):
        e = [_mse(x, g, 8, 8, sym=sym) for g in (32, 128, 512, 2048, 4096)]
        assert all(a < b for a, b in zip(e, e[1:])), e
        e = [_mse(x, g, 4, 4, sym=sym) for g in (32, 128, 512)]        # INT4 saturates beyond
        assert all(a < b for a, b in zip(e, e[1:])), e
        assert _mse(x, 4096, 4, 4, sym=sym) > 1.5 * _mse(x, 128, 4, 4, sym=sym)   # the coarse collapse


def test_two_step_error_exceeds_one_step_error():
    # quantizing twice (before the reduce and before the gather) cannot beat quantizing the
    # partials once and summing them exactly in fp32
    x = synth_inputs.make_partials(4, 8, 4096, seed=4)
    g, bits = 128, 4
    parts = [oracle.quantize(x[j], g, bits) for j in range(4)]
    c = np.stack([p[0] for p in parts]); s = np.stack([p[1] for p in parts]); z = np.stack([p[2] for p in parts])
    acc = oracle.dequant_reduce_f32(c, s, z, 4096, g, bits).astype(np.float64)
    exact = x.astype(np.float64).sum(0)
    one_step = float(np.mean((acc - exact) ** 2))
    assert one_step < _mse(x, g, bits, bits)
