"""Pins for the oracle's Hadamard rotation (Section 4 of the paper, rotation-based quantization): the
transform against scipy's Sylvester matrices in exact integer arithmetic, hand-worked examples that
expose the stage order (tests/golden/hand_rotation.txt), an exact-rational replay, involution, the
fp64 product, closed forms of the rotated all-reduce and its error bound.  CPU only."""
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.linalg

import oracle
import synth_inputs
from test_oracle_pins import bits_of, from_bits, parse_values, rn32

F32 = np.float32


def load_golden_rot(golden_dir):
    tr, q = {}, {}
    with open(os.path.join(golden_dir, "hand_rotation.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            f = [c.strip() for c in line.split("|")]
            if f[0].startswith("T"):
                tr[f[0]] = dict(x=parse_values(f[1]), y=from_bits(f[2].split()))
            else:
                q[f[0]] = dict(bits=int(f[1]), x=np.array(f[2].split(), dtype=np.float16),
                               scale=from_bits([f[3]])[0], zero=float(f[4]),
                               codes=np.array(f[5].split(), dtype=np.uint8),
                               out=np.array(f[6].split(), dtype=np.float16))
    assert len(tr) == 3 and len(q) == 1
    return tr, q


def test_hand_transforms(golden_dir):
    tr, _ = load_golden_rot(golden_dir)
    for name, g in tr.items():
        assert np.array_equal(bits_of(oracle.hadamard_f32(g["x"])), bits_of(g["y"])), name


def test_hand_rotated_quantization(golden_dir):
    _, q = load_golden_rot(golden_dir)
    for name, g in q.items():
        n = g["x"].size
        c, s, z = oracle.quantize_rot(g["x"][None, :], n, g["bits"], oracle.ASYM)
        codes = np.stack([c[0] & 0x0F, c[0] >> 4], -1).reshape(-1) if g["bits"] == 4 else c[0]
        assert np.array_equal(codes, g["codes"]), name
        assert bits_of(s)[0, 0] == bits_of(g["scale"]) and z[0, 0] == g["zero"], name
        y = oracle.dequantize_rot(c, s, z, n, n, g["bits"], oracle.ASYM)
        assert np.array_equal(y[0].view(np.uint16), g["out"].view(np.uint16)), name
        y2 = oracle.allreduce_sim_rot(g["x"][None, None, :], n, g["bits"], g["bits"], oracle.ASYM)
        assert np.array_equal(y2[0].view(np.uint16), g["out"].view(np.uint16)), name


@pytest.mark.parametrize("n", [1, 2, 4, 8, 64, 512, 4096])
def test_transform_is_the_sylvester_matrix_on_integers(n):
    # small integers: every fp32 sum is exact, so the result must equal the integer matrix product
    rng = np.random.default_rng(n)
    x = rng.integers(-50, 51, size=(3, n))
    want = x @ scipy.linalg.hadamard(n).astype(np.int64) if n > 1 else x
    got = oracle.hadamard_f32(x.astype(np.float32))
    assert np.array_equal(got.astype(np.int64), want)
    # involution: H(H(x)) = n x, exactly
    assert np.array_equal(oracle.hadamard_f32(got).astype(np.int64), n * x)


def test_transform_against_fp64_product_and_parseval():
    rng = np.random.default_rng(1)
    for n in (16, 1024, 8192):
        x = (rng.standard_normal((2, n)) * 3).astype(np.float32)
        got = oracle.hadamard_f32(x).astype(np.float64)
        want = x.astype(np.float64) @ scipy.linalg.hadamard(n).astype(np.float64)
        # log2(n) roundings, each relative 2^-24 of a partial sum bounded by the 1-norm
        bound = np.log2(n) * 2.0 ** -24 * np.abs(x).sum(-1, keepdims=True)
        assert np.all(np.abs(got - want) <= bound)
        assert np.allclose((got ** 2).sum(-1), n * (x.astype(np.float64) ** 2).sum(-1), rtol=1e-5)


def _replay(x, spans):
    v = [Fraction(float(a)) for a in x]
    for span in spans:
        for base in range(0, len(v), 2 * span):
            for i in range(base, base + span):
                a, b = v[i], v[i + span]
                v[i] = Fraction(float(rn32(a + b)))
                v[i + span] = Fraction(float(rn32(a - b)))
    return v


def test_stage_order_replayed_in_exact_arithmetic():
    rng = np.random.default_rng(2)
    differs = 0
    for trial in range(6):
        x = (rng.standard_normal(32) * np.exp(rng.uniform(-4, 4, 32))).astype(np.float32)
        got = [Fraction(float(v)) for v in oracle.hadamard_f32(x)]
        assert got == _replay(x, [1, 2, 4, 8, 16]), trial
        differs += got != _replay(x, [16, 8, 4, 2, 1])
    assert differs > 0          # the check above can tell the two stage orders apart


@pytest.mark.parametrize("quantizer", [oracle.ASYM, oracle.SYM, oracle.FP8])
def test_scalings_and_no_intermediate_binary16(quantizer):
    # forward scaling 2^-ceil(n/2): rotate+quantize equals quantizing the scaled fp32 transform
    for hidden, group in ((2048, 128), (4096, 4096), (8192, 1024)):
        n = int(np.log2(hidden))
        x = synth_inputs.make_partials(1, 3, hidden, seed=hidden)[0]
        rot = oracle.hadamard_f32(x.astype(np.float32)) * F32(2.0 ** -((n + 1) // 2))
        assert (rot.astype(np.float16).astype(np.float32) != rot).any()     # binary16 would lose bits
        c, s, z = oracle.quantize_rot(x, group, 8, quantizer)
        if quantizer == oracle.ASYM:
            want = oracle.quantize_f32(rot, group, 8)
        elif quantizer == oracle.SYM:
            want = oracle.quantize_sym_f32(rot, group, 8) + (np.zeros_like(s),)
        else:
            want = oracle.quantize_fp8_f32(rot, group) + (np.zeros_like(s),)
        assert np.array_equal(c, want[0]) and np.array_equal(bits_of(s), bits_of(want[1]))
        if quantizer == oracle.ASYM:
            assert np.array_equal(bits_of(z), bits_of(want[2]))
        # inverse scaling 2^-floor(n/2) after the transform of the dequantized values
        if quantizer == oracle.ASYM:
            d = oracle.dequantize_f32(c, s, z, hidden, group, 8)
        elif quantizer == oracle.SYM:
            d = oracle.dequantize_sym_f32(c, s, hidden, group, 8)
        else:
            d = oracle.dequantize_fp8_f32(c, s, hidden, group)
        back = (oracle.hadamard_f32(d) * F32(2.0 ** -(n // 2))).astype(np.float16)
        y = oracle.dequantize_rot(c, s, z, hidden, group, 8, quantizer)
        assert np.array_equal(y.view(np.uint16), back.view(np.uint16))


def test_walsh_function_partials_all_reduce_exactly():
    # a partial that is a multiple of one row of the Sylvester matrix rotates to a single non-zero
    # entry, which every quantizer represents exactly; 2^k such partials sum exactly
    hidden = 2048
    H = scipy.linalg.hadamard(hidden).astype(np.float32)
    x = np.stack([H[5] * 0.75, H[77] * -1.5, H[2047] * 0.25]).astype(np.float16)
    for quantizer, bits in ((oracle.ASYM, 4), (oracle.SYM, 4), (oracle.ASYM, 8), (oracle.FP8, 8)):
        for n_src in (1, 2, 4):
            y = oracle.allreduce_sim_rot(np.stack([x] * n_src), hidden, bits, bits, quantizer)
            assert np.array_equal(y.astype(np.float32), x.astype(np.float32) * n_src), (quantizer, bits, n_src)


@pytest.mark.parametrize("bits", [4, 8])
def test_rotated_allreduce_error_bound_and_gain_on_outlier_channels(bits):
    hidden, n_src = 4096, 4
    x = synth_inputs.make_partials(n_src, 6, hidden, seed=8)
    exact = x.astype(np.float64).sum(0)
    for group in (128, 4096):
        y = oracle.allreduce_sim_rot(x, group, bits, bits, oracle.ASYM).astype(np.float64)
        parts = [oracle.quantize_rot(x[j], group, bits, oracle.ASYM) for j in range(n_src)]
        c = np.stack([p[0] for p in parts]); s = np.stack([p[1] for p in parts]); z = np.stack([p[2] for p in parts])
        s2 = oracle.dequant_reduce_requant(c, s, z, hidden, group, bits, bits)[1]
        # per rotated element the two stages are off by at most sum_j s_j/2 + s'/2; the inverse transform
        # with its 2^-floor(n/2) scaling is orthonormal here (n = 12), so the 2-norm carries over
        per_elem = np.repeat(s.astype(np.float64).sum(0) / 2 + s2.astype(np.float64) / 2, group, axis=1)
        l2_bound = np.sqrt((per_elem ** 2).sum(-1)) * (1 + 1e-3) + np.sqrt(hidden) * np.abs(y).max() * 2.0 ** -11
        assert np.all(np.sqrt(((y - exact) ** 2).sum(-1)) <= l2_bound)
    # the paper's finding for coarse groups: the rotation repairs per-token quantization
    plain = oracle.allreduce_sim(x, hidden, bits, bits).astype(np.float64)
    rot = oracle.allreduce_sim_rot(x, hidden, bits, bits, oracle.ASYM).astype(np.float64)
    assert np.mean((rot - exact) ** 2) < np.mean((plain - exact) ** 2) / 3


def test_rot_bad_arguments():
    x = synth_inputs.make_partials(1, 2, 96, seed=1)[0]
    oracle.quantize_rot(x, 32, 8)                        # hidden 96 = 3 x 32: rotated block by block
    with pytest.raises(Exception):
        oracle.quantize_rot(x, 64, 8)                    # the group does not divide hidden
    with pytest.raises(Exception):
        oracle.quantize_rot(synth_inputs.make_partials(1, 2, 128, seed=1)[0], 32, 4, oracle.FP8)


# --------------------------------------------------------------------------- #
# rows whose length is not a power of two: the transform block by block (I (x) H_B, B the largest power of two
# dividing the length; the rotation table's LLaMA-2-13B row has hidden 5120 = 5 x 1024)
# --------------------------------------------------------------------------- #

@pytest.mark.parametrize("n,block", [(1, 1), (6, 2), (12, 4), (96, 32), (640, 128), (5120, 1024), (3072, 1024),
                                     (7168, 1024), (6144, 2048), (4096, 4096), (17, 1)])
def test_block_transform_is_the_kronecker_product_on_integers(n, block):
    rng = np.random.default_rng(n)
    x = rng.integers(-50, 51, size=(2, n))
    hb = scipy.linalg.hadamard(block).astype(np.int64) if block > 1 else np.ones((1, 1), np.int64)
    want = (x.reshape(2, n // block, block) @ hb).reshape(2, n)       # == x @ kron(I, H_B)
    got = oracle.hadamard_blocks_f32(x.astype(np.float32))
    assert np.array_equal(got.astype(np.int64), want)
    assert np.array_equal(oracle.hadamard_blocks_f32(got).astype(np.int64), block * x)     # involution up to B
    if n <= 640:                                                        # the dense orthogonal matrix itself
        dense = scipy.linalg.block_diag(*([hb] * (n // block)))
        assert np.array_equal(want, x @ dense)
        assert np.array_equal(dense @ dense.T, block * np.eye(n, dtype=np.int64))
    if block == n:                                                      # a power of two: the plain transform
        assert np.array_equal(bits_of(got), bits_of(oracle.hadamard_f32(x.astype(np.float32))))


@pytest.mark.parametrize("quantizer,bits", [(oracle.ASYM, 4), (oracle.ASYM, 8), (oracle.SYM, 4), (oracle.FP8, 8)])
@pytest.mark.parametrize("hidden,block", [(5120, 1024), (3072, 1024), (6144, 2048), (96, 32)])
def test_rotated_quantization_of_a_row_is_that_of_its_blocks(quantizer, bits, hidden, block):
    # blocks are independent and groups lie inside blocks: quantizing [tokens, hidden] must equal quantizing the
    # same memory viewed as [tokens * hidden / B, B], whose rows are powers of two (the case pinned above and by
    # the hand examples); likewise for Dequantize and for the whole all-reduce
    rng = np.random.default_rng(hidden + bits)
    tokens, n_src = 3, 2
    x = (rng.standard_normal((n_src, tokens, hidden)) * np.where(rng.random(hidden) < 0.02, 20.0, 1.0)).astype(np.float16)
    xb = x.reshape(n_src, tokens * hidden // block, block)
    for group in (32, block):
        c, s, z = oracle.quantize_rot(x[0], group, bits, quantizer)
        cb, sb, zb = oracle.quantize_rot(xb[0], group, bits, quantizer)
        assert c.tobytes() == cb.tobytes() and bits_of(s).tobytes() == bits_of(sb).tobytes()
        if quantizer == oracle.ASYM:
            assert bits_of(z).tobytes() == bits_of(zb).tobytes()
        y = oracle.dequantize_rot(c, s, z, hidden, group, bits, quantizer)
        yb = oracle.dequantize_rot(cb, sb, zb, block, group, bits, quantizer)
        assert y.view(np.uint16).tobytes() == yb.view(np.uint16).tobytes()
        a = oracle.allreduce_sim_rot(x, group, bits, bits, quantizer)
        ab = oracle.allreduce_sim_rot(xb, group, bits, bits, quantizer)
        assert a.view(np.uint16).tobytes() == ab.view(np.uint16).tobytes()


def test_block_rotation_spreads_outlier_channels_within_blocks():
    # what the rotation is for (Section 4): with outlier channels the coarse-group error drops by a large factor
    x = synth_inputs.make_partials(4, 8, 5120, seed=5, outlier_frac=0.01)
    exact = x.astype(np.float64).sum(0)
    plain = oracle.allreduce_sim(x, 1024, 4, 4).astype(np.float64)
    rot = oracle.allreduce_sim_rot(x, 1024, 4, 4, oracle.ASYM).astype(np.float64)
    assert ((rot - exact) ** 2).mean() * 3 < ((plain - exact) ** 2).mean()
