"""Pins for the CPU oracle: everything here checks ``oracle/`` against something
other than itself -- hand-worked groups (tests/golden/hand_groups.txt), numpy's
own float16 conversion, exact rational arithmetic, closed forms, invariants of
Eq. 1-2 and the error bound that Section 3.2.1 of the paper implies for the
two-step scheme.  No GPU is used.
"""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
import synth_inputs

F32 = np.float32


def bits_of(x) -> np.ndarray:
    return np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)


def from_bits(words) -> np.ndarray:
    return np.array([int(w, 16) for w in words], dtype=np.uint32).view(np.float32)


def parse_values(field) -> np.ndarray:
    # decimal tokens are exact fp32 values; 0x tokens are fp32 bit patterns
    return np.array([from_bits([t])[0] if t.lower().startswith("0x") else F32(t)
                     for t in field.split()], dtype=np.float32)


def load_golden(golden_dir):
    groups, reductions = {}, {}
    with open(os.path.join(golden_dir, "hand_groups.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            f = [c.strip() for c in line.split("|")]
            if f[0].startswith("W"):
                groups[f[0]] = dict(bits=int(f[1]), x=parse_values(f[2]),
                                    scale=from_bits([f[3]])[0], zero=F32(f[4]),
                                    codes=np.array(f[5].split(), dtype=np.uint8),
                                    xhat=from_bits(f[6].split()))
            else:
                reductions[f[0]] = dict(bits_in=int(f[1]), bits_out=int(f[2]), sources=f[3].split(),
                                        acc=np.array(f[4].split(), dtype=np.float32),
                                        scale=from_bits([f[5]])[0], zero=F32(f[6]),
                                        codes=np.array(f[7].split(), dtype=np.uint8),
                                        xhat=from_bits(f[8].split()))
    assert len(groups) >= 10 and len(reductions) == 2
    return groups, reductions


def unpack(codes, bits):
    codes = np.asarray(codes, np.uint8)
    if bits == 8:
        return codes.copy()
    out = np.empty(codes.shape[:-1] + (codes.shape[-1] * 2,), np.uint8)
    out[..., 0::2] = codes & 0x0F
    out[..., 1::2] = codes >> 4
    return out


# --------------------------------------------------------------------------- #
# float16 <-> float32 against numpy's conversion (an independent implementation)
# --------------------------------------------------------------------------- #

def test_half_to_float_all_65536_patterns():
    h = np.arange(65536, dtype=np.uint16)
    want = h.view(np.float16).astype(np.float32)
    got = np.array([oracle.half_to_float(int(b)) for b in h], dtype=np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(bits_of(got)[~nan], bits_of(want)[~nan])


def test_float_to_half_against_numpy():
    rng = np.random.default_rng(7)
    xs = [rng.standard_normal(20000).astype(np.float32) * F32(s)
          for s in (1e-8, 1e-6, 1e-4, 1e-2, 1.0, 50.0, 3000.0, 40000.0, 1e6)]
    # every float16 value, the midpoints between neighbours (ties) and their
    # float32 neighbours on both sides
    h = np.arange(0x7C00, dtype=np.uint16).view(np.float16).astype(np.float64)
    mid = ((h[:-1] + h[1:]) / 2).astype(np.float32)
    xs += [h.astype(np.float32), mid, np.nextafter(mid, F32(np.inf)), np.nextafter(mid, F32(-np.inf))]
    xs += [np.array([65504.0, 65519.996, 65520.0, 65536.0, 1e30, np.inf, 0.0, 2.0 ** -24, 2.0 ** -25,
                     np.nextafter(F32(2.0 ** -25), F32(1)), 2.0 ** -14, 6.0975552e-05], dtype=np.float32)]
    x = np.concatenate(xs)
    x = np.concatenate([x, -x])
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    got = np.array([oracle.float_to_half(v) for v in x], dtype=np.uint16)
    assert np.array_equal(got, want)


# --------------------------------------------------------------------------- #
# hand-worked groups: Eq. 1-2, Dequantize, Algorithm 1's reduce
# --------------------------------------------------------------------------- #

def test_hand_groups_quantize_and_dequantize(golden_dir):
    groups, _ = load_golden(golden_dir)
    for name, g in groups.items():
        q, s, z = oracle.quantize_group_f32(g["x"], g["bits"])
        assert np.array_equal(q, g["codes"]), name
        assert bits_of(s) == bits_of(g["scale"]), name
        assert bits_of(z) == bits_of(g["zero"]), name       # also pins +0 for the zero group
        n = g["x"].size
        if g["bits"] == 8 or n % 2 == 0:
            c, ss, zz = oracle.quantize_f32(g["x"][None, :], n, g["bits"])
            assert np.array_equal(unpack(c, g["bits"])[0], g["codes"]), name
            xhat = oracle.dequantize_f32(c, ss, zz, n, n, g["bits"])
            assert np.array_equal(bits_of(xhat[0]), bits_of(g["xhat"])), name


def test_int4_packing_order_low_nibble_is_even_element(golden_dir):
    groups, _ = load_golden(golden_dir)
    c, _, _ = oracle.quantize_f32(groups["W1"]["x"][None, :], 4, 4)
    assert c.tolist() == [[0x20, 0xF4]]


def test_hand_reduction(golden_dir):
    groups, reds = load_golden(golden_dir)
    for name, r in reds.items():
        srcs = [groups[s] for s in r["sources"]]
        n = srcs[0]["x"].size
        parts = [oracle.quantize_f32(s["x"][None, :], n, r["bits_in"]) for s in srcs]
        c = np.stack([p[0] for p in parts])
        s = np.stack([p[1] for p in parts])
        z = np.stack([p[2] for p in parts])
        acc = oracle.dequant_reduce_f32(c, s, z, n, n, r["bits_in"])
        assert np.array_equal(bits_of(acc[0]), bits_of(r["acc"])), name
        co, so, zo = oracle.dequant_reduce_requant(c, s, z, n, n, r["bits_in"], r["bits_out"])
        assert np.array_equal(unpack(co, r["bits_out"])[0], r["codes"]), name
        assert bits_of(so)[0, 0] == bits_of(r["scale"]) and bits_of(zo)[0, 0] == bits_of(r["zero"]), name
        xh = oracle.dequantize_f32(co, so, zo, n, n, r["bits_out"])
        assert np.array_equal(bits_of(xh[0]), bits_of(r["xhat"])), name
        # the end-to-end entry point on the same float16 inputs
        x16 = np.stack([s_["x"][None, :] for s_ in srcs]).astype(np.float16)
        y = oracle.allreduce_sim(x16, n, r["bits_in"], r["bits_out"])
        assert np.array_equal(y[0].view(np.uint16), r["xhat"].astype(np.float16).view(np.uint16)), name


# --------------------------------------------------------------------------- #
# invariants of Eq. 1-2
# --------------------------------------------------------------------------- #

def _datasets():
    rng = np.random.default_rng(3)
    yield "normal", rng.standard_normal((24, 1024)).astype(np.float32)
    yield "outliers", synth_inputs.make_partials(1, 24, 1024, seed=5)[0].astype(np.float32)
    yield "positive", (np.abs(rng.standard_normal((8, 1024))) + 3).astype(np.float32)
    yield "negative", (-np.abs(rng.standard_normal((8, 1024))) - 100).astype(np.float32)
    yield "tiny", (rng.standard_normal((8, 1024)) * 1e-6).astype(np.float32)
    yield "adversarial", synth_inputs.adversarial_groups(128).astype(np.float32)
    for kind in range(synth_inputs.STRESS_KINDS):
        yield "stress %d" % kind, synth_inputs.make_partials_stress(1, 8, 1024, kind, seed=kind)[0].astype(np.float32)


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("group", [32, 64, 128, 1024])
def test_quantizer_invariants(bits, group):
    qmax = (1 << bits) - 1
    for name, x in _datasets():
        t, h = x.shape
        c, s, z = oracle.quantize_f32(x, group, bits)
        q = unpack(c, bits).reshape(t, h // group, group)
        xg = x.reshape(t, h // group, group)
        assert q.max() <= qmax, name
        assert np.all(s > 0) and np.all(np.isfinite(s)), name
        assert np.array_equal(z, np.rint(z)), name
        # the group minimum always gets code 0; the maximum gets qmax or qmax-1
        amin = xg.argmin(-1)[..., None]
        amax = xg.argmax(-1)[..., None]
        const = (xg.max(-1) == xg.min(-1))
        assert np.all(np.take_along_axis(q, amin, -1) == 0), name
        top = np.take_along_axis(q, amax, -1)[..., 0]
        assert np.all((top[~const] == qmax) | (top[~const] == qmax - 1)), name
        assert np.all(q[const] == 0), name
        # reconstruction: within half a step (plus fp32 slop), exact for constant groups
        xh = oracle.dequantize_f32(c, s, z, h, group, bits).reshape(xg.shape)
        err = np.abs(xh.astype(np.float64) - xg.astype(np.float64))
        slop = 1.0 + 2.0 ** -20 * (np.abs(z) + qmax + 4)
        assert np.all(err[~const] <= (0.5 * s.astype(np.float64) * slop)[~const][..., None] + 1e-45), name
        assert np.array_equal(xh[const], xg[const]), name          # by value: a group of mixed +-0 gives +0
        nz = const & (xg[..., 0] != 0)
        assert np.array_equal(bits_of(xh[nz]), bits_of(xg[nz])), name
        # monotone: a larger value never gets a smaller code
        order = np.argsort(xg, axis=-1, kind="stable")
        qs = np.take_along_axis(q, order, -1).astype(np.int32)
        assert np.all(np.diff(qs, axis=-1) >= 0), name


@pytest.mark.parametrize("bits", [4, 8])
def test_power_of_two_scaling_and_permutation(bits):
    rng = np.random.default_rng(11)
    x = rng.standard_normal((6, 512)).astype(np.float32)
    c0, s0, z0 = oracle.quantize_f32(x, 128, bits)
    for k in (-20, -3, 5, 17):
        c, s, z = oracle.quantize_f32(x * F32(2.0 ** k), 128, bits)
        assert np.array_equal(c, c0) and np.array_equal(z, z0)
        assert np.array_equal(bits_of(s), bits_of(s0 * F32(2.0 ** k)))
    perm = rng.permutation(128)
    xp = x.reshape(6, 4, 128)[:, :, perm].reshape(6, 512)
    c, s, z = oracle.quantize_f32(xp, 128, bits)
    assert np.array_equal(bits_of(s), bits_of(s0)) and np.array_equal(z, z0)
    q0 = unpack(c0, bits).reshape(6, 4, 128)
    assert np.array_equal(unpack(c, bits).reshape(6, 4, 128), q0[:, :, perm])


@pytest.mark.parametrize("bits", [4, 8])
def test_arithmetic_progression_is_exact(bits):
    # x_k = mn + k*2^e for k = 0..qmax: codes are k, zero-point is -mn/2^e, exact round trip
    qmax = (1 << bits) - 1
    g = qmax + 1
    rows = []
    params = [(-3, -2), (0, 0), (7, 3), (-200, -4), (5, -10)]
    for (m, e) in params:
        rows.append((m + np.arange(g)) * 2.0 ** e)
    x = np.stack(rows).astype(np.float32)
    c, s, z = oracle.quantize_f32(x, g, bits)
    assert np.array_equal(unpack(c, bits), np.tile(np.arange(g, dtype=np.uint8), (len(params), 1)))
    assert np.array_equal(s[:, 0], np.array([2.0 ** e for _, e in params], np.float32))
    assert np.array_equal(z[:, 0], np.array([-m for m, _ in params], np.float32))
    assert np.array_equal(oracle.dequantize_f32(c, s, z, g, g, bits), x)
    # N identical partials, N a power of two: the two-step all-reduce returns exactly N*x
    x16 = x.astype(np.float16)
    assert np.array_equal(x16.astype(np.float32), x)
    for n in (1, 2, 4, 8):
        y = oracle.allreduce_sim(np.stack([x16] * n), g, bits, bits)
        assert np.array_equal(y.astype(np.float32), x * n)


def test_groups_run_along_hidden_and_meta_is_row_major():
    # 3 tokens x 2 groups, each group its own progression: scale 2^(t+2c), zero-point t+5c
    g = 16
    x = np.zeros((3, 2 * g), np.float32)
    for t in range(3):
        for c in range(2):
            x[t, c * g:(c + 1) * g] = (np.arange(g) - (t + 5 * c)) * 2.0 ** (t + 2 * c)
    cds, s, z = oracle.quantize_f32(x, g, 4)
    assert s.shape == (3, 2) and cds.shape == (3, g)
    for t in range(3):
        for c in range(2):
            assert s[t, c] == 2.0 ** (t + 2 * c) and z[t, c] == t + 5 * c
    assert np.array_equal(unpack(cds, 4), np.tile(np.arange(g, dtype=np.uint8), (3, 2)))


# --------------------------------------------------------------------------- #
# the reduce: exact rational arithmetic pins the fused-multiply-add chain
# --------------------------------------------------------------------------- #

def rn32(v: Fraction) -> np.float32:
    """Correctly rounded (nearest, ties to even) binary32 of a rational, normal range."""
    if v == 0:
        return F32(0.0)
    sign = -1 if v < 0 else 1
    a = abs(v)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    assert Fraction(2) ** e <= a < Fraction(2) ** (e + 1) and -126 <= e <= 127
    scaled = a / Fraction(2) ** (e - 23)
    n = scaled.numerator // scaled.denominator
    rem = scaled - n
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (n & 1)):
        n += 1
    return F32(sign * float(n) * 2.0 ** (e - 23))


def rint_half_even(v: Fraction) -> int:
    n = v.numerator // v.denominator            # floor
    rem = v - n
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (n & 1)):
        n += 1
    return n


@pytest.mark.parametrize("bits", [4, 8])
def test_group_quantizer_follows_the_stated_fp32_operation_order(bits):
    # Every fp32 operation of Eq. 1-2 (under the readings in the oracle's header) is
    # replayed in exact rational arithmetic with an explicit round-to-nearest-even
    # after each step: s = RN(r / qmax), inv = RN(1 / s), z = -rint(RN(mn * inv)),
    # q = clamp(rint(RN(x * inv)) + z).  A fused product or a different rounding
    # of any step changes some code below; hand example W9 separates the per-group
    # reciprocal from a per-element divide.
    rng = np.random.default_rng(31 + bits)
    qmax = (1 << bits) - 1
    for trial in range(12):
        x = (rng.standard_normal(32) * rng.choice([0.3, 1.0, 11.0, 170.0])).astype(np.float32)
        if trial % 4 == 3:
            x = np.abs(x) + F32(2.0)
        q, s, z = oracle.quantize_group_f32(x, bits)
        fx = [Fraction(float(v)) for v in x]
        mn, mx = min(fx), max(fx)
        r = Fraction(float(rn32(mx - mn)))
        es = Fraction(float(rn32(r / qmax)))
        einv = Fraction(float(rn32(1 / es)))
        ez = -rint_half_even(Fraction(float(rn32(mn * einv))))
        assert Fraction(float(s)) == es and int(z) == ez
        for k, v in enumerate(fx):
            t = rint_half_even(Fraction(float(rn32(v * einv)))) if v != 0 else 0
            assert int(q[k]) == min(max(t + ez, 0), qmax), (trial, k)


def test_reduce_is_an_fma_chain_in_source_order():
    rng = np.random.default_rng(19)
    n_src, g = 3, 32
    x = (rng.standard_normal((n_src, 4, g)) * np.array([1.0, 7.3, 0.11])[:, None, None]).astype(np.float16)
    parts = [oracle.quantize(x[j], g, 8) for j in range(n_src)]
    c = np.stack([p[0] for p in parts]); s = np.stack([p[1] for p in parts]); z = np.stack([p[2] for p in parts])
    acc = oracle.dequant_reduce_f32(c, s, z, g, g, 8)
    differs_from_mul_add = 0
    differs_from_reversed = 0
    for t in range(4):
        for k in range(g):
            a = Fraction(0)
            b = F32(0)
            for j in range(n_src):
                d = int(c[j, t, k]) - int(z[j, t, 0])
                a = Fraction(float(rn32(Fraction(d) * Fraction(float(s[j, t, 0])) + a)))
                b = F32(F32(d) * s[j, t, 0]) + b
            rv = Fraction(0)
            for j in reversed(range(n_src)):
                d = int(c[j, t, k]) - int(z[j, t, 0])
                rv = Fraction(float(rn32(Fraction(d) * Fraction(float(s[j, t, 0])) + rv)))
            assert bits_of(acc[t, k]) == bits_of(F32(float(a))), (t, k)
            differs_from_mul_add += int(F32(b).tobytes() != F32(acc[t, k]).tobytes())
            differs_from_reversed += int(float(rv) != float(a))
    # the case set really separates the readings
    assert differs_from_mul_add > 0 and differs_from_reversed > 0


def test_each_source_uses_its_own_scale_and_zero():
    # 4-bit progressions of 16 values: both sources are exact, with different (s, z)
    g = 16
    a = ((np.arange(g) - 3) * 0.5).astype(np.float32)[None, :]
    b = ((np.arange(g)[::-1] + 40) * 4.0).astype(np.float32)[None, :]
    pa = oracle.quantize_f32(a, g, 4); pb = oracle.quantize_f32(b, g, 4)
    assert pa[1][0, 0] == 0.5 and pa[2][0, 0] == 3 and pb[1][0, 0] == 4.0 and pb[2][0, 0] == -40
    c = np.stack([pa[0], pb[0]]); s = np.stack([pa[1], pb[1]]); z = np.stack([pa[2], pb[2]])
    assert np.array_equal(oracle.dequant_reduce_f32(c, s, z, g, g, 4), a + b)


# --------------------------------------------------------------------------- #
# brute force: the two-step all-reduce against the unquantized sum
# --------------------------------------------------------------------------- #

@pytest.mark.parametrize("bits_rs,bits_ag", [(8, 8), (4, 4), (4, 8)])
@pytest.mark.parametrize("n_src", [1, 2, 4, 8])
def test_allreduce_error_bound_against_exact_sum(bits_rs, bits_ag, n_src):
    # Section 3.2.1: the first quantization adds only rounding error (<= s_j/2 per source),
    # the second adds its own rounding on top of the accumulated error (<= s'/2).
    g, t, h = 128, 6, 1024
    x = synth_inputs.make_partials(n_src, t, h, seed=100 + n_src)
    exact = x.astype(np.float64).sum(0)
    parts = [oracle.quantize(x[j], g, bits_rs) for j in range(n_src)]
    c = np.stack([p[0] for p in parts]); s = np.stack([p[1] for p in parts]); z = np.stack([p[2] for p in parts])
    co, so, zo = oracle.dequant_reduce_requant(c, s, z, h, g, bits_rs, bits_ag)
    y = oracle.allreduce_sim(x, g, bits_rs, bits_ag)
    assert np.array_equal(y.view(np.uint16), oracle.dequantize(co, so, zo, h, g, bits_ag).view(np.uint16))
    bound = 0.5 * (s.astype(np.float64).sum(0) + so.astype(np.float64))          # per group
    bound = np.repeat(bound, g, axis=1) * (1 + 1e-5)
    y64 = y.astype(np.float64)
    half_ulp16 = np.maximum(np.abs(y64), 2.0 ** -14) * 2.0 ** -11
    assert np.all(np.abs(y64 - exact) <= bound + half_ulp16)
    # and the bound is not vacuous: the result is far closer to the sum than the data scale
    assert np.abs(y64 - exact).mean() < 0.6 * bound.mean()
    if bits_rs == 8 and bits_ag == 8:
        rel = np.abs(y64 - exact).mean() / np.abs(exact).mean()
        assert rel < 0.05


def test_single_source_reduce_equals_dequantize():
    x = synth_inputs.make_partials(1, 4, 512, seed=2)
    c, s, z = oracle.quantize(x[0], 64, 4)
    acc = oracle.dequant_reduce_f32(c[None], s[None], z[None], 512, 64, 4)
    assert np.array_equal(bits_of(acc), bits_of(oracle.dequantize_f32(c, s, z, 512, 64, 4)))


# --------------------------------------------------------------------------- #
# library cross-check (INT8, zero-point inside [0,255]): torch's affine quantizer
# --------------------------------------------------------------------------- #

def test_int8_codes_match_torch_quantize_per_tensor():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(23)
    x = rng.standard_normal((16, 128)).astype(np.float32) * 3
    c, s, z = oracle.quantize_f32(x, 128, 8)
    checked = 0
    for t in range(16):
        zp = int(z[t, 0])
        if not 0 <= zp <= 255:
            continue
        q = torch.quantize_per_tensor(torch.from_numpy(x[t]), float(s[t, 0]), zp, torch.quint8)
        assert np.array_equal(q.int_repr().numpy(), c[t])
        assert np.array_equal(bits_of(q.dequantize().numpy()),
                              bits_of(oracle.dequantize_f32(c[t:t + 1], s[t:t + 1], z[t:t + 1], 128, 128, 8)[0]))
        checked += 1
    assert checked >= 12


def test_bad_arguments_are_rejected():
    x = np.zeros((2, 96), np.float16)
    with pytest.raises(ValueError):
        oracle.quantize(x, 64, 8)          # hidden not a multiple of group
    with pytest.raises(ValueError):
        oracle.quantize(x, 32, 5)          # unsupported bit-width
    c, s, z = oracle.quantize(x, 32, 8)
    assert c.shape == (2, 96) and s.shape == (2, 3)
    e = oracle.quantize(np.zeros((0, 64), np.float16), 32, 4)
    assert e[0].shape == (0, 32)
