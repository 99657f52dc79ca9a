"""Pins for the oracle's asymmetric quantizer with binary16 metadata (Eq. 1-2 with the group's
scale and zero-point stored in 4 bytes): hand-worked groups (tests/golden/hand_groups_cmeta.txt),
reduction to the fp32-metadata functions wherever both numbers fit binary16, numpy's own binary16
rounding, exact-rational replay of the operation order, invariants and the two-step error bound.
CPU only."""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
import synth_inputs
from test_oracle_pins import (_datasets, bits_of, from_bits, parse_values, rint_half_even, rn32, unpack)

F32 = np.float32
F16 = np.float16


def load_golden_cmeta(golden_dir):
    groups, reds = {}, {}
    with open(os.path.join(golden_dir, "hand_groups_cmeta.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            f = [c.strip() for c in line.split("|")]
            if f[0].startswith("C"):
                groups[f[0]] = dict(bits=int(f[1]), x=parse_values(f[2]), meta=int(f[3], 16),
                                    codes=np.array(f[4].split(), dtype=np.uint8), xhat=from_bits(f[5].split()))
            else:
                reds[f[0]] = dict(bits_in=int(f[1]), bits_out=int(f[2]), sources=f[3].split(),
                                  acc=np.array(f[4].split(), dtype=np.float32), meta=int(f[5], 16),
                                  codes=np.array(f[6].split(), dtype=np.uint8), xhat=from_bits(f[7].split()),
                                  half=np.array([int(w, 16) for w in f[8].split()], dtype=np.uint16))
    assert len(groups) == 13 and len(reds) == 2
    return groups, reds


def half_rne_saturating(v, lo_floor=False):
    """numpy's binary16 rounding of fp32 values, with the oracle's two fix-ups."""
    with np.errstate(over="ignore"):
        h = np.asarray(v, F32).astype(F16)
    h = np.where(np.isinf(h), np.sign(h) * F16(65504), h).astype(F16)
    if lo_floor:
        h = np.where(h == 0, F16(2.0 ** -24), h).astype(F16)
    return h


def test_hand_groups_cmeta(golden_dir):
    groups, _ = load_golden_cmeta(golden_dir)
    for name, g in groups.items():
        q, m = oracle.quantize_group_cmeta_f32(g["x"], g["bits"])
        assert m == g["meta"], (name, hex(m))
        assert np.array_equal(q, g["codes"]), name
        n = g["x"].size
        c, mm = oracle.quantize_cmeta_f32(g["x"][None, :], n, g["bits"])
        assert np.array_equal(unpack(c, g["bits"])[0], g["codes"]) and int(mm[0, 0]) == g["meta"], name
        xh = oracle.dequantize_cmeta_f32(c, mm, n, n, g["bits"])
        assert np.array_equal(bits_of(xh[0]), bits_of(g["xhat"])), name


def test_hand_reduction_cmeta(golden_dir):
    groups, reds = load_golden_cmeta(golden_dir)
    for name, r in reds.items():
        srcs = [groups[s] for s in r["sources"]]
        n = srcs[0]["x"].size
        parts = [oracle.quantize_cmeta_f32(s["x"][None, :], n, r["bits_in"]) for s in srcs]
        c = np.stack([p[0] for p in parts]); m = np.stack([p[1] for p in parts])
        acc = oracle.dequant_reduce_cmeta_f32(c, m, n, n, r["bits_in"])
        assert np.array_equal(bits_of(acc[0]), bits_of(r["acc"])), name
        co, mo = oracle.dequant_reduce_requant_cmeta(c, m, n, n, r["bits_in"], r["bits_out"])
        assert np.array_equal(unpack(co, r["bits_out"])[0], r["codes"]) and int(mo[0, 0]) == r["meta"], name
        xh = oracle.dequantize_cmeta_f32(co, mo, n, n, r["bits_out"])
        assert np.array_equal(bits_of(xh[0]), bits_of(r["xhat"])), name
        x16 = np.stack([s_["x"][None, :] for s_ in srcs]).astype(F16)
        y = oracle.allreduce_sim_cmeta(x16, n, r["bits_in"], r["bits_out"])
        assert np.array_equal(y[0].view(np.uint16), r["half"]), name


def _exact_meta_inputs(rng, t, h, group, bits):
    """Groups whose Eq. 1 scale is a power of two and whose zero-point is a small integer."""
    qmax = (1 << bits) - 1
    k = rng.integers(0, qmax + 1, size=(t, h // group, group))
    k[..., 0] = 0
    k[..., 1] = qmax
    k = rng.permuted(k, axis=-1)
    z0 = rng.integers(0, qmax + 1, size=(t, h // group, 1))
    e = rng.integers(-6, 3, size=(t, h // group, 1))
    return ((k - z0) * 2.0 ** e).reshape(t, h).astype(F32), z0[..., 0], e[..., 0]


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("group", [32, 128])
def test_cmeta_reduces_to_fp32_metadata_when_scale_and_zero_fit_binary16(bits, group):
    rng = np.random.default_rng(bits * group)
    x, z0, e = _exact_meta_inputs(rng, 6, 512, group, bits)
    c, s, z = oracle.quantize_f32(x, group, bits)
    assert np.array_equal(s, (2.0 ** e).astype(F32)) and np.array_equal(z, z0.astype(F32))
    cc, m = oracle.quantize_cmeta_f32(x, group, bits)
    ms, mz = oracle.meta_unpack(m)
    assert np.array_equal(cc, c) and np.array_equal(ms, s) and np.array_equal(mz, z)
    assert np.array_equal(oracle.dequantize_cmeta_f32(cc, m, 512, group, bits), x)
    # binary16 input, several identical partials: the sums keep power-of-two scales
    x16 = x.astype(F16)
    assert np.array_equal(x16.astype(F32), x)
    for n in (1, 2, 4, 8):
        xs = np.stack([x16] * n)
        y = oracle.allreduce_sim_cmeta(xs, group, bits, bits)
        assert np.array_equal(y.view(np.uint16), oracle.allreduce_sim(xs, group, bits, bits).view(np.uint16))
        assert np.array_equal(y.astype(F32), x * n)


@pytest.mark.parametrize("bits", [4, 8])
def test_cmeta_decoders_equal_the_fp32_metadata_decoders_on_the_unpacked_numbers(bits):
    # Dequantize and the N-way reduction only read the stored numbers: with the halves widened by
    # numpy they must agree bit for bit with the fp32-metadata functions (pinned on their own)
    rng = np.random.default_rng(90 + bits)
    n_src, t, h, g = 3, 5, 512, 64
    c = rng.integers(0, 256, size=(n_src, t, h * bits // 8), dtype=np.uint8)
    sh = rng.integers(1, 0x7C00, size=(n_src, t, h // g)).astype(np.uint32)             # positive finite
    zh = rng.integers(0, 0x7C00, size=(n_src, t, h // g)).astype(np.uint32) | \
        (rng.integers(0, 2, size=(n_src, t, h // g)).astype(np.uint32) << 15)
    zh[0, 0, :4] = [0x0000, 0x7BFF, 0xFBFF, 0x3555]                                     # 0, +-65504, a non-integer
    m = sh | (zh << 16)
    s, z = oracle.meta_unpack(m)
    assert np.all(np.isfinite(s)) and np.all(s > 0) and np.all(np.isfinite(z))
    for j in range(n_src):
        assert np.array_equal(bits_of(oracle.dequantize_cmeta_f32(c[j], m[j], h, g, bits)),
                              bits_of(oracle.dequantize_f32(c[j], s[j], z[j], h, g, bits)))
        assert np.array_equal(oracle.dequantize_cmeta(c[j], m[j], h, g, bits).view(np.uint16),
                              oracle.dequantize(c[j], s[j], z[j], h, g, bits).view(np.uint16))
    assert np.array_equal(bits_of(oracle.dequant_reduce_cmeta_f32(c, m, h, g, bits)),
                          bits_of(oracle.dequant_reduce_f32(c, s, z, h, g, bits)))


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("group", [32, 128, 1024])
def test_cmeta_scale_is_numpy_binary16_of_the_eq1_scale(bits, group):
    for name, x in _datasets():
        _, s32, _ = oracle.quantize_f32(x, group, bits)
        _, m = oracle.quantize_cmeta_f32(x, group, bits)
        want = half_rne_saturating(s32, lo_floor=True).view(np.uint16)
        assert np.array_equal((m & 0xFFFF).astype(np.uint16), want), name
        ms, mz = oracle.meta_unpack(m)
        assert np.all(ms > 0) and np.all(np.isfinite(ms)) and np.all(np.abs(mz) <= 65504), name


@pytest.mark.parametrize("bits", [4, 8])
def test_cmeta_operation_order_replayed_in_exact_arithmetic(bits):
    # given the stored scale: inv = RN(1/s16), z = half(-rint(RN(mn*inv))), q = clamp(rint(RN(x*inv)) + z16)
    rng = np.random.default_rng(51 + bits)
    qmax = (1 << bits) - 1
    big_z = 0
    for trial in range(16):
        x = (rng.standard_normal(32) * rng.choice([0.3, 1.0, 11.0, 170.0])).astype(F32)
        if trial % 4 == 3:
            x = np.abs(rng.standard_normal(32)).astype(F32) + F32([2.0, 900.0, 30000.0, 4000.0][trial // 4])          # zero-points beyond 2048 and beyond 65504
        q, m = oracle.quantize_group_cmeta_f32(x, bits)
        fx = [Fraction(float(v)) for v in x]
        mn, mx = min(fx), max(fx)
        s32 = rn32(Fraction(float(rn32(mx - mn))) / qmax)
        s16 = half_rne_saturating(s32, lo_floor=True)
        assert (m & 0xFFFF) == int(s16.view(np.uint16))
        es = Fraction(float(s16))
        einv = Fraction(float(rn32(1 / es)))
        z_exact = -rint_half_even(Fraction(float(rn32(mn * einv))))
        z16 = half_rne_saturating(F32(float(z_exact)))
        assert (m >> 16) == int(z16.view(np.uint16)), trial
        ez = Fraction(float(z16))
        big_z += int(abs(z_exact) > 2048)
        for k, v in enumerate(fx):
            t = rint_half_even(Fraction(float(rn32(v * einv)))) if v != 0 else 0
            assert int(q[k]) == min(max(t + ez, 0), qmax), (trial, k)
    assert big_z >= 3


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("group", [32, 128, 1024])
def test_cmeta_invariants(bits, group):
    qmax = (1 << bits) - 1
    for name, x in _datasets():
        t, h = x.shape
        c, m = oracle.quantize_cmeta_f32(x, group, bits)
        s, z = oracle.meta_unpack(m)
        q = unpack(c, bits).reshape(t, h // group, group)
        xg = x.reshape(t, h // group, group)
        assert q.max() <= qmax and np.array_equal(z, np.rint(z)), name
        # groups whose scale is a normal binary16 number and whose zero-point is exact in binary16
        _, s32, z32 = oracle.quantize_f32(x, group, bits)
        const = xg.max(-1) == xg.min(-1)
        plain = (s32 >= 2.0 ** -14) & (s32 <= 65504) & (np.abs(z) <= 2048) & ~const
        if not plain.any():
            continue
        amin = xg.argmin(-1)[..., None]
        assert np.all(np.take_along_axis(q, amin, -1)[..., 0][plain] == 0), name
        assert np.all(np.abs(s.astype(np.float64) - s32)[plain] <= s32[plain] * 2.0 ** -11), name
        # half a step of rounding, plus what the top of the range loses when the rounded scale is too small
        xh = oracle.dequantize_cmeta_f32(c, m, h, group, bits).reshape(xg.shape)
        err = np.abs(xh.astype(np.float64) - xg.astype(np.float64))
        lim = s.astype(np.float64) * (0.5 + qmax * 2.0 ** -11) * (1.0 + 2.0 ** -18 * (np.abs(z) + qmax + 4))
        assert np.all(err[plain] <= lim[plain][..., None]), name
        order = np.argsort(xg, axis=-1, kind="stable")
        qs = np.take_along_axis(q, order, -1).astype(np.int32)
        assert np.all(np.diff(qs, axis=-1) >= 0), name
    # constant groups of binary16 values reconstruct exactly (R5: s = |min| is a binary16 number)
    v = np.repeat(np.array([[0.0, 2.5, -0.375, 65504.0, -6.1e-5, 5.96e-8]], F16).astype(F32), group, axis=1)
    c, m = oracle.quantize_cmeta_f32(v, group, bits)
    assert np.array_equal(oracle.dequantize_cmeta_f32(c, m, v.shape[1], group, bits), v)


@pytest.mark.parametrize("bits", [4, 8])
def test_cmeta_power_of_two_scaling(bits):
    rng = np.random.default_rng(13)
    x = rng.standard_normal((6, 512)).astype(F32)
    c0, m0 = oracle.quantize_cmeta_f32(x, 128, bits)
    s0, z0 = oracle.meta_unpack(m0)
    for k in (-8, -3, 5, 11):                    # scales stay normal binary16 numbers
        c, m = oracle.quantize_cmeta_f32(x * F32(2.0 ** k), 128, bits)
        s, z = oracle.meta_unpack(m)
        assert np.array_equal(c, c0) and np.array_equal(z, z0) and np.array_equal(s, s0 * F32(2.0 ** k)), k


@pytest.mark.parametrize("bits_rs,bits_ag", [(8, 8), (4, 4), (4, 8)])
@pytest.mark.parametrize("n_src", [1, 2, 4, 8])
def test_cmeta_allreduce_error_bound(bits_rs, bits_ag, n_src):
    g, t, h = 128, 6, 1024
    x = synth_inputs.make_partials(n_src, t, h, seed=300 + n_src)
    exact = x.astype(np.float64).sum(0)
    parts = [oracle.quantize_cmeta(x[j], g, bits_rs) for j in range(n_src)]
    c = np.stack([p[0] for p in parts]); m = np.stack([p[1] for p in parts])
    co, mo = oracle.dequant_reduce_requant_cmeta(c, m, h, g, bits_rs, bits_ag)
    y = oracle.allreduce_sim_cmeta(x, g, bits_rs, bits_ag)
    assert np.array_equal(y.view(np.uint16), oracle.dequantize_cmeta(co, mo, h, g, bits_ag).view(np.uint16))
    s, _ = oracle.meta_unpack(m)
    so, _ = oracle.meta_unpack(mo)
    step = lambda sc, b: sc.astype(np.float64) * (0.5 + ((1 << b) - 1) * 2.0 ** -11)
    bound = np.repeat(step(s, bits_rs).sum(0) + step(so, bits_ag), g, axis=1) * (1 + 1e-5)
    y64 = y.astype(np.float64)
    assert np.all(np.abs(y64 - exact) <= bound + np.maximum(np.abs(y64), 2.0 ** -14) * 2.0 ** -11)
    assert np.abs(y64 - exact).mean() < 0.6 * bound.mean()
    # and it stays close to the fp32-metadata scheme: same order of error
    y32 = oracle.allreduce_sim(x, g, bits_rs, bits_ag).astype(np.float64)
    e16, e32 = np.abs(y64 - exact).mean(), np.abs(y32 - exact).mean()
    assert 0.8 * e32 <= e16 <= 1.25 * e32


def test_cmeta_layout_and_bad_arguments():
    x = synth_inputs.make_partials(1, 3, 256, seed=8)[0]
    c, m = oracle.quantize_cmeta(x, 64, 4)
    assert c.shape == (3, 128) and m.shape == (3, 4) and m.dtype == np.uint32
    for t in range(3):                            # row-major metadata, groups along hidden
        for gi in range(4):
            q, w = oracle.quantize_group_cmeta_f32(x[t, 64 * gi:64 * gi + 64].astype(F32), 4)
            assert w == int(m[t, gi]) and np.array_equal(unpack(c[t:t + 1], 4)[0, 64 * gi:64 * gi + 64], q)
    with pytest.raises(ValueError):
        oracle.quantize_cmeta(np.zeros((2, 96), F16), 64, 8)
    with pytest.raises(ValueError):
        oracle.quantize_cmeta(np.zeros((2, 96), F16), 32, 5)
    e = oracle.quantize_cmeta(np.zeros((0, 64), F16), 32, 4)
    assert e[0].shape == (0, 32) and e[1].shape == (0, 2)
