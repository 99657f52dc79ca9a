"""Pins for the oracle's FP8 (E4M3) per-group symmetric variant: the format against torch's
float8_e4m3fn and a nearest-value search, hand-worked groups (tests/golden/hand_groups_fp8.txt),
exact-rational replay of the fp32 operation order, invariants, closed forms and the two-step error
bound.  CPU only."""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
import synth_inputs
from test_oracle_pins import bits_of, from_bits, parse_values, rn32

F32 = np.float32
torch = pytest.importorskip("torch")

# the 127 non-negative finite E4M3 numbers, straight from the format's definition
# (sign, 4 exponent bits with bias 7, 3 fraction bits; e = 0 subnormal; 1111.111 is NaN)
E4M3 = []
for _c in range(127):
    _e, _m = _c >> 3, _c & 7
    E4M3.append(Fraction(_m, 512) if _e == 0 else Fraction(8 + _m, 8) * Fraction(2) ** (_e - 7))


def nearest_e4m3(v: Fraction) -> int:
    """code of the nearest E4M3 number to the exact value v; ties to the even fraction; saturating"""
    sign = 0x80 if v < 0 else 0
    a = abs(v)
    if a >= 448:
        return sign | 0x7E
    best, code = None, None
    for c, r in enumerate(E4M3):
        d = abs(r - a)
        if best is None or d < best or (d == best and c % 2 == 0):
            best, code = d, c
    return sign | code


def load_golden_fp8(golden_dir):
    groups, reds = {}, {}
    with open(os.path.join(golden_dir, "hand_groups_fp8.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            f = [c.strip() for c in line.split("|")]
            if f[0].startswith("P"):
                groups[f[0]] = dict(x=parse_values(f[1]), scale=from_bits([f[2]])[0],
                                    codes=np.array([int(b, 16) for b in f[3].split()], dtype=np.uint8),
                                    xhat=from_bits(f[4].split()))
            else:
                reds[f[0]] = dict(sources=f[1].split(), acc=np.array(f[2].split(), dtype=np.float32),
                                  scale=from_bits([f[3]])[0],
                                  codes=np.array([int(b, 16) for b in f[4].split()], dtype=np.uint8),
                                  xhat=from_bits(f[5].split()))
    assert len(groups) == 7 and len(reds) == 1
    return groups, reds


def test_e4m3_decode_all_codes_against_torch_and_the_format():
    codes = np.arange(256, dtype=np.uint8)
    got = np.array([oracle.e4m3_to_float(int(c)) for c in codes], dtype=np.float32)
    want = torch.from_numpy(codes).view(torch.float8_e4m3fn).to(torch.float32).numpy()
    ok = ~np.isnan(want)
    assert np.array_equal(bits_of(got[ok]), bits_of(want[ok]))
    assert np.isnan(got[0x7F]) and np.isnan(got[0xFF]) and np.isnan(want[0x7F])
    # facts of the format: largest value, smallest normal, smallest subnormal, no infinities
    assert got[0x7E] == 448.0 and got[0x08] == 2.0 ** -6 and got[0x01] == 2.0 ** -9
    assert not np.isinf(got).any() and bits_of(got[0x80]) == 0x80000000
    for c in range(127):
        assert Fraction(float(got[c])) == E4M3[c] and got[c | 0x80] == -got[c]


def test_e4m3_encode_against_nearest_value_search_and_torch():
    rng = np.random.default_rng(0)
    # every binary16 value in range, every tie between neighbours and the fp32 numbers next to it,
    # and random fp32 values over the whole range
    h = np.arange(65536, dtype=np.uint16).view(np.float16).astype(np.float32)
    h = h[np.isfinite(h) & (np.abs(h) <= 448)]
    ties = np.array([float((a + b) / 2) for a, b in zip(E4M3, E4M3[1:])], dtype=np.float32)
    near = np.concatenate([ties, np.nextafter(ties, F32(0)), np.nextafter(ties, F32(1e9))])
    rnd = (rng.standard_normal(60000) * np.exp(rng.uniform(-9, 6, 60000))).astype(np.float32)
    rnd = rnd[np.abs(rnd) <= 448]
    x = np.concatenate([h, near, -near, rnd, np.array([0.0, -0.0, 448.0, -448.0], np.float32)])
    got = np.array([oracle.float_to_e4m3(float(v)) for v in x], dtype=np.uint8)
    want_t = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(got, want_t)
    sample = np.concatenate([near, -near, rnd[:3000], h[::37]])
    for v in sample:
        c = oracle.float_to_e4m3(float(v))
        want = nearest_e4m3(Fraction(float(v)))
        if v == 0 or want & 0x7F == 0:
            want = (0x80 if np.signbit(v) else 0) | (want & 0x7F)      # the sign of a zero result is the input's
        assert c == want, (float(v), hex(c), hex(want))
    # saturation beyond the largest value (cannot occur inside the quantizer)
    for v in (448.5, 464.0, 500.0, 3e38):
        assert oracle.float_to_e4m3(v) == 0x7E and oracle.float_to_e4m3(-v) == 0xFE


def test_e4m3_round_trip_and_monotone():
    for c in range(256):
        if c & 0x7F == 0x7F:
            continue
        assert oracle.float_to_e4m3(oracle.e4m3_to_float(c)) == c
    xs = np.sort(np.concatenate([np.linspace(-460, 460, 20001), np.linspace(-0.05, 0.05, 4001)])).astype(np.float32)
    v = np.array([oracle.e4m3_to_float(oracle.float_to_e4m3(float(a))) for a in xs])
    assert np.all(np.diff(v) >= 0)
    big = np.abs(xs) >= 2.0 ** -6
    assert np.all(np.abs(v - xs)[big & (np.abs(xs) <= 448)] <= np.abs(xs)[big & (np.abs(xs) <= 448)] / 16 * (1 + 1e-6))
    assert np.all(np.abs(v - xs)[~big] <= 2.0 ** -10)


def test_hand_groups_fp8(golden_dir):
    groups, _ = load_golden_fp8(golden_dir)
    for name, g in groups.items():
        q, s = oracle.quantize_group_fp8_f32(g["x"])
        assert np.array_equal(q, g["codes"]), name
        assert bits_of(s) == bits_of(g["scale"]), name
        n = g["x"].size
        c, ss = oracle.quantize_fp8_f32(g["x"][None, :], n)
        assert np.array_equal(c[0], g["codes"]), name
        xh = oracle.dequantize_fp8_f32(c, ss, n, n)
        assert np.array_equal(bits_of(xh[0]), bits_of(g["xhat"])), name


def test_hand_reduction_fp8(golden_dir):
    groups, reds = load_golden_fp8(golden_dir)
    for name, r in reds.items():
        srcs = [groups[s] for s in r["sources"]]
        n = srcs[0]["x"].size
        parts = [oracle.quantize_fp8_f32(s["x"][None, :], n) for s in srcs]
        c = np.stack([p[0] for p in parts]); s = np.stack([p[1] for p in parts])
        acc = oracle.dequant_reduce_fp8_f32(c, s, n, n)
        assert np.array_equal(bits_of(acc[0]), bits_of(r["acc"])), name
        co, so = oracle.dequant_reduce_requant_fp8(c, s, n, n)
        assert np.array_equal(co[0], r["codes"]), name
        assert bits_of(so)[0, 0] == bits_of(r["scale"]), name
        xh = oracle.dequantize_fp8_f32(co, so, n, n)
        assert np.array_equal(bits_of(xh[0]), bits_of(r["xhat"])), name
        x16 = np.stack([s_["x"][None, :] for s_ in srcs]).astype(np.float16)
        y = oracle.allreduce_sim_fp8(x16, n)
        assert np.array_equal(y[0].view(np.uint16), r["xhat"].astype(np.float16).view(np.uint16)), name


def test_fp8_operation_order_replayed_in_exact_arithmetic():
    rng = np.random.default_rng(43)
    for trial in range(12):
        x = (rng.standard_normal(32) * rng.choice([0.3, 1.0, 11.0, 170.0])).astype(np.float32)
        q, s = oracle.quantize_group_fp8_f32(x)
        fx = [Fraction(float(v)) for v in x]
        amax = max(abs(v) for v in fx)
        es = Fraction(float(rn32(amax / 448)))
        einv = Fraction(float(rn32(1 / es)))
        assert Fraction(float(s)) == es
        for k, v in enumerate(fx):
            assert int(q[k]) == nearest_e4m3(Fraction(float(rn32(v * einv)))), (trial, k)
    # the reduction: fused multiply-add chain in source order from +0, each source's own scale
    c = rng.integers(0, 256, size=(3, 1, 64), dtype=np.uint8)
    c[(c & 0x7F) == 0x7F] = 0x12
    s = np.exp(rng.uniform(-3, 3, size=(3, 1, 2))).astype(np.float32)
    acc = oracle.dequant_reduce_fp8_f32(c, s, 64, 32)
    for h in range(64):
        a = Fraction(0)
        for j in range(3):
            sign = -1 if c[j, 0, h] & 0x80 else 1
            a = Fraction(float(rn32(sign * E4M3[c[j, 0, h] & 0x7F] * Fraction(float(s[j, 0, h // 32])) + a)))
        assert Fraction(float(acc[0, h])) == a, h


@pytest.mark.parametrize("group", [32, 128, 1024])
def test_fp8_invariants(group):
    rng = np.random.default_rng(group)
    data = [rng.standard_normal((16, 1024)).astype(np.float32),
            synth_inputs.make_partials(1, 16, 1024, seed=3)[0].astype(np.float32),
            synth_inputs.adversarial_groups(128).astype(np.float32)]
    for x in data:
        t, h = x.shape
        c, s = oracle.quantize_fp8_f32(x, group)
        assert not ((c & 0x7F) == 0x7F).any() and np.all(s > 0)
        xg = x.reshape(t, h // group, group)
        cg = c.reshape(xg.shape)
        amax_idx = np.abs(xg).argmax(-1)[..., None]
        top = np.take_along_axis(cg, amax_idx, -1)[..., 0]
        zero = np.abs(xg).max(-1) == 0
        assert np.all((top[~zero] & 0x7F) == 0x7E) and np.all((cg[zero] & 0x7F) == 0)   # max|x| -> +-448
        xh = oracle.dequantize_fp8_f32(c, s, h, group).reshape(xg.shape).astype(np.float64)
        # relative error 2^-4 per element, floored by the subnormal step 2^-10 * s
        bound = np.maximum(np.abs(xg) / 16, s.astype(np.float64)[..., None] * 2.0 ** -10) * (1 + 1e-5)
        assert np.all(np.abs(xh - xg) <= bound)
        # odd symmetry and power-of-two scaling
        c2, s2 = oracle.quantize_fp8_f32(-x, group)
        assert np.array_equal(c2 ^ 0x80, c) and np.array_equal(s2, s)
        c3, s3 = oracle.quantize_fp8_f32(x * F32(8), group)
        nz = ~zero
        assert np.array_equal(c3.reshape(cg.shape)[nz], cg[nz]) and np.array_equal(s3[nz], s[nz] * F32(8))


def test_fp8_closed_forms():
    # a group made of E4M3 numbers times a power of two that contains +-448*2^k is reproduced exactly
    vals = np.array([float(v) for v in E4M3], dtype=np.float32)
    rng = np.random.default_rng(5)
    x = rng.choice(vals, size=(4, 128)) * rng.choice([-1.0, 1.0], size=(4, 128))
    x[:, 0] = 448.0
    x = (x * F32(2.0 ** -5)).astype(np.float32)
    c, s = oracle.quantize_fp8_f32(x, 128)
    assert np.all(s == F32(2.0 ** -5))
    assert np.array_equal(bits_of(oracle.dequantize_fp8_f32(c, s, 128, 128)), bits_of(x))
    # 2^k identical partials of such a tensor all-reduce to exactly 2^k * x
    x16 = x.astype(np.float16)
    assert np.array_equal(x16.astype(np.float32), x)
    for n in (1, 2, 4, 8):
        y = oracle.allreduce_sim_fp8(np.stack([x16] * n), 128)
        assert np.array_equal(y.astype(np.float32), x * n)


@pytest.mark.parametrize("n_src", [2, 4, 8])
def test_fp8_allreduce_error_bound_against_exact_sum(n_src):
    # each stage is off by at most 2^-4 of the value (or the subnormal floor); sum the two stages' bounds
    group = 128
    x = synth_inputs.make_partials(n_src, 8, 1024, seed=9)
    y = oracle.allreduce_sim_fp8(x, group).astype(np.float64)
    exact = x.astype(np.float64).sum(0)
    parts = [oracle.quantize_fp8(x[j], group) for j in range(n_src)]
    s1 = np.stack([p[1] for p in parts]).astype(np.float64)
    s2 = oracle.dequant_reduce_requant_fp8(np.stack([p[0] for p in parts]), np.stack([p[1] for p in parts]),
                                           1024, group)[1].astype(np.float64)
    st1 = np.maximum(np.abs(x.astype(np.float64)) / 16, np.repeat(s1, group, axis=2) * 2.0 ** -10).sum(0)
    reduced = np.abs(exact) + st1
    st2 = np.maximum(reduced / 16, np.repeat(s2, group, axis=1) * 2.0 ** -10)
    bound = (st1 + st2) * (1 + 1e-3) + np.abs(y) * 2.0 ** -11
    assert np.all(np.abs(y - exact) <= bound)
    assert np.abs(y - exact).max() > 0


def test_fp8_single_source_reduce_equals_dequantize_and_bad_arguments():
    x = synth_inputs.make_partials(1, 4, 512, seed=2)[0]
    c, s = oracle.quantize_fp8(x, 64)
    acc = oracle.dequant_reduce_fp8_f32(c[None], s[None], 512, 64)
    assert np.array_equal(bits_of(acc), bits_of(oracle.dequantize_fp8_f32(c, s, 512, 64)))
    with pytest.raises(Exception):
        oracle.quantize_fp8(x, 96)


def test_fp8_dequantize_to_binary16_against_the_format_table_and_numpy():
    """The last step of the FP8 all-reduce (Appendix "FP8 and FP4 Format"; Algorithm 1, final Dequantize):
    every byte decoded by the format's definition, times the scale of ITS group (rows, groups and scales all
    different, so a wrong group or row index shows), one fp32 product, numpy's binary16 rounding."""
    rng = np.random.default_rng(11)
    t, h, g = 5, 384, 64
    codes = rng.integers(0, 256, size=(t, h), dtype=np.uint8)
    codes[(codes & 0x7F) == 0x7F] = 0x3C                               # the two NaN bytes are outside the domain
    scales = np.exp(rng.uniform(-9, 7, size=(t, h // g))).astype(F32)
    scales[1, 2] = F32(3.0e2)                                          # 448 * 300 overflows binary16
    scales[3, 0] = F32(2.0 ** -20)                                     # binary16 subnormals
    table = np.array([float(v) for v in E4M3] + [0.0], dtype=F32)      # index 127 unused
    val = table[codes & 0x7F] * np.where(codes & 0x80, F32(-1), F32(1))
    want32 = (val * np.repeat(scales, g, axis=1)).astype(F32)
    with np.errstate(over="ignore"):
        want16 = want32.astype(np.float16)
    got32 = oracle.dequantize_fp8_f32(codes, scales, h, g)
    assert np.array_equal(bits_of(got32), bits_of(want32))
    got16 = oracle.dequantize_fp8(codes, scales, h, g)
    assert got16.dtype == np.float16 and got16.shape == (t, h)
    assert np.array_equal(got16.view(np.uint16), want16.view(np.uint16))
    assert np.isinf(want16).any() and ((want16.view(np.uint16) & 0x7C00) == 0).any()
    # -0 bytes keep their sign through the product and the rounding
    z = np.full((1, 64), 0x80, np.uint8)
    assert (oracle.dequantize_fp8(z, np.ones((1, 1), F32), 64, 64).view(np.uint16) == 0x8000).all()
    # and the end-to-end function is the composition of the three pinned steps
    x = synth_inputs.make_partials(3, 4, 512, seed=9, outlier_frac=0.02)
    parts = [oracle.quantize_fp8(x[j], 128) for j in range(3)]
    c = np.stack([p[0] for p in parts]); s = np.stack([p[1] for p in parts])
    co, so = oracle.dequant_reduce_requant_fp8(c, s, 512, 128)
    assert np.array_equal(oracle.allreduce_sim_fp8(x, 128).view(np.uint16),
                          oracle.dequantize_fp8(co, so, 512, 128).view(np.uint16))
