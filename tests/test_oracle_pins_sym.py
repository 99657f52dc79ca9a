"""Pins for the oracle's symmetric quantizer (Appendix Eq. 3-4): hand-worked groups
(tests/golden/hand_groups_sym.txt), exact-rational replay of the fp32 operation order, invariants,
closed forms, the two-step error bound, and torch's qint8 quantizer.  CPU only."""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
import synth_inputs
from test_oracle_pins import bits_of, from_bits, parse_values, rn32, rint_half_even

F32 = np.float32


def load_golden_sym(golden_dir):
    groups, reds = {}, {}
    with open(os.path.join(golden_dir, "hand_groups_sym.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            f = [c.strip() for c in line.split("|")]
            if f[0].startswith("S"):
                groups[f[0]] = dict(bits=int(f[1]), x=parse_values(f[2]), scale=from_bits([f[3]])[0],
                                    codes=np.array(f[4].split(), dtype=np.int8),
                                    packed=np.array([int(b, 16) for b in f[5].split()], dtype=np.uint8),
                                    xhat=from_bits(f[6].split()))
            else:
                reds[f[0]] = dict(bits_in=int(f[1]), bits_out=int(f[2]), sources=f[3].split(),
                                  acc=np.array(f[4].split(), dtype=np.float32), scale=from_bits([f[5]])[0],
                                  codes=np.array(f[6].split(), dtype=np.int8), xhat=from_bits(f[7].split()))
    assert len(groups) == 7 and len(reds) == 2
    return groups, reds


def unpack_signed(codes, bits):
    codes = np.asarray(codes, np.uint8)
    if bits == 8:
        return codes.view(np.int8).copy()
    out = np.empty(codes.shape[:-1] + (codes.shape[-1] * 2,), np.int8)
    lo = (codes & 0x0F).astype(np.int16); hi = (codes >> 4).astype(np.int16)
    out[..., 0::2] = np.where(lo >= 8, lo - 16, lo)
    out[..., 1::2] = np.where(hi >= 8, hi - 16, hi)
    return out


def test_hand_groups_sym(golden_dir):
    groups, _ = load_golden_sym(golden_dir)
    for name, g in groups.items():
        q, s = oracle.quantize_group_sym_f32(g["x"], g["bits"])
        assert np.array_equal(q, g["codes"]), name
        assert bits_of(s) == bits_of(g["scale"]), name
        n = g["x"].size
        c, ss = oracle.quantize_sym_f32(g["x"][None, :], n, g["bits"])
        assert np.array_equal(c[0], g["packed"]), name            # two's complement, low nibble first
        xh = oracle.dequantize_sym_f32(c, ss, n, n, g["bits"])
        assert np.array_equal(bits_of(xh[0]), bits_of(g["xhat"])), name


def test_hand_reduction_sym(golden_dir):
    groups, reds = load_golden_sym(golden_dir)
    for name, r in reds.items():
        srcs = [groups[s] for s in r["sources"]]
        n = srcs[0]["x"].size
        parts = [oracle.quantize_sym_f32(s["x"][None, :], n, r["bits_in"]) for s in srcs]
        c = np.stack([p[0] for p in parts]); s = np.stack([p[1] for p in parts])
        acc = oracle.dequant_reduce_sym_f32(c, s, n, n, r["bits_in"])
        assert np.array_equal(bits_of(acc[0]), bits_of(r["acc"])), name
        co, so = oracle.dequant_reduce_requant_sym(c, s, n, n, r["bits_in"], r["bits_out"])
        assert np.array_equal(unpack_signed(co, r["bits_out"])[0], r["codes"]), name
        assert bits_of(so)[0, 0] == bits_of(r["scale"]), name
        xh = oracle.dequantize_sym_f32(co, so, n, n, r["bits_out"])
        assert np.array_equal(bits_of(xh[0]), bits_of(r["xhat"])), name
        x16 = np.stack([s_["x"][None, :] for s_ in srcs]).astype(np.float16)
        y = oracle.allreduce_sim_sym(x16, n, r["bits_in"], r["bits_out"])
        assert np.array_equal(y[0].view(np.uint16), r["xhat"].astype(np.float16).view(np.uint16)), name


@pytest.mark.parametrize("bits", [4, 8])
def test_sym_operation_order_replayed_in_exact_arithmetic(bits):
    rng = np.random.default_rng(41 + bits)
    qm = (1 << (bits - 1)) - 1
    for trial in range(10):
        x = (rng.standard_normal(32) * rng.choice([0.3, 1.0, 11.0, 170.0])).astype(np.float32)
        q, s = oracle.quantize_group_sym_f32(x, bits)
        fx = [Fraction(float(v)) for v in x]
        amax = max(abs(v) for v in fx)
        es = Fraction(float(rn32(amax / qm)))
        einv = Fraction(float(rn32(1 / es)))
        assert Fraction(float(s)) == es
        for k, v in enumerate(fx):
            t = rint_half_even(Fraction(float(rn32(v * einv)))) if v != 0 else 0
            assert int(q[k]) == min(max(t, -qm - 1), qm), (trial, k)


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("group", [32, 128, 1024])
def test_sym_invariants(bits, group):
    qm = (1 << (bits - 1)) - 1
    rng = np.random.default_rng(group + bits)
    data = [rng.standard_normal((16, 1024)).astype(np.float32),
            synth_inputs.make_partials(1, 16, 1024, seed=3)[0].astype(np.float32),
            (np.abs(rng.standard_normal((8, 1024))) + 3).astype(np.float32),
            synth_inputs.adversarial_groups(128).astype(np.float32)]
    for x in data:
        t, h = x.shape
        c, s = oracle.quantize_sym_f32(x, group, bits)
        q = unpack_signed(c, bits).reshape(t, h // group, group).astype(np.int32)
        xg = x.reshape(t, h // group, group)
        assert q.max() <= qm and q.min() >= -qm            # -2^(n-1) is never produced
        assert np.all(s > 0)
        amax_idx = np.abs(xg).argmax(-1)[..., None]
        top = np.take_along_axis(q, amax_idx, -1)[..., 0]
        zero = np.abs(xg).max(-1) == 0
        assert np.all(np.abs(top[~zero]) == qm) and np.all(q[zero] == 0)
        xh = oracle.dequantize_sym_f32(c, s, h, group, bits).reshape(xg.shape)
        assert np.all(np.abs(xh.astype(np.float64) - xg) <= 0.5 * s.astype(np.float64)[..., None] * (1 + 1e-5))
        # odd symmetry: quantizing -x negates every code and keeps the scale
        c2, s2 = oracle.quantize_sym_f32(-x, group, bits)
        assert np.array_equal(unpack_signed(c2, bits).astype(np.int32), -unpack_signed(c, bits).astype(np.int32))
        assert np.array_equal(bits_of(s2), bits_of(s))
        # power-of-two scaling leaves the codes alone
        c3, s3 = oracle.quantize_sym_f32(x * F32(8.0), group, bits)
        assert np.array_equal(c3, c)
        assert np.array_equal(bits_of(s3)[~zero], bits_of(s * F32(8.0))[~zero]) and np.all(s3[zero] == 1)


def test_sym_progression_is_exact_and_sums_exactly():
    # x_k = k * 2^e for k = -qm..qm: s = 2^e, codes k, exact round trip; 2^m identical partials sum exactly
    for bits in (4, 8):
        qm = (1 << (bits - 1)) - 1
        g = 2 * qm + 2
        k = np.concatenate([np.arange(-qm, qm + 1), [0]])
        x = np.stack([k * 2.0 ** e for e in (-3, 0, 5)]).astype(np.float32)
        c, s = oracle.quantize_sym_f32(x, g, bits)
        assert np.array_equal(unpack_signed(c, bits), np.tile(k.astype(np.int8), (3, 1)))
        assert np.array_equal(s[:, 0], np.array([2.0 ** e for e in (-3, 0, 5)], np.float32))
        assert np.array_equal(oracle.dequantize_sym_f32(c, s, g, g, bits), x)
        x16 = x.astype(np.float16)
        for n in (1, 2, 4, 8):
            y = oracle.allreduce_sim_sym(np.stack([x16] * n), g, bits, bits)
            assert np.array_equal(y.astype(np.float32), x * n)


@pytest.mark.parametrize("bits_rs,bits_ag", [(8, 8), (4, 4), (4, 8)])
@pytest.mark.parametrize("n_src", [1, 2, 4, 8])
def test_sym_allreduce_error_bound(bits_rs, bits_ag, n_src):
    g, t, h = 128, 6, 1024
    x = synth_inputs.make_partials(n_src, t, h, seed=200 + n_src)
    exact = x.astype(np.float64).sum(0)
    parts = [oracle.quantize_sym(x[j], g, bits_rs) for j in range(n_src)]
    c = np.stack([p[0] for p in parts]); s = np.stack([p[1] for p in parts])
    co, so = oracle.dequant_reduce_requant_sym(c, s, h, g, bits_rs, bits_ag)
    y = oracle.allreduce_sim_sym(x, g, bits_rs, bits_ag)
    assert np.array_equal(y.view(np.uint16), oracle.dequantize_sym(co, so, h, g, bits_ag).view(np.uint16))
    bound = np.repeat(0.5 * (s.astype(np.float64).sum(0) + so), g, axis=1) * (1 + 1e-5)
    y64 = y.astype(np.float64)
    assert np.all(np.abs(y64 - exact) <= bound + np.maximum(np.abs(y64), 2.0 ** -14) * 2.0 ** -11)
    assert np.abs(y64 - exact).mean() < 0.6 * bound.mean()


def test_sym_reduce_is_an_fma_chain_in_source_order():
    rng = np.random.default_rng(77)
    n_src, g = 3, 32
    x = (rng.standard_normal((n_src, 4, g)) * np.array([1.0, 7.3, 0.11])[:, None, None]).astype(np.float16)
    parts = [oracle.quantize_sym(x[j], g, 8) for j in range(n_src)]
    c = np.stack([p[0] for p in parts]); s = np.stack([p[1] for p in parts])
    q = unpack_signed(c, 8)
    acc = oracle.dequant_reduce_sym_f32(c, s, g, g, 8)
    differs = 0
    for t in range(4):
        for k in range(g):
            a = Fraction(0); b = F32(0)
            for j in range(n_src):
                a = Fraction(float(rn32(Fraction(int(q[j, t, k])) * Fraction(float(s[j, t, 0])) + a)))
                b = F32(F32(int(q[j, t, k])) * s[j, t, 0]) + b
            assert F32(float(a)).tobytes() == F32(acc[t, k]).tobytes(), (t, k)
            differs += int(F32(b).tobytes() != F32(acc[t, k]).tobytes())
    assert differs > 0


def test_sym_int8_matches_torch_qint8():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(5)
    x = rng.standard_normal((12, 128)).astype(np.float32) * 2
    c, s = oracle.quantize_sym_f32(x, 128, 8)
    for t in range(12):
        q = torch.quantize_per_tensor(torch.from_numpy(x[t]), float(s[t, 0]), 0, torch.qint8)
        assert np.array_equal(q.int_repr().numpy(), c[t].view(np.int8))
