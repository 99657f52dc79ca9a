"""GPU parity of the compact-metadata entry points (Eq. 1-2 with the group's scale and
zero-point stored as two binary16 numbers in one 32-bit word) against the CPU oracle, bit for
bit, through the C ABI.  Run with ``-m gpu`` on an MI355X."""
import numpy as np
import pytest

import oracle
import synth_inputs
from test_gpu_parity import (Guarded, SHAPES, assert_f16, dev, first_diff, groups_for, same_bits,
                             fc)  # noqa: F401  (fc is the module-scoped fixture)

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def dev_meta(m):
    return torch.from_numpy(np.ascontiguousarray(m, np.uint32).view(np.int32)).cuda()


def host_meta(t):
    return t.cpu().numpy().view(np.uint32)


def gpu_quantize_cmeta(fc, x16, group, bits):
    t, h = x16.shape
    c = Guarded((t, h * bits // 8), torch.uint8)
    m = Guarded((t, h // group), torch.int32)
    fc.quantize_cmeta(dev(x16.view(np.uint16)).view(torch.float16), group, bits, out=(c.t, m.t))
    torch.cuda.synchronize()
    c.check(); m.check()
    return c.t.cpu().numpy(), host_meta(m.t)


def gpu_fused_cmeta(fc, c, m, hidden, group, bits_in, bits_out):
    t = c.shape[1]
    co = Guarded((t, hidden * bits_out // 8), torch.uint8)
    mo = Guarded((t, hidden // group), torch.int32)
    fc.dequant_reduce_requant_cmeta(dev(c), dev_meta(m), hidden, group, bits_in, bits_out, out=(co.t, mo.t))
    torch.cuda.synchronize()
    co.check(); mo.check()
    return co.t.cpu().numpy(), host_meta(mo.t)


def gpu_dequantize_cmeta(fc, c, m, hidden, group, bits):
    y = Guarded((c.shape[0], hidden), torch.float16)
    fc.dequantize_cmeta(dev(c), dev_meta(m), hidden, group, bits, out=y.t)
    torch.cuda.synchronize()
    y.check()
    return y.t.cpu().numpy()


def assert_pair(got, want, what):
    for name, g, w in zip(("codes", "meta"), got, want):
        assert same_bits(g, w), "%s %s: %s" % (what, name, first_diff(g, w))


def oracle_stage1_cmeta(x, group, bits):
    parts = [oracle.quantize_cmeta(x[j], group, bits) for j in range(x.shape[0])]
    return tuple(np.stack([p[i] for p in parts]) for i in range(2))


def random_meta(rng, shape):
    """positive finite binary16 scales over all binades; zero-points: small integers, large ones, +-65504"""
    sh = rng.integers(1, 0x7C00, size=shape).astype(np.uint32)
    z = np.rint(rng.standard_normal(shape) * rng.choice([3.0, 40.0, 900.0, 30000.0], size=shape))
    zh = np.clip(z, -65504, 65504).astype(np.float16).view(np.uint16).astype(np.uint32)
    return sh | (zh << 16)


# --------------------------------------------------------------------------- #
# fc_quantize_cmeta
# --------------------------------------------------------------------------- #

@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("shape", SHAPES)
def test_quantize_cmeta_matches_oracle(fc, bits, shape):
    t, h = shape
    x = synth_inputs.make_partials(1, t, h, seed=t + h + 4, outlier_frac=0.01)[0]
    for group in groups_for(h):
        assert_pair(gpu_quantize_cmeta(fc, x, group, bits), oracle.quantize_cmeta(x, group, bits),
                    "quantize_cmeta %s g=%d b=%d" % (shape, group, bits))


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("group", [32, 64, 128, 256])
def test_quantize_cmeta_adversarial_groups(fc, bits, group):
    # constant groups, float16 extremes, subnormal-only groups (scale floored at 2^-24), exact .5 ties
    x = synth_inputs.adversarial_groups(group, seed=group + 7)
    want = oracle.quantize_cmeta(x, group, bits)
    assert ((want[1] & 0xFFFF) == 0x0001).any() or ((want[1] & 0xFFFF) < 0x0400).any()
    assert_pair(gpu_quantize_cmeta(fc, x, group, bits), want, "adversarial g=%d b=%d" % (group, bits))


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("kind", range(synth_inputs.STRESS_KINDS))
def test_quantize_cmeta_value_distributions(fc, bits, kind):
    # offsets far above the range (zero-points beyond 2048 and beyond 65504), near-degenerate groups, ties
    x = synth_inputs.make_partials_stress(1, 12, 4096, kind, seed=kind + 11)[0]
    for group in (32, 128, 1024, 4096):
        want = oracle.quantize_cmeta(x, group, bits)
        assert_pair(gpu_quantize_cmeta(fc, x, group, bits), want, "stress %d g=%d b=%d" % (kind, group, bits))


def test_quantize_cmeta_zero_point_ranges_are_reached(fc):
    # binary16 inputs with offsets: zero-points exact (<= 2048), rounded (2048..65504) and saturated
    rng = np.random.default_rng(21)
    base = rng.standard_normal((3, 16, 1024)).astype(np.float32)
    x = np.concatenate([base[0] * 0.05 + 1.0, base[1] * 0.05 + 60.0, base[2] * 0.01 + 3000.0]).astype(np.float16)
    for bits in (4, 8):
        want = oracle.quantize_cmeta(x, 128, bits)
        z = np.abs(oracle.meta_unpack(want[1])[1])
        assert (z <= 2048).any() and ((z > 2048) & (z < 65504)).any()
        assert bits == 4 or (z == 65504).any()        # 4-bit zero-points of binary16 data stay below 15 * 1024
        assert_pair(gpu_quantize_cmeta(fc, x, 128, bits), want, "zero-point ranges b=%d" % bits)


# --------------------------------------------------------------------------- #
# fc_dequant_reduce_requant_cmeta
# --------------------------------------------------------------------------- #

@pytest.mark.parametrize("bits_in,bits_out", [(4, 4), (8, 8), (4, 8), (8, 4)])
@pytest.mark.parametrize("n_src", [1, 2, 3, 4, 5, 6, 7, 8])
def test_fused_cmeta_matches_oracle(fc, bits_in, bits_out, n_src):
    for (t, h) in [(16, 4096), (3, 1056), (7, 2080)]:
        x = synth_inputs.make_partials(n_src, t, h, seed=40 * n_src + bits_in)
        for group in groups_for(h)[:4]:
            c, m = oracle_stage1_cmeta(x, group, bits_in)
            want = oracle.dequant_reduce_requant_cmeta(c, m, h, group, bits_in, bits_out)
            got = gpu_fused_cmeta(fc, c, m, h, group, bits_in, bits_out)
            assert_pair(got, want, "fused_cmeta N=%d %dx%d g=%d %d->%d" % (n_src, t, h, group, bits_in, bits_out))


@pytest.mark.parametrize("bits_in,bits_out", [(4, 4), (8, 8), (4, 8)])
def test_fused_cmeta_large_and_wide_groups(fc, bits_in, bits_out):
    for (t, h, groups) in [(5, 8192, (256, 512, 1024, 2048, 8192)), (2, 16384, (4096, 16384))]:
        for n_src in (1, 3, 8):
            x = synth_inputs.make_partials(n_src, t, h, seed=79 + n_src)
            for group in groups:
                c, m = oracle_stage1_cmeta(x, group, bits_in)
                assert_pair(gpu_quantize_cmeta(fc, x[0], group, bits_in), (c[0], m[0]), "quantize_cmeta g=%d" % group)
                want = oracle.dequant_reduce_requant_cmeta(c, m, h, group, bits_in, bits_out)
                assert_pair(gpu_fused_cmeta(fc, c, m, h, group, bits_in, bits_out), want,
                            "fused_cmeta N=%d h=%d g=%d" % (n_src, h, group))


@pytest.mark.parametrize("bits_in", [4, 8])
def test_fused_cmeta_arbitrary_codes_and_meta(fc, bits_in):
    # every code value under scales from every binary16 binade and zero-points of every size:
    # the fast and the general dequantization path, sums of every magnitude into the requantizer
    rng = np.random.default_rng(16)
    for (n_src, t, h, group) in [(4, 6, 4096, 128), (3, 5, 2048, 32), (5, 3, 4096, 1024), (2, 3, 8192, 8192)]:
        c = rng.integers(0, 256, size=(n_src, t, h * bits_in // 8), dtype=np.uint8)
        m = random_meta(rng, (n_src, t, h // group))
        for bits_out in (4, 8):
            want = oracle.dequant_reduce_requant_cmeta(c, m, h, group, bits_in, bits_out)
            assert_pair(gpu_fused_cmeta(fc, c, m, h, group, bits_in, bits_out), want,
                        "arbitrary N=%d g=%d %d->%d" % (n_src, group, bits_in, bits_out))
    # small zero-points only: the whole tile takes the fast path
    n_src, t, h, group = 4, 4, 4096, 128
    c = rng.integers(0, 256, size=(n_src, t, h * bits_in // 8), dtype=np.uint8)
    sh = rng.integers(0x0400, 0x7C00, size=(n_src, t, h // group)).astype(np.uint32)
    zh = rng.integers(-20, 300, size=(n_src, t, h // group)).astype(np.float16).view(np.uint16).astype(np.uint32)
    m = sh | (zh << 16)
    want = oracle.dequant_reduce_requant_cmeta(c, m, h, group, bits_in, 4)
    assert_pair(gpu_fused_cmeta(fc, c, m, h, group, bits_in, 4), want, "fast path")


@pytest.mark.parametrize("bits_out", [4, 8])
def test_fused_cmeta_zero_point_rounded_to_2048(fc, bits_out):
    # Sums whose Eq. 1 zero-point is +-2049 (stored as +-2048) or sits just around it: the minimum's code is then
    # rint(min/s) + 2048 = -1 and must be clamped, next to neighbours packed in the same word.  Two INT8 sources
    # with a power-of-two scale produce such sums exactly: the first spans the code range under a zero-point of
    # +-2040, the second is a constant that shifts the sum by a few steps.
    qmax = (1 << bits_out) - 1
    s_in = 0.25 if bits_out == 4 else 2.0 ** -6
    h, group = 4096, 128
    rng = np.random.default_rng(44)
    targets = (2049, 2048, 2047, 2050, 2051, -2049, -2048, -2050)
    c = np.zeros((2, len(targets), h), np.uint8)
    m = np.zeros((2, len(targets), h // group), np.uint32)
    half = lambda v: int(np.float16(v).view(np.uint16))
    for r, z_target in enumerate(targets):
        z1 = 2040 if z_target > 0 else -2040
        q = rng.integers(0, qmax + 1, size=h).astype(np.uint8)
        q[0::group] = 0                        # every group holds its minimum ...
        q[1::group] = 0                        # ... twice in one packed word ...
        q[5::group] = qmax                     # ... and its maximum
        c[0, r] = q
        m[0, r] = half(s_in) | (half(z1) << 16)
        m[1, r] = half(s_in) | (half(z_target - z1) << 16)      # codes 0: contributes -(z_target - z1) steps
    want = oracle.dequant_reduce_requant_cmeta(c, m, h, group, 8, bits_out)
    s_out, z_out = oracle.meta_unpack(want[1])
    assert (s_out == np.float32(s_in)).all()
    assert [float(v) for v in z_out[:, 0]] == [2048.0, 2048.0, 2047.0, 2050.0, 2052.0, -2048.0, -2048.0, -2050.0]
    assert_pair(gpu_fused_cmeta(fc, c, m, h, group, 8, bits_out), want, "zero-point around 2048, %d bit" % bits_out)


@pytest.mark.parametrize("kind", range(synth_inputs.STRESS_KINDS))
def test_fused_cmeta_value_distributions(fc, kind):
    rng = np.random.default_rng(60 + kind)
    for case in range(6):
        group = int(rng.choice([32, 128, 512, 2048]))
        hidden = group * int(rng.integers(1, max(2, 8192 // group) + 1))
        tokens, n_src = int(rng.integers(1, 6)), int(rng.integers(1, 9))
        bits_in, bits_out = int(rng.choice([4, 8])), int(rng.choice([4, 8]))
        x = synth_inputs.make_partials_stress(n_src, tokens, hidden, kind, seed=kind * 10 + case)
        c, m = oracle_stage1_cmeta(x, group, bits_in)
        what = "stress %d case %d: N=%d %dx%d g=%d %d->%d" % (kind, case, n_src, tokens, hidden, group, bits_in, bits_out)
        assert_pair(gpu_quantize_cmeta(fc, x[0], group, bits_in), (c[0], m[0]), what + " quantize")
        want = oracle.dequant_reduce_requant_cmeta(c, m, hidden, group, bits_in, bits_out)
        assert_pair(gpu_fused_cmeta(fc, c, m, hidden, group, bits_in, bits_out), want, what + " fused")
        wy = oracle.dequantize_cmeta(*want, hidden, group, bits_out)
        gy = gpu_dequantize_cmeta(fc, *want, hidden, group, bits_out)
        assert same_bits(gy.view(np.uint16), wy.view(np.uint16)), what + " dequantize"
        y = fc.allreduce_sim_cmeta(dev(x.view(np.uint16)).view(torch.float16), group, bits_in, bits_out)
        assert same_bits(y.cpu().numpy().view(np.uint16), wy.view(np.uint16)), what + " sim"


def test_fused_cmeta_source_stride_with_padding(fc):
    n_src, t, h, group, bits = 3, 4, 2048, 128, 4
    x = synth_inputs.make_partials(n_src, t, h, seed=13)
    c, m = oracle_stage1_cmeta(x, group, bits)
    want = oracle.dequant_reduce_requant_cmeta(c, m, h, group, bits, bits)
    cp = torch.zeros((n_src, t + 2, h // 2), dtype=torch.uint8, device="cuda")
    mp = torch.zeros((n_src, t + 1, h // group), dtype=torch.int32, device="cuda")
    cp[:, :t] = dev(c); mp[:, :t] = dev_meta(m)
    co = torch.empty((t, h // 2), dtype=torch.uint8, device="cuda")
    mo = torch.empty((t, h // group), dtype=torch.int32, device="cuda")
    rc = fc.lib().fc_dequant_reduce_requant_cmeta(cp.data_ptr(), cp.stride(0), mp.data_ptr(), mp.stride(0),
                                                  n_src, t, h, group, bits, bits, co.data_ptr(),
                                                  mo.data_ptr(), torch.cuda.current_stream().cuda_stream)
    assert rc == 0
    torch.cuda.synchronize()
    assert_pair((co.cpu().numpy(), host_meta(mo)), want, "padded stride")


# --------------------------------------------------------------------------- #
# fc_dequantize_cmeta, fc_allreduce_sim_cmeta
# --------------------------------------------------------------------------- #

@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("shape", [(16, 4096), (3, 1056), (7, 2080), (2, 16384)])
def test_dequantize_cmeta_matches_oracle(fc, bits, shape):
    t, h = shape
    x = synth_inputs.make_partials(1, t, h, seed=14)[0]
    for group in groups_for(h)[:4] + ([h] if h & (h - 1) == 0 else []):
        c, m = oracle.quantize_cmeta(x, group, bits)
        want = oracle.dequantize_cmeta(c, m, h, group, bits)
        got = gpu_dequantize_cmeta(fc, c, m, h, group, bits)
        s = oracle.meta_unpack(m)[0]
        assert_f16(got, want, np.repeat(s, group, axis=1), "dequantize_cmeta %s g=%d b=%d" % (shape, group, bits))


@pytest.mark.parametrize("bits", [4, 8])
def test_dequantize_cmeta_extremes(fc, bits):
    rng = np.random.default_rng(19)
    t, h, group = 5, 2048, 128
    c = rng.integers(0, 256, size=(t, h * bits // 8), dtype=np.uint8)
    m = random_meta(rng, (t, h // group))
    want = oracle.dequantize_cmeta(c, m, h, group, bits)
    got = gpu_dequantize_cmeta(fc, c, m, h, group, bits)
    assert same_bits(got.view(np.uint16), want.view(np.uint16)), first_diff(got.view(np.uint16), want.view(np.uint16))
    assert np.isinf(want.astype(np.float32)).any() and (want.view(np.uint16) & 0x7C00 == 0).any()


@pytest.mark.parametrize("bits_rs,bits_ag", [(8, 8), (4, 4), (4, 8)])
@pytest.mark.parametrize("n_src", [2, 4, 8])
def test_allreduce_sim_cmeta_matches_oracle(fc, bits_rs, bits_ag, n_src):
    for t, h, group in ((9, 4096, 128), (3, 4096, 4096), (130, 512, 64)):
        x = synth_inputs.make_partials(n_src, t, h, seed=n_src + 70)
        want = oracle.allreduce_sim_cmeta(x, group, bits_rs, bits_ag)
        y = Guarded((t, h), torch.float16)
        fc.allreduce_sim_cmeta(dev(x.view(np.uint16)).view(torch.float16), group, bits_rs, bits_ag, out=y.t)
        torch.cuda.synchronize(); y.check()
        got = y.t.cpu().numpy()
        assert same_bits(got.view(np.uint16), want.view(np.uint16)), first_diff(got.view(np.uint16), want.view(np.uint16))


def test_cmeta_empty_input_is_a_noop(fc):
    x = torch.empty((0, 4096), dtype=torch.float16, device="cuda")
    c, m = fc.quantize_cmeta(x, 128, 4)
    assert c.shape == (0, 2048) and m.shape == (0, 32)
    y = fc.allreduce_sim_cmeta(torch.empty((4, 0, 4096), dtype=torch.float16, device="cuda"), 128, 4, 4)
    assert y.shape == (0, 4096)
    torch.cuda.synchronize()


@pytest.mark.parametrize("name", ["llama3_8b_prefill", "llama3_70b_prefill"])
def test_cmeta_full_size_configs_on_sampled_rows(fc, name):
    w = synth_inputs.WORKLOADS[name]
    x = synth_inputs.make_partials_device(w.n_src, w.tokens, w.hidden, w.seed + 3, "cuda",
                                          w.outlier_frac, w.outlier_gain)
    rows = np.unique(np.concatenate([[0, 1, w.tokens - 1],
                                     np.random.default_rng(3).integers(0, w.tokens, 61)]))
    ridx = torch.from_numpy(rows).cuda()
    stage1 = [fc.quantize_cmeta(x[j], w.group, w.bits_in) for j in range(w.n_src)]
    c = torch.stack([p[0] for p in stage1]); m = torch.stack([p[1] for p in stage1])
    co, mo = fc.dequant_reduce_requant_cmeta(c, m, w.hidden, w.group, w.bits_in, w.bits_out)
    y = fc.dequantize_cmeta(co, mo, w.hidden, w.group, w.bits_out)
    y2 = fc.allreduce_sim_cmeta(x, w.group, w.bits_in, w.bits_out)
    torch.cuda.synchronize()
    assert torch.equal(y.view(torch.int16), y2.view(torch.int16))

    xs = x[:, ridx].cpu().numpy()
    oc, om = oracle_stage1_cmeta(xs, w.group, w.bits_in)
    assert_pair((c[:, ridx].cpu().numpy(), host_meta(m[:, ridx])), (oc, om), name + " stage 1")
    want = oracle.dequant_reduce_requant_cmeta(oc, om, w.hidden, w.group, w.bits_in, w.bits_out)
    assert_pair((co[ridx].cpu().numpy(), host_meta(mo[ridx])), want, name + " fused")
    wy = oracle.dequantize_cmeta(*want, w.hidden, w.group, w.bits_out)
    s = oracle.meta_unpack(want[1])[0]
    assert_f16(y[ridx].cpu().numpy(), wy, np.repeat(s, w.group, axis=1), name + " output")
    assert bool(((mo & 0x7FFF) > 0).all()) and bool(((mo & 0x7C00) != 0x7C00).all())     # positive finite scales
