"""GPU parity of the symmetric entry points (Appendix Eq. 3-4: signed codes, no
zero-point) against the CPU oracle, bit for bit, through the C ABI.  Run with
``-m gpu`` on an MI355X."""
import numpy as np
import pytest

import oracle
import synth_inputs
from test_gpu_parity import (Guarded, SHAPES, assert_f16, dev, first_diff, groups_for, same_bits,
                             fc)  # noqa: F401  (fc is the module-scoped fixture)

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def gpu_quantize_sym(fc, x16, group, bits):
    t, h = x16.shape
    c = Guarded((t, h * bits // 8), torch.uint8)
    s = Guarded((t, h // group), torch.float32)
    fc.quantize_sym(dev(x16.view(np.uint16)).view(torch.float16), group, bits, out=(c.t, s.t))
    torch.cuda.synchronize()
    c.check(); s.check()
    return c.t.cpu().numpy(), s.t.cpu().numpy()


def gpu_fused_sym(fc, c, s, hidden, group, bits_in, bits_out):
    t = c.shape[1]
    co = Guarded((t, hidden * bits_out // 8), torch.uint8)
    so = Guarded((t, hidden // group), torch.float32)
    fc.dequant_reduce_requant_sym(dev(c), dev(s), hidden, group, bits_in, bits_out, out=(co.t, so.t))
    torch.cuda.synchronize()
    co.check(); so.check()
    return co.t.cpu().numpy(), so.t.cpu().numpy()


def gpu_dequantize_sym(fc, c, s, hidden, group, bits):
    y = Guarded((c.shape[0], hidden), torch.float16)
    fc.dequantize_sym(dev(c), dev(s), hidden, group, bits, out=y.t)
    torch.cuda.synchronize()
    y.check()
    return y.t.cpu().numpy()


def assert_pair(got, want, what):
    for name, g, w in zip(("codes", "scales"), got, want):
        assert same_bits(g, w), "%s %s: %s" % (what, name, first_diff(g, w))


def oracle_stage1_sym(x, group, bits):
    parts = [oracle.quantize_sym(x[j], group, bits) for j in range(x.shape[0])]
    return tuple(np.stack([p[i] for p in parts]) for i in range(2))


# --------------------------------------------------------------------------- #
# fc_quantize_sym
# --------------------------------------------------------------------------- #

@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("shape", SHAPES)
def test_quantize_sym_matches_oracle(fc, bits, shape):
    t, h = shape
    x = synth_inputs.make_partials(1, t, h, seed=t + h + 1, outlier_frac=0.01)[0]
    for group in groups_for(h):
        assert_pair(gpu_quantize_sym(fc, x, group, bits), oracle.quantize_sym(x, group, bits),
                    "quantize_sym %s g=%d b=%d" % (shape, group, bits))


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("group", [32, 64, 128, 256])
def test_quantize_sym_adversarial_groups(fc, bits, group):
    # all-zero groups (scale 1), float16 extremes, subnormal-only groups, exact .5 ties
    x = synth_inputs.adversarial_groups(group, seed=group + 3)
    want = oracle.quantize_sym(x, group, bits)
    assert (want[1] == 1.0).any()
    assert_pair(gpu_quantize_sym(fc, x, group, bits), want, "adversarial g=%d b=%d" % (group, bits))


# --------------------------------------------------------------------------- #
# fc_dequant_reduce_requant_sym
# --------------------------------------------------------------------------- #

@pytest.mark.parametrize("bits_in,bits_out", [(4, 4), (8, 8), (4, 8), (8, 4)])
@pytest.mark.parametrize("n_src", [1, 2, 3, 4, 5, 6, 7, 8])
def test_fused_sym_matches_oracle(fc, bits_in, bits_out, n_src):
    for (t, h) in [(16, 4096), (3, 1056), (7, 2080)]:
        x = synth_inputs.make_partials(n_src, t, h, seed=20 * n_src + bits_in)
        for group in groups_for(h)[:4]:
            c, s = oracle_stage1_sym(x, group, bits_in)
            want = oracle.dequant_reduce_requant_sym(c, s, h, group, bits_in, bits_out)
            got = gpu_fused_sym(fc, c, s, h, group, bits_in, bits_out)
            assert_pair(got, want, "fused_sym N=%d %dx%d g=%d %d->%d" % (n_src, t, h, group, bits_in, bits_out))


@pytest.mark.parametrize("bits_in,bits_out", [(4, 4), (8, 8), (4, 8)])
def test_fused_sym_large_groups(fc, bits_in, bits_out):
    t, h = 5, 8192
    x = synth_inputs.make_partials(3, t, h, seed=78)
    for group in (256, 512, 1024):
        c, s = oracle_stage1_sym(x, group, bits_in)
        want = oracle.dequant_reduce_requant_sym(c, s, h, group, bits_in, bits_out)
        assert_pair(gpu_fused_sym(fc, c, s, h, group, bits_in, bits_out), want, "fused_sym g=%d" % group)


@pytest.mark.parametrize("bits_in", [4, 8])
def test_fused_sym_arbitrary_codes_and_scales(fc, bits_in):
    # every code value of the field, including the most negative one the quantizer
    # itself never emits (-8 / -128), under scales spread over many binades
    rng = np.random.default_rng(6)
    n_src, t, h, group = 4, 6, 4096, 128
    c = rng.integers(0, 256, size=(n_src, t, h * bits_in // 8), dtype=np.uint8)
    c[0, 0, :64] = 0x88 if bits_in == 4 else 0x80
    s = np.exp(rng.uniform(-12, 8, size=(n_src, t, h // group))).astype(np.float32)
    for bits_out in (4, 8):
        want = oracle.dequant_reduce_requant_sym(c, s, h, group, bits_in, bits_out)
        assert_pair(gpu_fused_sym(fc, c, s, h, group, bits_in, bits_out), want,
                    "arbitrary codes %d->%d" % (bits_in, bits_out))


LADDER = np.array([1.4e-45, 1e-42, 1e-40, 1.1754944e-38, 1.2e-38, 1e-30, 1.0, 1e30, 2.0 ** 100, 2.0 ** 101, 1e35],
                  np.float32)


def extreme_scales(rng, shape):
    """per-group scales from the smallest subnormal to 1e35, with some rows uniform"""
    s = LADDER[rng.integers(0, LADDER.size, size=shape)]
    s[:, 0] = LADDER[0]; s[:, 1] = LADDER[3]; s[:, 2] = LADDER[8]; s[:, 3] = LADDER[10]
    s[0, 4] = LADDER[9]; s[-1, 4] = LADDER[1]
    return s


@pytest.mark.parametrize("bits_in", [4, 8])
def test_fused_sym_extreme_scales(fc, bits_in):
    # sums that are subnormal or vanish (scale 1) and output scales beyond 2^100 (the reciprocal's slow branch)
    rng = np.random.default_rng(25)
    n_src, t, h, group = 2, 9, 2048, 128
    c = rng.integers(0, 256, size=(n_src, t, h * bits_in // 8), dtype=np.uint8)
    s = extreme_scales(rng, (n_src, t, h // group))
    for bits_out in (4, 8):
        want = oracle.dequant_reduce_requant_sym(c, s, h, group, bits_in, bits_out)
        assert np.isfinite(want[1]).all() and (want[1] > 2.0 ** 100).any() and (want[1] == 1.0).any()
        assert_pair(gpu_fused_sym(fc, c, s, h, group, bits_in, bits_out), want, "extreme scales %d->%d" % (bits_in, bits_out))
        y = oracle.dequantize_sym(*want, h, group, bits_out)
        got = gpu_dequantize_sym(fc, *want, h, group, bits_out)
        assert same_bits(got.view(np.uint16), y.view(np.uint16)), "extreme scales, dequantize_sym"


def test_fused_sym_cancelling_sums(fc):
    # x + (-x): the codes are exact negatives, so what the fused multiply-adds leave is the rounding
    # error of the first product q*s (or an exact zero): sums some 2^-24 below the inputs
    group = 128
    a = synth_inputs.adversarial_groups(group, seed=4)
    x = np.stack([a, (-a.astype(np.float32)).astype(np.float16), a[::-1].copy()])
    for bits in (4, 8):
        c, s = oracle_stage1_sym(x, group, bits)
        want2 = oracle.dequant_reduce_requant_sym(c[:2], s[:2], a.shape[1], group, bits, bits)
        assert (want2[1] == 1.0).any() and (want2[1] < 1e-3).any()
        assert_pair(gpu_fused_sym(fc, c[:2], s[:2], a.shape[1], group, bits, bits), want2, "x + (-x)")
        want3 = oracle.dequant_reduce_requant_sym(c, s, a.shape[1], group, bits, bits)
        assert_pair(gpu_fused_sym(fc, c, s, a.shape[1], group, bits, bits), want3, "three sources")


def test_fused_sym_source_stride_with_padding(fc):
    n_src, t, h, group, bits = 3, 4, 2048, 128, 4
    x = synth_inputs.make_partials(n_src, t, h, seed=10)
    c, s = oracle_stage1_sym(x, group, bits)
    want = oracle.dequant_reduce_requant_sym(c, s, h, group, bits, bits)
    cp = torch.zeros((n_src, t + 2, h // 2), dtype=torch.uint8, device="cuda")
    sp = torch.zeros((n_src, t + 1, h // group), dtype=torch.float32, device="cuda")
    cp[:, :t] = dev(c); sp[:, :t] = dev(s)
    co = torch.empty((t, h // 2), dtype=torch.uint8, device="cuda")
    so = torch.empty((t, h // group), dtype=torch.float32, device="cuda")
    rc = fc.lib().fc_dequant_reduce_requant_sym(cp.data_ptr(), cp.stride(0), sp.data_ptr(), sp.stride(0),
                                                n_src, t, h, group, bits, bits, co.data_ptr(),
                                                so.data_ptr(), torch.cuda.current_stream().cuda_stream)
    assert rc == 0
    torch.cuda.synchronize()
    assert_pair((co.cpu().numpy(), so.cpu().numpy()), want, "padded stride")


# --------------------------------------------------------------------------- #
# fc_dequantize_sym, fc_allreduce_sim_sym
# --------------------------------------------------------------------------- #

@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("shape", [(16, 4096), (3, 1056), (7, 2080)])
def test_dequantize_sym_matches_oracle(fc, bits, shape):
    t, h = shape
    x = synth_inputs.make_partials(1, t, h, seed=4)[0]
    for group in groups_for(h)[:4]:
        c, s = oracle.quantize_sym(x, group, bits)
        want = oracle.dequantize_sym(c, s, h, group, bits)
        got = gpu_dequantize_sym(fc, c, s, h, group, bits)
        assert_f16(got, want, np.repeat(s, group, axis=1), "dequantize_sym %s g=%d b=%d" % (shape, group, bits))


@pytest.mark.parametrize("bits", [4, 8])
def test_dequantize_sym_extremes(fc, bits):
    # every code value under scales from subnormal-producing to overflowing
    rng = np.random.default_rng(9)
    t, h, group = 5, 2048, 128
    c = rng.integers(0, 256, size=(t, h * bits // 8), dtype=np.uint8)
    s = np.exp(rng.uniform(-30, 12, size=(t, h // group))).astype(np.float32)
    want = oracle.dequantize_sym(c, s, h, group, bits)
    got = gpu_dequantize_sym(fc, c, s, h, group, bits)
    assert same_bits(got.view(np.uint16), want.view(np.uint16)), first_diff(got.view(np.uint16), want.view(np.uint16))
    assert np.isinf(want.astype(np.float32)).any() and (want.view(np.uint16) & 0x7C00 == 0).any()


@pytest.mark.parametrize("bits_rs,bits_ag", [(8, 8), (4, 4), (4, 8)])
@pytest.mark.parametrize("n_src", [2, 4, 8])
def test_allreduce_sim_sym_matches_oracle(fc, bits_rs, bits_ag, n_src):
    t, h, group = 9, 4096, 128
    x = synth_inputs.make_partials(n_src, t, h, seed=n_src + 50)
    want = oracle.allreduce_sim_sym(x, group, bits_rs, bits_ag)
    y = Guarded((t, h), torch.float16)
    fc.allreduce_sim_sym(dev(x.view(np.uint16)).view(torch.float16), group, bits_rs, bits_ag, out=y.t)
    torch.cuda.synchronize(); y.check()
    got = y.t.cpu().numpy()
    assert same_bits(got.view(np.uint16), want.view(np.uint16)), first_diff(got.view(np.uint16), want.view(np.uint16))


def test_sym_empty_input_is_a_noop(fc):
    x = torch.empty((0, 4096), dtype=torch.float16, device="cuda")
    c, s = fc.quantize_sym(x, 128, 4)
    assert c.shape == (0, 2048) and s.shape == (0, 32)
    y = fc.allreduce_sim_sym(torch.empty((4, 0, 4096), dtype=torch.float16, device="cuda"), 128, 4, 4)
    assert y.shape == (0, 4096)
    torch.cuda.synchronize()


@pytest.mark.parametrize("name", ["llama3_8b_prefill", "llama3_70b_prefill"])
def test_sym_full_size_configs_on_sampled_rows(fc, name):
    w = synth_inputs.WORKLOADS[name]
    x = synth_inputs.make_partials_device(w.n_src, w.tokens, w.hidden, w.seed + 1, "cuda",
                                          w.outlier_frac, w.outlier_gain)
    rows = np.unique(np.concatenate([[0, 1, w.tokens - 1],
                                     np.random.default_rng(2).integers(0, w.tokens, 61)]))
    ridx = torch.from_numpy(rows).cuda()
    stage1 = [fc.quantize_sym(x[j], w.group, w.bits_in) for j in range(w.n_src)]
    c = torch.stack([p[0] for p in stage1]); s = torch.stack([p[1] for p in stage1])
    co, so = fc.dequant_reduce_requant_sym(c, s, w.hidden, w.group, w.bits_in, w.bits_out)
    y = fc.dequantize_sym(co, so, w.hidden, w.group, w.bits_out)
    y2 = fc.allreduce_sim_sym(x, w.group, w.bits_in, w.bits_out)
    torch.cuda.synchronize()
    assert torch.equal(y.view(torch.int16), y2.view(torch.int16))

    xs = x[:, ridx].cpu().numpy()
    oc, os_ = oracle_stage1_sym(xs, w.group, w.bits_in)
    assert_pair((c[:, ridx].cpu().numpy(), s[:, ridx].cpu().numpy()), (oc, os_), name + " stage 1")
    want = oracle.dequant_reduce_requant_sym(oc, os_, w.hidden, w.group, w.bits_in, w.bits_out)
    assert_pair((co[ridx].cpu().numpy(), so[ridx].cpu().numpy()), want, name + " fused")
    wy = oracle.dequantize_sym(*want, w.hidden, w.group, w.bits_out)
    assert_f16(y[ridx].cpu().numpy(), wy, np.repeat(want[1], w.group, axis=1), name + " output")
    assert bool((so > 0).all()) and bool(torch.isfinite(so).all())
