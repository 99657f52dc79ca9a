"""GPU parity of the FP8 (E4M3) per-group symmetric entry points against the CPU
oracle, bit for bit, through the C ABI.  Run with ``-m gpu`` on an MI355X."""
import numpy as np
import pytest

import oracle
import synth_inputs
from test_gpu_parity import (Guarded, SHAPES, assert_f16, dev, first_diff, groups_for, same_bits,
                             fc)  # noqa: F401  (fc is the module-scoped fixture)
from test_gpu_parity_sym import assert_pair

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def gpu_quantize_fp8(fc, x16, group):
    t, h = x16.shape
    c = Guarded((t, h), torch.uint8)
    s = Guarded((t, h // group), torch.float32)
    fc.quantize_fp8(dev(x16.view(np.uint16)).view(torch.float16), group, out=(c.t, s.t))
    torch.cuda.synchronize()
    c.check(); s.check()
    return c.t.cpu().numpy(), s.t.cpu().numpy()


def gpu_fused_fp8(fc, c, s, hidden, group):
    t = c.shape[1]
    co = Guarded((t, hidden), torch.uint8)
    so = Guarded((t, hidden // group), torch.float32)
    fc.dequant_reduce_requant_fp8(dev(c), dev(s), hidden, group, out=(co.t, so.t))
    torch.cuda.synchronize()
    co.check(); so.check()
    return co.t.cpu().numpy(), so.t.cpu().numpy()


def gpu_dequantize_fp8(fc, c, s, hidden, group):
    y = Guarded((c.shape[0], hidden), torch.float16)
    fc.dequantize_fp8(dev(c), dev(s), hidden, group, out=y.t)
    torch.cuda.synchronize()
    y.check()
    return y.t.cpu().numpy()


def oracle_stage1_fp8(x, group):
    parts = [oracle.quantize_fp8(x[j], group) for j in range(x.shape[0])]
    return tuple(np.stack([p[i] for p in parts]) for i in range(2))


def finite_codes(rng, shape):
    c = rng.integers(0, 256, size=shape, dtype=np.uint8)
    c[(c & 0x7F) == 0x7F] = 0x7E           # NaN bytes are outside the domain
    return c


WIDE = [(5, 4096, 2048), (3, 4096, 4096), (3, 8192, 8192), (2, 16384, 16384)]


@pytest.mark.parametrize("shape", SHAPES)
def test_quantize_fp8_matches_oracle(fc, shape):
    t, h = shape
    x = synth_inputs.make_partials(1, t, h, seed=t + h + 2, outlier_frac=0.01)[0]
    for group in groups_for(h):
        assert_pair(gpu_quantize_fp8(fc, x, group), oracle.quantize_fp8(x, group),
                    "quantize_fp8 %s g=%d" % (shape, group))


@pytest.mark.parametrize("group", [32, 64, 128, 256])
def test_quantize_fp8_adversarial_groups(fc, group):
    # all-zero groups, float16 extremes and subnormals, negative zeros, values that round to +-0
    x = synth_inputs.adversarial_groups(group, seed=group + 5)
    x[0, 2 * group:2 * group + 8] = np.float16(-0.0)
    want = oracle.quantize_fp8(x, group)
    assert (want[1] == 1.0).any() and (want[0] == 0x80).any()
    assert_pair(gpu_quantize_fp8(fc, x, group), want, "adversarial g=%d" % group)


def test_quantize_fp8_every_float16_value(fc):
    # every finite binary16 pattern, in groups whose scale is 1 (an element of 448 in each group)
    h = np.arange(65536, dtype=np.uint16).view(np.float16)
    h = h[np.isfinite(h) & (np.abs(h.astype(np.float32)) <= 448)]
    group, per = 32, 31
    rows = -(-h.size // per)
    body = np.zeros(rows * per, np.float16)
    body[:h.size] = h
    x = np.empty((rows, group), np.float16)
    x[:, 0] = 448.0
    x[:, 1:] = body.reshape(rows, per)
    x = x.reshape(1, rows * group)
    want = oracle.quantize_fp8(x, group)
    assert (want[1] == 1.0).all()
    assert_pair(gpu_quantize_fp8(fc, x, group), want, "all binary16 values")


@pytest.mark.parametrize("n_src", [1, 2, 3, 4, 5, 6, 7, 8])
def test_fused_fp8_matches_oracle(fc, n_src):
    for (t, h) in [(16, 4096), (3, 1056), (7, 2080)]:
        x = synth_inputs.make_partials(n_src, t, h, seed=30 * n_src)
        for group in groups_for(h)[:4]:
            c, s = oracle_stage1_fp8(x, group)
            want = oracle.dequant_reduce_requant_fp8(c, s, h, group)
            assert_pair(gpu_fused_fp8(fc, c, s, h, group), want,
                        "fused_fp8 N=%d %dx%d g=%d" % (n_src, t, h, group))


def test_fused_fp8_arbitrary_codes_and_scales(fc):
    # every finite byte value (subnormals, -0, +-448) under scales spread over many binades:
    # the requantizer then sees fp32 sums of every magnitude
    rng = np.random.default_rng(7)
    for n_src, t, h, group in ((4, 6, 4096, 128), (1, 9, 2048, 64), (3, 4, 4096, 1024)):
        c = finite_codes(rng, (n_src, t, h))
        s = np.exp(rng.uniform(-12, 8, size=(n_src, t, h // group))).astype(np.float32)
        want = oracle.dequant_reduce_requant_fp8(c, s, h, group)
        assert_pair(gpu_fused_fp8(fc, c, s, h, group), want, "arbitrary codes N=%d g=%d" % (n_src, group))


def test_fused_fp8_extreme_scales(fc):
    from test_gpu_parity_sym import extreme_scales
    rng = np.random.default_rng(26)
    n_src, t, h, group = 2, 9, 2048, 128
    c = finite_codes(rng, (n_src, t, h))
    s = extreme_scales(rng, (n_src, t, h // group))
    want = oracle.dequant_reduce_requant_fp8(c, s, h, group)
    assert np.isfinite(want[1]).all() and (want[1] > 2.0 ** 100).any() and (want[1] == 1.0).any()
    assert_pair(gpu_fused_fp8(fc, c, s, h, group), want, "extreme scales")
    y = oracle.dequantize_fp8(*want, h, group)
    got = gpu_dequantize_fp8(fc, *want, h, group)
    assert same_bits(got.view(np.uint16), y.view(np.uint16)), "extreme scales, dequantize_fp8"


def test_fused_fp8_wide_groups_and_padding(fc):
    for (t, h, g) in WIDE:
        for n_src in (1, 4, 8):
            x = synth_inputs.make_partials(n_src, t, h, seed=n_src + g + 1)
            c, s = oracle_stage1_fp8(x, g)
            assert_pair(gpu_quantize_fp8(fc, x[0], g), (c[0], s[0]), "quantize_fp8 wide %s" % ((t, h, g),))
            want = oracle.dequant_reduce_requant_fp8(c, s, h, g)
            assert_pair(gpu_fused_fp8(fc, c, s, h, g), want, "fused_fp8 wide N=%d %s" % (n_src, (t, h, g)))
    # sources separated by more than one slab
    n_src, t, h, group = 3, 4, 2048, 128
    x = synth_inputs.make_partials(n_src, t, h, seed=12)
    c, s = oracle_stage1_fp8(x, group)
    want = oracle.dequant_reduce_requant_fp8(c, s, h, group)
    cp = torch.zeros((n_src, t + 2, h), dtype=torch.uint8, device="cuda")
    sp = torch.zeros((n_src, t + 1, h // group), dtype=torch.float32, device="cuda")
    cp[:, :t] = dev(c); sp[:, :t] = dev(s)
    co = torch.empty((t, h), dtype=torch.uint8, device="cuda")
    so = torch.empty((t, h // group), dtype=torch.float32, device="cuda")
    rc = fc.lib().fc_dequant_reduce_requant_fp8(cp.data_ptr(), cp.stride(0), sp.data_ptr(), sp.stride(0),
                                                n_src, t, h, group, co.data_ptr(), so.data_ptr(),
                                                torch.cuda.current_stream().cuda_stream)
    assert rc == 0
    torch.cuda.synchronize()
    assert_pair((co.cpu().numpy(), so.cpu().numpy()), want, "padded stride")


def test_dequantize_fp8_matches_oracle(fc):
    rng = np.random.default_rng(10)
    for (t, h) in [(16, 4096), (3, 1056), (7, 2080)]:
        x = synth_inputs.make_partials(1, t, h, seed=6)[0]
        for group in groups_for(h)[:4]:
            c, s = oracle.quantize_fp8(x, group)
            want = oracle.dequantize_fp8(c, s, h, group)
            assert_f16(gpu_dequantize_fp8(fc, c, s, h, group), want, np.repeat(s, group, axis=1) * 2.0 ** -9,
                       "dequantize_fp8 %dx%d g=%d" % (t, h, group))
    # every finite byte under scales from subnormal-producing to overflowing
    t, h, group = 5, 2048, 128
    c = finite_codes(rng, (t, h))
    s = np.exp(rng.uniform(-30, 12, size=(t, h // group))).astype(np.float32)
    want = oracle.dequantize_fp8(c, s, h, group)
    got = gpu_dequantize_fp8(fc, c, s, h, group)
    assert same_bits(got.view(np.uint16), want.view(np.uint16)), first_diff(got.view(np.uint16), want.view(np.uint16))
    assert np.isinf(want.astype(np.float32)).any() and (want.view(np.uint16) == 0x8000).any()


@pytest.mark.parametrize("n_src", [2, 4, 8])
def test_allreduce_sim_fp8_matches_oracle(fc, n_src):
    for t, h, group in ((9, 4096, 128), (3, 4096, 4096)):
        x = synth_inputs.make_partials(n_src, t, h, seed=n_src + 60)
        want = oracle.allreduce_sim_fp8(x, group)
        y = Guarded((t, h), torch.float16)
        fc.allreduce_sim_fp8(dev(x.view(np.uint16)).view(torch.float16), group, out=y.t)
        torch.cuda.synchronize(); y.check()
        got = y.t.cpu().numpy()
        assert same_bits(got.view(np.uint16), want.view(np.uint16)), first_diff(got.view(np.uint16), want.view(np.uint16))


def test_fp8_empty_input_is_a_noop(fc):
    x = torch.empty((0, 4096), dtype=torch.float16, device="cuda")
    c, s = fc.quantize_fp8(x, 128)
    assert c.shape == (0, 4096) and s.shape == (0, 32)
    y = fc.allreduce_sim_fp8(torch.empty((4, 0, 4096), dtype=torch.float16, device="cuda"), 128)
    assert y.shape == (0, 4096)
    torch.cuda.synchronize()


def test_fp8_full_size_config_on_sampled_rows(fc):
    w = synth_inputs.WORKLOADS["llama3_8b_prefill"]
    x = synth_inputs.make_partials_device(w.n_src, w.tokens, w.hidden, w.seed + 2, "cuda",
                                          w.outlier_frac, w.outlier_gain)
    rows = np.unique(np.concatenate([[0, 1, w.tokens - 1],
                                     np.random.default_rng(4).integers(0, w.tokens, 61)]))
    ridx = torch.from_numpy(rows).cuda()
    stage1 = [fc.quantize_fp8(x[j], w.group) for j in range(w.n_src)]
    c = torch.stack([p[0] for p in stage1]); s = torch.stack([p[1] for p in stage1])
    co, so = fc.dequant_reduce_requant_fp8(c, s, w.hidden, w.group)
    y = fc.dequantize_fp8(co, so, w.hidden, w.group)
    y2 = fc.allreduce_sim_fp8(x, w.group)
    torch.cuda.synchronize()
    assert torch.equal(y.view(torch.int16), y2.view(torch.int16))
    xs = x[:, ridx].cpu().numpy()
    oc, os_ = oracle_stage1_fp8(xs, w.group)
    assert_pair((c[:, ridx].cpu().numpy(), s[:, ridx].cpu().numpy()), (oc, os_), "fp8 stage 1")
    want = oracle.dequant_reduce_requant_fp8(oc, os_, w.hidden, w.group)
    assert_pair((co[ridx].cpu().numpy(), so[ridx].cpu().numpy()), want, "fp8 fused")
    wy = oracle.dequantize_fp8(*want, w.hidden, w.group)
    assert_f16(y[ridx].cpu().numpy(), wy, np.repeat(want[1], w.group, axis=1) * 2.0 ** -9, "fp8 output")
    assert bool((so > 0).all()) and bool(torch.isfinite(so).all())
    assert not bool(((co & 0x7F) == 0x7F).any())
