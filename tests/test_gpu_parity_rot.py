"""GPU parity of the rotation entry points (Hadamard transform fused into the first
quantization and the last dequantization; paper Section 4) against the CPU oracle,
bit for bit, through the C ABI.  Run with ``-m gpu`` on an MI355X."""
import numpy as np
import pytest

import oracle
import synth_inputs
from test_gpu_parity import Guarded, dev, first_diff, same_bits, fc  # noqa: F401

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

QUANTIZERS = [(oracle.ASYM, 4), (oracle.ASYM, 8), (oracle.SYM, 4), (oracle.SYM, 8), (oracle.FP8, 8)]


def groups_of(hidden):
    return [g for g in (32, 128, 1024, 2048, 4096, 8192) if g <= hidden and hidden % g == 0]


# power-of-two rows (one block) and rows rotated block by block: 5 x 1024 (the rotation table's LLaMA-2-13B
# row), 3 x 1024, 7 x 1024, 3 x 2048, 3 x 4096, and a single block of 1024
HIDDENS = [2048, 4096, 8192, 1024, 5120, 3072, 7168, 6144, 12288]


def gpu_quantize_rot(fc, x16, group, bits, quantizer):
    t, h = x16.shape
    c = Guarded((t, h * bits // 8), torch.uint8)
    s = Guarded((t, h // group), torch.float32)
    z = Guarded((t, h // group), torch.float32)
    fc.quantize_rot(dev(x16.view(np.uint16)).view(torch.float16), group, bits, quantizer, out=(c.t, s.t, z.t))
    torch.cuda.synchronize()
    for g in (c, s, z):
        g.check()
    return c.t.cpu().numpy(), s.t.cpu().numpy(), z.t.cpu().numpy()


def assert_rot_triplet(got, want, quantizer, what):
    names = ("codes", "scales", "zeros") if quantizer == oracle.ASYM else ("codes", "scales")
    for name, g, w in zip(names, got, want):
        assert same_bits(g, w), "%s %s: %s" % (what, name, first_diff(g, w))


@pytest.mark.parametrize("quantizer,bits", QUANTIZERS)
@pytest.mark.parametrize("hidden", HIDDENS)
def test_quantize_rot_matches_oracle(fc, quantizer, bits, hidden):
    # 5 rows: with 1024-element blocks (two to a workgroup) 5 x 5, 5 x 3 and 5 x 7 blocks end in a half-filled chunk
    x = synth_inputs.make_partials(1, 5, hidden, seed=hidden + bits)[0]
    for group in groups_of(hidden):
        want = oracle.quantize_rot(x, group, bits, quantizer)
        got = gpu_quantize_rot(fc, x, group, bits, quantizer)
        assert_rot_triplet(got, want, quantizer, "quantize_rot h=%d g=%d b=%d q=%d" % (hidden, group, bits, quantizer))


@pytest.mark.parametrize("hidden", [2048, 4096, 8192])
def test_quantize_rot_special_rows(fc, hidden):
    # rows that rotate to a single spike (Walsh functions), a spike that rotates to a flat row, zeros,
    # binary16 extremes, and values whose transform rounds in every stage
    import scipy.linalg
    H = scipy.linalg.hadamard(hidden).astype(np.float32)
    rng = np.random.default_rng(hidden)
    x = np.zeros((8, hidden), np.float16)
    x[0] = H[3] * 0.5
    x[1] = H[hidden - 1] * -2.0
    x[2, 7] = 1000.0
    x[4] = 60000.0 * H[hidden // 2 + 1]
    x[5] = (rng.standard_normal(hidden) * np.exp(rng.uniform(-8, 8, hidden))).astype(np.float16)
    x[6] = np.float16(6e-8) * (np.arange(hidden) % 5)
    x[7] = rng.standard_normal(hidden) * 1e-3 + 3.0
    for quantizer, bits in QUANTIZERS:
        for group in (128, hidden):
            want = oracle.quantize_rot(x, group, bits, quantizer)
            got = gpu_quantize_rot(fc, x, group, bits, quantizer)
            assert_rot_triplet(got, want, quantizer, "special rows h=%d g=%d b=%d q=%d" % (hidden, group, bits, quantizer))


@pytest.mark.parametrize("quantizer,bits", QUANTIZERS)
@pytest.mark.parametrize("hidden", HIDDENS)
def test_dequantize_rot_matches_oracle(fc, quantizer, bits, hidden):
    x = synth_inputs.make_partials(1, 3, hidden, seed=hidden + 7)[0]
    rng = np.random.default_rng(hidden + bits)
    for group in groups_of(hidden)[::2]:
        c, s, z = oracle.quantize_rot(x, group, bits, quantizer)
        cases = [(c, s, z)]
        # arbitrary codes and metadata: every code value, scales over many binades, odd zero-points
        c2 = rng.integers(0, 256, size=c.shape, dtype=np.uint8)
        if quantizer == oracle.FP8:
            c2[(c2 & 0x7F) == 0x7F] = 0x7E
        s2 = np.exp(rng.uniform(-10, 6, size=s.shape)).astype(np.float32)
        z2 = np.rint(rng.uniform(-20, 300, size=s.shape)).astype(np.float32)
        z2[0, ::3] = rng.uniform(-3e4, 3e4, size=z2[0, ::3].shape).astype(np.float32)
        cases.append((c2, s2, z2))
        for cc, ss, zz in cases:
            want = oracle.dequantize_rot(cc, ss, zz, hidden, group, bits, quantizer)
            y = Guarded((cc.shape[0], hidden), torch.float16)
            fc.dequantize_rot(dev(cc), dev(ss), dev(zz), hidden, group, bits, quantizer, out=y.t)
            torch.cuda.synchronize(); y.check()
            got = y.t.cpu().numpy()
            assert same_bits(got.view(np.uint16), want.view(np.uint16)), \
                "dequantize_rot h=%d g=%d b=%d q=%d: %s" % (hidden, group, bits, quantizer,
                                                          first_diff(got.view(np.uint16), want.view(np.uint16)))


@pytest.mark.parametrize("quantizer,bits_rs,bits_ag", [(oracle.ASYM, 4, 4), (oracle.ASYM, 4, 8), (oracle.ASYM, 8, 8),
                                                       (oracle.SYM, 4, 4), (oracle.FP8, 8, 8)])
def test_allreduce_sim_rot_matches_oracle(fc, quantizer, bits_rs, bits_ag):
    for n_src, t, hidden, group in ((4, 5, 4096, 128), (2, 3, 8192, 8192), (8, 3, 2048, 2048), (3, 4, 8192, 1024),
                                    (4, 7, 5120, 1024), (2, 3, 5120, 128), (3, 1, 1024, 32), (2, 5, 12288, 4096)):
        x = synth_inputs.make_partials(n_src, t, hidden, seed=n_src + hidden)
        want = oracle.allreduce_sim_rot(x, group, bits_rs, bits_ag, quantizer)
        y = Guarded((t, hidden), torch.float16)
        fc.allreduce_sim_rot(dev(x.view(np.uint16)).view(torch.float16), group, bits_rs, bits_ag, quantizer, out=y.t)
        torch.cuda.synchronize(); y.check()
        got = y.t.cpu().numpy()
        assert same_bits(got.view(np.uint16), want.view(np.uint16)), \
            "allreduce_sim_rot N=%d h=%d g=%d: %s" % (n_src, hidden, group,
                                                      first_diff(got.view(np.uint16), want.view(np.uint16)))


def test_rot_rejects_unsupported_rows_and_empty_is_noop(fc):
    x = torch.zeros((2, 2560), dtype=torch.float16, device="cuda")           # 5 x 512: blocks below 1024
    with pytest.raises(fc.FcError):
        fc.quantize_rot(x, 128, 4)
    with pytest.raises(fc.FcError):
        fc.quantize_rot(torch.zeros((2, 4096), dtype=torch.float16, device="cuda"), 128, 4, fc.QUANTIZER_FP8)
    c, s, z = fc.quantize_rot(torch.empty((0, 4096), dtype=torch.float16, device="cuda"), 128, 4)
    assert c.shape == (0, 2048) and z.shape == (0, 32)
    torch.cuda.synchronize()


def test_rot_full_size_on_sampled_rows(fc):
    # the headline shape with per-token groups (where the paper finds the rotation pays off)
    w = synth_inputs.WORKLOADS["llama3_70b_prefill"]
    g = w.hidden
    x = synth_inputs.make_partials_device(w.n_src, w.tokens, w.hidden, 11, "cuda", w.outlier_frac, w.outlier_gain)
    rows = np.unique(np.concatenate([[0, w.tokens - 1], np.random.default_rng(5).integers(0, w.tokens, 20)]))
    ridx = torch.from_numpy(rows).cuda()
    y = fc.allreduce_sim_rot(x, g, w.bits_in, w.bits_out)
    stage1 = [fc.quantize_rot(x[j], g, w.bits_in) for j in range(w.n_src)]
    torch.cuda.synchronize()
    xs = x[:, ridx].cpu().numpy()
    for j in range(w.n_src):
        want = oracle.quantize_rot(xs[j], g, w.bits_in)
        got = tuple(a[ridx].cpu().numpy() for a in stage1[j])
        assert_rot_triplet(got, want, oracle.ASYM, "full size stage 1 source %d" % j)
    want = oracle.allreduce_sim_rot(xs, g, w.bits_in, w.bits_out)
    got = y[ridx].cpu().numpy()
    assert same_bits(got.view(np.uint16), want.view(np.uint16)), first_diff(got.view(np.uint16), want.view(np.uint16))


@pytest.mark.parametrize("hidden", [8192, 5120])
def test_rot_volume_beyond_2_to_32_elements(fc, hidden):
    # element indices and the byte offsets of the input pass 2^32 inside the tensor (for hidden 5120 the blocks of
    # 1024 also end in a half-filled chunk); sampled token rows against the oracle
    group, bits = 128, 4
    tokens = (1 << 32) // hidden + 3
    free, _ = torch.cuda.mem_get_info()
    if free < 40 * (1 << 30):
        pytest.skip("needs 40 GB of free device memory")
    g = torch.Generator(device="cuda"); g.manual_seed(hidden)
    x = torch.empty((tokens, hidden), dtype=torch.float16, device="cuda")
    chunk = 1 << 16
    for r0 in range(0, tokens, chunk):
        r1 = min(tokens, r0 + chunk)
        x[r0:r1] = (torch.randn((r1 - r0, hidden), generator=g, device="cuda") * (1.0 + (r0 // chunk) % 3)).half()
    c, s, z = fc.quantize_rot(x, group, bits)
    y = fc.dequantize_rot(c, s, z, hidden, group, bits)
    torch.cuda.synchronize()
    marks = [0, 1, (1 << 31) // hidden, (1 << 32) // hidden - 1, (1 << 32) // hidden, tokens - 2, tokens - 1]
    rows = np.unique(np.array(marks + list(np.random.default_rng(hidden).integers(0, tokens, 12))))
    ridx = torch.from_numpy(rows).cuda()
    xs = x[ridx].cpu().numpy()
    want = oracle.quantize_rot(xs, group, bits, oracle.ASYM)
    got = (c[ridx].cpu().numpy(), s[ridx].cpu().numpy(), z[ridx].cpu().numpy())
    assert_rot_triplet(got, want, oracle.ASYM, "rows around 2^32 elements, hidden %d" % hidden)
    wy = oracle.dequantize_rot(*want, hidden, group, bits, oracle.ASYM)
    assert same_bits(y[ridx].cpu().numpy().view(np.uint16), wy.view(np.uint16)), "dequantize_rot around 2^32 elements"
