"""GPU parity for coarse granularities: groups of 2048 ... 16384 elements, up to
one group per token (the block sizes of the paper's granularity study, Section
3.2.1 and the rotation table of Section 4), asymmetric and symmetric, against
the CPU oracle, bit for bit.  Run with ``-m gpu`` on an MI355X."""
import numpy as np
import pytest

import oracle
import synth_inputs
from test_gpu_parity import (assert_f16, assert_triplet, dev, first_diff, gpu_dequantize, gpu_fused,
                             gpu_quantize, oracle_stage1, same_bits, fc)  # noqa: F401
from test_gpu_parity_sym import (assert_pair, gpu_dequantize_sym, gpu_fused_sym, gpu_quantize_sym,
                                 oracle_stage1_sym)

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

# (tokens, hidden, group): groups spanning one wavefront exactly, 2 and 4 wavefronts, and 2 or 4
# sub-tiles of a workgroup; several groups per row and one group per row
CASES = [(5, 4096, 2048), (3, 4096, 4096), (4, 8192, 2048), (3, 8192, 8192), (2, 16384, 4096),
         (3, 16384, 16384), (1, 32768, 16384)]


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("case", CASES)
def test_quantize_wide_groups(fc, bits, case):
    t, h, g = case
    x = synth_inputs.make_partials(1, t, h, seed=h + g)[0]
    assert_triplet(gpu_quantize(fc, x, g, bits), oracle.quantize(x, g, bits), "quantize %s b=%d" % (case, bits))
    assert_pair(gpu_quantize_sym(fc, x, g, bits), oracle.quantize_sym(x, g, bits),
                "quantize_sym %s b=%d" % (case, bits))


@pytest.mark.parametrize("bits", [4, 8])
def test_quantize_wide_extreme_element_positions(fc, bits):
    # the group's minimum / maximum sits in the first or last lane of any wavefront or sub-tile
    t, h, g = 16, 8192, 8192
    rng = np.random.default_rng(3)
    x = rng.standard_normal((t, h)).astype(np.float16)
    pos = [0, 31, 2047, 2048, 4095, 4096, 6143, 8191]
    for r in range(t):
        x[r, pos[r % 8]] = 30.0 + r
        x[r, pos[(r + 3) % 8]] = -40.0 - r
    assert_triplet(gpu_quantize(fc, x, g, bits), oracle.quantize(x, g, bits), "extreme positions")
    assert_pair(gpu_quantize_sym(fc, x, g, bits), oracle.quantize_sym(x, g, bits), "extreme positions sym")


@pytest.mark.parametrize("bits_in,bits_out", [(4, 4), (8, 8), (4, 8), (8, 4)])
@pytest.mark.parametrize("n_src", [1, 2, 4, 5, 8])
def test_fused_wide_groups(fc, bits_in, bits_out, n_src):
    for (t, h, g) in CASES[:6]:
        x = synth_inputs.make_partials(n_src, t, h, seed=n_src + g)
        c, s, z = oracle_stage1(x, g, bits_in)
        want = oracle.dequant_reduce_requant(c, s, z, h, g, bits_in, bits_out)
        assert_triplet(gpu_fused(fc, c, s, z, h, g, bits_in, bits_out), want,
                       "fused N=%d %s %d->%d" % (n_src, (t, h, g), bits_in, bits_out))
        c, s = oracle_stage1_sym(x, g, bits_in)
        want = oracle.dequant_reduce_requant_sym(c, s, h, g, bits_in, bits_out)
        assert_pair(gpu_fused_sym(fc, c, s, h, g, bits_in, bits_out), want,
                    "fused_sym N=%d %s %d->%d" % (n_src, (t, h, g), bits_in, bits_out))


@pytest.mark.parametrize("bits_in", [4, 8])
def test_fused_wide_arbitrary_meta(fc, bits_in):
    # zero-points outside the fast range, fractional, huge: the literal fp32 path per source
    rng = np.random.default_rng(11)
    n_src, t, h, g = 4, 6, 8192, 4096
    c = rng.integers(0, 256, size=(n_src, t, h * bits_in // 8), dtype=np.uint8)
    s = np.exp(rng.uniform(-12, 8, size=(n_src, t, h // g))).astype(np.float32)
    z = np.rint(rng.uniform(-20, 300, size=(n_src, t, h // g))).astype(np.float32)
    z[0, :, 0] = rng.uniform(-3e6, 3e6, size=t).astype(np.float32)
    z[1, 1::2, 1] += 0.25
    z[2, 0] = -1701.0
    z[2, 1] = 1001.0
    z[3, 2] = 2.0 ** 24 + 2
    for bits_out in (4, 8):
        want = oracle.dequant_reduce_requant(c, s, z, h, g, bits_in, bits_out)
        assert_triplet(gpu_fused(fc, c, s, z, h, g, bits_in, bits_out), want,
                       "wide arbitrary meta %d->%d" % (bits_in, bits_out))
        want = oracle.dequant_reduce_requant_sym(c, s, h, g, bits_in, bits_out)
        assert_pair(gpu_fused_sym(fc, c, s, h, g, bits_in, bits_out), want,
                    "wide arbitrary codes sym %d->%d" % (bits_in, bits_out))


@pytest.mark.parametrize("bits", [4, 8])
def test_dequantize_wide_groups(fc, bits):
    for (t, h, g) in CASES:
        x = synth_inputs.make_partials(1, t, h, seed=5)[0]
        c, s, z = oracle.quantize(x, g, bits)
        want = oracle.dequantize(c, s, z, h, g, bits)
        assert_f16(gpu_dequantize(fc, c, s, z, h, g, bits), want, np.repeat(s, g, axis=1),
                   "dequantize %s b=%d" % ((t, h, g), bits))
        c, s = oracle.quantize_sym(x, g, bits)
        want = oracle.dequantize_sym(c, s, h, g, bits)
        assert_f16(gpu_dequantize_sym(fc, c, s, h, g, bits), want, np.repeat(s, g, axis=1),
                   "dequantize_sym %s b=%d" % ((t, h, g), bits))


@pytest.mark.parametrize("hidden", [4096, 8192])
@pytest.mark.parametrize("bits_rs,bits_ag", [(4, 4), (8, 8), (4, 8)])
def test_allreduce_sim_per_token(fc, hidden, bits_rs, bits_ag):
    # one group per token: the coarsest point of the paper's granularity study
    n_src, t = 4, 6
    x = synth_inputs.make_partials(n_src, t, hidden, seed=hidden + bits_rs)
    xd = dev(x.view(np.uint16)).view(torch.float16)
    want = oracle.allreduce_sim(x, hidden, bits_rs, bits_ag)
    got = fc.allreduce_sim(xd, hidden, bits_rs, bits_ag).cpu().numpy()
    assert same_bits(got.view(np.uint16), want.view(np.uint16)), first_diff(got.view(np.uint16), want.view(np.uint16))
    want = oracle.allreduce_sim_sym(x, hidden, bits_rs, bits_ag)
    got = fc.allreduce_sim_sym(xd, hidden, bits_rs, bits_ag).cpu().numpy()
    assert same_bits(got.view(np.uint16), want.view(np.uint16)), first_diff(got.view(np.uint16), want.view(np.uint16))


def test_per_token_full_size_on_sampled_rows(fc):
    # the headline shape with one group per token, whole tensor through the GPU
    w = synth_inputs.WORKLOADS["llama3_70b_prefill"]
    g = w.hidden
    x = synth_inputs.make_partials_device(w.n_src, w.tokens, w.hidden, 7, "cuda", w.outlier_frac, w.outlier_gain)
    rows = np.unique(np.concatenate([[0, w.tokens - 1], np.random.default_rng(3).integers(0, w.tokens, 30)]))
    ridx = torch.from_numpy(rows).cuda()
    stage1 = [fc.quantize(x[j], g, w.bits_in) for j in range(w.n_src)]
    c = torch.stack([p[0] for p in stage1]); s = torch.stack([p[1] for p in stage1])
    z = torch.stack([p[2] for p in stage1])
    co, so, zo = fc.dequant_reduce_requant(c, s, z, w.hidden, g, w.bits_in, w.bits_out)
    y = fc.dequantize(co, so, zo, w.hidden, g, w.bits_out)
    torch.cuda.synchronize()
    xs = x[:, ridx].cpu().numpy()
    oc, os_, oz = oracle_stage1(xs, g, w.bits_in)
    assert_triplet((c[:, ridx].cpu().numpy(), s[:, ridx].cpu().numpy(), z[:, ridx].cpu().numpy()),
                   (oc, os_, oz), "per-token stage 1")
    want = oracle.dequant_reduce_requant(oc, os_, oz, w.hidden, g, w.bits_in, w.bits_out)
    assert_triplet((co[ridx].cpu().numpy(), so[ridx].cpu().numpy(), zo[ridx].cpu().numpy()), want,
                   "per-token fused")
    wy = oracle.dequantize(*want, w.hidden, g, w.bits_out)
    assert_f16(y[ridx].cpu().numpy(), wy, np.repeat(want[1], g, axis=1), "per-token output")


def test_ablation_sweep_matches_oracle_errors(fc):
    # the error table of the granularity / precision sweep equals what the oracle's outputs give
    from paper_2412_04964_amd import ablation
    x = synth_inputs.make_partials(4, 8, 4096, seed=6)
    rows = ablation.sweep(dev(x.view(np.uint16)).view(torch.float16), [128, 1024, 4096], rotation=True)
    assert len(rows) == (3 * 3 * 3 + 3) + (3 * 2 * 3 + 3)
    exact = x.astype(np.float64).sum(0)
    for r in rows:
        if r["quantizer"].endswith("+ht"):
            if r["precision"] == "FP8":
                y = oracle.allreduce_sim_rot(x, r["group"], 8, 8, oracle.FP8)
            else:
                b_rs, b_ag = ablation.PRECISIONS[r["precision"]]
                y = oracle.allreduce_sim_rot(x, r["group"], b_rs, b_ag,
                                             oracle.SYM if r["quantizer"] == "sym+ht" else oracle.ASYM)
        elif r["precision"] == "FP8":
            y = oracle.allreduce_sim_fp8(x, r["group"])
        else:
            b_rs, b_ag = ablation.PRECISIONS[r["precision"]]
            fn = {"sym": oracle.allreduce_sim_sym, "cmeta": oracle.allreduce_sim_cmeta,
                  "asym": oracle.allreduce_sim}[r["quantizer"]]
            y = fn(x, r["group"], b_rs, b_ag)
        want = float(np.mean((y.astype(np.float64) - exact) ** 2))
        assert abs(r["mse"] - want) <= 1e-4 * want, r


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_random_shapes_all_quantizers(fc, seed):
    # seeded sweep over shapes, group sizes, fan-ins and code widths that no other test names explicitly
    from test_gpu_parity_fp8 import gpu_fused_fp8, gpu_quantize_fp8, oracle_stage1_fp8
    rng = np.random.default_rng(1000 + seed)
    for case in range(14):
        group = int(rng.choice([32, 64, 128, 256, 512, 1024, 2048, 4096]))
        hidden = group * int(rng.integers(1, max(2, 12288 // group) + 1))
        tokens = int(rng.integers(1, 7))
        n_src = int(rng.integers(1, 9))
        bits_in, bits_out = int(rng.choice([4, 8])), int(rng.choice([4, 8]))
        what = "seed %d case %d: N=%d %dx%d g=%d %d->%d" % (seed, case, n_src, tokens, hidden, group, bits_in, bits_out)
        x = synth_inputs.make_partials(n_src, tokens, hidden, seed=seed * 100 + case,
                                       outlier_frac=float(rng.choice([0.0, 0.01, 0.1])))
        c, s, z = oracle_stage1(x, group, bits_in)
        assert_triplet(gpu_quantize(fc, x[0], group, bits_in), (c[0], s[0], z[0]), what + " quantize")
        want = oracle.dequant_reduce_requant(c, s, z, hidden, group, bits_in, bits_out)
        assert_triplet(gpu_fused(fc, c, s, z, hidden, group, bits_in, bits_out), want, what + " fused")
        wy = oracle.dequantize(*want, hidden, group, bits_out)
        gy = gpu_dequantize(fc, *want, hidden, group, bits_out)
        assert same_bits(gy.view(np.uint16), wy.view(np.uint16)), what + " dequantize"
        c, s = oracle_stage1_sym(x, group, bits_in)
        assert_pair(gpu_quantize_sym(fc, x[0], group, bits_in), (c[0], s[0]), what + " quantize_sym")
        want = oracle.dequant_reduce_requant_sym(c, s, hidden, group, bits_in, bits_out)
        assert_pair(gpu_fused_sym(fc, c, s, hidden, group, bits_in, bits_out), want, what + " fused_sym")
        wy = oracle.dequantize_sym(*want, hidden, group, bits_out)
        gy = gpu_dequantize_sym(fc, *want, hidden, group, bits_out)
        assert same_bits(gy.view(np.uint16), wy.view(np.uint16)), what + " dequantize_sym"
        c, s = oracle_stage1_fp8(x, group)
        assert_pair(gpu_quantize_fp8(fc, x[0], group), (c[0], s[0]), what + " quantize_fp8")
        want = oracle.dequant_reduce_requant_fp8(c, s, hidden, group)
        assert_pair(gpu_fused_fp8(fc, c, s, hidden, group), want, what + " fused_fp8")


def test_large_volume_offsets_beyond_32_bits(fc):
    # 2^33 elements: byte offsets of the input exceed 2^34 and element indices 2^32, with a ragged last tile;
    # sampled rows (first, last, around the 2^32-element and 2^32-byte marks) are checked against the oracle
    hidden, group, bits = 8192, 128, 4
    tokens = (1 << 20) + 3
    free, _ = torch.cuda.mem_get_info()
    if free < 80 * (1 << 30):
        pytest.skip("needs 80 GB of free device memory")
    g = torch.Generator(device="cuda"); g.manual_seed(5)
    x = torch.empty((tokens, hidden), dtype=torch.float16, device="cuda")
    chunk = 1 << 16
    for r0 in range(0, tokens, chunk):
        r1 = min(tokens, r0 + chunk)
        x[r0:r1] = (torch.randn((r1 - r0, hidden), generator=g, device="cuda") * (1.0 + (r0 // chunk) % 5)).half()
    c = torch.empty((2, tokens, hidden // 2), dtype=torch.uint8, device="cuda")
    s = torch.empty((2, tokens, hidden // group), dtype=torch.float32, device="cuda")
    z = torch.empty_like(s)
    fc.quantize(x, group, bits, out=(c[0], s[0], z[0]))
    x2 = x.flip(1)                                        # second partial: the same values mirrored along hidden
    fc.quantize(x2, group, bits, out=(c[1], s[1], z[1]))
    co, so, zo = fc.dequant_reduce_requant(c, s, z, hidden, group, bits, bits)
    y = fc.dequantize(co, so, zo, hidden, group, bits)
    torch.cuda.synchronize()
    marks = [0, 1, (1 << 32) // hidden - 1, (1 << 32) // hidden, (1 << 31) // hidden, (1 << 33) // (2 * hidden) - 1,
             (1 << 19) + 1, tokens - 4, tokens - 3, tokens - 2, tokens - 1]
    rows = np.unique(np.array(marks + list(np.random.default_rng(6).integers(0, tokens, 20))))
    ridx = torch.from_numpy(rows).cuda()
    xs = np.stack([x[ridx].cpu().numpy(), x2[ridx].cpu().numpy()])
    oc, os_, oz = oracle_stage1(xs, group, bits)
    assert_triplet((c[:, ridx].cpu().numpy(), s[:, ridx].cpu().numpy(), z[:, ridx].cpu().numpy()), (oc, os_, oz),
                   "large volume stage 1")
    want = oracle.dequant_reduce_requant(oc, os_, oz, hidden, group, bits, bits)
    assert_triplet((co[ridx].cpu().numpy(), so[ridx].cpu().numpy(), zo[ridx].cpu().numpy()), want, "large volume fused")
    wy = oracle.dequantize(*want, hidden, group, bits)
    assert same_bits(y[ridx].cpu().numpy().view(np.uint16), wy.view(np.uint16)), "large volume output"


@pytest.mark.parametrize("seed", [11, 12])
def test_randomized_sweep_of_every_quantizer_end_to_end(fc, seed):
    # 250 random (shape, group, fan-in, bit-width, value distribution) draws per seed; every quantizer's
    # fc_allreduce_sim* and the compact-metadata stages against the oracle.  (A sweep of this kind found the
    # zero-point-2049 case of the compact-metadata packer.)
    rng = np.random.default_rng(seed)

    def draw(n, t, h):
        kind = int(rng.integers(0, 6))
        if kind == 0:
            x = rng.standard_normal((n, t, h))
        elif kind == 1:
            x = rng.standard_normal((n, t, h)) * np.exp(rng.uniform(-12, 10, (n, t, 1)))
        elif kind == 2:
            x = rng.uniform(100, 101, (n, t, h)) * rng.choice([-1, 1])
        elif kind == 3:
            x = np.round(rng.standard_normal((n, t, h)) * 4) / 2
        elif kind == 4:
            x = rng.standard_normal((n, t, h)) * (rng.random((n, t, h)) < 0.02) * 1000
        else:
            x = rng.standard_normal((n, t, h)) * 1e-6 + rng.choice([0, 3, -500, 60000])
        return np.clip(x, -65504, 65504).astype(np.float16)

    def same16(got, want, what):
        assert same_bits(got.cpu().numpy().view(np.uint16), want.view(np.uint16)), what

    for case in range(250):
        group = int(rng.choice([32, 64, 128, 256, 512, 1024, 2048, 4096, 8192]))
        hidden = group * int(rng.integers(1, max(2, 8192 // group) + 1))
        tokens, n = int(rng.integers(1, 5)), int(rng.integers(1, 9))
        bi, bo = int(rng.choice([4, 8])), int(rng.choice([4, 8]))
        x = draw(n, tokens, hidden)
        xd = dev(x.view(np.uint16)).view(torch.float16)
        what = "seed %d case %d: N=%d %dx%d g=%d %d->%d" % (seed, case, n, tokens, hidden, group, bi, bo)
        same16(fc.allreduce_sim(xd, group, bi, bo), oracle.allreduce_sim(x, group, bi, bo), what + " asym")
        same16(fc.allreduce_sim_sym(xd, group, bi, bo), oracle.allreduce_sim_sym(x, group, bi, bo), what + " sym")
        same16(fc.allreduce_sim_fp8(xd, group), oracle.allreduce_sim_fp8(x, group), what + " fp8")
        same16(fc.allreduce_sim_cmeta(xd, group, bi, bo), oracle.allreduce_sim_cmeta(x, group, bi, bo), what + " cmeta")
        # the asymmetric fused step on its own: the launch-bound kernel at this volume and, with the token rows
        # repeated, the bulk kernel (gpu_fused runs both and compares them)
        pa = [oracle.quantize(x[j], group, bi) for j in range(n)]
        ca = np.stack([p[0] for p in pa]); sa = np.stack([p[1] for p in pa]); za = np.stack([p[2] for p in pa])
        assert_triplet(gpu_fused(fc, ca, sa, za, hidden, group, bi, bo),
                       oracle.dequant_reduce_requant(ca, sa, za, hidden, group, bi, bo), what + " fused asym")
        pm = [oracle.quantize_cmeta(x[j], group, bi) for j in range(n)]
        cm = np.stack([p[0] for p in pm]); mm = np.stack([p[1] for p in pm])
        gq = fc.quantize_cmeta(xd[0], group, bi)
        assert same_bits(gq[0].cpu().numpy(), pm[0][0]) and same_bits(gq[1].cpu().numpy().view(np.uint32), pm[0][1]), what
        gf = fc.dequant_reduce_requant_cmeta(dev(cm), dev(mm.view(np.int32)), hidden, group, bi, bo)
        wf = oracle.dequant_reduce_requant_cmeta(cm, mm, hidden, group, bi, bo)
        assert same_bits(gf[0].cpu().numpy(), wf[0]) and same_bits(gf[1].cpu().numpy().view(np.uint32), wf[1]), what
        if (hidden & -hidden) in (1024, 2048, 4096, 8192):      # the rotation's block: largest power of two dividing hidden
            q = int(rng.integers(0, 3))
            b8 = (8, 8) if q == 2 else (bi, bo)
            same16(fc.allreduce_sim_rot(xd, group, b8[0], b8[1], q), oracle.allreduce_sim_rot(x, group, b8[0], b8[1], q),
                   what + " rot %d" % q)


@pytest.mark.parametrize("variant", ["sym", "fp8", "cmeta"])
def test_large_volume_other_quantizers(fc, variant):
    # 2^32 + 24576 elements through the symmetric, FP8 and compact-metadata kernels at 8 bit: element
    # indices and the byte offsets of the input and of the codes all pass 2^32 inside the volume
    hidden, group, bits = 8192, 128, 8
    tokens = (1 << 19) + 3
    free, _ = torch.cuda.mem_get_info()
    if free < 60 * (1 << 30):
        pytest.skip("needs 60 GB of free device memory")
    g = torch.Generator(device="cuda"); g.manual_seed(9)
    x = torch.empty((2, tokens, hidden), dtype=torch.float16, device="cuda")
    chunk = 1 << 16
    for r0 in range(0, tokens, chunk):
        r1 = min(tokens, r0 + chunk)
        x[0, r0:r1] = (torch.randn((r1 - r0, hidden), generator=g, device="cuda") * (1.0 + (r0 // chunk) % 3)).half()
    x[1] = x[0].flip(1)
    if variant == "sym":
        q = lambda t, out: fc.quantize_sym(t, group, bits, out=out)
        f = lambda c, m: fc.dequant_reduce_requant_sym(c, m, hidden, group, bits, bits)
        d = lambda c, m: fc.dequantize_sym(c, m, hidden, group, bits)
        oq = lambda a: oracle.quantize_sym(a, group, bits)
        of = lambda c, m: oracle.dequant_reduce_requant_sym(c, m, hidden, group, bits, bits)
        od = lambda c, m: oracle.dequantize_sym(c, m, hidden, group, bits)
        mdt = torch.float32
    elif variant == "fp8":
        q = lambda t, out: fc.quantize_fp8(t, group, out=out)
        f = lambda c, m: fc.dequant_reduce_requant_fp8(c, m, hidden, group)
        d = lambda c, m: fc.dequantize_fp8(c, m, hidden, group)
        oq = lambda a: oracle.quantize_fp8(a, group)
        of = lambda c, m: oracle.dequant_reduce_requant_fp8(c, m, hidden, group)
        od = lambda c, m: oracle.dequantize_fp8(c, m, hidden, group)
        mdt = torch.float32
    else:
        q = lambda t, out: fc.quantize_cmeta(t, group, bits, out=out)
        f = lambda c, m: fc.dequant_reduce_requant_cmeta(c, m, hidden, group, bits, bits)
        d = lambda c, m: fc.dequantize_cmeta(c, m, hidden, group, bits)
        oq = lambda a: oracle.quantize_cmeta(a, group, bits)
        of = lambda c, m: oracle.dequant_reduce_requant_cmeta(c, m.view(np.uint32), hidden, group, bits, bits)
        od = lambda c, m: oracle.dequantize_cmeta(c, m.view(np.uint32), hidden, group, bits)
        mdt = torch.int32
    c = torch.empty((2, tokens, hidden), dtype=torch.uint8, device="cuda")
    m = torch.empty((2, tokens, hidden // group), dtype=mdt, device="cuda")
    for j in range(2):
        q(x[j], (c[j], m[j]))
    co, mo = f(c, m)
    y = d(co, mo)
    torch.cuda.synchronize()
    marks = [0, 1, (1 << 32) // hidden - 1, (1 << 32) // hidden, (1 << 31) // hidden, (1 << 18) + 1,
             tokens - 3, tokens - 2, tokens - 1]
    rows = np.unique(np.array(marks + list(np.random.default_rng(8).integers(0, tokens, 16))))
    ridx = torch.from_numpy(rows).cuda()
    bits_of = lambda a: np.ascontiguousarray(a).view(np.uint32) if a.dtype != np.uint8 else a
    ref = [oq(x[j, ridx].cpu().numpy()) for j in range(2)]
    for j in range(2):
        assert same_bits(c[j, ridx].cpu().numpy(), ref[j][0]), "%s stage 1 codes, source %d" % (variant, j)
        assert same_bits(bits_of(m[j, ridx].cpu().numpy()), bits_of(ref[j][1])), "%s stage 1 meta, source %d" % (variant, j)
    rc = np.stack([r[0] for r in ref]); rm = np.stack([bits_of(r[1]) for r in ref]).view(ref[0][1].dtype)
    want = of(rc, rm)
    assert same_bits(co[ridx].cpu().numpy(), want[0]), variant + " fused codes"
    assert same_bits(bits_of(mo[ridx].cpu().numpy()), bits_of(want[1])), variant + " fused meta"
    wy = od(*want)
    assert same_bits(y[ridx].cpu().numpy().view(np.uint16), wy.view(np.uint16)), variant + " output"


@pytest.mark.parametrize("kind", range(synth_inputs.STRESS_KINDS))
def test_value_distributions_end_to_end(fc, kind):
    # every quantizer and the rotation, end to end, on value distributions that reach the corners
    # (ties, huge zero-points, near-degenerate groups, mostly-zero groups, 22 octaves of scale)
    rng = np.random.default_rng(50 + kind)
    for case in range(10):
        group = int(rng.choice([32, 128, 512, 2048, 8192]))
        hidden = group * int(rng.integers(1, max(2, 8192 // group) + 1))
        tokens, n_src = int(rng.integers(1, 5)), int(rng.integers(1, 9))
        bi, bo = int(rng.choice([4, 8])), int(rng.choice([4, 8]))
        x = synth_inputs.make_partials_stress(n_src, tokens, hidden, kind, seed=kind * 100 + case)
        xd = dev(x.view(np.uint16)).view(torch.float16)
        what = "kind %d case %d: N=%d %dx%d g=%d %d->%d" % (kind, case, n_src, tokens, hidden, group, bi, bo)
        pairs = [("asym", fc.allreduce_sim(xd, group, bi, bo), oracle.allreduce_sim(x, group, bi, bo)),
                 ("sym", fc.allreduce_sim_sym(xd, group, bi, bo), oracle.allreduce_sim_sym(x, group, bi, bo)),
                 ("fp8", fc.allreduce_sim_fp8(xd, group), oracle.allreduce_sim_fp8(x, group))]
        if (hidden & -hidden) in (1024, 2048, 4096, 8192):      # the rotation's block: largest power of two dividing hidden
            q = int(rng.integers(0, 3))
            b = (8, 8) if q == 2 else (bi, bo)
            pairs.append(("rot q=%d" % q, fc.allreduce_sim_rot(xd, group, b[0], b[1], q),
                          oracle.allreduce_sim_rot(x, group, b[0], b[1], q)))
        c, s, z = oracle_stage1(x, group, bi)
        assert_triplet(gpu_fused(fc, c, s, z, hidden, group, bi, bo),
                       oracle.dequant_reduce_requant(c, s, z, hidden, group, bi, bo), what + " fused")
        for name, got, want in pairs:
            got = got.cpu().numpy()
            assert same_bits(got.view(np.uint16), want.view(np.uint16)), "%s %s: %s" % (
                what, name, first_diff(got.view(np.uint16), want.view(np.uint16)))
