"""Corners of the C ABI on the GPU, called raw through ctypes: per-source metadata slabs that are only
4-byte aligned (odd source strides), on both ways the fused kernel fetches group parameters (the shared table
for narrow groups, per-lane loads for wide ones), and the launch-bound kernel that small volumes take (one code word
per lane and source), for every fan-in, bit-width pair and group size, on both sides of its size limit.  Bit for bit against the CPU oracle.  Run with ``-m gpu``."""
import numpy as np
import pytest

import oracle
import synth_inputs
from test_gpu_parity import Guarded, bulk_reps, dev, first_diff, oracle_stage1, same_bits, tile_tokens, fc  # noqa: F401
from test_gpu_parity_cmeta import oracle_stage1_cmeta

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _padded_slabs(arrs, stride_elems, dtype, lead):
    """The per-source arrays of `arrs` [N, ...] laid out `stride_elems` apart after `lead` elements of poison,
    in one device buffer whose base is 16-byte aligned; returns (buffer, view of element `lead`)."""
    n = arrs.shape[0]
    per = arrs[0].size
    assert stride_elems >= per
    buf = torch.full((lead + n * stride_elems + 8,), -12345, dtype=dtype, device="cuda")
    flat = torch.from_numpy(np.ascontiguousarray(arrs).reshape(n, per).view(
        {torch.float32: np.float32, torch.int32: np.int32}[dtype])).cuda()
    for j in range(n):
        buf[lead + j * stride_elems: lead + j * stride_elems + per] = flat[j]
    return buf, buf[lead:]


@pytest.mark.parametrize("group", [32, 128, 512, 2048])
@pytest.mark.parametrize("bits_in,bits_out", [(4, 4), (8, 8), (4, 8)])
@pytest.mark.parametrize("n_src", [2, 5])
def test_fused_with_odd_metadata_strides(fc, group, bits_in, bits_out, n_src):
    # scales and zero-points of source j start at +j*stride floats with an odd stride, so slabs 1, 3, ... are
    # only 4-byte aligned; base pointers stay 16-byte aligned as the header requires
    t0, h = 11, 4096
    x = synth_inputs.make_partials(n_src, t0, h, seed=300 + group + n_src, outlier_frac=0.01)
    c0, s0, z0 = oracle_stage1(x, group, bits_in)
    want0 = oracle.dequant_reduce_requant(c0, s0, z0, h, group, bits_in, bits_out)
    # the case as it is (narrow groups: the launch-bound kernel) and repeated up to the bulk kernel's volumes, where
    # narrow groups go through the shared table and wide ones through per-lane loads
    for reps, extras in ((1, (1, 3, 7)), (bulk_reps(t0, h), (1, 7))):
        c, s, z = tile_tokens(c0, reps), tile_tokens(s0, reps), tile_tokens(z0, reps)
        want = tuple(tile_tokens(w, reps) for w in want0)
        t = t0 * reps
        per = t * h // group
        for extra in extras:
            stride = per + extra + (0 if (per + extra) % 2 else 1)            # odd number of floats
            assert stride % 2 == 1
            sbuf, sview = _padded_slabs(s, stride, torch.float32, 0)
            zbuf, zview = _padded_slabs(z, stride, torch.float32, 0)
            cd = dev(c)
            co = Guarded((t, h * bits_out // 8), torch.uint8)
            so = Guarded((t, h // group), torch.float32)
            zo = Guarded((t, h // group), torch.float32)
            rc = fc.lib().fc_dequant_reduce_requant(cd.data_ptr(), cd.stride(0), sview.data_ptr(), zview.data_ptr(),
                                                    stride, n_src, t, h, group, bits_in, bits_out, co.t.data_ptr(),
                                                    so.t.data_ptr(), zo.t.data_ptr(), _stream())
            assert rc == 0
            torch.cuda.synchronize()
            for g_ in (co, so, zo):
                g_.check()
            for part, got, w_ in zip(("codes", "scales", "zeros"), (co, so, zo), want):
                assert same_bits(got.t.cpu().numpy(), w_), "x%d stride %d g=%d %s: %s" % (
                    reps, stride, group, part, first_diff(got.t.cpu().numpy(), w_))


@pytest.mark.parametrize("group", [128, 512])
@pytest.mark.parametrize("bits_in,bits_out", [(4, 4), (8, 8)])
def test_fused_cmeta_with_odd_metadata_strides(fc, group, bits_in, bits_out):
    n_src, t, h = 3, 11, 4096
    x = synth_inputs.make_partials(n_src, t, h, seed=500 + group, outlier_frac=0.01)
    c, m = oracle_stage1_cmeta(x, group, bits_in)
    want = oracle.dequant_reduce_requant_cmeta(c, m, h, group, bits_in, bits_out)
    per = t * h // group
    stride = per + (1 if per % 2 == 0 else 2)
    mbuf, mview = _padded_slabs(m.view(np.int32), stride, torch.int32, 0)
    cd = dev(c)
    co = Guarded((t, h * bits_out // 8), torch.uint8)
    mo = Guarded((t, h // group), torch.int32)
    rc = fc.lib().fc_dequant_reduce_requant_cmeta(cd.data_ptr(), cd.stride(0), mview.data_ptr(), stride, n_src, t, h,
                                                  group, bits_in, bits_out, co.t.data_ptr(), mo.t.data_ptr(), _stream())
    assert rc == 0
    torch.cuda.synchronize()
    co.check(); mo.check()
    assert same_bits(co.t.cpu().numpy(), want[0]), first_diff(co.t.cpu().numpy(), want[0])
    assert same_bits(mo.t.cpu().numpy().view(np.uint32), want[1])


def test_fused_rejects_misaligned_bases_and_short_strides(fc):
    L = fc.lib()
    t, h, g = 4, 1024, 128
    c = torch.zeros((2, t, h // 2), dtype=torch.uint8, device="cuda")
    s = torch.zeros((2 * t * h // g + 8,), dtype=torch.float32, device="cuda")
    o = torch.zeros((t, h // 2), dtype=torch.uint8, device="cuda")
    so = torch.zeros((t, h // g), dtype=torch.float32, device="cuda")
    args = lambda sp, zp, ms: (c.data_ptr(), c.stride(0), sp, zp, ms, 2, t, h, g, 4, 4, o.data_ptr(), so.data_ptr(),
                               so.data_ptr(), _stream())
    assert L.fc_dequant_reduce_requant(*args(s.data_ptr() + 4, s.data_ptr(), t * h // g)) == -5      # base not 16-byte aligned
    assert L.fc_dequant_reduce_requant(*args(s.data_ptr(), s.data_ptr(), t * h // g - 1)) == -4      # stride below one slab


# Volumes of at most 2048 wavefronts of one 32-bit code word per lane (asymmetric quantizer, groups that fit such a
# wavefront) take the launch-bound kernel: every fan-in and bit-width pair, with a ragged last wavefront and rows
# that straddle wavefronts
@pytest.mark.parametrize("bits_in,bits_out", [(8, 8), (4, 4), (4, 8), (8, 4)])
@pytest.mark.parametrize("n_src", [1, 2, 3, 4, 5, 6, 7, 8])
def test_fused_small_volumes_every_fan_in(fc, bits_in, bits_out, n_src):
    for (t, h) in [(7, 2176), (1, 128), (8, 8192), (31, 8192)]:
        waves = -(-t * h // (64 * 32 // bits_in))
        assert waves <= 2048
        x = synth_inputs.make_partials(n_src, t, h, seed=7 * n_src + bits_in + t, outlier_frac=0.02)
        c, s, z = oracle_stage1(x, 128, bits_in)
        want = oracle.dequant_reduce_requant(c, s, z, h, 128, bits_in, bits_out)
        cd, sd, zd = dev(c), dev(s), dev(z)
        co = Guarded((t, h * bits_out // 8), torch.uint8)
        so = Guarded((t, h // 128), torch.float32)
        zo = Guarded((t, h // 128), torch.float32)
        rc = fc.lib().fc_dequant_reduce_requant(cd.data_ptr(), cd.stride(0), sd.data_ptr(), zd.data_ptr(), sd.stride(0),
                                                n_src, t, h, 128, bits_in, bits_out, co.t.data_ptr(), so.t.data_ptr(),
                                                zo.t.data_ptr(), _stream())
        assert rc == 0
        torch.cuda.synchronize()
        for part, got, w_ in zip(("codes", "scales", "zeros"), (co, so, zo), want):
            got.check()
            assert same_bits(got.t.cpu().numpy(), w_), "N=%d %dx%d %d->%d %s: %s" % (
                n_src, t, h, bits_in, bits_out, part, first_diff(got.t.cpu().numpy(), w_))


# The fused kernels read their landing zones with hand-ordered waits.  libfc_plainreads.so is the same library with
# those reads compiled the plain way (full wait, compiler-visible LDS loads): both must give the oracle's bits for
# every fan-in and bit-width pair, on narrow, wide and cross-wavefront groups, asymmetric and symmetric.
@pytest.fixture(scope="module")
def plain_lib():
    import ctypes
    import os
    import paper_2412_04964_amd as m
    path = os.path.join(os.path.dirname(m.lib_path()), "libfc_plainreads.so")
    if not os.path.exists(path):
        pytest.fail("%s missing: build with `python -m paper_2412_04964_amd.build`" % path)
    L = ctypes.CDLL(path)
    i64, i32, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
    L.fc_dequant_reduce_requant.argtypes = [vp, i64, vp, vp, i64, i32, i64, i64, i32, i32, i32, vp, vp, vp, vp]
    L.fc_dequant_reduce_requant.restype = i32
    L.fc_dequant_reduce_requant_sym.argtypes = [vp, i64, vp, i64, i32, i64, i64, i32, i32, i32, vp, vp, vp]
    L.fc_dequant_reduce_requant_sym.restype = i32
    sz = ctypes.c_size_t
    for name in ("fc_allreduce_sim", "fc_allreduce_sim_sym", "fc_allreduce_sim_cmeta"):
        getattr(L, name).argtypes = [vp, i32, i64, i64, i32, i32, i32, vp, vp, sz, vp]
        getattr(L, name).restype = i32
    L.fc_allreduce_sim_fp8.argtypes = [vp, i32, i64, i64, i32, vp, vp, sz, vp]
    L.fc_allreduce_sim_fp8.restype = i32
    return L


@pytest.mark.parametrize("bits_in,bits_out", [(4, 4), (8, 8), (4, 8), (8, 4)])
@pytest.mark.parametrize("n_src", [1, 2, 3, 4, 5, 6, 7, 8])
def test_hand_ordered_and_plain_landing_reads_agree_with_the_oracle(fc, plain_lib, bits_in, bits_out, n_src):
    t0, h = 6, 8192
    x = synth_inputs.make_partials(n_src, t0, h, seed=900 + n_src, outlier_frac=0.01)
    reps = bulk_reps(t0, h)                             # the bulk kernel is the one with landing zones
    t = t0 * reps
    for group in (32, 128, 1024, 8192):
        c0, s0, z0 = oracle_stage1(x, group, bits_in)
        want = tuple(tile_tokens(w, reps) for w in oracle.dequant_reduce_requant(c0, s0, z0, h, group, bits_in, bits_out))
        cd, sd, zd = dev(tile_tokens(c0, reps)), dev(tile_tokens(s0, reps)), dev(tile_tokens(z0, reps))
        for which, L in (("hand-ordered", fc.lib()), ("plain", plain_lib)):
            co = Guarded((t, h * bits_out // 8), torch.uint8)
            so = Guarded((t, h // group), torch.float32)
            zo = Guarded((t, h // group), torch.float32)
            rc = L.fc_dequant_reduce_requant(cd.data_ptr(), cd.stride(0), sd.data_ptr(), zd.data_ptr(), sd.stride(0), n_src,
                                             t, h, group, bits_in, bits_out, co.t.data_ptr(), so.t.data_ptr(),
                                             zo.t.data_ptr(), _stream())
            assert rc == 0
            torch.cuda.synchronize()
            for part, got, w_ in zip(("codes", "scales", "zeros"), (co, so, zo), want):
                got.check()
                assert same_bits(got.t.cpu().numpy(), w_), "%s reads, N=%d g=%d %d->%d %s: %s" % (
                    which, n_src, group, bits_in, bits_out, part, first_diff(got.t.cpu().numpy(), w_))
    t = t0
    # symmetric kernels share the staging
    group = 128
    parts = [oracle.quantize_sym(x[j], group, bits_in) for j in range(n_src)]
    c = np.stack([p[0] for p in parts]); s = np.stack([p[1] for p in parts])
    want = oracle.dequant_reduce_requant_sym(c, s, h, group, bits_in, bits_out)
    cd, sd = dev(c), dev(s)
    for which, L in (("hand-ordered", fc.lib()), ("plain", plain_lib)):
        co = Guarded((t, h * bits_out // 8), torch.uint8)
        so = Guarded((t, h // group), torch.float32)
        rc = L.fc_dequant_reduce_requant_sym(cd.data_ptr(), cd.stride(0), sd.data_ptr(), sd.stride(0), n_src, t, h, group,
                                             bits_in, bits_out, co.t.data_ptr(), so.t.data_ptr(), _stream())
        assert rc == 0
        torch.cuda.synchronize()
        co.check(); so.check()
        assert same_bits(co.t.cpu().numpy(), want[0]) and same_bits(so.t.cpu().numpy(), want[1]), which + " reads, symmetric"


@pytest.mark.parametrize("n_src", [1, 2, 3, 4, 5, 6, 7, 8])
def test_one_launch_allreduce_with_hand_ordered_and_plain_landing_reads(fc, plain_lib, n_src):
    # the bandwidth-bound one-launch kernel stages its partials the same way (two loads per source and wavefront)
    t, h, group = 129, 8192, 128                       # above the limit of the launch-bound kernel
    x = synth_inputs.make_partials(n_src, t, h, seed=700 + n_src, outlier_frac=0.01)
    xd = dev(x.view(np.uint16)).view(torch.float16)
    ws = torch.empty(fc.allreduce_sim_workspace_bytes(n_src, t, h, group, 8, 8), dtype=torch.uint8, device="cuda")
    cases = [("fc_allreduce_sim", (4, 4), oracle.allreduce_sim(x, group, 4, 4)),
             ("fc_allreduce_sim_sym", (4, 8), oracle.allreduce_sim_sym(x, group, 4, 8)),
             ("fc_allreduce_sim_cmeta", (8, 4), oracle.allreduce_sim_cmeta(x, group, 8, 4)),
             ("fc_allreduce_sim_fp8", (), oracle.allreduce_sim_fp8(x, group))]
    for which, L in (("hand-ordered", fc.lib()), ("plain", plain_lib)):
        for name, bits, want in cases:
            y = Guarded((t, h), torch.float16)
            rc = getattr(L, name)(xd.data_ptr(), n_src, t, h, group, *bits, y.t.data_ptr(), ws.data_ptr(), ws.numel(),
                                  _stream())
            assert rc == 0
            torch.cuda.synchronize(); y.check()
            got = y.t.cpu().numpy().view(np.uint16)
            assert same_bits(got, want.view(np.uint16)), "%s reads, %s N=%d: %s" % (
                which, name, n_src, first_diff(got, want.view(np.uint16)))


# Volumes of at most 2^20 elements per partial with groups of at most 512 elements take fc_allreduce_sim's
# one-launch kernel: same bits as the three separate entry points and as the oracle, for every fan-in, bit-width
# pair and group size, with ragged last tiles, adversarial groups, and on both sides of the size limit.
def _three_kernel_path(fc, xd, group, bits_rs, bits_ag):
    stage1 = [fc.quantize(xd[j], group, bits_rs) for j in range(xd.shape[0])]
    c = torch.stack([p[0] for p in stage1]); s = torch.stack([p[1] for p in stage1]); z = torch.stack([p[2] for p in stage1])
    co, so, zo = fc.dequant_reduce_requant(c, s, z, xd.shape[2], group, bits_rs, bits_ag)
    return fc.dequantize(co, so, zo, xd.shape[2], group, bits_ag)


@pytest.mark.parametrize("bits_rs,bits_ag", [(8, 8), (4, 4), (4, 8), (8, 4)])
@pytest.mark.parametrize("n_src", [1, 2, 3, 4, 5, 6, 7, 8])
def test_one_launch_allreduce_every_fan_in_and_group(fc, bits_rs, bits_ag, n_src):
    for (t, h, group) in [(8, 8192, 128), (3, 1056, 32), (5, 2112, 64), (7, 2304, 256), (2, 1536, 512), (1, 32, 32)]:
        x = synth_inputs.make_partials(n_src, t, h, seed=50 * n_src + bits_rs + t, outlier_frac=0.02)
        xd = dev(x.view(np.uint16)).view(torch.float16)
        y = Guarded((t, h), torch.float16)
        fc.allreduce_sim(xd, group, bits_rs, bits_ag, out=y.t)
        y3 = _three_kernel_path(fc, xd, group, bits_rs, bits_ag)
        torch.cuda.synchronize(); y.check()
        got = y.t.cpu().numpy().view(np.uint16)
        want = oracle.allreduce_sim(x, group, bits_rs, bits_ag).view(np.uint16)
        what = "N=%d %dx%d g=%d %d->%d" % (n_src, t, h, group, bits_rs, bits_ag)
        assert same_bits(got, want), what + " vs oracle: " + first_diff(got, want)
        assert same_bits(got, y3.cpu().numpy().view(np.uint16)), what + " vs the three entry points"


@pytest.mark.parametrize("bits", [4, 8])
def test_one_launch_allreduce_adversarial_and_stress_values(fc, bits):
    for group in (32, 128, 512):
        a = synth_inputs.adversarial_groups(group, seed=3 + group)
        x = np.stack([a, a[::-1].copy(), (-a.astype(np.float32)).astype(np.float16)])
        for n in (1, 2, 3):
            want = oracle.allreduce_sim(x[:n], group, bits, bits).view(np.uint16)
            got = fc.allreduce_sim(dev(x[:n].view(np.uint16)).view(torch.float16), group, bits, bits)
            torch.cuda.synchronize()
            got = got.cpu().numpy().view(np.uint16)
            assert same_bits(got, want), "adversarial g=%d b=%d n=%d: %s" % (group, bits, n, first_diff(got, want))
    for kind in range(6):
        x = synth_inputs.make_partials_stress(3, 24, 2048, seed=70 + kind, kind=kind)
        want = oracle.allreduce_sim(x, 128, bits, bits).view(np.uint16)
        got = fc.allreduce_sim(dev(x.view(np.uint16)).view(torch.float16), 128, bits, bits).cpu().numpy().view(np.uint16)
        assert same_bits(got, want), "stress kind %d b=%d: %s" % (kind, bits, first_diff(got, want))


def test_one_launch_allreduce_on_both_sides_of_its_size_limit(fc):
    h, group = 8192, 128
    for t in (128, 129):                                   # 2^20 elements per partial: one launch; above: three kernels
        x = synth_inputs.make_partials(2, t, h, seed=t, outlier_frac=0.01)
        xd = dev(x.view(np.uint16)).view(torch.float16)
        got = fc.allreduce_sim(xd, group, 4, 8).cpu().numpy().view(np.uint16)
        y3 = _three_kernel_path(fc, xd, group, 4, 8).cpu().numpy().view(np.uint16)
        want = oracle.allreduce_sim(x, group, 4, 8).view(np.uint16)
        assert same_bits(got, want), "t=%d: %s" % (t, first_diff(got, want))
        assert same_bits(got, y3)


def test_loading_the_library_before_torch_still_shares_torchs_hip_runtime():
    # a process that touches the package first and torch afterwards: the library must end up on the HIP runtime
    # that owns torch's device memory (a second copy of the runtime fails every launch with "no device")
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    code = (
        "import sys; sys.path.insert(0, %r)\n"
        "import paper_2412_04964_amd as fc\n"
        "assert fc.version() >= 100\n"                       # loads libfc.so
        "import torch\n"
        "x = torch.randn(2, 4, 4096, device='cuda', dtype=torch.float16)\n"
        "y = fc.allreduce_sim(x, 128, 8, 8)\n"
        "torch.cuda.synchronize()\n"
        "assert torch.isfinite(y.float()).all() and (y.float() - x.float().sum(0)).abs().max() < 0.2\n"
        "print('ok')\n" % root)
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and r.stdout.strip().endswith("ok"), r.stdout + r.stderr


def test_three_entry_points_captured_into_one_graph_at_the_decode_shape(fc):
    # quantize (all partials in one launch), the launch-bound fused kernel and dequantize captured once, replayed on
    # new inputs with eager work and synchronizations in between; every replay against the oracle
    n, t, h, g, b = 8, 8, 8192, 128, 8
    xd = torch.zeros((n, t, h), dtype=torch.float16, device="cuda")
    c = torch.empty((n, t, h * b // 8), dtype=torch.uint8, device="cuda")
    s = torch.empty((n, t, h // g), dtype=torch.float32, device="cuda")
    z = torch.empty_like(s)
    co = torch.empty((t, h * b // 8), dtype=torch.uint8, device="cuda")
    so = torch.empty((t, h // g), dtype=torch.float32, device="cuda")
    zo = torch.empty_like(so)
    y = torch.empty((t, h), dtype=torch.float16, device="cuda")

    def chain():
        fc.quantize(xd.view(n * t, h), g, b, out=(c.view(n * t, -1), s.view(n * t, -1), z.view(n * t, -1)))
        fc.dequant_reduce_requant(c, s, z, h, g, b, b, out=(co, so, zo))
        fc.dequantize(co, so, zo, h, g, b, out=y)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        chain()                                                      # every kernel loaded before capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        chain()
    for rep in range(4):
        x = synth_inputs.make_partials(n, t, h, seed=1200 + rep, outlier_frac=0.01)
        xd.copy_(dev(x.view(np.uint16)).view(torch.float16))
        _ = float(xd.float().abs().max())                            # eager work and a synchronization
        graph.replay()
        torch.cuda.synchronize()
        want = oracle.allreduce_sim(x, g, b, b).view(np.uint16)
        got = y.cpu().numpy().view(np.uint16)
        assert same_bits(got, want), "replay %d: %s" % (rep, first_diff(got, want))
