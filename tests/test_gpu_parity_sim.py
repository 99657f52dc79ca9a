"""GPU parity of the single-kernel all-reduce for bandwidth-bound volumes (fc_allreduce_sim above 2^20 elements per
partial, its symmetric / FP8 / binary16-metadata counterparts at any volume; groups of at most 1024 elements) against
the CPU oracle, bit for bit, and against the three-kernel sequence (quantize x N, dequant-reduce-requant, dequantize
called one by one through the binding).  Volumes are just above the threshold so that the oracle finishes in a
fraction of a second per case."""
import numpy as np
import pytest

import oracle
import synth_inputs

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

SMALL_LIMIT = 1 << 20        # elements per partial up to which fc_allreduce_sim takes the launch-bound kernel


@pytest.fixture(scope="module")
def fc():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests selected but no GPU is visible")
    import paper_2412_04964_amd as m
    m.lib()
    return m


def dev16(x):
    return torch.from_numpy(np.ascontiguousarray(x).view(np.uint16)).cuda().view(torch.float16)


def run_sim(fc, x, group, b_rs, b_ag):
    n, t, h = x.shape
    assert t * h > SMALL_LIMIT, "the case must reach the bandwidth-bound kernel"
    guard = 64
    raw = torch.full((t * h + 2 * guard,), 7.0, dtype=torch.float16, device="cuda")
    y = raw[guard:guard + t * h].view(t, h)
    fc.allreduce_sim(dev16(x), group, b_rs, b_ag, out=y)
    torch.cuda.synchronize()
    edge = raw.cpu().numpy()
    assert (edge[:guard] == 7.0).all() and (edge[guard + t * h:] == 7.0).all(), "write outside the output"
    return y.cpu().numpy()


def three_steps(fc, x, group, b_rs, b_ag):
    n, t, h = x.shape
    xd = dev16(x)
    parts = [fc.quantize(xd[j], group, b_rs) for j in range(n)]
    c = torch.stack([p[0] for p in parts]); s = torch.stack([p[1] for p in parts]); z = torch.stack([p[2] for p in parts])
    co, so, zo = fc.dequant_reduce_requant(c, s, z, h, group, b_rs, b_ag)
    y = fc.dequantize(co, so, zo, h, group, b_ag)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def check(got, want, what):
    g = np.ascontiguousarray(got).view(np.uint16); w = np.ascontiguousarray(want).view(np.uint16)
    if g.tobytes() != w.tobytes():
        idx = np.flatnonzero(g.ravel() != w.ravel())
        raise AssertionError("%s: %d mismatches, first at %s: gpu=%s ref=%s" % (
            what, idx.size, idx[:5], got.ravel()[idx[:5]], want.ravel()[idx[:5]]))


@pytest.mark.parametrize("bits_rs,bits_ag", [(4, 4), (8, 8), (4, 8), (8, 4)])
@pytest.mark.parametrize("n_src", [1, 2, 3, 4, 5, 6, 7, 8])
def test_every_fan_in_and_bit_width_pair(fc, bits_rs, bits_ag, n_src):
    # 129 rows of 8192: 516 whole workgroup tiles of 2048 elements; 1% outlier channels as in the workloads
    x = synth_inputs.make_partials(n_src, 129, 8192, seed=100 + n_src, outlier_frac=0.01)
    got = run_sim(fc, x, 128, bits_rs, bits_ag)
    check(got, oracle.allreduce_sim(x, 128, bits_rs, bits_ag), "N=%d %d->%d" % (n_src, bits_rs, bits_ag))


RAGGED = [(t, h, g) for (t, h) in ((257, 5120), (1025, 1024), (911, 1152), (1000, 1056))
          for g in (32, 64, 128, 256, 512, 1024) if h % g == 0]


@pytest.mark.parametrize("tokens,hidden,group", RAGGED)
def test_group_sizes_and_ragged_tails(fc, tokens, hidden, group):
    # 257 x 5120 and 1025 x 1024 end after the first wavefront of a workgroup tile, 911 x 1152 and 1000 x 1056 in
    # the middle of a wavefront
    x = synth_inputs.make_partials(3, tokens, hidden, seed=group + tokens, outlier_frac=0.01)
    for b_rs, b_ag in ((4, 4), (8, 8)):
        got = run_sim(fc, x, group, b_rs, b_ag)
        check(got, oracle.allreduce_sim(x, group, b_rs, b_ag), "g=%d %dx%d %d->%d" % (group, tokens, hidden, b_rs, b_ag))


@pytest.mark.parametrize("kind", range(synth_inputs.STRESS_KINDS))
def test_corner_reaching_distributions(fc, kind):
    # per-row scales over 22 octaves, bands on large offsets (zero-points in the hundreds of thousands),
    # half-integers (ties), sparse spikes, micro-noise on constants
    for n_src, group in ((2, 32), (4, 128), (8, 1024)):
        x = synth_inputs.make_partials_stress(n_src, 130, 8192, kind, seed=7 * kind + n_src)
        for b_rs, b_ag in ((4, 4), (8, 8), (4, 8)):
            got = run_sim(fc, x, group, b_rs, b_ag)
            check(got, oracle.allreduce_sim(x, group, b_rs, b_ag),
                  "kind %d N=%d g=%d %d->%d" % (kind, n_src, group, b_rs, b_ag))


@pytest.mark.parametrize("group", [32, 128, 512])
def test_hand_picked_hard_groups(fc, group):
    # constant, one-sided, zero, tiny-range-on-offset, binary16-extreme and subnormal groups, tiled to the volume;
    # the partials carry the rows in different orders so that hard groups meet ordinary ones in the sum
    rows = synth_inputs.adversarial_groups(group, seed=group)              # [r, 8 * group]
    hidden = rows.shape[1]
    reps = SMALL_LIMIT // (rows.shape[0] * hidden) + 2
    base = np.tile(rows, (reps, 1))
    x = np.stack([np.roll(base, j, axis=0) if j % 2 == 0 else np.roll(base[:, ::-1].copy(), j, axis=0)
                  for j in range(4)])
    for b_rs, b_ag in ((4, 4), (8, 8), (8, 4)):
        got = run_sim(fc, x, group, b_rs, b_ag)
        check(got, oracle.allreduce_sim(x, group, b_rs, b_ag), "hard groups g=%d %d->%d" % (group, b_rs, b_ag))


@pytest.mark.parametrize("n_src,group,bits", [(4, 128, 4), (8, 64, 4), (2, 256, 8)])
def test_identical_to_the_three_kernel_sequence(fc, n_src, group, bits):
    x = synth_inputs.make_partials(n_src, 160, 8192, seed=n_src * group, outlier_frac=0.01)
    check(run_sim(fc, x, group, bits, bits), three_steps(fc, x, group, bits, bits), "one launch vs three")


def test_under_graph_capture_and_replay(fc):
    # the call only enqueues one kernel: captured once, replayed on new inputs with eager work in between
    n, t, h, g = 4, 136, 8192, 128
    xd = torch.zeros((n, t, h), dtype=torch.float16, device="cuda")
    y = torch.zeros((t, h), dtype=torch.float16, device="cuda")
    ws = torch.empty(fc.allreduce_sim_workspace_bytes(n, t, h, g, 4, 4), dtype=torch.uint8, device="cuda")
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        fc.allreduce_sim(xd, g, 4, 4, out=y, workspace=ws)           # warm-up outside capture
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        fc.allreduce_sim(xd, g, 4, 4, out=y, workspace=ws)
    for rep in range(3):
        x = synth_inputs.make_partials(n, t, h, seed=900 + rep, outlier_frac=0.01)
        xd.copy_(dev16(x))
        _ = (xd.float().sum()).item()                                    # eager work and a synchronization
        graph.replay()
        torch.cuda.synchronize()
        check(y.cpu().numpy(), oracle.allreduce_sim(x, g, 4, 4), "replay %d" % rep)


# --------------------------------------------------------------------------- #
# the other quantizers: symmetric (Eq. 3-4), FP8 E4M3, asymmetric with binary16 metadata
# --------------------------------------------------------------------------- #

def variant(fc, name):
    if name == "sym":
        return (lambda xd, g, bi, bo: fc.allreduce_sim_sym(xd, g, bi, bo)), \
               (lambda x, g, bi, bo: oracle.allreduce_sim_sym(x, g, bi, bo))
    if name == "fp8":
        return (lambda xd, g, bi, bo: fc.allreduce_sim_fp8(xd, g)), (lambda x, g, bi, bo: oracle.allreduce_sim_fp8(x, g))
    return (lambda xd, g, bi, bo: fc.allreduce_sim_cmeta(xd, g, bi, bo)), \
           (lambda x, g, bi, bo: oracle.allreduce_sim_cmeta(x, g, bi, bo))


def bit_pairs(name):
    return ((8, 8),) if name == "fp8" else ((4, 4), (8, 8), (4, 8), (8, 4))


@pytest.mark.parametrize("name", ["sym", "fp8", "cmeta"])
@pytest.mark.parametrize("n_src", [1, 2, 3, 4, 5, 6, 7, 8])
def test_variants_every_fan_in_and_bit_width_pair(fc, name, n_src):
    gpu, ref = variant(fc, name)
    x = synth_inputs.make_partials(n_src, 40, 4096, seed=300 + n_src, outlier_frac=0.01)
    xd = dev16(x)
    for bi, bo in bit_pairs(name):
        got = gpu(xd, 128, bi, bo)
        torch.cuda.synchronize()
        check(got.cpu().numpy(), ref(x, 128, bi, bo), "%s N=%d %d->%d" % (name, n_src, bi, bo))


@pytest.mark.parametrize("name", ["sym", "fp8", "cmeta"])
@pytest.mark.parametrize("tokens,hidden", [(1, 32), (3, 1056), (7, 2080), (33, 4096 + 1024), (9, 1152)])
def test_variants_group_sizes_and_ragged_tails(fc, name, tokens, hidden):
    gpu, ref = variant(fc, name)
    x = synth_inputs.make_partials(3, tokens, hidden, seed=tokens + hidden, outlier_frac=0.01)
    xd = dev16(x)
    for group in (32, 64, 128, 256, 512, 1024):
        if hidden % group:
            continue
        for bi, bo in bit_pairs(name)[:2]:
            got = gpu(xd, group, bi, bo)
            torch.cuda.synchronize()
            check(got.cpu().numpy(), ref(x, group, bi, bo), "%s g=%d %dx%d %d->%d" % (name, group, tokens, hidden, bi, bo))


@pytest.mark.parametrize("name", ["sym", "fp8", "cmeta"])
@pytest.mark.parametrize("kind", range(synth_inputs.STRESS_KINDS))
def test_variants_corner_reaching_distributions(fc, name, kind):
    gpu, ref = variant(fc, name)
    for n_src, group in ((2, 32), (4, 128), (8, 1024)):
        x = synth_inputs.make_partials_stress(n_src, 12, 8192, kind, seed=11 * kind + n_src)
        xd = dev16(x)
        for bi, bo in bit_pairs(name):
            got = gpu(xd, group, bi, bo)
            torch.cuda.synchronize()
            check(got.cpu().numpy(), ref(x, group, bi, bo), "%s kind %d N=%d g=%d %d->%d" % (name, kind, n_src, group, bi, bo))


@pytest.mark.parametrize("name", ["sym", "fp8", "cmeta"])
@pytest.mark.parametrize("group", [32, 128, 512])
def test_variants_hand_picked_hard_groups(fc, name, group):
    gpu, ref = variant(fc, name)
    rows = synth_inputs.adversarial_groups(group, seed=group + 1)
    base = np.tile(rows, (3, 1))
    x = np.stack([np.roll(base, j, axis=0) if j % 2 == 0 else np.roll(base[:, ::-1].copy(), j, axis=0)
                  for j in range(4)])
    xd = dev16(x)
    for bi, bo in bit_pairs(name):
        got = gpu(xd, group, bi, bo)
        torch.cuda.synchronize()
        check(got.cpu().numpy(), ref(x, group, bi, bo), "%s hard groups g=%d %d->%d" % (name, group, bi, bo))


def test_variants_identical_to_their_three_kernel_sequences(fc):
    n, t, h, g = 4, 24, 8192, 128
    x = synth_inputs.make_partials(n, t, h, seed=77, outlier_frac=0.01)
    xd = dev16(x)
    # symmetric
    parts = [fc.quantize_sym(xd[j], g, 4) for j in range(n)]
    co, so = fc.dequant_reduce_requant_sym(torch.stack([p[0] for p in parts]), torch.stack([p[1] for p in parts]), h, g, 4, 8)
    check(fc.allreduce_sim_sym(xd, g, 4, 8).cpu().numpy(), fc.dequantize_sym(co, so, h, g, 8).cpu().numpy(), "sym")
    # FP8
    parts = [fc.quantize_fp8(xd[j], g) for j in range(n)]
    co, so = fc.dequant_reduce_requant_fp8(torch.stack([p[0] for p in parts]), torch.stack([p[1] for p in parts]), h, g)
    check(fc.allreduce_sim_fp8(xd, g).cpu().numpy(), fc.dequantize_fp8(co, so, h, g).cpu().numpy(), "fp8")
    # binary16 metadata
    parts = [fc.quantize_cmeta(xd[j], g, 8) for j in range(n)]
    co, mo = fc.dequant_reduce_requant_cmeta(torch.stack([p[0] for p in parts]), torch.stack([p[1] for p in parts]), h, g, 8, 4)
    check(fc.allreduce_sim_cmeta(xd, g, 8, 4).cpu().numpy(), fc.dequantize_cmeta(co, mo, h, g, 4).cpu().numpy(), "cmeta")


@pytest.mark.parametrize("which", ["asym", "sym"])
def test_volume_beyond_2_to_32_elements(fc, which):
    # 2^32 + 24576 elements per partial through the one-launch kernel: element indices, the byte offset of the
    # second partial and the byte offsets inside a partial all pass 2^32; sampled token rows against the oracle
    # (groups never cross rows)
    hidden, group, bits = 8192, 128, 4
    tokens = (1 << 19) + 3
    free, _ = torch.cuda.mem_get_info()
    if free < 60 * (1 << 30):
        pytest.skip("needs 60 GB of free device memory")
    g = torch.Generator(device="cuda"); g.manual_seed(19)
    x = torch.empty((2, tokens, hidden), dtype=torch.float16, device="cuda")
    chunk = 1 << 16
    for r0 in range(0, tokens, chunk):
        r1 = min(tokens, r0 + chunk)
        x[0, r0:r1] = (torch.randn((r1 - r0, hidden), generator=g, device="cuda") * (1.0 + (r0 // chunk) % 3)).half()
    x[1] = x[0].flip(1) * 0.5
    y = torch.full((tokens, hidden), 7.0, dtype=torch.float16, device="cuda")
    L = fc.lib()
    need = L.fc_allreduce_sim_workspace_bytes(2, tokens, hidden, group, bits, bits)
    ws = torch.full((need,), 0x5A, dtype=torch.uint8, device="cuda")     # the one-launch kernel leaves it untouched
    fn = L.fc_allreduce_sim if which == "asym" else L.fc_allreduce_sim_sym
    rc = fn(x.data_ptr(), 2, tokens, hidden, group, bits, bits, y.data_ptr(), ws.data_ptr(), ws.numel(),
            torch.cuda.current_stream().cuda_stream)
    assert rc == 0
    torch.cuda.synchronize()
    assert bool((ws == 0x5A).all()), "the one-launch kernel wrote to the workspace"
    marks = [0, 1, (1 << 32) // hidden - 1, (1 << 32) // hidden, (1 << 31) // hidden, (1 << 18) + 1,
             tokens - 3, tokens - 2, tokens - 1]
    rows = np.unique(np.array(marks + list(np.random.default_rng(18).integers(0, tokens, 16))))
    ridx = torch.from_numpy(rows).cuda()
    xs = x[:, ridx].cpu().numpy()
    ref = oracle.allreduce_sim if which == "asym" else oracle.allreduce_sim_sym
    check(y[ridx].cpu().numpy(), ref(xs, group, bits, bits), "rows around 2^32 elements, " + which)
    # nothing outside the sampled rows is left unwritten: the fill value 7.0 would survive only by accident
    assert int((y == 7.0).sum().item()) < tokens
