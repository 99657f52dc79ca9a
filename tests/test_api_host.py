"""Host-only checks of the C-ABI library: it loads, exports every function that
include/fc.h declares, and rejects bad arguments before touching a GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    import paper_2412_04964_amd as fc
    if not os.path.exists(fc.lib_path()):
        from paper_2412_04964_amd.build import build
        build()
    return fc.lib()


def declared_functions(header="fc.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fc_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(L):
    names = declared_functions()
    assert {"fc_quantize", "fc_dequant_reduce_requant", "fc_dequantize", "fc_allreduce_sim",
            "fc_allreduce_sim_workspace_bytes", "fc_strerror", "fc_last_hip_error",
            "fc_version"} <= set(names)
    for n in names:
        assert hasattr(L, n), n


def test_no_internal_symbols_leak(L):
    import subprocess
    import paper_2412_04964_amd as fc
    out = subprocess.run(["nm", "-D", "--defined-only", fc.lib_path()], capture_output=True, text=True).stdout
    exported = [l.split()[-1] for l in out.splitlines() if " T " in l]
    assert sorted(exported) == declared_functions()


P = 0x10000      # a fake, 16-byte aligned, non-NULL device address; never dereferenced


def test_quantize_argument_checks(L):
    q = L.fc_quantize
    assert q(P, 4, 256, 128, 5, P, P, P, None) == -2          # bits
    assert q(P, 4, 256, 100, 8, P, P, P, None) == -3          # group not a power of two
    assert q(P, 4, 256, 16, 8, P, P, P, None) == -3           # group too small
    assert q(P, 4, 32768, 32768, 8, P, P, P, None) == -3      # group too large
    assert q(P, 4, 192, 128, 8, P, P, P, None) == -3          # hidden % group
    assert q(P, -1, 256, 128, 8, P, P, P, None) == -4         # tokens
    assert q(P, 4, 0, 128, 8, P, P, P, None) == -4            # hidden
    assert q(P, 1 << 40, 1 << 20, 128, 8, P, P, P, None) == -4  # too many elements
    assert q(None, 4, 256, 128, 8, P, P, P, None) == -1
    assert q(P, 4, 256, 128, 8, P, None, P, None) == -1
    assert q(P + 8, 4, 256, 128, 8, P, P, P, None) == -5
    assert q(P, 4, 256, 128, 8, P, P, P + 4, None) == -5
    assert q(None, 0, 256, 128, 8, None, None, None, None) == 0   # empty input is a no-op


def test_fused_argument_checks(L):
    f = L.fc_dequant_reduce_requant
    ok = dict(tokens=4, hidden=256, group=128)
    cs, ms = 4 * 256 // 2, 8      # 4-bit slab bytes, groups per slab

    def call(codes=P, cstride=cs, sc=P, ze=P, mstride=ms, n=4, bits_in=4, bits_out=4, co=P, so=P, zo=P,
             **kw):
        a = dict(ok); a.update(kw)
        return f(codes, cstride, sc, ze, mstride, n, a["tokens"], a["hidden"], a["group"], bits_in,
                 bits_out, co, so, zo, None)

    assert call(bits_in=3) == -2 and call(bits_out=16) == -2
    assert call(n=0) == -4 and call(n=9) == -4
    assert call(cstride=cs - 16) == -4                        # slabs would overlap
    assert call(mstride=4) == -4
    assert call(cstride=cs + 8) == -5
    assert call(codes=None) == -1 and call(zo=None) == -1
    assert call(sc=P + 4) == -5
    assert call(group=64, hidden=96) == -3
    assert call(tokens=0, codes=None, sc=None, ze=None, co=None, so=None, zo=None) == 0


def test_dequantize_and_sim_argument_checks(L):
    d = L.fc_dequantize
    assert d(P, P, P, 4, 256, 128, 7, P, None) == -2
    assert d(P, P, P, 4, 256, 128, 8, None, None) == -1
    assert d(P, P, P, 4, 256, 128, 8, P + 2, None) == -5
    w = L.fc_allreduce_sim_workspace_bytes
    assert w(4, 4, 256, 128, 3, 4) == 0 and w(0, 4, 256, 128, 4, 4) == 0
    need = w(4, 16, 4096, 128, 4, 8)
    m = 16 * 4096
    assert need >= 4 * (m // 2 + 2 * 4 * m // 128) + m + 2 * 4 * m // 128
    s = L.fc_allreduce_sim
    assert s(P, 4, 16, 4096, 128, 4, 8, P, P, need - 1, None) == -6
    assert s(P, 4, 16, 4096, 128, 4, 8, P, None, need, None) == -6
    assert s(P, 4, 16, 4096, 128, 4, 9, P, P, need, None) == -2
    assert s(P, 9, 16, 4096, 128, 4, 8, P, P, need, None) == -4
    assert s(None, 4, 16, 4096, 128, 4, 8, P, P, need, None) == -1


def test_strerror_and_version(L):
    assert L.fc_version() >= 100
    for code in range(-8, 1):
        msg = L.fc_strerror(code)
        assert isinstance(msg, bytes) and len(msg) > 0
    assert L.fc_last_hip_error() == 0


def test_binding_refuses_cpu_tensors():
    torch = pytest.importorskip("torch")
    import paper_2412_04964_amd as fc
    with pytest.raises(TypeError):
        fc.quantize(torch.zeros(4, 256, dtype=torch.float16), 128, 8)


def test_variant_entry_points_argument_checks(L):
    # symmetric and FP8: the same checks minus the zero-point arrays
    assert L.fc_quantize_sym(P, 4, 256, 128, 5, P, P, None) == -2
    assert L.fc_quantize_sym(P, 4, 256, 128, 4, P, None, None) == -1
    assert L.fc_quantize_sym(P, 4, 256, 128, 4, P + 8, P, None) == -5
    assert L.fc_quantize_sym(None, 0, 256, 128, 4, None, None, None) == 0
    assert L.fc_quantize_fp8(P, 4, 256, 100, P, P, None) == -3
    assert L.fc_quantize_fp8(None, 4, 256, 128, P, P, None) == -1
    cs = 4 * 256
    assert L.fc_dequant_reduce_requant_fp8(P, cs - 16, P, 8, 4, 4, 256, 128, P, P, None) == -4
    assert L.fc_dequant_reduce_requant_fp8(P, cs, P, 1, 4, 4, 256, 128, P, P, None) == -4
    assert L.fc_dequant_reduce_requant_sym(P, cs // 2, P, 8, 9, 4, 256, 128, 4, 4, P, P, None) == -4
    assert L.fc_dequant_reduce_requant_sym(P, cs // 2, P, 8, 4, 4, 256, 128, 4, 4, P, None, None) == -1
    assert L.fc_dequantize_sym(P, P, 4, 256, 128, 4, None, None) == -1
    assert L.fc_dequantize_fp8(P, P + 4, 4, 256, 128, P, None) == -5
    need = L.fc_allreduce_sim_workspace_bytes(4, 16, 4096, 128, 8, 8)
    assert L.fc_allreduce_sim_fp8(P, 4, 16, 4096, 128, P, P, need - 1, None) == -6
    assert L.fc_allreduce_sim_sym(P, 4, 16, 4096, 128, 4, 4, P, None, need, None) == -6
    # binary16 metadata: one array of 32-bit words in place of scales and zero-points
    assert L.fc_quantize_cmeta(P, 4, 256, 128, 5, P, P, None) == -2
    assert L.fc_quantize_cmeta(P, 4, 256, 128, 4, P, None, None) == -1
    assert L.fc_quantize_cmeta(P, 4, 256, 128, 4, P, P + 4, None) == -5
    assert L.fc_quantize_cmeta(P, 4, 256, 48, 4, P, P, None) == -3
    assert L.fc_quantize_cmeta(None, 0, 256, 128, 4, None, None, None) == 0
    assert L.fc_dequant_reduce_requant_cmeta(P, cs // 2, P, 7, 4, 4, 256, 128, 4, 4, P, P, None) == -4
    assert L.fc_dequant_reduce_requant_cmeta(P, cs // 2, None, 8, 4, 4, 256, 128, 4, 4, P, P, None) == -1
    assert L.fc_dequant_reduce_requant_cmeta(P, cs // 2, P, 8, 4, 4, 256, 128, 4, 6, P, P, None) == -2
    assert L.fc_dequantize_cmeta(P, None, 4, 256, 128, 4, P, None) == -1
    need44 = L.fc_allreduce_sim_workspace_bytes(4, 16, 4096, 128, 4, 4)
    assert L.fc_allreduce_sim_cmeta(P, 4, 16, 4096, 128, 4, 4, P, P, need44 - 1, None) == -6
    assert L.fc_allreduce_sim_cmeta(P, 9, 16, 4096, 128, 4, 4, P, P, need, None) == -4


def test_bench_library_exports_exactly_its_header_and_the_product_library_none_of_it(L):
    import subprocess
    import paper_2412_04964_amd as fc
    B = fc.bench_lib()
    names = declared_functions("fc_bench.h")
    assert names == ["fc_fused_compute_probe", "fc_stream_reference"]
    out = subprocess.run(["nm", "-D", "--defined-only", B._name], capture_output=True, text=True).stdout
    assert sorted(l.split()[-1] for l in out.splitlines() if " T " in l) == names
    assert not hasattr(L, "fc_stream_reference")
    assert "fc_stream_reference" not in declared_functions()


def test_rotation_and_stream_reference_argument_checks(L):
    q = L.fc_quantize_rot
    # the largest power of two dividing hidden (the rotation's block) must be 1024 ... 8192
    assert q(P, 4, 512, 128, 4, 0, P, P, P, None) == -4
    assert q(P, 4, 2560, 128, 4, 0, P, P, P, None) == -4          # 5 x 512
    assert q(P, 4, 16384, 128, 4, 0, P, P, P, None) == -4
    assert q(P, 4, 4096 + 128, 128, 4, 0, P, P, P, None) == -4    # block 128
    assert q(P, 4, 4096, 128, 4, 3, P, P, P, None) == -4          # unknown quantizer
    assert q(P, 4, 4096, 128, 4, 2, P, P, P, None) == -2          # FP8 needs 8 bits
    assert q(P, 4, 4096, 128, 4, 0, P, P, None, None) == -1       # asymmetric needs zero-points
    assert q(P, 4, 4096, 8192, 4, 0, P, P, P, None) == -3         # group > hidden
    assert q(None, 0, 4096, 128, 4, 1, None, None, None, None) == 0
    d = L.fc_dequantize_rot
    assert d(P, P, None, 4, 4096, 128, 8, 0, P, None) == -1
    assert d(P, P, P, 4, 4096, 128, 8, 1, P + 2, None) == -5
    need = L.fc_allreduce_sim_workspace_bytes(4, 16, 4096, 128, 4, 8)
    s = L.fc_allreduce_sim_rot
    assert s(P, 4, 16, 4096, 128, 4, 8, 0, P, P, need - 1, None) == -6
    assert s(P, 4, 16, 4096, 128, 4, 8, 2, P, P, need, None) == -2
    assert s(P, 4, 16, 2560, 128, 4, 8, 0, P, P, need, None) == -4
    import paper_2412_04964_amd as fc
    r = fc.bench_lib().fc_stream_reference
    assert r(P, 4096, 4, 4096 + 8, P, None) == -4                 # bytes % 16
    assert r(P, 2048, 4, 4096, P, None) == -4                     # sources would overlap
    assert r(P, 4096, 0, 4096, P, None) == -4
    assert r(None, 4096, 4, 4096, P, None) == -1
    assert r(P, 4096, 4, 0, None, None) == 0


def test_header_is_plain_c_and_links_against_the_library(tmp_path, L):
    # include/fc.h must be usable from C99 and C++ and every declaration must resolve in libfc.so
    import subprocess
    import paper_2412_04964_amd as fc
    calls = "\n".join("    p[%d] = (void *)%s;" % (i, n) for i, n in enumerate(declared_functions()))
    src = tmp_path / "use_fc.c"
    src.write_text('#include "fc.h"\n#include <stdio.h>\nint main(void) {\n    void *p[64];\n%s\n'
                   '    printf("%%d %%s\\n", fc_version(), fc_strerror(FC_ERR_GROUP));\n    return p[0] == 0;\n}\n' % calls)
    inc = os.path.join(ROOT, "include")
    exe = tmp_path / "use_fc"
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-Wno-pedantic", "-I", inc, str(src),
                        fc.lib_path(), "-o", str(exe)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run(["g++", "-std=c++11", "-Wall", "-Wextra", "-fsyntax-only", "-x", "c++", "-I", inc, str(src)],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr


def test_missing_library_fails_loudly():
    # no CPU fallback: without libfc.so every compute entry of the binding raises at load time
    import subprocess
    import sys
    code = ("import paper_2412_04964_amd as fc\n"
            "try:\n    fc.lib()\nexcept ImportError as e:\n    print('ImportError:', e)\n    raise SystemExit(3)\n")
    env = dict(os.environ, FC_LIBRARY="/nonexistent/libfc.so", PYTHONPATH=ROOT)
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, env=env, cwd=ROOT)
    assert r.returncode == 3 and "no CPU fallback" in r.stdout, (r.returncode, r.stdout, r.stderr)


def test_binding_checks_every_tensor_against_the_geometry_before_the_c_call(monkeypatch):
    # The kernels take their buffer ranges from (tokens, hidden, group, bits): a tensor that disagrees with them
    # must be refused on the host.  CPU tensors stand in for device tensors here (the device check is switched
    # off) and the C library is replaced by an object that fails the test when any entry point is reached.
    torch = pytest.importorskip("torch")
    from paper_2412_04964_amd import binding as b

    class Unreachable:
        def __getattr__(self, name):
            if name in ("fc_strerror",):
                return lambda code: b"x"
            if name == "fc_last_hip_error":
                return lambda: 0
            if name == "fc_allreduce_sim_workspace_bytes":
                return lambda *a: 1 << 20
            raise AssertionError("C entry point %s reached with inconsistent tensors" % name)

    def dev(t, dtype, what):
        if t.dtype != dtype:
            raise TypeError(what)
        return t

    monkeypatch.setattr(b, "_dev", dev)
    monkeypatch.setattr(b, "lib", lambda: Unreachable())
    monkeypatch.setattr(b, "bench_lib", lambda: Unreachable())
    monkeypatch.setattr(b, "_stream", lambda: 0)
    f16, u8, f32, i32 = torch.float16, torch.uint8, torch.float32, torch.int32
    T, H, G = 4, 256, 128
    x = torch.zeros(T, H, dtype=f16)
    codes4 = torch.zeros(T, H // 2, dtype=u8); codes8 = torch.zeros(T, H, dtype=u8)
    meta = torch.zeros(T, H // G, dtype=f32)
    y = torch.zeros(T, H, dtype=f16)

    bad = pytest.raises(ValueError)
    with bad: b.quantize(x, G, 4, out=(codes8, meta, meta))                     # codes sized for 8 bit
    with bad: b.quantize(x, G, 4, out=(codes4, meta[:, :1], meta))              # too few scales
    with bad: b.quantize(x, G, 4, out=(codes4, meta, meta[:3]))                 # too few rows of zero-points
    with bad: b.quantize(x.view(-1), G, 4)                                      # not [tokens, hidden]
    with bad: b.quantize_sym(x, G, 8, out=(codes4, meta))
    with bad: b.quantize_fp8(x, G, out=(codes4, meta))
    with bad: b.quantize_cmeta(x, G, 4, out=(codes4, torch.zeros(T, 1, dtype=i32)))
    with bad: b.quantize_rot(x, G, 4, out=(codes8, meta, meta))
    with bad: b.dequantize(codes4, meta, meta, H, G, 8)                         # bits disagree with the codes
    with bad: b.dequantize(codes4, meta, meta, 2 * H, G, 4)                     # hidden disagrees
    with bad: b.dequantize(codes4, meta, meta[:, :1], H, G, 4)
    with bad: b.dequantize(codes4, meta, meta, H, G, 4, out=y[:2])              # short output
    with bad: b.dequantize_sym(codes8, meta, H, G, 4)
    with bad: b.dequantize_fp8(codes4, meta, H, G)
    with bad: b.dequantize_cmeta(codes4, torch.zeros(T, 1, dtype=i32), H, G, 4)
    with bad: b.dequantize_rot(codes4, meta, meta[:2], H, G, 4)
    c_in = torch.zeros(3, T, H // 2, dtype=u8); m_in = torch.zeros(3, T, H // G, dtype=f32)
    with bad: b.dequant_reduce_requant(c_in, m_in, m_in, H, G, 8, 8)            # bits_in disagrees with the codes
    with bad: b.dequant_reduce_requant(c_in, m_in[:2], m_in, H, G, 4, 4)        # fewer scale slabs than sources
    with bad: b.dequant_reduce_requant(c_in, m_in, m_in[:, :2], H, G, 4, 4)
    with bad: b.dequant_reduce_requant(c_in, m_in, m_in, H, G, 4, 8, out=(codes4, meta, meta))   # out sized for 4 bit
    with bad: b.dequant_reduce_requant(c_in[0], m_in[0], m_in[0], H, G, 4, 4)   # missing source axis
    with bad: b.dequant_reduce_requant_sym(c_in, m_in[:, :, :1], H, G, 4, 4)
    with bad: b.dequant_reduce_requant_fp8(c_in, m_in, H, G)
    with bad: b.dequant_reduce_requant_cmeta(c_in, torch.zeros(3, T, 1, dtype=i32), H, G, 4, 4)
    x3 = torch.zeros(2, T, H, dtype=f16)
    with bad: b.allreduce_sim(x3, G, 4, 4, out=y[:, :128])
    with bad: b.allreduce_sim(x, G, 4, 4)                                       # missing source axis
    with bad: b.allreduce_sim_static(x3, G, 4, 4, out=y[:3])
    with pytest.raises(b.FcError): b.allreduce_sim(x3, G, 4, 4, workspace=torch.zeros(16, dtype=u8))   # short workspace
    with pytest.raises(b.FcError): b.allreduce_sim(torch.zeros(9, T, H, dtype=f16), G, 4, 4)           # too many sources
    with bad: b.stream_reference(torch.zeros(2, 64, dtype=u8), torch.zeros(48, dtype=u8))
    # argument errors keep the C library's codes
    for call, code in ((lambda: b.quantize(x, G, 5), -2), (lambda: b.quantize(x, 96, 4), -3),
                       (lambda: b.quantize(x, 512, 4), -3), (lambda: b.dequantize(codes4, meta, meta, H, 16, 4), -3)):
        with pytest.raises(b.FcError) as ei:
            call()
        assert ei.value.code == code
    with pytest.raises(TypeError): b.quantize(x.float(), G, 4)


def test_binding_refuses_tensors_of_another_device(monkeypatch):
    # the C ABI works on the device that is current on the calling thread; a tensor of another device is refused
    torch = pytest.importorskip("torch")
    from paper_2412_04964_amd import binding as b

    class OnDevice1(torch.Tensor):
        is_cuda = property(lambda self: True)
        device = property(lambda self: torch.device("cuda", 1))

    monkeypatch.setattr(torch.cuda, "current_device", lambda: 0)
    fake = torch.zeros(2, 2, dtype=torch.float16).as_subclass(OnDevice1)
    with pytest.raises(ValueError, match="current device"):
        b._dev(fake, torch.float16, "x")


def test_the_user_scripts_import_and_describe_themselves_without_a_gpu():
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    for mod in ("paper_2412_04964_amd.volume_sweep", "paper_2412_04964_amd.ablation"):
        r = subprocess.run([sys.executable, "-m", mod, "--help"], capture_output=True, text=True, cwd=root, timeout=300)
        assert r.returncode == 0 and "usage" in r.stdout.lower(), mod + ": " + r.stderr[-500:]
