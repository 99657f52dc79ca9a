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


def declared_functions():
    text = open(os.path.join(ROOT, "include", "fc.h")).read()
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


def test_rotation_and_stream_reference_argument_checks(L):
    q = L.fc_quantize_rot
    assert q(P, 4, 1024, 128, 4, 0, P, P, P, None) == -4          # hidden must be 2048, 4096 or 8192
    assert q(P, 4, 6144, 128, 4, 0, P, P, P, None) == -4
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
    r = L.fc_stream_reference
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
