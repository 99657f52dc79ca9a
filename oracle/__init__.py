"""numpy front end of the plain-C CPU oracle (``fc_oracle.c``).

Test infrastructure only: tests, the smoke check and the benchmark's
CPU-baseline leg import this; the GPU package never does.  All arrays are host
numpy arrays; nothing here touches a GPU or the HIP library.

Array conventions (Algorithm 1 of the paper; groups run along ``hidden``):
  x_f16   uint16 view or float16 ``[tokens, hidden]``
  codes   uint8 ``[tokens, hidden*bits/8]`` (INT4: element 2k low nibble, 2k+1 high)
  scales  float32 ``[tokens, hidden/group]``
  zeros   float32 ``[tokens, hidden/group]`` (integer-valued, not clamped)
  meta    uint32 ``[tokens, hidden/group]`` (compact variant: binary16 scale | binary16 zero << 16)
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fc_oracle.c")
_LIB = os.path.join(_HERE, "libfc_oracle.so")

CFLAGS = ["-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared"]


def build(force: bool = False) -> str:
    """Compile fc_oracle.c with the host C compiler; returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.run(["gcc", *CFLAGS, "-o", tmp, _SRC, "-lm"], check=True)
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        i64, i32, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
        L.fc_ref_half_to_float.restype = ctypes.c_float
        L.fc_ref_half_to_float.argtypes = [ctypes.c_uint16]
        L.fc_ref_float_to_half.restype = ctypes.c_uint16
        L.fc_ref_float_to_half.argtypes = [ctypes.c_float]
        L.fc_ref_quantize_group_f32.restype = None
        L.fc_ref_quantize_group_f32.argtypes = [vp, i32, i32, vp, vp, vp]
        L.fc_ref_quantize_f32.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp]
        L.fc_ref_quantize.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp]
        L.fc_ref_dequantize_f32.argtypes = [vp, vp, vp, i64, i64, i32, i32, vp]
        L.fc_ref_dequantize.argtypes = [vp, vp, vp, i64, i64, i32, i32, vp]
        L.fc_ref_dequant_reduce_f32.argtypes = [vp, i64, vp, vp, i64, i32, i64, i64, i32, i32, vp]
        L.fc_ref_dequant_reduce_requant.argtypes = [vp, i64, vp, vp, i64, i32, i64, i64, i32, i32,
                                                    i32, vp, vp, vp]
        L.fc_ref_allreduce_sim.argtypes = [vp, i32, i64, i64, i32, i32, i32, vp]
        L.fc_ref_quantize_group_sym_f32.restype = None
        L.fc_ref_quantize_group_sym_f32.argtypes = [vp, i32, i32, vp, vp]
        L.fc_ref_quantize_sym_f32.argtypes = [vp, i64, i64, i32, i32, vp, vp]
        L.fc_ref_quantize_sym.argtypes = [vp, i64, i64, i32, i32, vp, vp]
        L.fc_ref_dequantize_sym_f32.argtypes = [vp, vp, i64, i64, i32, i32, vp]
        L.fc_ref_dequantize_sym.argtypes = [vp, vp, i64, i64, i32, i32, vp]
        L.fc_ref_dequant_reduce_sym_f32.argtypes = [vp, i64, vp, i64, i32, i64, i64, i32, i32, vp]
        L.fc_ref_dequant_reduce_requant_sym.argtypes = [vp, i64, vp, i64, i32, i64, i64, i32, i32, i32,
                                                        vp, vp]
        L.fc_ref_allreduce_sim_sym.argtypes = [vp, i32, i64, i64, i32, i32, i32, vp]
        L.fc_ref_e4m3_to_float.restype = ctypes.c_float
        L.fc_ref_e4m3_to_float.argtypes = [ctypes.c_uint8]
        L.fc_ref_float_to_e4m3.restype = ctypes.c_uint8
        L.fc_ref_float_to_e4m3.argtypes = [ctypes.c_float]
        L.fc_ref_quantize_group_fp8_f32.restype = None
        L.fc_ref_quantize_group_fp8_f32.argtypes = [vp, i32, vp, vp]
        L.fc_ref_quantize_fp8_f32.argtypes = [vp, i64, i64, i32, vp, vp]
        L.fc_ref_quantize_fp8.argtypes = [vp, i64, i64, i32, vp, vp]
        L.fc_ref_dequantize_fp8_f32.argtypes = [vp, vp, i64, i64, i32, vp]
        L.fc_ref_dequantize_fp8.argtypes = [vp, vp, i64, i64, i32, vp]
        L.fc_ref_dequant_reduce_fp8_f32.argtypes = [vp, i64, vp, i64, i32, i64, i64, i32, vp]
        L.fc_ref_dequant_reduce_requant_fp8.argtypes = [vp, i64, vp, i64, i32, i64, i64, i32, vp, vp]
        L.fc_ref_allreduce_sim_fp8.argtypes = [vp, i32, i64, i64, i32, vp]
        L.fc_ref_hadamard_f32.argtypes = [vp, i64]
        L.fc_ref_hadamard_blocks_f32.argtypes = [vp, i64]
        L.fc_ref_quantize_rot.argtypes = [vp, i64, i64, i32, i32, i32, vp, vp, vp]
        L.fc_ref_dequantize_rot.argtypes = [vp, vp, vp, i64, i64, i32, i32, i32, vp]
        L.fc_ref_allreduce_sim_rot.argtypes = [vp, i32, i64, i64, i32, i32, i32, i32, vp]
        L.fc_ref_quantize_group_cmeta_f32.restype = None
        L.fc_ref_quantize_group_cmeta_f32.argtypes = [vp, i32, i32, vp, vp]
        L.fc_ref_quantize_cmeta_f32.argtypes = [vp, i64, i64, i32, i32, vp, vp]
        L.fc_ref_quantize_cmeta.argtypes = [vp, i64, i64, i32, i32, vp, vp]
        L.fc_ref_dequantize_cmeta_f32.argtypes = [vp, vp, i64, i64, i32, i32, vp]
        L.fc_ref_dequantize_cmeta.argtypes = [vp, vp, i64, i64, i32, i32, vp]
        L.fc_ref_dequant_reduce_cmeta_f32.argtypes = [vp, i64, vp, i64, i32, i64, i64, i32, i32, vp]
        L.fc_ref_dequant_reduce_requant_cmeta.argtypes = [vp, i64, vp, i64, i32, i64, i64, i32, i32, i32,
                                                          vp, vp]
        L.fc_ref_allreduce_sim_cmeta.argtypes = [vp, i32, i64, i64, i32, i32, i32, vp]
        for name in ("fc_ref_quantize_cmeta_f32", "fc_ref_quantize_cmeta", "fc_ref_dequantize_cmeta_f32",
                     "fc_ref_dequantize_cmeta", "fc_ref_dequant_reduce_cmeta_f32",
                     "fc_ref_dequant_reduce_requant_cmeta", "fc_ref_allreduce_sim_cmeta"):
            getattr(L, name).restype = i32
        for name in ("fc_ref_hadamard_f32", "fc_ref_hadamard_blocks_f32", "fc_ref_quantize_rot", "fc_ref_dequantize_rot",
                     "fc_ref_allreduce_sim_rot"):
            getattr(L, name).restype = i32
        for name in ("fc_ref_quantize_fp8_f32", "fc_ref_quantize_fp8", "fc_ref_dequantize_fp8_f32",
                     "fc_ref_dequantize_fp8", "fc_ref_dequant_reduce_fp8_f32",
                     "fc_ref_dequant_reduce_requant_fp8", "fc_ref_allreduce_sim_fp8"):
            getattr(L, name).restype = i32
        for name in ("fc_ref_quantize_f32", "fc_ref_quantize", "fc_ref_dequantize_f32",
                     "fc_ref_dequantize", "fc_ref_dequant_reduce_f32",
                     "fc_ref_dequant_reduce_requant", "fc_ref_allreduce_sim",
                     "fc_ref_quantize_sym_f32", "fc_ref_quantize_sym", "fc_ref_dequantize_sym_f32",
                     "fc_ref_dequantize_sym", "fc_ref_dequant_reduce_sym_f32",
                     "fc_ref_dequant_reduce_requant_sym", "fc_ref_allreduce_sim_sym"):
            getattr(L, name).restype = i32
        _lib = L
    return _lib


def _p(a: np.ndarray) -> ctypes.c_void_p:
    return ctypes.c_void_p(a.ctypes.data)


def _chk(rc: int, what: str) -> None:
    if rc != 0:
        raise ValueError("%s: oracle returned %d (bad argument or out of memory)" % (what, rc))


def _as_u16(x) -> np.ndarray:
    x = np.asarray(x)
    if x.dtype == np.float16:
        x = x.view(np.uint16)
    if x.dtype != np.uint16:
        raise TypeError("expected float16 (or its uint16 bits), got %s" % x.dtype)
    return np.ascontiguousarray(x)


def half_to_float(bits: int) -> float:
    return float(lib().fc_ref_half_to_float(int(bits)))


def float_to_half(x: float) -> int:
    return int(lib().fc_ref_float_to_half(float(np.float32(x))))


def quantize_group_f32(x, bits: int):
    """Eq. 1-2 on one group of fp32 values -> (codes uint8[g] unpacked, scale, zero)."""
    x = np.ascontiguousarray(x, dtype=np.float32).ravel()
    q = np.zeros(x.size, np.uint8)
    s = np.zeros(1, np.float32)
    z = np.zeros(1, np.float32)
    lib().fc_ref_quantize_group_f32(_p(x), x.size, bits, _p(q), _p(s), _p(z))
    return q, s[0], z[0]


def _alloc_q(tokens: int, hidden: int, group: int, bits: int):
    codes = np.zeros((tokens, hidden * bits // 8), np.uint8)
    scales = np.zeros((tokens, hidden // group), np.float32)
    zeros = np.zeros((tokens, hidden // group), np.float32)
    return codes, scales, zeros


def quantize_f32(x, group: int, bits: int):
    x = np.ascontiguousarray(x, dtype=np.float32)
    t, h = x.shape
    _chk(0 if (h % group == 0 and bits in (4, 8)) else -1, "quantize_f32")
    c, s, z = _alloc_q(t, h, group, bits)
    _chk(lib().fc_ref_quantize_f32(_p(x), t, h, group, bits, _p(c), _p(s), _p(z)), "quantize_f32")
    return c, s, z


def quantize(x_f16, group: int, bits: int):
    x = _as_u16(x_f16)
    t, h = x.shape
    _chk(0 if (h % group == 0 and bits in (4, 8)) else -1, "quantize")
    c, s, z = _alloc_q(t, h, group, bits)
    _chk(lib().fc_ref_quantize(_p(x), t, h, group, bits, _p(c), _p(s), _p(z)), "quantize")
    return c, s, z


def dequantize_f32(codes, scales, zeros, hidden: int, group: int, bits: int):
    codes = np.ascontiguousarray(codes, np.uint8)
    scales = np.ascontiguousarray(scales, np.float32)
    zeros = np.ascontiguousarray(zeros, np.float32)
    t = codes.shape[0]
    y = np.zeros((t, hidden), np.float32)
    _chk(lib().fc_ref_dequantize_f32(_p(codes), _p(scales), _p(zeros), t, hidden, group, bits, _p(y)),
         "dequantize_f32")
    return y


def dequantize(codes, scales, zeros, hidden: int, group: int, bits: int):
    codes = np.ascontiguousarray(codes, np.uint8)
    scales = np.ascontiguousarray(scales, np.float32)
    zeros = np.ascontiguousarray(zeros, np.float32)
    t = codes.shape[0]
    y = np.zeros((t, hidden), np.uint16)
    _chk(lib().fc_ref_dequantize(_p(codes), _p(scales), _p(zeros), t, hidden, group, bits, _p(y)),
         "dequantize")
    return y.view(np.float16)


def _stacked(codes_in, scales_in, zeros_in):
    c = np.ascontiguousarray(codes_in, np.uint8)
    s = np.ascontiguousarray(scales_in, np.float32)
    z = np.ascontiguousarray(zeros_in, np.float32)
    if c.ndim != 3 or s.ndim != 3 or z.shape != s.shape or s.shape[0] != c.shape[0]:
        raise ValueError("expected codes [N,T,bytes], scales/zeros [N,T,groups]")
    return c, s, z


def dequant_reduce_f32(codes_in, scales_in, zeros_in, hidden: int, group: int, bits_in: int):
    """fp32 FMA-chain sum of the N dequantized sources (stacked on axis 0)."""
    c, s, z = _stacked(codes_in, scales_in, zeros_in)
    n, t = c.shape[0], c.shape[1]
    acc = np.zeros((t, hidden), np.float32)
    _chk(lib().fc_ref_dequant_reduce_f32(_p(c), c[0].nbytes, _p(s), _p(z), s[0].size, n, t, hidden,
                                         group, bits_in, _p(acc)), "dequant_reduce_f32")
    return acc


def dequant_reduce_requant(codes_in, scales_in, zeros_in, hidden: int, group: int,
                           bits_in: int, bits_out: int):
    c, s, z = _stacked(codes_in, scales_in, zeros_in)
    n, t = c.shape[0], c.shape[1]
    co, so, zo = _alloc_q(t, hidden, group, bits_out)
    _chk(lib().fc_ref_dequant_reduce_requant(_p(c), c[0].nbytes, _p(s), _p(z), s[0].size, n, t,
                                             hidden, group, bits_in, bits_out,
                                             _p(co), _p(so), _p(zo)), "dequant_reduce_requant")
    return co, so, zo


def allreduce_sim(x_f16, group: int, bits_rs: int, bits_ag: int):
    """x_f16: [N, tokens, hidden] float16 -> [tokens, hidden] float16."""
    x = _as_u16(x_f16)
    n, t, h = x.shape
    y = np.zeros((t, h), np.uint16)
    _chk(lib().fc_ref_allreduce_sim(_p(x), n, t, h, group, bits_rs, bits_ag, _p(y)), "allreduce_sim")
    return y.view(np.float16)


# --------------------------------------------------------------------------- #
# symmetric variant (Eq. 3-4): signed codes in two's complement, scales only
# --------------------------------------------------------------------------- #

def quantize_group_sym_f32(x, bits: int):
    """Eq. 3-4 on one group of fp32 values -> (signed codes int8[g] unpacked, scale)."""
    x = np.ascontiguousarray(x, dtype=np.float32).ravel()
    q = np.zeros(x.size, np.int8)
    s = np.zeros(1, np.float32)
    lib().fc_ref_quantize_group_sym_f32(_p(x), x.size, bits, _p(q), _p(s))
    return q, s[0]


def quantize_sym_f32(x, group: int, bits: int):
    x = np.ascontiguousarray(x, dtype=np.float32)
    t, h = x.shape
    _chk(0 if (h % group == 0 and bits in (4, 8)) else -1, "quantize_sym_f32")
    c, s, _ = _alloc_q(t, h, group, bits)
    _chk(lib().fc_ref_quantize_sym_f32(_p(x), t, h, group, bits, _p(c), _p(s)), "quantize_sym_f32")
    return c, s


def quantize_sym(x_f16, group: int, bits: int):
    x = _as_u16(x_f16)
    t, h = x.shape
    _chk(0 if (h % group == 0 and bits in (4, 8)) else -1, "quantize_sym")
    c, s, _ = _alloc_q(t, h, group, bits)
    _chk(lib().fc_ref_quantize_sym(_p(x), t, h, group, bits, _p(c), _p(s)), "quantize_sym")
    return c, s


def dequantize_sym_f32(codes, scales, hidden: int, group: int, bits: int):
    codes = np.ascontiguousarray(codes, np.uint8)
    scales = np.ascontiguousarray(scales, np.float32)
    t = codes.shape[0]
    y = np.zeros((t, hidden), np.float32)
    _chk(lib().fc_ref_dequantize_sym_f32(_p(codes), _p(scales), t, hidden, group, bits, _p(y)),
         "dequantize_sym_f32")
    return y


def dequantize_sym(codes, scales, hidden: int, group: int, bits: int):
    codes = np.ascontiguousarray(codes, np.uint8)
    scales = np.ascontiguousarray(scales, np.float32)
    t = codes.shape[0]
    y = np.zeros((t, hidden), np.uint16)
    _chk(lib().fc_ref_dequantize_sym(_p(codes), _p(scales), t, hidden, group, bits, _p(y)),
         "dequantize_sym")
    return y.view(np.float16)


def _stacked_sym(codes_in, scales_in):
    c = np.ascontiguousarray(codes_in, np.uint8)
    s = np.ascontiguousarray(scales_in, np.float32)
    if c.ndim != 3 or s.ndim != 3 or s.shape[0] != c.shape[0]:
        raise ValueError("expected codes [N,T,bytes], scales [N,T,groups]")
    return c, s


def dequant_reduce_sym_f32(codes_in, scales_in, hidden: int, group: int, bits_in: int):
    c, s = _stacked_sym(codes_in, scales_in)
    n, t = c.shape[0], c.shape[1]
    acc = np.zeros((t, hidden), np.float32)
    _chk(lib().fc_ref_dequant_reduce_sym_f32(_p(c), c[0].nbytes, _p(s), s[0].size, n, t, hidden, group,
                                             bits_in, _p(acc)), "dequant_reduce_sym_f32")
    return acc


def dequant_reduce_requant_sym(codes_in, scales_in, hidden: int, group: int, bits_in: int, bits_out: int):
    c, s = _stacked_sym(codes_in, scales_in)
    n, t = c.shape[0], c.shape[1]
    co, so, _ = _alloc_q(t, hidden, group, bits_out)
    _chk(lib().fc_ref_dequant_reduce_requant_sym(_p(c), c[0].nbytes, _p(s), s[0].size, n, t, hidden,
                                                 group, bits_in, bits_out, _p(co), _p(so)),
         "dequant_reduce_requant_sym")
    return co, so


def allreduce_sim_sym(x_f16, group: int, bits_rs: int, bits_ag: int):
    x = _as_u16(x_f16)
    n, t, h = x.shape
    y = np.zeros((t, h), np.uint16)
    _chk(lib().fc_ref_allreduce_sim_sym(_p(x), n, t, h, group, bits_rs, bits_ag, _p(y)),
         "allreduce_sim_sym")
    return y.view(np.float16)


# --------------------------------------------------------------------------- #
# FP8 E4M3 per-group symmetric variant: one E4M3 byte per element, scales only
# --------------------------------------------------------------------------- #

def e4m3_to_float(code: int) -> float:
    return float(lib().fc_ref_e4m3_to_float(int(code) & 0xFF))


def float_to_e4m3(x: float) -> int:
    return int(lib().fc_ref_float_to_e4m3(float(np.float32(x))))


def quantize_group_fp8_f32(x):
    """one group of fp32 values -> (E4M3 bytes uint8[g], scale)."""
    x = np.ascontiguousarray(x, dtype=np.float32).ravel()
    q = np.zeros(x.size, np.uint8)
    s = np.zeros(1, np.float32)
    lib().fc_ref_quantize_group_fp8_f32(_p(x), x.size, _p(q), _p(s))
    return q, s[0]


def quantize_fp8_f32(x, group: int):
    x = np.ascontiguousarray(x, dtype=np.float32)
    t, h = x.shape
    _chk(0 if h % group == 0 else -1, "quantize_fp8_f32")
    c, s, _ = _alloc_q(t, h, group, 8)
    _chk(lib().fc_ref_quantize_fp8_f32(_p(x), t, h, group, _p(c), _p(s)), "quantize_fp8_f32")
    return c, s


def quantize_fp8(x_f16, group: int):
    x = _as_u16(x_f16)
    t, h = x.shape
    _chk(0 if h % group == 0 else -1, "quantize_fp8")
    c, s, _ = _alloc_q(t, h, group, 8)
    _chk(lib().fc_ref_quantize_fp8(_p(x), t, h, group, _p(c), _p(s)), "quantize_fp8")
    return c, s


def dequantize_fp8_f32(codes, scales, hidden: int, group: int):
    codes = np.ascontiguousarray(codes, np.uint8)
    scales = np.ascontiguousarray(scales, np.float32)
    t = codes.shape[0]
    y = np.zeros((t, hidden), np.float32)
    _chk(lib().fc_ref_dequantize_fp8_f32(_p(codes), _p(scales), t, hidden, group, _p(y)), "dequantize_fp8_f32")
    return y


def dequantize_fp8(codes, scales, hidden: int, group: int):
    codes = np.ascontiguousarray(codes, np.uint8)
    scales = np.ascontiguousarray(scales, np.float32)
    t = codes.shape[0]
    y = np.zeros((t, hidden), np.uint16)
    _chk(lib().fc_ref_dequantize_fp8(_p(codes), _p(scales), t, hidden, group, _p(y)), "dequantize_fp8")
    return y.view(np.float16)


def dequant_reduce_fp8_f32(codes_in, scales_in, hidden: int, group: int):
    c, s = _stacked_sym(codes_in, scales_in)
    n, t = c.shape[0], c.shape[1]
    acc = np.zeros((t, hidden), np.float32)
    _chk(lib().fc_ref_dequant_reduce_fp8_f32(_p(c), c[0].nbytes, _p(s), s[0].size, n, t, hidden, group,
                                             _p(acc)), "dequant_reduce_fp8_f32")
    return acc


def dequant_reduce_requant_fp8(codes_in, scales_in, hidden: int, group: int):
    c, s = _stacked_sym(codes_in, scales_in)
    n, t = c.shape[0], c.shape[1]
    co, so, _ = _alloc_q(t, hidden, group, 8)
    _chk(lib().fc_ref_dequant_reduce_requant_fp8(_p(c), c[0].nbytes, _p(s), s[0].size, n, t, hidden,
                                                 group, _p(co), _p(so)), "dequant_reduce_requant_fp8")
    return co, so


def allreduce_sim_fp8(x_f16, group: int):
    x = _as_u16(x_f16)
    n, t, h = x.shape
    y = np.zeros((t, h), np.uint16)
    _chk(lib().fc_ref_allreduce_sim_fp8(_p(x), n, t, h, group, _p(y)), "allreduce_sim_fp8")
    return y.view(np.float16)


# --------------------------------------------------------------------------- #
# Hadamard rotation around the quantized all-reduce (quantizer: 0 asym, 1 sym, 2 fp8)
# --------------------------------------------------------------------------- #

ASYM, SYM, FP8 = 0, 1, 2


def hadamard_f32(x):
    """unnormalised Walsh-Hadamard transform (natural order) of the last axis, fp32 butterflies."""
    x = np.array(x, dtype=np.float32, order="C")
    n = x.shape[-1]
    flat = x.reshape(-1, n)
    for r in range(flat.shape[0]):
        row = np.ascontiguousarray(flat[r])
        _chk(lib().fc_ref_hadamard_f32(_p(row), n), "hadamard_f32")
        flat[r] = row
    return flat.reshape(x.shape)


def hadamard_blocks_f32(x):
    """the transform the rotated entry points apply to a row of any length: hadamard_f32 over every aligned
    block of B elements of the last axis, B the largest power of two dividing its length."""
    x = np.array(x, dtype=np.float32, order="C")
    n = x.shape[-1]
    flat = x.reshape(-1, n)
    for r in range(flat.shape[0]):
        row = np.ascontiguousarray(flat[r])
        _chk(lib().fc_ref_hadamard_blocks_f32(_p(row), n), "hadamard_blocks_f32")
        flat[r] = row
    return flat.reshape(x.shape)


def quantize_rot(x_f16, group: int, bits: int, quantizer: int = ASYM):
    """-> (codes, scales, zeros); zeros is all-zero and meaningless unless quantizer == ASYM."""
    x = _as_u16(x_f16)
    t, h = x.shape
    _chk(0 if (h % group == 0 and bits in (4, 8)) else -1, "quantize_rot")
    c, s, z = _alloc_q(t, h, group, bits)
    _chk(lib().fc_ref_quantize_rot(_p(x), t, h, group, bits, quantizer, _p(c), _p(s), _p(z)), "quantize_rot")
    return c, s, z


def dequantize_rot(codes, scales, zeros, hidden: int, group: int, bits: int, quantizer: int = ASYM):
    codes = np.ascontiguousarray(codes, np.uint8)
    scales = np.ascontiguousarray(scales, np.float32)
    zeros = np.ascontiguousarray(zeros if zeros is not None else np.zeros_like(scales), np.float32)
    t = codes.shape[0]
    y = np.zeros((t, hidden), np.uint16)
    _chk(lib().fc_ref_dequantize_rot(_p(codes), _p(scales), _p(zeros), t, hidden, group, bits, quantizer,
                                     _p(y)), "dequantize_rot")
    return y.view(np.float16)


def allreduce_sim_rot(x_f16, group: int, bits_rs: int, bits_ag: int, quantizer: int = ASYM):
    x = _as_u16(x_f16)
    n, t, h = x.shape
    y = np.zeros((t, h), np.uint16)
    _chk(lib().fc_ref_allreduce_sim_rot(_p(x), n, t, h, group, bits_rs, bits_ag, quantizer, _p(y)),
         "allreduce_sim_rot")
    return y.view(np.float16)


# --------------------------------------------------------------------------- #
# asymmetric quantizer with binary16 metadata: one uint32 word per group,
# bits 0-15 the scale, bits 16-31 the zero-point (both binary16)
# --------------------------------------------------------------------------- #

def meta_unpack(meta):
    """uint32 words -> (scales, zeros) as the float32 values of the two binary16 halves."""
    m = np.ascontiguousarray(meta, np.uint32)
    s = (m & 0xFFFF).astype(np.uint16).view(np.float16).astype(np.float32)
    z = (m >> 16).astype(np.uint16).view(np.float16).astype(np.float32)
    return s, z


def quantize_group_cmeta_f32(x, bits: int):
    """one group of fp32 values -> (codes uint8[g] unpacked, metadata word)."""
    x = np.ascontiguousarray(x, dtype=np.float32).ravel()
    q = np.zeros(x.size, np.uint8)
    m = np.zeros(1, np.uint32)
    lib().fc_ref_quantize_group_cmeta_f32(_p(x), x.size, bits, _p(q), _p(m))
    return q, int(m[0])


def _alloc_cmeta(tokens: int, hidden: int, group: int, bits: int):
    return np.zeros((tokens, hidden * bits // 8), np.uint8), np.zeros((tokens, hidden // group), np.uint32)


def quantize_cmeta_f32(x, group: int, bits: int):
    x = np.ascontiguousarray(x, dtype=np.float32)
    t, h = x.shape
    _chk(0 if (h % group == 0 and bits in (4, 8)) else -1, "quantize_cmeta_f32")
    c, m = _alloc_cmeta(t, h, group, bits)
    _chk(lib().fc_ref_quantize_cmeta_f32(_p(x), t, h, group, bits, _p(c), _p(m)), "quantize_cmeta_f32")
    return c, m


def quantize_cmeta(x_f16, group: int, bits: int):
    x = _as_u16(x_f16)
    t, h = x.shape
    _chk(0 if (h % group == 0 and bits in (4, 8)) else -1, "quantize_cmeta")
    c, m = _alloc_cmeta(t, h, group, bits)
    _chk(lib().fc_ref_quantize_cmeta(_p(x), t, h, group, bits, _p(c), _p(m)), "quantize_cmeta")
    return c, m


def dequantize_cmeta_f32(codes, meta, hidden: int, group: int, bits: int):
    codes = np.ascontiguousarray(codes, np.uint8)
    meta = np.ascontiguousarray(meta, np.uint32)
    t = codes.shape[0]
    y = np.zeros((t, hidden), np.float32)
    _chk(lib().fc_ref_dequantize_cmeta_f32(_p(codes), _p(meta), t, hidden, group, bits, _p(y)),
         "dequantize_cmeta_f32")
    return y


def dequantize_cmeta(codes, meta, hidden: int, group: int, bits: int):
    codes = np.ascontiguousarray(codes, np.uint8)
    meta = np.ascontiguousarray(meta, np.uint32)
    t = codes.shape[0]
    y = np.zeros((t, hidden), np.uint16)
    _chk(lib().fc_ref_dequantize_cmeta(_p(codes), _p(meta), t, hidden, group, bits, _p(y)), "dequantize_cmeta")
    return y.view(np.float16)


def _stacked_cmeta(codes_in, meta_in):
    c = np.ascontiguousarray(codes_in, np.uint8)
    m = np.ascontiguousarray(meta_in, np.uint32)
    if c.ndim != 3 or m.ndim != 3 or m.shape[0] != c.shape[0]:
        raise ValueError("expected codes [N,T,bytes], meta [N,T,groups]")
    return c, m


def dequant_reduce_cmeta_f32(codes_in, meta_in, hidden: int, group: int, bits_in: int):
    c, m = _stacked_cmeta(codes_in, meta_in)
    n, t = c.shape[0], c.shape[1]
    acc = np.zeros((t, hidden), np.float32)
    _chk(lib().fc_ref_dequant_reduce_cmeta_f32(_p(c), c[0].nbytes, _p(m), m[0].size, n, t, hidden, group,
                                               bits_in, _p(acc)), "dequant_reduce_cmeta_f32")
    return acc


def dequant_reduce_requant_cmeta(codes_in, meta_in, hidden: int, group: int, bits_in: int, bits_out: int):
    c, m = _stacked_cmeta(codes_in, meta_in)
    n, t = c.shape[0], c.shape[1]
    co, mo = _alloc_cmeta(t, hidden, group, bits_out)
    _chk(lib().fc_ref_dequant_reduce_requant_cmeta(_p(c), c[0].nbytes, _p(m), m[0].size, n, t, hidden, group,
                                                   bits_in, bits_out, _p(co), _p(mo)),
         "dequant_reduce_requant_cmeta")
    return co, mo


def allreduce_sim_cmeta(x_f16, group: int, bits_rs: int, bits_ag: int):
    x = _as_u16(x_f16)
    n, t, h = x.shape
    y = np.zeros((t, h), np.uint16)
    _chk(lib().fc_ref_allreduce_sim_cmeta(_p(x), n, t, h, group, bits_rs, bits_ag, _p(y)), "allreduce_sim_cmeta")
    return y.view(np.float16)
