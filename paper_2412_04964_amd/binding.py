"""ctypes front end of libfc.so.  Same names as the C entry points, minus the
``fc_`` prefix.  Tensors must be contiguous torch tensors on the current CUDA
(HIP) device; outputs are allocated by torch when not supplied.  Every call is
asynchronous on ``torch.cuda.current_stream()``.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
# FC_LIBRARY overrides the location of the shared library (e.g. a differently tuned build)
_LIB_PATH = os.environ.get("FC_LIBRARY") or os.path.join(_HERE, "libfc.so")
_lib = None

FC_MAX_SRC = 8
QUANTIZER_ASYM, QUANTIZER_SYM, QUANTIZER_FP8 = 0, 1, 2


class FcError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        msg = lib().fc_strerror(code).decode()
        if code == -7:
            msg += " [hipError %d]" % lib().fc_last_hip_error()
        super().__init__("%s: %s (code %d)" % (what, msg, code))


def lib_path() -> str:
    return _LIB_PATH


def lib() -> ctypes.CDLL:
    """Load libfc.so (built by ``python -m paper_2412_04964_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(
                "%s not found: build it with `python -m paper_2412_04964_amd.build` "
                "(there is no CPU fallback)" % _LIB_PATH)
        L = ctypes.CDLL(_LIB_PATH)
        i64, i32, vp, sz = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
        L.fc_quantize.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp, vp]
        L.fc_quantize.restype = i32
        L.fc_dequant_reduce_requant.argtypes = [vp, i64, vp, vp, i64, i32, i64, i64, i32, i32, i32,
                                                vp, vp, vp, vp]
        L.fc_dequant_reduce_requant.restype = i32
        L.fc_dequantize.argtypes = [vp, vp, vp, i64, i64, i32, i32, vp, vp]
        L.fc_dequantize.restype = i32
        L.fc_allreduce_sim.argtypes = [vp, i32, i64, i64, i32, i32, i32, vp, vp, sz, vp]
        L.fc_allreduce_sim.restype = i32
        L.fc_allreduce_sim_static.argtypes = [vp, i32, i64, i64, i32, i32, i32, vp, vp]
        L.fc_allreduce_sim_static.restype = i32
        L.fc_allreduce_sim_workspace_bytes.argtypes = [i32, i64, i64, i32, i32, i32]
        L.fc_allreduce_sim_workspace_bytes.restype = sz
        L.fc_quantize_sym.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp]
        L.fc_quantize_sym.restype = i32
        L.fc_dequant_reduce_requant_sym.argtypes = [vp, i64, vp, i64, i32, i64, i64, i32, i32, i32,
                                                    vp, vp, vp]
        L.fc_dequant_reduce_requant_sym.restype = i32
        L.fc_dequantize_sym.argtypes = [vp, vp, i64, i64, i32, i32, vp, vp]
        L.fc_dequantize_sym.restype = i32
        L.fc_allreduce_sim_sym.argtypes = [vp, i32, i64, i64, i32, i32, i32, vp, vp, sz, vp]
        L.fc_allreduce_sim_sym.restype = i32
        L.fc_quantize_fp8.argtypes = [vp, i64, i64, i32, vp, vp, vp]
        L.fc_quantize_fp8.restype = i32
        L.fc_dequant_reduce_requant_fp8.argtypes = [vp, i64, vp, i64, i32, i64, i64, i32, vp, vp, vp]
        L.fc_dequant_reduce_requant_fp8.restype = i32
        L.fc_dequantize_fp8.argtypes = [vp, vp, i64, i64, i32, vp, vp]
        L.fc_dequantize_fp8.restype = i32
        L.fc_allreduce_sim_fp8.argtypes = [vp, i32, i64, i64, i32, vp, vp, sz, vp]
        L.fc_allreduce_sim_fp8.restype = i32
        L.fc_quantize_cmeta.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp]
        L.fc_quantize_cmeta.restype = i32
        L.fc_dequant_reduce_requant_cmeta.argtypes = [vp, i64, vp, i64, i32, i64, i64, i32, i32, i32,
                                                      vp, vp, vp]
        L.fc_dequant_reduce_requant_cmeta.restype = i32
        L.fc_dequantize_cmeta.argtypes = [vp, vp, i64, i64, i32, i32, vp, vp]
        L.fc_dequantize_cmeta.restype = i32
        L.fc_allreduce_sim_cmeta.argtypes = [vp, i32, i64, i64, i32, i32, i32, vp, vp, sz, vp]
        L.fc_allreduce_sim_cmeta.restype = i32
        L.fc_quantize_rot.argtypes = [vp, i64, i64, i32, i32, i32, vp, vp, vp, vp]
        L.fc_quantize_rot.restype = i32
        L.fc_dequantize_rot.argtypes = [vp, vp, vp, i64, i64, i32, i32, i32, vp, vp]
        L.fc_dequantize_rot.restype = i32
        L.fc_allreduce_sim_rot.argtypes = [vp, i32, i64, i64, i32, i32, i32, i32, vp, vp, sz, vp]
        L.fc_allreduce_sim_rot.restype = i32
        L.fc_stream_reference.argtypes = [vp, i64, i32, i64, vp, vp]
        L.fc_stream_reference.restype = i32
        L.fc_strerror.argtypes = [i32]
        L.fc_strerror.restype = ctypes.c_char_p
        L.fc_last_hip_error.argtypes = []
        L.fc_last_hip_error.restype = i32
        L.fc_version.argtypes = []
        L.fc_version.restype = i32
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().fc_strerror(code).decode()


def last_hip_error() -> int:
    return lib().fc_last_hip_error()


def version() -> int:
    return lib().fc_version()


def _torch():
    import torch
    return torch


def _stream() -> int:
    return _torch().cuda.current_stream().cuda_stream


def _dev(t, dtype, what):
    torch = _torch()
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("%s must be a CUDA (HIP) tensor; this library has no CPU path" % what)
    if t.dtype != dtype:
        raise TypeError("%s must be %s, got %s" % (what, dtype, t.dtype))
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % what)
    return t


def _check(rc: int, what: str):
    if rc != 0:
        raise FcError(rc, what)


def quantize(x, group: int, bits: int, out=None):
    """fc_quantize.  x: float16 [tokens, hidden] -> (codes u8 [tokens, hidden*bits/8],
    scales f32 [tokens, hidden/group], zeros f32 [tokens, hidden/group])."""
    torch = _torch()
    _dev(x, torch.float16, "x")
    t, h = x.shape
    if out is None:
        if bits not in (4, 8) or group <= 0 or h % group:
            _check(lib().fc_quantize(None, t, h, group, bits, None, None, None, None), "fc_quantize")
        codes = torch.empty((t, h * bits // 8), dtype=torch.uint8, device=x.device)
        scales = torch.empty((t, h // group), dtype=torch.float32, device=x.device)
        zeros = torch.empty_like(scales)
    else:
        codes, scales, zeros = out
        _dev(codes, torch.uint8, "codes"); _dev(scales, torch.float32, "scales")
        _dev(zeros, torch.float32, "zeros")
    _check(lib().fc_quantize(x.data_ptr(), t, h, group, bits, codes.data_ptr(), scales.data_ptr(),
                             zeros.data_ptr(), _stream()), "fc_quantize")
    return codes, scales, zeros


def dequant_reduce_requant(codes_in, scales_in, zeros_in, hidden: int, group: int,
                           bits_in: int, bits_out: int, out=None):
    """fc_dequant_reduce_requant.  Inputs stacked on a leading source axis:
    codes_in u8 [N, tokens, hidden*bits_in/8], scales_in / zeros_in f32 [N, tokens, hidden/group]."""
    torch = _torch()
    _dev(codes_in, torch.uint8, "codes_in"); _dev(scales_in, torch.float32, "scales_in")
    _dev(zeros_in, torch.float32, "zeros_in")
    n, t = codes_in.shape[0], codes_in.shape[1]
    if out is None:
        if bits_out not in (4, 8) or group <= 0 or hidden % group:
            _check(lib().fc_dequant_reduce_requant(None, 0, None, None, 0, n, t, hidden, group,
                                                   bits_in, bits_out, None, None, None, None),
                   "fc_dequant_reduce_requant")
        codes = torch.empty((t, hidden * bits_out // 8), dtype=torch.uint8, device=codes_in.device)
        scales = torch.empty((t, hidden // group), dtype=torch.float32, device=codes_in.device)
        zeros = torch.empty_like(scales)
    else:
        codes, scales, zeros = out
        _dev(codes, torch.uint8, "codes_out"); _dev(scales, torch.float32, "scales_out")
        _dev(zeros, torch.float32, "zeros_out")
    cstride = codes_in.stride(0) if n > 1 else 0
    mstride = scales_in.stride(0) if n > 1 else 0
    if n > 1 and zeros_in.stride(0) != mstride:
        raise ValueError("scales_in and zeros_in must share the source stride")
    _check(lib().fc_dequant_reduce_requant(
        codes_in.data_ptr(), cstride, scales_in.data_ptr(), zeros_in.data_ptr(), mstride, n, t,
        hidden, group, bits_in, bits_out, codes.data_ptr(), scales.data_ptr(), zeros.data_ptr(),
        _stream()), "fc_dequant_reduce_requant")
    return codes, scales, zeros


def dequantize(codes, scales, zeros, hidden: int, group: int, bits: int, out=None):
    """fc_dequantize -> float16 [tokens, hidden]."""
    torch = _torch()
    _dev(codes, torch.uint8, "codes"); _dev(scales, torch.float32, "scales")
    _dev(zeros, torch.float32, "zeros")
    t = codes.shape[0]
    y = out if out is not None else torch.empty((t, hidden), dtype=torch.float16, device=codes.device)
    _dev(y, torch.float16, "y")
    _check(lib().fc_dequantize(codes.data_ptr(), scales.data_ptr(), zeros.data_ptr(), t, hidden,
                               group, bits, y.data_ptr(), _stream()), "fc_dequantize")
    return y


def allreduce_sim_workspace_bytes(n_src: int, tokens: int, hidden: int, group: int,
                                  bits_rs: int, bits_ag: int) -> int:
    return int(lib().fc_allreduce_sim_workspace_bytes(n_src, tokens, hidden, group, bits_rs, bits_ag))


def allreduce_sim(x, group: int, bits_rs: int, bits_ag: int, out=None, workspace=None):
    """fc_allreduce_sim.  x: float16 [N, tokens, hidden] -> float16 [tokens, hidden]."""
    torch = _torch()
    _dev(x, torch.float16, "x")
    n, t, h = x.shape
    need = allreduce_sim_workspace_bytes(n, t, h, group, bits_rs, bits_ag)
    if need == 0 and t != 0:
        _check(lib().fc_allreduce_sim(None, n, t, h, group, bits_rs, bits_ag, None, None, 0, None),
               "fc_allreduce_sim")
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=x.device)
    _dev(workspace, torch.uint8, "workspace")
    y = out if out is not None else torch.empty((t, h), dtype=torch.float16, device=x.device)
    _dev(y, torch.float16, "y")
    _check(lib().fc_allreduce_sim(x.data_ptr(), n, t, h, group, bits_rs, bits_ag, y.data_ptr(),
                                  workspace.data_ptr(), workspace.numel(), _stream()),
           "fc_allreduce_sim")
    return y


STATIC_SCRATCH_BYTES = 32 << 20      # FC_STATIC_SCRATCH_BYTES of include/fc.h


def allreduce_sim_static(x, group: int, bits_rs: int, bits_ag: int, out=None):
    """fc_allreduce_sim_static: fc_allreduce_sim with the intermediates in the library's own fixed
    scratch array.  The C call allocates nothing; pass `out` to keep this wrapper from allocating too."""
    torch = _torch()
    _dev(x, torch.float16, "x")
    n, t, h = x.shape
    y = out if out is not None else torch.empty((t, h), dtype=torch.float16, device=x.device)
    _dev(y, torch.float16, "y")
    _check(lib().fc_allreduce_sim_static(x.data_ptr(), n, t, h, group, bits_rs, bits_ag, y.data_ptr(),
                                         _stream()), "fc_allreduce_sim_static")
    return y


# ---- symmetric variant (Appendix Eq. 3-4): signed two's-complement codes, no zero-points ----

def quantize_sym(x, group: int, bits: int, out=None):
    """fc_quantize_sym.  x: float16 [tokens, hidden] -> (codes u8 [tokens, hidden*bits/8] holding
    signed codes, scales f32 [tokens, hidden/group])."""
    torch = _torch()
    _dev(x, torch.float16, "x")
    t, h = x.shape
    if out is None:
        if bits not in (4, 8) or group <= 0 or h % group:
            _check(lib().fc_quantize_sym(None, t, h, group, bits, None, None, None), "fc_quantize_sym")
        codes = torch.empty((t, h * bits // 8), dtype=torch.uint8, device=x.device)
        scales = torch.empty((t, h // group), dtype=torch.float32, device=x.device)
    else:
        codes, scales = out
        _dev(codes, torch.uint8, "codes"); _dev(scales, torch.float32, "scales")
    _check(lib().fc_quantize_sym(x.data_ptr(), t, h, group, bits, codes.data_ptr(), scales.data_ptr(),
                                 _stream()), "fc_quantize_sym")
    return codes, scales


def dequant_reduce_requant_sym(codes_in, scales_in, hidden: int, group: int,
                               bits_in: int, bits_out: int, out=None):
    """fc_dequant_reduce_requant_sym.  codes_in u8 [N, tokens, hidden*bits_in/8],
    scales_in f32 [N, tokens, hidden/group]."""
    torch = _torch()
    _dev(codes_in, torch.uint8, "codes_in"); _dev(scales_in, torch.float32, "scales_in")
    n, t = codes_in.shape[0], codes_in.shape[1]
    if out is None:
        if bits_out not in (4, 8) or group <= 0 or hidden % group:
            _check(lib().fc_dequant_reduce_requant_sym(None, 0, None, 0, n, t, hidden, group,
                                                       bits_in, bits_out, None, None, None),
                   "fc_dequant_reduce_requant_sym")
        codes = torch.empty((t, hidden * bits_out // 8), dtype=torch.uint8, device=codes_in.device)
        scales = torch.empty((t, hidden // group), dtype=torch.float32, device=codes_in.device)
    else:
        codes, scales = out
        _dev(codes, torch.uint8, "codes_out"); _dev(scales, torch.float32, "scales_out")
    cstride = codes_in.stride(0) if n > 1 else 0
    mstride = scales_in.stride(0) if n > 1 else 0
    _check(lib().fc_dequant_reduce_requant_sym(
        codes_in.data_ptr(), cstride, scales_in.data_ptr(), mstride, n, t, hidden, group, bits_in,
        bits_out, codes.data_ptr(), scales.data_ptr(), _stream()), "fc_dequant_reduce_requant_sym")
    return codes, scales


def dequantize_sym(codes, scales, hidden: int, group: int, bits: int, out=None):
    """fc_dequantize_sym -> float16 [tokens, hidden]."""
    torch = _torch()
    _dev(codes, torch.uint8, "codes"); _dev(scales, torch.float32, "scales")
    t = codes.shape[0]
    y = out if out is not None else torch.empty((t, hidden), dtype=torch.float16, device=codes.device)
    _dev(y, torch.float16, "y")
    _check(lib().fc_dequantize_sym(codes.data_ptr(), scales.data_ptr(), t, hidden, group, bits,
                                   y.data_ptr(), _stream()), "fc_dequantize_sym")
    return y


def allreduce_sim_sym(x, group: int, bits_rs: int, bits_ag: int, out=None, workspace=None):
    """fc_allreduce_sim_sym.  x: float16 [N, tokens, hidden] -> float16 [tokens, hidden]."""
    torch = _torch()
    _dev(x, torch.float16, "x")
    n, t, h = x.shape
    need = allreduce_sim_workspace_bytes(n, t, h, group, bits_rs, bits_ag)
    if need == 0 and t != 0:
        _check(lib().fc_allreduce_sim_sym(None, n, t, h, group, bits_rs, bits_ag, None, None, 0, None),
               "fc_allreduce_sim_sym")
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=x.device)
    _dev(workspace, torch.uint8, "workspace")
    y = out if out is not None else torch.empty((t, h), dtype=torch.float16, device=x.device)
    _dev(y, torch.float16, "y")
    _check(lib().fc_allreduce_sim_sym(x.data_ptr(), n, t, h, group, bits_rs, bits_ag, y.data_ptr(),
                                      workspace.data_ptr(), workspace.numel(), _stream()),
           "fc_allreduce_sim_sym")
    return y


# ---- asymmetric quantizer with binary16 metadata: one 32-bit word per group ----
# (int32 tensors: bits 0-15 the binary16 scale, bits 16-31 the binary16 zero-point)

def quantize_cmeta(x, group: int, bits: int, out=None):
    """fc_quantize_cmeta.  x: float16 [tokens, hidden] -> (codes u8 [tokens, hidden*bits/8],
    meta i32 [tokens, hidden/group])."""
    torch = _torch()
    _dev(x, torch.float16, "x")
    t, h = x.shape
    if out is None:
        if bits not in (4, 8) or group <= 0 or h % group:
            _check(lib().fc_quantize_cmeta(None, t, h, group, bits, None, None, None), "fc_quantize_cmeta")
        codes = torch.empty((t, h * bits // 8), dtype=torch.uint8, device=x.device)
        meta = torch.empty((t, h // group), dtype=torch.int32, device=x.device)
    else:
        codes, meta = out
        _dev(codes, torch.uint8, "codes"); _dev(meta, torch.int32, "meta")
    _check(lib().fc_quantize_cmeta(x.data_ptr(), t, h, group, bits, codes.data_ptr(), meta.data_ptr(),
                                   _stream()), "fc_quantize_cmeta")
    return codes, meta


def dequant_reduce_requant_cmeta(codes_in, meta_in, hidden: int, group: int,
                                 bits_in: int, bits_out: int, out=None):
    """fc_dequant_reduce_requant_cmeta.  codes_in u8 [N, tokens, hidden*bits_in/8],
    meta_in i32 [N, tokens, hidden/group]."""
    torch = _torch()
    _dev(codes_in, torch.uint8, "codes_in"); _dev(meta_in, torch.int32, "meta_in")
    n, t = codes_in.shape[0], codes_in.shape[1]
    if out is None:
        if bits_out not in (4, 8) or group <= 0 or hidden % group:
            _check(lib().fc_dequant_reduce_requant_cmeta(None, 0, None, 0, n, t, hidden, group,
                                                         bits_in, bits_out, None, None, None),
                   "fc_dequant_reduce_requant_cmeta")
        codes = torch.empty((t, hidden * bits_out // 8), dtype=torch.uint8, device=codes_in.device)
        meta = torch.empty((t, hidden // group), dtype=torch.int32, device=codes_in.device)
    else:
        codes, meta = out
        _dev(codes, torch.uint8, "codes_out"); _dev(meta, torch.int32, "meta_out")
    cstride = codes_in.stride(0) if n > 1 else 0
    mstride = meta_in.stride(0) if n > 1 else 0
    _check(lib().fc_dequant_reduce_requant_cmeta(
        codes_in.data_ptr(), cstride, meta_in.data_ptr(), mstride, n, t, hidden, group, bits_in,
        bits_out, codes.data_ptr(), meta.data_ptr(), _stream()), "fc_dequant_reduce_requant_cmeta")
    return codes, meta


def dequantize_cmeta(codes, meta, hidden: int, group: int, bits: int, out=None):
    """fc_dequantize_cmeta -> float16 [tokens, hidden]."""
    torch = _torch()
    _dev(codes, torch.uint8, "codes"); _dev(meta, torch.int32, "meta")
    t = codes.shape[0]
    y = out if out is not None else torch.empty((t, hidden), dtype=torch.float16, device=codes.device)
    _dev(y, torch.float16, "y")
    _check(lib().fc_dequantize_cmeta(codes.data_ptr(), meta.data_ptr(), t, hidden, group, bits,
                                     y.data_ptr(), _stream()), "fc_dequantize_cmeta")
    return y


def allreduce_sim_cmeta(x, group: int, bits_rs: int, bits_ag: int, out=None, workspace=None):
    """fc_allreduce_sim_cmeta.  x: float16 [N, tokens, hidden] -> float16 [tokens, hidden]."""
    torch = _torch()
    _dev(x, torch.float16, "x")
    n, t, h = x.shape
    need = allreduce_sim_workspace_bytes(n, t, h, group, bits_rs, bits_ag)
    if need == 0 and t != 0:
        _check(lib().fc_allreduce_sim_cmeta(None, n, t, h, group, bits_rs, bits_ag, None, None, 0, None),
               "fc_allreduce_sim_cmeta")
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=x.device)
    _dev(workspace, torch.uint8, "workspace")
    y = out if out is not None else torch.empty((t, h), dtype=torch.float16, device=x.device)
    _dev(y, torch.float16, "y")
    _check(lib().fc_allreduce_sim_cmeta(x.data_ptr(), n, t, h, group, bits_rs, bits_ag, y.data_ptr(),
                                        workspace.data_ptr(), workspace.numel(), _stream()),
           "fc_allreduce_sim_cmeta")
    return y


# ---- FP8 E4M3 variant: one E4M3 byte per element, scales only ----

def quantize_fp8(x, group: int, out=None):
    """fc_quantize_fp8.  x: float16 [tokens, hidden] -> (E4M3 bytes u8 [tokens, hidden],
    scales f32 [tokens, hidden/group])."""
    torch = _torch()
    _dev(x, torch.float16, "x")
    t, h = x.shape
    if out is None:
        if group <= 0 or h % group:
            _check(lib().fc_quantize_fp8(None, t, h, group, None, None, None), "fc_quantize_fp8")
        codes = torch.empty((t, h), dtype=torch.uint8, device=x.device)
        scales = torch.empty((t, h // group), dtype=torch.float32, device=x.device)
    else:
        codes, scales = out
        _dev(codes, torch.uint8, "codes"); _dev(scales, torch.float32, "scales")
    _check(lib().fc_quantize_fp8(x.data_ptr(), t, h, group, codes.data_ptr(), scales.data_ptr(), _stream()),
           "fc_quantize_fp8")
    return codes, scales


def dequant_reduce_requant_fp8(codes_in, scales_in, hidden: int, group: int, out=None):
    """fc_dequant_reduce_requant_fp8.  codes_in u8 [N, tokens, hidden], scales_in f32 [N, tokens, hidden/group]."""
    torch = _torch()
    _dev(codes_in, torch.uint8, "codes_in"); _dev(scales_in, torch.float32, "scales_in")
    n, t = codes_in.shape[0], codes_in.shape[1]
    if out is None:
        if group <= 0 or hidden % group:
            _check(lib().fc_dequant_reduce_requant_fp8(None, 0, None, 0, n, t, hidden, group, None, None, None),
                   "fc_dequant_reduce_requant_fp8")
        codes = torch.empty((t, hidden), dtype=torch.uint8, device=codes_in.device)
        scales = torch.empty((t, hidden // group), dtype=torch.float32, device=codes_in.device)
    else:
        codes, scales = out
        _dev(codes, torch.uint8, "codes_out"); _dev(scales, torch.float32, "scales_out")
    cstride = codes_in.stride(0) if n > 1 else 0
    mstride = scales_in.stride(0) if n > 1 else 0
    _check(lib().fc_dequant_reduce_requant_fp8(
        codes_in.data_ptr(), cstride, scales_in.data_ptr(), mstride, n, t, hidden, group,
        codes.data_ptr(), scales.data_ptr(), _stream()), "fc_dequant_reduce_requant_fp8")
    return codes, scales


def dequantize_fp8(codes, scales, hidden: int, group: int, out=None):
    """fc_dequantize_fp8 -> float16 [tokens, hidden]."""
    torch = _torch()
    _dev(codes, torch.uint8, "codes"); _dev(scales, torch.float32, "scales")
    t = codes.shape[0]
    y = out if out is not None else torch.empty((t, hidden), dtype=torch.float16, device=codes.device)
    _dev(y, torch.float16, "y")
    _check(lib().fc_dequantize_fp8(codes.data_ptr(), scales.data_ptr(), t, hidden, group, y.data_ptr(),
                                   _stream()), "fc_dequantize_fp8")
    return y


def allreduce_sim_fp8(x, group: int, out=None, workspace=None):
    """fc_allreduce_sim_fp8.  x: float16 [N, tokens, hidden] -> float16 [tokens, hidden]."""
    torch = _torch()
    _dev(x, torch.float16, "x")
    n, t, h = x.shape
    need = allreduce_sim_workspace_bytes(n, t, h, group, 8, 8)
    if need == 0 and t != 0:
        _check(lib().fc_allreduce_sim_fp8(None, n, t, h, group, None, None, 0, None), "fc_allreduce_sim_fp8")
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=x.device)
    _dev(workspace, torch.uint8, "workspace")
    y = out if out is not None else torch.empty((t, h), dtype=torch.float16, device=x.device)
    _dev(y, torch.float16, "y")
    _check(lib().fc_allreduce_sim_fp8(x.data_ptr(), n, t, h, group, y.data_ptr(), workspace.data_ptr(),
                                      workspace.numel(), _stream()), "fc_allreduce_sim_fp8")
    return y


# ---- Hadamard rotation fused into the first quantization and the last dequantization ----

def quantize_rot(x, group: int, bits: int, quantizer: int = QUANTIZER_ASYM, out=None):
    """fc_quantize_rot.  x: float16 [tokens, hidden] -> (codes, scales, zeros); zeros is None
    unless quantizer == QUANTIZER_ASYM."""
    torch = _torch()
    _dev(x, torch.float16, "x")
    t, h = x.shape
    asym = quantizer == QUANTIZER_ASYM
    if out is None:
        if bits not in (4, 8) or group <= 0 or h % group:
            _check(lib().fc_quantize_rot(None, t, h, group, bits, quantizer, None, None, None, None),
                   "fc_quantize_rot")
        codes = torch.empty((t, h * bits // 8), dtype=torch.uint8, device=x.device)
        scales = torch.empty((t, h // group), dtype=torch.float32, device=x.device)
        zeros = torch.empty_like(scales) if asym else None
    else:
        codes, scales, zeros = out
        _dev(codes, torch.uint8, "codes"); _dev(scales, torch.float32, "scales")
        if asym:
            _dev(zeros, torch.float32, "zeros")
    _check(lib().fc_quantize_rot(x.data_ptr(), t, h, group, bits, quantizer, codes.data_ptr(),
                                 scales.data_ptr(), zeros.data_ptr() if asym else None, _stream()),
           "fc_quantize_rot")
    return codes, scales, (zeros if asym else None)


def dequantize_rot(codes, scales, zeros, hidden: int, group: int, bits: int,
                   quantizer: int = QUANTIZER_ASYM, out=None):
    """fc_dequantize_rot -> float16 [tokens, hidden]."""
    torch = _torch()
    _dev(codes, torch.uint8, "codes"); _dev(scales, torch.float32, "scales")
    asym = quantizer == QUANTIZER_ASYM
    if asym:
        _dev(zeros, torch.float32, "zeros")
    t = codes.shape[0]
    y = out if out is not None else torch.empty((t, hidden), dtype=torch.float16, device=codes.device)
    _dev(y, torch.float16, "y")
    _check(lib().fc_dequantize_rot(codes.data_ptr(), scales.data_ptr(), zeros.data_ptr() if asym else None,
                                   t, hidden, group, bits, quantizer, y.data_ptr(), _stream()),
           "fc_dequantize_rot")
    return y


def allreduce_sim_rot(x, group: int, bits_rs: int, bits_ag: int, quantizer: int = QUANTIZER_ASYM,
                      out=None, workspace=None):
    """fc_allreduce_sim_rot.  x: float16 [N, tokens, hidden] -> float16 [tokens, hidden]."""
    torch = _torch()
    _dev(x, torch.float16, "x")
    n, t, h = x.shape
    need = allreduce_sim_workspace_bytes(n, t, h, group, bits_rs, bits_ag)
    if need == 0 and t != 0:
        _check(lib().fc_allreduce_sim_rot(None, n, t, h, group, bits_rs, bits_ag, quantizer, None, None, 0,
                                          None), "fc_allreduce_sim_rot")
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=x.device)
    _dev(workspace, torch.uint8, "workspace")
    y = out if out is not None else torch.empty((t, h), dtype=torch.float16, device=x.device)
    _dev(y, torch.float16, "y")
    _check(lib().fc_allreduce_sim_rot(x.data_ptr(), n, t, h, group, bits_rs, bits_ag, quantizer,
                                      y.data_ptr(), workspace.data_ptr(), workspace.numel(), _stream()),
           "fc_allreduce_sim_rot")
    return y


def stream_reference(src, out):
    """fc_stream_reference (measurement aid): src u8 [N, bytes], out u8 [bytes] = XOR over the N rows."""
    torch = _torch()
    _dev(src, torch.uint8, "src"); _dev(out, torch.uint8, "out")
    n, nbytes = src.shape[0], src[0].numel()
    _check(lib().fc_stream_reference(src.data_ptr(), src.stride(0) if n > 1 else 0, n, nbytes, out.data_ptr(),
                                     _stream()), "fc_stream_reference")
    return out
