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
_BENCH_LIB_PATH = os.environ.get("FC_BENCH_LIBRARY") or os.path.join(_HERE, "libfc_bench.so")
_lib = None
_bench_lib = None

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
        # PyTorch ships its own copy of the HIP runtime.  The library must bind to the copy that owns the
        # tensors' device memory, so torch is loaded first: the loader then resolves libfc.so's dependency to
        # the runtime already in the process instead of bringing in a second one (whose launches on torch's
        # pointers fail with "no device").
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
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
    if t.device.index != torch.cuda.current_device():
        raise ValueError("%s lives on %s but the current device is cuda:%d; the C ABI works on the current device"
                         % (what, t.device, torch.cuda.current_device()))
    return t


# The kernels take every buffer range from (tokens, hidden, group, bits), never from the allocation, so a tensor
# whose shape disagrees with those numbers would be read or written out of bounds: each wrapper compares every
# tensor's shape with the geometry before the C call.

def _geometry(what: str, hidden: int, group: int, *bits: int):
    """The C library's own argument errors, raised before any shape arithmetic that would divide by them."""
    for b in bits:
        if b not in (4, 8):
            raise FcError(-2, what)
    if group < 32 or group > 16384 or (group & (group - 1)):
        raise FcError(-3, what)
    if hidden <= 0:
        raise FcError(-4, what)
    if hidden % group:
        raise FcError(-3, what)


def _shape(t, want, what: str):
    if tuple(t.shape) != tuple(want):
        raise ValueError("%s must have shape %s for these arguments, got %s" % (what, tuple(want), tuple(t.shape)))
    return t


def _sources(t, what: str):
    """[N, tokens, bytes-or-groups] stacked on the source axis, each source's slab dense"""
    if t.dim() != 3:
        raise ValueError("%s must be [n_src, tokens, ...], got shape %s" % (what, tuple(t.shape)))
    if not 1 <= t.shape[0] <= FC_MAX_SRC:
        raise FcError(-4, what)
    return t


def _check(rc: int, what: str):
    if rc != 0:
        raise FcError(rc, what)


def _x2(x, what="x"):
    torch = _torch()
    _dev(x, torch.float16, what)
    if x.dim() != 2:
        raise ValueError("%s must be float16 [tokens, hidden], got shape %s" % (what, tuple(x.shape)))
    return x.shape


def _x3(x):
    torch = _torch()
    _dev(x, torch.float16, "x")
    _sources(x, "x")
    return x.shape


def _coded_outputs(device, t, h, group, bits, out, meta):
    """codes u8 [t, h*bits/8] plus one [t, h/group] array per entry of `meta` (its dtype, its name): allocated
    here, or the caller's `out` tuple checked against those shapes."""
    torch = _torch()
    if out is None:
        return (torch.empty((t, h * bits // 8), dtype=torch.uint8, device=device),
                *[torch.empty((t, h // group), dtype=dt, device=device) for dt, _ in meta])
    if len(out) != 1 + len(meta):
        raise ValueError("out must hold %d tensors" % (1 + len(meta)))
    _shape(_dev(out[0], torch.uint8, "codes (out)"), (t, h * bits // 8), "codes (out)")
    for o, (dt, name) in zip(out[1:], meta):
        _shape(_dev(o, dt, name + " (out)"), (t, h // group), name + " (out)")
    return tuple(out)


def _coded_inputs(codes, metas, hidden, group, bits, meta):
    """codes u8 [t, hidden*bits/8] and the [t, hidden/group] metadata arrays of one quantized tensor"""
    torch = _torch()
    _dev(codes, torch.uint8, "codes")
    if codes.dim() != 2:
        raise ValueError("codes must be [tokens, hidden*bits/8], got shape %s" % (tuple(codes.shape),))
    t = codes.shape[0]
    _shape(codes, (t, hidden * bits // 8), "codes")
    for m, (dt, name) in zip(metas, meta):
        _shape(_dev(m, dt, name), (t, hidden // group), name)
    return t


def _stacked_inputs(codes_in, metas, hidden, group, bits_in, meta):
    """codes_in u8 [N, t, hidden*bits_in/8] and metadata [N, t, hidden/group]; returns (N, t, code stride in
    bytes, metadata stride in elements) of the dense slabs"""
    torch = _torch()
    _sources(_dev(codes_in, torch.uint8, "codes_in"), "codes_in")
    n, t = codes_in.shape[0], codes_in.shape[1]
    _shape(codes_in, (n, t, hidden * bits_in // 8), "codes_in")
    for m, (dt, name) in zip(metas, meta):
        _shape(_dev(m, dt, name), (n, t, hidden // group), name)
    return n, t, (codes_in.stride(0) if n > 1 else 0), (metas[0].stride(0) if n > 1 else 0)


def _y_out(device, t, h, out):
    torch = _torch()
    if out is None:
        return torch.empty((t, h), dtype=torch.float16, device=device)
    return _shape(_dev(out, torch.float16, "y (out)"), (t, h), "y (out)")


def _f32(name):
    return (_torch().float32, name)


def _i32(name):
    return (_torch().int32, name)


def quantize(x, group: int, bits: int, out=None):
    """fc_quantize.  x: float16 [tokens, hidden] -> (codes u8 [tokens, hidden*bits/8],
    scales f32 [tokens, hidden/group], zeros f32 [tokens, hidden/group])."""
    t, h = _x2(x)
    _geometry("fc_quantize", h, group, bits)
    codes, scales, zeros = _coded_outputs(x.device, t, h, group, bits, out, [_f32("scales"), _f32("zeros")])
    _check(lib().fc_quantize(x.data_ptr(), t, h, group, bits, codes.data_ptr(), scales.data_ptr(),
                             zeros.data_ptr(), _stream()), "fc_quantize")
    return codes, scales, zeros


def dequant_reduce_requant(codes_in, scales_in, zeros_in, hidden: int, group: int,
                           bits_in: int, bits_out: int, out=None):
    """fc_dequant_reduce_requant.  Inputs stacked on a leading source axis:
    codes_in u8 [N, tokens, hidden*bits_in/8], scales_in / zeros_in f32 [N, tokens, hidden/group]."""
    _geometry("fc_dequant_reduce_requant", hidden, group, bits_in, bits_out)
    n, t, cstride, mstride = _stacked_inputs(codes_in, (scales_in, zeros_in), hidden, group, bits_in,
                                             [_f32("scales_in"), _f32("zeros_in")])
    codes, scales, zeros = _coded_outputs(codes_in.device, t, hidden, group, bits_out, out,
                                          [_f32("scales"), _f32("zeros")])
    _check(lib().fc_dequant_reduce_requant(
        codes_in.data_ptr(), cstride, scales_in.data_ptr(), zeros_in.data_ptr(), mstride, n, t,
        hidden, group, bits_in, bits_out, codes.data_ptr(), scales.data_ptr(), zeros.data_ptr(),
        _stream()), "fc_dequant_reduce_requant")
    return codes, scales, zeros


def dequantize(codes, scales, zeros, hidden: int, group: int, bits: int, out=None):
    """fc_dequantize -> float16 [tokens, hidden]."""
    _geometry("fc_dequantize", hidden, group, bits)
    t = _coded_inputs(codes, (scales, zeros), hidden, group, bits, [_f32("scales"), _f32("zeros")])
    y = _y_out(codes.device, t, hidden, out)
    _check(lib().fc_dequantize(codes.data_ptr(), scales.data_ptr(), zeros.data_ptr(), t, hidden,
                               group, bits, y.data_ptr(), _stream()), "fc_dequantize")
    return y


def allreduce_sim_workspace_bytes(n_src: int, tokens: int, hidden: int, group: int,
                                  bits_rs: int, bits_ag: int) -> int:
    return int(lib().fc_allreduce_sim_workspace_bytes(n_src, tokens, hidden, group, bits_rs, bits_ag))


def _sim(fn_name, x, group, bits_rs, bits_ag, out, workspace, bits_args=True, extra=()):
    """the fc_allreduce_sim* family: x float16 [N, tokens, hidden] -> float16 [tokens, hidden]"""
    torch = _torch()
    n, t, h = _x3(x)
    _geometry(fn_name, h, group, bits_rs, bits_ag)
    need = allreduce_sim_workspace_bytes(n, t, h, group, bits_rs, bits_ag)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=x.device)
    _dev(workspace, torch.uint8, "workspace")
    if workspace.numel() < need:
        raise FcError(-6, fn_name)
    y = _y_out(x.device, t, h, out)
    bits = (bits_rs, bits_ag) if bits_args else ()
    _check(getattr(lib(), fn_name)(x.data_ptr(), n, t, h, group, *bits, *extra, y.data_ptr(),
                                   workspace.data_ptr(), workspace.numel(), _stream()), fn_name)
    return y


def allreduce_sim(x, group: int, bits_rs: int, bits_ag: int, out=None, workspace=None):
    """fc_allreduce_sim.  x: float16 [N, tokens, hidden] -> float16 [tokens, hidden]."""
    return _sim("fc_allreduce_sim", x, group, bits_rs, bits_ag, out, workspace)


STATIC_SCRATCH_BYTES = 32 << 20      # FC_STATIC_SCRATCH_BYTES of include/fc.h


def allreduce_sim_static(x, group: int, bits_rs: int, bits_ag: int, out=None):
    """fc_allreduce_sim_static: fc_allreduce_sim with the intermediates in the library's own fixed
    scratch array.  The C call allocates nothing; pass `out` to keep this wrapper from allocating too."""
    n, t, h = _x3(x)
    _geometry("fc_allreduce_sim_static", h, group, bits_rs, bits_ag)
    y = _y_out(x.device, t, h, out)
    _check(lib().fc_allreduce_sim_static(x.data_ptr(), n, t, h, group, bits_rs, bits_ag, y.data_ptr(),
                                         _stream()), "fc_allreduce_sim_static")
    return y


# ---- symmetric variant (Appendix Eq. 3-4): signed two's-complement codes, no zero-points ----

def quantize_sym(x, group: int, bits: int, out=None):
    """fc_quantize_sym.  x: float16 [tokens, hidden] -> (codes u8 [tokens, hidden*bits/8] holding
    signed codes, scales f32 [tokens, hidden/group])."""
    t, h = _x2(x)
    _geometry("fc_quantize_sym", h, group, bits)
    codes, scales = _coded_outputs(x.device, t, h, group, bits, out, [_f32("scales")])
    _check(lib().fc_quantize_sym(x.data_ptr(), t, h, group, bits, codes.data_ptr(), scales.data_ptr(),
                                 _stream()), "fc_quantize_sym")
    return codes, scales


def dequant_reduce_requant_sym(codes_in, scales_in, hidden: int, group: int,
                               bits_in: int, bits_out: int, out=None):
    """fc_dequant_reduce_requant_sym.  codes_in u8 [N, tokens, hidden*bits_in/8],
    scales_in f32 [N, tokens, hidden/group]."""
    _geometry("fc_dequant_reduce_requant_sym", hidden, group, bits_in, bits_out)
    n, t, cstride, mstride = _stacked_inputs(codes_in, (scales_in,), hidden, group, bits_in, [_f32("scales_in")])
    codes, scales = _coded_outputs(codes_in.device, t, hidden, group, bits_out, out, [_f32("scales")])
    _check(lib().fc_dequant_reduce_requant_sym(
        codes_in.data_ptr(), cstride, scales_in.data_ptr(), mstride, n, t, hidden, group, bits_in,
        bits_out, codes.data_ptr(), scales.data_ptr(), _stream()), "fc_dequant_reduce_requant_sym")
    return codes, scales


def dequantize_sym(codes, scales, hidden: int, group: int, bits: int, out=None):
    """fc_dequantize_sym -> float16 [tokens, hidden]."""
    _geometry("fc_dequantize_sym", hidden, group, bits)
    t = _coded_inputs(codes, (scales,), hidden, group, bits, [_f32("scales")])
    y = _y_out(codes.device, t, hidden, out)
    _check(lib().fc_dequantize_sym(codes.data_ptr(), scales.data_ptr(), t, hidden, group, bits,
                                   y.data_ptr(), _stream()), "fc_dequantize_sym")
    return y


def allreduce_sim_sym(x, group: int, bits_rs: int, bits_ag: int, out=None, workspace=None):
    """fc_allreduce_sim_sym.  x: float16 [N, tokens, hidden] -> float16 [tokens, hidden]."""
    return _sim("fc_allreduce_sim_sym", x, group, bits_rs, bits_ag, out, workspace)


# ---- asymmetric quantizer with binary16 metadata: one 32-bit word per group ----
# (int32 tensors: bits 0-15 the binary16 scale, bits 16-31 the binary16 zero-point)

def quantize_cmeta(x, group: int, bits: int, out=None):
    """fc_quantize_cmeta.  x: float16 [tokens, hidden] -> (codes u8 [tokens, hidden*bits/8],
    meta i32 [tokens, hidden/group])."""
    t, h = _x2(x)
    _geometry("fc_quantize_cmeta", h, group, bits)
    codes, meta = _coded_outputs(x.device, t, h, group, bits, out, [_i32("meta")])
    _check(lib().fc_quantize_cmeta(x.data_ptr(), t, h, group, bits, codes.data_ptr(), meta.data_ptr(),
                                   _stream()), "fc_quantize_cmeta")
    return codes, meta


def dequant_reduce_requant_cmeta(codes_in, meta_in, hidden: int, group: int,
                                 bits_in: int, bits_out: int, out=None):
    """fc_dequant_reduce_requant_cmeta.  codes_in u8 [N, tokens, hidden*bits_in/8],
    meta_in i32 [N, tokens, hidden/group]."""
    _geometry("fc_dequant_reduce_requant_cmeta", hidden, group, bits_in, bits_out)
    n, t, cstride, mstride = _stacked_inputs(codes_in, (meta_in,), hidden, group, bits_in, [_i32("meta_in")])
    codes, meta = _coded_outputs(codes_in.device, t, hidden, group, bits_out, out, [_i32("meta")])
    _check(lib().fc_dequant_reduce_requant_cmeta(
        codes_in.data_ptr(), cstride, meta_in.data_ptr(), mstride, n, t, hidden, group, bits_in,
        bits_out, codes.data_ptr(), meta.data_ptr(), _stream()), "fc_dequant_reduce_requant_cmeta")
    return codes, meta


def dequantize_cmeta(codes, meta, hidden: int, group: int, bits: int, out=None):
    """fc_dequantize_cmeta -> float16 [tokens, hidden]."""
    _geometry("fc_dequantize_cmeta", hidden, group, bits)
    t = _coded_inputs(codes, (meta,), hidden, group, bits, [_i32("meta")])
    y = _y_out(codes.device, t, hidden, out)
    _check(lib().fc_dequantize_cmeta(codes.data_ptr(), meta.data_ptr(), t, hidden, group, bits,
                                     y.data_ptr(), _stream()), "fc_dequantize_cmeta")
    return y


def allreduce_sim_cmeta(x, group: int, bits_rs: int, bits_ag: int, out=None, workspace=None):
    """fc_allreduce_sim_cmeta.  x: float16 [N, tokens, hidden] -> float16 [tokens, hidden]."""
    return _sim("fc_allreduce_sim_cmeta", x, group, bits_rs, bits_ag, out, workspace)


# ---- FP8 E4M3 variant: one E4M3 byte per element, scales only ----

def quantize_fp8(x, group: int, out=None):
    """fc_quantize_fp8.  x: float16 [tokens, hidden] -> (E4M3 bytes u8 [tokens, hidden],
    scales f32 [tokens, hidden/group])."""
    t, h = _x2(x)
    _geometry("fc_quantize_fp8", h, group)
    codes, scales = _coded_outputs(x.device, t, h, group, 8, out, [_f32("scales")])
    _check(lib().fc_quantize_fp8(x.data_ptr(), t, h, group, codes.data_ptr(), scales.data_ptr(), _stream()),
           "fc_quantize_fp8")
    return codes, scales


def dequant_reduce_requant_fp8(codes_in, scales_in, hidden: int, group: int, out=None):
    """fc_dequant_reduce_requant_fp8.  codes_in u8 [N, tokens, hidden], scales_in f32 [N, tokens, hidden/group]."""
    _geometry("fc_dequant_reduce_requant_fp8", hidden, group)
    n, t, cstride, mstride = _stacked_inputs(codes_in, (scales_in,), hidden, group, 8, [_f32("scales_in")])
    codes, scales = _coded_outputs(codes_in.device, t, hidden, group, 8, out, [_f32("scales")])
    _check(lib().fc_dequant_reduce_requant_fp8(
        codes_in.data_ptr(), cstride, scales_in.data_ptr(), mstride, n, t, hidden, group,
        codes.data_ptr(), scales.data_ptr(), _stream()), "fc_dequant_reduce_requant_fp8")
    return codes, scales


def dequantize_fp8(codes, scales, hidden: int, group: int, out=None):
    """fc_dequantize_fp8 -> float16 [tokens, hidden]."""
    _geometry("fc_dequantize_fp8", hidden, group)
    t = _coded_inputs(codes, (scales,), hidden, group, 8, [_f32("scales")])
    y = _y_out(codes.device, t, hidden, out)
    _check(lib().fc_dequantize_fp8(codes.data_ptr(), scales.data_ptr(), t, hidden, group, y.data_ptr(),
                                   _stream()), "fc_dequantize_fp8")
    return y


def allreduce_sim_fp8(x, group: int, out=None, workspace=None):
    """fc_allreduce_sim_fp8.  x: float16 [N, tokens, hidden] -> float16 [tokens, hidden]."""
    return _sim("fc_allreduce_sim_fp8", x, group, 8, 8, out, workspace, bits_args=False)


# ---- Hadamard rotation fused into the first quantization and the last dequantization ----

def quantize_rot(x, group: int, bits: int, quantizer: int = QUANTIZER_ASYM, out=None):
    """fc_quantize_rot.  x: float16 [tokens, hidden] -> (codes, scales, zeros); zeros is None
    unless quantizer == QUANTIZER_ASYM."""
    t, h = _x2(x)
    _geometry("fc_quantize_rot", h, group, bits)
    asym = quantizer == QUANTIZER_ASYM
    if out is not None and not asym:
        out = tuple(out)[:2]
    res = _coded_outputs(x.device, t, h, group, bits, out, [_f32("scales")] + ([_f32("zeros")] if asym else []))
    codes, scales, zeros = res[0], res[1], (res[2] if asym else None)
    _check(lib().fc_quantize_rot(x.data_ptr(), t, h, group, bits, quantizer, codes.data_ptr(),
                                 scales.data_ptr(), zeros.data_ptr() if asym else None, _stream()),
           "fc_quantize_rot")
    return codes, scales, zeros


def dequantize_rot(codes, scales, zeros, hidden: int, group: int, bits: int,
                   quantizer: int = QUANTIZER_ASYM, out=None):
    """fc_dequantize_rot -> float16 [tokens, hidden]."""
    _geometry("fc_dequantize_rot", hidden, group, bits)
    asym = quantizer == QUANTIZER_ASYM
    metas = (scales, zeros) if asym else (scales,)
    t = _coded_inputs(codes, metas, hidden, group, bits, [_f32("scales"), _f32("zeros")][:len(metas)])
    y = _y_out(codes.device, t, hidden, out)
    _check(lib().fc_dequantize_rot(codes.data_ptr(), scales.data_ptr(), zeros.data_ptr() if asym else None,
                                   t, hidden, group, bits, quantizer, y.data_ptr(), _stream()),
           "fc_dequantize_rot")
    return y


def allreduce_sim_rot(x, group: int, bits_rs: int, bits_ag: int, quantizer: int = QUANTIZER_ASYM,
                      out=None, workspace=None):
    """fc_allreduce_sim_rot.  x: float16 [N, tokens, hidden] -> float16 [tokens, hidden]."""
    return _sim("fc_allreduce_sim_rot", x, group, bits_rs, bits_ag, out, workspace, extra=(quantizer,))


# ---- measurement aid (libfc_bench.so, include/fc_bench.h): not part of the product library ----

def bench_lib() -> ctypes.CDLL:
    global _bench_lib
    if _bench_lib is None:
        if not os.path.exists(_BENCH_LIB_PATH):
            raise ImportError("%s not found: build it with `python -m paper_2412_04964_amd.build`" % _BENCH_LIB_PATH)
        lib()                                          # torch's HIP runtime first (see lib())
        L = ctypes.CDLL(_BENCH_LIB_PATH)
        L.fc_stream_reference.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_int64,
                                          ctypes.c_void_p, ctypes.c_void_p]
        L.fc_stream_reference.restype = ctypes.c_int
        i64, i32, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
        L.fc_fused_compute_probe.argtypes = [vp, i64, vp, vp, i64, i32, i64, i64, i32, i32, i32, vp, vp, vp, vp]
        L.fc_fused_compute_probe.restype = i32
        _bench_lib = L
    return _bench_lib


def stream_reference(src, out):
    """fc_stream_reference: src u8 [N, bytes], out u8 [bytes] = XOR over the N rows."""
    torch = _torch()
    _dev(src, torch.uint8, "src"); _dev(out, torch.uint8, "out")
    if src.dim() != 2 or not 1 <= src.shape[0] <= FC_MAX_SRC:
        raise ValueError("src must be u8 [n_src, bytes] with 1 <= n_src <= %d" % FC_MAX_SRC)
    n, nbytes = src.shape
    _shape(out, (nbytes,), "out")
    _check(bench_lib().fc_stream_reference(src.data_ptr(), src.stride(0) if n > 1 else 0, n, nbytes, out.data_ptr(),
                                           _stream()), "fc_stream_reference")
    return out


def fused_compute_probe(codes_in, scales_in, zeros_in, hidden: int, group: int, bits_in: int, bits_out: int, out):
    """fc_fused_compute_probe: the launch of dequant_reduce_requant with its memory traffic confined to the L2
    (benchmark configurations only); `out` as for dequant_reduce_requant, contents meaningless afterwards."""
    _geometry("fc_fused_compute_probe", hidden, group, bits_in, bits_out)
    n, t, cstride, mstride = _stacked_inputs(codes_in, (scales_in, zeros_in), hidden, group, bits_in,
                                             [_f32("scales_in"), _f32("zeros_in")])
    codes, scales, zeros = _coded_outputs(codes_in.device, t, hidden, group, bits_out, out,
                                          [_f32("scales"), _f32("zeros")])
    _check(bench_lib().fc_fused_compute_probe(
        codes_in.data_ptr(), cstride, scales_in.data_ptr(), zeros_in.data_ptr(), mstride, n, t, hidden, group,
        bits_in, bits_out, codes.data_ptr(), scales.data_ptr(), zeros.data_ptr(), _stream()), "fc_fused_compute_probe")
