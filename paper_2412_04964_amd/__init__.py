"""MI355X-native Flash Communication quantization path (arXiv 2412.04964).

Thin ctypes binding over ``libfc.so`` (the C ABI in ``include/fc.h``).  The
functions here only marshal arguments: they take torch CUDA tensors for device
memory, pass raw pointers and the current HIP stream, and raise on any error
code.  There is no CPU fallback: if the HIP library is missing or no GPU is
present the compute calls fail loudly.
"""
from .binding import (  # noqa: F401
    QUANTIZER_ASYM,
    QUANTIZER_FP8,
    QUANTIZER_SYM,
    FcError,
    STATIC_SCRATCH_BYTES,
    allreduce_sim_rot,
    allreduce_sim_static,
    bench_lib,
    fused_compute_probe,
    dequantize_rot,
    quantize_rot,
    stream_reference,
    allreduce_sim,
    allreduce_sim_cmeta,
    allreduce_sim_fp8,
    allreduce_sim_sym,
    allreduce_sim_workspace_bytes,
    dequant_reduce_requant,
    dequant_reduce_requant_cmeta,
    dequant_reduce_requant_fp8,
    dequant_reduce_requant_sym,
    dequantize,
    dequantize_cmeta,
    dequantize_fp8,
    dequantize_sym,
    last_hip_error,
    lib,
    lib_path,
    quantize,
    quantize_cmeta,
    quantize_fp8,
    quantize_sym,
    strerror,
    version,
)

__all__ = [
    "QUANTIZER_ASYM", "QUANTIZER_FP8", "QUANTIZER_SYM", "allreduce_sim_rot", "dequantize_rot", "quantize_rot",
    "stream_reference", "allreduce_sim_static", "STATIC_SCRATCH_BYTES", "bench_lib", "fused_compute_probe",
    "FcError", "allreduce_sim", "allreduce_sim_fp8", "allreduce_sim_sym", "allreduce_sim_workspace_bytes",
    "dequant_reduce_requant", "dequant_reduce_requant_fp8", "dequant_reduce_requant_sym", "dequantize",
    "dequantize_fp8", "dequantize_sym", "last_hip_error", "lib", "lib_path", "quantize", "quantize_fp8",
    "quantize_sym", "strerror", "version",
    "allreduce_sim_cmeta", "dequant_reduce_requant_cmeta", "dequantize_cmeta", "quantize_cmeta",
]
