/*
 * fc_bench.h -- measurement aid of the MI355X Flash Communication quantization path, exported by
 * libfc_bench.so (NOT by the product library libfc.so; nothing in it is part of the paper's method).
 *
 * fc_stream_reference reproduces the memory access pattern of fc_dequant_reduce_requant (the fused
 * Dequantize x N, ReduceSum, FinegrainedQuantize body of Algorithm 1) with the arithmetic taken out:
 * it reads n_src device arrays of `bytes` bytes (source j at in + j*in_src_stride_bytes) and writes
 * their bytewise XOR to `out` (`bytes` bytes), with the fused kernel's tiling, staging, tile order and
 * cache policy.  bench.py times it next to the fused kernel to show how much bandwidth this access
 * pattern can reach on the machine at hand.
 *
 * All pointers are device pointers owned by the caller, 16-byte aligned; bytes % 16 == 0;
 * 1 <= n_src <= 8; in_src_stride_bytes >= bytes and a multiple of 16 (ignored when n_src == 1).
 * Work is enqueued on `hip_stream` (hipStream_t as void*, NULL = default stream); nothing is
 * allocated and nothing synchronizes.  Returns 0, or the negative code that fc.h names
 * (-1 NULL pointer, -4 shape, -5 alignment, -7 launch failure).  Argument checks make no HIP call.
 */
#ifndef FC_BENCH_H
#define FC_BENCH_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#if defined(__GNUC__)
__attribute__((visibility("default")))
#endif
int fc_stream_reference(const void *in, int64_t in_src_stride_bytes, int n_src, int64_t bytes,
                        void *out, void *hip_stream);

/*
 * The other cut through the same kernel: fc_dequant_reduce_requant's whole instruction stream with HBM
 * taken out.  Same arguments as fc_dequant_reduce_requant and the same launch (grid, workgroup size,
 * instructions per wavefront), but every workgroup works on one of the first 64 tiles of the volume, which
 * stay in the L2; the outputs are meaningless beyond those tiles.  Its launch time is what the kernel's
 * arithmetic costs on the part at hand, to be read next to fc_stream_reference (what its traffic costs).
 * Only the benchmark configurations are instantiated: (n_src, bits_in, bits_out, group) in
 * {(4,4,4,128), (4,8,8,128), (8,4,4,64)}, at least 64 tiles; anything else returns -4.  No alignment or
 * stride checks beyond NULL pointers: pass what fc_dequant_reduce_requant accepted.
 */
#if defined(__GNUC__)
__attribute__((visibility("default")))
#endif
int fc_fused_compute_probe(const void *codes_in, int64_t codes_src_stride_bytes, const float *scales_in,
                           const float *zeros_in, int64_t meta_src_stride_elems, int n_src, int64_t tokens,
                           int64_t hidden, int group, int bits_in, int bits_out, void *codes_out,
                           float *scales_out, float *zeros_out, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* FC_BENCH_H */
