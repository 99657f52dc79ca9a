// fc_launch.hpp -- host-side launch functions implemented by the .hip units.
// Internal to the library; the public interface is include/fc.h.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <tuple>
#include <utility>

namespace fc {

// Launch `kernel` and return the status of THIS launch.  (The <<< >>> syntax reports failures only
// through the thread's last-error slot, which hipGetLastError would also clear of errors that other
// code left there, and a stale one would be taken for a failure of a launch that succeeded.)
template <typename... P, size_t... I>
inline hipError_t launch_kernel_impl(void (*kernel)(P...), dim3 grid, dim3 block, hipStream_t stream,
                                     std::tuple<P...> &args, std::index_sequence<I...>)
{
    void *ptrs[] = {static_cast<void *>(&std::get<I>(args))...};
    return hipLaunchKernel(reinterpret_cast<const void *>(kernel), grid, block, ptrs, 0, stream);
}

template <typename... P, typename... A>
inline hipError_t launch_kernel(void (*kernel)(P...), dim3 grid, dim3 block, hipStream_t stream, A... a)
{
    static_assert(sizeof...(P) == sizeof...(A), "one argument per kernel parameter");
    std::tuple<P...> args{static_cast<P>(a)...};
    return launch_kernel_impl(kernel, grid, block, stream, args, std::index_sequence_for<P...>{});
}

// Quantizer: 0 = asymmetric (Eq. 1-2), 1 = symmetric (Eq. 3-4), 2 = FP8 E4M3 (8 bit only),
// 3 = asymmetric with binary16 metadata (one 32-bit word per group, passed where the other
// codecs pass `scales`); the values match kAsym / kSym / kFp8 / kAsymH of the device code.
// Only codec 0 uses the zero-point arrays.
enum { CODEC_ASYM = 0, CODEC_SYM = 1, CODEC_FP8 = 2, CODEC_ASYMH = 3 };

// n_elems = tokens*hidden (a multiple of `group`, which is a power of two in
// [32, 16384]).  All pointers are device pointers.
hipError_t launch_quantize(int bits, int codec, const void *x_f16, int64_t n_elems, int group,
                           void *codes, float *scales, float *zeros, hipStream_t stream);

hipError_t launch_dequantize(int bits, int codec, const void *codes, const float *scales, const float *zeros,
                             int64_t n_elems, int group, void *y_f16, hipStream_t stream);

struct FusedArgs {
    int codec;
    const void *codes_in;
    int64_t codes_stride;
    const float *scales_in;
    const float *zeros_in;
    int64_t meta_stride;
    int n_src;
    int64_t n_elems;
    int group;
    void *codes_out;
    float *scales_out;
    float *zeros_out;
};

// one translation unit per (bits_in, bits_out) pair
hipError_t launch_fused_4_4(const FusedArgs &a, hipStream_t stream);
hipError_t launch_fused_4_8(const FusedArgs &a, hipStream_t stream);
hipError_t launch_fused_8_4(const FusedArgs &a, hipStream_t stream);
hipError_t launch_fused_8_8(const FusedArgs &a, hipStream_t stream);

// fc_wide.hip holds one-group-per-workgroup kernels for coarse groups.  The
// stand-alone quantizer uses them for every group wider than one wavefront (64
// lanes x 128 bits of codes); the fused kernel reduces across the wavefronts of
// its workgroup itself and hands over only groups wider than its 256-lane tile.
inline bool is_wide_group(int bits, int group) { return group * bits / 128 > 64; }
inline bool exceeds_tile(int bits, int group) { return group * bits / 128 > 256; }

hipError_t launch_quantize_wide(int bits, int codec, const void *x_f16, int64_t n_elems, int group,
                                void *codes, float *scales, float *zeros, hipStream_t stream);
hipError_t launch_fused_wide(int bits_in, int bits_out, const FusedArgs &a, hipStream_t stream);

// Hadamard rotation fused into the quantizer / dequantizer (fc_rot.hip), applied to every aligned block of
// rotation_block(hidden) elements, which must be 1024, 2048, 4096 or 8192.
inline int rotation_block(int64_t hidden) { return (int)(hidden & -hidden); }     // largest power of two dividing hidden
hipError_t launch_quantize_rot(int bits, int codec, const void *x_f16, int64_t tokens, int hidden, int group,
                               void *codes, float *scales, float *zeros, hipStream_t stream);
hipError_t launch_dequantize_rot(int bits, int codec, const void *codes, const float *scales, const float *zeros,
                                 int64_t tokens, int hidden, int group, void *y_f16, hipStream_t stream);

// fc_small.hip: the whole all-reduce (asymmetric quantizer, fp32 metadata) in one launch, for launch-bound
// volumes: at most kSmallAllreduceMaxElems elements per partial and groups of at most 512 elements.
constexpr int64_t kSmallAllreduceMaxElems = (int64_t)1 << 20;
bool allreduce_small_applies(int64_t n_elems, int group);
hipError_t launch_allreduce_small(int bits_rs, int bits_ag, const void *x_f16, int n_src, int64_t n_elems, int group,
                                  void *y_f16, hipStream_t stream);

// fc_sim.hip (one translation unit per quantizer): the same in one launch for volumes that memory bandwidth bounds
// (the N binary16 partials are read once, the binary16 result is written once, nothing else touches memory);
// groups of at most 1024 elements, every quantizer.
constexpr int kFusedAllreduceMaxGroup = 1024;         // one wavefront's 64 lanes x 16 elements
constexpr int kFusedAllreduceTileElems = 2048;        // one workgroup; the tile count must fit the 32-bit workgroup index
inline bool allreduce_fused_applies(int64_t n_elems, int group)
{
    return group <= kFusedAllreduceMaxGroup && n_elems / kFusedAllreduceTileElems < 0x7FFFFFFF;
}
#define FC_DECLARE_SIM(name)                                                                                       \
    hipError_t launch_allreduce_fused_##name(int bits_rs, int bits_ag, const void *x_f16, int n_src, int64_t n_elems, \
                                             int group, void *y_f16, hipStream_t stream);
FC_DECLARE_SIM(asym) FC_DECLARE_SIM(sym) FC_DECLARE_SIM(fp8) FC_DECLARE_SIM(cmeta)
#undef FC_DECLARE_SIM
inline hipError_t launch_allreduce_fused(int codec, int bits_rs, int bits_ag, const void *x_f16, int n_src,
                                         int64_t n_elems, int group, void *y_f16, hipStream_t stream)
{
    switch (codec) {
    case CODEC_ASYM: return launch_allreduce_fused_asym(bits_rs, bits_ag, x_f16, n_src, n_elems, group, y_f16, stream);
    case CODEC_SYM: return launch_allreduce_fused_sym(bits_rs, bits_ag, x_f16, n_src, n_elems, group, y_f16, stream);
    case CODEC_FP8: return launch_allreduce_fused_fp8(bits_rs, bits_ag, x_f16, n_src, n_elems, group, y_f16, stream);
    case CODEC_ASYMH: return launch_allreduce_fused_cmeta(bits_rs, bits_ag, x_f16, n_src, n_elems, group, y_f16, stream);
    default: return hipErrorInvalidValue;
    }
}

inline int log2_int(int v)
{
    int s = 0;
    while ((1 << s) < v) ++s;
    return s;
}

}  // namespace fc
