// fc_fused.hip -- instantiations of the fused Dequantize-ReduceSum-Quantize
// kernel for one (FC_BITS_IN, FC_BITS_OUT) pair and every fan-in 1..8.
// Compiled once per pair (the build defines the two macros).
#include "fc_device.hpp"
#include "fc_fused_small.hpp"
#include "fc_launch.hpp"

#if !defined(FC_BITS_IN) || !defined(FC_BITS_OUT)
#error "define FC_BITS_IN and FC_BITS_OUT (4 or 8)"
#endif

#define FC_CAT3(a, b, c) a##b##_##c
#define FC_NAME(in, out) FC_CAT3(launch_fused_, in, out)

namespace fc {

template <int NSRC, int LPG>
static hipError_t launch_nl(const FusedArgs &a, hipStream_t stream)
{
    constexpr int BT = fused_block_threads(LPG);
    const int64_t tile = (int64_t)BT * lane_elems(FC_BITS_IN);
    const int64_t blocks = (a.n_elems + tile - 1) / tile;
#if FC_BITS_IN == 8 && FC_BITS_OUT == 8
    if (a.codec == CODEC_FP8) {
        return launch_kernel(k_dequant_reduce_requant_sym<8, 8, NSRC, LPG, true>, dim3((unsigned)blocks), dim3(BT), stream,
                static_cast<const uint8_t *>(a.codes_in), a.codes_stride, a.scales_in, a.meta_stride,
                a.n_elems, log2_int(a.group),
                static_cast<uint8_t *>(a.codes_out), a.scales_out);
    }
#endif
    if (a.codec == CODEC_SYM) {
        return launch_kernel(k_dequant_reduce_requant_sym<FC_BITS_IN, FC_BITS_OUT, NSRC, LPG>, dim3((unsigned)blocks), dim3(BT), stream,
                static_cast<const uint8_t *>(a.codes_in), a.codes_stride, a.scales_in, a.meta_stride,
                a.n_elems, log2_int(a.group),
                static_cast<uint8_t *>(a.codes_out), a.scales_out);
    }
    if (a.codec == CODEC_ASYMH) {
        return launch_kernel(k_dequant_reduce_requant<FC_BITS_IN, FC_BITS_OUT, NSRC, LPG, true>, dim3((unsigned)blocks), dim3(BT), stream,
                static_cast<const uint8_t *>(a.codes_in), a.codes_stride, a.scales_in, nullptr,
                a.meta_stride, a.n_elems, log2_int(a.group),
                static_cast<uint8_t *>(a.codes_out), a.scales_out, nullptr);
    }
    if (a.codec != CODEC_ASYM) return hipErrorInvalidValue;
    return launch_kernel(k_dequant_reduce_requant<FC_BITS_IN, FC_BITS_OUT, NSRC, LPG>, dim3((unsigned)blocks), dim3(BT), stream,
            static_cast<const uint8_t *>(a.codes_in), a.codes_stride, a.scales_in, a.zeros_in,
            a.meta_stride, a.n_elems, log2_int(a.group),
            static_cast<uint8_t *>(a.codes_out), a.scales_out, a.zeros_out);
}

// one instantiation per group width in lanes: 1 ... 128 lanes in 128-thread workgroups, 256 lanes in
// 256-thread workgroups (wider groups go to fc_wide.hip before this point)
template <int NSRC>
static hipError_t launch_n(const FusedArgs &a, hipStream_t stream)
{
    // launch-bound volumes (asymmetric quantizer, fp32 metadata): one code word per lane and source
    if (a.codec == CODEC_ASYM && fused_small_applies(FC_BITS_IN, a.n_elems, a.group)) {
        const int64_t wave_elems = fused_small_wave_elems(FC_BITS_IN);
        const int64_t waves = (a.n_elems + wave_elems - 1) / wave_elems;
        return launch_kernel(k_fused_small<FC_BITS_IN, FC_BITS_OUT, NSRC>, dim3((unsigned)waves), dim3(64), stream,
                static_cast<const uint8_t *>(a.codes_in), a.codes_stride, a.scales_in, a.zeros_in,
                a.meta_stride, a.n_elems, log2_int(a.group), a.group / fused_small_lane_elems(FC_BITS_IN),
                static_cast<uint8_t *>(a.codes_out), a.scales_out, a.zeros_out);
    }
    switch (a.group / lane_elems(FC_BITS_IN)) {
    case 1: return launch_nl<NSRC, 1>(a, stream);
    case 2: return launch_nl<NSRC, 2>(a, stream);
    case 4: return launch_nl<NSRC, 4>(a, stream);
    case 8: return launch_nl<NSRC, 8>(a, stream);
    case 16: return launch_nl<NSRC, 16>(a, stream);
    case 32: return launch_nl<NSRC, 32>(a, stream);
    case 64: return launch_nl<NSRC, 64>(a, stream);
    case 128: return launch_nl<NSRC, 128>(a, stream);
    case 256: return launch_nl<NSRC, 256>(a, stream);
    default: return hipErrorInvalidValue;
    }
}

hipError_t FC_NAME(FC_BITS_IN, FC_BITS_OUT)(const FusedArgs &a, hipStream_t stream)
{
    switch (a.n_src) {
    case 1: return launch_n<1>(a, stream);
    case 2: return launch_n<2>(a, stream);
    case 3: return launch_n<3>(a, stream);
    case 4: return launch_n<4>(a, stream);
    case 5: return launch_n<5>(a, stream);
    case 6: return launch_n<6>(a, stream);
    case 7: return launch_n<7>(a, stream);
    case 8: return launch_n<8>(a, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace fc
