// fc_codec.hip -- launchers of the stand-alone quantize and dequantize kernels.
#include "fc_device.hpp"
#include "fc_launch.hpp"

namespace fc {

template <int BITS, int LPG>
static hipError_t launch_q(int codec, hipStream_t stream, const uint16_t *x, int64_t n_elems, int lpg,
                     int group_shift, uint8_t *c, float *scales, float *zeros)
{
    constexpr int BT = quantize_block_threads(BITS, LPG);
    const int64_t tile = (int64_t)BT * lane_elems(BITS);
    const dim3 grid((unsigned)((n_elems + tile - 1) / tile)), block(BT);
    if (codec == CODEC_ASYM)
        return launch_kernel(k_quantize<BITS, LPG, kAsym>, grid, block, stream, x, n_elems, lpg, group_shift, c, scales, zeros);
    else if (codec == CODEC_SYM)
        return launch_kernel(k_quantize<BITS, LPG, kSym>, grid, block, stream, x, n_elems, lpg, group_shift, c, scales, nullptr);
    else if (codec == CODEC_ASYMH)
        return launch_kernel(k_quantize<BITS, LPG, kAsymH>, grid, block, stream, x, n_elems, lpg, group_shift, c, scales, nullptr);
    else if constexpr (BITS == 8)
        return launch_kernel(k_quantize<8, LPG, kFp8>, grid, block, stream, x, n_elems, lpg, group_shift, c, scales, nullptr);
    return hipErrorInvalidValue;
}

template <int BITS>
static hipError_t launch_q_bits(int codec, hipStream_t stream, const uint16_t *x, int64_t n_elems, int group,
                          uint8_t *c, float *scales, float *zeros)
{
    const int lpg = group / lane_elems(BITS), sh = log2_int(group);
    switch (lpg) {
    case 1: return launch_q<BITS, 1>(codec, stream, x, n_elems, lpg, sh, c, scales, zeros);
    case 2: return launch_q<BITS, 2>(codec, stream, x, n_elems, lpg, sh, c, scales, zeros);
    case 4: return launch_q<BITS, 4>(codec, stream, x, n_elems, lpg, sh, c, scales, zeros);
    case 8: return launch_q<BITS, 8>(codec, stream, x, n_elems, lpg, sh, c, scales, zeros);
    default: return launch_q<BITS, 0>(codec, stream, x, n_elems, lpg, sh, c, scales, zeros);
    }
}

hipError_t launch_quantize(int bits, int codec, const void *x_f16, int64_t n_elems, int group,
                           void *codes, float *scales, float *zeros, hipStream_t stream)
{
    if (codec == CODEC_FP8 && bits != 8) return hipErrorInvalidValue;
    if (is_wide_group(bits, group))
        return launch_quantize_wide(bits, codec, x_f16, n_elems, group, codes, scales, zeros, stream);
    const uint16_t *x = static_cast<const uint16_t *>(x_f16);
    uint8_t *c = static_cast<uint8_t *>(codes);
    if (bits == 4) return launch_q_bits<4>(codec, stream, x, n_elems, group, c, scales, zeros);
    return launch_q_bits<8>(codec, stream, x, n_elems, group, c, scales, zeros);
}

hipError_t launch_dequantize(int bits, int codec, const void *codes, const float *scales, const float *zeros,
                             int64_t n_elems, int group, void *y_f16, hipStream_t stream)
{
    const uint8_t *c = static_cast<const uint8_t *>(codes);
    uint16_t *y = static_cast<uint16_t *>(y_f16);
    const int sh = log2_int(group);
    const int64_t tile = block_elems(bits);
    const dim3 grid((unsigned)((n_elems + tile - 1) / tile)), block(kBlockThreads);
    if (codec == CODEC_FP8) {
        if (bits != 8) return hipErrorInvalidValue;
        return launch_kernel(k_dequantize<8, kFp8>, grid, block, stream, c, scales, nullptr, n_elems, sh, y);
    } else if (codec == CODEC_ASYMH) {
        if (bits == 4)
            return launch_kernel(k_dequantize<4, kAsymH>, grid, block, stream, c, scales, nullptr, n_elems, sh, y);
        else
            return launch_kernel(k_dequantize<8, kAsymH>, grid, block, stream, c, scales, nullptr, n_elems, sh, y);
    } else if (bits == 4 && codec == CODEC_ASYM)
        return launch_kernel(k_dequantize<4, kAsym>, grid, block, stream, c, scales, zeros, n_elems, sh, y);
    else if (bits == 4)
        return launch_kernel(k_dequantize<4, kSym>, grid, block, stream, c, scales, nullptr, n_elems, sh, y);
    else if (codec == CODEC_ASYM)
        return launch_kernel(k_dequantize<8, kAsym>, grid, block, stream, c, scales, zeros, n_elems, sh, y);
    else
        return launch_kernel(k_dequantize<8, kSym>, grid, block, stream, c, scales, nullptr, n_elems, sh, y);
}

}  // namespace fc
