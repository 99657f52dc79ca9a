// fc_codec.hip -- launchers of the stand-alone quantize and dequantize kernels.
#include "fc_device.hpp"
#include "fc_launch.hpp"

namespace fc {

template <int BITS, int LPG>
static void launch_q(int codec, hipStream_t stream, const uint16_t *x, int64_t n_elems, int lpg,
                     int group_shift, uint8_t *c, float *scales, float *zeros)
{
    constexpr int BT = quantize_block_threads(BITS, LPG);
    const int64_t tile = (int64_t)BT * lane_elems(BITS);
    const dim3 grid((unsigned)((n_elems + tile - 1) / tile)), block(BT);
    if (codec == CODEC_ASYM)
        k_quantize<BITS, LPG, kAsym><<<grid, block, 0, stream>>>(x, n_elems, lpg, group_shift, c, scales, zeros);
    else if (codec == CODEC_SYM)
        k_quantize<BITS, LPG, kSym><<<grid, block, 0, stream>>>(x, n_elems, lpg, group_shift, c, scales, nullptr);
    else if (codec == CODEC_ASYMH)
        k_quantize<BITS, LPG, kAsymH><<<grid, block, 0, stream>>>(x, n_elems, lpg, group_shift, c, scales, nullptr);
    else if constexpr (BITS == 8)
        k_quantize<8, LPG, kFp8><<<grid, block, 0, stream>>>(x, n_elems, lpg, group_shift, c, scales, nullptr);
}

template <int BITS>
static void launch_q_bits(int codec, hipStream_t stream, const uint16_t *x, int64_t n_elems, int group,
                          uint8_t *c, float *scales, float *zeros)
{
    const int lpg = group / lane_elems(BITS), sh = log2_int(group);
    switch (lpg) {
    case 1: launch_q<BITS, 1>(codec, stream, x, n_elems, lpg, sh, c, scales, zeros); break;
    case 2: launch_q<BITS, 2>(codec, stream, x, n_elems, lpg, sh, c, scales, zeros); break;
    case 4: launch_q<BITS, 4>(codec, stream, x, n_elems, lpg, sh, c, scales, zeros); break;
    case 8: launch_q<BITS, 8>(codec, stream, x, n_elems, lpg, sh, c, scales, zeros); break;
    default: launch_q<BITS, 0>(codec, stream, x, n_elems, lpg, sh, c, scales, zeros); break;
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
    if (bits == 4)
        launch_q_bits<4>(codec, stream, x, n_elems, group, c, scales, zeros);
    else
        launch_q_bits<8>(codec, stream, x, n_elems, group, c, scales, zeros);
    return hipGetLastError();
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
        k_dequantize<8, kFp8><<<grid, block, 0, stream>>>(c, scales, nullptr, n_elems, sh, y);
    } else if (codec == CODEC_ASYMH) {
        if (bits == 4)
            k_dequantize<4, kAsymH><<<grid, block, 0, stream>>>(c, scales, nullptr, n_elems, sh, y);
        else
            k_dequantize<8, kAsymH><<<grid, block, 0, stream>>>(c, scales, nullptr, n_elems, sh, y);
    } else if (bits == 4 && codec == CODEC_ASYM)
        k_dequantize<4, kAsym><<<grid, block, 0, stream>>>(c, scales, zeros, n_elems, sh, y);
    else if (bits == 4)
        k_dequantize<4, kSym><<<grid, block, 0, stream>>>(c, scales, nullptr, n_elems, sh, y);
    else if (codec == CODEC_ASYM)
        k_dequantize<8, kAsym><<<grid, block, 0, stream>>>(c, scales, zeros, n_elems, sh, y);
    else
        k_dequantize<8, kSym><<<grid, block, 0, stream>>>(c, scales, nullptr, n_elems, sh, y);
    return hipGetLastError();
}

template <int NSRC>
static void launch_sr(dim3 grid, hipStream_t stream, const uint8_t *in, int64_t in_stride, int64_t bytes, uint8_t *out)
{
    k_stream_reference<NSRC><<<grid, dim3(fused_block_threads(1)), 0, stream>>>(in, in_stride, bytes, out);
}

hipError_t launch_stream_reference(const void *in, int64_t in_stride, int n_src, int64_t bytes, void *out,
                                   hipStream_t stream)
{
    const uint8_t *i = static_cast<const uint8_t *>(in);
    uint8_t *o = static_cast<uint8_t *>(out);
    const int64_t tile = fused_block_threads(1) * 16;
    const dim3 grid((unsigned)((bytes + tile - 1) / tile));
    switch (n_src) {
    case 1: launch_sr<1>(grid, stream, i, in_stride, bytes, o); break;
    case 2: launch_sr<2>(grid, stream, i, in_stride, bytes, o); break;
    case 3: launch_sr<3>(grid, stream, i, in_stride, bytes, o); break;
    case 4: launch_sr<4>(grid, stream, i, in_stride, bytes, o); break;
    case 5: launch_sr<5>(grid, stream, i, in_stride, bytes, o); break;
    case 6: launch_sr<6>(grid, stream, i, in_stride, bytes, o); break;
    case 7: launch_sr<7>(grid, stream, i, in_stride, bytes, o); break;
    case 8: launch_sr<8>(grid, stream, i, in_stride, bytes, o); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace fc
