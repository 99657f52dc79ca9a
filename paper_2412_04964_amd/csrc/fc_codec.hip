// fc_codec.hip -- launchers of the stand-alone quantize and dequantize kernels.
#include "fc_device.hpp"
#include "fc_launch.hpp"

namespace fc {

template <int BITS, int LPG>
static void launch_q(dim3 grid, hipStream_t stream, const uint16_t *x, int64_t n_elems, int lpg,
                     int group_shift, uint8_t *c, float *scales, float *zeros)
{
    if (zeros)
        k_quantize<BITS, LPG, false><<<grid, dim3(kBlockThreads), 0, stream>>>(x, n_elems, lpg, group_shift,
                                                                              c, scales, zeros);
    else
        k_quantize<BITS, LPG, true><<<grid, dim3(kBlockThreads), 0, stream>>>(x, n_elems, lpg, group_shift,
                                                                             c, scales, nullptr);
}

template <int BITS>
static void launch_q_bits(hipStream_t stream, const uint16_t *x, int64_t n_elems, int group,
                          uint8_t *c, float *scales, float *zeros)
{
    const int64_t tile = block_elems(BITS);
    const dim3 grid((unsigned)((n_elems + tile - 1) / tile));
    const int lpg = group / lane_elems(BITS), sh = log2_int(group);
    switch (lpg) {
    case 1: launch_q<BITS, 1>(grid, stream, x, n_elems, lpg, sh, c, scales, zeros); break;
    case 2: launch_q<BITS, 2>(grid, stream, x, n_elems, lpg, sh, c, scales, zeros); break;
    case 4: launch_q<BITS, 4>(grid, stream, x, n_elems, lpg, sh, c, scales, zeros); break;
    case 8: launch_q<BITS, 8>(grid, stream, x, n_elems, lpg, sh, c, scales, zeros); break;
    default: launch_q<BITS, 0>(grid, stream, x, n_elems, lpg, sh, c, scales, zeros); break;
    }
}

hipError_t launch_quantize(int bits, const void *x_f16, int64_t n_elems, int group,
                           void *codes, float *scales, float *zeros, hipStream_t stream)
{
    if (is_wide_group(bits, group))
        return launch_quantize_wide(bits, x_f16, n_elems, group, codes, scales, zeros, stream);
    const uint16_t *x = static_cast<const uint16_t *>(x_f16);
    uint8_t *c = static_cast<uint8_t *>(codes);
    if (bits == 4)
        launch_q_bits<4>(stream, x, n_elems, group, c, scales, zeros);
    else
        launch_q_bits<8>(stream, x, n_elems, group, c, scales, zeros);
    return hipGetLastError();
}

hipError_t launch_dequantize(int bits, const void *codes, const float *scales, const float *zeros,
                             int64_t n_elems, int group, void *y_f16, hipStream_t stream)
{
    const uint8_t *c = static_cast<const uint8_t *>(codes);
    uint16_t *y = static_cast<uint16_t *>(y_f16);
    const int sh = log2_int(group);
    const int64_t tile = block_elems(bits);
    const dim3 grid((unsigned)((n_elems + tile - 1) / tile)), block(kBlockThreads);
    if (bits == 4 && zeros)
        k_dequantize<4, false><<<grid, block, 0, stream>>>(c, scales, zeros, n_elems, sh, y);
    else if (bits == 4)
        k_dequantize<4, true><<<grid, block, 0, stream>>>(c, scales, nullptr, n_elems, sh, y);
    else if (zeros)
        k_dequantize<8, false><<<grid, block, 0, stream>>>(c, scales, zeros, n_elems, sh, y);
    else
        k_dequantize<8, true><<<grid, block, 0, stream>>>(c, scales, nullptr, n_elems, sh, y);
    return hipGetLastError();
}

}  // namespace fc
