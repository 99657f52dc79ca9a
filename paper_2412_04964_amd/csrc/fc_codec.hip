// fc_codec.hip -- launchers of the stand-alone quantize and dequantize kernels.
#include "fc_device.hpp"
#include "fc_launch.hpp"

namespace fc {

template <int BITS, int LPG>
static void launch_q(dim3 grid, hipStream_t stream, const uint16_t *x, int64_t n_elems, int lpg,
                     int group_shift, uint8_t *c, float *scales, float *zeros)
{
    k_quantize<BITS, LPG><<<grid, dim3(kBlockThreads), 0, stream>>>(x, n_elems, lpg, group_shift, c,
                                                                   scales, zeros);
}

template <int BITS>
static void launch_q_bits(dim3 grid, hipStream_t stream, const uint16_t *x, int64_t n_elems, int lpg,
                          int group_shift, uint8_t *c, float *scales, float *zeros)
{
    switch (lpg) {
    case 1: launch_q<BITS, 1>(grid, stream, x, n_elems, lpg, group_shift, c, scales, zeros); break;
    case 2: launch_q<BITS, 2>(grid, stream, x, n_elems, lpg, group_shift, c, scales, zeros); break;
    case 4: launch_q<BITS, 4>(grid, stream, x, n_elems, lpg, group_shift, c, scales, zeros); break;
    default: launch_q<BITS, 0>(grid, stream, x, n_elems, lpg, group_shift, c, scales, zeros); break;
    }
}

hipError_t launch_quantize(int bits, const void *x_f16, int64_t n_elems, int lpg, int group_shift,
                           void *codes, float *scales, float *zeros, hipStream_t stream)
{
    const int64_t blocks = (n_elems + kBlockElems - 1) / kBlockElems;
    const dim3 grid((unsigned)blocks);
    const uint16_t *x = static_cast<const uint16_t *>(x_f16);
    uint8_t *c = static_cast<uint8_t *>(codes);
    if (bits == 4)
        launch_q_bits<4>(grid, stream, x, n_elems, lpg, group_shift, c, scales, zeros);
    else
        launch_q_bits<8>(grid, stream, x, n_elems, lpg, group_shift, c, scales, zeros);
    return hipGetLastError();
}

hipError_t launch_dequantize(int bits, const void *codes, const float *scales, const float *zeros,
                             int64_t n_elems, int group_shift, void *y_f16, hipStream_t stream)
{
    const int64_t blocks = (n_elems + kBlockElems - 1) / kBlockElems;
    const dim3 grid((unsigned)blocks), block(kBlockThreads);
    const uint8_t *c = static_cast<const uint8_t *>(codes);
    uint16_t *y = static_cast<uint16_t *>(y_f16);
    if (bits == 4)
        k_dequantize<4><<<grid, block, 0, stream>>>(c, scales, zeros, n_elems, group_shift, y);
    else
        k_dequantize<8><<<grid, block, 0, stream>>>(c, scales, zeros, n_elems, group_shift, y);
    return hipGetLastError();
}

}  // namespace fc
