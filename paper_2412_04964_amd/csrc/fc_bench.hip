// fc_bench.hip -- measurement aid, built into its own shared library (libfc_bench.so, declared in
// include/fc_bench.h) so that the product library exports the method's entry points only.
//
// fc_stream_reference: the memory access pattern of the fused Dequantize x N -> ReduceSum ->
// FinegrainedQuantize kernel with the arithmetic and the scales / zero-points taken out.
// fc_fused_compute_probe: the opposite cut, that kernel's whole instruction stream with HBM taken out.
#include "fc_bench.h"

#include "fc_device.hpp"
#include "fc_launch.hpp"

namespace fc {

// NSRC input streams of `bytes` each, one output stream, out = XOR of the inputs; same 4 KB tile per
// workgroup, buffer-to-LDS staging, tile dealing and cache policy as k_dequant_reduce_requant.
template <int NSRC>
__global__ __launch_bounds__(fused_block_threads(1)) void k_stream_reference(const uint8_t *__restrict__ in, int64_t in_stride,
                                                   int64_t bytes, uint8_t *__restrict__ out)
{
    __shared__ __attribute__((aligned(16))) uint8_t landing[fused_block_threads(1) / 64][NSRC][1024];
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    constexpr int kTileBytes = fused_block_threads(1) * 16;
    const int64_t b_tile = (int64_t)xcd_tile<xcd_chunk(kTileBytes)>((u32)((bytes + kTileBytes - 1) / kTileBytes)) * kTileBytes;
#pragma unroll
    for (int j = 0; j < NSRC; ++j) {
        const rsrc_t r = make_rsrc(in + (int64_t)j * in_stride + b_tile, bytes - b_tile);
        dma_piece(r, tid * 16, &landing[wave][j][0]);
    }
    issue_order_fence();
    u32x4 acc = u32x4{0, 0, 0, 0};
#pragma unroll
    for (int j = 0; j < NSRC; ++j) {
        wait_vmem_outstanding(NSRC - 1 - j);
        u32x4 a = lds_read_b128_issue(&landing[wave][0][lane * 16], j * 1024);
        lds_read_complete(a);
        acc ^= a;
    }
    const rsrc_t ro = make_rsrc(out + b_tile, bytes - b_tile);
    __builtin_amdgcn_raw_buffer_store_b128(acc, ro, tid * 16, 0, kStreamStorePolicy);
}

template <int NSRC>
static hipError_t launch_sr(dim3 grid, hipStream_t stream, const uint8_t *in, int64_t in_stride, int64_t bytes, uint8_t *out)
{
    return launch_kernel(k_stream_reference<NSRC>, grid, dim3(fused_block_threads(1)), stream, in, in_stride, bytes, out);
}

}  // namespace fc

extern "C" int fc_stream_reference(const void *in, int64_t in_src_stride_bytes, int n_src, int64_t bytes, void *out,
                                   void *hip_stream)
{
    const auto aligned16 = [](const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; };
    if (n_src < 1 || n_src > 8 || bytes < 0 || (bytes & 15) != 0 || bytes > ((int64_t)1 << 36)) return -4;
    if (bytes == 0) return 0;
    if (!in || !out) return -1;
    if (n_src > 1) {
        if (in_src_stride_bytes < bytes) return -4;
        if ((in_src_stride_bytes & 15) != 0) return -5;
    } else {
        in_src_stride_bytes = 0;
    }
    if (!aligned16(in) || !aligned16(out)) return -5;
    const uint8_t *i = static_cast<const uint8_t *>(in);
    uint8_t *o = static_cast<uint8_t *>(out);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int64_t tile = fc::fused_block_threads(1) * 16;
    const dim3 grid((unsigned)((bytes + tile - 1) / tile));
    hipError_t e = hipErrorInvalidValue;
    switch (n_src) {
    case 1: e = fc::launch_sr<1>(grid, stream, i, in_src_stride_bytes, bytes, o); break;
    case 2: e = fc::launch_sr<2>(grid, stream, i, in_src_stride_bytes, bytes, o); break;
    case 3: e = fc::launch_sr<3>(grid, stream, i, in_src_stride_bytes, bytes, o); break;
    case 4: e = fc::launch_sr<4>(grid, stream, i, in_src_stride_bytes, bytes, o); break;
    case 5: e = fc::launch_sr<5>(grid, stream, i, in_src_stride_bytes, bytes, o); break;
    case 6: e = fc::launch_sr<6>(grid, stream, i, in_src_stride_bytes, bytes, o); break;
    case 7: e = fc::launch_sr<7>(grid, stream, i, in_src_stride_bytes, bytes, o); break;
    case 8: e = fc::launch_sr<8>(grid, stream, i, in_src_stride_bytes, bytes, o); break;
    }
    return e == hipSuccess ? 0 : -7;
}

// The fused kernel as the library launches it for the benchmark shapes, except that every workgroup works in the
// first 64 tiles of the volume (which stay in the L2): same grid, same instructions per wavefront, no HBM traffic.
extern "C" int fc_fused_compute_probe(const void *codes_in, int64_t codes_src_stride_bytes, const float *scales_in,
                                      const float *zeros_in, int64_t meta_src_stride_elems, int n_src, int64_t tokens,
                                      int64_t hidden, int group, int bits_in, int bits_out, void *codes_out,
                                      float *scales_out, float *zeros_out, void *hip_stream)
{
    using namespace fc;
    if (!codes_in || !scales_in || !zeros_in || !codes_out || !scales_out || !zeros_out) return -1;
    if (tokens <= 0 || hidden <= 0 || hidden % group != 0) return -4;
    const int64_t n = tokens * hidden;
    const uint8_t *ci = static_cast<const uint8_t *>(codes_in);
    uint8_t *co = static_cast<uint8_t *>(codes_out);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    constexpr int kWrap = 64;
    hipError_t e = hipErrorInvalidValue;
    auto grid = [&](int bits) { const int64_t tile = 128 * lane_elems(bits); return dim3((unsigned)((n + tile - 1) / tile)); };
    if (n < (int64_t)kWrap * 128 * 32) return -4;                       // the wrapped tiles must exist
    if (n_src == 4 && bits_in == 4 && bits_out == 4 && group == 128)
        e = launch_kernel(k_dequant_reduce_requant<4, 4, 4, 4, false, 128, kWrap>, grid(4), dim3(128), st, ci,
                          codes_src_stride_bytes, scales_in, zeros_in, meta_src_stride_elems, n, 7, co, scales_out,
                          zeros_out);
    else if (n_src == 4 && bits_in == 8 && bits_out == 8 && group == 128)
        e = launch_kernel(k_dequant_reduce_requant<8, 8, 4, 8, false, 128, kWrap>, grid(8), dim3(128), st, ci,
                          codes_src_stride_bytes, scales_in, zeros_in, meta_src_stride_elems, n, 7, co, scales_out,
                          zeros_out);
    else if (n_src == 8 && bits_in == 4 && bits_out == 4 && group == 64)
        e = launch_kernel(k_dequant_reduce_requant<4, 4, 8, 2, false, 128, kWrap>, grid(4), dim3(128), st, ci,
                          codes_src_stride_bytes, scales_in, zeros_in, meta_src_stride_elems, n, 6, co, scales_out,
                          zeros_out);
    else
        return -4;
    return e == hipSuccess ? 0 : -7;
}
