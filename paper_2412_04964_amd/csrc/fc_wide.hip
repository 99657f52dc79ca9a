// fc_wide.hip -- kernels for groups wider than one wavefront's span (more than
// 64 lanes x 128 bits of codes): the coarse granularities of the paper's
// block-size study, up to one group per token (Section 3.2.1, block-size
// figure; rotation table of Section 4).
//
// One workgroup owns one group.  It is 128 or 256 threads wide and walks the
// group in P sub-tiles of blockDim.x 128-bit code pieces, so every global access
// stays one coalesced 16 bytes per lane; the lane's values of all P sub-tiles
// stay in registers between the min/max pass and the packing pass.  min/max are
// reduced in the lane, across the wavefront (DPP / shuffles), then across the
// wavefronts through a few LDS words and one barrier.  The group's scale and
// zero-point are uniform over the workgroup.  Arithmetic is the same
// device functions as the narrow kernels use, so results are bit-identical to
// the definition in include/fc.h.
#include "fc_device.hpp"
#include "fc_launch.hpp"

namespace fc {

// min and max over the whole workgroup; every wavefront must call it once
__device__ __forceinline__ void block_minmax(float &mn, float &mx, float (*slot)[2], u32 wave, u32 lane)
{
    group_minmax<0>(mn, mx, 64);
    if (lane == 0) {
        slot[wave][0] = mn;
        slot[wave][1] = mx;
    }
    __syncthreads();
    const u32 n_waves = blockDim.x >> 6;
    for (u32 w = 0; w < n_waves; ++w) {
        mn = fminf(mn, slot[w][0]);
        mx = fmaxf(mx, slot[w][1]);
    }
}

// FinegrainedQuantize of binary16 input, one group per workgroup.
template <int BITS, int P, int CODEC>
__global__ __launch_bounds__(kBlockThreads) void k_quantize_wide(
    const uint16_t *__restrict__ x, int group, uint8_t *__restrict__ codes,
    float *__restrict__ scales, float *__restrict__ zeros)
{
    constexpr int EPL = lane_elems(BITS);
    constexpr int kPieces = EPL * 2 / 16;                       // 1 KB input pieces per wavefront
    __shared__ __attribute__((aligned(16))) uint8_t img[P][kBlockWaves][kPieces * 1024];
    __shared__ float slot[kBlockWaves][2];

    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const int64_t e0 = (int64_t)blockIdx.x * group;
    const u32 sub_elems = blockDim.x * EPL;
    const rsrc_t rx = make_rsrc(x + e0, (int64_t)group * 2);
    const rsrc_t rc = make_rsrc(codes + e0 * BITS / 8, (int64_t)group * BITS / 8);

#pragma unroll
    for (int p = 0; p < P; ++p)
#pragma unroll
        for (int k = 0; k < kPieces; ++k)
            dma_piece(rx, (p * sub_elems + wave * 64 * EPL) * 2 + k * 1024 + lane * 16, &img[p][wave][k * 1024]);
    wait_vmem_outstanding(0);

    float v[P][EPL];
#pragma unroll
    for (int p = 0; p < P; ++p) {
        const u32x4 *mine = reinterpret_cast<const u32x4 *>(&img[p][wave][lane * (EPL * 2)]);
#pragma unroll
        for (int k = 0; k < kPieces; ++k) {
            const u32x4 a = mine[k];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const h2 h = as_h2(a[i]);
                v[p][8 * k + 2 * i] = (float)h.x;
                v[p][8 * k + 2 * i + 1] = (float)h.y;
            }
        }
    }

    float mn, mx;
    lane_minmax(v[0], mn, mx);
#pragma unroll
    for (int p = 1; p < P; ++p) {
        float a, b;
        lane_minmax(v[p], a, b);
        mn = fminf(mn, a);
        mx = fmaxf(mx, b);
    }
    block_minmax(mn, mx, slot, wave, lane);

    float s, inv, zf = 0.0f;
    if constexpr (CODEC == kFp8)
        group_params_absmax<448>(fmaxf(fabsf(mn), fabsf(mx)), s, inv);
    else if constexpr (CODEC == kSym)
        group_params_sym<BITS>(fmaxf(fabsf(mn), fabsf(mx)), s, inv);   // max|x| = max(|min|, |max|)
    else
        group_params<BITS, CODEC == kAsymH>(mn, mx, s, inv, zf);
#pragma unroll
    for (int p = 0; p < P; ++p) {
        u32 word[EPL * BITS / 32];
        if constexpr (CODEC == kFp8)
            pack_lane_fp8<EPL>(v[p], inv, word);
        else if constexpr (CODEC == kSym)
            pack_lane_sym<BITS, EPL>(v[p], inv, word);
        else
            pack_lane<BITS, EPL>(v[p], inv, zf, mx, word);
        __builtin_amdgcn_raw_buffer_store_b128(u32x4{word[0], word[1], word[2], word[3]}, rc,
                                               (p * blockDim.x + tid) * 16, 0, kStreamStorePolicy);
    }
    if (tid == 0) {
        scales[blockIdx.x] = CODEC == kAsymH ? __builtin_bit_cast(float, pack_meta(s, zf)) : s;
        if constexpr (CODEC == kAsym) zeros[blockIdx.x] = zf;
    }
}

// Dequantize x n_src, ReduceSum, FinegrainedQuantize, one group per workgroup.
template <int BITS_IN, int BITS_OUT, int P, int CODEC>
__global__ __launch_bounds__(kBlockThreads) void k_dequant_reduce_requant_wide(
    const uint8_t *__restrict__ codes_in, int64_t codes_stride,
    const float *__restrict__ scales_in, const float *__restrict__ zeros_in, int64_t meta_stride,
    int n_src, int group, uint8_t *__restrict__ codes_out,
    float *__restrict__ scales_out, float *__restrict__ zeros_out)
{
    constexpr int EPL = lane_elems(BITS_IN);
    constexpr int kOutBytes = EPL * BITS_OUT / 8;             // code bytes a lane writes per sub-tile
    __shared__ float slot[kBlockWaves][2];
    __shared__ __attribute__((aligned(16))) uint8_t out_img[kOutBytes == 32 ? kBlockWaves : 1]
                                                            [kOutBytes == 32 ? 2048 : 16];

    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const int64_t g_idx = blockIdx.x;
    const int64_t in_bytes = (int64_t)group * BITS_IN / 8;    // code bytes of the group per source
    const uint8_t *base = codes_in + g_idx * in_bytes;

    float acc[P][EPL];
#pragma unroll
    for (int p = 0; p < P; ++p)
#pragma unroll
        for (int i = 0; i < EPL; ++i) acc[p][i] = 0.0f;

    // Sources are taken in chunks of D = 4/P, so that a chunk is four 128-bit
    // pieces per lane; the next chunk is fetched while the current one is
    // folded in (two register buffers), which keeps up to eight pieces per
    // lane in flight.
    constexpr int D = 4 / P;
    auto fetch_chunk = [&](int j0, u32x4 (&dst)[D][P]) {
#pragma unroll
        for (int d = 0; d < D; ++d)
            if (j0 + d < n_src) {
                const rsrc_t r = make_rsrc(base + (int64_t)(j0 + d) * codes_stride, in_bytes);
#pragma unroll
                for (int p = 0; p < P; ++p)
                    dst[d][p] = __builtin_amdgcn_raw_buffer_load_b128(r, (p * blockDim.x + tid) * 16, 0,
                                                                      kStreamLoadPolicy);
            }
    };
    auto fold_chunk = [&](int j0, const u32x4 (&src)[D][P]) {
#pragma unroll
        for (int d = 0; d < D; ++d)
            if (j0 + d < n_src) {
                const int j = j0 + d;
                float s = scales_in[(int64_t)j * meta_stride + g_idx];
                if constexpr (CODEC == kFp8) {
#pragma unroll
                    for (int p = 0; p < P; ++p) {
                        const u32 w[4] = {src[d][p][0], src[d][p][1], src[d][p][2], src[d][p][3]};
                        accumulate_fp8(w, s, acc[p]);
                    }
                } else if constexpr (CODEC == kSym) {
                    const ZeroConst zc = sym_zero_const<BITS_IN>();
#pragma unroll
                    for (int p = 0; p < P; ++p) {
                        const u32 w[4] = {to_offset_binary<BITS_IN>(src[d][p][0]),
                                          to_offset_binary<BITS_IN>(src[d][p][1]),
                                          to_offset_binary<BITS_IN>(src[d][p][2]),
                                          to_offset_binary<BITS_IN>(src[d][p][3])};
                        accumulate_fast<BITS_IN>(w, s, zc, acc[p]);
                    }
                } else {
                    float zf;
                    if constexpr (CODEC == kAsymH)
                        unpack_meta(__builtin_bit_cast(u32, s), s, zf);
                    else
                        zf = zeros_in[(int64_t)j * meta_stride + g_idx];
                    const bool fast = zero_is_fast(zf);       // uniform over the workgroup
                    const ZeroConst zc = unpack_zero_const(pack_zero_const(fast ? zf : 0.0f));
#pragma unroll
                    for (int p = 0; p < P; ++p) {
                        const u32 w[4] = {src[d][p][0], src[d][p][1], src[d][p][2], src[d][p][3]};
                        if (fast)
                            accumulate_fast<BITS_IN>(w, s, zc, acc[p]);
                        else
                            accumulate_general<BITS_IN>(w, s, zf, acc[p]);
                    }
                }
            }
    };

    u32x4 buf0[D][P], buf1[D][P];
    fetch_chunk(0, buf0);
    for (int j0 = 0; j0 < n_src; j0 += 2 * D) {
        fetch_chunk(j0 + D, buf1);
        fold_chunk(j0, buf0);
        fetch_chunk(j0 + 2 * D, buf0);
        fold_chunk(j0 + D, buf1);
    }

    float mn, mx;
    lane_minmax(acc[0], mn, mx);
#pragma unroll
    for (int p = 1; p < P; ++p) {
        float a, b;
        lane_minmax(acc[p], a, b);
        mn = fminf(mn, a);
        mx = fmaxf(mx, b);
    }
    block_minmax(mn, mx, slot, wave, lane);

    float s, inv, zf = 0.0f;
    if constexpr (CODEC == kFp8)
        group_params_absmax<448>(fmaxf(fabsf(mn), fabsf(mx)), s, inv);
    else if constexpr (CODEC == kSym)
        group_params_sym<BITS_OUT>(fmaxf(fabsf(mn), fabsf(mx)), s, inv);
    else
        group_params<BITS_OUT, CODEC == kAsymH>(mn, mx, s, inv, zf);

    const int64_t out_bytes = (int64_t)group * BITS_OUT / 8;
    const u32 sub_out = blockDim.x * kOutBytes;               // output bytes of one sub-tile
#pragma unroll
    for (int p = 0; p < P; ++p) {
        u32 word[EPL * BITS_OUT / 32];
        if constexpr (CODEC == kFp8)
            pack_lane_fp8<EPL>(acc[p], inv, word);
        else if constexpr (CODEC == kSym)
            pack_lane_sym<BITS_OUT, EPL>(acc[p], inv, word);
        else
            pack_lane<BITS_OUT, EPL>(acc[p], inv, zf, mx, word);
        const rsrc_t rc = make_rsrc(codes_out + g_idx * out_bytes + (int64_t)p * sub_out,
                                    out_bytes - (int64_t)p * sub_out);
        store_codes<kOutBytes>(word, rc, wave, lane, &out_img[kOutBytes == 32 ? wave : 0][0]);
    }
    if (tid == 0) {
        scales_out[g_idx] = CODEC == kAsymH ? __builtin_bit_cast(float, pack_meta(s, zf)) : s;
        if constexpr (CODEC == kAsym) zeros_out[g_idx] = zf;
    }
}

// ---------------------------------------------------------------------------
// launchers.  The group is a power of two, at least two wavefront spans
// (128 lanes) and at most 16384 elements; threads = min(256, group/EPL) and
// P = group / (threads * EPL) is 1, 2 or 4.
// ---------------------------------------------------------------------------
namespace {

struct WideShape {
    int threads;
    int p;
};

WideShape wide_shape(int bits, int group)
{
    const int lanes = group / lane_elems(bits);
    WideShape w;
    w.threads = lanes < kBlockThreads ? lanes : kBlockThreads;
    w.p = lanes / w.threads;
    return w;
}

template <int BITS, int CODEC>
hipError_t quantize_wide_bits(const uint16_t *x, int64_t n_elems, int group, uint8_t *c,
                              float *scales, float *zeros, hipStream_t stream)
{
    const WideShape w = wide_shape(BITS, group);
    const dim3 grid((unsigned)(n_elems / group)), block(w.threads);
    switch (w.p) {
    case 1: return launch_kernel(k_quantize_wide<BITS, 1, CODEC>, grid, block, stream, x, group, c, scales, zeros);
    case 2: return launch_kernel(k_quantize_wide<BITS, 2, CODEC>, grid, block, stream, x, group, c, scales, zeros);
    case 4:
        if constexpr (BITS == 8)
            return launch_kernel(k_quantize_wide<BITS, 4, CODEC>, grid, block, stream, x, group, c, scales, zeros);
        [[fallthrough]];
    default: return hipErrorInvalidValue;
    }
}

template <int BI, int BO, int CODEC>
hipError_t fused_wide_bits(const FusedArgs &a, hipStream_t stream)
{
    const WideShape w = wide_shape(BI, a.group);
    const dim3 grid((unsigned)(a.n_elems / a.group)), block(w.threads);
    const uint8_t *ci = static_cast<const uint8_t *>(a.codes_in);
    uint8_t *co = static_cast<uint8_t *>(a.codes_out);
#define FC_WIDE_LAUNCH(PP)                                                                                  \
    launch_kernel(k_dequant_reduce_requant_wide<BI, BO, PP, CODEC>, grid, block, stream, ci, a.codes_stride, \
                  a.scales_in, a.zeros_in, a.meta_stride, a.n_src, a.group, co, a.scales_out, a.zeros_out)
    switch (w.p) {
    case 1: return FC_WIDE_LAUNCH(1);
    case 2: return FC_WIDE_LAUNCH(2);
    case 4:
        if constexpr (BI == 8) return FC_WIDE_LAUNCH(4);
        [[fallthrough]];
    default: return hipErrorInvalidValue;
    }
#undef FC_WIDE_LAUNCH
}

}  // namespace

hipError_t launch_quantize_wide(int bits, int codec, const void *x_f16, int64_t n_elems, int group,
                                void *codes, float *scales, float *zeros, hipStream_t stream)
{
    const uint16_t *x = static_cast<const uint16_t *>(x_f16);
    uint8_t *c = static_cast<uint8_t *>(codes);
    if (codec == CODEC_FP8)
        return bits == 8 ? quantize_wide_bits<8, kFp8>(x, n_elems, group, c, scales, nullptr, stream)
                         : hipErrorInvalidValue;
    if (codec == CODEC_ASYMH)
        return bits == 4 ? quantize_wide_bits<4, kAsymH>(x, n_elems, group, c, scales, nullptr, stream)
                         : quantize_wide_bits<8, kAsymH>(x, n_elems, group, c, scales, nullptr, stream);
    if (bits == 4)
        return codec == CODEC_ASYM ? quantize_wide_bits<4, kAsym>(x, n_elems, group, c, scales, zeros, stream)
                                   : quantize_wide_bits<4, kSym>(x, n_elems, group, c, scales, nullptr, stream);
    return codec == CODEC_ASYM ? quantize_wide_bits<8, kAsym>(x, n_elems, group, c, scales, zeros, stream)
                               : quantize_wide_bits<8, kSym>(x, n_elems, group, c, scales, nullptr, stream);
}

hipError_t launch_fused_wide(int bits_in, int bits_out, const FusedArgs &a, hipStream_t stream)
{
    if (a.codec == CODEC_FP8)
        return (bits_in == 8 && bits_out == 8) ? fused_wide_bits<8, 8, kFp8>(a, stream) : hipErrorInvalidValue;
    if (a.codec == CODEC_ASYMH) {
        if (bits_in == 4)
            return bits_out == 4 ? fused_wide_bits<4, 4, kAsymH>(a, stream) : fused_wide_bits<4, 8, kAsymH>(a, stream);
        return bits_out == 4 ? fused_wide_bits<8, 4, kAsymH>(a, stream) : fused_wide_bits<8, 8, kAsymH>(a, stream);
    }
    const bool sym = a.codec == CODEC_SYM;
    if (bits_in == 4 && bits_out == 4)
        return sym ? fused_wide_bits<4, 4, kSym>(a, stream) : fused_wide_bits<4, 4, kAsym>(a, stream);
    if (bits_in == 4)
        return sym ? fused_wide_bits<4, 8, kSym>(a, stream) : fused_wide_bits<4, 8, kAsym>(a, stream);
    if (bits_out == 4)
        return sym ? fused_wide_bits<8, 4, kSym>(a, stream) : fused_wide_bits<8, 4, kAsym>(a, stream);
    return sym ? fused_wide_bits<8, 8, kSym>(a, stream) : fused_wide_bits<8, 8, kAsym>(a, stream);
}

}  // namespace fc
