// fc_sim.hip -- Algorithm 1 in ONE launch for volumes that memory bandwidth bounds.
//
// The paper's design is a single fused kernel around its two exchanges (Section 3.2.3, "Kernel Design").  On one
// device the exchanges are the identity, and the counterpart is a kernel that reads the N binary16 partials once and
// writes the binary16 result once: FinegrainedQuantize of every partial (Eq. 1-2), Dequantize and ReduceSum in
// source order, FinegrainedQuantize of the sum with the second bit-width and the final Dequantize all happen in
// registers, and no code, scale or zero-point travels through HBM.  Per output element that is 2 N + 2 bytes
// instead of the 2 N + 2 (N + 1) (b/8 + 8/g) + ... of the three-kernel sequence: 10 against 15.6 bytes at N = 4,
// INT4, g = 128.  Every rounding of the three-kernel sequence is kept, so the result is bit-identical to
// fc_quantize x N -> fc_dequant_reduce_requant -> fc_dequantize.
//
// Arithmetic, and why the shortcuts are exact:
//  * first quantization (binary16 input): s, 1/s and z come from group_params, the function the stand-alone
//    quantizer uses.  With t = rint(x * (1/s)) the code is q = clamp(t + z, 0, qmax) and Dequantize forms q - z.
//    For binary16 inputs z and t are integers below 2^20 (|z| <= 2^11 * 255), so both additions are exact and
//    q - z = clamp(t, -z, qmax - z): one median-of-three.  x * (1/s) is evaluated as a mixed-precision
//    multiply-add with a +0 addend straight from the binary16 value (widening is exact; adding +0 changes only the
//    sign of a zero product); the sign of a zero difference cannot reach the result, because the sum
//    acc = fma(q - z, s, acc) starts at +0 and a round-to-nearest sum is -0 only if both terms are.
//  * the group's min and max are taken on the binary16 pairs (packed min / max are exact in any format) and widened
//    afterwards; whether a zero minimum is +0 or -0 does not matter to Eq. 1 (the range, |min| and 0 - rint(min/s)
//    are the same).
//  * second quantization (fp32 sums) and final Dequantize: literally Eq. 2 and its inverse in fp32, because the
//    zero-point of a sum can be any fp32 integer: u = rint(acc * (1/s')) + z', q = clamp(u, 0, qmax),
//    y = half((q - z') * s').
//
//  * the other quantizers (one translation unit per quantizer, selected by FC_SIM_CODEC).  Symmetric (Eq. 3-4):
//    max|x| of a lane is max(|min|, |max|) of its packed min / max; neither clamp of Eq. 4 can act on a group's own
//    values, so the first stage contributes rint(x * (1/s)) itself, and the second stage adds +0 to its rint so that
//    a code of zero dequantizes to +0 as the stored integer does.  FP8: both stages go through the same conversion
//    instructions as the stand-alone kernels (the format keeps the sign of zero).  Binary16 metadata: group_params
//    rounds the scale and the zero-point as the stored word does; the zero-point stays an integer below 2^17, so
//    the median-of-three form of the first stage remains exact, lower clamp included.
//
// Decomposition: a lane owns 16 consecutive elements (two 128-bit pieces of binary16 per partial), a wavefront
// 1024, a workgroup of two wavefronts 2048; a group of g <= 1024 elements is g/16 adjacent lanes.  At wavefront
// start all N x 2 KB of the tile are requested as buffer-to-LDS loads (nothing sits in vector registers while in
// flight); the partials are then consumed in source order as they land.  The binary16 result leaves through the
// first landing zone as coalesced 1 KB pieces.
#include "fc_device.hpp"
#include "fc_launch.hpp"

namespace fc {

constexpr int kSimLaneElems = 16;
constexpr int kSimWaveElems = 64 * kSimLaneElems;
constexpr int kSimBlockThreads = 128;
constexpr int kSimTileElems = kSimBlockThreads * kSimLaneElems;
static_assert(kSimWaveElems == kFusedAllreduceMaxGroup && kSimTileElems == kFusedAllreduceTileElems,
              "the launcher's applicability test describes this decomposition");

// Packed binary16 min / max as single instructions (the compiler's own sequence first canonicalizes each input
// with a v_pk_max x, x; the inputs here come from memory and the result only has to be one of them).
__device__ __forceinline__ h2 pk_min(h2 a, h2 b)
{
    h2 r;
    asm("v_pk_min_f16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ h2 pk_max(h2 a, h2 b)
{
    h2 r;
    asm("v_pk_max_f16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

template <int CODEC, int BITS_RS, int BITS_AG, int NSRC, int LPG>
__global__ __launch_bounds__(kSimBlockThreads) void k_allreduce_fused(const uint16_t *__restrict__ x, int64_t n_elems,
                                                                     int lpg, uint16_t *__restrict__ y)
{
    constexpr int E = kSimLaneElems;
    constexpr int kZone = E * 2 * 64;                                  // bytes of one partial per wavefront: 2 KB
    constexpr int kWaves = kSimBlockThreads / 64;
    constexpr bool HM = CODEC == kAsymH;
    static_assert(2 * (NSRC - 1) <= kMaxCountedVmem, "landing-zone waits count the loads of the later sources");
    static_assert(CODEC != kFp8 || (BITS_RS == 8 && BITS_AG == 8), "E4M3 codes are bytes");
    __shared__ __attribute__((aligned(16))) uint8_t landing[kWaves][NSRC][kZone];

    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const u32 tile = xcd_tile<xcd_chunk(kSimTileElems * 2)>((u32)((n_elems + kSimTileElems - 1) / kSimTileElems));
    const int64_t e_tile = (int64_t)tile * kSimTileElems;
    const int64_t left = (n_elems - e_tile) * 2;                       // bytes from the tile to the end of a partial

#pragma unroll
    for (int j = 0; j < NSRC; ++j) {
        const rsrc_t rx = make_rsrc(x + (int64_t)j * n_elems + e_tile, left);
        dma_piece(rx, wave * kZone + lane * 16, &landing[wave][j][0]);
        dma_piece(rx, wave * kZone + 1024 + lane * 16, &landing[wave][j][1024]);
    }
    issue_order_fence();

    float acc[E];
#pragma unroll
    for (int i = 0; i < E; ++i) acc[i] = 0.0f;
#pragma unroll
    for (int j = 0; j < NSRC; ++j) {
        // source j has landed once no more than the loads of the later sources are outstanding
        wait_vmem_outstanding(2 * (NSRC - 1 - j));
        u32x4 a0 = lds_read_b128_issue(&landing[wave][0][lane * (E * 2)], j * kZone);
        u32x4 a1 = lds_read_b128_issue(&landing[wave][0][lane * (E * 2)], j * kZone + 16);
        lds_read_complete(a0);
        lds_read_complete(a1);
        const h2 p[8] = {as_h2(a0[0]), as_h2(a0[1]), as_h2(a0[2]), as_h2(a0[3]),
                         as_h2(a1[0]), as_h2(a1[1]), as_h2(a1[2]), as_h2(a1[3])};
        h2 lo = pk_min(p[0], p[1]), hi = pk_max(p[0], p[1]);
#pragma unroll
        for (int k = 2; k < 8; ++k) {
            lo = pk_min(lo, p[k]);
            hi = pk_max(hi, p[k]);
        }
        float mn = fminf((float)lo.x, (float)lo.y), mx = fmaxf((float)hi.x, (float)hi.y);
        float s, inv;
        if constexpr (is_asym(CODEC)) {
            group_minmax<LPG>(mn, mx, lpg);
            float zf;
            group_params<BITS_RS, HM>(mn, mx, s, inv, zf);
            const float d_lo = 0.0f - zf, d_hi = (float)((1 << BITS_RS) - 1) - zf;
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const float t0 = rintf(fmaf((float)p[k].x, inv, 0.0f));
                const float t1 = rintf(fmaf((float)p[k].y, inv, 0.0f));
                acc[2 * k] = fmaf(__builtin_amdgcn_fmed3f(t0, d_lo, d_hi), s, acc[2 * k]);
                acc[2 * k + 1] = fmaf(__builtin_amdgcn_fmed3f(t1, d_lo, d_hi), s, acc[2 * k + 1]);
            }
        } else {
            const float amax = group_max<LPG>(fmaxf(fabsf(mn), fabsf(mx)), lpg);
            if constexpr (CODEC == kSym) {
                group_params_sym<BITS_RS>(amax, s, inv);
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    acc[2 * k] = fmaf(rintf(fmaf((float)p[k].x, inv, 0.0f)), s, acc[2 * k]);
                    acc[2 * k + 1] = fmaf(rintf(fmaf((float)p[k].y, inv, 0.0f)), s, acc[2 * k + 1]);
                }
            } else {
                group_params_absmax<448>(amax, s, inv);
                float v[E];
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    v[2 * k] = (float)p[k].x;
                    v[2 * k + 1] = (float)p[k].y;
                }
                u32 word[4];
                pack_lane_fp8<E>(v, inv, word);
                accumulate_fp8(word, s, acc);
            }
        }
        pin_values(acc);              // source j is folded in before source j+1 is waited for
    }

    // FinegrainedQuantize of the sums and the final Dequantize: d[i] = the dequantized code before the scale
    float s, inv, d[E];
    if constexpr (is_asym(CODEC)) {
        float mn, mx, zf;
        lane_minmax(acc, mn, mx);
        group_minmax<LPG>(mn, mx, lpg);
        group_params<BITS_AG, HM>(mn, mx, s, inv, zf);
        constexpr float qmax = (float)((1 << BITS_AG) - 1);
#pragma unroll
        for (int i = 0; i < E; ++i) {
            const float u = rintf(acc[i] * inv) + zf;
            d[i] = __builtin_amdgcn_fmed3f(u, 0.0f, qmax) - zf;
        }
    } else {
        const float amax = group_max<LPG>(lane_absmax(acc), lpg);
        if constexpr (CODEC == kSym) {
            group_params_sym<BITS_AG>(amax, s, inv);
#pragma unroll
            for (int i = 0; i < E; ++i) d[i] = rintf(acc[i] * inv) + 0.0f;
        } else {
            group_params_absmax<448>(amax, s, inv);
            u32 word[4];
            pack_lane_fp8<E>(acc, inv, word);
            decode_fp8(word, d);
        }
    }
    u32x4 *mine = reinterpret_cast<u32x4 *>(&landing[wave][0][lane * (E * 2)]);
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        u32x4 out;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            h2 r;
            r.x = (_Float16)(d[8 * k + 2 * i] * s);
            r.y = (_Float16)(d[8 * k + 2 * i + 1] * s);
            out[i] = as_u32(r);
        }
        mine[k] = out;
    }
    const rsrc_t ry = make_rsrc(y + e_tile, left);
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const u32x4 o = *reinterpret_cast<const u32x4 *>(&landing[wave][0][k * 1024 + lane * 16]);
        __builtin_amdgcn_raw_buffer_store_b128(o, ry, wave * kZone + k * 1024 + lane * 16, 0, kStreamStorePolicy);
    }
}

#ifndef FC_SIM_CODEC
#error "compile with -DFC_SIM_CODEC=0..3 (kAsym, kSym, kFp8, kAsymH): one translation unit per quantizer"
#endif

namespace {

constexpr int CODEC = FC_SIM_CODEC;

template <int BITS_RS, int BITS_AG, int NSRC>
hipError_t launch_sim_src(const uint16_t *x, int64_t n_elems, int group, uint16_t *y, hipStream_t stream)
{
    const dim3 grid((unsigned)((n_elems + kSimTileElems - 1) / kSimTileElems)), block(kSimBlockThreads);
    const int lpg = group / kSimLaneElems;
    if (lpg == 8)                                                      // g = 128: the lane pattern is a constant
        return launch_kernel(k_allreduce_fused<CODEC, BITS_RS, BITS_AG, NSRC, 8>, grid, block, stream, x, n_elems,
                             lpg, y);
    return launch_kernel(k_allreduce_fused<CODEC, BITS_RS, BITS_AG, NSRC, 0>, grid, block, stream, x, n_elems, lpg, y);
}

template <int BITS_RS, int BITS_AG>
hipError_t launch_sim_bits(const uint16_t *x, int n_src, int64_t n_elems, int group, uint16_t *y, hipStream_t stream)
{
    switch (n_src) {
    case 1: return launch_sim_src<BITS_RS, BITS_AG, 1>(x, n_elems, group, y, stream);
    case 2: return launch_sim_src<BITS_RS, BITS_AG, 2>(x, n_elems, group, y, stream);
    case 3: return launch_sim_src<BITS_RS, BITS_AG, 3>(x, n_elems, group, y, stream);
    case 4: return launch_sim_src<BITS_RS, BITS_AG, 4>(x, n_elems, group, y, stream);
    case 5: return launch_sim_src<BITS_RS, BITS_AG, 5>(x, n_elems, group, y, stream);
    case 6: return launch_sim_src<BITS_RS, BITS_AG, 6>(x, n_elems, group, y, stream);
    case 7: return launch_sim_src<BITS_RS, BITS_AG, 7>(x, n_elems, group, y, stream);
    case 8: return launch_sim_src<BITS_RS, BITS_AG, 8>(x, n_elems, group, y, stream);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_sim_codec(int bits_rs, int bits_ag, const void *x_f16, int n_src, int64_t n_elems, int group,
                            void *y_f16, hipStream_t stream)
{
    const uint16_t *x = static_cast<const uint16_t *>(x_f16);
    uint16_t *y = static_cast<uint16_t *>(y_f16);
    if constexpr (CODEC == kFp8) {
        return (bits_rs == 8 && bits_ag == 8) ? launch_sim_bits<8, 8>(x, n_src, n_elems, group, y, stream)
                                              : hipErrorInvalidValue;
    } else {
        if (bits_rs == 4)
            return bits_ag == 4 ? launch_sim_bits<4, 4>(x, n_src, n_elems, group, y, stream)
                                : launch_sim_bits<4, 8>(x, n_src, n_elems, group, y, stream);
        return bits_ag == 4 ? launch_sim_bits<8, 4>(x, n_src, n_elems, group, y, stream)
                            : launch_sim_bits<8, 8>(x, n_src, n_elems, group, y, stream);
    }
}

}  // namespace

#if FC_SIM_CODEC == 0
hipError_t launch_allreduce_fused_asym(int bits_rs, int bits_ag, const void *x_f16, int n_src, int64_t n_elems,
                                       int group, void *y_f16, hipStream_t stream)
{
    return launch_sim_codec(bits_rs, bits_ag, x_f16, n_src, n_elems, group, y_f16, stream);
}
#elif FC_SIM_CODEC == 1
hipError_t launch_allreduce_fused_sym(int bits_rs, int bits_ag, const void *x_f16, int n_src, int64_t n_elems,
                                      int group, void *y_f16, hipStream_t stream)
{
    return launch_sim_codec(bits_rs, bits_ag, x_f16, n_src, n_elems, group, y_f16, stream);
}
#elif FC_SIM_CODEC == 2
hipError_t launch_allreduce_fused_fp8(int bits_rs, int bits_ag, const void *x_f16, int n_src, int64_t n_elems,
                                      int group, void *y_f16, hipStream_t stream)
{
    return launch_sim_codec(bits_rs, bits_ag, x_f16, n_src, n_elems, group, y_f16, stream);
}
#else
hipError_t launch_allreduce_fused_cmeta(int bits_rs, int bits_ag, const void *x_f16, int n_src, int64_t n_elems,
                                        int group, void *y_f16, hipStream_t stream)
{
    return launch_sim_codec(bits_rs, bits_ag, x_f16, n_src, n_elems, group, y_f16, stream);
}
#endif

}  // namespace fc
