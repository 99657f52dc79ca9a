// fc_fused_small.hpp -- Dequantize x NSRC, ReduceSum, FinegrainedQuantize for volumes that launching bounds.
//
// A decode-sized volume (N = 8 partials of 8 x 8192 codes) is 64 wavefront tiles of the bulk kernel: a quarter of
// the compute units get one wavefront each, and that wavefront walks through 16 or 32 elements per lane and
// source as one chain of dependent instructions.  Here a lane owns ONE 32-bit word of codes per source (4
// elements at 8 bit, 8 at 4 bit), so the same volume spreads over four times as many single-wavefront workgroups
// and every chain is a quarter as long; all loads (codes, scales, zero-points of every source) are issued before
// the first use.  The arithmetic is the literal form of the contract in include/fc.h, the same that the bulk
// kernel's general path evaluates: d = (float)q - z, acc = fma(d, s, acc) in source order from +0, then Eq. 1-2
// on the sums.  Groups span g / E adjacent lanes (at most the wavefront: g <= 256 at 8 bit, 512 at 4 bit).
#pragma once

#include "fc_device.hpp"

namespace fc {

constexpr int fused_small_lane_elems(int bits_in) { return 32 / bits_in; }
constexpr int fused_small_wave_elems(int bits_in) { return 64 * fused_small_lane_elems(bits_in); }
// Up to this many wavefronts (eight per compute unit of the part) the launch is latency-bound and this kernel wins
// (decode shape, N = 8 at 8 bit: 2.63 -> 2.14 us per launch under graph replay; the two forms cross between 2048
// and 4096 wavefronts).
constexpr int kFusedSmallMaxWaves = 2048;

inline bool fused_small_applies(int bits_in, int64_t n_elems, int group)
{
    return group <= fused_small_wave_elems(bits_in) &&
           (n_elems + fused_small_wave_elems(bits_in) - 1) / fused_small_wave_elems(bits_in) <= kFusedSmallMaxWaves;
}

template <int BITS_IN, int BITS_OUT, int NSRC>
__global__ __launch_bounds__(64) void k_fused_small(
    const uint8_t *__restrict__ codes_in, int64_t codes_stride,
    const float *__restrict__ scales_in, const float *__restrict__ zeros_in, int64_t meta_stride,
    int64_t n_elems, int group_shift, int lpg,
    uint8_t *__restrict__ codes_out, float *__restrict__ scales_out, float *__restrict__ zeros_out)
{
    constexpr int E = fused_small_lane_elems(BITS_IN);
    constexpr u32 kMask = (1u << BITS_IN) - 1u;
    constexpr int kOutBytes = E * BITS_OUT / 8;                 // 2, 4 or 8 code bytes per lane
    const u32 lane = threadIdx.x;
    const int64_t e_wave = (int64_t)blockIdx.x * (64 * E);
    const int64_t e_lane = e_wave + (int64_t)lane * E;
    const bool live = e_lane < n_elems;                         // (the volume is a multiple of the group, hence of E)
    const int64_t n_groups = n_elems >> group_shift;
    const int64_t g_mine = e_lane >> group_shift;
    const int64_t gi = g_mine < n_groups ? g_mine : n_groups - 1;   // lanes beyond the end stay inside the arrays

    u32 w[NSRC];
    float s[NSRC], z[NSRC];
#pragma unroll
    for (int j = 0; j < NSRC; ++j) {
        const rsrc_t rc = make_rsrc(codes_in + (int64_t)j * codes_stride + e_wave * BITS_IN / 8,
                                    (n_elems - e_wave) * BITS_IN / 8);
        w[j] = __builtin_amdgcn_raw_buffer_load_b32(rc, lane * 4, 0, 0);
        s[j] = scales_in[(int64_t)j * meta_stride + gi];
        z[j] = zeros_in[(int64_t)j * meta_stride + gi];
    }

    float acc[E];
#pragma unroll
    for (int i = 0; i < E; ++i) acc[i] = 0.0f;
#pragma unroll
    for (int j = 0; j < NSRC; ++j)
#pragma unroll
        for (int i = 0; i < E; ++i) {
            const float d = (float)((w[j] >> (BITS_IN * i)) & kMask) - z[j];
            acc[i] = fmaf(d, s[j], acc[i]);
        }

    float mn, mx, s2, inv, zf;
    lane_minmax(acc, mn, mx);
    group_minmax<0>(mn, mx, lpg);
    group_params<BITS_OUT>(mn, mx, s2, inv, zf);
    uint64_t packed = 0;
#pragma unroll
    for (int i = 0; i < E; ++i) packed |= (uint64_t)encode<BITS_OUT>(acc[i], inv, zf) << (BITS_OUT * i);

    const rsrc_t ro = make_rsrc(codes_out + e_wave * BITS_OUT / 8, (n_elems - e_wave) * BITS_OUT / 8);
    if constexpr (kOutBytes == 8)
        __builtin_amdgcn_raw_buffer_store_b64(u32x2{(u32)packed, (u32)(packed >> 32)}, ro, lane * 8, 0, 0);
    else if constexpr (kOutBytes == 4)
        __builtin_amdgcn_raw_buffer_store_b32((u32)packed, ro, lane * 4, 0, 0);
    else
        __builtin_amdgcn_raw_buffer_store_b16((uint16_t)packed, ro, lane * 2, 0, 0);
    if (live && (lane & (u32)(lpg - 1)) == 0) {
        scales_out[g_mine] = s2;
        zeros_out[g_mine] = zf;
    }
}

}  // namespace fc
