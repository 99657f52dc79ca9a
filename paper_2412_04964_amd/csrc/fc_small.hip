// fc_small.hip -- Algorithm 1 in ONE launch for volumes that launching, not memory, bounds.
//
// The paper's own design is a single fused kernel around its exchanges (Section 3.2.3, "Kernel Design"); on one
// device with identity exchanges the counterpart is a kernel that takes the N binary16 partials and writes the
// binary16 result, with both quantizations happening in registers.  Every rounding of the three-kernel path is
// kept: FinegrainedQuantize of each partial (Eq. 1-2) gives codes q_j, scale s_j and zero-point z_j of the group;
// the sum is acc = fma(q_j - z_j, s_j, acc) in source order from +0; FinegrainedQuantize of acc with the second
// bit-width; Dequantize to binary16.  Codes are formed literally as in Eq. 2 (the packed fast paths of the bulk
// kernels are proven equal to this form) and never leave the lane, so the result is bit-identical to
// fc_quantize x N -> fc_dequant_reduce_requant -> fc_dequantize while a decode-sized all-reduce costs one launch
// instead of three.
//
// Decomposition: a lane owns 8 consecutive elements (one 128-bit access of binary16), a wavefront 512; a group of
// g <= 512 elements is g/8 adjacent lanes, reduced with DPP / cross-lane steps.  A workgroup of NSRC wavefronts
// owns one 512-element tile of the result: wavefront j quantizes that tile of partial j (the expensive, independent
// part: min / max, Eq. 1, Eq. 2) and leaves q - z and the scale in LDS; after one barrier wavefront 0 runs the
// sequential fp32 FMA chain over the sources, requantizes, dequantizes and stores.  For a decode-sized volume a
// wavefront's work is a chain of dependent instructions with nothing to overlap it, so spreading the NSRC
// quantizations over wavefronts is what shortens the launch (N = 8: 7.4 -> about 4 us).
#include "fc_device.hpp"
#include "fc_launch.hpp"

namespace fc {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kSmallLaneElems = 8;
constexpr int kSmallWaveElems = 64 * kSmallLaneElems;

template <int BITS_RS, int BITS_AG, int NSRC>
__global__ __launch_bounds__(64 * NSRC) void k_allreduce_small(const uint16_t *__restrict__ x, int64_t n_elems, int lpg,
                                                              uint16_t *__restrict__ y)
{
    constexpr int E = kSmallLaneElems;
    // per source: q - z of the tile's 512 elements as fp32 (exact small integers, or the literal fp32 difference
    // for extreme zero-points) and the scale of each lane's group
    __shared__ __attribute__((aligned(16))) float diff[NSRC][64][E];
    __shared__ float scale[NSRC][64];

    const u32 lane = threadIdx.x & 63u, j = threadIdx.x >> 6;            // wavefront j <-> source j
    const int64_t e_tile = (int64_t)blockIdx.x * kSmallWaveElems;
    const int64_t left = (n_elems - e_tile) * 2;                         // bytes from the tile to the end of a partial

    {
        const rsrc_t rx = make_rsrc(x + (int64_t)j * n_elems + e_tile, left);
        const u32x4 raw = __builtin_amdgcn_raw_buffer_load_b128(rx, lane * 16, 0, kStreamLoadPolicy);
        float v[E];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const h2 p = as_h2(raw[k]);
            v[2 * k] = (float)p.x;
            v[2 * k + 1] = (float)p.y;
        }
        float mn, mx, s, inv, zf;
        lane_minmax(v, mn, mx);
        group_minmax<0>(mn, mx, lpg);
        group_params<BITS_RS>(mn, mx, s, inv, zf);
        float d[E];
#pragma unroll
        for (int i = 0; i < E; ++i) d[i] = (float)encode<BITS_RS>(v[i], inv, zf) - zf;      // Dequantize: q - z
        if constexpr (NSRC > 1) {
            f32x4 *mine = reinterpret_cast<f32x4 *>(&diff[j][lane][0]);
            mine[0] = f32x4{d[0], d[1], d[2], d[3]};
            mine[1] = f32x4{d[4], d[5], d[6], d[7]};
            scale[j][lane] = s;
            __syncthreads();
            if (j != 0) return;
        }

        float acc[E];
#pragma unroll
        for (int i = 0; i < E; ++i) acc[i] = 0.0f;
        if constexpr (NSRC > 1) {
#pragma unroll
            for (int k = 0; k < NSRC; ++k) {                                               // ReduceSum, source order
                const f32x4 lo = *reinterpret_cast<const f32x4 *>(&diff[k][lane][0]);
                const f32x4 hi = *reinterpret_cast<const f32x4 *>(&diff[k][lane][4]);
                const float sk = scale[k][lane];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    acc[i] = fmaf(lo[i], sk, acc[i]);
                    acc[4 + i] = fmaf(hi[i], sk, acc[4 + i]);
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < E; ++i) acc[i] = fmaf(d[i], s, acc[i]);
        }

        float mn2, mx2, s2, inv2, zf2;
        lane_minmax(acc, mn2, mx2);
        group_minmax<0>(mn2, mx2, lpg);
        group_params<BITS_AG>(mn2, mx2, s2, inv2, zf2);
        u32x4 out;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            h2 p;
            p.x = (_Float16)(((float)encode<BITS_AG>(acc[2 * k], inv2, zf2) - zf2) * s2);
            p.y = (_Float16)(((float)encode<BITS_AG>(acc[2 * k + 1], inv2, zf2) - zf2) * s2);
            out[k] = as_u32(p);
        }
        const rsrc_t ry = make_rsrc(y + e_tile, left);
        __builtin_amdgcn_raw_buffer_store_b128(out, ry, lane * 16, 0, kStreamStorePolicy);
    }
}

template <int BITS_RS, int BITS_AG>
static hipError_t launch_small_bits(const uint16_t *x, int n_src, int64_t n_elems, int group, uint16_t *y, hipStream_t stream)
{
    const dim3 grid((unsigned)((n_elems + kSmallWaveElems - 1) / kSmallWaveElems));
    const int lpg = group / kSmallLaneElems;
    switch (n_src) {
    case 1: return launch_kernel(k_allreduce_small<BITS_RS, BITS_AG, 1>, grid, dim3(64 * 1), stream, x, n_elems, lpg, y);
    case 2: return launch_kernel(k_allreduce_small<BITS_RS, BITS_AG, 2>, grid, dim3(64 * 2), stream, x, n_elems, lpg, y);
    case 3: return launch_kernel(k_allreduce_small<BITS_RS, BITS_AG, 3>, grid, dim3(64 * 3), stream, x, n_elems, lpg, y);
    case 4: return launch_kernel(k_allreduce_small<BITS_RS, BITS_AG, 4>, grid, dim3(64 * 4), stream, x, n_elems, lpg, y);
    case 5: return launch_kernel(k_allreduce_small<BITS_RS, BITS_AG, 5>, grid, dim3(64 * 5), stream, x, n_elems, lpg, y);
    case 6: return launch_kernel(k_allreduce_small<BITS_RS, BITS_AG, 6>, grid, dim3(64 * 6), stream, x, n_elems, lpg, y);
    case 7: return launch_kernel(k_allreduce_small<BITS_RS, BITS_AG, 7>, grid, dim3(64 * 7), stream, x, n_elems, lpg, y);
    case 8: return launch_kernel(k_allreduce_small<BITS_RS, BITS_AG, 8>, grid, dim3(64 * 8), stream, x, n_elems, lpg, y);
    default: return hipErrorInvalidValue;
    }
}

bool allreduce_small_applies(int64_t n_elems, int group)
{
    return group <= kSmallWaveElems && n_elems <= kSmallAllreduceMaxElems;
}

hipError_t launch_allreduce_small(int bits_rs, int bits_ag, const void *x_f16, int n_src, int64_t n_elems, int group,
                                  void *y_f16, hipStream_t stream)
{
    const uint16_t *x = static_cast<const uint16_t *>(x_f16);
    uint16_t *y = static_cast<uint16_t *>(y_f16);
    if (bits_rs == 4)
        return bits_ag == 4 ? launch_small_bits<4, 4>(x, n_src, n_elems, group, y, stream)
                            : launch_small_bits<4, 8>(x, n_src, n_elems, group, y, stream);
    return bits_ag == 4 ? launch_small_bits<8, 4>(x, n_src, n_elems, group, y, stream)
                        : launch_small_bits<8, 8>(x, n_src, n_elems, group, y, stream);
}

}  // namespace fc
