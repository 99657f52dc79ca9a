// fc_device.hpp -- gfx950 device code of the Flash Communication quantization
// path: the group quantizer (paper Appendix, Eq. 1-2), its inverse, and the fused
// Dequantize x N -> ReduceSum -> FinegrainedQuantize body of Algorithm 1.
//
// Work decomposition (wave64): every lane owns 32 consecutive elements of the
// flattened [tokens*hidden] volume, so a group of g elements is g/32 adjacent
// lanes (4 lanes = one DPP quad for g = 128), a wavefront covers 2048 elements
// and a 256-thread workgroup covers 8192.  32 elements are exactly one 128-bit
// access of 4-bit codes, two of 8-bit codes and four of binary16 values.
// The per-group min/max is reduced in-lane first and then across the lanes of
// the group with DPP row operations; nothing goes through LDS or memory.
//
// Arithmetic contract (must match the header of include/fc.h operation by
// operation; the build passes -ffp-contract=off so that no product is fused
// into a sum unless written as fmaf here).
#pragma once

#include <hip/hip_runtime.h>
#include <float.h>
#include <stdint.h>

namespace fc {

constexpr int kLaneElems = 32;                       // elements per lane
constexpr int kBlockThreads = 256;                   // 4 wavefronts
constexpr int kBlockElems = kLaneElems * kBlockThreads;

typedef uint32_t u32;
typedef u32 u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ h2 as_h2(u32 v) { return __builtin_bit_cast(h2, v); }
__device__ __forceinline__ u32 as_u32(h2 v) { return __builtin_bit_cast(u32, v); }

// ---------------------------------------------------------------------------
// cross-lane min / max over the LPG adjacent lanes that share a group
// ---------------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ float dpp_read(float v)
{
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

constexpr int kDppQuadXor1 = 0xB1;      // quad_perm:[1,0,3,2]
constexpr int kDppQuadXor2 = 0x4E;      // quad_perm:[2,3,0,1]
constexpr int kDppRowHalfMirror = 0x141;  // lane i <-> 7-i inside each 8 lanes
constexpr int kDppRowMirror = 0x140;      // lane i <-> 15-i inside each 16 lanes

// All 64 lanes must be active when this is called.  lpg is a power of two, 1..64.
__device__ __forceinline__ void group_minmax(float &mn, float &mx, int lpg)
{
    if (lpg >= 2) {
        mn = fminf(mn, dpp_read<kDppQuadXor1>(mn));
        mx = fmaxf(mx, dpp_read<kDppQuadXor1>(mx));
    }
    if (lpg >= 4) {
        mn = fminf(mn, dpp_read<kDppQuadXor2>(mn));
        mx = fmaxf(mx, dpp_read<kDppQuadXor2>(mx));
    }
    if (lpg >= 8) {
        mn = fminf(mn, dpp_read<kDppRowHalfMirror>(mn));
        mx = fmaxf(mx, dpp_read<kDppRowHalfMirror>(mx));
    }
    if (lpg >= 16) {
        mn = fminf(mn, dpp_read<kDppRowMirror>(mn));
        mx = fmaxf(mx, dpp_read<kDppRowMirror>(mx));
    }
    if (lpg >= 32) {
        mn = fminf(mn, __shfl_xor(mn, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 16));
    }
    if (lpg >= 64) {
        mn = fminf(mn, __shfl_xor(mn, 32));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
    }
}

// ---------------------------------------------------------------------------
// Eq. 1: scale, reciprocal and zero-point of one group from its min and max
// ---------------------------------------------------------------------------
template <int BITS>
__device__ __forceinline__ void group_params(float mn, float mx, float &s, float &inv, float &zf)
{
    constexpr float qmax = (float)((1 << BITS) - 1);
    const float r = mx - mn;
    s = r / qmax;
    if (!(s >= FLT_MIN)) {                 // constant (or nearly constant) group
        const float a = fabsf(mn);
        s = (a >= FLT_MIN) ? a : 1.0f;
    }
    inv = 1.0f / s;
    zf = 0.0f - rintf(mn * inv);
}

// Eq. 2 for one element; returns the code as an integer in [0, 2^BITS-1].
template <int BITS>
__device__ __forceinline__ u32 encode(float x, float inv, float zf)
{
    constexpr float qmax = (float)((1 << BITS) - 1);
    const float t = rintf(x * inv);
    const float u = t + zf;
    return (u32)fminf(fmaxf(u, 0.0f), qmax);
}

// Quantize the lane's 32 fp32 values and store codes (+ the group's scale and
// zero-point from the group's first lane).  `e0` is the lane's first element.
template <int BITS>
__device__ __forceinline__ void quantize_and_store(const float (&v)[kLaneElems], bool live, int64_t e0,
                                                   int lpg, int group_shift,
                                                   uint8_t *__restrict__ codes,
                                                   float *__restrict__ scales,
                                                   float *__restrict__ zeros)
{
    float mn = v[0], mx = v[0];
#pragma unroll
    for (int i = 1; i < kLaneElems; ++i) {
        mn = fminf(mn, v[i]);
        mx = fmaxf(mx, v[i]);
    }
    group_minmax(mn, mx, lpg);
    float s, inv, zf;
    group_params<BITS>(mn, mx, s, inv, zf);

    if (!live) return;
    if (BITS == 4) {
        u32x4 out;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            u32 word = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) word |= encode<4>(v[8 * w + i], inv, zf) << (4 * i);
            out[w] = word;
        }
        *reinterpret_cast<u32x4 *>(codes + (e0 >> 1)) = out;
    } else {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            u32x4 out;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                u32 word = 0;
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    word |= encode<8>(v[16 * h + 4 * w + i], inv, zf) << (8 * i);
                out[w] = word;
            }
            *reinterpret_cast<u32x4 *>(codes + e0 + 16 * h) = out;
        }
    }
    if ((threadIdx.x & (lpg - 1)) == 0) {
        const int64_t gi = e0 >> group_shift;
        scales[gi] = s;
        zeros[gi] = zf;
    }
}

// ---------------------------------------------------------------------------
// Dequantize: d = q - z for the codes of one 32-bit word.
//
// Fast path (z an integer in [-1700, 1000], which covers every group whose
// range is not tiny against its offset): the code bits are OR-ed under a
// binary16 exponent so that the half reads 1024+q (or 64+q for a nibble that
// sits in bits 4-7); subtracting the half 1024+z (64+z) with one packed
// binary16 subtract gives the integer q-z for two codes at once.  All three
// numbers are integers of magnitude <= 2048, hence exact in binary16, and
// widening to fp32 is exact, so d is bit-identical to the fp32 (float)q - z.
// Slow path: convert and subtract in fp32.
// ---------------------------------------------------------------------------
struct ZeroConst {
    h2 c1024;   // (1024 + z, 1024 + z)
    h2 c64;     // (64 + z, 64 + z)
};

__device__ __forceinline__ bool zero_is_fast(float zf)
{
    return (zf == rintf(zf)) && (zf >= -1700.0f) && (zf <= 1000.0f);
}

__device__ __forceinline__ ZeroConst make_zero_const(float zf)
{
    ZeroConst c;
    const _Float16 a = (_Float16)(1024.0f + zf);
    const _Float16 b = (_Float16)(64.0f + zf);
    c.c1024 = h2{a, a};
    c.c64 = h2{b, b};
    return c;
}

// d[0..7] for the 8 nibbles of w (element i in bits 4i..4i+3), as binary16 pairs:
// p[0] = (d0, d4), p[1] = (d1, d5), p[2] = (d2, d6), p[3] = (d3, d7)
__device__ __forceinline__ void nibbles_minus_zero(u32 w, const ZeroConst &c, h2 (&p)[4])
{
    const u32 w8 = w >> 8;
    p[0] = as_h2((w & 0x000F000Fu) | 0x64006400u) - c.c1024;
    p[1] = as_h2((w & 0x00F000F0u) | 0x54005400u) - c.c64;
    p[2] = as_h2((w8 & 0x000F000Fu) | 0x64006400u) - c.c1024;
    p[3] = as_h2((w8 & 0x00F000F0u) | 0x54005400u) - c.c64;
}

// p[0] = (d0, d2), p[1] = (d1, d3) for the 4 bytes of w
__device__ __forceinline__ void bytes_minus_zero(u32 w, const ZeroConst &c, h2 (&p)[2])
{
    p[0] = as_h2((w & 0x00FF00FFu) | 0x64006400u) - c.c1024;
    p[1] = as_h2(((w >> 8) & 0x00FF00FFu) | 0x64006400u) - c.c1024;
}

// acc[i] = fma(q_i - z, s, acc[i]) for the lane's 32 codes of one source.
// `w` holds the raw code words: 4 words (4 bit) or 8 words (8 bit).
template <int BITS>
__device__ __forceinline__ void accumulate_source(const u32 *w, float s, float zf, bool wave_fast,
                                                  float (&acc)[kLaneElems])
{
    if (wave_fast) {
        const ZeroConst c = make_zero_const(zf);
        if (BITS == 4) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                h2 p[4];
                nibbles_minus_zero(w[k], c, p);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    acc[8 * k + i] = fmaf((float)p[i].x, s, acc[8 * k + i]);
                    acc[8 * k + 4 + i] = fmaf((float)p[i].y, s, acc[8 * k + 4 + i]);
                }
            }
        } else {
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                h2 p[2];
                bytes_minus_zero(w[k], c, p);
                acc[4 * k + 0] = fmaf((float)p[0].x, s, acc[4 * k + 0]);
                acc[4 * k + 2] = fmaf((float)p[0].y, s, acc[4 * k + 2]);
                acc[4 * k + 1] = fmaf((float)p[1].x, s, acc[4 * k + 1]);
                acc[4 * k + 3] = fmaf((float)p[1].y, s, acc[4 * k + 3]);
            }
        }
    } else {
        constexpr int per_word = 32 / BITS;
        constexpr u32 mask = (1u << BITS) - 1u;
#pragma unroll
        for (int k = 0; k < kLaneElems / per_word; ++k)
#pragma unroll
            for (int i = 0; i < per_word; ++i) {
                const float d = (float)((w[k] >> (BITS * i)) & mask) - zf;
                acc[per_word * k + i] = fmaf(d, s, acc[per_word * k + i]);
            }
    }
}

template <int BITS>
__device__ __forceinline__ void load_codes(const uint8_t *__restrict__ base, int64_t e0, u32 *w)
{
    if (BITS == 4) {
        const u32x4 a = *reinterpret_cast<const u32x4 *>(base + (e0 >> 1));
        w[0] = a[0]; w[1] = a[1]; w[2] = a[2]; w[3] = a[3];
    } else {
        const u32x4 a = *reinterpret_cast<const u32x4 *>(base + e0);
        const u32x4 b = *reinterpret_cast<const u32x4 *>(base + e0 + 16);
        w[0] = a[0]; w[1] = a[1]; w[2] = a[2]; w[3] = a[3];
        w[4] = b[0]; w[5] = b[1]; w[6] = b[2]; w[7] = b[3];
    }
}

// ---------------------------------------------------------------------------
// Kernels
// ---------------------------------------------------------------------------

// FinegrainedQuantize of binary16 input (Algorithm 1, first quantization).
template <int BITS>
__global__ __launch_bounds__(kBlockThreads) void k_quantize(
    const uint16_t *__restrict__ x, int64_t n_elems, int lpg, int group_shift,
    uint8_t *__restrict__ codes, float *__restrict__ scales, float *__restrict__ zeros)
{
    const int64_t e0 = ((int64_t)blockIdx.x * kBlockThreads + threadIdx.x) * kLaneElems;
    const bool live = e0 < n_elems;
    float v[kLaneElems];
    if (live) {
        const u32x4 *src = reinterpret_cast<const u32x4 *>(x + e0);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const u32x4 a = src[k];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const h2 p = as_h2(a[i]);
                v[8 * k + 2 * i] = (float)p.x;
                v[8 * k + 2 * i + 1] = (float)p.y;
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < kLaneElems; ++i) v[i] = 0.0f;
    }
    quantize_and_store<BITS>(v, live, e0, lpg, group_shift, codes, scales, zeros);
}

// Dequantize x NSRC, ReduceSum, FinegrainedQuantize (Algorithm 1, loop body
// between the two exchanges).  The fp32 sum lives in registers only.
template <int BITS_IN, int BITS_OUT, int NSRC>
__global__ __launch_bounds__(kBlockThreads) void k_dequant_reduce_requant(
    const uint8_t *__restrict__ codes_in, int64_t codes_stride,
    const float *__restrict__ scales_in, const float *__restrict__ zeros_in, int64_t meta_stride,
    int64_t n_elems, int lpg, int group_shift,
    uint8_t *__restrict__ codes_out, float *__restrict__ scales_out, float *__restrict__ zeros_out)
{
    constexpr int kWords = kLaneElems * BITS_IN / 32;
    const int64_t e0 = ((int64_t)blockIdx.x * kBlockThreads + threadIdx.x) * kLaneElems;
    const bool live = e0 < n_elems;
    const int64_t gi = e0 >> group_shift;

    u32 w[NSRC][kWords];
    float s[NSRC], zf[NSRC];
    if (live) {
#pragma unroll
        for (int j = 0; j < NSRC; ++j) {
            load_codes<BITS_IN>(codes_in + (int64_t)j * codes_stride, e0, w[j]);
            s[j] = scales_in[(int64_t)j * meta_stride + gi];
            zf[j] = zeros_in[(int64_t)j * meta_stride + gi];
        }
    } else {
#pragma unroll
        for (int j = 0; j < NSRC; ++j) {
#pragma unroll
            for (int k = 0; k < kWords; ++k) w[j][k] = 0;
            s[j] = 1.0f;
            zf[j] = 0.0f;
        }
    }

    float acc[kLaneElems];
#pragma unroll
    for (int i = 0; i < kLaneElems; ++i) acc[i] = 0.0f;
#pragma unroll
    for (int j = 0; j < NSRC; ++j) {
        const bool wave_fast = __builtin_amdgcn_ballot_w64(!zero_is_fast(zf[j])) == 0;
        accumulate_source<BITS_IN>(w[j], s[j], zf[j], wave_fast, acc);
    }
    quantize_and_store<BITS_OUT>(acc, live, e0, lpg, group_shift, codes_out, scales_out, zeros_out);
}

// Dequantize to binary16 (Algorithm 1, last step): y = half_rne((q - z) * s).
template <int BITS>
__global__ __launch_bounds__(kBlockThreads) void k_dequantize(
    const uint8_t *__restrict__ codes, const float *__restrict__ scales,
    const float *__restrict__ zeros, int64_t n_elems, int group_shift, uint16_t *__restrict__ y)
{
    constexpr int kWords = kLaneElems * BITS / 32;
    const int64_t e0 = ((int64_t)blockIdx.x * kBlockThreads + threadIdx.x) * kLaneElems;
    if (e0 >= n_elems) return;
    const int64_t gi = e0 >> group_shift;
    u32 w[kWords];
    load_codes<BITS>(codes, e0, w);
    const float s = scales[gi];
    const float zf = zeros[gi];

    // acc = fma(d, s, +0) equals the plain product d * s for every finite d, s
    // except that a negative-zero product becomes +0; (q - z) * s must keep its
    // sign, so the product is formed with an explicit multiply instead.
    float d[kLaneElems];
    const bool wave_fast = __builtin_amdgcn_ballot_w64(!zero_is_fast(zf)) == 0;
    if (wave_fast) {
        const ZeroConst c = make_zero_const(zf);
        if (BITS == 4) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                h2 p[4];
                nibbles_minus_zero(w[k], c, p);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    d[8 * k + i] = (float)p[i].x;
                    d[8 * k + 4 + i] = (float)p[i].y;
                }
            }
        } else {
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                h2 p[2];
                bytes_minus_zero(w[k], c, p);
                d[4 * k + 0] = (float)p[0].x;
                d[4 * k + 2] = (float)p[0].y;
                d[4 * k + 1] = (float)p[1].x;
                d[4 * k + 3] = (float)p[1].y;
            }
        }
    } else {
        constexpr int per_word = 32 / BITS;
        constexpr u32 mask = (1u << BITS) - 1u;
#pragma unroll
        for (int k = 0; k < kWords; ++k)
#pragma unroll
            for (int i = 0; i < per_word; ++i)
                d[per_word * k + i] = (float)((w[k] >> (BITS * i)) & mask) - zf;
    }

    u32x4 *dst = reinterpret_cast<u32x4 *>(y + e0);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        u32x4 out;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            h2 p;
            p.x = (_Float16)(d[8 * k + 2 * i] * s);
            p.y = (_Float16)(d[8 * k + 2 * i + 1] * s);
            out[i] = as_u32(p);
        }
        dst[k] = out;
    }
}

}  // namespace fc
