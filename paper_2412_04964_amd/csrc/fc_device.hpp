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

#ifdef FC_WAVES_PER_EU
#define FC_KERNEL_ATTRS __launch_bounds__(kBlockThreads) __attribute__((amdgpu_waves_per_eu(FC_WAVES_PER_EU)))
#else
#define FC_KERNEL_ATTRS __launch_bounds__(kBlockThreads)
#endif

constexpr int kLaneElems = 32;                       // elements per lane
constexpr int kBlockThreads = 256;                   // 4 wavefronts
constexpr int kBlockElems = kLaneElems * kBlockThreads;

typedef uint32_t u32;
typedef u32 u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ h2 as_h2(u32 v) { return __builtin_bit_cast(h2, v); }
__device__ __forceinline__ u32 as_u32(h2 v) { return __builtin_bit_cast(u32, v); }

// ---------------------------------------------------------------------------
// Buffer addressing.  Every global access goes through a raw buffer resource
// whose base is the (wave-uniform) start of the workgroup's tile and whose
// size is the number of bytes from there to the end of the array: the lane's
// position is a 32-bit offset, no 64-bit address lives in vector registers,
// and lanes beyond the end of the volume (the ragged last tile) read zeros and
// have their stores dropped by the hardware range check.
// ---------------------------------------------------------------------------
typedef __amdgpu_buffer_rsrc_t rsrc_t;
typedef __attribute__((address_space(3))) void lds_void;

// Cache policy of the bulk streams (codes, binary16 values): every byte is
// touched exactly once, so they are marked non-temporal, which measurably
// raises streaming bandwidth on this part (about +10 % for 4 reads : 1 write).
constexpr int kStreamPolicy = 2;      // "nt" bit of the buffer instruction

__device__ __forceinline__ rsrc_t make_rsrc(const void *base, int64_t bytes_left)
{
    const int n = bytes_left > 0x7FFFFFF0 ? 0x7FFFFFF0 : (bytes_left < 0 ? 0 : (int)bytes_left);
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, n, 0x00020000);
}

// Wait until at most `N` vector-memory operations of this wavefront are still
// outstanding (they complete in issue order).  The compiler does not order LDS
// reads after buffer-to-LDS loads by itself, so the landing-zone reads below are
// fenced explicitly; the "memory" clobber keeps the compiler from moving any
// memory access across the wait.
#define FC_WAIT_VM_CASE(k) case k: asm volatile("s_waitcnt vmcnt(" #k ")" ::: "memory"); break;
__device__ __forceinline__ void wait_vmem_outstanding(int n)
{
    switch (n) {   // n is a compile-time constant after unrolling; at most 8 sources x 2 pieces
        FC_WAIT_VM_CASE(1) FC_WAIT_VM_CASE(2) FC_WAIT_VM_CASE(3) FC_WAIT_VM_CASE(4) FC_WAIT_VM_CASE(5)
        FC_WAIT_VM_CASE(6) FC_WAIT_VM_CASE(7) FC_WAIT_VM_CASE(8) FC_WAIT_VM_CASE(9) FC_WAIT_VM_CASE(10)
        FC_WAIT_VM_CASE(11) FC_WAIT_VM_CASE(12) FC_WAIT_VM_CASE(13) FC_WAIT_VM_CASE(14)
    default: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
    }
}
#undef FC_WAIT_VM_CASE

__device__ __forceinline__ float load_f32(rsrc_t r, u32 byte_off)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, byte_off, 0, 0));
}

__device__ __forceinline__ void store_f32(rsrc_t r, u32 byte_off, float v)
{
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(u32, v), r, byte_off, 0, 0);
}

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

// All 64 lanes must be active when this is called.  The group spans `lpg`
// adjacent lanes (a power of two, 1..64); LPG > 0 fixes it at compile time,
// LPG == 0 reads the run-time value.
template <int LPG>
__device__ __forceinline__ void group_minmax(float &mn, float &mx, int lpg_rt)
{
    const int lpg = LPG > 0 ? LPG : lpg_rt;
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

// Fast packing of the lane's 32 codes (see quantize_and_store): Horner merge of
// t = rint(x*inv), optionally capped at tmax = qmax - z, plus z on every digit.
template <int BITS, bool CAP>
__device__ __forceinline__ void pack_codes(const float (&v)[kLaneElems], float inv, float zf, float tmax,
                                           u32 (&word)[kLaneElems * BITS / 32])
{
    auto digit = [&](float x) {
        const float t = rintf(x * inv);
        return CAP ? fminf(t, tmax) : t;
    };
    if constexpr (BITS == 4) {
        const float zc = zf * 4369.0f;               // z * (1 + 16 + 256 + 4096)
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            float t[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) t[i] = digit(v[8 * w + i]);
            const float lo = fmaf(fmaf(fmaf(t[3], 16.0f, t[2]), 16.0f, t[1]), 16.0f, t[0]) + zc;
            const float hi = fmaf(fmaf(fmaf(t[7], 16.0f, t[6]), 16.0f, t[5]), 16.0f, t[4]) + zc;
            word[w] = (u32)lo | ((u32)hi << 16);
        }
    } else {
        const float zc = zf * 257.0f;                // z * (1 + 256)
#pragma unroll
        for (int w = 0; w < 8; ++w) {
            float t[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) t[i] = digit(v[4 * w + i]);
            const float lo = fmaf(t[1], 256.0f, t[0]) + zc;
            const float hi = fmaf(t[3], 256.0f, t[2]) + zc;
            word[w] = (u32)lo | ((u32)hi << 16);
        }
    }
}

// Quantize the lane's 32 fp32 values and store codes (+ the group's scale and
// zero-point from the group's first lane).
//
// Packing, fast path (|z| <= 2048 in every lane of the wavefront): with
// t = rint(x*inv) the code is q = clamp(t + z, 0, qmax).  t >= rint(mn*inv) = -z
// because x >= mn and both the product and rint are monotone, so the lower clamp
// never acts, and since t, z and qmax are small integers the upper clamp can be
// applied to t: q = min(t, qmax - z) + z exactly.  Several codes are then merged
// in fp32 by Horner steps (t3*16 + t2)*16 + ... , every partial sum an integer
// below 2^24 and therefore exact, and z*(1 + 16 + 16^2 + 16^3) is added once.
// Otherwise each code is formed literally as in Eq. 2.
// `codes`, `scales`, `zeros` address the workgroup's tile; `code_off` is the
// lane's first output byte and `group_idx` the lane's group inside the tile.
template <int BITS, int LPG>
__device__ __forceinline__ void quantize_and_store(const float (&v)[kLaneElems], int lpg_rt,
                                                   rsrc_t codes, u32 code_off,
                                                   rsrc_t scales, rsrc_t zeros, u32 group_idx)
{
    constexpr float qmax = (float)((1 << BITS) - 1);
    float mn = v[0], mx = v[0];
#pragma unroll
    for (int i = 1; i < kLaneElems; ++i) {
        mn = fminf(mn, v[i]);
        mx = fmaxf(mx, v[i]);
    }
    group_minmax<LPG>(mn, mx, lpg_rt);
    float s, inv, zf;
    group_params<BITS>(mn, mx, s, inv, zf);
    const bool pack_fast = __builtin_amdgcn_ballot_w64(!(fabsf(zf) <= 2048.0f)) == 0;

    u32 word[kLaneElems * BITS / 32];
    if (pack_fast) {
        // every t of the group is <= rint(mx*inv); the cap is needed only if that exceeds qmax - z
        const float tmax = qmax - zf;
        const bool need_cap = __builtin_amdgcn_ballot_w64(rintf(mx * inv) > tmax) != 0;
        if (need_cap)
            pack_codes<BITS, true>(v, inv, zf, tmax, word);
        else
            pack_codes<BITS, false>(v, inv, zf, tmax, word);
    } else {
        constexpr int per_word = 32 / BITS;
#pragma unroll
        for (int w = 0; w < kLaneElems / per_word; ++w) {
            u32 acc = 0;
#pragma unroll
            for (int i = 0; i < per_word; ++i)
                acc |= encode<BITS>(v[per_word * w + i], inv, zf) << (BITS * i);
            word[w] = acc;
        }
    }
    __builtin_amdgcn_raw_buffer_store_b128(u32x4{word[0], word[1], word[2], word[3]}, codes, code_off, 0,
                                           kStreamPolicy);
    if constexpr (BITS == 8)
        __builtin_amdgcn_raw_buffer_store_b128(u32x4{word[4], word[5], word[6], word[7]}, codes,
                                               code_off + 16, 0, kStreamPolicy);
    const int lpg = LPG > 0 ? LPG : lpg_rt;
    if ((threadIdx.x & (lpg - 1)) == 0) {
        store_f32(scales, group_idx * 4, s);
        store_f32(zeros, group_idx * 4, zf);
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

// (a & mask) | orv in one VALU operation.  The compiler splits this into two
// VOP2 instructions when both constants are literals, so it is spelled out:
// the mask travels in an SGPR, the OR-ed exponent pattern in a VGPR.
__device__ __forceinline__ u32 and_or(u32 a, u32 mask, u32 orv)
{
    u32 r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "s"(mask), "v"(orv));
    return r;
}

// d[0..7] for the 8 nibbles of w (element i in bits 4i..4i+3), as binary16 pairs:
// p[0] = (d0, d4), p[1] = (d1, d5), p[2] = (d2, d6), p[3] = (d3, d7)
__device__ __forceinline__ void nibbles_minus_zero(u32 w, const ZeroConst &c, h2 (&p)[4])
{
    const u32 w8 = w >> 8;
    p[0] = as_h2(and_or(w, 0x000F000Fu, 0x64006400u)) - c.c1024;
    p[1] = as_h2(and_or(w, 0x00F000F0u, 0x54005400u)) - c.c64;
    p[2] = as_h2(and_or(w8, 0x000F000Fu, 0x64006400u)) - c.c1024;
    p[3] = as_h2(and_or(w8, 0x00F000F0u, 0x54005400u)) - c.c64;
}

// p[0] = (d0, d2), p[1] = (d1, d3) for the 4 bytes of w
__device__ __forceinline__ void bytes_minus_zero(u32 w, const ZeroConst &c, h2 (&p)[2])
{
    // v_perm_b32 picks each result byte from the pool {S1 = w: 0-3, S0 = magic: 4-7}
    p[0] = as_h2(__builtin_amdgcn_perm(0x64006400u, w, 0x05020500u)) - c.c1024;   // (b0, b2)
    p[1] = as_h2(__builtin_amdgcn_perm(0x64006400u, w, 0x05030501u)) - c.c1024;   // (b1, b3)
}

// acc[i] = fma(q_i - z, s, acc[i]) for the lane's 32 codes of one source.
// `w` holds the raw code words: 4 words (4 bit) or 8 words (8 bit).
template <int BITS>
__device__ __forceinline__ void accumulate_fast(const u32 *w, float s, const ZeroConst &c,
                                                float (&acc)[kLaneElems])
{
    if constexpr (BITS == 4) {
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
}

template <int BITS>
__device__ __forceinline__ void accumulate_general(const u32 *w, float s, float zf,
                                                   float (&acc)[kLaneElems])
{
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

// ---------------------------------------------------------------------------
// Kernels.  One workgroup = 256 threads = 4 wavefronts = one tile of 8192
// consecutive elements; wavefronts never synchronize with each other.
// ---------------------------------------------------------------------------

// FinegrainedQuantize of binary16 input (Algorithm 1, first quantization).
template <int BITS, int LPG>
__global__ FC_KERNEL_ATTRS void k_quantize(
    const uint16_t *__restrict__ x, int64_t n_elems, int lpg, int group_shift,
    uint8_t *__restrict__ codes, float *__restrict__ scales, float *__restrict__ zeros)
{
    const u32 tid = threadIdx.x;
    const int64_t e_tile = (int64_t)blockIdx.x * kBlockElems;
    const int64_t g_tile = e_tile >> group_shift;
    const int64_t n_groups = n_elems >> group_shift;
    const rsrc_t rx = make_rsrc(x + e_tile, (n_elems - e_tile) * 2);
    const rsrc_t rc = make_rsrc(codes + e_tile * BITS / 8, (n_elems - e_tile) * BITS / 8);
    const rsrc_t rs = make_rsrc(scales + g_tile, (n_groups - g_tile) * 4);
    const rsrc_t rz = make_rsrc(zeros + g_tile, (n_groups - g_tile) * 4);

    float v[kLaneElems];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const u32x4 a = __builtin_amdgcn_raw_buffer_load_b128(rx, tid * 64 + 16 * k, 0, kStreamPolicy);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const h2 p = as_h2(a[i]);
            v[8 * k + 2 * i] = (float)p.x;
            v[8 * k + 2 * i + 1] = (float)p.y;
        }
    }
    quantize_and_store<BITS, LPG>(v, lpg, rc, tid * (kLaneElems * BITS / 8), rs, rz,
                                  (tid * kLaneElems) >> group_shift);
}

// Dequantize x NSRC, ReduceSum, FinegrainedQuantize (Algorithm 1, loop body
// between the two exchanges).  The fp32 sum lives in registers only.
//
// Fan-in staging: at wavefront start every lane issues, for each of the NSRC
// sources, one (two for 8-bit codes) 128-bit buffer load that the memory
// pipeline writes straight into the wavefront's LDS landing zone, bypassing the
// vector registers.  All NSRC x 1 KB (2 KB) of a wavefront are therefore in
// flight at once while its registers hold only the 32 accumulators and the
// source currently being folded in, which keeps enough wavefronts resident per
// SIMD to cover HBM latency.  Each source is then read back with ds_read_b128
// (lane-contiguous, conflict-free) and accumulated.
template <int BITS_IN, int BITS_OUT, int NSRC, int LPG>
__global__ FC_KERNEL_ATTRS void k_dequant_reduce_requant(
    const uint8_t *__restrict__ codes_in, int64_t codes_stride,
    const float *__restrict__ scales_in, const float *__restrict__ zeros_in, int64_t meta_stride,
    int64_t n_elems, int lpg, int group_shift,
    uint8_t *__restrict__ codes_out, float *__restrict__ scales_out, float *__restrict__ zeros_out)
{
    constexpr int kLaneIn = kLaneElems * BITS_IN / 8;        // 16 or 32 bytes of codes per lane
    constexpr int kPieces = kLaneIn / 16;                     // 128-bit pieces per lane
    constexpr int kWords = kLaneElems * BITS_IN / 32;
    constexpr int kWaveElems = 64 * kLaneElems;
    constexpr int kMaxGw = LPG > 0 ? 64 / LPG : 8;            // groups per wavefront tile (upper bound)
    constexpr int kMetaIters = (NSRC * kMaxGw + 63) / 64;
    struct MetaRec { float s; u32 z; };                       // z: packed halves (fast) or fp32 bits
    __shared__ __attribute__((aligned(16))) uint8_t landing[kBlockThreads / 64][NSRC][kPieces][64 * 16];
    __shared__ MetaRec meta[kBlockThreads / 64][NSRC * kMaxGw];

    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const int64_t e_tile = (int64_t)blockIdx.x * kBlockElems;
    const int64_t g_tile = e_tile >> group_shift;
    const int64_t n_groups = n_elems >> group_shift;
    const u32 group_idx = (tid * kLaneElems) >> group_shift;

    // --- scale / zero-point table of the wavefront: its NSRC x gw entries are
    // spread over the lanes (one or a few entries each), checked and converted
    // once, and handed to the consuming lanes through LDS
    const int gw_shift = 11 - group_shift;                    // log2(groups per wavefront tile)
    const int gw = LPG > 0 ? 64 / LPG : (kWaveElems >> group_shift);
    const int entries = NSRC * gw;
    const int64_t g_wave = (e_tile + (int64_t)wave * kWaveElems) >> group_shift;
    float ms[kMetaIters], mz[kMetaIters];
    bool ok = true;
#pragma unroll
    for (int it = 0; it < kMetaIters; ++it) {
        const int idx = it * 64 + (int)lane;
        const int j = idx >> gw_shift, g = idx & (gw - 1);
        ms[it] = 0.0f;
        mz[it] = 0.0f;
        if (idx < entries && g_wave + g < n_groups) {
            const int64_t at = (int64_t)j * meta_stride + g_wave + g;
            ms[it] = scales_in[at];
            mz[it] = zeros_in[at];
        }
        ok = ok && zero_is_fast(mz[it]);
    }

    // --- codes: straight into the landing zone
#pragma unroll
    for (int j = 0; j < NSRC; ++j) {
        const rsrc_t rc = make_rsrc(codes_in + (int64_t)j * codes_stride + e_tile * BITS_IN / 8,
                                    (n_elems - e_tile) * BITS_IN / 8);
#pragma unroll
        for (int p = 0; p < kPieces; ++p)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rc, (lds_void *)&landing[wave][j][p][0], 16,
                                                     tid * kLaneIn + 16 * p, 0, 0, kStreamPolicy);
    }

    const bool all_fast = __builtin_amdgcn_ballot_w64(!ok) == 0;
#pragma unroll
    for (int it = 0; it < kMetaIters; ++it) {
        const int idx = it * 64 + (int)lane;
        if (idx < entries) {
            MetaRec r;
            r.s = ms[it];
            if (all_fast) {
                h2 c;
                c.x = (_Float16)(1024.0f + mz[it]);
                c.y = (_Float16)(64.0f + mz[it]);
                r.z = as_u32(c);
            } else {
                r.z = __builtin_bit_cast(u32, mz[it]);
            }
            meta[wave][idx] = r;
        }
    }
    const MetaRec *my_meta = &meta[wave][(lane * kLaneElems) >> group_shift];

    float acc[kLaneElems];
#pragma unroll
    for (int i = 0; i < kLaneElems; ++i) acc[i] = 0.0f;

    auto read_landing = [&](int j, u32 (&w)[kWords]) {
        // source j's pieces are complete once no more than the pieces of the
        // later sources (issued after it) are outstanding
        wait_vmem_outstanding((NSRC - 1 - j) * kPieces);
#pragma unroll
        for (int p = 0; p < kPieces; ++p) {
            const u32x4 a = *reinterpret_cast<const u32x4 *>(&landing[wave][j][p][lane * 16]);
            w[4 * p + 0] = a[0]; w[4 * p + 1] = a[1]; w[4 * p + 2] = a[2]; w[4 * p + 3] = a[3];
        }
    };

    if (all_fast) {
#pragma unroll
        for (int j = 0; j < NSRC; ++j) {
            u32 w[kWords];
            read_landing(j, w);
            const MetaRec r = my_meta[j * gw];
            const h2 c = as_h2(r.z);
            ZeroConst zc;
            zc.c1024 = h2{c.x, c.x};
            zc.c64 = h2{c.y, c.y};
            accumulate_fast<BITS_IN>(w, r.s, zc, acc);
        }
    } else {
#pragma unroll
        for (int j = 0; j < NSRC; ++j) {
            u32 w[kWords];
            read_landing(j, w);
            const MetaRec r = my_meta[j * gw];
            accumulate_general<BITS_IN>(w, r.s, __builtin_bit_cast(float, r.z), acc);
        }
    }

    const rsrc_t rc = make_rsrc(codes_out + e_tile * BITS_OUT / 8, (n_elems - e_tile) * BITS_OUT / 8);
    const rsrc_t rs = make_rsrc(scales_out + g_tile, (n_groups - g_tile) * 4);
    const rsrc_t rz = make_rsrc(zeros_out + g_tile, (n_groups - g_tile) * 4);
    quantize_and_store<BITS_OUT, LPG>(acc, lpg, rc, tid * (kLaneElems * BITS_OUT / 8), rs, rz, group_idx);
}

// Dequantize to binary16 (Algorithm 1, last step): y = half_rne((q - z) * s).
template <int BITS>
__global__ FC_KERNEL_ATTRS void k_dequantize(
    const uint8_t *__restrict__ codes, const float *__restrict__ scales,
    const float *__restrict__ zeros, int64_t n_elems, int group_shift, uint16_t *__restrict__ y)
{
    constexpr int kWords = kLaneElems * BITS / 32;
    const u32 tid = threadIdx.x;
    const int64_t e_tile = (int64_t)blockIdx.x * kBlockElems;
    const int64_t g_tile = e_tile >> group_shift;
    const int64_t n_groups = n_elems >> group_shift;
    const u32 group_idx = (tid * kLaneElems) >> group_shift;
    const rsrc_t rc = make_rsrc(codes + e_tile * BITS / 8, (n_elems - e_tile) * BITS / 8);
    const rsrc_t rs = make_rsrc(scales + g_tile, (n_groups - g_tile) * 4);
    const rsrc_t rz = make_rsrc(zeros + g_tile, (n_groups - g_tile) * 4);
    const rsrc_t ry = make_rsrc(y + e_tile, (n_elems - e_tile) * 2);

    const float s = load_f32(rs, group_idx * 4);
    const float zf = load_f32(rz, group_idx * 4);
    u32 w[kWords];
#pragma unroll
    for (int p = 0; p < kWords / 4; ++p) {
        const u32x4 a = __builtin_amdgcn_raw_buffer_load_b128(rc, tid * (kWords * 4) + 16 * p, 0, kStreamPolicy);
        w[4 * p + 0] = a[0]; w[4 * p + 1] = a[1]; w[4 * p + 2] = a[2]; w[4 * p + 3] = a[3];
    }

    float d[kLaneElems];
    const bool wave_fast = __builtin_amdgcn_ballot_w64(!zero_is_fast(zf)) == 0;
    if (wave_fast) {
        const ZeroConst c = make_zero_const(zf);
        if (BITS == 4) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                h2 p[4];
                nibbles_minus_zero(w[k % kWords], c, p);
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
                bytes_minus_zero(w[k % kWords], c, p);
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
        __builtin_amdgcn_raw_buffer_store_b128(out, ry, tid * 64 + 16 * k, 0, kStreamPolicy);
    }
}

}  // namespace fc
