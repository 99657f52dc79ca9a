// fc_device.hpp -- gfx950 device code of the Flash Communication quantization
// path: the group quantizers (paper Appendix, Eq. 1-2 asymmetric, Eq. 3-4
// symmetric, the FP8 E4M3 variant of the paper's precision table, and Eq. 1-2
// with binary16 metadata), their inverses, and the fused Dequantize x N -> ReduceSum -> FinegrainedQuantize body
// of Algorithm 1.  Groups wider than this file's kernels handle and the Hadamard
// rotation are in fc_wide.hip and fc_rot.hip, built from the same functions.
//
// Work decomposition (wave64).  On the code side every lane owns exactly one
// 128-bit access: EPL = 32 consecutive elements for 4-bit codes, 16 for 8-bit
// codes.  A group of g elements is therefore LPG = g/EPL adjacent lanes (4 lanes
// = one DPP quad for g = 128 at 4 bit), a wavefront covers 64*EPL elements and a
// workgroup of 2 or 4 wavefronts that many times more.  The per-group min/max is
// reduced in the lane first, then across the LPG lanes with DPP row operations
// (and, for groups of 128 or 256 lanes, across wavefronts through LDS).
//
// Memory access.  Every global access instruction of the bulk streams is one
// fully coalesced 128-bit-per-lane access (lane l of a wavefront touches bytes
// [16 l, 16 l + 16) of a 1 KB span).  Where a lane needs more than 16 contiguous
// bytes (binary16 values, 8-bit output of 32 elements) the wavefront's span is
// staged in LDS as an exact image of global memory and the lane reads or writes
// its contiguous part there.  Strided 16-byte pieces per lane, the obvious
// alternative, cost 25 % of the streaming bandwidth on this part (measured) and
// far more once the accesses are marked non-temporal.
//
// Arithmetic contract: must match the header of include/fc.h operation by
// operation; the build passes -ffp-contract=off so that no product is fused
// into a sum unless written as fmaf here.
#pragma once

#include <hip/hip_runtime.h>
#include <float.h>
#include <stdint.h>

#include <type_traits>

namespace fc {

constexpr int kBlockThreads = 256;                   // 4 wavefronts
constexpr int kBlockWaves = kBlockThreads / 64;

// quantizer selected by a template argument of the kernels
constexpr int kAsym = 0;    // Eq. 1-2: unsigned codes, scale and zero-point
constexpr int kSym = 1;     // Eq. 3-4: signed codes, scale only
constexpr int kFp8 = 2;     // FP8 E4M3 bytes, scale only (8-bit only)
constexpr int kAsymH = 3;   // Eq. 1-2 with the scale and zero-point stored as binary16, one 32-bit word per group
constexpr bool is_asym(int codec) { return codec == kAsym || codec == kAsymH; }

// elements per lane for a given code width: one 128-bit access of codes
constexpr int lane_elems(int bits) { return 128 / bits; }
constexpr int block_elems(int bits) { return kBlockThreads * lane_elems(bits); }

// The fused kernel runs 128-thread workgroups for groups of up to 128 lanes (128 lanes = both
// wavefronts of the workgroup): finer workgroups stream measurably faster (about 2 % on a bare
// 4-in/1-out copy, up to 3 % on the 8-bit fused kernel).  256-lane groups need 256 threads, the span
// over which the kernel reduces a group across wavefronts.
constexpr int fused_block_threads(int lpg) { return (lpg > 0 && lpg <= 128) ? 128 : kBlockThreads; }
// The stand-alone 4-bit quantizer gains the same way (1.8 %); the 8-bit one and the dequantizer do not.
constexpr int quantize_block_threads(int bits, int lpg) { return (bits == 4 && lpg > 0) ? 128 : kBlockThreads; }

typedef uint32_t u32;
typedef u32 u32x2 __attribute__((ext_vector_type(2)));
typedef u32 u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ h2 as_h2(u32 v) { return __builtin_bit_cast(h2, v); }
__device__ __forceinline__ u32 as_u32(h2 v) { return __builtin_bit_cast(u32, v); }

// ---------------------------------------------------------------------------
// Buffer addressing.  Bulk accesses go through a raw buffer resource whose base
// is the (wave-uniform) start of the workgroup's tile and whose size is the
// number of bytes from there to the end of the array: the lane's position is a
// 32-bit offset, no 64-bit address lives in vector registers, and lanes beyond
// the end of the volume (the ragged last tile) read zeros and have their stores
// dropped by the hardware range check.
// ---------------------------------------------------------------------------
typedef __amdgpu_buffer_rsrc_t rsrc_t;
typedef __attribute__((address_space(3))) void lds_void;

// Cache policy of the bulk streams (codes, binary16 values): every byte is
// touched exactly once.  Loads are marked non-temporal (+17 % on a bare 4 reads :
// 1 write stream against the default policy).  Stores are non-temporal with device
// scope: the scope bit makes them write through the XCD's L2 as they are issued,
// which is worth 2-5 % to the one-in / one-out codec kernels.  The non-temporal bit
// has to stay on the stores: without it a bare 4-in / 1-out stream gains 6 %, but as
// soon as a kernel also makes the small default-policy loads of scales and
// zero-points those loads stall (same HBM traffic by the counters, yet the fused
// kernel goes from 30.4 to 36.4 us and a bare stream with such loads added from
// 28.6 to 31.7 us).
constexpr int kStreamLoadPolicy = 2;       // "nt" bit of the buffer instruction
constexpr int kStreamStorePolicy = 2 | 16; // "nt" and "sc1" bits

__device__ __forceinline__ rsrc_t make_rsrc(const void *base, int64_t bytes_left)
{
    const int n = bytes_left > 0x7FFFFFF0 ? 0x7FFFFFF0 : (bytes_left < 0 ? 0 : (int)bytes_left);
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, n, 0x00020000);
}

// Landing zones: ordering by hand.
//
// A buffer-to-LDS load writes LDS when its data arrives, and the compiler does not reliably order LDS reads of
// that memory after it (in some control-flow shapes it waits for ALL outstanding vector-memory operations, in
// others for none).  The kernels therefore read a landing zone with an LDS instruction the compiler does not see
// (lds_read_b128_issue) and fence it themselves:
//     wait_vmem_outstanding(k);   a = lds_read_b128_issue(zone);   ...   lds_read_complete(a);   use a
// INVARIANT the callers keep: vector-memory operations of a wavefront complete in issue order, and vmcnt counts ALL
// of them, so "source j has landed" is "at most (number of vector-memory operations issued after source j's load)
// are outstanding".  Between the load of the first source and the read-out of the last one a kernel must
// therefore issue NO other vector-memory instruction (loads of scales and zero-points are issued BEFORE the first
// source; stores come after the last read-out), or `k` must count it.  The fan-in is at most 8, far below the 40
// cases spelled out below (beyond them the wait degrades to vmcnt(0), which is always sufficient).
//
// Building with -DFC_PLAIN_LANDING_READS replaces the scheme by its plain equivalent, a full vmcnt(0) before an
// ordinary LDS load that the compiler sees: slower, but free of hand-placed counts.  The build makes that variant
// of the fused kernels as well (libfc_plainreads.so) and the GPU tests run the fused parity cases through both,
// so that a compiler change that breaks the hand ordering shows up as a difference between the two.

// Wait until at most `n` vector-memory operations of this wavefront are still
// outstanding (they complete in issue order).  The "memory" clobber keeps the compiler
// from moving any memory access across the wait.  `n` must be wave-uniform.
#define FC_WAIT_VM_CASE(k) case k: asm volatile("s_waitcnt vmcnt(" #k ")" ::: "memory"); break;
__device__ __forceinline__ void wait_vmem_outstanding(int n)
{
#ifdef FC_PLAIN_LANDING_READS
    n = 0;
#endif
    switch (n) {
        FC_WAIT_VM_CASE(1) FC_WAIT_VM_CASE(2) FC_WAIT_VM_CASE(3) FC_WAIT_VM_CASE(4) FC_WAIT_VM_CASE(5)
        FC_WAIT_VM_CASE(6) FC_WAIT_VM_CASE(7) FC_WAIT_VM_CASE(8) FC_WAIT_VM_CASE(9) FC_WAIT_VM_CASE(10)
        FC_WAIT_VM_CASE(11) FC_WAIT_VM_CASE(12) FC_WAIT_VM_CASE(13) FC_WAIT_VM_CASE(14) FC_WAIT_VM_CASE(15)
        FC_WAIT_VM_CASE(16) FC_WAIT_VM_CASE(17) FC_WAIT_VM_CASE(18) FC_WAIT_VM_CASE(19) FC_WAIT_VM_CASE(20)
        FC_WAIT_VM_CASE(21) FC_WAIT_VM_CASE(22) FC_WAIT_VM_CASE(23) FC_WAIT_VM_CASE(24) FC_WAIT_VM_CASE(25)
        FC_WAIT_VM_CASE(26) FC_WAIT_VM_CASE(27) FC_WAIT_VM_CASE(28) FC_WAIT_VM_CASE(29) FC_WAIT_VM_CASE(30)
        FC_WAIT_VM_CASE(31) FC_WAIT_VM_CASE(32) FC_WAIT_VM_CASE(33) FC_WAIT_VM_CASE(34) FC_WAIT_VM_CASE(35)
        FC_WAIT_VM_CASE(36) FC_WAIT_VM_CASE(37) FC_WAIT_VM_CASE(38) FC_WAIT_VM_CASE(39) FC_WAIT_VM_CASE(40)
    default: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
    }
}
#undef FC_WAIT_VM_CASE
constexpr int kMaxCountedVmem = 40;      // largest count wait_vmem_outstanding spells out

// 128-bit LDS read that the compiler's wait-count bookkeeping does not see.  The value
// returned must not be used before lds_read_complete(v) has been called.
// `byte_off` (a compile-time constant once the caller's loop is unrolled, at most 65535) goes into the
// instruction's offset field, so one address register serves every landing slot of the wavefront.
__device__ __forceinline__ u32x4 lds_read_b128_issue(const void *p, int byte_off = 0)
{
#ifdef FC_PLAIN_LANDING_READS
    return *reinterpret_cast<const u32x4 *>(static_cast<const uint8_t *>(p) + byte_off);
#else
    u32x4 v;
    const u32 addr = (u32)(uintptr_t)(const __attribute__((address_space(3))) void *)p;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(byte_off) : "memory");
    return v;
#endif
}

// Waits for every LDS operation of the wavefront; `v` passes through so that
// no use of it can be scheduled in front of the wait.
__device__ __forceinline__ void lds_read_complete(u32x4 &v)
{
#ifdef FC_PLAIN_LANDING_READS
    asm volatile("" : "+v"(v) : : "memory");
#else
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(v) : : "memory");
#endif
}

// the compiler may not move memory operations across this point
__device__ __forceinline__ void issue_order_fence() { asm volatile("" ::: "memory"); }

// Pins the program position of the values in v[]: everything that produces them
// is emitted before this point and everything that consumes them after it.
// (Pure arithmetic is otherwise free to sink below later volatile statements,
// which here would collect all landing-zone reads first and keep every
// source's codes in registers at once.)  Generates no instruction.
template <int N>
__device__ __forceinline__ void pin_values(float (&v)[N])
{
    static_assert(N % 8 == 0, "pinned in groups of 8");
#pragma unroll
    for (int i = 0; i < N; i += 8)
        asm volatile("" : "+v"(v[i]), "+v"(v[i + 1]), "+v"(v[i + 2]), "+v"(v[i + 3]), "+v"(v[i + 4]),
                          "+v"(v[i + 5]), "+v"(v[i + 6]), "+v"(v[i + 7]));
}

// Workgroup -> tile.  Consecutive workgroup ids land on different XCDs (round
// robin over the 8 XCDs of the part).  Tiles are dealt in chunks: the i-th
// workgroup of XCD x takes tile ((i / CH) * 8 + x) * CH + i % CH, so each XCD
// streams runs of CH consecutive tiles (512 KB of every source) and the eight
// XCDs together advance through one window of 8 * CH tiles.  Measured on a bare
// 4-in / 1-out stream of the headline size: tile-by-tile interleaving of the XCDs
// 28.5 us, one contiguous eighth of the volume per XCD 25.8 us, chunks of 16 / 64 /
// 256 / 1024 tiles 25.7 / 25.5 / 25.1 / 25.6 us (fused kernels: 2-3 % where HBM
// bounds them).  Tiles beyond the last whole window keep the plain order; volumes
// smaller than a window use a smaller power-of-two chunk.
// n = number of workgroups of the launch.  The callers derive it from the volume instead of reading
// gridDim: the explicit kernel arguments are preloaded into scalar registers at wavefront start (see
// the build flags) while gridDim would cost a memory read before the first load can be issued, and
// these short-lived wavefronts are sensitive to that delay (1 % of the fused kernel's time).
template <int CH>
__device__ __forceinline__ u32 xcd_tile(u32 n)
{
    static_assert(CH > 0 && (CH & (CH - 1)) == 0, "chunk length is a power of two");
    const u32 b = blockIdx.x;
    if (n < 16u) return b;
    const u32 per_xcd = n >> 3;
    constexpr u32 kLogCh = (u32)__builtin_ctz((unsigned)CH);
    const u32 sh = per_xcd >= (u32)CH ? kLogCh : (u32)(31 - __builtin_clz(per_xcd));   // log2 of the chunk length
    const u32 window = 8u << sh;
    if (b >= (n & ~(window - 1u))) return b;
    const u32 x = b & 7u, i = b >> 3;
    return ((((i >> sh) << 3) + x) << sh) + (i & ((1u << sh) - 1u));
}
// chunk length for a tile of `tile_code_bytes` of every source: 512 KB runs
constexpr int xcd_chunk(int tile_code_bytes) { return (512 * 1024) / tile_code_bytes; }

// One coalesced 1 KB piece of a wavefront: lane l's 16 bytes at `off` (which
// already contains 16*l) go to lds_piece + 16*l.
__device__ __forceinline__ void dma_piece(rsrc_t r, u32 off, void *lds_piece)
{
    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lds_void *)lds_piece, 16, off, 0, 0, kStreamLoadPolicy);
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

constexpr int kDppQuadXor1 = 0xB1;        // quad_perm:[1,0,3,2]
constexpr int kDppQuadXor2 = 0x4E;        // quad_perm:[2,3,0,1]
constexpr int kDppRowHalfMirror = 0x141;  // lane i <-> 7-i inside each 8 lanes
constexpr int kDppRowMirror = 0x140;      // lane i <-> 15-i inside each 16 lanes

// min / max of a value with the same value in the lane that CTRL selects, in ONE instruction (the DPP operand
// modifier on v_min_f32 / v_max_f32 themselves).  Written as inline assembly because the compiler's own sequence
// is a DPP move, a canonicalizing v_max x, x and then the min: three instructions.  The instruction is the one
// fminf / fmaxf end in, so results are unchanged.  "s_nop 1": a DPP read of a register needs two wait states
// after the vector instruction that wrote it, which the compiler cannot insert for code it does not see.
template <int CTRL>
__device__ __forceinline__ float dpp_min(float v)
{
    float r;
    if constexpr (CTRL == kDppQuadXor1)
        asm("s_nop 1\n\tv_min_f32_dpp %0, %1, %1 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf bound_ctrl:1" : "=v"(r) : "v"(v));
    else if constexpr (CTRL == kDppQuadXor2)
        asm("s_nop 1\n\tv_min_f32_dpp %0, %1, %1 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf bound_ctrl:1" : "=v"(r) : "v"(v));
    else if constexpr (CTRL == kDppRowHalfMirror)
        asm("s_nop 1\n\tv_min_f32_dpp %0, %1, %1 row_half_mirror row_mask:0xf bank_mask:0xf bound_ctrl:1" : "=v"(r) : "v"(v));
    else {
        static_assert(CTRL == kDppRowMirror, "unsupported DPP control");
        asm("s_nop 1\n\tv_min_f32_dpp %0, %1, %1 row_mirror row_mask:0xf bank_mask:0xf bound_ctrl:1" : "=v"(r) : "v"(v));
    }
    return r;
}

template <int CTRL>
__device__ __forceinline__ float dpp_max(float v)
{
    float r;
    if constexpr (CTRL == kDppQuadXor1)
        asm("s_nop 1\n\tv_max_f32_dpp %0, %1, %1 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf bound_ctrl:1" : "=v"(r) : "v"(v));
    else if constexpr (CTRL == kDppQuadXor2)
        asm("s_nop 1\n\tv_max_f32_dpp %0, %1, %1 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf bound_ctrl:1" : "=v"(r) : "v"(v));
    else if constexpr (CTRL == kDppRowHalfMirror)
        asm("s_nop 1\n\tv_max_f32_dpp %0, %1, %1 row_half_mirror row_mask:0xf bank_mask:0xf bound_ctrl:1" : "=v"(r) : "v"(v));
    else {
        static_assert(CTRL == kDppRowMirror, "unsupported DPP control");
        asm("s_nop 1\n\tv_max_f32_dpp %0, %1, %1 row_mirror row_mask:0xf bank_mask:0xf bound_ctrl:1" : "=v"(r) : "v"(v));
    }
    return r;
}

// Second half of a wavefront-wide reduction: every lane holds the min (max) of its row of 16 lanes.
// row_bcast:15 gives rows 1 and 3 the value of the last lane of the row before them, row_bcast:31 gives rows 2
// and 3 the value of lane 31; afterwards lane 31 holds the result of lanes 0-31 and lane 63 that of the whole
// wavefront (lanes 32-63 after the first step alone).  Rows that a step does not address keep their value.
template <bool IS_MIN, bool FULL>
__device__ __forceinline__ float rows_reduce(float v)
{
    if constexpr (IS_MIN) {
        asm("s_nop 1\n\tv_min_f32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf" : "+v"(v));
        if constexpr (FULL) asm("s_nop 1\n\tv_min_f32_dpp %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf" : "+v"(v));
    } else {
        asm("s_nop 1\n\tv_max_f32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf" : "+v"(v));
        if constexpr (FULL) asm("s_nop 1\n\tv_max_f32_dpp %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf" : "+v"(v));
    }
    return v;
}

// min (max) over the 32-lane half (lpg == 32) or the whole wavefront (lpg == 64) that a lane belongs to, given
// the value already reduced over its row of 16 lanes
template <bool IS_MIN>
__device__ __forceinline__ float halves_or_wave(float v, int lpg, u32 lane)
{
    if (lpg >= 64) {
        const float t = rows_reduce<IS_MIN, true>(v);
        return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, t), 63));
    }
    const float t = rows_reduce<IS_MIN, false>(v);
    const float lo = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, t), 31));
    const float hi = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, t), 63));
    return lane < 32u ? lo : hi;
}

// All 64 lanes must be active when this is called.  The group spans `lpg`
// adjacent lanes (a power of two, 1..64); LPG > 0 fixes it at compile time,
// LPG == 0 reads the run-time value.
template <int LPG>
__device__ __forceinline__ void group_minmax(float &mn, float &mx, int lpg_rt)
{
    const int lpg = LPG > 0 ? LPG : lpg_rt;
    if (lpg >= 2) {
        mn = dpp_min<kDppQuadXor1>(mn);
        mx = dpp_max<kDppQuadXor1>(mx);
    }
    if (lpg >= 4) {
        mn = dpp_min<kDppQuadXor2>(mn);
        mx = dpp_max<kDppQuadXor2>(mx);
    }
    if (lpg >= 8) {
        mn = dpp_min<kDppRowHalfMirror>(mn);
        mx = dpp_max<kDppRowHalfMirror>(mx);
    }
    if (lpg >= 16) {
        mn = dpp_min<kDppRowMirror>(mn);
        mx = dpp_max<kDppRowMirror>(mx);
    }
    if (lpg >= 32) {
        const u32 lane = threadIdx.x & 63u;
        mn = halves_or_wave<true>(mn, lpg, lane);
        mx = halves_or_wave<false>(mx, lpg, lane);
    }
}

// ---------------------------------------------------------------------------
// Eq. 1: scale, reciprocal and zero-point of one group from its min and max.
//
// The two IEEE divisions are evaluated by short sequences that were checked on
// gfx950 against the `/` operator for every positive fp32 bit pattern:
//   r / qmax (qmax = 15, 255):  q0 = r*c,  e = fma(-qmax, q0, r),  q = fma(e, c, q0)
//       with c = RN(1/qmax): equal to the correctly rounded quotient for ALL
//       positive r, subnormal and huge included;
//   1 / s:  y0 = v_rcp_f32(s),  e = fma(-s, y0, 1),  y = fma(e, y0, y0): equal to
//       the correctly rounded reciprocal for all s in [2^-126, 2^126]; s is never
//       below FLT_MIN here, and a wavefront holding an s above 2^100 takes the
//       ordinary division.
// ---------------------------------------------------------------------------
//
// HM (binary16 metadata): the scale is rounded to binary16 (nearest even, kept in
// [2^-24, 65504]) before the reciprocal is taken, so that the zero-point and every
// code are computed from the number that is stored; the zero-point is then rounded
// to binary16 as well (saturating at +-65504; integers up to 2048 are unchanged).
template <int BITS, bool HM = false>
__device__ __forceinline__ void group_params(float mn, float mx, float &s, float &inv, float &zf)
{
    constexpr float qmax = (float)((1 << BITS) - 1);
    constexpr float c = 1.0f / qmax;
    const float r = mx - mn;
    const float q0 = r * c;
    const float e = fmaf(-qmax, q0, r);
    s = fmaf(e, c, q0);                    // == r / qmax
    if (!(s >= FLT_MIN)) {                 // constant (or nearly constant) group
        const float a = fabsf(mn);
        s = (a >= FLT_MIN) ? a : 1.0f;
    }
    if constexpr (HM) s = (float)(_Float16)__builtin_amdgcn_fmed3f(s, 0x1p-24f, 65504.0f);
    if (HM || __builtin_amdgcn_ballot_w64(!(s <= 0x1p100f)) == 0) {
        const float y0 = __builtin_amdgcn_rcpf(s);
        const float e1 = fmaf(-s, y0, 1.0f);
        inv = fmaf(e1, y0, y0);            // == 1 / s
    } else {
        inv = 1.0f / s;
    }
    float t = rintf(mn * inv);
    if constexpr (HM) t = __builtin_amdgcn_fmed3f(t, -65504.0f, 65504.0f);
    zf = 0.0f - t;
    if constexpr (HM) {
        // The difference is pinned in a register first: feeding it straight into the conversion lets
        // the compiler replace "0 - t" by a negation modifier on the operand, which turns the +0 that
        // a group starting at zero must store into -0.
        asm volatile("" : "+v"(zf));
        zf = (float)(_Float16)zf;
    }
}

// the metadata word of the binary16 variant: scale in bits 0-15, zero-point in bits 16-31
__device__ __forceinline__ u32 pack_meta(float s, float zf)
{
    h2 m;
    m.x = (_Float16)s;                     // both are binary16 numbers already
    m.y = (_Float16)zf;
    return as_u32(m);
}

__device__ __forceinline__ void unpack_meta(u32 w, float &s, float &zf)
{
    const h2 m = as_h2(w);
    s = (float)m.x;
    zf = (float)m.y;
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

// Fast packing of the lane's codes (see pack_lane): rounding and merging in the integer view of fp32 numbers.
//   u = x*inv + M with M = 1.5 * 2^23: every fp32 in [2^23, 2^24) is an integer, so this addition rounds x*inv to
//       an integer with ties to the even one (M is even): u = M + rint(x*inv) exactly, the same t = rint(x*inv)
//       that v_rndne_f32 gives, and the bit pattern of u is bits(M) + t as a 32-bit integer (t may be negative).
//   Horner steps h = (h << BITS) + bits(u_i) (one v_lshl_add_u32 per code) merge a whole 32-bit word of codes;
//       modulo 2^32 the result is bits(M) * 0x11..1 + sum t_i << (BITS * i).
//   Adding (z - bits(M)) * 0x11..1 once per word leaves sum (t_i + z) << (BITS * i), and every digit t_i + z lies in
//       [0, 2^BITS - 1] (lower clamp idle, upper clamp applied to u beforehand when CAP), so no carry crosses a digit.
// z * 0x11..1 = (z * 0x1111) * 0x10001 is formed from the exact fp32 product z * 4369 (|z| < 2048).
template <int BITS, int EPL, bool CAP>
__device__ __forceinline__ void pack_codes(const float (&v)[EPL], float inv, float zf, float tmax,
                                           u32 (&word)[EPL * BITS / 32])
{
    constexpr float kMagic = 12582912.0f;
    constexpr u32 kMagicBits = 0x4B400000u;
    constexpr int per_word = 32 / BITS;
    constexpr u32 kOnes = BITS == 4 ? 0x11111111u : 0x01010101u;
    const float cap = kMagic + tmax;
    const u32 zc = (u32)(int)(zf * (BITS == 4 ? 4369.0f : 257.0f));      // z * 0x1111 (z * 0x0101)
    const u32 fix = (zc + (zc << 16)) - kMagicBits * kOnes;
#pragma unroll
    for (int w = 0; w < EPL / per_word; ++w) {
        u32 h = 0;
#pragma unroll
        for (int i = per_word - 1; i >= 0; --i) {
            const float r = v[per_word * w + i] * inv;
            float u = r + kMagic;
            if constexpr (CAP) u = fminf(u, cap);
            h = (h << BITS) + __builtin_bit_cast(u32, u);
        }
        word[w] = h + fix;
    }
}

// FinegrainedQuantize of the lane's EPL fp32 values: packed code words plus the
// group's scale and zero-point (identical in all lanes of the group).
//
// Packing, fast path (|z| < 2048 in every lane of the wavefront): with
// t = rint(x*inv) the code is q = clamp(t + z, 0, qmax).  t >= rint(mn*inv) = -z
// because x >= mn and both the product and rint are monotone, so the lower clamp
// never acts, and since t, z and qmax are small integers the upper clamp can be
// applied to t: q = min(t, qmax - z) + z exactly; it is skipped altogether when
// rint(mx*inv), the largest t of the group, does not exceed qmax - z anywhere in
// the wavefront.  The codes are then rounded and merged as pack_codes describes.
// Otherwise each code is formed literally as in Eq. 2.
// `mx` is the group's maximum (the largest t of the group decides whether the
// upper clamp can act at all); inv and zf come from group_params.
template <int BITS, int EPL>
__device__ __forceinline__ void pack_lane(const float (&v)[EPL], float inv, float zf, float mx,
                                          u32 (&word)[EPL * BITS / 32])
{
    constexpr float qmax = (float)((1 << BITS) - 1);
    // strictly below 2048: a zero-point that was rounded to binary16 afterwards (compact metadata) equals the
    // one Eq. 1 gave only then (2049 rounds to 2048, and the minimum's code then needs the lower clamp)
    const bool pack_fast = __builtin_amdgcn_ballot_w64(!(fabsf(zf) < 2048.0f)) == 0;
    if (pack_fast) {
        const float tmax = qmax - zf;
        const bool need_cap = __builtin_amdgcn_ballot_w64(rintf(mx * inv) > tmax) != 0;
        if (need_cap)
            pack_codes<BITS, EPL, true>(v, inv, zf, tmax, word);
        else
            pack_codes<BITS, EPL, false>(v, inv, zf, tmax, word);
    } else {
        constexpr int per_word = 32 / BITS;
#pragma unroll
        for (int w = 0; w < EPL / per_word; ++w) {
            u32 acc = 0;
#pragma unroll
            for (int i = 0; i < per_word; ++i)
                acc |= encode<BITS>(v[per_word * w + i], inv, zf) << (BITS * i);
            word[w] = acc;
        }
    }
}

template <int EPL>
__device__ __forceinline__ void lane_minmax(const float (&v)[EPL], float &mn, float &mx)
{
    // three-input steps throughout (v_min3_f32 / v_max3_f32 take their inputs as they are; the two-input
    // forms would first be given a canonicalizing instruction per input by the compiler)
    static_assert(EPL % 2 == 0 && EPL >= 4, "three, then pairs, then the last one");
    mn = fminf(fminf(v[0], v[1]), v[2]);
    mx = fmaxf(fmaxf(v[0], v[1]), v[2]);
#pragma unroll
    for (int i = 3; i + 1 < EPL; i += 2) {
        mn = fminf(fminf(mn, v[i]), v[i + 1]);
        mx = fmaxf(fmaxf(mx, v[i]), v[i + 1]);
    }
    mn = fminf(mn, v[EPL - 1]);
    mx = fmaxf(mx, v[EPL - 1]);
}

template <int BITS, int EPL, int LPG, bool HM = false>
__device__ __forceinline__ void quantize_lane(const float (&v)[EPL], int lpg_rt,
                                              u32 (&word)[EPL * BITS / 32], float &s, float &zf)
{
    float mn, mx;
    lane_minmax(v, mn, mx);
    group_minmax<LPG>(mn, mx, lpg_rt);
    float inv;
    group_params<BITS, HM>(mn, mx, s, inv, zf);
    pack_lane<BITS, EPL>(v, inv, zf, mx, word);
}

// min / max across the `n_waves` (2 or 4, aligned) wavefronts of a workgroup
// that share one group; mn / mx are already reduced over each wavefront.  Every
// wavefront of the workgroup must call it (it contains a barrier).
__device__ __forceinline__ void cross_wave_minmax(float &mn, float &mx, float (*slot)[2], u32 wave,
                                                  u32 lane, u32 n_waves)
{
    if (lane == 0) {
        slot[wave][0] = mn;
        slot[wave][1] = mx;
    }
    __syncthreads();
    const u32 w0 = wave & ~(n_waves - 1u);
    for (u32 k = 0; k < n_waves; ++k) {
        mn = fminf(mn, slot[w0 + k][0]);
        mx = fmaxf(mx, slot[w0 + k][1]);
    }
}

// quantize_lane for a run-time group width of 16 ... 256 lanes (up to the whole workgroup)
template <int BITS, int EPL, bool HM = false>
__device__ __forceinline__ void quantize_lane_any(const float (&v)[EPL], int lpg, float (*slot)[2],
                                                  u32 wave, u32 lane,
                                                  u32 (&word)[EPL * BITS / 32], float &s, float &zf)
{
    float mn, mx;
    lane_minmax(v, mn, mx);
    group_minmax<0>(mn, mx, lpg);
    if (lpg > 64) cross_wave_minmax(mn, mx, slot, wave, lane, (u32)lpg >> 6);
    float inv;
    group_params<BITS, HM>(mn, mx, s, inv, zf);
    pack_lane<BITS, EPL>(v, inv, zf, mx, word);
}

struct ZeroConst {
    h2 c1024;   // (1024 + z, 1024 + z)
    h2 c64;     // (64 + z, 64 + z)
};

// ---------------------------------------------------------------------------
// Symmetric variant (paper Appendix, Eq. 3-4): s = max|X| / (2^(n-1) - 1),
// q = clamp(rint(X * (1/s)), -2^(n-1), 2^(n-1) - 1), signed codes stored in two's
// complement, no zero-point.
// ---------------------------------------------------------------------------
template <int LPG>
__device__ __forceinline__ float group_max(float m, int lpg_rt)
{
    const int lpg = LPG > 0 ? LPG : lpg_rt;
    if (lpg >= 2) m = dpp_max<kDppQuadXor1>(m);
    if (lpg >= 4) m = dpp_max<kDppQuadXor2>(m);
    if (lpg >= 8) m = dpp_max<kDppRowHalfMirror>(m);
    if (lpg >= 16) m = dpp_max<kDppRowMirror>(m);
    if (lpg >= 32) m = halves_or_wave<false>(m, lpg, threadIdx.x & 63u);
    return m;
}

// Eq. 3 (scale = max|X| / QM) with the same exhaustively checked division
// sequences as group_params: r/7, r/127 and r/448 match the IEEE quotient for
// every positive fp32 whose quotient is at least FLT_MIN, and smaller quotients
// are replaced by 1 on both sides.
template <int QM>
__device__ __forceinline__ void group_params_absmax(float amax, float &s, float &inv)
{
    constexpr float qm = (float)QM;
    constexpr float c = 1.0f / qm;
    const float q0 = amax * c;
    const float e = fmaf(-qm, q0, amax);
    s = fmaf(e, c, q0);                    // == amax / qm
    if (!(s >= FLT_MIN)) s = 1.0f;         // all-zero (or vanishing) group
    if (__builtin_amdgcn_ballot_w64(!(s <= 0x1p100f)) == 0) {
        const float y0 = __builtin_amdgcn_rcpf(s);
        const float e1 = fmaf(-s, y0, 1.0f);
        inv = fmaf(e1, y0, y0);            // == 1 / s
    } else {
        inv = 1.0f / s;
    }
}

template <int BITS>
__device__ __forceinline__ void group_params_sym(float amax, float &s, float &inv)
{
    group_params_absmax<(1 << (BITS - 1)) - 1>(amax, s, inv);
}

// Symmetric FinegrainedQuantize of the lane's EPL values.  |x| <= amax makes
// |x*inv| <= amax*inv = qm*(1 + O(2^-22)), so |rint(x*inv)| <= qm and neither
// clamp of Eq. 4 can act.  Digits are rounded and merged as in the asymmetric
// path (pack_codes) with a bias of 2^(n-1) per digit, and the bias is removed
// again by flipping each digit's top bit (offset binary -> two's complement).
template <int BITS, int EPL>
__device__ __forceinline__ void pack_lane_sym(const float (&v)[EPL], float inv, u32 (&word)[EPL * BITS / 32])
{
    // as pack_codes with the constant "zero-point" 2^(n-1): offset-binary digits t + 2^(n-1) in [1, 2^n - 1]
    constexpr float kMagic = 12582912.0f;
    constexpr u32 kMagicBits = 0x4B400000u;
    constexpr int per_word = 32 / BITS;
    constexpr u32 kOnes = BITS == 4 ? 0x11111111u : 0x01010101u;
    constexpr u32 kTop = BITS == 4 ? 0x88888888u : 0x80808080u;           // 2^(n-1) on every digit
    constexpr u32 fix = kTop - kMagicBits * kOnes;
#pragma unroll
    for (int w = 0; w < EPL / per_word; ++w) {
        u32 h = 0;
#pragma unroll
        for (int i = per_word - 1; i >= 0; --i) {
            const float r = v[per_word * w + i] * inv;
            const float u = r + kMagic;
            h = (h << BITS) + __builtin_bit_cast(u32, u);
        }
        word[w] = (h + fix) ^ kTop;
    }
}

template <int EPL>
__device__ __forceinline__ float lane_absmax(const float (&v)[EPL])
{
    float amax = fabsf(v[0]);
#pragma unroll
    for (int i = 1; i < EPL; ++i) amax = fmaxf(amax, fabsf(v[i]));
    return amax;
}

template <int BITS, int EPL, int LPG>
__device__ __forceinline__ void quantize_lane_sym(const float (&v)[EPL], int lpg_rt,
                                                  u32 (&word)[EPL * BITS / 32], float &s)
{
    const float amax = group_max<LPG>(lane_absmax(v), lpg_rt);
    float inv;
    group_params_sym<BITS>(amax, s, inv);
    pack_lane_sym<BITS, EPL>(v, inv, word);
}

template <int BITS, int EPL>
__device__ __forceinline__ void quantize_lane_sym_any(const float (&v)[EPL], int lpg, float (*slot)[2],
                                                      u32 wave, u32 lane,
                                                      u32 (&word)[EPL * BITS / 32], float &s)
{
    float amax = group_max<0>(lane_absmax(v), lpg);
    if (lpg > 64) {
        float lo = -amax;
        cross_wave_minmax(lo, amax, slot, wave, lane, (u32)lpg >> 6);
    }
    float inv;
    group_params_sym<BITS>(amax, s, inv);
    pack_lane_sym<BITS, EPL>(v, inv, word);
}

// ---------------------------------------------------------------------------
// FP8 variant (the paper's FP8_Sym rows): one OCP E4M3 byte per element,
// s = max|X| / 448, q = E4M3(X * (1/s)) to nearest-even, x^ = value(q) * s.
// gfx950's v_cvt_pk_fp8_f32 / v_cvt_pk_f32_fp8 implement exactly this format
// (round to nearest even, subnormals, signed zero; checked against a bitwise
// reference for every fp32 pattern up to |x| = 464, beyond which the hardware
// returns NaN instead of saturating).  |X * (1/s)| never exceeds
// 448 * (1 + 2^-22), which rounds to 448, so no clamp is needed.
// ---------------------------------------------------------------------------
typedef float f32x2 __attribute__((ext_vector_type(2)));

template <int EPL>
__device__ __forceinline__ void pack_lane_fp8(const float (&v)[EPL], float inv, u32 (&word)[EPL / 4])
{
#pragma unroll
    for (int w = 0; w < EPL / 4; ++w) {
        int a = __builtin_amdgcn_cvt_pk_fp8_f32(v[4 * w] * inv, v[4 * w + 1] * inv, 0, false);
        a = __builtin_amdgcn_cvt_pk_fp8_f32(v[4 * w + 2] * inv, v[4 * w + 3] * inv, a, true);
        word[w] = (u32)a;
    }
}

template <int EPL, int LPG>
__device__ __forceinline__ void quantize_lane_fp8(const float (&v)[EPL], int lpg_rt, u32 (&word)[EPL / 4],
                                                  float &s)
{
    const float amax = group_max<LPG>(lane_absmax(v), lpg_rt);
    float inv;
    group_params_absmax<448>(amax, s, inv);
    pack_lane_fp8<EPL>(v, inv, word);
}

template <int EPL>
__device__ __forceinline__ void quantize_lane_fp8_any(const float (&v)[EPL], int lpg, float (*slot)[2],
                                                      u32 wave, u32 lane, u32 (&word)[EPL / 4], float &s)
{
    float amax = group_max<0>(lane_absmax(v), lpg);
    if (lpg > 64) {
        float lo = -amax;
        cross_wave_minmax(lo, amax, slot, wave, lane, (u32)lpg >> 6);
    }
    float inv;
    group_params_absmax<448>(amax, s, inv);
    pack_lane_fp8<EPL>(v, inv, word);
}

// d[e] = value of the e-th E4M3 byte of the lane's 128 bits
__device__ __forceinline__ void decode_fp8(const u32 (&w)[4], float (&d)[16])
{
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const f32x2 lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[k], false);
        const f32x2 hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[k], true);
        d[4 * k + 0] = lo.x;
        d[4 * k + 1] = lo.y;
        d[4 * k + 2] = hi.x;
        d[4 * k + 3] = hi.y;
    }
}

// acc[e] = fma(value(q_e), s, acc[e])
__device__ __forceinline__ void accumulate_fp8(const u32 (&w)[4], float s, float (&acc)[16])
{
    float d[16];
    decode_fp8(w, d);
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = fmaf(d[i], s, acc[i]);
}

// signed codes -> offset binary (q + 2^(n-1)) and the matching "zero-point"
template <int BITS>
__device__ __forceinline__ u32 to_offset_binary(u32 w)
{
    return w ^ (BITS == 4 ? 0x88888888u : 0x80808080u);
}

template <int BITS>
__device__ __forceinline__ ZeroConst sym_zero_const()
{
    constexpr float bias = (float)(1 << (BITS - 1));
    ZeroConst z;
    const _Float16 a = (_Float16)(1024.0f + bias), b = (_Float16)(64.0f + bias);
    z.c1024 = h2{a, a};
    z.c64 = h2{b, b};
    return z;
}

// Store the lane's code words.  `r` addresses the workgroup's tile of the code
// array.  8 or 16 bytes per lane go out directly (coalesced); 32 bytes per lane
// are first laid out in the wavefront's LDS scratch `img` (2 KB) as they will
// sit in memory and then written as two coalesced 1 KB pieces.
template <int OUT_BYTES>
__device__ __forceinline__ void store_codes(const u32 *word, rsrc_t r, u32 wave, u32 lane, uint8_t *img)
{
    const u32 wave_off = wave * (64 * OUT_BYTES);
    if constexpr (OUT_BYTES == 8) {
        __builtin_amdgcn_raw_buffer_store_b64(u32x2{word[0], word[1]}, r, wave_off + lane * 8, 0,
                                              kStreamStorePolicy);
    } else if constexpr (OUT_BYTES == 16) {
        __builtin_amdgcn_raw_buffer_store_b128(u32x4{word[0], word[1], word[2], word[3]}, r,
                                               wave_off + lane * 16, 0, kStreamStorePolicy);
    } else {
        static_assert(OUT_BYTES == 32, "8, 16 or 32 code bytes per lane");
        u32x4 *mine = reinterpret_cast<u32x4 *>(img + lane * 32);
        mine[0] = u32x4{word[0], word[1], word[2], word[3]};
        mine[1] = u32x4{word[4], word[5], word[6], word[7]};
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const u32x4 a = *reinterpret_cast<const u32x4 *>(img + k * 1024 + lane * 16);
            __builtin_amdgcn_raw_buffer_store_b128(a, r, wave_off + k * 1024 + lane * 16, 0, kStreamStorePolicy);
        }
    }
}

__device__ __forceinline__ void store_f32(rsrc_t r, u32 byte_off, float v)
{
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(u32, v), r, byte_off, 0, 0);
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
// General path: convert and subtract in fp32.
// ---------------------------------------------------------------------------
__device__ __forceinline__ bool zero_is_fast(float zf)
{
    return (zf == rintf(zf)) && (zf >= -1700.0f) && (zf <= 1000.0f);
}

// lanes of the wavefront whose zf fails zero_is_fast, as a mask (the comparisons write lane masks directly;
// going through a per-lane bool costs two more vector instructions per use)
__device__ __forceinline__ uint64_t zero_is_slow_mask(float zf)
{
    constexpr int kUne = 14, kUlt = 12, kUgt = 10;            // unordered-or: not equal, less, greater
    return __builtin_amdgcn_fcmpf(zf, rintf(zf), kUne) | __builtin_amdgcn_fcmpf(zf, -1700.0f, kUlt) |
           __builtin_amdgcn_fcmpf(zf, 1000.0f, kUgt);
}

// (half(1024 + z), half(64 + z)) packed in one word
__device__ __forceinline__ u32 pack_zero_const(float zf)
{
    h2 c;
    c.x = (_Float16)(1024.0f + zf);
    c.y = (_Float16)(64.0f + zf);
    return as_u32(c);
}

__device__ __forceinline__ ZeroConst unpack_zero_const(u32 packed)
{
    const h2 c = as_h2(packed);
    ZeroConst z;
    z.c1024 = h2{c.x, c.x};
    z.c64 = h2{c.y, c.y};
    return z;
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

// d[e] = q_e - z (as fp32) for the lane's 128 bits of codes
template <int BITS>
__device__ __forceinline__ void codes_minus_zero_fast(const u32 (&w)[4], const ZeroConst &c,
                                                      float (&d)[128 / BITS])
{
    if constexpr (BITS == 4) {
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
        for (int k = 0; k < 4; ++k) {
            h2 p[2];
            bytes_minus_zero(w[k], c, p);
            d[4 * k + 0] = (float)p[0].x;
            d[4 * k + 2] = (float)p[0].y;
            d[4 * k + 1] = (float)p[1].x;
            d[4 * k + 3] = (float)p[1].y;
        }
    }
}

// v[e] = (q_e - z) * s for the lane's 128 bits of codes.  The widening of the binary16 difference folds into a
// mixed-precision multiply-add with a zero addend: the differences are integers (never -0) and s is positive, so
// adding +0 changes neither a nonzero product nor the sign of a zero one.
template <int BITS>
__device__ __forceinline__ void scaled_differences_fast(const u32 (&w)[4], const ZeroConst &c, float s,
                                                        float (&v)[128 / BITS])
{
    if constexpr (BITS == 4) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            h2 p[4];
            nibbles_minus_zero(w[k], c, p);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                v[8 * k + i] = fmaf((float)p[i].x, s, 0.0f);
                v[8 * k + 4 + i] = fmaf((float)p[i].y, s, 0.0f);
            }
        }
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            h2 p[2];
            bytes_minus_zero(w[k], c, p);
            v[4 * k + 0] = fmaf((float)p[0].x, s, 0.0f);
            v[4 * k + 2] = fmaf((float)p[0].y, s, 0.0f);
            v[4 * k + 1] = fmaf((float)p[1].x, s, 0.0f);
            v[4 * k + 3] = fmaf((float)p[1].y, s, 0.0f);
        }
    }
}

template <int BITS>
__device__ __forceinline__ void codes_minus_zero_general(const u32 (&w)[4], float zf,
                                                         float (&d)[128 / BITS])
{
    constexpr int per_word = 32 / BITS;
    constexpr u32 mask = (1u << BITS) - 1u;
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int i = 0; i < per_word; ++i)
            d[per_word * k + i] = (float)((w[k] >> (BITS * i)) & mask) - zf;
}

// acc[e] = fma(q_e - z, s, acc[e]) for the lane's codes of one source.  The
// widening of the binary16 difference folds into the multiply-add.
template <int BITS>
__device__ __forceinline__ void accumulate_fast(const u32 (&w)[4], float s, const ZeroConst &c,
                                                float (&acc)[128 / BITS])
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
        for (int k = 0; k < 4; ++k) {
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
__device__ __forceinline__ void accumulate_general(const u32 (&w)[4], float s, float zf,
                                                   float (&acc)[128 / BITS])
{
    constexpr int per_word = 32 / BITS;
    constexpr u32 mask = (1u << BITS) - 1u;
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int i = 0; i < per_word; ++i) {
            const float d = (float)((w[k] >> (BITS * i)) & mask) - zf;
            acc[per_word * k + i] = fmaf(d, s, acc[per_word * k + i]);
        }
}

// ---------------------------------------------------------------------------
// Kernels.  One workgroup = 2 or 4 wavefronts; wavefronts never synchronize
// with each other (every LDS region is private to one wavefront) except for the
// one barrier of a group that spans several wavefronts.
// ---------------------------------------------------------------------------

// FinegrainedQuantize of binary16 input (Algorithm 1, first quantization).
// One tile of BT*EPL elements per workgroup.  The wavefront's 64*EPL*2 input
// bytes are fetched as coalesced 1 KB pieces straight into LDS (an image of
// global memory) and each lane then reads its EPL contiguous values from there.
// CODEC selects the quantizer (`zeros` is used by kAsym only; with kAsymH `scales`
// is the array of 32-bit metadata words).
template <int BITS, int LPG, int CODEC>
__global__ __launch_bounds__(quantize_block_threads(BITS, LPG)) void k_quantize(
    const uint16_t *__restrict__ x, int64_t n_elems, int lpg, int group_shift,
    uint8_t *__restrict__ codes, float *__restrict__ scales, float *__restrict__ zeros)
{
    constexpr int EPL = lane_elems(BITS);
    constexpr int kPieces = EPL * 2 / 16;                       // 1 KB pieces per wavefront
    constexpr int BT = quantize_block_threads(BITS, LPG);
    __shared__ __attribute__((aligned(16))) uint8_t img[BT / 64][kPieces * 1024];

    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const int64_t e_tile = (int64_t)blockIdx.x * (BT * EPL);
    const int64_t g_tile = e_tile >> group_shift;
    const int64_t n_groups = n_elems >> group_shift;
    const rsrc_t rx = make_rsrc(x + e_tile, (n_elems - e_tile) * 2);
    const rsrc_t rc = make_rsrc(codes + e_tile * BITS / 8, (n_elems - e_tile) * BITS / 8);
    const rsrc_t rs = make_rsrc(scales + g_tile, (n_groups - g_tile) * 4);
    const rsrc_t rz = make_rsrc(CODEC != kAsym ? scales + g_tile : zeros + g_tile, (n_groups - g_tile) * 4);

#pragma unroll
    for (int k = 0; k < kPieces; ++k)
        dma_piece(rx, wave * (kPieces * 1024) + k * 1024 + lane * 16, &img[wave][k * 1024]);
    wait_vmem_outstanding(0);

    float v[EPL];
    const u32x4 *mine = reinterpret_cast<const u32x4 *>(&img[wave][lane * (EPL * 2)]);
#pragma unroll
    for (int k = 0; k < kPieces; ++k) {
        const u32x4 a = mine[k];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const h2 p = as_h2(a[i]);
            v[8 * k + 2 * i] = (float)p.x;
            v[8 * k + 2 * i + 1] = (float)p.y;
        }
    }

    u32 word[EPL * BITS / 32];
    float s, zf = 0.0f;
    if constexpr (CODEC == kFp8)
        quantize_lane_fp8<EPL, LPG>(v, lpg, word, s);
    else if constexpr (CODEC == kSym)
        quantize_lane_sym<BITS, EPL, LPG>(v, lpg, word, s);
    else
        quantize_lane<BITS, EPL, LPG, CODEC == kAsymH>(v, lpg, word, s, zf);
    store_codes<16>(word, rc, wave, lane, nullptr);
    const int lpg_v = LPG > 0 ? LPG : lpg;
    if ((tid & (lpg_v - 1)) == 0) {
        const u32 gi = (tid * EPL) >> group_shift;
        store_f32(rs, gi * 4, CODEC == kAsymH ? __builtin_bit_cast(float, pack_meta(s, zf)) : s);
        if constexpr (CODEC == kAsym) store_f32(rz, gi * 4, zf);
    }
}

// Dequantize x NSRC, ReduceSum, FinegrainedQuantize (Algorithm 1, loop body
// between the two exchanges).  The fp32 sum lives in registers only.
//
// One tile of BT*EPL elements per workgroup (BT = fused_block_threads(LPG)), one wavefront tile per wavefront.
// Fan-in staging: at wavefront start every lane issues, for each of the NSRC
// sources, one 128-bit buffer load that the memory pipeline writes straight into
// the wavefront's LDS landing zone (1 KB per source), bypassing the vector
// registers.  All NSRC KB of a wavefront are in flight at once while its
// registers hold only the accumulators and the source being folded in, which
// keeps 8 wavefronts resident per SIMD.  Each source is read back with one
// ds_read_b128 per lane (conflict-free) as soon as its load has retired.
// The group scales / zero-points reach the lanes in one of two ways, chosen at
// compile time by the group width (see kEntryMeta below).
// HM = true: binary16 metadata; scales_in / scales_out are the arrays of 32-bit
// metadata words and the zeros arrays are not used.
// BT: threads per workgroup.
// WRAP: 0 in the library.  The benchmark aid instantiates WRAP > 0, which makes every workgroup work on tile
// (its tile % WRAP): the instruction stream of a full launch with its memory traffic confined to a few tiles that
// stay in the L2, i.e. the time the kernel's arithmetic takes when HBM is out of the picture.
template <int BITS_IN, int BITS_OUT, int NSRC, int LPG, bool HM = false, int BT = fused_block_threads(LPG),
          int WRAP = 0>
__global__ __launch_bounds__(BT) void k_dequant_reduce_requant(
    const uint8_t *__restrict__ codes_in, int64_t codes_stride,
    const float *__restrict__ scales_in, const float *__restrict__ zeros_in, int64_t meta_stride,
    int64_t n_elems, int group_shift,
    uint8_t *__restrict__ codes_out, float *__restrict__ scales_out, float *__restrict__ zeros_out)
{
    constexpr int EPL = lane_elems(BITS_IN);
    constexpr int kWaveElems = 64 * EPL;
    constexpr int kWaves = BT / 64;
    static_assert(BT == fused_block_threads(LPG), "unsupported workgroup size");
    constexpr int kTileElems = BT * EPL;
    constexpr int kOutBytes = EPL * BITS_OUT / 8;             // code bytes a lane writes: 8, 16 or 32
    static_assert(LPG >= 1 && LPG <= 256 && (LPG & (LPG - 1)) == 0, "lanes per group: a power of two up to 256");
    static_assert(NSRC >= 1 && NSRC - 1 <= kMaxCountedVmem, "landing-zone waits count the loads of the later sources");
    constexpr int gw = LPG >= 64 ? 1 : 64 / LPG;              // groups per wavefront tile
    constexpr int gw_shift = __builtin_ctz((unsigned)gw);
    constexpr int entries = NSRC * gw;
    constexpr bool kSpansWaves = LPG > 64;                    // a group takes more than one wavefront
    constexpr int K = (entries + 63) / 64;                    // table entries per lane
    struct MetaRec { float s; u32 z; };                       // z: packed halves (fast) or fp32 bits

    __shared__ __attribute__((aligned(16))) uint8_t landing[kWaves][NSRC][1024];
    __shared__ MetaRec meta[LPG >= 8 ? 1 : kWaves][LPG >= 8 ? 1 : entries];
    __shared__ float slot[kSpansWaves ? kWaves : 1][2];       // cross-wavefront min / max (wide groups)
    __shared__ __attribute__((aligned(16))) uint8_t out_img[kOutBytes == 32 ? kWaves : 1]
                                                            [kOutBytes == 32 ? 2048 : 16];

    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const int64_t n_groups = n_elems >> group_shift;

    u32 tile = xcd_tile<xcd_chunk(BT * 16)>((u32)((n_elems + kTileElems - 1) / kTileElems));
    if constexpr (WRAP > 0) tile %= (u32)WRAP;
    const int64_t e_tile = (int64_t)tile * kTileElems;
    const int64_t g_tile = e_tile >> group_shift;

    // Scales and zero-points of the sources: the NSRC x (groups of the wavefront tile) pairs are loaded one per
    // lane, checked and converted once, and handed to the lanes of each group.  Narrow groups (up to 4 lanes: 16 or
    // more groups per wavefront tile, possibly several entries per lane) go through an LDS table; wider groups
    // (at most 8 groups per tile, so at most 64 entries: one per lane) are handed over with ds_bpermute, which
    // needs no table and no address arithmetic (0.2-0.7 us per launch at the headline shape against every lane
    // loading and converting the pairs of its own group; the LDS table measured up to 14 % slower there).
    constexpr bool kEntryMeta = LPG >= 8;
    // the code load of source j, straight into its landing slot
    auto issue_source = [&](int j) {
        const rsrc_t rc = make_rsrc(codes_in + (int64_t)j * codes_stride + e_tile * BITS_IN / 8,
                                    (n_elems - e_tile) * BITS_IN / 8);
        dma_piece(rc, tid * 16, &landing[wave][j][0]);
    };
    bool all_fast;
    MetaRec mrec[kEntryMeta ? NSRC : 1];
    const MetaRec *my_meta = nullptr;
    if constexpr (kEntryMeta) {
        // one lane per (source, group of the wavefront tile): entry e = j * gw + g
        static_assert(entries <= 64, "one entry per lane");
        const u32 e = lane < (u32)entries ? lane : 0u;            // surplus lanes repeat entry 0
        int64_t gi = ((e_tile + (int64_t)wave * kWaveElems) >> group_shift) + (e & (u32)(gw - 1));
        gi = gi < n_groups ? gi : n_groups - 1;                   // ragged tail: stay inside the array
        const int64_t at = (int64_t)(e >> gw_shift) * meta_stride + gi;
        float es = scales_in[at], ez;
        if constexpr (!HM) ez = zeros_in[at];
        issue_order_fence();
#pragma unroll
        for (int j = 0; j < NSRC; ++j) issue_source(j);
        issue_order_fence();
        if constexpr (HM) unpack_meta(__builtin_bit_cast(u32, es), es, ez);
        all_fast = zero_is_slow_mask(ez) == 0;
        const u32 ezc = all_fast ? pack_zero_const(ez) : __builtin_bit_cast(u32, ez);
        const u32 mine = ((LPG >= 64 ? 0u : lane / (u32)LPG)) * 4u;   // byte index of entry (0, my group)
#pragma unroll
        for (int j = 0; j < NSRC; ++j) {
            const int from = (int)mine + j * gw * 4;
            mrec[j].s = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(from, __builtin_bit_cast(int, es)));
            mrec[j].z = (u32)__builtin_amdgcn_ds_bpermute(from, (int)ezc);
        }
    } else {
        // --- table loads (small, first: vector-memory results return in issue order).
        // entry idx = j * gw + g  <->  (source j, group g of the wavefront tile)
        const int64_t g_wave = (e_tile + (int64_t)wave * kWaveElems) >> group_shift;
        float ms[K], mz[K];
#pragma unroll
        for (int it = 0; it < K; ++it) {
            int idx = it * 64 + (int)lane;
            idx = idx < entries ? idx : 0;                        // surplus lanes re-read entry 0
            const int j = idx >> gw_shift, g = idx & (gw - 1);
            int64_t gi = g_wave + g;
            gi = gi < n_groups ? gi : n_groups - 1;               // ragged tail: stay inside the array
            const int64_t at = (int64_t)j * meta_stride + gi;
            ms[it] = scales_in[at];
            if constexpr (!HM) mz[it] = zeros_in[at];
        }
        issue_order_fence();

        // --- codes: straight into the landing zone
#pragma unroll
        for (int j = 0; j < NSRC; ++j) issue_source(j);
        issue_order_fence();

        // --- table: check, convert, publish
        if constexpr (HM) {
#pragma unroll
            for (int it = 0; it < K; ++it) unpack_meta(__builtin_bit_cast(u32, ms[it]), ms[it], mz[it]);
        }
        uint64_t slow = 0;
#pragma unroll
        for (int it = 0; it < K; ++it) slow |= zero_is_slow_mask(mz[it]);
        all_fast = slow == 0;
#pragma unroll
        for (int it = 0; it < K; ++it) {
            const int idx = it * 64 + (int)lane;
            if (idx < entries) {
                MetaRec r;
                r.s = ms[it];
                r.z = all_fast ? pack_zero_const(mz[it]) : __builtin_bit_cast(u32, mz[it]);
                meta[wave][idx] = r;
            }
        }
        my_meta = &meta[wave][lane / (u32)LPG];
    }

    float acc[EPL];
#pragma unroll
    for (int i = 0; i < EPL; ++i) acc[i] = 0.0f;
    // one pass over the sources; the fast / general choice is made once per
    // tile so that the accumulators never cross a control-flow merge
    auto fold_sources = [&](auto fast_tag) {
#pragma unroll
        for (int j = 0; j < NSRC; ++j) {
            // source j has landed once no more than the loads of the later
            // sources (issued after it) are outstanding
            wait_vmem_outstanding(NSRC - 1 - j);
            u32x4 a = lds_read_b128_issue(&landing[wave][0][lane * 16], j * 1024);
            MetaRec r;
            if constexpr (kEntryMeta)
                r = mrec[j];
            else
                r = my_meta[j * gw];
            lds_read_complete(a);
            const u32 w[4] = {a[0], a[1], a[2], a[3]};
            if constexpr (decltype(fast_tag)::value)
                accumulate_fast<BITS_IN>(w, r.s, unpack_zero_const(r.z), acc);
            else
                accumulate_general<BITS_IN>(w, r.s, __builtin_bit_cast(float, r.z), acc);
            pin_values(acc);          // source j is folded in before source j+1 is waited for
        }
    };
    if (all_fast)
        fold_sources(std::true_type{});
    else
        fold_sources(std::false_type{});

    // --- requantize the sums and store
    u32 word[EPL * BITS_OUT / 32];
    float s, zf;
    if constexpr (kSpansWaves)
        quantize_lane_any<BITS_OUT, EPL, HM>(acc, LPG, slot, wave, lane, word, s, zf);
    else
        quantize_lane<BITS_OUT, EPL, LPG, HM>(acc, LPG, word, s, zf);
    const rsrc_t rc = make_rsrc(codes_out + e_tile * BITS_OUT / 8, (n_elems - e_tile) * BITS_OUT / 8);
    const rsrc_t rs = make_rsrc(scales_out + g_tile, (n_groups - g_tile) * 4);
    const rsrc_t rz = make_rsrc(HM ? scales_out + g_tile : zeros_out + g_tile, (n_groups - g_tile) * 4);
    store_codes<kOutBytes>(word, rc, wave, lane, &out_img[kOutBytes == 32 ? wave : 0][0]);
    if ((tid & (LPG - 1)) == 0) {
        const u32 gi = (tid * EPL) >> group_shift;
        // One group per lane (32-element groups at 4 bit): a wavefront writes whole 256-byte runs of scales and of
        // zero-points, and those stream best marked non-temporal like the codes (headline shape, g = 32: 48.2 ->
        // 37.7 us).  Wider groups write 128 bytes or less per wavefront and array; there the default policy, which
        // lets the L2 merge the pieces of a line, is the faster one (non-temporal: +1.4 us at g = 128).
        constexpr int kMetaStorePolicy = LPG == 1 ? kStreamStorePolicy : 0;
        const u32 first = HM ? pack_meta(s, zf) : __builtin_bit_cast(u32, s);
        __builtin_amdgcn_raw_buffer_store_b32(first, rs, gi * 4, 0, kMetaStorePolicy);
        if constexpr (!HM) __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(u32, zf), rz, gi * 4, 0, kMetaStorePolicy);
    }
}

// Symmetric version of the fused kernel (Eq. 3-4 on both sides): same staging
// and tiling; the signed codes are flipped to offset binary with one XOR per
// word and then take the fast path above with the constant "zero-point"
// 2^(n-1), so there is nothing to check or tabulate: each lane reads its
// group's scale of every source directly.
// FP8 = true: the bytes are E4M3 numbers instead of signed integers (8 bit on both sides).
template <int BITS_IN, int BITS_OUT, int NSRC, int LPG, bool FP8 = false>
__global__ __launch_bounds__(fused_block_threads(LPG)) void k_dequant_reduce_requant_sym(
    const uint8_t *__restrict__ codes_in, int64_t codes_stride,
    const float *__restrict__ scales_in, int64_t meta_stride,
    int64_t n_elems, int group_shift,
    uint8_t *__restrict__ codes_out, float *__restrict__ scales_out)
{
    constexpr int EPL = lane_elems(BITS_IN);
    constexpr int BT = fused_block_threads(LPG), kWaves = BT / 64;
    constexpr int kTileElems = BT * EPL;
    constexpr int kOutBytes = EPL * BITS_OUT / 8;
    __shared__ __attribute__((aligned(16))) uint8_t landing[kWaves][NSRC][1024];
    __shared__ __attribute__((aligned(16))) uint8_t out_img[kOutBytes == 32 ? kWaves : 1]
                                                            [kOutBytes == 32 ? 2048 : 16];
    static_assert(LPG >= 1 && LPG <= 256 && (LPG & (LPG - 1)) == 0, "lanes per group: a power of two up to 256");
    static_assert(NSRC >= 1 && NSRC - 1 <= kMaxCountedVmem, "landing-zone waits count the loads of the later sources");
    constexpr bool kSpansWaves = LPG > 64;
    __shared__ float slot[kSpansWaves ? kWaves : 1][2];       // cross-wavefront maximum (wide groups)

    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const int64_t n_groups = n_elems >> group_shift;
    const u32 tile = xcd_tile<xcd_chunk(BT * 16)>((u32)((n_elems + kTileElems - 1) / kTileElems));
    const int64_t e_tile = (int64_t)tile * kTileElems;
    const int64_t g_tile = e_tile >> group_shift;
    const u32 gi = (tid * EPL) >> group_shift;

    int64_t g_lane = g_tile + gi;
    g_lane = g_lane < n_groups ? g_lane : n_groups - 1;       // ragged tail: stay inside the array
    float sc[NSRC];
#pragma unroll
    for (int j = 0; j < NSRC; ++j) sc[j] = scales_in[(int64_t)j * meta_stride + g_lane];
    issue_order_fence();
    auto issue_source = [&](int j) {
        const rsrc_t rc = make_rsrc(codes_in + (int64_t)j * codes_stride + e_tile * BITS_IN / 8,
                                    (n_elems - e_tile) * BITS_IN / 8);
        dma_piece(rc, tid * 16, &landing[wave][j][0]);
    };
#pragma unroll
    for (int j = 0; j < NSRC; ++j) issue_source(j);
    issue_order_fence();

    const ZeroConst zc = sym_zero_const<BITS_IN>();
    float acc[EPL];
#pragma unroll
    for (int i = 0; i < EPL; ++i) acc[i] = 0.0f;
#pragma unroll
    for (int j = 0; j < NSRC; ++j) {
        wait_vmem_outstanding(NSRC - 1 - j);
        u32x4 a = lds_read_b128_issue(&landing[wave][0][lane * 16], j * 1024);
        lds_read_complete(a);
        if constexpr (FP8) {
            const u32 w[4] = {a[0], a[1], a[2], a[3]};
            accumulate_fp8(w, sc[j], acc);
        } else {
            const u32 w[4] = {to_offset_binary<BITS_IN>(a[0]), to_offset_binary<BITS_IN>(a[1]),
                              to_offset_binary<BITS_IN>(a[2]), to_offset_binary<BITS_IN>(a[3])};
            accumulate_fast<BITS_IN>(w, sc[j], zc, acc);
        }
        pin_values(acc);
    }

    u32 word[EPL * BITS_OUT / 32];
    float s;
    if constexpr (FP8) {
        static_assert(!FP8 || (BITS_IN == 8 && BITS_OUT == 8), "E4M3 is an 8-bit code");
        if constexpr (kSpansWaves)
            quantize_lane_fp8_any<EPL>(acc, LPG, slot, wave, lane, word, s);
        else
            quantize_lane_fp8<EPL, LPG>(acc, LPG, word, s);
    } else if constexpr (kSpansWaves)
        quantize_lane_sym_any<BITS_OUT, EPL>(acc, LPG, slot, wave, lane, word, s);
    else
        quantize_lane_sym<BITS_OUT, EPL, LPG>(acc, LPG, word, s);
    const rsrc_t rc = make_rsrc(codes_out + e_tile * BITS_OUT / 8, (n_elems - e_tile) * BITS_OUT / 8);
    const rsrc_t rs = make_rsrc(scales_out + g_tile, (n_groups - g_tile) * 4);
    store_codes<kOutBytes>(word, rc, wave, lane, &out_img[kOutBytes == 32 ? wave : 0][0]);
    if ((tid & (LPG - 1)) == 0) store_f32(rs, gi * 4, s);
}

// Dequantize to binary16 (Algorithm 1, last step): y = half_rne((q - z) * s).
// With kAsymH `scales` is the array of 32-bit metadata words.
// One tile of 256*EPL elements per workgroup; the EPL halves of a lane are laid
// out in the wavefront's LDS image and leave as coalesced 1 KB pieces.
template <int BITS, int CODEC>
__global__ __launch_bounds__(kBlockThreads) void k_dequantize(
    const uint8_t *__restrict__ codes, const float *__restrict__ scales,
    const float *__restrict__ zeros, int64_t n_elems, int group_shift, uint16_t *__restrict__ y)
{
    constexpr int EPL = lane_elems(BITS);
    constexpr int kPieces = EPL * 2 / 16;
    __shared__ __attribute__((aligned(16))) uint8_t img[kBlockWaves][kPieces * 1024];

    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const int64_t e_tile = (int64_t)blockIdx.x * block_elems(BITS);
    const int64_t g_tile = e_tile >> group_shift;
    const int64_t n_groups = n_elems >> group_shift;
    const u32 gi = (tid * EPL) >> group_shift;
    const rsrc_t rc = make_rsrc(codes + e_tile * BITS / 8, (n_elems - e_tile) * BITS / 8);
    const rsrc_t rs = make_rsrc(scales + g_tile, (n_groups - g_tile) * 4);
    const rsrc_t rz = make_rsrc(CODEC != kAsym ? scales + g_tile : zeros + g_tile, (n_groups - g_tile) * 4);
    const rsrc_t ry = make_rsrc(y + e_tile, (n_elems - e_tile) * 2);

    const float s_raw = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, gi * 4, 0, 0));
    float s = s_raw;
    const u32x4 a = __builtin_amdgcn_raw_buffer_load_b128(rc, tid * 16, 0, kStreamLoadPolicy);

    float d[EPL];
    if constexpr (CODEC == kFp8) {
        const u32 w[4] = {a[0], a[1], a[2], a[3]};
        decode_fp8(w, d);
    } else if constexpr (CODEC == kSym) {
        const u32 w[4] = {to_offset_binary<BITS>(a[0]), to_offset_binary<BITS>(a[1]),
                          to_offset_binary<BITS>(a[2]), to_offset_binary<BITS>(a[3])};
        codes_minus_zero_fast<BITS>(w, sym_zero_const<BITS>(), d);
    } else {
        float zf;
        if constexpr (CODEC == kAsymH)
            unpack_meta(__builtin_bit_cast(u32, s_raw), s, zf);
        else
            zf = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rz, gi * 4, 0, 0));
        const u32 w[4] = {a[0], a[1], a[2], a[3]};
        const bool wave_fast = __builtin_amdgcn_ballot_w64(!zero_is_fast(zf)) == 0;
        if (wave_fast)
            codes_minus_zero_fast<BITS>(w, unpack_zero_const(pack_zero_const(zf)), d);
        else
            codes_minus_zero_general<BITS>(w, zf, d);
    }

    u32x4 *mine = reinterpret_cast<u32x4 *>(&img[wave][lane * (EPL * 2)]);
#pragma unroll
    for (int k = 0; k < kPieces; ++k) {
        u32x4 out;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            h2 p;
            p.x = (_Float16)(d[8 * k + 2 * i] * s);
            p.y = (_Float16)(d[8 * k + 2 * i + 1] * s);
            out[i] = as_u32(p);
        }
        mine[k] = out;
    }
#pragma unroll
    for (int k = 0; k < kPieces; ++k) {
        const u32x4 o = *reinterpret_cast<const u32x4 *>(&img[wave][k * 1024 + lane * 16]);
        __builtin_amdgcn_raw_buffer_store_b128(o, ry, wave * (kPieces * 1024) + k * 1024 + lane * 16, 0,
                                               kStreamStorePolicy);
    }
}

}  // namespace fc
