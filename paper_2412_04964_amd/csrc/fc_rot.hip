// fc_rot.hip -- Hadamard rotation fused into the first quantization and the
// last dequantization of the all-reduce (paper Section 4, rotation-based
// quantization: the transform QuaRot applies before quantizing activations).
//
// Arithmetic contract (must match include/fc.h): the natural-order
// Walsh-Hadamard transform over every aligned block of B = 2^n elements of a
// token's row, B the largest power of two dividing hidden (the whole row when
// hidden is a power of two; five blocks of 1024 for hidden 5120), evaluated in
// fp32 as n butterfly stages with spans 1, 2, 4, ... in that order, each
// butterfly (a, b) -> (a + b, a - b); forward scaling 2^-ceil(n/2), inverse
// scaling 2^-floor(n/2).  A butterfly's result does not depend on which thread
// computes it, so any assignment of butterflies to threads that keeps the stage
// order is bit-identical.
//
// Blocks and quantization groups never cross block boundaries, so the tensor is
// handled as a flat sequence of chunks of 2^LOGH elements (LOGH = LB = n, except
// that 1024-element blocks go two to a chunk of 2048 and skip its last stage).
// One workgroup owns one chunk (2048, 4096 or 8192 elements) and keeps it
// in registers, R = 16 or 32 values per thread.  The stages over the bits of
// the index that live inside a thread run in registers; then the row goes to
// LDS and each further phase gives every thread the R values that differ in
// the next (up to) log2(R) index bits, with a barrier between phases.  The row
// is padded by 16 bytes per lane segment so that both the contiguous 128-bit
// accesses of the first / last step and the strided 32-bit accesses of the
// middle phases spread over the LDS banks.  The quantizer that follows (or the
// dequantizer that precedes) is the same device code as in the plain kernels.
#include "fc_device.hpp"
#include "fc_launch.hpp"

namespace fc {

constexpr int ilog2(int v) { return v <= 1 ? 0 : 1 + ilog2(v / 2); }

// Butterfly stages S0 ... NB-1 over the low NB bits of the register index, spans 2^S0, 2^(S0+1), ...
template <int R, int NB, int S0 = 0>
__device__ __forceinline__ void butterflies(float (&x)[R])
{
#pragma unroll
    for (int s = S0; s < NB; ++s)
#pragma unroll
        for (int q = 0; q < R; ++q)
            if (!(q & (1 << s))) {
                const float a = x[q], b = x[q | (1 << s)];
                x[q] = a + b;
                x[q | (1 << s)] = a - b;
            }
}

// First stage (span 1) on a pair of binary16 inputs held in one word: (lo + hi, lo - hi) in fp32.  Widening a
// binary16 number is exact, so a mixed-precision multiply-add lo * 1 +- hi rounds the same real sum once, as the
// conversion followed by an fp32 add does: one instruction per output instead of a conversion and an add.
__device__ __forceinline__ void first_stage(u32 pair, float &sum, float &diff)
{
    asm("v_fma_mix_f32 %0, %1, 1.0, %1 op_sel:[0,0,1] op_sel_hi:[1,0,1]" : "=v"(sum) : "v"(pair));
    asm("v_fma_mix_f32 %0, %1, 1.0, -%1 op_sel:[0,0,1] op_sel_hi:[1,0,1]" : "=v"(diff) : "v"(pair));
}

// word position of element e in the padded LDS row: 4 extra words per lane segment of 2^LE elements
template <int LE>
__device__ __forceinline__ constexpr u32 padded(u32 e)
{
    return e + 4u * (e >> LE);
}

// One LDS phase: stages over index bits [B0, B0 + NB).  Thread `tid` of T = 2^LT
// threads holds the R values whose index has register bits q_lo at [B0, B0+NB)
// and whose remaining bits are u = q_hi * T + tid; the position of the values is
// unchanged, so there is no hazard inside a phase.
template <int B0, int NB, int R, int LT, int LE>
__device__ __forceinline__ void lds_phase(float *row, u32 tid)
{
    const u32 et = ((tid >> B0) << (B0 + NB)) | (tid & ((1u << B0) - 1u));
    float *base = row + padded<LE>(et);
    auto at = [](int q) constexpr -> u32 {
        const u32 q_lo = (u32)q & ((1u << NB) - 1u), u = ((u32)q >> NB) << LT;
        const u32 e = ((u >> B0) << (B0 + NB)) | (q_lo << B0) | (u & ((1u << B0) - 1u));
        return e + 4u * (e >> LE);         // disjoint bit fields: padded(et | e) == padded(et) + padded(e)
    };
    float x[R];
#pragma unroll
    for (int q = 0; q < R; ++q) x[q] = base[at(q)];
    butterflies<R, NB>(x);
#pragma unroll
    for (int q = 0; q < R; ++q) base[at(q)] = x[q];
}

// Remaining stages for index bits [B0, END), R registers per thread, in phases of up to log2(R) bits.
template <int B0, int END, int R, int LT, int LE>
__device__ __forceinline__ void lds_phases(float *row, u32 tid)
{
    if constexpr (B0 < END) {
        constexpr int NB = (END - B0) < ilog2(R) ? (END - B0) : ilog2(R);
        lds_phase<B0, NB, R, LT, LE>(row, tid);
        __syncthreads();
        lds_phases<B0 + NB, END, R, LT, LE>(row, tid);
    }
}

// Shape of the workgroup for a code width and a row length.
template <int BITS, int LOGH>
struct RowShape {
    static constexpr int EPL = lane_elems(BITS);
    static constexpr int LE = ilog2(EPL);
    static constexpr int H = 1 << LOGH;
    static constexpr int LANES = H / EPL;
    static constexpr int T = LANES < kBlockThreads ? LANES : kBlockThreads;
    static constexpr int LT = ilog2(T);
    static constexpr int P = LANES / T;
    static constexpr int R = EPL * P;
    static constexpr int ROW_WORDS = H + 4 * (H / EPL);
    static_assert(T >= 64 && (P == 1 || P == 2), "rows of 2048 to 8192 elements");
};

// In-place transform of every aligned block of 2^LB elements of the chunk held as
// v[p][i] = element (p*T + tid)*EPL + i.  With S0 = 1 the caller has already applied the first stage (span 1).
template <int BITS, int LOGH, int LB, int S0, int NP, int NE>
__device__ __forceinline__ void hadamard_row(float (&v)[NP][NE], float *row, u32 tid)
{
    using S = RowShape<BITS, LOGH>;
    static_assert(NP == S::P && NE == S::EPL, "row held as v[P][EPL]");
    static_assert(LB <= LOGH && LB > S::LE, "blocks of at least two lanes, at most the chunk");
#pragma unroll
    for (int p = 0; p < S::P; ++p) butterflies<S::EPL, S::LE, S0>(v[p]);
#pragma unroll
    for (int p = 0; p < S::P; ++p) {
        u32x4 *dst = reinterpret_cast<u32x4 *>(row + padded<S::LE>((p * S::T + tid) * S::EPL));
#pragma unroll
        for (int k = 0; k < S::EPL / 4; ++k)
            dst[k] = u32x4{__builtin_bit_cast(u32, v[p][4 * k]), __builtin_bit_cast(u32, v[p][4 * k + 1]),
                           __builtin_bit_cast(u32, v[p][4 * k + 2]), __builtin_bit_cast(u32, v[p][4 * k + 3])};
    }
    __syncthreads();
    lds_phases<S::LE, LB, S::R, S::LT, S::LE>(row, tid);       // ends with a barrier
#pragma unroll
    for (int p = 0; p < S::P; ++p) {
        const u32x4 *src = reinterpret_cast<const u32x4 *>(row + padded<S::LE>((p * S::T + tid) * S::EPL));
#pragma unroll
        for (int k = 0; k < S::EPL / 4; ++k) {
            const u32x4 a = src[k];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const u32 w = a[i];        // (a bit_cast applied to the vector element itself reads element 0)
                v[p][4 * k + i] = __builtin_bit_cast(float, w);
            }
        }
    }
}

// Rotate one chunk block by block and quantize it (FinegrainedQuantize of Algorithm 1 on the rotated values).
// n_elems: elements of the whole tensor (a multiple of 2^LB; the last chunk may be a partial one when LB < LOGH:
// lanes beyond the end read zeros and have their stores dropped or skipped).
template <int BITS, int CODEC, int LOGH, int LB>
__global__ __launch_bounds__((RowShape<BITS, LOGH>::T)) void k_quantize_rot(
    const uint16_t *__restrict__ x, int64_t n_elems, int lpg, int group_shift, uint8_t *__restrict__ codes,
    float *__restrict__ scales, float *__restrict__ zeros)
{
    using S = RowShape<BITS, LOGH>;
    constexpr int EPL = S::EPL, T = S::T, P = S::P;
    constexpr int kPieces = EPL * 2 / 16;
    // the binary16 image of the row as it arrives and the padded fp32 row of the transform share their LDS (the
    // image is dead once every thread has its values in registers): 37 KB instead of 53 KB per workgroup at
    // hidden 8192, i.e. four resident workgroups per compute unit instead of three
    constexpr int kImgBytes = P * (T / 64) * kPieces * 1024;
    constexpr int kLdsBytes = kImgBytes > S::ROW_WORDS * 4 ? kImgBytes : S::ROW_WORDS * 4;
    __shared__ __attribute__((aligned(16))) uint8_t lds[kLdsBytes];
    __shared__ float slot[P][kBlockWaves][2];
    uint8_t (*img)[T / 64][kPieces * 1024] = reinterpret_cast<uint8_t (*)[T / 64][kPieces * 1024]>(lds);
    float *row = reinterpret_cast<float *>(lds);

    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const int64_t e0 = (int64_t)blockIdx.x << LOGH;
    const int64_t here = (n_elems - e0) < (int64_t)S::H ? (n_elems - e0) : (int64_t)S::H;      // elements of this chunk
    const rsrc_t rx = make_rsrc(x + e0, here * 2);
    const rsrc_t rc = make_rsrc(codes + e0 * BITS / 8, here * BITS / 8);

#pragma unroll
    for (int p = 0; p < P; ++p)
#pragma unroll
        for (int k = 0; k < kPieces; ++k)
            dma_piece(rx, (p * T * EPL + wave * 64 * EPL) * 2 + k * 1024 + lane * 16, &img[p][wave][k * 1024]);
    wait_vmem_outstanding(0);

    float v[P][EPL];
#pragma unroll
    for (int p = 0; p < P; ++p) {
        const u32x4 *mine = reinterpret_cast<const u32x4 *>(&img[p][wave][lane * (EPL * 2)]);
#pragma unroll
        for (int k = 0; k < kPieces; ++k) {
            const u32x4 a = mine[k];
#pragma unroll
            for (int i = 0; i < 4; ++i) first_stage(a[i], v[p][8 * k + 2 * i], v[p][8 * k + 2 * i + 1]);
        }
    }
    __syncthreads();                                   // the image is read; its LDS becomes the row

    hadamard_row<BITS, LOGH, LB, 1>(v, row, tid);
    // Forward scaling fwd = 2^-ceil(n/2), n = LB.  It is a power of two and nothing here is near the ends of
    // the fp32 range (the transformed values are multiples of 2^-24 below 2^30), so scaling commutes
    // with every rounding: instead of scaling all values, the group's min and max are scaled (which
    // gives the scale, reciprocal and zero-point of the scaled values exactly) and the codes are formed
    // from the unscaled values with the reciprocal times fwd, the same real product and hence the
    // same rounded one.
    constexpr float fwd = 1.0f / (float)(1 << ((LB + 1) / 2));

    // group min / max: inside the wavefront, then across the wavefronts of the sub-tile, then
    // (one group per row of two sub-tiles) across the sub-tiles
    float mn[P], mx[P];
#pragma unroll
    for (int p = 0; p < P; ++p) {
        lane_minmax(v[p], mn[p], mx[p]);
        group_minmax<0>(mn[p], mx[p], lpg);
        if (lpg > 64) cross_wave_minmax(mn[p], mx[p], slot[p], wave, lane, (u32)(lpg < T ? lpg : T) >> 6);
    }
    if (P == 2 && lpg > T) {
        mn[0] = mn[P - 1] = fminf(mn[0], mn[P - 1]);
        mx[0] = mx[P - 1] = fmaxf(mx[0], mx[P - 1]);
    }

    const int64_t g_row = ((int64_t)blockIdx.x << LOGH) >> group_shift;
#pragma unroll
    for (int p = 0; p < P; ++p) {
        float s, inv, zf = 0.0f;
        u32 word[4];
        const float mn_s = mn[p] * fwd, mx_s = mx[p] * fwd;
        if constexpr (CODEC == kFp8) {
            group_params_absmax<448>(fmaxf(fabsf(mn_s), fabsf(mx_s)), s, inv);
            pack_lane_fp8<EPL>(v[p], inv * fwd, word);
        } else if constexpr (CODEC == kSym) {
            group_params_sym<BITS>(fmaxf(fabsf(mn_s), fabsf(mx_s)), s, inv);
            pack_lane_sym<BITS, EPL>(v[p], inv * fwd, word);
        } else {
            group_params<BITS>(mn_s, mx_s, s, inv, zf);
            pack_lane<BITS, EPL>(v[p], inv * fwd, zf, mx[p], word);
        }
        __builtin_amdgcn_raw_buffer_store_b128(u32x4{word[0], word[1], word[2], word[3]}, rc,
                                               (p * T + tid) * 16, 0, kStreamStorePolicy);
        const u32 lane_in_row = p * T + tid;
        if ((lane_in_row & (u32)(lpg - 1)) == 0 && (int64_t)(lane_in_row * EPL) < here) {
            const int64_t gi = g_row + ((lane_in_row * EPL) >> group_shift);
            scales[gi] = s;
            if constexpr (CODEC == kAsym) zeros[gi] = zf;
        }
    }
}

// Dequantize one chunk, rotate it back block by block and round to binary16 (last step of Algorithm 1).
template <int BITS, int CODEC, int LOGH, int LB>
__global__ __launch_bounds__((RowShape<BITS, LOGH>::T)) void k_dequantize_rot(
    const uint8_t *__restrict__ codes, const float *__restrict__ scales, const float *__restrict__ zeros,
    int64_t n_elems, int group_shift, uint16_t *__restrict__ y)
{
    using S = RowShape<BITS, LOGH>;
    constexpr int EPL = S::EPL, T = S::T, P = S::P;
    constexpr int kPieces = EPL * 2 / 16;
    // the padded fp32 row and the binary16 image of the result share their LDS (see k_quantize_rot)
    constexpr int kImgBytes = (T / 64) * kPieces * 1024;
    constexpr int kLdsBytes = kImgBytes > S::ROW_WORDS * 4 ? kImgBytes : S::ROW_WORDS * 4;
    __shared__ __attribute__((aligned(16))) uint8_t lds[kLdsBytes];
    uint8_t (*img)[kPieces * 1024] = reinterpret_cast<uint8_t (*)[kPieces * 1024]>(lds);
    float *row = reinterpret_cast<float *>(lds);

    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const int64_t e0 = (int64_t)blockIdx.x << LOGH;
    const int64_t g_row = e0 >> group_shift;
    const int64_t here = (n_elems - e0) < (int64_t)S::H ? (n_elems - e0) : (int64_t)S::H;      // elements of this chunk
    const int64_t g_last = (n_elems >> group_shift) - 1;
    const rsrc_t rc = make_rsrc(codes + e0 * BITS / 8, here * BITS / 8);
    const rsrc_t ry = make_rsrc(y + e0, here * 2);

    float v[P][EPL];
#pragma unroll
    for (int p = 0; p < P; ++p) {
        const u32 lane_in_row = p * T + tid;
        int64_t gi = g_row + ((lane_in_row * EPL) >> group_shift);
        gi = gi < g_last ? gi : g_last;                    // lanes beyond a partial last chunk stay inside the arrays
        const float s = scales[gi];
        const u32x4 a = __builtin_amdgcn_raw_buffer_load_b128(rc, lane_in_row * 16, 0, kStreamLoadPolicy);
        if constexpr (CODEC == kFp8) {
            const u32 w[4] = {a[0], a[1], a[2], a[3]};
            float d[EPL];
            decode_fp8(w, d);
#pragma unroll
            for (int i = 0; i < EPL; ++i) v[p][i] = d[i] * s;
        } else if constexpr (CODEC == kSym) {
            const u32 w[4] = {to_offset_binary<BITS>(a[0]), to_offset_binary<BITS>(a[1]),
                              to_offset_binary<BITS>(a[2]), to_offset_binary<BITS>(a[3])};
            scaled_differences_fast<BITS>(w, sym_zero_const<BITS>(), s, v[p]);
        } else {
            const float zf = zeros[gi];
            const u32 w[4] = {a[0], a[1], a[2], a[3]};
            if (__builtin_amdgcn_ballot_w64(!zero_is_fast(zf)) == 0) {
                scaled_differences_fast<BITS>(w, unpack_zero_const(pack_zero_const(zf)), s, v[p]);
            } else {
                float d[EPL];
                codes_minus_zero_general<BITS>(w, zf, d);
#pragma unroll
                for (int i = 0; i < EPL; ++i) v[p][i] = d[i] * s;
            }
        }
    }

    hadamard_row<BITS, LOGH, LB, 0>(v, row, tid);
    __syncthreads();                                   // the row is read; its LDS becomes the output image
    constexpr float inv = 1.0f / (float)(1 << (LB / 2));               // 2^-floor(n/2), n = LB

#pragma unroll
    for (int p = 0; p < P; ++p) {
        u32x4 *mine = reinterpret_cast<u32x4 *>(&img[wave][lane * (EPL * 2)]);
#pragma unroll
        for (int k = 0; k < kPieces; ++k) {
            u32x4 out;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                h2 h;
                h.x = (_Float16)(v[p][8 * k + 2 * i] * inv);
                h.y = (_Float16)(v[p][8 * k + 2 * i + 1] * inv);
                out[i] = as_u32(h);
            }
            mine[k] = out;
        }
#pragma unroll
        for (int k = 0; k < kPieces; ++k) {
            const u32x4 o = *reinterpret_cast<const u32x4 *>(&img[wave][k * 1024 + lane * 16]);
            __builtin_amdgcn_raw_buffer_store_b128(o, ry, (p * T * EPL + wave * 64 * EPL) * 2 + k * 1024 + lane * 16,
                                                   0, kStreamStorePolicy);
        }
    }
}

// ---------------------------------------------------------------------------
// launchers: block = largest power of two dividing hidden, in {1024, 2048, 4096, 8192};
// group a power of two in [32, block]
// ---------------------------------------------------------------------------
namespace {

template <int BITS, int CODEC, int LOGH, int LB>
hipError_t quantize_rot_one(const uint16_t *x, int64_t n_elems, int group, uint8_t *c, float *scales,
                            float *zeros, hipStream_t stream)
{
    const unsigned grid = (unsigned)((n_elems + ((int64_t)1 << LOGH) - 1) >> LOGH);
    return launch_kernel(k_quantize_rot<BITS, CODEC, LOGH, LB>, dim3(grid), dim3(RowShape<BITS, LOGH>::T), stream, x,
                         n_elems, group / lane_elems(BITS), log2_int(group), c, scales, zeros);
}

template <int BITS, int CODEC>
hipError_t quantize_rot_h(int log_b, const uint16_t *x, int64_t n_elems, int group, uint8_t *c, float *scales,
                          float *zeros, hipStream_t stream)
{
    switch (log_b) {
    case 10: return quantize_rot_one<BITS, CODEC, 11, 10>(x, n_elems, group, c, scales, zeros, stream);
    case 11: return quantize_rot_one<BITS, CODEC, 11, 11>(x, n_elems, group, c, scales, zeros, stream);
    case 12: return quantize_rot_one<BITS, CODEC, 12, 12>(x, n_elems, group, c, scales, zeros, stream);
    case 13: return quantize_rot_one<BITS, CODEC, 13, 13>(x, n_elems, group, c, scales, zeros, stream);
    default: return hipErrorInvalidValue;
    }
}

template <int BITS, int CODEC, int LOGH, int LB>
hipError_t dequantize_rot_one(const uint8_t *c, const float *scales, const float *zeros, int64_t n_elems,
                              int group, uint16_t *y, hipStream_t stream)
{
    const unsigned grid = (unsigned)((n_elems + ((int64_t)1 << LOGH) - 1) >> LOGH);
    return launch_kernel(k_dequantize_rot<BITS, CODEC, LOGH, LB>, dim3(grid), dim3(RowShape<BITS, LOGH>::T), stream, c,
                         scales, zeros, n_elems, log2_int(group), y);
}

template <int BITS, int CODEC>
hipError_t dequantize_rot_h(int log_b, const uint8_t *c, const float *scales, const float *zeros,
                            int64_t n_elems, int group, uint16_t *y, hipStream_t stream)
{
    switch (log_b) {
    case 10: return dequantize_rot_one<BITS, CODEC, 11, 10>(c, scales, zeros, n_elems, group, y, stream);
    case 11: return dequantize_rot_one<BITS, CODEC, 11, 11>(c, scales, zeros, n_elems, group, y, stream);
    case 12: return dequantize_rot_one<BITS, CODEC, 12, 12>(c, scales, zeros, n_elems, group, y, stream);
    case 13: return dequantize_rot_one<BITS, CODEC, 13, 13>(c, scales, zeros, n_elems, group, y, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace

hipError_t launch_quantize_rot(int bits, int codec, const void *x_f16, int64_t tokens, int hidden, int group,
                               void *codes, float *scales, float *zeros, hipStream_t stream)
{
    const uint16_t *x = static_cast<const uint16_t *>(x_f16);
    uint8_t *c = static_cast<uint8_t *>(codes);
    const int lb = log2_int(rotation_block(hidden));
    const int64_t n = tokens * hidden;
    if (codec == CODEC_FP8)
        return bits == 8 ? quantize_rot_h<8, kFp8>(lb, x, n, group, c, scales, nullptr, stream)
                         : hipErrorInvalidValue;
    if (bits == 4)
        return codec == CODEC_ASYM ? quantize_rot_h<4, kAsym>(lb, x, n, group, c, scales, zeros, stream)
                                   : quantize_rot_h<4, kSym>(lb, x, n, group, c, scales, nullptr, stream);
    return codec == CODEC_ASYM ? quantize_rot_h<8, kAsym>(lb, x, n, group, c, scales, zeros, stream)
                               : quantize_rot_h<8, kSym>(lb, x, n, group, c, scales, nullptr, stream);
}

hipError_t launch_dequantize_rot(int bits, int codec, const void *codes, const float *scales, const float *zeros,
                                 int64_t tokens, int hidden, int group, void *y_f16, hipStream_t stream)
{
    const uint8_t *c = static_cast<const uint8_t *>(codes);
    uint16_t *y = static_cast<uint16_t *>(y_f16);
    const int lb = log2_int(rotation_block(hidden));
    const int64_t n = tokens * hidden;
    if (codec == CODEC_FP8)
        return bits == 8 ? dequantize_rot_h<8, kFp8>(lb, c, scales, nullptr, n, group, y, stream)
                         : hipErrorInvalidValue;
    if (bits == 4)
        return codec == CODEC_ASYM ? dequantize_rot_h<4, kAsym>(lb, c, scales, zeros, n, group, y, stream)
                                   : dequantize_rot_h<4, kSym>(lb, c, scales, nullptr, n, group, y, stream);
    return codec == CODEC_ASYM ? dequantize_rot_h<8, kAsym>(lb, c, scales, zeros, n, group, y, stream)
                               : dequantize_rot_h<8, kSym>(lb, c, scales, nullptr, n, group, y, stream);
}

}  // namespace fc
