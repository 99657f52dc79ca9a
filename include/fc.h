/*
 * fc.h -- C ABI of the MI355X (gfx950) Flash Communication quantization path.
 *
 * The library implements, on ONE GPU, the arithmetic that Flash Communication
 * (arXiv 2412.04964) wraps around its two exchanges (Algorithm 1, Section 3.2.2):
 *
 *     FinegrainedQuantize  ->  [All2All]  ->  Dequantize x N, ReduceSum,
 *     FinegrainedQuantize  ->  [All-Gather]  ->  Dequantize
 *
 * The exchanges themselves are not part of this library: the N partial tensors
 * (or their quantized slices) are simply N slabs in this GPU's memory.
 *
 * Quantizer (Appendix "Quantization Fundamentals", Eq. 1-2, asymmetric; groups
 * of `group` consecutive elements along `hidden`, Section 3.2.1), in fp32 with
 * round-to-nearest-even.  Results are bit-identical to evaluating, for every
 * group, exactly these operations in this order:
 *     mn, mx   = min, max of the group
 *     s        = (mx - mn) / (2^bits - 1)          one IEEE divide
 *     if !(s >= FLT_MIN):  s = |mn| >= FLT_MIN ? |mn| : 1       (constant group)
 *     inv      = 1 / s                              one IEEE divide
 *     z        = 0 - rint(mn * inv)                 integer-valued, NOT clamped
 *     q        = clamp(rint(x * inv) + z, 0, 2^bits - 1)
 * Dequantize (the inverse of Eq. 2):   x^ = (q - z) * s      (fp32 sub, fp32 mul)
 * ReduceSum: acc = +0; for j = 0..N-1 in order: acc = fma(q_j - z_j, s_j, acc).
 *
 * Data layouts (all device memory, dense, row-major):
 *   x, y     IEEE binary16 [tokens, hidden]
 *   codes    bytes [tokens, hidden*bits/8].  8 bit: one code per byte.  4 bit:
 *            two codes per byte, element 2k in bits 0-3, element 2k+1 in bits 4-7.
 *   scales   float [tokens, hidden/group]
 *   zeros    float [tokens, hidden/group]   (the zero-points z above)
 *
 * Common rules for every entry point
 *   - All pointers are DEVICE pointers unless stated otherwise, owned by the
 *     caller, 16-byte aligned (base pointers; the per-source meta slabs at
 *     +j*meta_src_stride_elems only need float alignment).  Inputs are never written; outputs must not
 *     overlap inputs.  The library allocates nothing and keeps no state except
 *     the last HIP error code.
 *   - Work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL is
 *     the default stream).  No call synchronizes.  The device that is current
 *     on the calling thread must own the buffers and the stream.
 *   - bits in {4, 8};  group a power of two in [32, 16384] (group == hidden: one group per token);
 *     hidden % group == 0;  tokens >= 0 (0 is a no-op returning FC_OK);
 *     tokens*hidden <= 2^36;  1 <= n_src <= FC_MAX_SRC.
 *   - Inputs must be finite.  NaN / Inf inputs give unspecified codes.
 *   - Return value: FC_OK or a negative FC_ERR_* code.  Argument checks come
 *     first and make no HIP call, so they work on a host without a GPU.
 *     FC_ERR_HIP reports the status that the launch call itself returned (kept for
 *     fc_last_hip_error); the library never reads or clears the calling thread's
 *     HIP last-error state, so an error left there by other code is neither
 *     reported as ours nor consumed.
 */
#ifndef FC_H
#define FC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#if defined(__GNUC__)
#define FC_API __attribute__((visibility("default")))
#else
#define FC_API
#endif

#define FC_MAX_SRC 8

enum {
    FC_OK = 0,
    FC_ERR_NULL = -1,       /* a required pointer is NULL */
    FC_ERR_BITS = -2,       /* bit-width not 4 or 8 */
    FC_ERR_GROUP = -3,      /* unsupported group size, or hidden % group != 0 */
    FC_ERR_SHAPE = -4,      /* tokens < 0, hidden <= 0, too many elements, n_src out of range,
                               or a source stride smaller than one slab */
    FC_ERR_ALIGN = -5,      /* pointer or stride not 16-byte aligned */
    FC_ERR_WORKSPACE = -6,  /* workspace NULL or too small */
    FC_ERR_HIP = -7         /* kernel launch failed; see fc_last_hip_error() */
};

/*
 * FinegrainedQuantize of Algorithm 1 (first call), Eq. 1-2.
 *   x_f16   in   binary16 [tokens, hidden]
 *   codes   out  [tokens, hidden*bits/8] bytes
 *   scales  out  float [tokens, hidden/group]
 *   zeros   out  float [tokens, hidden/group]
 */
FC_API int fc_quantize(const void *x_f16, int64_t tokens, int64_t hidden, int group, int bits,
                       void *codes, float *scales, float *zeros, void *hip_stream);

/*
 * The body of Algorithm 1 between the two exchanges, fused: Dequantize each of
 * the n_src received slices with its own scale and zero-point, ReduceSum (fp32
 * FMA chain, source order), FinegrainedQuantize of the sum with bits_out.  The
 * fp32 sum never goes to memory.  bits_in = 4 with bits_out = 8 is the paper's
 * "INT6" setting (Section 3.2.3).
 *   codes_in   in  source j's codes start at (char*)codes_in + j*codes_src_stride_bytes,
 *                  each [tokens, hidden*bits_in/8]
 *   scales_in, zeros_in
 *              in  source j's arrays start at +j*meta_src_stride_elems floats,
 *                  each [tokens, hidden/group]
 *   codes_src_stride_bytes >= tokens*hidden*bits_in/8, multiple of 16;
 *   meta_src_stride_elems  >= tokens*hidden/group (both ignored when
 *   n_src == 1).
 *   codes_out, scales_out, zeros_out   out, as in fc_quantize with bits_out.
 */
FC_API int fc_dequant_reduce_requant(const void *codes_in, int64_t codes_src_stride_bytes,
                                     const float *scales_in, const float *zeros_in,
                                     int64_t meta_src_stride_elems,
                                     int n_src, int64_t tokens, int64_t hidden, int group,
                                     int bits_in, int bits_out,
                                     void *codes_out, float *scales_out, float *zeros_out,
                                     void *hip_stream);

/*
 * Dequantize of Algorithm 1 (last call): y = binary16_rne((q - z) * s).
 * Values beyond the binary16 range become infinities.
 */
FC_API int fc_dequantize(const void *codes, const float *scales, const float *zeros,
                         int64_t tokens, int64_t hidden, int group, int bits,
                         void *y_f16, void *hip_stream);

/*
 * Algorithm 1 end to end on one device with identity exchanges:
 * n_src x fc_quantize(bits_rs) into the workspace, fc_dequant_reduce_requant
 * (bits_rs -> bits_ag), fc_dequantize.  The volume is quantized and dequantized
 * exactly twice (Table 1, "QDQ Step").
 *   x_f16      in   binary16 [n_src, tokens, hidden]
 *   y_f16      out  binary16 [tokens, hidden]
 *   workspace  device scratch of at least fc_allreduce_sim_workspace_bytes(...)
 *              bytes, 16-byte aligned; contents on return are unspecified.
 * With groups of at most 1024 elements the call runs as ONE kernel that keeps both quantizations in
 * registers (the single fused kernel of Section 3.2.3, "Kernel Design", with identity exchanges): the
 * partials are read once and the result is written once, 2 n_src + 2 bytes per element.  It evaluates
 * the same operations in the same order, so the result is bit-identical to the three steps, and it
 * does not touch the workspace (which must still be passed).  Wider groups run as the three steps.
 */
FC_API int fc_allreduce_sim(const void *x_f16, int n_src, int64_t tokens, int64_t hidden,
                            int group, int bits_rs, int bits_ag, void *y_f16,
                            void *workspace, size_t workspace_bytes, void *hip_stream);

/* Bytes fc_allreduce_sim needs; 0 if the arguments are invalid. */
FC_API size_t fc_allreduce_sim_workspace_bytes(int n_src, int64_t tokens, int64_t hidden, int group,
                                               int bits_rs, int bits_ag);

/*
 * fc_allreduce_sim for callers that cannot allocate device memory or keep a workspace (code
 * under HIP graph capture, tight serving loops, harnesses that forbid allocation): always the
 * three steps, with the intermediate codes, scales and zero-points in a fixed array of
 * FC_STATIC_SCRATCH_BYTES that lives in the library's device image (one copy per GPU, held until
 * the process ends).  The call allocates and frees nothing.  Same arguments, results and errors
 * as fc_allreduce_sim, plus:
 *   - FC_ERR_WORKSPACE when fc_allreduce_sim_workspace_bytes(...) exceeds
 *     FC_STATIC_SCRATCH_BYTES (e.g. 8 partials of 128 x 8192 at 8 bit, group 128, need 9.6 MB;
 *     the prefill volumes do not fit and must use fc_allreduce_sim);
 *   - all calls on one GPU share that GPU's array: calls that may overlap in time on one GPU
 *     (different streams, different threads) race; serialize them;
 *   - the first call on a device looks up the array's address (hipGetSymbolAddress); make
 *     that call outside graph capture.
 */
#define FC_STATIC_SCRATCH_BYTES (32u << 20)

FC_API int fc_allreduce_sim_static(const void *x_f16, int n_src, int64_t tokens, int64_t hidden,
                                   int group, int bits_rs, int bits_ag, void *y_f16, void *hip_stream);

/*
 * Symmetric variant (Appendix "Quantization Fundamentals", Eq. 3-4; the paper's
 * INT8_Sym / INT4_Sym ablation rows).  Same layouts and rules as above except:
 * there is no zero-point array, and codes are SIGNED, stored in two's
 * complement (8 bit: one int8 per byte; 4 bit: two per byte, element 2k in bits
 * 0-3).  Results are bit-identical to evaluating, for every group,
 *     s   = max|x| / (2^(bits-1) - 1)           one IEEE divide
 *     if !(s >= FLT_MIN): s = 1                  (all-zero group)
 *     inv = 1 / s                                 one IEEE divide
 *     q   = clamp(rint(x * inv), -2^(bits-1), 2^(bits-1) - 1)
 * Dequantize: x^ = q * s.  ReduceSum: acc = +0; acc = fma(q_j, s_j, acc), j = 0..N-1.
 */
FC_API int fc_quantize_sym(const void *x_f16, int64_t tokens, int64_t hidden, int group, int bits,
                           void *codes, float *scales, void *hip_stream);

FC_API int fc_dequant_reduce_requant_sym(const void *codes_in, int64_t codes_src_stride_bytes,
                                         const float *scales_in, int64_t meta_src_stride_elems,
                                         int n_src, int64_t tokens, int64_t hidden, int group,
                                         int bits_in, int bits_out,
                                         void *codes_out, float *scales_out, void *hip_stream);

FC_API int fc_dequantize_sym(const void *codes, const float *scales,
                             int64_t tokens, int64_t hidden, int group, int bits,
                             void *y_f16, void *hip_stream);

/* Algorithm 1 end to end with the symmetric quantizer; workspace as for fc_allreduce_sim
   (fc_allreduce_sim_workspace_bytes gives a sufficient size). */
FC_API int fc_allreduce_sim_sym(const void *x_f16, int n_src, int64_t tokens, int64_t hidden,
                                int group, int bits_rs, int bits_ag, void *y_f16,
                                void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * FP8 variant (the FP8_Sym rows of the paper's precision table and rotation table;
 * format: Appendix "FP8 and FP4 Format").  Layouts and rules as for the 8-bit symmetric
 * variant, except that each code byte is one OCP FP8 E4M3 number (1 sign, 4 exponent
 * bits with bias 7, 3 fraction bits, subnormals, no infinities, largest value 448).
 * Results are bit-identical to evaluating, for every group,
 *     s   = max|x| / 448                         one IEEE divide
 *     if !(s >= FLT_MIN): s = 1                  (all-zero group)
 *     inv = 1 / s                                 one IEEE divide
 *     q   = E4M3(x * inv)     nearest, ties to the even fraction, sign kept (-0 is byte 0x80)
 * Dequantize: x^ = value(q) * s.  ReduceSum: acc = +0; acc = fma(value(q_j), s_j, acc).
 * Input bytes 0x7F / 0xFF (NaN) are outside the domain.
 */
FC_API int fc_quantize_fp8(const void *x_f16, int64_t tokens, int64_t hidden, int group,
                           void *codes, float *scales, void *hip_stream);

FC_API int fc_dequant_reduce_requant_fp8(const void *codes_in, int64_t codes_src_stride_bytes,
                                         const float *scales_in, int64_t meta_src_stride_elems,
                                         int n_src, int64_t tokens, int64_t hidden, int group,
                                         void *codes_out, float *scales_out, void *hip_stream);

FC_API int fc_dequantize_fp8(const void *codes, const float *scales,
                             int64_t tokens, int64_t hidden, int group, void *y_f16, void *hip_stream);

/* Algorithm 1 end to end with FP8 on both sides; workspace of
   fc_allreduce_sim_workspace_bytes(n_src, tokens, hidden, group, 8, 8) bytes suffices. */
FC_API int fc_allreduce_sim_fp8(const void *x_f16, int n_src, int64_t tokens, int64_t hidden, int group,
                                void *y_f16, void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Compact-metadata variant of the asymmetric quantizer (Eq. 1-2; the paper does not say
 * how a group's scale and zero-point are stored or sent): both are kept in binary16, one
 * 32-bit word per group, so a group carries 4 bytes of metadata instead of 8.
 *   meta   uint32 [tokens, hidden/group]; bits 0-15 the scale, bits 16-31 the zero-point
 * Other layouts and rules as for fc_quantize.  Results are bit-identical to evaluating, for
 * every group,
 *     s   as in fc_quantize (including the constant-group rule), then
 *     s   = binary16_rne(s) kept inside [2^-24, 65504]  (zero -> 2^-24, overflow -> 65504)
 *     inv = 1 / s                                 one IEEE divide, of the stored scale
 *     z   = 0 - rint(mn * inv), then binary16_rne(z) saturated at +-65504
 *                                                 (integers up to 2048 are unchanged)
 *     q   = clamp(rint(x * inv) + z, 0, 2^bits - 1)
 * Dequantize: x^ = (q - z) * s with the two stored numbers widened to fp32; ReduceSum as in
 * fc_dequant_reduce_requant.  Input words must hold a positive finite scale and a finite
 * zero-point.  meta_src_stride_elems counts 32-bit words.
 */
FC_API int fc_quantize_cmeta(const void *x_f16, int64_t tokens, int64_t hidden, int group, int bits,
                             void *codes, uint32_t *meta, void *hip_stream);

FC_API int fc_dequant_reduce_requant_cmeta(const void *codes_in, int64_t codes_src_stride_bytes,
                                           const uint32_t *meta_in, int64_t meta_src_stride_elems,
                                           int n_src, int64_t tokens, int64_t hidden, int group,
                                           int bits_in, int bits_out,
                                           void *codes_out, uint32_t *meta_out, void *hip_stream);

FC_API int fc_dequantize_cmeta(const void *codes, const uint32_t *meta,
                               int64_t tokens, int64_t hidden, int group, int bits,
                               void *y_f16, void *hip_stream);

/* Algorithm 1 end to end with binary16 metadata; workspace as for fc_allreduce_sim
   (fc_allreduce_sim_workspace_bytes gives a sufficient size). */
FC_API int fc_allreduce_sim_cmeta(const void *x_f16, int n_src, int64_t tokens, int64_t hidden,
                                  int group, int bits_rs, int bits_ag, void *y_f16,
                                  void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Rotation variant (paper Section 4, "Naive vs. Rotation-based Quantization": the Hadamard
 * transform of QuaRot around the quantized all-reduce).  Every partial is rotated before
 * the first quantization; the rotation is linear, so the unchanged
 * fc_dequant_reduce_requant* step sums rotated partials; the inverse rotation follows the
 * last Dequantize.  `quantizer` selects the code (FC_QUANTIZER_*; FP8 needs bits == 8;
 * zeros may be NULL unless FC_QUANTIZER_ASYM).  The transform runs over every aligned block of
 * B elements of a token's row, B the largest power of two that divides hidden: the whole row when
 * hidden is a power of two, five blocks of 1024 for hidden 5120 (the rotation table's LLaMA-2-13B
 * row; the paper names no transform for such a length).  B must be 1024, 2048, 4096 or 8192
 * (FC_ERR_SHAPE otherwise); every group, a power of two dividing hidden, lies inside one block.
 * Other rules as above.  Results are bit-identical to:
 *     r = WHT_B(x) * 2^-ceil(n/2),  n = log2(B)          (fc_quantize_rot, then the quantizer on r in fp32)
 *     y = binary16(WHT_B(x^) * 2^-floor(n/2))            (fc_dequantize_rot on the dequantized fp32 x^)
 * where WHT_B applies, to each block, the natural-order Walsh-Hadamard transform evaluated in
 * fp32 as butterfly stages (a, b) -> (a + b, a - b) with spans 1, 2, 4, ..., B/2 in that order.
 */
#define FC_QUANTIZER_ASYM 0   /* Eq. 1-2 */
#define FC_QUANTIZER_SYM 1    /* Eq. 3-4 */
#define FC_QUANTIZER_FP8 2    /* E4M3 bytes */

FC_API int fc_quantize_rot(const void *x_f16, int64_t tokens, int64_t hidden, int group, int bits,
                           int quantizer, void *codes, float *scales, float *zeros, void *hip_stream);

FC_API int fc_dequantize_rot(const void *codes, const float *scales, const float *zeros,
                             int64_t tokens, int64_t hidden, int group, int bits, int quantizer,
                             void *y_f16, void *hip_stream);

/* Algorithm 1 with the rotation around it; workspace as for fc_allreduce_sim. */
FC_API int fc_allreduce_sim_rot(const void *x_f16, int n_src, int64_t tokens, int64_t hidden,
                                int group, int bits_rs, int bits_ag, int quantizer, void *y_f16,
                                void *workspace, size_t workspace_bytes, void *hip_stream);

/* Static, NUL-terminated description of an FC_* code.  Host pointer, never NULL. */
FC_API const char *fc_strerror(int code);

/* Raw hipError_t of the most recent failed launch on this thread (0 if none). */
FC_API int fc_last_hip_error(void);

/* major*10000 + minor*100 + patch */
FC_API int fc_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FC_H */
