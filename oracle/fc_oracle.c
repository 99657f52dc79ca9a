/*
 * fc_oracle.c -- plain CPU oracle for the Flash Communication quantization
 * arithmetic (arXiv 2412.04964).
 *
 * THIS FILE IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  It is a slow, scalar,
 * one-element-at-a-time statement of what the GPU library must compute and it
 * shares nothing with the HIP sources: no header, no helper, no table.  Only
 * tests, the smoke check and the benchmark's CPU-baseline leg may call it.
 *
 * What it follows in the paper
 *   - asymmetric group quantizer: Appendix "Quantization Fundamentals",
 *     Eq. 1 (scale, zero-point) and Eq. 2 (codes, clamp to [0, 2^n-1]);
 *   - two-step all-reduce: Algorithm 1 (FinegrainedQuantize -> exchange ->
 *     Dequantize each of the N slices -> ReduceSum -> FinegrainedQuantize ->
 *     exchange -> Dequantize), Section 3.2.2;
 *   - groups run along the hidden dimension of one token (Section 3.2.1,
 *     the block-size figure: 4096 = hidden down to 128);
 *   - mixed bit-widths ("INT6" = 4-bit before the reduce, 8-bit before the
 *     gather): Section 3.2.3, "INT6 Quantization".
 *
 * Readings taken where the paper is silent or garbled (every one of them is a
 * plain fp32 operation in the order written below, default rounding mode):
 *   R1  the rounding bracket of Eq. 1-2 is round-to-nearest, ties to even;
 *   R2  Dequantize, which the paper calls but never prints, is the inverse of
 *       Eq. 2:  x^ = (q - z) * s;
 *   R3  s and z are stored as fp32; z is integer-valued and is NOT clamped;
 *   R4  X/s is evaluated as X * (1/s) with one reciprocal per group, and the
 *       zero-point uses the same product, so the group minimum always gets
 *       code 0;
 *   R5  a group whose range is zero (or so small that s would be subnormal)
 *       takes s = |min| (1 if that is below FLT_MIN too): all codes are 0 and
 *       a constant group reconstructs exactly;
 *   R6  the N-way sum is an fp32 fused-multiply-add chain over the sources in
 *       index order, starting from +0;
 *   R7  Algorithm 1's Dequantize takes each slice's own scale (the symbol is
 *       dropped in the listing) and the sum has N terms;
 *   R8  INT4 codes are packed two per byte in linear order, element 2k in the
 *       low nibble and element 2k+1 in the high nibble.
 * Symmetric variant (Appendix, Eq. 3-4; the paper's INT8_Sym / INT4_Sym ablation
 * rows): the fc_ref_*_sym functions at the end of this file, with readings
 *   S1  rounding and the per-group reciprocal as R1 and R4;
 *   S2  s = max|X| / (2^(n-1) - 1) in fp32; a group whose s would be below
 *       FLT_MIN (in particular the all-zero group) takes s = 1, all codes 0;
 *   S3  codes are signed, clamped to [-2^(n-1), 2^(n-1)-1] as Eq. 4 says, and
 *       stored in two's complement in the same packing as R8;
 *   S4  Dequantize is x^ = q * s; the N-way sum is acc = fma(q_j, s_j, acc).
 * FP8 variant (the FP8_Sym rows of the precision table and of the rotation
 * table, "FP8 and FP4 Format" in the Appendix): the fc_ref_*_fp8 functions, with
 *   F1  the code is one OCP FP8 E4M3 number per byte (Micikevicius et al. 2022,
 *       which the paper cites): 1 sign, 4 exponent bits with bias 7, 3 fraction
 *       bits, subnormals of step 2^-9, no infinities, S.1111.111 is NaN, largest
 *       finite value 448;
 *   F2  per-group symmetric scale s = max|X| / 448 in fp32 (the paper prints
 *       no formula for FP8; this is Eq. 3 with the format's largest value in
 *       place of 2^(n-1) - 1); s below FLT_MIN -> s = 1 as in S2;
 *   F3  q = E4M3(X * (1/s)): round to nearest, ties to even fraction, sign kept
 *       (so a negative value that rounds to zero gives -0, byte 0x80);
 *       magnitudes beyond 448 saturate to 448 (cannot happen for a group's own
 *       values, as with the clamps of Eq. 4);
 *   F4  Dequantize is x^ = value(q) * s; the N-way sum is
 *       acc = fma(value(q_j), s_j, acc) from +0.
 * Rotation variant (Section 4, "Naive vs. Rotation-based Quantization": the
 * Hadamard transform of QuaRot applied around the quantized all-reduce; the paper
 * gives no formula): the fc_ref_*_rot functions, with
 *   H1  the transform is the Walsh-Hadamard transform in natural (Sylvester)
 *       order over the whole hidden dimension of one token, hidden a power of
 *       two; every partial is rotated before the first quantization, the sum of
 *       rotated partials is the rotated sum, and the inverse is applied once
 *       after the last Dequantize;
 *   H2  it is evaluated in fp32 as log2(hidden) butterfly stages with spans
 *       1, 2, 4, ..., hidden/2 in that order, each butterfly (a, b) -> (a+b, a-b);
 *   H3  the forward transform is scaled by 2^-ceil(n/2) and the inverse by
 *       2^-floor(n/2), n = log2(hidden): exact scalings whose product is 1/hidden
 *       (the orthonormal transform up to an exact power of two, to which the
 *       group quantizers are invariant);
 *   H4  the rotated values go into the quantizer in fp32 (no rounding to
 *       binary16 in between); the result is binary16(RNE) of the inverse transform
 *       of the dequantized fp32 values;
 *   H5  a hidden dimension that is not a power of two (the rotation table's
 *       LLaMA-2-13B row: 5120) is rotated block by block: the transform of H1-H3
 *       over every aligned run of B elements, B the largest power of two that
 *       divides hidden (5120 = 5 x 1024), i.e. the orthogonal matrix
 *       I (x) H_B.  A quantization group that is a power of two dividing hidden
 *       divides B, so it lies inside one block.  For a power of two B = hidden
 *       and nothing changes.
 * Compact metadata variant (the paper never says how a group's scale and
 * zero-point are stored or sent; this is the asymmetric quantizer of Eq. 1-2 with
 * both kept in binary16, 4 bytes per group instead of 8): the fc_ref_*_cmeta
 * functions, with R1, R2, R4-R8 unchanged and
 *   C1  the scale of Eq. 1 (after R5) is rounded to binary16, to nearest even,
 *       and kept inside the positive finite binary16 numbers: a result of zero
 *       becomes 2^-24 (the smallest subnormal), an overflow becomes 65504; from
 *       here on s is that binary16 number, so the reciprocal of R4, the
 *       zero-point and every code are computed from the scale that is stored;
 *   C2  the zero-point of Eq. 1, computed from that s, is rounded to binary16 the
 *       same way and saturates at +-65504; the codes of Eq. 2 use the rounded
 *       value.  Integers up to 2048 are exact in binary16, so nothing changes
 *       for a group whose range contains zero (0 <= z <= 2^n - 1 there);
 *   C3  Dequantize is x^ = (q - z) * s with the two stored binary16 numbers
 *       widened exactly to fp32; the N-way sum is R6;
 *   C4  one 32-bit word per group: bits 0-15 the scale, bits 16-31 the
 *       zero-point.
 * Domain: finite inputs.  NaN / Inf inputs: parity unpinned.
 *
 * Build: cc -O2 -std=c11 -ffp-contract=off -fno-fast-math -fPIC -shared
 *        (contraction must stay off: every product and sum below is rounded
 *        on its own, except the explicit fmaf of R6).
 */
#include <float.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define FC_REF_OK 0
#define FC_REF_BAD_ARG (-1)
#define FC_REF_NO_MEM (-2)

/* ------------------------------------------------------------------------ */
/* IEEE binary16 <-> binary32, written out on the bit fields (1 sign, 5      */
/* exponent bits with bias 15, 10 fraction bits: Appendix, "IEEE 754         */
/* standards for FP16").                                                     */
/* ------------------------------------------------------------------------ */

float fc_ref_half_to_float(uint16_t h)
{
    const int sign = (h >> 15) & 1;
    const int e = (h >> 10) & 0x1F;
    const int f = h & 0x3FF;
    double v;
    if (e == 0)
        v = ldexp((double)f, -24);               /* zero or subnormal: f * 2^-24 */
    else if (e == 31)
        v = f ? (double)NAN : (double)INFINITY;
    else
        v = ldexp((double)(1024 + f), e - 25);   /* (1 + f/1024) * 2^(e-15) */
    return (float)(sign ? -v : v);               /* every binary16 is exact in binary32 */
}

/* Round-to-nearest-even conversion; overflow goes to infinity. */
uint16_t fc_ref_float_to_half(float x)
{
    uint32_t u;
    memcpy(&u, &x, 4);
    const uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    if (isnan(x)) return (uint16_t)(sign | 0x7E00u);
    const double a = fabs((double)x);
    if (a == 0.0) return sign;
    if (isinf(x)) return (uint16_t)(sign | 0x7C00u);
    int e2;
    (void)frexp(a, &e2);                         /* a = m * 2^e2, m in [0.5, 1) */
    int e = e2 - 1;                              /* a in [2^e, 2^(e+1)) */
    if (e < -14) e = -14;                        /* subnormal range shares the 2^-24 grid */
    /* spacing of binary16 numbers around a is 2^(e-10); a / spacing is exact
       in double, nearbyint rounds half to even in the default mode */
    const double n = nearbyint(ldexp(a, 10 - e));
    uint32_t mant = (uint32_t)n;                 /* in [0, 2048] */
    int be = e + 15;                             /* biased exponent when mant >= 1024 */
    if (mant >= 2048u) { mant = 1024u; be += 1; }
    if (mant < 1024u) return (uint16_t)(sign | mant);           /* subnormal (or zero) */
    if (be >= 31) return (uint16_t)(sign | 0x7C00u);            /* overflow */
    return (uint16_t)(sign | ((uint32_t)be << 10) | (mant - 1024u));
}

/* ------------------------------------------------------------------------ */
/* FinegrainedQuantize of ONE group (Eq. 1-2 under R1, R3, R4, R5).          */
/* x: g fp32 values.  q: g codes, one per byte (not packed).                 */
/* ------------------------------------------------------------------------ */

void fc_ref_quantize_group_f32(const float *x, int g, int bits,
                               uint8_t *q, float *scale, float *zero)
{
    const float qmax = (float)((1 << bits) - 1);
    float mn = x[0], mx = x[0];
    for (int k = 1; k < g; ++k) {
        if (x[k] < mn) mn = x[k];
        if (x[k] > mx) mx = x[k];
    }
    const float r = mx - mn;
    float s = r / qmax;                          /* Eq. 1, scale */
    if (!(s >= FLT_MIN)) {                       /* R5: degenerate range */
        const float a = fabsf(mn);
        s = (a >= FLT_MIN) ? a : 1.0f;
    }
    const float inv = 1.0f / s;                  /* R4 */
    const float zf = 0.0f - rintf(mn * inv);     /* Eq. 1, zero-point; 0 - (-0) = +0 */
    for (int k = 0; k < g; ++k) {
        const float t = rintf(x[k] * inv);       /* Eq. 2: round(X / s) */
        float u = t + zf;                        /*        + z          */
        if (u < 0.0f) u = 0.0f;                  /*        clamp        */
        if (u > qmax) u = qmax;
        q[k] = (uint8_t)u;
    }
    *scale = s;
    *zero = zf;
}

static int check_shape(int64_t tokens, int64_t hidden, int group, int bits)
{
    if (tokens < 0 || hidden <= 0 || group <= 0) return 0;
    if (bits != 4 && bits != 8) return 0;
    if (hidden % group != 0) return 0;
    if (bits == 4 && (hidden % 2) != 0) return 0;
    return 1;
}

/* store one row of codes: one byte each (8 bit) or two per byte (R8) */
static void pack_row(const uint8_t *q, int64_t hidden, int bits, uint8_t *dst)
{
    if (bits == 8) {
        memcpy(dst, q, (size_t)hidden);
    } else {
        for (int64_t k = 0; k < hidden / 2; ++k)
            dst[k] = (uint8_t)(q[2 * k] | (q[2 * k + 1] << 4));
    }
}

static unsigned code_at(const uint8_t *row, int64_t h, int bits)
{
    if (bits == 8) return row[h];
    const uint8_t b = row[h / 2];
    return (h & 1) ? (unsigned)(b >> 4) : (unsigned)(b & 0x0F);
}

/* FinegrainedQuantize of an fp32 matrix [tokens, hidden], groups along hidden. */
int fc_ref_quantize_f32(const float *x, int64_t tokens, int64_t hidden, int group, int bits,
                        uint8_t *codes, float *scales, float *zeros)
{
    if (!check_shape(tokens, hidden, group, bits)) return FC_REF_BAD_ARG;
    if (tokens == 0) return FC_REF_OK;
    if (!x || !codes || !scales || !zeros) return FC_REF_BAD_ARG;
    const int64_t gpr = hidden / group;          /* groups per row */
    const int64_t row_bytes = hidden * bits / 8;
    uint8_t *q = (uint8_t *)malloc((size_t)hidden);
    if (!q) return FC_REF_NO_MEM;
    for (int64_t t = 0; t < tokens; ++t) {
        for (int64_t c = 0; c < gpr; ++c)
            fc_ref_quantize_group_f32(x + t * hidden + c * group, group, bits,
                                      q + c * group, &scales[t * gpr + c], &zeros[t * gpr + c]);
        pack_row(q, hidden, bits, codes + t * row_bytes);
    }
    free(q);
    return FC_REF_OK;
}

/* Algorithm 1, first FinegrainedQuantize: the input is binary16 and is widened
   exactly to fp32 before Eq. 1-2. */
int fc_ref_quantize(const uint16_t *x_f16, int64_t tokens, int64_t hidden, int group, int bits,
                    uint8_t *codes, float *scales, float *zeros)
{
    if (!check_shape(tokens, hidden, group, bits)) return FC_REF_BAD_ARG;
    if (tokens == 0) return FC_REF_OK;
    if (!x_f16 || !codes || !scales || !zeros) return FC_REF_BAD_ARG;
    const int64_t gpr = hidden / group;
    const int64_t row_bytes = hidden * bits / 8;
    float *xf = (float *)malloc(sizeof(float) * (size_t)hidden);
    uint8_t *q = (uint8_t *)malloc((size_t)hidden);
    if (!xf || !q) { free(xf); free(q); return FC_REF_NO_MEM; }
    for (int64_t t = 0; t < tokens; ++t) {
        for (int64_t h = 0; h < hidden; ++h) xf[h] = fc_ref_half_to_float(x_f16[t * hidden + h]);
        for (int64_t c = 0; c < gpr; ++c)
            fc_ref_quantize_group_f32(xf + c * group, group, bits,
                                      q + c * group, &scales[t * gpr + c], &zeros[t * gpr + c]);
        pack_row(q, hidden, bits, codes + t * row_bytes);
    }
    free(xf);
    free(q);
    return FC_REF_OK;
}

/* Dequantize (R2) to fp32: x^ = (q - z) * s, one subtraction and one product. */
int fc_ref_dequantize_f32(const uint8_t *codes, const float *scales, const float *zeros,
                          int64_t tokens, int64_t hidden, int group, int bits, float *y)
{
    if (!check_shape(tokens, hidden, group, bits)) return FC_REF_BAD_ARG;
    if (tokens == 0) return FC_REF_OK;
    if (!codes || !scales || !zeros || !y) return FC_REF_BAD_ARG;
    const int64_t gpr = hidden / group;
    const int64_t row_bytes = hidden * bits / 8;
    for (int64_t t = 0; t < tokens; ++t)
        for (int64_t h = 0; h < hidden; ++h) {
            const int64_t gi = t * gpr + h / group;
            const float d = (float)code_at(codes + t * row_bytes, h, bits) - zeros[gi];
            y[t * hidden + h] = d * scales[gi];
        }
    return FC_REF_OK;
}

/* Algorithm 1, last Dequantize: the recovered values are binary16 (RNE). */
int fc_ref_dequantize(const uint8_t *codes, const float *scales, const float *zeros,
                      int64_t tokens, int64_t hidden, int group, int bits, uint16_t *y_f16)
{
    if (!check_shape(tokens, hidden, group, bits)) return FC_REF_BAD_ARG;
    if (tokens == 0) return FC_REF_OK;
    if (!codes || !scales || !zeros || !y_f16) return FC_REF_BAD_ARG;
    const int64_t gpr = hidden / group;
    const int64_t row_bytes = hidden * bits / 8;
    for (int64_t t = 0; t < tokens; ++t)
        for (int64_t h = 0; h < hidden; ++h) {
            const int64_t gi = t * gpr + h / group;
            const float d = (float)code_at(codes + t * row_bytes, h, bits) - zeros[gi];
            y_f16[t * hidden + h] = fc_ref_float_to_half(d * scales[gi]);
        }
    return FC_REF_OK;
}

/* Algorithm 1, the Dequantize loop over the N received slices followed by
   ReduceSum (R6, R7).  Source j's codes start at codes_in + j*codes_stride
   bytes, its scales/zeros at +j*meta_stride floats.  acc: fp32 [tokens,hidden]. */
int fc_ref_dequant_reduce_f32(const uint8_t *codes_in, int64_t codes_stride,
                              const float *scales_in, const float *zeros_in, int64_t meta_stride,
                              int n_src, int64_t tokens, int64_t hidden, int group, int bits_in,
                              float *acc)
{
    if (!check_shape(tokens, hidden, group, bits_in) || n_src < 1) return FC_REF_BAD_ARG;
    if (tokens == 0) return FC_REF_OK;
    if (!codes_in || !scales_in || !zeros_in || !acc) return FC_REF_BAD_ARG;
    const int64_t gpr = hidden / group;
    const int64_t row_bytes = hidden * bits_in / 8;
    for (int64_t t = 0; t < tokens; ++t)
        for (int64_t h = 0; h < hidden; ++h) {
            const int64_t gi = t * gpr + h / group;
            float a = 0.0f;
            for (int j = 0; j < n_src; ++j) {
                const uint8_t *row = codes_in + (int64_t)j * codes_stride + t * row_bytes;
                const float d = (float)code_at(row, h, bits_in) - zeros_in[(int64_t)j * meta_stride + gi];
                a = fmaf(d, scales_in[(int64_t)j * meta_stride + gi], a);
            }
            acc[t * hidden + h] = a;
        }
    return FC_REF_OK;
}

/* Algorithm 1, middle of the loop body: Dequantize x N, ReduceSum, then the
   second FinegrainedQuantize with bits_out. */
int fc_ref_dequant_reduce_requant(const uint8_t *codes_in, int64_t codes_stride,
                                  const float *scales_in, const float *zeros_in, int64_t meta_stride,
                                  int n_src, int64_t tokens, int64_t hidden, int group,
                                  int bits_in, int bits_out,
                                  uint8_t *codes_out, float *scales_out, float *zeros_out)
{
    if (!check_shape(tokens, hidden, group, bits_in) || !check_shape(tokens, hidden, group, bits_out)
        || n_src < 1)
        return FC_REF_BAD_ARG;
    if (tokens == 0) return FC_REF_OK;
    float *acc = (float *)malloc(sizeof(float) * (size_t)(tokens * hidden));
    if (!acc) return FC_REF_NO_MEM;
    int rc = fc_ref_dequant_reduce_f32(codes_in, codes_stride, scales_in, zeros_in, meta_stride,
                                       n_src, tokens, hidden, group, bits_in, acc);
    if (rc == FC_REF_OK)
        rc = fc_ref_quantize_f32(acc, tokens, hidden, group, bits_out, codes_out, scales_out, zeros_out);
    free(acc);
    return rc;
}

/* Algorithm 1 end to end on one device, the two exchanges being identity
   copies: x_f16 is [n_src, tokens, hidden] (the N ranks' partial activations),
   y_f16 is [tokens, hidden].  The volume is quantized and dequantized exactly
   twice (Table 1, "QDQ Step"). */
int fc_ref_allreduce_sim(const uint16_t *x_f16, int n_src, int64_t tokens, int64_t hidden,
                         int group, int bits_rs, int bits_ag, uint16_t *y_f16)
{
    if (!check_shape(tokens, hidden, group, bits_rs) || !check_shape(tokens, hidden, group, bits_ag)
        || n_src < 1)
        return FC_REF_BAD_ARG;
    if (tokens == 0) return FC_REF_OK;
    const int64_t m = tokens * hidden, ng = m / group;
    const int64_t cb_rs = m * bits_rs / 8, cb_ag = m * bits_ag / 8;
    uint8_t *c1 = (uint8_t *)malloc((size_t)(cb_rs * n_src));
    float *s1 = (float *)malloc(sizeof(float) * (size_t)(ng * n_src));
    float *z1 = (float *)malloc(sizeof(float) * (size_t)(ng * n_src));
    uint8_t *c2 = (uint8_t *)malloc((size_t)cb_ag);
    float *s2 = (float *)malloc(sizeof(float) * (size_t)ng);
    float *z2 = (float *)malloc(sizeof(float) * (size_t)ng);
    int rc = (c1 && s1 && z1 && c2 && s2 && z2) ? FC_REF_OK : FC_REF_NO_MEM;
    for (int j = 0; rc == FC_REF_OK && j < n_src; ++j)
        rc = fc_ref_quantize(x_f16 + (int64_t)j * m, tokens, hidden, group, bits_rs,
                             c1 + (int64_t)j * cb_rs, s1 + (int64_t)j * ng, z1 + (int64_t)j * ng);
    if (rc == FC_REF_OK)
        rc = fc_ref_dequant_reduce_requant(c1, cb_rs, s1, z1, ng, n_src, tokens, hidden, group,
                                           bits_rs, bits_ag, c2, s2, z2);
    if (rc == FC_REF_OK)
        rc = fc_ref_dequantize(c2, s2, z2, tokens, hidden, group, bits_ag, y_f16);
    free(c1); free(s1); free(z1); free(c2); free(s2); free(z2);
    return rc;
}

/* ======================================================================== */
/* Symmetric quantization (Appendix, Eq. 3-4) -- readings S1-S4 above.       */
/* ======================================================================== */

/* Eq. 3-4 on ONE group.  q: g signed codes, one per byte (not packed). */
void fc_ref_quantize_group_sym_f32(const float *x, int g, int bits, int8_t *q, float *scale)
{
    const float qm = (float)((1 << (bits - 1)) - 1);          /* 2^(n-1) - 1 */
    const float lo = -(float)(1 << (bits - 1));               /* -2^(n-1)   */
    float amax = 0.0f;
    for (int k = 0; k < g; ++k) {
        const float a = fabsf(x[k]);
        if (a > amax) amax = a;
    }
    float s = amax / qm;                                      /* Eq. 3 */
    if (!(s >= FLT_MIN)) s = 1.0f;                            /* S2 */
    const float inv = 1.0f / s;
    for (int k = 0; k < g; ++k) {
        float t = rintf(x[k] * inv);                          /* Eq. 4: round(X / s) */
        if (t < lo) t = lo;                                   /*        clamp        */
        if (t > qm) t = qm;
        q[k] = (int8_t)t;
    }
    *scale = s;
}

static void pack_row_signed(const int8_t *q, int64_t hidden, int bits, uint8_t *dst)
{
    if (bits == 8) {
        for (int64_t k = 0; k < hidden; ++k) dst[k] = (uint8_t)q[k];
    } else {
        for (int64_t k = 0; k < hidden / 2; ++k)
            dst[k] = (uint8_t)((q[2 * k] & 0x0F) | ((q[2 * k + 1] & 0x0F) << 4));
    }
}

static int signed_code_at(const uint8_t *row, int64_t h, int bits)
{
    if (bits == 8) return (int)(int8_t)row[h];
    const uint8_t b = row[h / 2];
    const int n = (h & 1) ? (b >> 4) : (b & 0x0F);
    return n >= 8 ? n - 16 : n;                               /* two's complement nibble */
}

int fc_ref_quantize_sym_f32(const float *x, int64_t tokens, int64_t hidden, int group, int bits,
                            uint8_t *codes, float *scales)
{
    if (!check_shape(tokens, hidden, group, bits)) return FC_REF_BAD_ARG;
    if (tokens == 0) return FC_REF_OK;
    if (!x || !codes || !scales) return FC_REF_BAD_ARG;
    const int64_t gpr = hidden / group;
    const int64_t row_bytes = hidden * bits / 8;
    int8_t *q = (int8_t *)malloc((size_t)hidden);
    if (!q) return FC_REF_NO_MEM;
    for (int64_t t = 0; t < tokens; ++t) {
        for (int64_t c = 0; c < gpr; ++c)
            fc_ref_quantize_group_sym_f32(x + t * hidden + c * group, group, bits, q + c * group,
                                          &scales[t * gpr + c]);
        pack_row_signed(q, hidden, bits, codes + t * row_bytes);
    }
    free(q);
    return FC_REF_OK;
}

int fc_ref_quantize_sym(const uint16_t *x_f16, int64_t tokens, int64_t hidden, int group, int bits,
                        uint8_t *codes, float *scales)
{
    if (!check_shape(tokens, hidden, group, bits)) return FC_REF_BAD_ARG;
    if (tokens == 0) return FC_REF_OK;
    if (!x_f16 || !codes || !scales) return FC_REF_BAD_ARG;
    float *xf = (float *)malloc(sizeof(float) * (size_t)(tokens * hidden));
    if (!xf) return FC_REF_NO_MEM;
    for (int64_t i = 0; i < tokens * hidden; ++i) xf[i] = fc_ref_half_to_float(x_f16[i]);
    const int rc = fc_ref_quantize_sym_f32(xf, tokens, hidden, group, bits, codes, scales);
    free(xf);
    return rc;
}

/* x^ = q * s (S4), fp32 */
int fc_ref_dequantize_sym_f32(const uint8_t *codes, const float *scales,
                              int64_t tokens, int64_t hidden, int group, int bits, float *y)
{
    if (!check_shape(tokens, hidden, group, bits)) return FC_REF_BAD_ARG;
    if (tokens == 0) return FC_REF_OK;
    if (!codes || !scales || !y) return FC_REF_BAD_ARG;
    const int64_t gpr = hidden / group;
    const int64_t row_bytes = hidden * bits / 8;
    for (int64_t t = 0; t < tokens; ++t)
        for (int64_t h = 0; h < hidden; ++h)
            y[t * hidden + h] = (float)signed_code_at(codes + t * row_bytes, h, bits)
                                * scales[t * gpr + h / group];
    return FC_REF_OK;
}

int fc_ref_dequantize_sym(const uint8_t *codes, const float *scales,
                          int64_t tokens, int64_t hidden, int group, int bits, uint16_t *y_f16)
{
    if (!check_shape(tokens, hidden, group, bits)) return FC_REF_BAD_ARG;
    if (tokens == 0) return FC_REF_OK;
    if (!codes || !scales || !y_f16) return FC_REF_BAD_ARG;
    const int64_t gpr = hidden / group;
    const int64_t row_bytes = hidden * bits / 8;
    for (int64_t t = 0; t < tokens; ++t)
        for (int64_t h = 0; h < hidden; ++h)
            y_f16[t * hidden + h] = fc_ref_float_to_half(
                (float)signed_code_at(codes + t * row_bytes, h, bits) * scales[t * gpr + h / group]);
    return FC_REF_OK;
}

int fc_ref_dequant_reduce_sym_f32(const uint8_t *codes_in, int64_t codes_stride,
                                  const float *scales_in, int64_t meta_stride,
                                  int n_src, int64_t tokens, int64_t hidden, int group, int bits_in,
                                  float *acc)
{
    if (!check_shape(tokens, hidden, group, bits_in) || n_src < 1) return FC_REF_BAD_ARG;
    if (tokens == 0) return FC_REF_OK;
    if (!codes_in || !scales_in || !acc) return FC_REF_BAD_ARG;
    const int64_t gpr = hidden / group;
    const int64_t row_bytes = hidden * bits_in / 8;
    for (int64_t t = 0; t < tokens; ++t)
        for (int64_t h = 0; h < hidden; ++h) {
            const int64_t gi = t * gpr + h / group;
            float a = 0.0f;
            for (int j = 0; j < n_src; ++j) {
                const uint8_t *row = codes_in + (int64_t)j * codes_stride + t * row_bytes;
                a = fmaf((float)signed_code_at(row, h, bits_in),
                         scales_in[(int64_t)j * meta_stride + gi], a);
            }
            acc[t * hidden + h] = a;
        }
    return FC_REF_OK;
}

int fc_ref_dequant_reduce_requant_sym(const uint8_t *codes_in, int64_t codes_stride,
                                      const float *scales_in, int64_t meta_stride,
                                      int n_src, int64_t tokens, int64_t hidden, int group,
                                      int bits_in, int bits_out,
                                      uint8_t *codes_out, float *scales_out)
{
    if (!check_shape(tokens, hidden, group, bits_in) || !check_shape(tokens, hidden, group, bits_out)
        || n_src < 1)
        return FC_REF_BAD_ARG;
    if (tokens == 0) return FC_REF_OK;
    float *acc = (float *)malloc(sizeof(float) * (size_t)(tokens * hidden));
    if (!acc) return FC_REF_NO_MEM;
    int rc = fc_ref_dequant_reduce_sym_f32(codes_in, codes_stride, scales_in, meta_stride, n_src,
                                           tokens, hidden, group, bits_in, acc);
    if (rc == FC_REF_OK)
        rc = fc_ref_quantize_sym_f32(acc, tokens, hidden, group, bits_out, codes_out, scales_out);
    free(acc);
    return rc;
}

int fc_ref_allreduce_sim_sym(const uint16_t *x_f16, int n_src, int64_t tokens, int64_t hidden,
                             int group, int bits_rs, int bits_ag, uint16_t *y_f16)
{
    if (!check_shape(tokens, hidden, group, bits_rs) || !check_shape(tokens, hidden, group, bits_ag)
        || n_src < 1)
        return FC_REF_BAD_ARG;
    if (tokens == 0) return FC_REF_OK;
    const int64_t m = tokens * hidden, ng = m / group;
    const int64_t cb_rs = m * bits_rs / 8, cb_ag = m * bits_ag / 8;
    uint8_t *c1 = (uint8_t *)malloc((size_t)(cb_rs * n_src));
    float *s1 = (float *)malloc(sizeof(float) * (size_t)(ng * n_src));
    uint8_t *c2 = (uint8_t *)malloc((size_t)cb_ag);
    float *s2 = (float *)malloc(sizeof(float) * (size_t)ng);
    int rc = (c1 && s1 && c2 && s2) ? FC_REF_OK : FC_REF_NO_MEM;
    for (int j = 0; rc == FC_REF_OK && j < n_src; ++j)
        rc = fc_ref_quantize_sym(x_f16 + (int64_t)j * m, tokens, hidden, group, bits_rs,
                                 c1 + (int64_t)j * cb_rs, s1 + (int64_t)j * ng);
    if (rc == FC_REF_OK)
        rc = fc_ref_dequant_reduce_requant_sym(c1, cb_rs, s1, ng, n_src, tokens, hidden, group,
                                               bits_rs, bits_ag, c2, s2);
    if (rc == FC_REF_OK)
        rc = fc_ref_dequantize_sym(c2, s2, tokens, hidden, group, bits_ag, y_f16);
    free(c1); free(s1); free(c2); free(s2);
    return rc;
}

/* ======================================================================== */
/* FP8 E4M3 per-group symmetric quantization -- readings F1-F4 above.        */
/* ======================================================================== */

/* value of one E4M3 byte (F1) */
float fc_ref_e4m3_to_float(uint8_t c)
{
    const int sign = (c >> 7) & 1;
    const int e = (c >> 3) & 0xF;
    const int f = c & 7;
    double v;
    if (e == 15 && f == 7)
        v = (double)NAN;
    else if (e == 0)
        v = ldexp((double)f, -9);                /* zero or subnormal: f * 2^-9 */
    else
        v = ldexp((double)(8 + f), e - 10);      /* (1 + f/8) * 2^(e-7) */
    return (float)(sign ? -v : v);
}

/* nearest E4M3 number, ties to even, saturating at +-448 (F3) */
uint8_t fc_ref_float_to_e4m3(float x)
{
    uint32_t u;
    memcpy(&u, &x, 4);
    const uint8_t sign = (uint8_t)((u >> 24) & 0x80u);
    if (isnan(x)) return (uint8_t)(sign | 0x7Fu);
    const double a = fabs((double)x);
    if (a >= 448.0) return (uint8_t)(sign | 0x7Eu);            /* 448 = 0.1111.110 */
    if (a == 0.0) return sign;
    int e2;
    (void)frexp(a, &e2);
    int e = e2 - 1;                              /* a in [2^e, 2^(e+1)) */
    if (e < -6) e = -6;                          /* subnormals share the grid of the first binade */
    /* spacing of E4M3 numbers around a is 2^(e-3); a / spacing is exact in
       double and nearbyint rounds half to even */
    uint32_t mant = (uint32_t)nearbyint(ldexp(a, 3 - e));      /* in [0, 16] */
    int be = e + 7;
    if (mant >= 16u) { mant = 8u; be += 1; }
    if (mant < 8u) return (uint8_t)(sign | mant);              /* subnormal (or zero) */
    return (uint8_t)(sign | ((uint32_t)be << 3) | (mant - 8u)); /* be <= 15 and never 1111.111 since a < 448 */
}

/* F2-F3 on ONE group */
void fc_ref_quantize_group_fp8_f32(const float *x, int g, uint8_t *q, float *scale)
{
    float amax = 0.0f;
    for (int k = 0; k < g; ++k) {
        const float a = fabsf(x[k]);
        if (a > amax) amax = a;
    }
    float s = amax / 448.0f;
    if (!(s >= FLT_MIN)) s = 1.0f;
    const float inv = 1.0f / s;
    for (int k = 0; k < g; ++k) q[k] = fc_ref_float_to_e4m3(x[k] * inv);
    *scale = s;
}

int fc_ref_quantize_fp8_f32(const float *x, int64_t tokens, int64_t hidden, int group,
                            uint8_t *codes, float *scales)
{
    if (!check_shape(tokens, hidden, group, 8)) return FC_REF_BAD_ARG;
    if (tokens == 0) return FC_REF_OK;
    if (!x || !codes || !scales) return FC_REF_BAD_ARG;
    const int64_t gpr = hidden / group;
    for (int64_t t = 0; t < tokens; ++t)
        for (int64_t c = 0; c < gpr; ++c)
            fc_ref_quantize_group_fp8_f32(x + t * hidden + c * group, group,
                                          codes + t * hidden + c * group, &scales[t * gpr + c]);
    return FC_REF_OK;
}

int fc_ref_quantize_fp8(const uint16_t *x_f16, int64_t tokens, int64_t hidden, int group,
                        uint8_t *codes, float *scales)
{
    if (!check_shape(tokens, hidden, group, 8)) return FC_REF_BAD_ARG;
    if (tokens == 0) return FC_REF_OK;
    if (!x_f16 || !codes || !scales) return FC_REF_BAD_ARG;
    float *xf = (float *)malloc(sizeof(float) * (size_t)(tokens * hidden));
    if (!xf) return FC_REF_NO_MEM;
    for (int64_t i = 0; i < tokens * hidden; ++i) xf[i] = fc_ref_half_to_float(x_f16[i]);
    const int rc = fc_ref_quantize_fp8_f32(xf, tokens, hidden, group, codes, scales);
    free(xf);
    return rc;
}

/* x^ = value(q) * s (F4), fp32 */
int fc_ref_dequantize_fp8_f32(const uint8_t *codes, const float *scales,
                              int64_t tokens, int64_t hidden, int group, float *y)
{
    if (!check_shape(tokens, hidden, group, 8)) return FC_REF_BAD_ARG;
    if (tokens == 0) return FC_REF_OK;
    if (!codes || !scales || !y) return FC_REF_BAD_ARG;
    const int64_t gpr = hidden / group;
    for (int64_t t = 0; t < tokens; ++t)
        for (int64_t h = 0; h < hidden; ++h)
            y[t * hidden + h] = fc_ref_e4m3_to_float(codes[t * hidden + h]) * scales[t * gpr + h / group];
    return FC_REF_OK;
}

int fc_ref_dequantize_fp8(const uint8_t *codes, const float *scales,
                          int64_t tokens, int64_t hidden, int group, uint16_t *y_f16)
{
    if (!check_shape(tokens, hidden, group, 8)) return FC_REF_BAD_ARG;
    if (tokens == 0) return FC_REF_OK;
    if (!codes || !scales || !y_f16) return FC_REF_BAD_ARG;
    const int64_t gpr = hidden / group;
    for (int64_t t = 0; t < tokens; ++t)
        for (int64_t h = 0; h < hidden; ++h)
            y_f16[t * hidden + h] = fc_ref_float_to_half(
                fc_ref_e4m3_to_float(codes[t * hidden + h]) * scales[t * gpr + h / group]);
    return FC_REF_OK;
}

int fc_ref_dequant_reduce_fp8_f32(const uint8_t *codes_in, int64_t codes_stride,
                                  const float *scales_in, int64_t meta_stride,
                                  int n_src, int64_t tokens, int64_t hidden, int group, float *acc)
{
    if (!check_shape(tokens, hidden, group, 8) || n_src < 1) return FC_REF_BAD_ARG;
    if (tokens == 0) return FC_REF_OK;
    if (!codes_in || !scales_in || !acc) return FC_REF_BAD_ARG;
    const int64_t gpr = hidden / group;
    for (int64_t t = 0; t < tokens; ++t)
        for (int64_t h = 0; h < hidden; ++h) {
            const int64_t gi = t * gpr + h / group;
            float a = 0.0f;
            for (int j = 0; j < n_src; ++j)
                a = fmaf(fc_ref_e4m3_to_float(codes_in[(int64_t)j * codes_stride + t * hidden + h]),
                         scales_in[(int64_t)j * meta_stride + gi], a);
            acc[t * hidden + h] = a;
        }
    return FC_REF_OK;
}

int fc_ref_dequant_reduce_requant_fp8(const uint8_t *codes_in, int64_t codes_stride,
                                      const float *scales_in, int64_t meta_stride,
                                      int n_src, int64_t tokens, int64_t hidden, int group,
                                      uint8_t *codes_out, float *scales_out)
{
    if (!check_shape(tokens, hidden, group, 8) || n_src < 1) return FC_REF_BAD_ARG;
    if (tokens == 0) return FC_REF_OK;
    float *acc = (float *)malloc(sizeof(float) * (size_t)(tokens * hidden));
    if (!acc) return FC_REF_NO_MEM;
    int rc = fc_ref_dequant_reduce_fp8_f32(codes_in, codes_stride, scales_in, meta_stride, n_src,
                                           tokens, hidden, group, acc);
    if (rc == FC_REF_OK)
        rc = fc_ref_quantize_fp8_f32(acc, tokens, hidden, group, codes_out, scales_out);
    free(acc);
    return rc;
}

int fc_ref_allreduce_sim_fp8(const uint16_t *x_f16, int n_src, int64_t tokens, int64_t hidden,
                             int group, uint16_t *y_f16)
{
    if (!check_shape(tokens, hidden, group, 8) || n_src < 1) return FC_REF_BAD_ARG;
    if (tokens == 0) return FC_REF_OK;
    const int64_t m = tokens * hidden, ng = m / group;
    uint8_t *c1 = (uint8_t *)malloc((size_t)(m * n_src));
    float *s1 = (float *)malloc(sizeof(float) * (size_t)(ng * n_src));
    uint8_t *c2 = (uint8_t *)malloc((size_t)m);
    float *s2 = (float *)malloc(sizeof(float) * (size_t)ng);
    int rc = (c1 && s1 && c2 && s2) ? FC_REF_OK : FC_REF_NO_MEM;
    for (int j = 0; rc == FC_REF_OK && j < n_src; ++j)
        rc = fc_ref_quantize_fp8(x_f16 + (int64_t)j * m, tokens, hidden, group,
                                 c1 + (int64_t)j * m, s1 + (int64_t)j * ng);
    if (rc == FC_REF_OK)
        rc = fc_ref_dequant_reduce_requant_fp8(c1, m, s1, ng, n_src, tokens, hidden, group, c2, s2);
    if (rc == FC_REF_OK)
        rc = fc_ref_dequantize_fp8(c2, s2, tokens, hidden, group, y_f16);
    free(c1); free(s1); free(c2); free(s2);
    return rc;
}

/* ======================================================================== */
/* Hadamard rotation around the quantized all-reduce -- readings H1-H4.      */
/* ======================================================================== */

#define FC_REF_ASYM 0
#define FC_REF_SYM 1
#define FC_REF_FP8 2

static int log2_exact(int64_t v)
{
    int n = 0;
    while (((int64_t)1 << n) < v) ++n;
    return (((int64_t)1 << n) == v) ? n : -1;
}

/* In-place unnormalised Walsh-Hadamard transform of n = 2^k fp32 values (H2). */
int fc_ref_hadamard_f32(float *x, int64_t n)
{
    if (n < 1 || log2_exact(n) < 0 || !x) return FC_REF_BAD_ARG;
    for (int64_t span = 1; span < n; span *= 2)
        for (int64_t base = 0; base < n; base += 2 * span)
            for (int64_t i = base; i < base + span; ++i) {
                const float a = x[i], b = x[i + span];
                x[i] = a + b;
                x[i + span] = a - b;
            }
    return FC_REF_OK;
}

/* H5: the largest power of two that divides n, and the transform applied to every aligned block of that length */
static int64_t rotation_block(int64_t n) { return n & -n; }

int fc_ref_hadamard_blocks_f32(float *x, int64_t n)
{
    if (n < 1 || !x) return FC_REF_BAD_ARG;
    const int64_t b = rotation_block(n);
    for (int64_t at = 0; at < n; at += b) {
        const int rc = fc_ref_hadamard_f32(x + at, b);
        if (rc != FC_REF_OK) return rc;
    }
    return FC_REF_OK;
}

static int quantize_any_f32(int quantizer, const float *x, int64_t tokens, int64_t hidden, int group,
                            int bits, uint8_t *codes, float *scales, float *zeros)
{
    if (quantizer == FC_REF_ASYM) return fc_ref_quantize_f32(x, tokens, hidden, group, bits, codes, scales, zeros);
    if (quantizer == FC_REF_SYM) return fc_ref_quantize_sym_f32(x, tokens, hidden, group, bits, codes, scales);
    if (quantizer == FC_REF_FP8 && bits == 8) return fc_ref_quantize_fp8_f32(x, tokens, hidden, group, codes, scales);
    return FC_REF_BAD_ARG;
}

static int dequantize_any_f32(int quantizer, const uint8_t *codes, const float *scales, const float *zeros,
                              int64_t tokens, int64_t hidden, int group, int bits, float *y)
{
    if (quantizer == FC_REF_ASYM) return fc_ref_dequantize_f32(codes, scales, zeros, tokens, hidden, group, bits, y);
    if (quantizer == FC_REF_SYM) return fc_ref_dequantize_sym_f32(codes, scales, tokens, hidden, group, bits, y);
    if (quantizer == FC_REF_FP8 && bits == 8) return fc_ref_dequantize_fp8_f32(codes, scales, tokens, hidden, group, y);
    return FC_REF_BAD_ARG;
}

/* rotate each token row (H1-H3, forward scaling), then FinegrainedQuantize in fp32 (H4) */
int fc_ref_quantize_rot(const uint16_t *x_f16, int64_t tokens, int64_t hidden, int group, int bits,
                        int quantizer, uint8_t *codes, float *scales, float *zeros)
{
    if (hidden < 1 || !check_shape(tokens, hidden, group, bits)) return FC_REF_BAD_ARG;
    const int n = log2_exact(rotation_block(hidden));         /* H5: per block of 2^n elements */
    if (tokens == 0) return FC_REF_OK;
    if (!x_f16 || !codes || !scales) return FC_REF_BAD_ARG;
    float *xf = (float *)malloc(sizeof(float) * (size_t)(tokens * hidden));
    if (!xf) return FC_REF_NO_MEM;
    const float fwd = ldexpf(1.0f, -((n + 1) / 2));          /* 2^-ceil(n/2) */
    for (int64_t t = 0; t < tokens; ++t) {
        float *row = xf + t * hidden;
        for (int64_t h = 0; h < hidden; ++h) row[h] = fc_ref_half_to_float(x_f16[t * hidden + h]);
        fc_ref_hadamard_blocks_f32(row, hidden);
        for (int64_t h = 0; h < hidden; ++h) row[h] *= fwd;
    }
    const int rc = quantize_any_f32(quantizer, xf, tokens, hidden, group, bits, codes, scales, zeros);
    free(xf);
    return rc;
}

/* Dequantize in fp32, rotate back (inverse scaling), round to binary16 (H4) */
int fc_ref_dequantize_rot(const uint8_t *codes, const float *scales, const float *zeros,
                          int64_t tokens, int64_t hidden, int group, int bits, int quantizer,
                          uint16_t *y_f16)
{
    if (hidden < 1 || !check_shape(tokens, hidden, group, bits)) return FC_REF_BAD_ARG;
    const int n = log2_exact(rotation_block(hidden));         /* H5: per block of 2^n elements */
    if (tokens == 0) return FC_REF_OK;
    if (!codes || !scales || !y_f16) return FC_REF_BAD_ARG;
    float *yf = (float *)malloc(sizeof(float) * (size_t)(tokens * hidden));
    if (!yf) return FC_REF_NO_MEM;
    int rc = dequantize_any_f32(quantizer, codes, scales, zeros, tokens, hidden, group, bits, yf);
    const float inv = ldexpf(1.0f, -(n / 2));                /* 2^-floor(n/2) */
    for (int64_t t = 0; rc == FC_REF_OK && t < tokens; ++t) {
        float *row = yf + t * hidden;
        fc_ref_hadamard_blocks_f32(row, hidden);
        for (int64_t h = 0; h < hidden; ++h) y_f16[t * hidden + h] = fc_ref_float_to_half(row[h] * inv);
    }
    free(yf);
    return rc;
}

/* Algorithm 1 with the rotation around it: rotate+quantize each partial, the unchanged
   Dequantize-ReduceSum-FinegrainedQuantize step, dequantize+rotate back. */
int fc_ref_allreduce_sim_rot(const uint16_t *x_f16, int n_src, int64_t tokens, int64_t hidden,
                             int group, int bits_rs, int bits_ag, int quantizer, uint16_t *y_f16)
{
    if (!check_shape(tokens, hidden, group, bits_rs) || !check_shape(tokens, hidden, group, bits_ag)
        || n_src < 1 || hidden < 1)
        return FC_REF_BAD_ARG;
    if (tokens == 0) return FC_REF_OK;
    const int64_t m = tokens * hidden, ng = m / group;
    const int64_t cb_rs = m * bits_rs / 8, cb_ag = m * bits_ag / 8;
    uint8_t *c1 = (uint8_t *)malloc((size_t)(cb_rs * n_src));
    float *s1 = (float *)malloc(sizeof(float) * (size_t)(ng * n_src));
    float *z1 = (float *)malloc(sizeof(float) * (size_t)(ng * n_src));
    uint8_t *c2 = (uint8_t *)malloc((size_t)cb_ag);
    float *s2 = (float *)malloc(sizeof(float) * (size_t)ng);
    float *z2 = (float *)malloc(sizeof(float) * (size_t)ng);
    int rc = (c1 && s1 && z1 && c2 && s2 && z2) ? FC_REF_OK : FC_REF_NO_MEM;
    for (int j = 0; rc == FC_REF_OK && j < n_src; ++j)
        rc = fc_ref_quantize_rot(x_f16 + (int64_t)j * m, tokens, hidden, group, bits_rs, quantizer,
                                 c1 + (int64_t)j * cb_rs, s1 + (int64_t)j * ng, z1 + (int64_t)j * ng);
    if (rc == FC_REF_OK) {
        if (quantizer == FC_REF_ASYM)
            rc = fc_ref_dequant_reduce_requant(c1, cb_rs, s1, z1, ng, n_src, tokens, hidden, group,
                                               bits_rs, bits_ag, c2, s2, z2);
        else if (quantizer == FC_REF_SYM)
            rc = fc_ref_dequant_reduce_requant_sym(c1, cb_rs, s1, ng, n_src, tokens, hidden, group,
                                                   bits_rs, bits_ag, c2, s2);
        else if (bits_rs == 8 && bits_ag == 8)
            rc = fc_ref_dequant_reduce_requant_fp8(c1, cb_rs, s1, ng, n_src, tokens, hidden, group, c2, s2);
        else
            rc = FC_REF_BAD_ARG;
    }
    if (rc == FC_REF_OK)
        rc = fc_ref_dequantize_rot(c2, s2, z2, tokens, hidden, group, bits_ag, quantizer, y_f16);
    free(c1); free(s1); free(z1); free(c2); free(s2); free(z2);
    return rc;
}

/* ======================================================================== */
/* Asymmetric quantization with binary16 metadata -- readings C1-C4 above.   */
/* ======================================================================== */

static float meta_scale(uint32_t m) { return fc_ref_half_to_float((uint16_t)(m & 0xFFFFu)); }
static float meta_zero(uint32_t m) { return fc_ref_half_to_float((uint16_t)(m >> 16)); }

/* Eq. 1-2 on ONE group with the scale and the zero-point held in binary16.
   q: g codes, one per byte (not packed); *meta: the group's word (C4). */
void fc_ref_quantize_group_cmeta_f32(const float *x, int g, int bits, uint8_t *q, uint32_t *meta)
{
    const float qmax = (float)((1 << bits) - 1);
    float mn = x[0], mx = x[0];
    for (int k = 1; k < g; ++k) {
        if (x[k] < mn) mn = x[k];
        if (x[k] > mx) mx = x[k];
    }
    float s = (mx - mn) / qmax;                  /* Eq. 1, scale */
    if (!(s >= FLT_MIN)) {                       /* R5 */
        const float a = fabsf(mn);
        s = (a >= FLT_MIN) ? a : 1.0f;
    }
    uint16_t sh = fc_ref_float_to_half(s);       /* C1 */
    if (sh == 0x0000u) sh = 0x0001u;             /*   2^-24 */
    if (sh == 0x7C00u) sh = 0x7BFFu;             /*   65504 */
    s = fc_ref_half_to_float(sh);
    const float inv = 1.0f / s;                  /* R4 */
    float zf = 0.0f - rintf(mn * inv);           /* Eq. 1, zero-point */
    uint16_t zh = fc_ref_float_to_half(zf);      /* C2 */
    if ((zh & 0x7FFFu) == 0x7C00u) zh = (uint16_t)((zh & 0x8000u) | 0x7BFFu);
    zf = fc_ref_half_to_float(zh);
    for (int k = 0; k < g; ++k) {
        const float t = rintf(x[k] * inv);       /* Eq. 2 */
        float u = t + zf;
        if (u < 0.0f) u = 0.0f;
        if (u > qmax) u = qmax;
        q[k] = (uint8_t)u;
    }
    *meta = (uint32_t)sh | ((uint32_t)zh << 16);
}

int fc_ref_quantize_cmeta_f32(const float *x, int64_t tokens, int64_t hidden, int group, int bits,
                              uint8_t *codes, uint32_t *meta)
{
    if (!check_shape(tokens, hidden, group, bits)) return FC_REF_BAD_ARG;
    if (tokens == 0) return FC_REF_OK;
    if (!x || !codes || !meta) return FC_REF_BAD_ARG;
    const int64_t gpr = hidden / group;
    const int64_t row_bytes = hidden * bits / 8;
    uint8_t *q = (uint8_t *)malloc((size_t)hidden);
    if (!q) return FC_REF_NO_MEM;
    for (int64_t t = 0; t < tokens; ++t) {
        for (int64_t c = 0; c < gpr; ++c)
            fc_ref_quantize_group_cmeta_f32(x + t * hidden + c * group, group, bits, q + c * group,
                                            &meta[t * gpr + c]);
        pack_row(q, hidden, bits, codes + t * row_bytes);
    }
    free(q);
    return FC_REF_OK;
}

int fc_ref_quantize_cmeta(const uint16_t *x_f16, int64_t tokens, int64_t hidden, int group, int bits,
                          uint8_t *codes, uint32_t *meta)
{
    if (!check_shape(tokens, hidden, group, bits)) return FC_REF_BAD_ARG;
    if (tokens == 0) return FC_REF_OK;
    if (!x_f16 || !codes || !meta) return FC_REF_BAD_ARG;
    float *xf = (float *)malloc(sizeof(float) * (size_t)(tokens * hidden));
    if (!xf) return FC_REF_NO_MEM;
    for (int64_t i = 0; i < tokens * hidden; ++i) xf[i] = fc_ref_half_to_float(x_f16[i]);
    const int rc = fc_ref_quantize_cmeta_f32(xf, tokens, hidden, group, bits, codes, meta);
    free(xf);
    return rc;
}

/* C3, fp32 result */
int fc_ref_dequantize_cmeta_f32(const uint8_t *codes, const uint32_t *meta,
                                int64_t tokens, int64_t hidden, int group, int bits, float *y)
{
    if (!check_shape(tokens, hidden, group, bits)) return FC_REF_BAD_ARG;
    if (tokens == 0) return FC_REF_OK;
    if (!codes || !meta || !y) return FC_REF_BAD_ARG;
    const int64_t gpr = hidden / group;
    const int64_t row_bytes = hidden * bits / 8;
    for (int64_t t = 0; t < tokens; ++t)
        for (int64_t h = 0; h < hidden; ++h) {
            const uint32_t m = meta[t * gpr + h / group];
            const float d = (float)code_at(codes + t * row_bytes, h, bits) - meta_zero(m);
            y[t * hidden + h] = d * meta_scale(m);
        }
    return FC_REF_OK;
}

/* C3, binary16 result (Algorithm 1, last Dequantize) */
int fc_ref_dequantize_cmeta(const uint8_t *codes, const uint32_t *meta,
                            int64_t tokens, int64_t hidden, int group, int bits, uint16_t *y_f16)
{
    if (!check_shape(tokens, hidden, group, bits)) return FC_REF_BAD_ARG;
    if (tokens == 0) return FC_REF_OK;
    if (!codes || !meta || !y_f16) return FC_REF_BAD_ARG;
    const int64_t gpr = hidden / group;
    const int64_t row_bytes = hidden * bits / 8;
    for (int64_t t = 0; t < tokens; ++t)
        for (int64_t h = 0; h < hidden; ++h) {
            const uint32_t m = meta[t * gpr + h / group];
            const float d = (float)code_at(codes + t * row_bytes, h, bits) - meta_zero(m);
            y_f16[t * hidden + h] = fc_ref_float_to_half(d * meta_scale(m));
        }
    return FC_REF_OK;
}

/* Dequantize x N and ReduceSum (R6); source j's words start at meta_in + j*meta_stride. */
int fc_ref_dequant_reduce_cmeta_f32(const uint8_t *codes_in, int64_t codes_stride,
                                    const uint32_t *meta_in, int64_t meta_stride,
                                    int n_src, int64_t tokens, int64_t hidden, int group, int bits_in,
                                    float *acc)
{
    if (!check_shape(tokens, hidden, group, bits_in) || n_src < 1) return FC_REF_BAD_ARG;
    if (tokens == 0) return FC_REF_OK;
    if (!codes_in || !meta_in || !acc) return FC_REF_BAD_ARG;
    const int64_t gpr = hidden / group;
    const int64_t row_bytes = hidden * bits_in / 8;
    for (int64_t t = 0; t < tokens; ++t)
        for (int64_t h = 0; h < hidden; ++h) {
            const int64_t gi = t * gpr + h / group;
            float a = 0.0f;
            for (int j = 0; j < n_src; ++j) {
                const uint8_t *row = codes_in + (int64_t)j * codes_stride + t * row_bytes;
                const uint32_t m = meta_in[(int64_t)j * meta_stride + gi];
                const float d = (float)code_at(row, h, bits_in) - meta_zero(m);
                a = fmaf(d, meta_scale(m), a);
            }
            acc[t * hidden + h] = a;
        }
    return FC_REF_OK;
}

int fc_ref_dequant_reduce_requant_cmeta(const uint8_t *codes_in, int64_t codes_stride,
                                        const uint32_t *meta_in, int64_t meta_stride,
                                        int n_src, int64_t tokens, int64_t hidden, int group,
                                        int bits_in, int bits_out,
                                        uint8_t *codes_out, uint32_t *meta_out)
{
    if (!check_shape(tokens, hidden, group, bits_in) || !check_shape(tokens, hidden, group, bits_out)
        || n_src < 1)
        return FC_REF_BAD_ARG;
    if (tokens == 0) return FC_REF_OK;
    float *acc = (float *)malloc(sizeof(float) * (size_t)(tokens * hidden));
    if (!acc) return FC_REF_NO_MEM;
    int rc = fc_ref_dequant_reduce_cmeta_f32(codes_in, codes_stride, meta_in, meta_stride, n_src,
                                             tokens, hidden, group, bits_in, acc);
    if (rc == FC_REF_OK)
        rc = fc_ref_quantize_cmeta_f32(acc, tokens, hidden, group, bits_out, codes_out, meta_out);
    free(acc);
    return rc;
}

int fc_ref_allreduce_sim_cmeta(const uint16_t *x_f16, int n_src, int64_t tokens, int64_t hidden,
                               int group, int bits_rs, int bits_ag, uint16_t *y_f16)
{
    if (!check_shape(tokens, hidden, group, bits_rs) || !check_shape(tokens, hidden, group, bits_ag)
        || n_src < 1)
        return FC_REF_BAD_ARG;
    if (tokens == 0) return FC_REF_OK;
    const int64_t m = tokens * hidden, ng = m / group;
    const int64_t cb_rs = m * bits_rs / 8, cb_ag = m * bits_ag / 8;
    uint8_t *c1 = (uint8_t *)malloc((size_t)(cb_rs * n_src));
    uint32_t *m1 = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)(ng * n_src));
    uint8_t *c2 = (uint8_t *)malloc((size_t)cb_ag);
    uint32_t *m2 = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)ng);
    int rc = (c1 && m1 && c2 && m2) ? FC_REF_OK : FC_REF_NO_MEM;
    for (int j = 0; rc == FC_REF_OK && j < n_src; ++j)
        rc = fc_ref_quantize_cmeta(x_f16 + (int64_t)j * m, tokens, hidden, group, bits_rs,
                                   c1 + (int64_t)j * cb_rs, m1 + (int64_t)j * ng);
    if (rc == FC_REF_OK)
        rc = fc_ref_dequant_reduce_requant_cmeta(c1, cb_rs, m1, ng, n_src, tokens, hidden, group,
                                                 bits_rs, bits_ag, c2, m2);
    if (rc == FC_REF_OK)
        rc = fc_ref_dequantize_cmeta(c2, m2, tokens, hidden, group, bits_ag, y_f16);
    free(c1); free(m1); free(c2); free(m2);
    return rc;
}
