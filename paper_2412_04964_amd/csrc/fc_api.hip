// fc_api.hip -- the extern "C" boundary declared in include/fc.h: argument
// checks (no HIP call before they pass), shape bookkeeping and kernel dispatch.
#include "fc.h"

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "fc_launch.hpp"

// Scratch of fc_allreduce_sim_static: the intermediate codes, scales and zero-points of one
// all-reduce.  Every GPU the library runs on holds its own copy at its own address until the
// process ends.  In host code the name is only a handle for hipGetSymbolAddress; the device
// address it returns is what the kernels receive.
static __device__ __align__(256) unsigned char scratch[FC_STATIC_SCRATCH_BYTES];

namespace {

thread_local int g_last_hip_error = 0;

constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];     // device address of `scratch`, per device

constexpr int64_t kMaxElems = (int64_t)1 << 36;   // keeps grid*block below 2^32 threads

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int log2_exact(int v)
{
    if (v <= 0 || v > (1 << 20)) return -1;
    int s = 0;
    while ((1 << s) < v) ++s;
    return ((1 << s) == v) ? s : -1;
}

// Checks common to every entry point.  On success *n_elems = tokens*hidden.
int check_shape(int64_t tokens, int64_t hidden, int group, int bits, int64_t *n_elems)
{
    if (bits != 4 && bits != 8) return FC_ERR_BITS;
    const int sh = log2_exact(group);
    if (sh < 5 || sh > 14) return FC_ERR_GROUP;            // 32 .. 16384
    if (tokens < 0 || hidden <= 0) return FC_ERR_SHAPE;
    if (hidden % group != 0) return FC_ERR_GROUP;
    if (hidden > kMaxElems || (tokens > 0 && tokens > kMaxElems / hidden)) return FC_ERR_SHAPE;
    *n_elems = tokens * hidden;
    return FC_OK;
}

int hip_result(hipError_t e)
{
    if (e == hipSuccess) return FC_OK;
    g_last_hip_error = (int)e;
    return FC_ERR_HIP;
}

struct SimLayout {
    size_t codes_rs;     // bytes of one source's codes
    size_t meta;         // bytes of one scales (or zeros) array
    size_t off_codes1, off_scales1, off_zeros1, off_codes2, off_scales2, off_zeros2, total;
};

size_t round16(size_t v) { return (v + 15u) & ~(size_t)15u; }

SimLayout sim_layout(int n_src, int64_t n_elems, int group, int bits_rs, int bits_ag)
{
    SimLayout L;
    L.codes_rs = round16((size_t)(n_elems * bits_rs / 8));
    L.meta = round16((size_t)(n_elems / group) * sizeof(float));
    const size_t codes_ag = round16((size_t)(n_elems * bits_ag / 8));
    size_t off = 0;
    L.off_codes1 = off;  off += L.codes_rs * n_src;
    L.off_scales1 = off; off += L.meta * n_src;
    L.off_zeros1 = off;  off += L.meta * n_src;
    L.off_codes2 = off;  off += codes_ag;
    L.off_scales2 = off; off += L.meta;
    L.off_zeros2 = off;  off += L.meta;
    L.total = off;
    return L;
}

// All quantizer variants share these; every codec but the fp32-metadata asymmetric
// one drops the zero-point arrays (passed as nullptr to the launchers).  The
// binary16-metadata codec passes its array of 32-bit words where the others pass
// `scales`: the kernels move those words as raw bits.
int quantize_impl(int codec, const void *x_f16, int64_t tokens, int64_t hidden, int group, int bits,
                  void *codes, float *scales, float *zeros, void *hip_stream)
{
    const bool sym = codec != fc::CODEC_ASYM;
    int64_t n = 0;
    const int rc = check_shape(tokens, hidden, group, bits, &n);
    if (rc != FC_OK) return rc;
    if (n == 0) return FC_OK;
    if (!x_f16 || !codes || !scales || (!sym && !zeros)) return FC_ERR_NULL;
    if (!aligned16(x_f16) || !aligned16(codes) || !aligned16(scales) || (!sym && !aligned16(zeros)))
        return FC_ERR_ALIGN;
    return hip_result(fc::launch_quantize(bits, codec, x_f16, n, group, codes, scales, sym ? nullptr : zeros,
                                          static_cast<hipStream_t>(hip_stream)));
}

int fused_impl(int codec, const void *codes_in, int64_t codes_src_stride_bytes,
               const float *scales_in, const float *zeros_in, int64_t meta_src_stride_elems,
               int n_src, int64_t tokens, int64_t hidden, int group, int bits_in, int bits_out,
               void *codes_out, float *scales_out, float *zeros_out, void *hip_stream)
{
    const bool sym = codec != fc::CODEC_ASYM;
    int64_t n = 0;
    int rc = check_shape(tokens, hidden, group, bits_in, &n);
    if (rc != FC_OK) return rc;
    if (bits_out != 4 && bits_out != 8) return FC_ERR_BITS;
    if (n_src < 1 || n_src > FC_MAX_SRC) return FC_ERR_SHAPE;
    if (n == 0) return FC_OK;
    if (!codes_in || !scales_in || !codes_out || !scales_out || (!sym && (!zeros_in || !zeros_out)))
        return FC_ERR_NULL;
    if (n_src > 1) {
        if (codes_src_stride_bytes < n * bits_in / 8 || meta_src_stride_elems < n / group)
            return FC_ERR_SHAPE;
        if ((codes_src_stride_bytes & 15) != 0) return FC_ERR_ALIGN;
    } else {
        codes_src_stride_bytes = 0;
        meta_src_stride_elems = 0;
    }
    if (!aligned16(codes_in) || !aligned16(scales_in) || !aligned16(codes_out) || !aligned16(scales_out) ||
        (!sym && (!aligned16(zeros_in) || !aligned16(zeros_out))))
        return FC_ERR_ALIGN;

    fc::FusedArgs a;
    a.codec = codec;
    a.codes_in = codes_in;
    a.codes_stride = codes_src_stride_bytes;
    a.scales_in = scales_in;
    a.zeros_in = sym ? nullptr : zeros_in;
    a.meta_stride = meta_src_stride_elems;
    a.n_src = n_src;
    a.n_elems = n;
    a.group = group;
    a.codes_out = codes_out;
    a.scales_out = scales_out;
    a.zeros_out = sym ? nullptr : zeros_out;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    hipError_t e;
    if (fc::exceeds_tile(bits_in, group))
        e = fc::launch_fused_wide(bits_in, bits_out, a, st);
    else if (bits_in == 4)
        e = (bits_out == 4) ? fc::launch_fused_4_4(a, st) : fc::launch_fused_4_8(a, st);
    else
        e = (bits_out == 4) ? fc::launch_fused_8_4(a, st) : fc::launch_fused_8_8(a, st);
    return hip_result(e);
}

int dequantize_impl(int codec, const void *codes, const float *scales, const float *zeros,
                    int64_t tokens, int64_t hidden, int group, int bits, void *y_f16, void *hip_stream)
{
    const bool sym = codec != fc::CODEC_ASYM;
    int64_t n = 0;
    const int rc = check_shape(tokens, hidden, group, bits, &n);
    if (rc != FC_OK) return rc;
    if (n == 0) return FC_OK;
    if (!codes || !scales || !y_f16 || (!sym && !zeros)) return FC_ERR_NULL;
    if (!aligned16(codes) || !aligned16(scales) || !aligned16(y_f16) || (!sym && !aligned16(zeros)))
        return FC_ERR_ALIGN;
    return hip_result(fc::launch_dequantize(bits, codec, codes, scales, sym ? nullptr : zeros, n, group, y_f16,
                                            static_cast<hipStream_t>(hip_stream)));
}

// one_launch: whether the single-kernel forms (which leave the workspace untouched) may stand in for the
// three-kernel sequence
int allreduce_sim_impl(int codec, const void *x_f16, int n_src, int64_t tokens, int64_t hidden,
                       int group, int bits_rs, int bits_ag, void *y_f16,
                       void *workspace, size_t workspace_bytes, void *hip_stream, bool one_launch = true)
{
    int64_t n = 0;
    const int rc = check_shape(tokens, hidden, group, bits_rs, &n);
    if (rc != FC_OK) return rc;
    if (bits_ag != 4 && bits_ag != 8) return FC_ERR_BITS;
    if (n_src < 1 || n_src > FC_MAX_SRC) return FC_ERR_SHAPE;
    if (n == 0) return FC_OK;
    if (!x_f16 || !y_f16) return FC_ERR_NULL;
    if (!aligned16(x_f16) || !aligned16(y_f16)) return FC_ERR_ALIGN;
    const SimLayout L = sim_layout(n_src, n, group, bits_rs, bits_ag);
    if (!workspace || workspace_bytes < L.total) return FC_ERR_WORKSPACE;
    if (!aligned16(workspace)) return FC_ERR_ALIGN;

    // the three steps in one kernel, bit-identical, nothing goes through the workspace: one form for launch-bound
    // volumes (asymmetric quantizer; the partials' quantizations spread over wavefronts), one for bandwidth-bound
    // volumes (every quantizer)
    if (one_launch) {
        if (codec == fc::CODEC_ASYM && fc::allreduce_small_applies(n, group))
            return hip_result(fc::launch_allreduce_small(bits_rs, bits_ag, x_f16, n_src, n, group, y_f16,
                                                         static_cast<hipStream_t>(hip_stream)));
        if (fc::allreduce_fused_applies(n, group))
            return hip_result(fc::launch_allreduce_fused(codec, bits_rs, bits_ag, x_f16, n_src, n, group, y_f16,
                                                         static_cast<hipStream_t>(hip_stream)));
    }

    char *ws = static_cast<char *>(workspace);
    const char *x = static_cast<const char *>(x_f16);
    // the N partials are N*tokens rows of one tensor; when the workspace slabs need no padding they
    // are quantized by one launch (what matters for launch-bound volumes), otherwise one by one
    const bool packed = L.codes_rs == (size_t)n * bits_rs / 8 && L.meta == (size_t)(n / group) * sizeof(float) &&
                        tokens <= kMaxElems / hidden / n_src;
    const int launches = packed ? 1 : n_src;
    for (int j = 0; j < launches; ++j) {
        const int q = quantize_impl(codec, x + (size_t)j * (size_t)n * 2, packed ? tokens * n_src : tokens, hidden,
                                    group, bits_rs, ws + L.off_codes1 + (size_t)j * L.codes_rs,
                                    reinterpret_cast<float *>(ws + L.off_scales1 + (size_t)j * L.meta),
                                    reinterpret_cast<float *>(ws + L.off_zeros1 + (size_t)j * L.meta),
                                    hip_stream);
        if (q != FC_OK) return q;
    }
    const int f = fused_impl(codec, ws + L.off_codes1, (int64_t)L.codes_rs,
                             reinterpret_cast<const float *>(ws + L.off_scales1),
                             reinterpret_cast<const float *>(ws + L.off_zeros1),
                             (int64_t)(L.meta / sizeof(float)), n_src, tokens, hidden, group, bits_rs,
                             bits_ag, ws + L.off_codes2, reinterpret_cast<float *>(ws + L.off_scales2),
                             reinterpret_cast<float *>(ws + L.off_zeros2), hip_stream);
    if (f != FC_OK) return f;
    return dequantize_impl(codec, ws + L.off_codes2, reinterpret_cast<const float *>(ws + L.off_scales2),
                           reinterpret_cast<const float *>(ws + L.off_zeros2), tokens, hidden, group,
                           bits_ag, y_f16, hip_stream);
}

// Device address of the current device's copy of `scratch`, looked up once per device.
int static_scratch(void **ptr)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_result(e);
    if (dev < 0 || dev >= kMaxDevices) return hip_result(hipErrorInvalidDevice);
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_result(e);
        if (!p) return hip_result(hipErrorInvalidSymbol);
        g_scratch_ptr[dev].store(p, std::memory_order_release);   // every thread finds the same address
    }
    *ptr = p;
    return FC_OK;
}

// the rotation runs over aligned blocks of the largest power of two dividing hidden
bool rot_hidden_ok(int64_t hidden)
{
    if (hidden <= 0 || hidden > 0x7FFFFFFF) return false;
    const int b = fc::rotation_block(hidden);
    return b == 1024 || b == 2048 || b == 4096 || b == 8192;
}

int check_quantizer(int quantizer, int bits)
{
    if (quantizer != fc::CODEC_ASYM && quantizer != fc::CODEC_SYM && quantizer != fc::CODEC_FP8) return FC_ERR_SHAPE;
    if (quantizer == fc::CODEC_FP8 && bits != 8) return FC_ERR_BITS;
    return FC_OK;
}

int quantize_rot_impl(int codec, const void *x_f16, int64_t tokens, int64_t hidden, int group, int bits,
                      void *codes, float *scales, float *zeros, void *hip_stream)
{
    const bool sym = codec != fc::CODEC_ASYM;
    int64_t n = 0;
    int rc = check_shape(tokens, hidden, group, bits, &n);
    if (rc != FC_OK) return rc;
    if ((rc = check_quantizer(codec, bits)) != FC_OK) return rc;
    if (!rot_hidden_ok(hidden) || tokens > 0x7FFFFFFF) return FC_ERR_SHAPE;
    if (n == 0) return FC_OK;
    if (!x_f16 || !codes || !scales || (!sym && !zeros)) return FC_ERR_NULL;
    if (!aligned16(x_f16) || !aligned16(codes) || !aligned16(scales) || (!sym && !aligned16(zeros)))
        return FC_ERR_ALIGN;
    return hip_result(fc::launch_quantize_rot(bits, codec, x_f16, tokens, (int)hidden, group, codes, scales,
                                              sym ? nullptr : zeros, static_cast<hipStream_t>(hip_stream)));
}

int dequantize_rot_impl(int codec, const void *codes, const float *scales, const float *zeros,
                        int64_t tokens, int64_t hidden, int group, int bits, void *y_f16, void *hip_stream)
{
    const bool sym = codec != fc::CODEC_ASYM;
    int64_t n = 0;
    int rc = check_shape(tokens, hidden, group, bits, &n);
    if (rc != FC_OK) return rc;
    if ((rc = check_quantizer(codec, bits)) != FC_OK) return rc;
    if (!rot_hidden_ok(hidden) || tokens > 0x7FFFFFFF) return FC_ERR_SHAPE;
    if (n == 0) return FC_OK;
    if (!codes || !scales || !y_f16 || (!sym && !zeros)) return FC_ERR_NULL;
    if (!aligned16(codes) || !aligned16(scales) || !aligned16(y_f16) || (!sym && !aligned16(zeros)))
        return FC_ERR_ALIGN;
    return hip_result(fc::launch_dequantize_rot(bits, codec, codes, scales, sym ? nullptr : zeros, tokens,
                                                (int)hidden, group, y_f16, static_cast<hipStream_t>(hip_stream)));
}

}  // namespace

extern "C" {

int fc_quantize(const void *x_f16, int64_t tokens, int64_t hidden, int group, int bits,
                void *codes, float *scales, float *zeros, void *hip_stream)
{
    return quantize_impl(fc::CODEC_ASYM, x_f16, tokens, hidden, group, bits, codes, scales, zeros, hip_stream);
}

int fc_quantize_sym(const void *x_f16, int64_t tokens, int64_t hidden, int group, int bits,
                    void *codes, float *scales, void *hip_stream)
{
    return quantize_impl(fc::CODEC_SYM, x_f16, tokens, hidden, group, bits, codes, scales, nullptr, hip_stream);
}

int fc_dequant_reduce_requant(const void *codes_in, int64_t codes_src_stride_bytes,
                              const float *scales_in, const float *zeros_in,
                              int64_t meta_src_stride_elems,
                              int n_src, int64_t tokens, int64_t hidden, int group,
                              int bits_in, int bits_out,
                              void *codes_out, float *scales_out, float *zeros_out,
                              void *hip_stream)
{
    return fused_impl(fc::CODEC_ASYM, codes_in, codes_src_stride_bytes, scales_in, zeros_in, meta_src_stride_elems,
                      n_src, tokens, hidden, group, bits_in, bits_out, codes_out, scales_out, zeros_out,
                      hip_stream);
}

int fc_dequant_reduce_requant_sym(const void *codes_in, int64_t codes_src_stride_bytes,
                                  const float *scales_in, int64_t meta_src_stride_elems,
                                  int n_src, int64_t tokens, int64_t hidden, int group,
                                  int bits_in, int bits_out,
                                  void *codes_out, float *scales_out, void *hip_stream)
{
    return fused_impl(fc::CODEC_SYM, codes_in, codes_src_stride_bytes, scales_in, nullptr, meta_src_stride_elems,
                      n_src, tokens, hidden, group, bits_in, bits_out, codes_out, scales_out, nullptr,
                      hip_stream);
}

int fc_dequantize(const void *codes, const float *scales, const float *zeros,
                  int64_t tokens, int64_t hidden, int group, int bits,
                  void *y_f16, void *hip_stream)
{
    return dequantize_impl(fc::CODEC_ASYM, codes, scales, zeros, tokens, hidden, group, bits, y_f16, hip_stream);
}

int fc_dequantize_sym(const void *codes, const float *scales,
                      int64_t tokens, int64_t hidden, int group, int bits,
                      void *y_f16, void *hip_stream)
{
    return dequantize_impl(fc::CODEC_SYM, codes, scales, nullptr, tokens, hidden, group, bits, y_f16, hip_stream);
}

size_t fc_allreduce_sim_workspace_bytes(int n_src, int64_t tokens, int64_t hidden, int group,
                                        int bits_rs, int bits_ag)
{
    int64_t n = 0;
    if (check_shape(tokens, hidden, group, bits_rs, &n) != FC_OK) return 0;
    if (bits_ag != 4 && bits_ag != 8) return 0;
    if (n_src < 1 || n_src > FC_MAX_SRC) return 0;
    return sim_layout(n_src, n, group, bits_rs, bits_ag).total;
}

int fc_allreduce_sim(const void *x_f16, int n_src, int64_t tokens, int64_t hidden,
                     int group, int bits_rs, int bits_ag, void *y_f16,
                     void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return allreduce_sim_impl(fc::CODEC_ASYM, x_f16, n_src, tokens, hidden, group, bits_rs, bits_ag, y_f16,
                              workspace, workspace_bytes, hip_stream);
}

int fc_allreduce_sim_static(const void *x_f16, int n_src, int64_t tokens, int64_t hidden,
                            int group, int bits_rs, int bits_ag, void *y_f16, void *hip_stream)
{
    int64_t n = 0;
    const int rc = check_shape(tokens, hidden, group, bits_rs, &n);
    if (rc != FC_OK) return rc;
    if (bits_ag != 4 && bits_ag != 8) return FC_ERR_BITS;
    if (n_src < 1 || n_src > FC_MAX_SRC) return FC_ERR_SHAPE;
    if (n == 0) return FC_OK;
    if (!x_f16 || !y_f16) return FC_ERR_NULL;
    if (!aligned16(x_f16) || !aligned16(y_f16)) return FC_ERR_ALIGN;
    if (sim_layout(n_src, n, group, bits_rs, bits_ag).total > (size_t)FC_STATIC_SCRATCH_BYTES)
        return FC_ERR_WORKSPACE;
    void *ws = nullptr;
    const int sc = static_scratch(&ws);
    if (sc != FC_OK) return sc;
    // nothing in the scratch has to start at zero: every byte a kernel reads there was written by
    // the kernel before it in this call
    // always the three-kernel sequence through the scratch array (the single-kernel forms need no intermediates
    // at all; fc_allreduce_sim takes them where they apply)
    return allreduce_sim_impl(fc::CODEC_ASYM, x_f16, n_src, tokens, hidden, group, bits_rs, bits_ag, y_f16,
                              ws, (size_t)FC_STATIC_SCRATCH_BYTES, hip_stream, false);
}

int fc_allreduce_sim_sym(const void *x_f16, int n_src, int64_t tokens, int64_t hidden,
                         int group, int bits_rs, int bits_ag, void *y_f16,
                         void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return allreduce_sim_impl(fc::CODEC_SYM, x_f16, n_src, tokens, hidden, group, bits_rs, bits_ag, y_f16,
                              workspace, workspace_bytes, hip_stream);
}

int fc_quantize_fp8(const void *x_f16, int64_t tokens, int64_t hidden, int group,
                    void *codes, float *scales, void *hip_stream)
{
    return quantize_impl(fc::CODEC_FP8, x_f16, tokens, hidden, group, 8, codes, scales, nullptr, hip_stream);
}

int fc_dequant_reduce_requant_fp8(const void *codes_in, int64_t codes_src_stride_bytes,
                                  const float *scales_in, int64_t meta_src_stride_elems,
                                  int n_src, int64_t tokens, int64_t hidden, int group,
                                  void *codes_out, float *scales_out, void *hip_stream)
{
    return fused_impl(fc::CODEC_FP8, codes_in, codes_src_stride_bytes, scales_in, nullptr,
                      meta_src_stride_elems, n_src, tokens, hidden, group, 8, 8, codes_out, scales_out,
                      nullptr, hip_stream);
}

int fc_dequantize_fp8(const void *codes, const float *scales, int64_t tokens, int64_t hidden, int group,
                      void *y_f16, void *hip_stream)
{
    return dequantize_impl(fc::CODEC_FP8, codes, scales, nullptr, tokens, hidden, group, 8, y_f16, hip_stream);
}

int fc_allreduce_sim_fp8(const void *x_f16, int n_src, int64_t tokens, int64_t hidden, int group,
                         void *y_f16, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return allreduce_sim_impl(fc::CODEC_FP8, x_f16, n_src, tokens, hidden, group, 8, 8, y_f16,
                              workspace, workspace_bytes, hip_stream);
}

int fc_quantize_cmeta(const void *x_f16, int64_t tokens, int64_t hidden, int group, int bits,
                      void *codes, uint32_t *meta, void *hip_stream)
{
    return quantize_impl(fc::CODEC_ASYMH, x_f16, tokens, hidden, group, bits, codes,
                         reinterpret_cast<float *>(meta), nullptr, hip_stream);
}

int fc_dequant_reduce_requant_cmeta(const void *codes_in, int64_t codes_src_stride_bytes,
                                    const uint32_t *meta_in, int64_t meta_src_stride_elems,
                                    int n_src, int64_t tokens, int64_t hidden, int group,
                                    int bits_in, int bits_out,
                                    void *codes_out, uint32_t *meta_out, void *hip_stream)
{
    return fused_impl(fc::CODEC_ASYMH, codes_in, codes_src_stride_bytes, reinterpret_cast<const float *>(meta_in),
                      nullptr, meta_src_stride_elems, n_src, tokens, hidden, group, bits_in, bits_out, codes_out,
                      reinterpret_cast<float *>(meta_out), nullptr, hip_stream);
}

int fc_dequantize_cmeta(const void *codes, const uint32_t *meta, int64_t tokens, int64_t hidden, int group,
                        int bits, void *y_f16, void *hip_stream)
{
    return dequantize_impl(fc::CODEC_ASYMH, codes, reinterpret_cast<const float *>(meta), nullptr, tokens, hidden,
                           group, bits, y_f16, hip_stream);
}

int fc_allreduce_sim_cmeta(const void *x_f16, int n_src, int64_t tokens, int64_t hidden,
                           int group, int bits_rs, int bits_ag, void *y_f16,
                           void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return allreduce_sim_impl(fc::CODEC_ASYMH, x_f16, n_src, tokens, hidden, group, bits_rs, bits_ag, y_f16,
                              workspace, workspace_bytes, hip_stream);
}

int fc_quantize_rot(const void *x_f16, int64_t tokens, int64_t hidden, int group, int bits,
                    int quantizer, void *codes, float *scales, float *zeros, void *hip_stream)
{
    return quantize_rot_impl(quantizer, x_f16, tokens, hidden, group, bits, codes, scales, zeros, hip_stream);
}

int fc_dequantize_rot(const void *codes, const float *scales, const float *zeros,
                      int64_t tokens, int64_t hidden, int group, int bits, int quantizer,
                      void *y_f16, void *hip_stream)
{
    return dequantize_rot_impl(quantizer, codes, scales, zeros, tokens, hidden, group, bits, y_f16, hip_stream);
}

int fc_allreduce_sim_rot(const void *x_f16, int n_src, int64_t tokens, int64_t hidden,
                         int group, int bits_rs, int bits_ag, int quantizer, void *y_f16,
                         void *workspace, size_t workspace_bytes, void *hip_stream)
{
    int64_t n = 0;
    int rc = check_shape(tokens, hidden, group, bits_rs, &n);
    if (rc != FC_OK) return rc;
    if (bits_ag != 4 && bits_ag != 8) return FC_ERR_BITS;
    if ((rc = check_quantizer(quantizer, bits_rs)) != FC_OK) return rc;
    if ((rc = check_quantizer(quantizer, bits_ag)) != FC_OK) return rc;
    if (n_src < 1 || n_src > FC_MAX_SRC || !rot_hidden_ok(hidden)) return FC_ERR_SHAPE;
    if (n == 0) return FC_OK;
    if (!x_f16 || !y_f16) return FC_ERR_NULL;
    if (!aligned16(x_f16) || !aligned16(y_f16)) return FC_ERR_ALIGN;
    const SimLayout L = sim_layout(n_src, n, group, bits_rs, bits_ag);
    if (!workspace || workspace_bytes < L.total) return FC_ERR_WORKSPACE;
    if (!aligned16(workspace)) return FC_ERR_ALIGN;

    char *ws = static_cast<char *>(workspace);
    const char *x = static_cast<const char *>(x_f16);
    const bool packed = L.codes_rs == (size_t)n * bits_rs / 8 && L.meta == (size_t)(n / group) * sizeof(float) &&
                        tokens * n_src <= 0x7FFFFFFF;
    const int launches = packed ? 1 : n_src;
    for (int j = 0; j < launches; ++j) {
        rc = quantize_rot_impl(quantizer, x + (size_t)j * (size_t)n * 2, packed ? tokens * n_src : tokens, hidden,
                               group, bits_rs,
                               ws + L.off_codes1 + (size_t)j * L.codes_rs,
                               reinterpret_cast<float *>(ws + L.off_scales1 + (size_t)j * L.meta),
                               reinterpret_cast<float *>(ws + L.off_zeros1 + (size_t)j * L.meta), hip_stream);
        if (rc != FC_OK) return rc;
    }
    rc = fused_impl(quantizer, ws + L.off_codes1, (int64_t)L.codes_rs,
                    reinterpret_cast<const float *>(ws + L.off_scales1),
                    reinterpret_cast<const float *>(ws + L.off_zeros1), (int64_t)(L.meta / sizeof(float)),
                    n_src, tokens, hidden, group, bits_rs, bits_ag, ws + L.off_codes2,
                    reinterpret_cast<float *>(ws + L.off_scales2), reinterpret_cast<float *>(ws + L.off_zeros2),
                    hip_stream);
    if (rc != FC_OK) return rc;
    return dequantize_rot_impl(quantizer, ws + L.off_codes2, reinterpret_cast<const float *>(ws + L.off_scales2),
                               reinterpret_cast<const float *>(ws + L.off_zeros2), tokens, hidden, group,
                               bits_ag, y_f16, hip_stream);
}

const char *fc_strerror(int code)
{
    switch (code) {
    case FC_OK: return "success";
    case FC_ERR_NULL: return "a required pointer is NULL";
    case FC_ERR_BITS: return "bit-width must be 4 or 8";
    case FC_ERR_GROUP: return "group must be a power of two in [32, 16384] that divides hidden";
    case FC_ERR_SHAPE: return "bad tokens / hidden / n_src / source stride";
    case FC_ERR_ALIGN: return "pointers and strides must be 16-byte aligned";
    case FC_ERR_WORKSPACE: return "workspace missing or too small (or volume beyond the static scratch)";
    case FC_ERR_HIP: return "HIP launch failed (see fc_last_hip_error)";
    default: return "unknown error code";
    }
}

int fc_last_hip_error(void) { return g_last_hip_error; }

int fc_version(void) { return 100; }

}  // extern "C"
