// C ABI of libfp4mr.so: argument validation on the host, then dispatch to the kernel launchers.
// Nothing here allocates, frees or keeps device memory.
#include "../../include/fp4mr.h"

#include <cstdlib>
#include <cstring>
#include <mutex>

#include "internal.hpp"
#include "layout.hpp"

using namespace fp4mr;

// Scratch of fp4_rotate_quantize_static: the abs-max partials and the reduced abs-max of the NVFP4 tensor-scale pass
// (what fp4_rotate_quantize takes as its workspace).  One copy per GPU, held until the process ends.  Host code never
// uses this name as an address: static_scratch() asks the runtime for the array's device address once per device.
constexpr size_t kStaticScratchBytes = 256 + 4096 * 4;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
static_assert(kStaticScratchBytes == FP4MR_STATIC_SCRATCH_BYTES, "the header states the size of the static scratch");

namespace {

constexpr uint32_t kQuantFlags = FP4MR_LAYOUT_GEMM | FP4MR_INPUT_F32 | FP4MR_STATIC_TENSOR_SCALE | FP4MR_SCALE_MSE | FP4MR_SCALE_ROUND43 | FP4MR_SCALE_FIT_TENSOR |
                                 FP4MR_SCALE_FIT_RANGE;
constexpr uint32_t kGemmFlags = FP4MR_A_LAYOUT_GEMM | FP4MR_W_LAYOUT_GEMM | FP4MR_OUT_F32 | FP4MR_A_SCALE43 | FP4MR_W_SCALE43;

// result factor for operands whose scales carry the tensor-level 4/3 (FP4MR_SCALE_ROUND43)
float scale43_factor(uint32_t flags)
{
    float f = 1.0f;
    if (flags & FP4MR_A_SCALE43) f *= 4.0f / 3.0f;
    if (flags & FP4MR_W_SCALE43) f *= 4.0f / 3.0f;
    return f;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }

int group_of(fp4mr_fmt_t fmt) { return fmt == FP4MR_MXFP4 ? 32 : 16; }

size_t quant_workspace(fp4mr_fmt_t fmt, uint32_t flags)
{
    // 256 bytes for the tensor abs-max plus one 4-byte partial per wave of the abs-max pass (1024 blocks x 4 waves)
    // (+ two fp64 sums per wave of the tensor-scale fit pass with FP4MR_SCALE_FIT_TENSOR)
    // (the range pre-pass of FP4MR_SCALE_FIT_RANGE: two 4-byte extremes per wave of 512 blocks x 4 waves, the same size)
    if (flags & FP4MR_STATIC_TENSOR_SCALE) return 0;
    if (fmt != FP4MR_NVFP4) return (flags & FP4MR_SCALE_FIT_RANGE) ? 256 + 4096 * 4 : 0;
    return 256 + 4096 * 4 + ((flags & FP4MR_SCALE_FIT_TENSOR) ? 4096 * 16 : 0);
}

size_t repack_bytes(int64_t rows, int64_t K, fp4mr_fmt_t fmt)
{
    return align256((size_t)gemm_codes_bytes(rows, K)) + align256((size_t)gemm_scales_bytes(rows, K, (int)fmt));
}

fp4mr_status_t static_scratch(void** out)
{
    static std::mutex mu;
    static void* ptr[64] = {};  // per device: each GPU holds its own copy of the array at its own address
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return FP4MR_ERR_DEVICE;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return FP4MR_ERR_DEVICE;
        ptr[dev] = p;
    }
    *out = ptr[dev];
    return FP4MR_OK;
}

fp4mr_status_t quantize_common(const void* x, int64_t rows, int64_t K, int had_block, const void* rot, fp4mr_fmt_t fmt,
                               void* codes, void* scales, float* tensor_scale, void* workspace, size_t workspace_bytes,
                               uint32_t flags, void* stream, bool library_scratch = false)
{
    if (fmt != FP4MR_MXFP4 && fmt != FP4MR_NVFP4) return FP4MR_ERR_FMT;
    if (flags & ~kQuantFlags) return FP4MR_ERR_FMT;
    if ((flags & FP4MR_SCALE_ROUND43) && (fmt != FP4MR_MXFP4 || (flags & FP4MR_SCALE_MSE))) return FP4MR_ERR_FMT;
    // the tensor-scale fit is the NVFP4 squared-error search plus a fitted (hence not caller-supplied) tensor scale
    if ((flags & FP4MR_SCALE_FIT_TENSOR) && (fmt != FP4MR_NVFP4 || !(flags & FP4MR_SCALE_MSE) || (flags & FP4MR_STATIC_TENSOR_SCALE))) return FP4MR_ERR_FMT;
    // the fitted scale range is a format of its own: MXFP4 groups, no other scale policy beside it
    if ((flags & FP4MR_SCALE_FIT_RANGE) && (fmt != FP4MR_MXFP4 || (flags & (FP4MR_SCALE_MSE | FP4MR_SCALE_ROUND43 | FP4MR_SCALE_FIT_TENSOR)))) return FP4MR_ERR_FMT;
    if (!x || !codes || !scales) return FP4MR_ERR_NULL;
    if ((fmt == FP4MR_NVFP4 || (flags & FP4MR_SCALE_FIT_RANGE)) && !tensor_scale) return FP4MR_ERR_NULL;
    if (had_block != 1 && had_block != 16 && had_block != 32 && had_block != 64 && had_block != 128) return FP4MR_ERR_HAD_BLOCK;
    if ((flags & FP4MR_INPUT_F32) && had_block != 1) return FP4MR_ERR_HAD_BLOCK;
    if (rot && (had_block == 1 || !aligned16(rot))) return had_block == 1 ? FP4MR_ERR_HAD_BLOCK : FP4MR_ERR_ALIGN;
    if (rows <= 0 || K <= 0) return FP4MR_ERR_SHAPE;
    const int G = group_of(fmt);
    const int lcm = had_block > G ? had_block : G;  // both are powers of two
    if (K % lcm != 0) return FP4MR_ERR_SHAPE;
    if ((flags & FP4MR_LAYOUT_GEMM) && K % 128 != 0) return FP4MR_ERR_SHAPE;
    if (rows > ((int64_t)1 << 40) / K) return FP4MR_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(codes) || !aligned16(scales)) return FP4MR_ERR_ALIGN;
    const size_t need = quant_workspace(fmt, flags);
    if (library_scratch) {
        // the allocation-free entry point: its scratch is the library's own device array (looked up after validation)
        if (need > kStaticScratchBytes) return FP4MR_ERR_WORKSPACE;
        if (need) {
            const fp4mr_status_t s = static_scratch(&workspace);
            if (s != FP4MR_OK) return s;
        }
    } else if (need && (!workspace || workspace_bytes < need || !aligned16(workspace))) {
        return FP4MR_ERR_WORKSPACE;
    }

    const hipError_t e = launch_rotate_quantize(x, rows, K, had_block, rot, (int)fmt, (flags & FP4MR_INPUT_F32) != 0,
                                                (flags & FP4MR_LAYOUT_GEMM) ? 1 : 0, (flags & FP4MR_STATIC_TENSOR_SCALE) != 0,
                                                (flags & FP4MR_SCALE_FIT_RANGE) ? 4 : (flags & FP4MR_SCALE_FIT_TENSOR) ? 3 : ((flags & FP4MR_SCALE_MSE) ? 1 : ((flags & FP4MR_SCALE_ROUND43) ? 2 : 0)), codes, scales, tensor_scale,
                                                workspace, options().sw_codec == 0,
                                                static_cast<hipStream_t>(stream));
    return e == hipSuccess ? FP4MR_OK : FP4MR_ERR_DEVICE;
}


// shared by fp4_fused_linear (activations quantized) and fp4_w4a16_linear (activations kept in bf16)
fp4mr_status_t few_token_linear(const void* x, int64_t M, int64_t K, int had_block, const void* w_codes, const void* w_scales,
                                int64_t N, fp4mr_fmt_t fmt, void* out, uint32_t flags, void* stream, bool weight_only)
{
    if (fmt != FP4MR_MXFP4) return FP4MR_ERR_FMT;  // NVFP4 needs the tensor abs-max first: not a one-pass operation
    if (flags & ~(uint32_t)(FP4MR_OUT_F32 | FP4MR_W_LAYOUT_GEMM | FP4MR_W_SCALE43)) return FP4MR_ERR_FMT;
    if (!(flags & FP4MR_W_LAYOUT_GEMM)) return FP4MR_ERR_FMT;
    if (!x || !w_codes || !w_scales || !out) return FP4MR_ERR_NULL;
    if (had_block != 16 && had_block != 32 && had_block != 64 && had_block != 128) return FP4MR_ERR_HAD_BLOCK;
    // the quantizing variant repeats the quantization per workgroup: beyond four tokens the two-call path is faster
    if (M <= 0 || M > (weight_only ? 16 : 4) || N <= 0 || K <= 0 || K % 128 != 0 || N > (1 << 24) || K > (1 << 24)) return FP4MR_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(w_codes) || !aligned16(w_scales) || !aligned16(out)) return FP4MR_ERR_ALIGN;
    const hipError_t e = launch_fused_decode(x, M, K, had_block, w_codes, w_scales, N, out, (flags & FP4MR_OUT_F32) != 0,
                                             weight_only, scale43_factor(flags), static_cast<hipStream_t>(stream));
    return e == hipSuccess ? FP4MR_OK : FP4MR_ERR_DEVICE;
}

}  // namespace

namespace fp4mr {
Options& options()
{
    static Options o;
    return o;
}
}  // namespace fp4mr

extern "C" {

fp4mr_status_t fp4_set_option(int option, int value)
{
    Options& o = options();
    switch (option) {
        case FP4MR_OPT_GEMM_VARIANT:
            if (value < 0 || value > kMaxGemmVariantMx) return FP4MR_ERR_FMT;
            o.gemm_variant = value;
            return FP4MR_OK;
        case FP4MR_OPT_GEMM_GRID:
            if (value < 0) return FP4MR_ERR_FMT;
            o.gemm_grid = value;
            return FP4MR_OK;
        case FP4MR_OPT_SW_CODEC:
            o.sw_codec = value != 0;
            return FP4MR_OK;
        default: return FP4MR_ERR_FMT;
    }
}

fp4mr_status_t fp4_rotate_quantize(const void* x, int64_t M, int64_t K, int had_block, fp4mr_fmt_t fmt, void* codes_out,
                                   void* scales_out, float* tensor_scale, void* workspace, size_t workspace_bytes,
                                   uint32_t flags, void* stream)
{
    return quantize_common(x, M, K, had_block, nullptr, fmt, codes_out, scales_out, tensor_scale, workspace, workspace_bytes, flags, stream);
}

fp4mr_status_t fp4_rotate_quantize_static(const void* x, int64_t M, int64_t K, int had_block, fp4mr_fmt_t fmt, void* codes_out,
                                          void* scales_out, float* tensor_scale, uint32_t flags, void* stream)
{
    if (M > 0 && K > 0 && M > (int64_t)FP4MR_STATIC_MAX_ELEMENTS / K) return FP4MR_ERR_SHAPE;
    return quantize_common(x, M, K, had_block, nullptr, fmt, codes_out, scales_out, tensor_scale, nullptr, 0, flags, stream, true);
}

fp4mr_status_t fp4_rotate_quantize_dense(const void* x, int64_t M, int64_t K, int block, const void* rot_bf16, fp4mr_fmt_t fmt,
                                         void* codes_out, void* scales_out, float* tensor_scale, void* workspace,
                                         size_t workspace_bytes, uint32_t flags, void* stream)
{
    if (!rot_bf16) return FP4MR_ERR_NULL;
    return quantize_common(x, M, K, block, rot_bf16, fmt, codes_out, scales_out, tensor_scale, workspace, workspace_bytes, flags, stream);
}

fp4mr_status_t fp4_quantize_weights(const void* w, int64_t N, int64_t K, int had_block, fp4mr_fmt_t fmt, void* codes_out,
                                    void* scales_out, float* tensor_scale, void* workspace, size_t workspace_bytes,
                                    uint32_t flags, void* stream)
{
    return quantize_common(w, N, K, had_block, nullptr, fmt, codes_out, scales_out, tensor_scale, workspace, workspace_bytes, flags, stream);
}

fp4mr_status_t fp4_gemm(const void* a_codes, const void* a_scales, const float* a_tensor_scale, const void* w_codes,
                        const void* w_scales, const float* w_tensor_scale, int64_t M, int64_t N, int64_t K,
                        fp4mr_fmt_t fmt, void* out, void* workspace, size_t workspace_bytes, uint32_t flags, void* stream)
{
    if (fmt != FP4MR_MXFP4 && fmt != FP4MR_NVFP4) return FP4MR_ERR_FMT;
    if (flags & ~kGemmFlags) return FP4MR_ERR_FMT;
    if (!a_codes || !a_scales || !w_codes || !w_scales || !out) return FP4MR_ERR_NULL;
    if (fmt == FP4MR_NVFP4 && (!a_tensor_scale || !w_tensor_scale)) return FP4MR_ERR_NULL;
    if (fmt == FP4MR_NVFP4 && (flags & (FP4MR_A_SCALE43 | FP4MR_W_SCALE43))) return FP4MR_ERR_FMT;
    if (M <= 0 || N <= 0 || K <= 0 || K % 128 != 0) return FP4MR_ERR_SHAPE;
    if (M > (1 << 24) || N > (1 << 24) || K > (1 << 24)) return FP4MR_ERR_SHAPE;
    if (!aligned16(a_codes) || !aligned16(a_scales) || !aligned16(w_codes) || !aligned16(w_scales) || !aligned16(out)) return FP4MR_ERR_ALIGN;
    const size_t need = fp4_workspace_bytes(FP4MR_OP_GEMM, M, N, K, fmt, flags);
    if (need && (!workspace || workspace_bytes < need || !aligned16(workspace))) return FP4MR_ERR_WORKSPACE;
    const int variant = options().gemm_variant;
    if (variant < 0 || variant > (fmt == FP4MR_MXFP4 ? kMaxGemmVariantMx : kMaxGemmVariantNv)) return FP4MR_ERR_FMT;

    hipStream_t st = static_cast<hipStream_t>(stream);
    char* ws = static_cast<char*>(workspace);
    hipError_t e;
    if (!(flags & FP4MR_A_LAYOUT_GEMM)) {
        void* c = ws;
        void* s = ws + align256((size_t)gemm_codes_bytes(M, K));
        if ((e = launch_repack_to_gemm(a_codes, a_scales, M, K, (int)fmt, c, s, st)) != hipSuccess) return FP4MR_ERR_DEVICE;
        a_codes = c;
        a_scales = s;
        ws += repack_bytes(M, K, fmt);
    }
    if (!(flags & FP4MR_W_LAYOUT_GEMM)) {
        void* c = ws;
        void* s = ws + align256((size_t)gemm_codes_bytes(N, K));
        if ((e = launch_repack_to_gemm(w_codes, w_scales, N, K, (int)fmt, c, s, st)) != hipSuccess) return FP4MR_ERR_DEVICE;
        w_codes = c;
        w_scales = s;
        ws += repack_bytes(N, K, fmt);
    }
    const bool out_f32 = (flags & FP4MR_OUT_F32) != 0;
    const float alpha = scale43_factor(flags);
    // Few tokens: the weight-streaming kernels, except MXFP4 with more than two 16-token blocks on a very wide layer with
    // K > 4096, where the 64 x 256 tile kernel's time hardly grows with the token count and the streaming kernels' does
    // (N = 57344, K = 14336, M = 48: 87 us against 113; K = 6144, M = 64: 39 against 45; below N = 40960 the streaming
    // kernels win at every token count: N = 28672, K = 8192, M = 64: 27.7 us against 38.4).
    const bool wide_mx = fmt == FP4MR_MXFP4 && M > 32 && N >= 40960 && K > 4096;
    // Optional split-K room behind what the call needs (FP4MR_OP_GEMM_SPLIT_K): used when the caller passed that much
    void* partial = nullptr;
    const bool few = variant == 0 && !wide_mx && gemm_skinny_takes(M, N, K, (int)fmt);
    if (M > 64 && variant == 0 && !few) {
        const size_t extra = fmt == FP4MR_MXFP4 ? gemm_mx_split_k_bytes(M, N, K) : nv16_split_k_bytes(M, N, K);
        if (extra && workspace && aligned16(workspace) && workspace_bytes >= align256(need) + extra) partial = static_cast<char*>(workspace) + align256(need);
    }
    if (few)
        e = launch_gemm_skinny(a_codes, a_scales, a_tensor_scale, w_codes, w_scales, w_tensor_scale, M, N, K, (int)fmt, out, out_f32, alpha, st);
    else if (fmt == FP4MR_MXFP4)
        e = launch_gemm_mxfp4(a_codes, a_scales, w_codes, w_scales, M, N, K, out, out_f32, variant, alpha, partial, st);
    else
        e = launch_gemm_nvfp4(a_codes, a_scales, a_tensor_scale, w_codes, w_scales, w_tensor_scale, M, N, K, out, out_f32, variant, ws, partial, st);
    return e == hipSuccess ? FP4MR_OK : FP4MR_ERR_DEVICE;
}

fp4mr_status_t fp4_gptq_quantize_weights(const void* w, int64_t N, int64_t K, int had_block, fp4mr_fmt_t fmt,
                                         const float* hinv_u, const int32_t* perm, void* codes_out, void* scales_out,
                                         float* tensor_scale, void* workspace, size_t workspace_bytes, uint32_t flags,
                                         void* stream)
{
    if (fmt != FP4MR_MXFP4 && fmt != FP4MR_NVFP4) return FP4MR_ERR_FMT;
    if (flags & ~(uint32_t)(FP4MR_SCALE_MSE | FP4MR_SCALE_ROUND43 | FP4MR_SCALE_FIT_TENSOR | FP4MR_SCALE_FIT_RANGE)) return FP4MR_ERR_FMT;
    if (!hinv_u) return FP4MR_ERR_NULL;
    if (N > (1 << 24) || K <= 0 || K % 64 != 0 || K > 24576) return FP4MR_ERR_SHAPE;
    if (!aligned16(hinv_u) || (perm && !aligned16(perm))) return FP4MR_ERR_ALIGN;
    const size_t need = fp4_workspace_bytes(FP4MR_OP_GPTQ, N, 0, K, fmt, flags);
    if (!workspace || workspace_bytes < need || !aligned16(workspace)) return FP4MR_ERR_WORKSPACE;
    // 1. the grid: scales (and the NVFP4 tensor scale) of the rotated weights in their original order; the codes this
    //    writes are the round-to-nearest ones, replaced below
    const size_t qws = align256(quant_workspace(fmt, flags));
    const fp4mr_status_t s = quantize_common(w, N, K, had_block, nullptr, fmt, codes_out, scales_out, tensor_scale, workspace, qws, flags, stream);
    if (s != FP4MR_OK) return s;
    // 2. the sweep
    const hipError_t e = launch_gptq_sweep(w, N, K, had_block, (int)fmt, hinv_u, reinterpret_cast<const int*>(perm), scales_out,
                                           fmt == FP4MR_NVFP4 ? tensor_scale : nullptr,
                                           (flags & FP4MR_SCALE_FIT_RANGE) ? tensor_scale + 2 : nullptr,  // the scale values just published
                                           (flags & FP4MR_SCALE_ROUND43) ? 4.0f / 3.0f : 1.0f, codes_out,
                                           static_cast<char*>(workspace) + qws, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? FP4MR_OK : FP4MR_ERR_DEVICE;
}

fp4mr_status_t fp4_gptq_accumulate_hessian(const void* x, int64_t T, int64_t K, int had_block, float* hessian, int accumulate,
                                           void* workspace, size_t workspace_bytes, void* stream)
{
    if (!x || !hessian) return FP4MR_ERR_NULL;
    if (had_block != 1 && had_block != 16 && had_block != 32 && had_block != 64 && had_block != 128) return FP4MR_ERR_HAD_BLOCK;
    if (T <= 0 || T > (1 << 24) || K <= 0 || K > 24576 || K % had_block != 0 || K % 2 != 0) return FP4MR_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(hessian)) return FP4MR_ERR_ALIGN;
    const size_t need = align256((size_t)T * K * 4);
    if (!workspace || workspace_bytes < need || !aligned16(workspace)) return FP4MR_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    float* xr = static_cast<float*>(workspace);
    if (launch_gptq_rotate_rows(x, T, K, had_block, xr, st) != hipSuccess) return FP4MR_ERR_DEVICE;
    return launch_gptq_hessian_product(xr, T, K, hessian, accumulate != 0, st) == hipSuccess ? FP4MR_OK : FP4MR_ERR_DEVICE;
}

fp4mr_status_t fp4_gptq_prepare(const float* hessian, int64_t K, float damp, int act_order, int32_t* perm_out, float* hinv_u_out,
                                void* workspace, size_t workspace_bytes, void* stream)
{
    if (!hessian || !perm_out || !hinv_u_out) return FP4MR_ERR_NULL;
    if (K <= 0 || K > 24576 || !(damp >= 0.0f)) return FP4MR_ERR_SHAPE;
    if (!aligned16(hessian) || !aligned16(perm_out) || !aligned16(hinv_u_out)) return FP4MR_ERR_ALIGN;
    const size_t need = gptq_prepare_workspace_bytes(K);
    if (!workspace || workspace_bytes < need || !aligned16(workspace)) return FP4MR_ERR_WORKSPACE;
    const hipError_t e = launch_gptq_prepare(hessian, K, damp, act_order != 0, reinterpret_cast<int*>(perm_out), hinv_u_out, workspace,
                                             static_cast<hipStream_t>(stream));
    return e == hipSuccess ? FP4MR_OK : FP4MR_ERR_DEVICE;
}

fp4mr_status_t fp4_fused_linear(const void* x, int64_t M, int64_t K, int had_block, const void* w_codes, const void* w_scales,
                                int64_t N, fp4mr_fmt_t fmt, void* out, uint32_t flags, void* stream)
{
    return few_token_linear(x, M, K, had_block, w_codes, w_scales, N, fmt, out, flags, stream, false);
}

fp4mr_status_t fp4_w4a16_linear(const void* x, int64_t M, int64_t K, int had_block, const void* w_codes, const void* w_scales,
                                int64_t N, fp4mr_fmt_t fmt, void* out, uint32_t flags, void* stream)
{
    return few_token_linear(x, M, K, had_block, w_codes, w_scales, N, fmt, out, flags, stream, true);
}

fp4mr_status_t fp4_probe(int which, void* buf, size_t bytes, int iters, void* stream)
{
    if (!buf) return FP4MR_ERR_NULL;
    if (!aligned16(buf)) return FP4MR_ERR_ALIGN;
    if (which < FP4MR_PROBE_MFMA_FP4 || which > FP4MR_PROBE_READ) return FP4MR_ERR_SHAPE;
    if ((which <= FP4MR_PROBE_MFMA_F16 && iters < 1) || bytes < 32) return FP4MR_ERR_SHAPE;
    const hipError_t e = launch_probe(which, buf, bytes, iters, static_cast<hipStream_t>(stream));
    if (e == hipErrorInvalidValue) return FP4MR_ERR_SHAPE;  // buffer smaller than one record per compute unit
    return e == hipSuccess ? FP4MR_OK : FP4MR_ERR_DEVICE;
}

size_t fp4_workspace_bytes(int op, int64_t M, int64_t N, int64_t K, fp4mr_fmt_t fmt, uint32_t flags)
{
    if (fmt != FP4MR_MXFP4 && fmt != FP4MR_NVFP4) return 0;
    if (op == FP4MR_OP_ROTATE_QUANTIZE || op == FP4MR_OP_QUANTIZE_WEIGHTS) return quant_workspace(fmt, flags);
    if (op == FP4MR_OP_GPTQ_HESSIAN) return (M > 0 && K > 0) ? align256((size_t)M * K * 4) : 0;
    if (op == FP4MR_OP_GPTQ_PREPARE) return K > 0 ? gptq_prepare_workspace_bytes(K) : 0;
    if (op == FP4MR_OP_GPTQ) return (M > 0 && K > 0) ? align256(quant_workspace(fmt, flags)) + gptq_workspace_bytes(M, K) : 0;
    if (op == FP4MR_OP_GEMM || op == FP4MR_OP_GEMM_SPLIT_K) {
        if (M <= 0 || N <= 0 || K <= 0 || K % 128 != 0) return 0;
        size_t n = 0;
        if (!(flags & FP4MR_A_LAYOUT_GEMM)) n += repack_bytes(M, K, fmt);
        if (!(flags & FP4MR_W_LAYOUT_GEMM)) n += repack_bytes(N, K, fmt);
        // NVFP4 with more than 64 tokens: the activations are dequantized once to fp16 (2 bytes per element)
        if (fmt == FP4MR_NVFP4 && M > 64 && !gemm_skinny_takes(M, N, K, (int)fmt)) n += align256(nv16_workspace_bytes(M, K));
        // what fp4_gemm needs, plus -- optional -- the fp32 partials of a split-K run where the shape has one
        if (op == FP4MR_OP_GEMM_SPLIT_K && M > 64 && !gemm_skinny_takes(M, N, K, (int)fmt)) {
            const size_t extra = fmt == FP4MR_MXFP4 ? gemm_mx_split_k_bytes(M, N, K) : nv16_split_k_bytes(M, N, K);
            if (extra) n = align256(n) + extra;
        }
        return n;
    }
    return 0;
}

fp4mr_status_t fp4_dequantize(const void* codes, const void* scales, const float* tensor_scale, int64_t rows, int64_t K,
                              fp4mr_fmt_t fmt, void* out, uint32_t flags, void* stream)
{
    if (fmt != FP4MR_MXFP4 && fmt != FP4MR_NVFP4) return FP4MR_ERR_FMT;
    if (flags & ~(uint32_t)(FP4MR_LAYOUT_GEMM | FP4MR_OUT_F32 | FP4MR_SCALE_ROUND43 | FP4MR_SCALE_FIT_RANGE)) return FP4MR_ERR_FMT;
    if ((flags & (FP4MR_SCALE_ROUND43 | FP4MR_SCALE_FIT_RANGE)) && fmt != FP4MR_MXFP4) return FP4MR_ERR_FMT;
    if ((flags & FP4MR_SCALE_ROUND43) && (flags & FP4MR_SCALE_FIT_RANGE)) return FP4MR_ERR_FMT;
    if (!codes || !scales || !out) return FP4MR_ERR_NULL;
    if ((fmt == FP4MR_NVFP4 || (flags & FP4MR_SCALE_FIT_RANGE)) && !tensor_scale) return FP4MR_ERR_NULL;
    if (rows <= 0 || K <= 0 || K % group_of(fmt) != 0) return FP4MR_ERR_SHAPE;
    if ((flags & FP4MR_LAYOUT_GEMM) && K % 128 != 0) return FP4MR_ERR_SHAPE;
    if (rows > ((int64_t)1 << 40) / K) return FP4MR_ERR_SHAPE;
    if (!aligned16(codes) || !aligned16(scales) || !aligned16(out)) return FP4MR_ERR_ALIGN;
    const int mode = fmt == FP4MR_NVFP4 ? 2 : ((flags & FP4MR_SCALE_FIT_RANGE) ? 3 : ((flags & FP4MR_SCALE_ROUND43) ? 1 : 0));
    const hipError_t e = launch_dequantize(codes, scales, tensor_scale, rows, K, mode, (flags & FP4MR_LAYOUT_GEMM) != 0, out,
                                           (flags & FP4MR_OUT_F32) != 0, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? FP4MR_OK : FP4MR_ERR_DEVICE;
}

fp4mr_status_t fp4_packed_bytes(int64_t rows, int64_t K, fp4mr_fmt_t fmt, uint32_t flags, size_t* codes_bytes, size_t* scales_bytes)
{
    if (fmt != FP4MR_MXFP4 && fmt != FP4MR_NVFP4) return FP4MR_ERR_FMT;
    if (!codes_bytes || !scales_bytes) return FP4MR_ERR_NULL;
    const int G = group_of(fmt);
    if (rows <= 0 || K <= 0 || K % G != 0) return FP4MR_ERR_SHAPE;
    if (flags & FP4MR_LAYOUT_GEMM) {
        if (K % 128 != 0) return FP4MR_ERR_SHAPE;
        *codes_bytes = (size_t)gemm_codes_bytes(rows, K);
        *scales_bytes = (size_t)gemm_scales_bytes(rows, K, (int)fmt);
    } else {
        *codes_bytes = (size_t)(rows * K / 2);
        *scales_bytes = (size_t)(rows * K / G);
    }
    return FP4MR_OK;
}

const char* fp4_status_string(fp4mr_status_t s)
{
    switch (s) {
        case FP4MR_OK: return "ok";
        case FP4MR_ERR_NULL: return "a required pointer is NULL";
        case FP4MR_ERR_SHAPE: return "bad shape: sizes must be positive and K a multiple of the group, the Hadamard block and (GEMM layout) 128; fp4_fused_linear takes 1..4 tokens (beyond: fp4_rotate_quantize + fp4_gemm), fp4_w4a16_linear 1..16";
        case FP4MR_ERR_HAD_BLOCK: return "had_block must be 1, 16, 32, 64 or 128 (1 with fp32 input)";
        case FP4MR_ERR_FMT: return "unknown format, flag bits or option value";
        case FP4MR_ERR_ALIGN: return "pointers must be 16-byte aligned";
        case FP4MR_ERR_WORKSPACE: return "workspace missing, misaligned or smaller than fp4_workspace_bytes()";
        case FP4MR_ERR_DEVICE: return "HIP runtime error at launch";
    }
    return "unknown status";
}

int fp4_version(void) { return 100; }

}  // extern "C"
