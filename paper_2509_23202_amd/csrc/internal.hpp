// Host-side launchers behind the C ABI (one per kernel family).  All pointers are device pointers that the
// C-ABI layer has already validated.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

namespace fp4mr {

// Process-wide tuning / cross-check switches behind fp4_set_option (plain ints: set them before concurrent use).
struct Options {
    int gemm_variant = 0;  // 0 = tile shape by the cost model, else a forced tile configuration of the GEMM kernels
    int gemm_grid = 0;     // > 0: cap on the number of persistent workgroups (a small grid walks many tiles each)
    int sw_codec = 0;      // != 0: element and scale codecs in integer arithmetic instead of the converting instructions
};
Options& options();

// Raises a kernel's dynamic-LDS limit the first time the kernel is launched on a device (one object per kernel).
struct LdsAttrOnce {
    std::atomic<uint64_t> done{0};  // bit d: set on device d
    hipError_t ensure(const void* kernel, int lds_bytes)
    {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = 63;  // (unknown device: set it every time)
        const uint64_t bit = 1ull << dev;
        if (dev != 63 && (done.load(std::memory_order_relaxed) & bit)) return hipSuccess;
        const hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e == hipSuccess) done.fetch_or(bit, std::memory_order_relaxed);
        return e;
    }
};

// compute units of the current device (cached per device)
int compute_units();

// largest valid forced tile configuration per format (fp4_gemm rejects anything else before it launches)
constexpr int kMaxGemmVariantMx = 18;
constexpr int kMaxGemmVariantNv = 3;

// policy: group scales by 0 abs-max, 1 squared-error search, 2 rounded exponent with the 4/3 factor (MXFP4 only).
// rot: null for the normalised Hadamard of size b, else a bf16 [b, b] row-major matrix (y = x . rot per block)
hipError_t launch_rotate_quantize(const void* x, int64_t rows, int64_t K, int b, const void* rot, int fmt, bool in_f32,
                                  int layout_gemm, bool static_scale, int policy, void* codes, void* scales,
                                  float* tensor_scale, void* workspace, bool hw_codec, hipStream_t st);

// canonical -> GEMM layout copy of one quantized operand (codes and scales)
hipError_t launch_repack_to_gemm(const void* codes, const void* scales, int64_t rows, int64_t K, int fmt,
                                 void* codes_gemm, void* scales_gemm, hipStream_t st);

// both operands in GEMM layout; alpha multiplies the result (1, or powers of 4/3 for operands quantized with the
// rounded-exponent rule whose scale bytes leave that tensor-level factor out)
hipError_t launch_gemm_mxfp4(const void* a_codes, const void* a_scales, const void* w_codes, const void* w_scales,
                             int64_t M, int64_t N, int64_t K, void* out, bool out_f32, int variant, float alpha, void* partial,
                             hipStream_t st);
// fp32 partials of a split-K run (few tiles, long K: every tile's K range shared by several workgroups); 0 = not split
size_t gemm_mx_split_k_bytes(int64_t M, int64_t N, int64_t K);

// variant 0: the fp16-activation kernel below (needs its workspace); 1..3: the tile kernels that dequantize both operands
hipError_t launch_gemm_nvfp4(const void* a_codes, const void* a_scales, const float* a_ts, const void* w_codes,
                             const void* w_scales, const float* w_ts, int64_t M, int64_t N, int64_t K, void* out,
                             bool out_f32, int variant, void* workspace, void* partial, hipStream_t st);

// NVFP4 product for many tokens: the activations are dequantized once to fp16 into `workspace`
// (nv16_workspace_bytes(M, K) bytes, 256-byte aligned), then multiplied against W dequantized on the fly
size_t nv16_workspace_bytes(int64_t M, int64_t K);
hipError_t launch_gemm_nv16(const void* a_codes, const void* a_scales, const float* a_ts, const void* w_codes,
                            const void* w_scales, const float* w_ts, int64_t M, int64_t N, int64_t K, void* out,
                            bool out_f32, void* workspace, void* partial, hipStream_t st);
// fp32 partials of a split-K run of that product (`partial`, may be null: then it is never split); 0 = not split
size_t nv16_split_k_bytes(int64_t M, int64_t N, int64_t K);

// few-token weight-streaming GEMM, both formats, operands in GEMM layout: every shape up to 64 tokens, and the shapes
// gemm_skinny_takes() accepts above that
bool gemm_skinny_takes(int64_t M, int64_t N, int64_t K, int fmt);
hipError_t launch_gemm_skinny(const void* a_codes, const void* a_scales, const float* a_ts, const void* w_codes,
                              const void* w_scales, const float* w_ts, int64_t M, int64_t N, int64_t K, int fmt, void* out,
                              bool out_f32, float alpha, hipStream_t st);

// M <= 16, MXFP4: rotation + quantization of the activations inside the weight-streaming GEMM (W in GEMM layout);
// weight_only: the rotated activations stay bf16 (W4A16)
hipError_t launch_fused_decode(const void* x, int64_t M, int64_t K, int b, const void* w_codes, const void* w_scales,
                               int64_t N, void* out, bool out_f32, bool weight_only, float alpha, hipStream_t st);

// MR-GPTQ sweep over fixed scales (canonical layout) with the factor U of the damped inverse Hessian in visiting order;
// workspace of gptq_workspace_bytes(N, K) bytes; K % 64 == 0, K <= 24576
size_t gptq_workspace_bytes(int64_t N, int64_t K);
hipError_t launch_gptq_sweep(const void* w, int64_t N, int64_t K, int b, int fmt, const float* U, const int* perm,
                             const void* scales, const float* s_T, const float* table, float factor, void* codes, void* workspace,
                             hipStream_t st);

// Hessian [K,K] fp32 -> static activation order and the upper-triangular U with U^T U = (H[perm][:,perm] + damp mean(diag) I)^-1
size_t gptq_prepare_workspace_bytes(int64_t K);
hipError_t launch_gptq_prepare(const float* H, int64_t K, float damp, bool use_order, int* perm, float* U, void* workspace,
                               hipStream_t st);

// Hessian of rotated calibration rows: Xr = x H_b (fp32 scratch [T,K]), H (+)= Xr^T Xr
hipError_t launch_gptq_rotate_rows(const void* x, int64_t T, int64_t K, int b, float* out, hipStream_t st);
hipError_t launch_gptq_hessian_product(const float* Xr, int64_t T, int64_t K, float* H, bool accumulate, hipStream_t st);

// measurement aids (fp4_probe): which = 0 scaled-FP4 MFMA issue loop, 1 fp16 MFMA issue loop (buf: one 24-byte record per
// compute unit), 2 streaming copy of the first half of buf to the second, 3 streaming read of the first half
// mode: 0 MXFP4, 1 MXFP4 with the tensor-level 4/3, 2 NVFP4, 3 scale byte fitted to the tensor's range (table at tensor_scale + 2)
hipError_t launch_dequantize(const void* codes, const void* scales, const float* tensor_scale, int64_t rows, int64_t K, int mode,
                             bool gemm_layout, void* out, bool out_f32, hipStream_t st);

hipError_t launch_probe(int which, void* buf, size_t bytes, int iters, hipStream_t st);

}  // namespace fp4mr
