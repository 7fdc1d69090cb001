// The decoding side of the formats (arXiv 2509.23202, Section 2: a microscaling tensor is scale x element per group;
// Section 4.1 "Ingredient 1": NVFP4 with its tensor scale; appendix on MXFP scale fitting: the rescaled E8M0 rule and the
// scale byte fitted to the tensor's range).  xhat[m, k] = E2M1(code) * scale of the group, from either layout, to bf16
// or fp32.  What an emulated evaluation multiplies, and the only consumer of the fitted-range format.
//
// One lane decodes the eight elements of one code dword (they share a group in both formats) and writes 16 bytes of
// bf16 or 32 bytes of fp32: HBM-bound, 0.5 + 1/G bytes in, 2 or 4 bytes out per element.  All arithmetic is binary32:
//   MXFP4          E2M1 * 2^(byte - 127): exact;  with the 4/3 rule one multiplication by the binary32 value of 4/3
//   NVFP4          (E2M1 * E4M3) exact (at most 6 significant bits), times the tensor scale: one rounding
//   fitted range   E2M1 * table[byte]: one rounding
// bf16 output rounds that binary32 value to nearest even.
#include "device_util.hpp"
#include "internal.hpp"
#include "layout.hpp"

namespace fp4mr {
namespace {

struct DqArgs {
    const uint8_t* codes;
    const uint8_t* scales;
    const float* tensor_scale;
    void* out;
    int64_t rows, K;
};

// MODE 0 MXFP4 (E8M0), 1 MXFP4 with the 4/3 factor, 2 NVFP4, 3 fitted range (table at tensor_scale + 2)
template <int MODE, bool GEMM_LAYOUT, bool OUT_F32>
__global__ __launch_bounds__(256) void dequantize_kernel(DqArgs a)
{
    typedef float v2f_t __attribute__((ext_vector_type(2)));
    constexpr int G = MODE == 2 ? 16 : 32;
    const int64_t n8 = a.rows * a.K / 8;
    const int64_t KC = a.K >> 7, KS = (a.K + 511) >> 9;
    float s_T = 1.0f;
    if constexpr (MODE == 2) s_T = *a.tensor_scale;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n8; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t e0 = i * 8, row = e0 / a.K, k = e0 - row * a.K;
        uint32_t p;
        uint8_t sb;
        if constexpr (GEMM_LAYOUT) {
            p = *reinterpret_cast<const uint32_t*>(a.codes + gemm_codes_offset(row, k, KC));
            sb = (G == 32) ? a.scales[gemm_mx_scale_offset(row, k >> 5, KS)] : a.scales[gemm_nv_scale_offset(row, k >> 4, KC)];
        } else {
            p = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(a.codes + (e0 >> 1)));  // read once
            sb = a.scales[e0 / G];
        }
        float s;
        if constexpr (MODE == 0 || MODE == 1) s = __uint_as_float(sb == 0 ? 0x00400000u : (uint32_t)sb << 23);  // 2^(byte - 127); byte 0 is the subnormal 2^-127
        else if constexpr (MODE == 2) s = e4m3_decode<true>(sb);
        else s = a.tensor_scale[2 + sb];
        const v2f_t q0 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(p, 1.0f, 0);
        const v2f_t q1 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(p, 1.0f, 1);
        const v2f_t q2 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(p, 1.0f, 2);
        const v2f_t q3 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(p, 1.0f, 3);
        float v[8] = {q0[0], q0[1], q1[0], q1[1], q2[0], q2[1], q3[0], q3[1]};
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            v[j] *= s;
            if constexpr (MODE == 1) v[j] *= 4.0f / 3.0f;
            if constexpr (MODE == 2) v[j] *= s_T;
        }
        if constexpr (OUT_F32) {
            // written once, never read here: streaming stores
            v4f* o = reinterpret_cast<v4f*>(static_cast<float*>(a.out) + e0);
            __builtin_nontemporal_store(v4f{v[0], v[1], v[2], v[3]}, o);
            __builtin_nontemporal_store(v4f{v[4], v[5], v[6], v[7]}, o + 1);
        } else {
            typedef __bf16 v8b __attribute__((ext_vector_type(8)));
            const v8b o = {(__bf16)v[0], (__bf16)v[1], (__bf16)v[2], (__bf16)v[3], (__bf16)v[4], (__bf16)v[5], (__bf16)v[6], (__bf16)v[7]};
            __builtin_nontemporal_store(__builtin_bit_cast(v4i, o), reinterpret_cast<v4i*>(static_cast<__bf16*>(a.out) + e0));
        }
    }
}

template <int MODE>
hipError_t launch_mode(const DqArgs& a, bool gemm_layout, bool out_f32, hipStream_t st)
{
    const int64_t n8 = a.rows * a.K / 8;
    int64_t blocks = (n8 + 255) / 256;
    if (blocks > 256 * 64) blocks = 256 * 64;  // grid-stride beyond: 64 workgroups per compute unit keep HBM busy
    if (blocks < 1) blocks = 1;
    const dim3 grid((unsigned)blocks), block(256);
    if (gemm_layout) {
        if (out_f32) hipLaunchKernelGGL((dequantize_kernel<MODE, true, true>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((dequantize_kernel<MODE, true, false>), grid, block, 0, st, a);
    } else {
        if (out_f32) hipLaunchKernelGGL((dequantize_kernel<MODE, false, true>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((dequantize_kernel<MODE, false, false>), grid, block, 0, st, a);
    }
    return hipGetLastError();
}

}  // namespace

// mode: 0 MXFP4, 1 MXFP4 with the 4/3 factor, 2 NVFP4, 3 fitted range
hipError_t launch_dequantize(const void* codes, const void* scales, const float* tensor_scale, int64_t rows, int64_t K, int mode,
                             bool gemm_layout, void* out, bool out_f32, hipStream_t st)
{
    DqArgs a{static_cast<const uint8_t*>(codes), static_cast<const uint8_t*>(scales), tensor_scale, out, rows, K};
    switch (mode) {
        case 0: return launch_mode<0>(a, gemm_layout, out_f32, st);
        case 1: return launch_mode<1>(a, gemm_layout, out_f32, st);
        case 2: return launch_mode<2>(a, gemm_layout, out_f32, st);
        case 3: return launch_mode<3>(a, gemm_layout, out_f32, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace fp4mr
