// In-register NVFP4 fragment dequantization shared by the NVFP4 GEMM kernels: 32 E2M1 codes of one lane (16 bytes)
// times the two E4M3 group scales of that lane -> 32 fp16 values (exact: <= 6 significant bits, range [2^-10, 2688]).
#pragma once

#include "device_util.hpp"

namespace fp4mr {

// 8 codes (one dword) times one scale -> 8 fp16
__device__ __forceinline__ v8h nv_dequant8(uint32_t codes, v2h scale2)
{
    // byte i of the dword: low nibble -> .x, high nibble -> .y
    const v2h p0 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(codes, 1.0f, 0) * scale2;
    const v2h p1 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(codes, 1.0f, 1) * scale2;
    const v2h p2 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(codes, 1.0f, 2) * scale2;
    const v2h p3 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(codes, 1.0f, 3) * scale2;
    const v8h r = {p0[0], p0[1], p1[0], p1[1], p2[0], p2[1], p3[0], p3[1]};
    return r;
}

struct NvFrag16 {
    v8h s[4];  // s[i] = elements 8i..8i+7 of the lane's 32
};

__device__ __forceinline__ NvFrag16 nv_dequant_frag(const v4i& codes, uint32_t scale_bytes)
{
    const _Float16 s0 = (_Float16)e4m3_decode<true>(scale_bytes & 0xffu);
    const _Float16 s1 = (_Float16)e4m3_decode<true>((scale_bytes >> 8) & 0xffu);
    const v2h a = {s0, s0}, b = {s1, s1};
    NvFrag16 f;
    f.s[0] = nv_dequant8((uint32_t)codes[0], a);
    f.s[1] = nv_dequant8((uint32_t)codes[1], a);
    f.s[2] = nv_dequant8((uint32_t)codes[2], b);
    f.s[3] = nv_dequant8((uint32_t)codes[3], b);
    return f;
}

}  // namespace fp4mr
