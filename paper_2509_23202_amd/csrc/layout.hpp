// Index arithmetic of the GEMM layout, shared by the quantize kernels (writers) and the GEMM kernels
// (readers).  Host and device.
//
// The unit is a FRAGMENT: 16 rows x 128 K-elements of E2M1 codes = 1024 bytes, ordered the way one
// block-scaled FP4 MFMA (16x16x128) wants its operand: lane l of a wavefront owns row (l % 16) and the 32
// consecutive K-elements of K-block (l / 16), i.e. 16 contiguous bytes at offset 16*l.  Fragments of one
// 16-row block are consecutive along K:
//     codes byte offset (row, k) = ((row/16) * (K/128) + k/128) * 1024 + (((k%128)/32) * 16 + row%16) * 16 + (k%32)/2
// MXFP4 scales: one dword per lane holds the E8M0 bytes of four consecutive fragments along K (so one
// 32-bit load feeds four MFMAs through the op_sel byte selector):
//     scale byte offset (row, kg=k/32) = (((row/16) * ceil(K/512) + kg/16) * 64 + ((kg%4) * 16 + row%16)) * 4 + (kg/4)%4
// NVFP4 scales: two E4M3 bytes (the two groups of 16 inside the lane's 32 elements) per lane per fragment:
//     scale byte offset (row, g16=k/16) = (((row/16) * (K/128) + g16/8) * 64 + (((g16%8)/2) * 16 + row%16)) * 2 + g16%2
#pragma once

#include <stdint.h>

#ifndef __HIPCC__
#define __host__
#define __device__
#endif

namespace fp4mr {

constexpr int kFragRows = 16;
constexpr int kFragK = 128;
constexpr int kFragBytes = 1024;

__host__ __device__ inline int64_t round_up(int64_t a, int64_t b) { return (a + b - 1) / b * b; }

__host__ __device__ inline int64_t gemm_codes_bytes(int64_t rows, int64_t K)
{
    return round_up(rows, kFragRows) / kFragRows * (K / kFragK) * (int64_t)kFragBytes;
}

__host__ __device__ inline int64_t gemm_scales_bytes(int64_t rows, int64_t K, int fmt)
{
    const int64_t rb = round_up(rows, kFragRows) / kFragRows;
    if (fmt == 0) return rb * ((K + 511) / 512) * 256;  // MXFP4: 64 lanes x 4 bytes per 512 K-elements
    return rb * (K / kFragK) * 128;                      // NVFP4: 64 lanes x 2 bytes per fragment
}

// byte offsets of the formulas above (row = row of the tensor, k = element along K, kg = k / 32, g16 = k / 16;
// KC = K / 128, KS = ceil(K / 512))
__host__ __device__ inline int64_t gemm_codes_offset(int64_t row, int64_t k, int64_t KC)
{
    return ((row >> 4) * KC + (k >> 7)) * 1024 + ((((k & 127) >> 5) * 16 + (row & 15)) << 4) + ((k & 31) >> 1);
}

__host__ __device__ inline int64_t gemm_mx_scale_offset(int64_t row, int64_t kg, int64_t KS)
{
    return ((((row >> 4) * KS + (kg >> 4)) * 64 + ((kg & 3) * 16 + (row & 15))) << 2) + ((kg >> 2) & 3);
}

__host__ __device__ inline int64_t gemm_nv_scale_offset(int64_t row, int64_t g16, int64_t KC)
{
    return ((((row >> 4) * KC + (g16 >> 3)) * 64 + (((g16 & 7) >> 1) * 16 + (row & 15))) << 1) + (g16 & 1);
}

}  // namespace fp4mr
