// Device-side helpers shared by the fp4mr kernels (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fp4mr {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v2f __attribute__((ext_vector_type(2)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v2h __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;

// ---------------------------------------------------------------- E2M1 element codec
// Software encoder: exact round-to-nearest-even onto {0,.5,1,1.5,2,3,4,6} with saturation, sign bit
// kept (so -0.0 and tiny negatives give 0x8).  Integer arithmetic on the binary32 pattern only.
__device__ __forceinline__ uint32_t e2m1_encode_sw(float t)
{
    const uint32_t u = __float_as_uint(t);
    const uint32_t sign = (u >> 28) & 8u;
    const uint32_t a = u & 0x7fffffffu;
    uint32_t mag;
    if (a < 0x3f800000u) {
        // |t| < 1: the grid step is 0.5.  Adding 2^22 aligns the binary32 ulp to 0.5, so the hardware's
        // round-to-nearest-even of the addition performs the rounding; the low bits then count halves.
        const float r = __uint_as_float(a) + 4194304.0f;
        mag = __float_as_uint(r) & 3u;  // 0, 1 (=0.5) or 2 (=1.0)
    } else {
        // |t| >= 1: keep one mantissa bit.  Round to nearest even at bit 22, carry may bump the exponent.
        const uint32_t r = a + 0x1fffffu + ((a >> 22) & 1u);
        mag = (r >> 22) - (126u << 1);  // exponent 127 (1.0) -> code 2
        mag = mag > 7u ? 7u : mag;      // saturate at 6.0
    }
    return sign | mag;
}

// Eight values -> one dword of codes, element i in nibble i.
template <bool HW>
__device__ __forceinline__ uint32_t e2m1_pack8(const float (&t)[8])
{
    if constexpr (HW) {
        // v_cvt_scalef32_pk_fp4_f32 with unit scale: two binary32 -> two E2M1 into byte `sel` of the dword.
        uint32_t p = 0;
        p = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p, t[0], t[1], 1.0f, 0);
        p = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p, t[2], t[3], 1.0f, 1);
        p = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p, t[4], t[5], 1.0f, 2);
        p = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p, t[6], t[7], 1.0f, 3);
        return p;
    } else {
        uint32_t p = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) p |= e2m1_encode_sw(t[i]) << (4 * i);
        return p;
    }
}

// Eight values divided by the E8M0 scale 2^(byte - 127) -> one dword of codes.  The hardware convert takes the scale
// as the exponent field of a binary32 operand, so the division is free (checked against multiply-then-convert over
// every scale byte, subnormal inputs included); the software codec multiplies by the exact reciprocal.
template <bool HW>
__device__ __forceinline__ uint32_t e2m1_pack8_e8m0(const float (&y)[8], uint32_t byte)
{
    if constexpr (HW) {
        const float sc = __uint_as_float(byte << 23);
        uint32_t p = 0;
        p = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p, y[0], y[1], sc, 0);
        p = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p, y[2], y[3], sc, 1);
        p = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p, y[4], y[5], sc, 2);
        p = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p, y[6], y[7], sc, 3);
        return p;
    } else {
        const float inv = __uint_as_float((254u - byte) << 23);  // 2^(127 - byte), a normal number for byte <= 253
        float t[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) t[i] = y[i] * inv;
        return e2m1_pack8<false>(t);
    }
}

// ---------------------------------------------------------------- E4M3 scale codec (non-negative input)
// Software encoder: round-to-nearest-even onto the e4m3fn grid (bias 7, subnormal step 2^-9), saturating
// at 448.
__device__ __forceinline__ uint32_t e4m3_encode_sw(float t)
{
    if (!(t > 0.0f)) return 0u;
    if (t >= 448.0f) return 0x7eu;
    const uint32_t a = __float_as_uint(t);
    if (a < 0x3c800000u) {  // t < 2^-6: subnormal range, step 2^-9; 2^-9 * 2^23 = 2^14
        const float r = t + 16384.0f;
        return __float_as_uint(r) & 0xfu;  // 0..8 (8 = 2^-6, the first normal: code 0x08)
    }
    const uint32_t r = a + 0x7ffffu + ((a >> 20) & 1u);  // keep three mantissa bits
    return (r >> 20) - ((127u - 7u) << 3);
}

__device__ __forceinline__ float e4m3_decode_sw(uint32_t c)
{
    const uint32_t e = (c >> 3) & 15u, m = c & 7u;
    if (e == 0u) return (float)m * 0.001953125f;              // m * 2^-9
    return __uint_as_float(((e + 120u) << 23) | (m << 20));  // (1 + m/8) * 2^(e-7)
}

template <bool HW>
__device__ __forceinline__ uint32_t e4m3_encode(float t)
{
    if constexpr (HW) {
        const float c = fminf(t, 448.0f);
        return (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(c, 0.0f, 0, false) & 0xffu;
    } else {
        return e4m3_encode_sw(t);
    }
}

template <bool HW>
__device__ __forceinline__ float e4m3_decode(uint32_t c)
{
    if constexpr (HW) {
        return __builtin_amdgcn_cvt_f32_fp8((int)c, 0);
    } else {
        return e4m3_decode_sw(c);
    }
}

// ---------------------------------------------------------------- misc
__device__ __forceinline__ float fabs_max(float a, float b) { return fmaxf(a, fabsf(b)); }

// Fast exact division by a runtime constant d (2 <= d < 2^31) for n < 2^31: q = umulhi(n, magic) >> shift.
struct FastDiv {
    uint32_t magic;
    uint32_t shift;
    uint32_t d;
};

__device__ __forceinline__ uint32_t fast_div(uint32_t n, const FastDiv& f)
{
    return f.d == 1u ? n : (__umulhi(n, f.magic) >> f.shift);
}

}  // namespace fp4mr
