// Pieces of the fused rotation + quantization shared by the kernels that contain it (the stand-alone quantizers and the
// few-token GEMM that quantizes its activations itself): the group quantizers, the +-1 Hadamard operand of the
// rotation MFMA and the butterfly levels that widen a 32-block to 64 / 128.
#pragma once

#include "device_util.hpp"

namespace fp4mr {

// ------------------------------------------------------------------------------------------------------
// Quantize NO consecutive fp32 values held by one lane (NO in {8,16,32}) whose group of G elements spans LG
// lanes (lanes differ in bits 4/5 of the lane id for the MFMA kernel, bits 0/1 for the direct kernel).
// XOR_LO is the lane-id distance of the first partner.
template <int G, int NO, int XOR_LO, bool HW>
struct GroupQuant {
    static constexpr int LG = (G > NO) ? G / NO : 1;   // lanes per group
    static constexpr int NG = (NO > G) ? NO / G : 1;   // groups per lane
    static constexpr int VG = NO / NG;                 // values per lane per group
    static constexpr int ND = NO / 8;                  // dwords of codes per lane

    // MXFP4: returns scale bytes in sc[NG], codes in out[ND]
    __device__ static __forceinline__ void mx(const float (&y)[NO], uint32_t (&out)[ND], uint32_t (&sc)[NG])
    {
#pragma unroll
        for (int gi = 0; gi < NG; ++gi) {
            float amax = 0.0f;
#pragma unroll
            for (int i = 0; i < VG; ++i) amax = fabs_max(amax, y[gi * VG + i]);
            if constexpr (LG >= 2) amax = fmaxf(amax, __shfl_xor(amax, XOR_LO));
            if constexpr (LG >= 4) amax = fmaxf(amax, __shfl_xor(amax, XOR_LO * 2));
            // OCP MX: shared exponent = floor(log2 amax) - 2 -> biased byte = exponent field - 2, clamped at 0
            const int ef = (int)((__float_as_uint(amax) >> 23) & 0xffu);
            const uint32_t byte = (uint32_t)max(ef - 2, 0);
            sc[gi] = byte;
#pragma unroll
            for (int d = 0; d < VG / 8; ++d) {
                float t[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) t[i] = y[gi * VG + d * 8 + i];
                out[gi * (VG / 8) + d] = e2m1_pack8_e8m0<HW>(t, byte);
            }
        }
    }

    // NVFP4 with tensor scale s_T
    __device__ static __forceinline__ void nv(const float (&y)[NO], float s_T, uint32_t (&out)[ND], uint32_t (&sc)[NG])
    {
        const float six_sT = 6.0f * s_T;
#pragma unroll
        for (int gi = 0; gi < NG; ++gi) {
            float amax = 0.0f;
#pragma unroll
            for (int i = 0; i < VG; ++i) amax = fabs_max(amax, y[gi * VG + i]);
            if constexpr (LG >= 2) amax = fmaxf(amax, __shfl_xor(amax, XOR_LO));
            if constexpr (LG >= 4) amax = fmaxf(amax, __shfl_xor(amax, XOR_LO * 2));
            uint32_t c = 0;
            if (s_T > 0.0f) c = e4m3_encode<HW>(__fdiv_rn(amax, six_sT));
            sc[gi] = c;
            const float d = s_T * e4m3_decode<HW>(c);
            const float r = (d == 0.0f) ? 0.0f : __fdiv_rn(1.0f, d);
#pragma unroll
            for (int dd = 0; dd < VG / 8; ++dd) {
                float t[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) t[i] = y[gi * VG + dd * 8 + i] * r;
                uint32_t p = e2m1_pack8<HW>(t);
                out[gi * (VG / 8) + dd] = (d == 0.0f) ? 0u : p;
            }
        }
    }

    // ---- MSE scale policy (Section 4.1 "Ingredient 1": the scales that minimise sum (Xhat - X)^2; the "MSE" method of
    // Section 4.2 item 1).  Per group the scale code is searched in a window around the abs-max code (MXFP4: the code
    // and its two neighbours, tried in the order abs-max, one above, one below; NVFP4: see nv_mse); a candidate wins
    // only with a strictly smaller squared error.
    // The error is accumulated in fp32 per lane and added across the lanes of the group symmetrically, so that every
    // lane of a group takes the same decision.  Hardware converts only (encode and decode).
    typedef float v2f_t __attribute__((ext_vector_type(2)));

    // codes of 8 values at scale `sc` (E8M0 in the exponent field) and the squared error they leave
    __device__ static __forceinline__ uint32_t try8(const float (&t)[8], float sc, float mul, float& err)
    {
        uint32_t p = 0;
        p = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p, t[0], t[1], sc, 0);
        p = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p, t[2], t[3], sc, 1);
        p = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p, t[4], t[5], sc, 2);
        p = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p, t[6], t[7], sc, 3);
        const v2f_t q0 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(p, sc, 0);
        const v2f_t q1 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(p, sc, 1);
        const v2f_t q2 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(p, sc, 2);
        const v2f_t q3 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(p, sc, 3);
        const float q[8] = {q0[0], q0[1], q1[0], q1[1], q2[0], q2[1], q3[0], q3[1]};
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float d = t[i] - q[i];
            err = __fmaf_rn(d * mul, d * mul, err);
        }
        return p;
    }

    __device__ static __forceinline__ float group_sum(float e)
    {
        if constexpr (LG >= 2) e += __shfl_xor(e, XOR_LO);
        if constexpr (LG >= 4) e += __shfl_xor(e, XOR_LO * 2);
        return e;
    }

    __device__ static __forceinline__ void mx_mse(const float (&y)[NO], uint32_t (&out)[ND], uint32_t (&sc)[NG])
    {
#pragma unroll
        for (int gi = 0; gi < NG; ++gi) {
            float amax = 0.0f;
#pragma unroll
            for (int i = 0; i < VG; ++i) amax = fabs_max(amax, y[gi * VG + i]);
            if constexpr (LG >= 2) amax = fmaxf(amax, __shfl_xor(amax, XOR_LO));
            if constexpr (LG >= 4) amax = fmaxf(amax, __shfl_xor(amax, XOR_LO * 2));
            const int ef = (int)((__float_as_uint(amax) >> 23) & 0xffu);
            const int byte0 = max(ef - 2, 0);
            float best_err = 0.0f;
            uint32_t best_byte = 0, best[VG / 8];
#pragma unroll
            for (int k = 0; k < 3; ++k) {
                const int byte = min(max(byte0 + (k == 0 ? 0 : (k == 1 ? 1 : -1)), 0), 254);
                const float scf = __uint_as_float((uint32_t)byte << 23);
                float err = 0.0f;
                uint32_t cand[VG / 8];
#pragma unroll
                for (int d = 0; d < VG / 8; ++d) {
                    float t[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) t[i] = y[gi * VG + d * 8 + i];
                    cand[d] = try8(t, scf, 1.0f, err);
                }
                err = group_sum(err);
                if (k == 0 || err < best_err) {
                    best_err = err;
                    best_byte = (uint32_t)byte;
#pragma unroll
                    for (int d = 0; d < VG / 8; ++d) best[d] = cand[d];
                }
            }
            sc[gi] = best_byte;
#pragma unroll
            for (int d = 0; d < VG / 8; ++d) out[gi * (VG / 8) + d] = best[d];
        }
    }

    // NVFP4: E4M3 has eight codes per octave and the minimiser sits either next to the abs-max code c0 or about half an
    // octave above it (the scale that puts the largest element on 4 instead of 6), so the window is c0 - 2 .. c0 + 7,
    // tried in the order c0, +1, -1, +2, -2, +3, +4, +5, +6, +7 (a brute force over every code finds the global minimiser
    // inside this window in all but about 1e-4 of the groups of heavy-tailed data; within +-1 in only half of them).
    __device__ static __forceinline__ void nv_mse(const float (&y)[NO], float s_T, uint32_t (&out)[ND], uint32_t (&sc)[NG])
    {
        const float six_sT = 6.0f * s_T;
#pragma unroll
        for (int gi = 0; gi < NG; ++gi) {
            float amax = 0.0f;
#pragma unroll
            for (int i = 0; i < VG; ++i) amax = fabs_max(amax, y[gi * VG + i]);
            if constexpr (LG >= 2) amax = fmaxf(amax, __shfl_xor(amax, XOR_LO));
            if constexpr (LG >= 4) amax = fmaxf(amax, __shfl_xor(amax, XOR_LO * 2));
            int c0 = 0;
            if (s_T > 0.0f) c0 = (int)e4m3_encode<true>(__fdiv_rn(amax, six_sT));
            float best_err = 0.0f;
            uint32_t best_c = 0, best[VG / 8];
            // a rolled loop: ten copies of the body would not fit the instruction cache's share of a wave
#pragma unroll 1
            for (int k = 0; k < 10; ++k) {
                const int off = k < 5 ? ((k & 1) ? (k + 1) >> 1 : -(k >> 1)) : k - 2;   // 0, +1, -1, +2, -2, +3 .. +7
                const int c = min(max(c0 + off, 0), 0x7e);
                const float d = s_T * e4m3_decode<true>((uint32_t)c);
                const float r = (d == 0.0f) ? 0.0f : __fdiv_rn(1.0f, d);
                float err = 0.0f;
                uint32_t cand[VG / 8];
#pragma unroll
                for (int dd = 0; dd < VG / 8; ++dd) {
                    // the error is measured in units of d: (y r - q)^2 d^2 = (y - q d)^2 up to the rounding of y r
                    float t[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) t[i] = y[gi * VG + dd * 8 + i] * r;
                    if (d == 0.0f) {
                        cand[dd] = 0u;
#pragma unroll
                        for (int i = 0; i < 8; ++i) err = __fmaf_rn(y[gi * VG + dd * 8 + i], y[gi * VG + dd * 8 + i], err);
                    } else {
                        cand[dd] = try8(t, 1.0f, d, err);
                    }
                }
                err = group_sum(err);
                if (k == 0 || err < best_err) {
                    best_err = err;
                    best_c = (uint32_t)c;
#pragma unroll
                    for (int dd = 0; dd < VG / 8; ++dd) best[dd] = cand[dd];
                }
            }
            sc[gi] = best_c;
#pragma unroll
            for (int dd = 0; dd < VG / 8; ++dd) out[gi * (VG / 8) + dd] = best[dd];
        }
    }

    // ---- rounded, 4/3-rescaled E8M0 scale (appendix on MXFP scale fitting, first equation): exponent
    // k = round(log2(amax / 6)), scale (4/3) 2^k; the byte stores k, the factor 4/3 is the tensor's.
    // With amax = m 2^e (1 <= m < 2): log2(amax / 6) = e - 2 + log2(m / 1.5) and m / 1.5 lies in [2/3, 4/3), so the
    // rounded exponent is e - 2, less one when m / 1.5 < 2^-1/2, i.e. when m < 1.5 / sqrt 2 -- decided on the
    // mantissa field against the smallest binary32 mantissa above that (irrational) bound: an exact decision.
    // Elements: E2M1(0.75 y 2^-k).  0.75 y is not always a binary32 number, and rounding it to one before the
    // convert rounds again could land on (or cross) a tie of the E2M1 grid; the product is therefore rounded TO ODD
    // (truncate, then set the last mantissa bit if anything was lost -- the fma gives the lost part exactly), after
    // which the convert's round-to-nearest-even returns the correctly rounded code (24 bits against the grid's 2).
    __device__ static __forceinline__ float mul_075_to_odd(float v)
    {
        const float p = v * 0.75f;
        const float r = __fmaf_rn(v, 0.75f, -p);  // exact: what the rounding of p dropped
        const uint32_t pb = __float_as_uint(p);
        // r and p of opposite sign: |p| was rounded up, step back to the truncated magnitude
        const uint32_t odd = (pb - ((pb ^ __float_as_uint(r)) >> 31)) | 1u;
        return __uint_as_float((r != 0.0f && (pb << 1) != 0u) ? odd : pb);  // (a product that underflowed to zero stays zero)
    }

    __device__ static __forceinline__ void mx43(const float (&y)[NO], uint32_t (&out)[ND], uint32_t (&sc)[NG])
    {
#pragma unroll
        for (int gi = 0; gi < NG; ++gi) {
            float amax = 0.0f;
#pragma unroll
            for (int i = 0; i < VG; ++i) amax = fabs_max(amax, y[gi * VG + i]);
            if constexpr (LG >= 2) amax = fmaxf(amax, __shfl_xor(amax, XOR_LO));
            if constexpr (LG >= 4) amax = fmaxf(amax, __shfl_xor(amax, XOR_LO * 2));
            const uint32_t ab = __float_as_uint(amax);
            const int ef = (int)((ab >> 23) & 0xffu);
            const int below = (ab & 0x7fffffu) < 0x7c3b7u ? 1 : 0;  // mantissa under 1.5 / sqrt 2
            const uint32_t byte = (uint32_t)max(ef - 2 - below, 0);
            sc[gi] = byte;
#pragma unroll
            for (int d = 0; d < VG / 8; ++d) {
                float t[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) t[i] = mul_075_to_odd(y[gi * VG + d * 8 + i]);
                out[gi * (VG / 8) + d] = e2m1_pack8_e8m0<HW>(t, byte);
            }
        }
    }

    // ---- scale byte fitted to the tensor's range of scales (appendix on MXFP scale fitting: s = 2^(alpha q + beta), the
    // modified format MXFP4-dagger).  The byte is the index of the nearest of 256 scale values that are evenly spaced
    // in the log domain between the smallest and the largest ideal group scale (amax / 6) of the tensor:
    //     q = clamp(round((log2 amax - lmin) * inv), 0, 255),  lmin = beta + log2 6,  inv = 1 / alpha  (0 when alpha = 0)
    // and the group's scale is table[q], the binary32 value of 2^(alpha q + beta) that the range pre-pass published.
    // Elements follow the NVFP4 chain (correctly rounded reciprocal, one multiply, the converting pack: saturating).
    // A group that is all zero gets byte 0 and zero codes.
    __device__ static __forceinline__ float group_amax(const float (&y)[NO], int gi)
    {
        float amax = 0.0f;
#pragma unroll
        for (int i = 0; i < VG; ++i) amax = fabs_max(amax, y[gi * VG + i]);
        if constexpr (LG >= 2) amax = fmaxf(amax, __shfl_xor(amax, XOR_LO));
        if constexpr (LG >= 4) amax = fmaxf(amax, __shfl_xor(amax, XOR_LO * 2));
        return amax;
    }

    __device__ static __forceinline__ void mx_fit(const float (&y)[NO], float lmin, float inv, const float* __restrict__ table,
                                                  uint32_t (&out)[ND], uint32_t (&sc)[NG])
    {
#pragma unroll
        for (int gi = 0; gi < NG; ++gi) {
            const float amax = group_amax(y, gi);
            int q = 0;
            if (amax > 0.0f) q = min(max((int)rintf((__log2f(amax) - lmin) * inv), 0), 255);
            sc[gi] = (uint32_t)q;
            const float d = table[q];
            const float r = (amax > 0.0f && d > 0.0f) ? __fdiv_rn(1.0f, d) : 0.0f;
#pragma unroll
            for (int dd = 0; dd < VG / 8; ++dd) {
                float t[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) t[i] = y[gi * VG + dd * 8 + i] * r;
                const uint32_t p = e2m1_pack8<HW>(t);
                out[gi * (VG / 8) + dd] = (r == 0.0f) ? 0u : p;
            }
        }
    }

    // POL: 0 abs-max, 1 squared-error search, 2 rounded exponent with the 4/3 factor (MXFP4 only)
    template <int POL>
    __device__ static __forceinline__ void run(const float (&y)[NO], float s_T, uint32_t (&out)[ND], uint32_t (&sc)[NG])
    {
        static_assert(POL >= 0 && POL <= 2 && (POL != 2 || G == 32), "scale policy");
        if constexpr (G == 32) {
            if constexpr (POL == 1) mx_mse(y, out, sc);
            else if constexpr (POL == 2) mx43(y, out, sc);
            else mx(y, out, sc);
        } else {
            if constexpr (POL == 1) nv_mse(y, s_T, out, sc); else nv(y, s_T, out, sc);
        }
    }
};


// Hadamard operand of the rotation MFMA: A[i][k] = H[32s + k][c(t,i)] with c(t,i) = (i/4)*NO + 4t + i%4 (the column
// permutation that leaves every lane with NO = BP/4 consecutive outputs); the lane holds i = g, k = 8q .. 8q+7.
// Entries are +-1 in bf16 inside the b x b diagonal block of the column, 0 outside (b < BP: block-diagonal).
// Sylvester: H[r][c] = (-1)^popcount(r & c).  With r = r_hi + e (e = 0..7, b >= 8) the sign factors into
// parity(r_hi & c) times parity(e & (c & 7)), and c & 7 = (4t + g%4) & 7 takes two values (t even / odd): two
// 8-element patterns are built once and every register group costs a sign flip and a block test.
template <int BP>
__device__ __forceinline__ void build_hadamard_operand(v8bf (&hop)[BP / 16][BP / 32], int g, int q, int b)
{
    constexpr int S = BP / 32, T = BP / 16, NO = BP / 4;
    const unsigned bm = (unsigned)b - 1u;
    const unsigned b0 = (unsigned)g & 1u, b1 = ((unsigned)g >> 1) & 1u;
    uint32_t pat[2][4];  // [t & 1][d]: elements e = 2d (low half) and 2d+1 (high half)
#pragma unroll
    for (unsigned b2 = 0; b2 < 2; ++b2)
#pragma unroll
        for (unsigned d = 0; d < 4; ++d) {
            const unsigned lo = ((d & 1u) & b1) ^ (((d >> 1) & 1u) & b2);  // parity(2d & c3), c3 = b0 + 2 b1 + 4 b2
            const unsigned hi = lo ^ b0;                                     // parity((2d + 1) & c3)
            pat[b2][d] = 0x3f803f80u | (lo << 15) | (hi << 31);
        }
#pragma unroll
    for (int t = 0; t < T; ++t) {
        const unsigned c = (unsigned)((g >> 2) * NO + 4 * t + (g & 3));
#pragma unroll
        for (int s = 0; s < S; ++s) {
            const unsigned r_hi = (unsigned)(32 * s + 8 * q);
            const bool same = (r_hi & ~bm) == (c & ~bm);
            const uint32_t flip = (__popc(r_hi & c & bm) & 1u) ? 0x80008000u : 0u;
            v4i w;
#pragma unroll
            for (int d = 0; d < 4; ++d) w[d] = same ? (int)(pat[t & 1][d] ^ flip) : 0;
            hop[t][s] = __builtin_bit_cast(v8bf, w);
        }
    }
}

// Hadamard blocks of 64 and 128 on the 32-wide operand.  Sylvester's matrix is a Kronecker product,
// H_64 = H_2 (x) H_32 and H_128 = H_4 (x) H_32: after the MFMA has applied H_32 to every 32-element vector, the
// 2 (4) vectors of one block sit in the lanes g, g^1 (g, g^1, g^2, g^3) of a quad -- the 16 vectors of an MFMA group
// are consecutive along K and blocks are aligned -- and one (two) butterfly levels across those lanes finish the
// transform: lane bit clear -> self + partner, set -> partner - self.  The 128 x 128 operand (128 registers) and
// its MFMAs are never needed.
template <int CTRL>
__device__ __forceinline__ float quad_partner(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}

template <int T>
__device__ __forceinline__ void kronecker_levels(v4f (&acc)[T], int g, int levels)
{
    float h[4 * T], p[4 * T];
#pragma unroll
    for (int i = 0; i < 4 * T; ++i) h[i] = acc[i >> 2][i & 3];
    if (levels >= 1) {
        const float sg = (g & 1) ? -1.0f : 1.0f;
#pragma unroll
        for (int i = 0; i < 4 * T; ++i) p[i] = quad_partner<0xB1>(h[i]);  // quad_perm [1,0,3,2]: lane ^ 1
#pragma unroll
        for (int i = 0; i < 4 * T; ++i) h[i] = __fmaf_rn(h[i], sg, p[i]);
    }
    if (levels >= 2) {
        const float sg = (g & 2) ? -1.0f : 1.0f;
#pragma unroll
        for (int i = 0; i < 4 * T; ++i) p[i] = quad_partner<0x4E>(h[i]);  // quad_perm [2,3,0,1]: lane ^ 2
#pragma unroll
        for (int i = 0; i < 4 * T; ++i) h[i] = __fmaf_rn(h[i], sg, p[i]);
    }
#pragma unroll
    for (int i = 0; i < 4 * T; ++i) acc[i >> 2][i & 3] = h[i];
}

}  // namespace fp4mr
