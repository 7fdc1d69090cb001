// One launch for a handful of tokens (M <= 16), MXFP4:  out = Q(X H_b) Q(W H_b)^T  with the activations rotated and
// quantized inside the GEMM (arXiv 2509.23202, Section 4.2 items 1 and 2 in one kernel; the appendix on inference regimes
// notes that at small batch the separate kernels give little: here the activation side costs no launch of its own).
//
// Same decomposition as the few-token weight-streaming kernel: a workgroup owns one 16-column block of the output
// (one row-block of W in GEMM layout), its 8 waves split K, W fragments go straight from global memory to registers.
// The activation fragments are not loaded but made: a wave's share of K is walked in chunks of four fragments
// (512 K-elements = 16 vectors of 32), and for every token the 16 vectors of the chunk are one rotation MFMA group
// (vectors consecutive along K in one row, so Hadamard blocks of 64 / 128 finish with butterfly levels across lanes),
// quantized by the same group quantizer as the stand-alone kernels, and scattered through LDS into the lane order of
// the GEMM's B operand.  A token's 512 activations are 1 KB of bf16: less L2 traffic than the 4 x 1 KB of 16-row padded
// code fragments the unfused path reads.  The codes are the stand-alone quantizer's codes, the K split and the order
// of additions are the weight-streaming kernel's: the result is bit-identical to the two-launch path.
#include "device_util.hpp"
#include "internal.hpp"
#include "layout.hpp"
#include "rq_core.hpp"

namespace fp4mr {
namespace {

constexpr int kFusedWaves = 8;

struct FusedArgs {
    const uint16_t* x;       // [M, K] bf16
    const uint8_t* w_codes;  // GEMM layout
    const uint8_t* w_scales;
    void* out;
    int M, N, K, b;
    float c_hi, c_lo;        // 1/sqrt(b) split in two floats
    float alpha;             // factor on the result (4/3 when the weights' scales carry the tensor-level 4/3), else 1
};

// MP = token rows kept in the staging area (4 or 16): rows of the activation fragments beyond MP are zero by construction
// and never touch LDS, which keeps the workgroup small enough for four of them per compute unit when M <= 4.
template <bool OUT_F32, int MP>
__global__ __launch_bounds__(kFusedWaves * 64) void gemm_fused_decode_kernel(FusedArgs a)
{
    constexpr int U = 4;    // fragments per chunk = 16 vectors of 32
    constexpr int TOK = 4;  // tokens whose loads are in flight together
    using GQ = GroupQuant<32, 8, 16, true>;

    // staging: entry (vector v of the chunk, token m) at v * MP + m: four code dwords and one scale dword (byte in bits 7:0)
    __shared__ __attribute__((aligned(16))) uint32_t st_codes[kFusedWaves][16 * MP * 4];
    __shared__ __attribute__((aligned(16))) uint32_t st_scales[kFusedWaves][16 * MP];
    __shared__ float partial[kFusedWaves][256];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int g = lane & 15, q = lane >> 4;
    const int rb = blockIdx.x;
    const int KC = a.K >> 7, KS = (a.K + 511) >> 9;
    const int per = (KC + kFusedWaves - 1) / kFusedWaves;
    const int k_begin = min(wave * per, KC), k_end = min(k_begin + per, KC);

    v8bf hop[2][1];
    build_hadamard_operand<32>(hop, g, q, a.b < 32 ? a.b : 32);
    const int kron = a.b > 32 ? (a.b == 64 ? 1 : 2) : 0;

    // rows of the staged fragments that belong to no token stay zero for the whole kernel
    uint32_t* const sc_codes = st_codes[wave];
    uint32_t* const sc_scales = st_scales[wave];
    for (int i = lane; i < 16 * MP * 4; i += 64) sc_codes[i] = 0u;
    for (int i = lane; i < 16 * MP; i += 64) sc_scales[i] = 0u;

    const v4i* wfrag = reinterpret_cast<const v4i*>(a.w_codes + (int64_t)rb * KC * 1024) + lane;
    v4f acc = {0.f, 0.f, 0.f, 0.f};

    for (int kc0 = k_begin; kc0 < k_end; kc0 += U) {
        // activations of the chunk: vector g of the chunk starts at element (kc0 * 4 + g) * 32; it exists if its fragment
        // is inside this wave's share of K
        const bool v_ok = kc0 + (g >> 2) < k_end;
        const int64_t k_lane = (int64_t)kc0 * 128 + g * 32 + 8 * q;
        for (int m0 = 0; m0 < a.M; m0 += TOK) {
            v4i xin[TOK];
#pragma unroll
            for (int t = 0; t < TOK; ++t) {
                const v4i z = {0, 0, 0, 0};
                const int m = m0 + t;
                xin[t] = (m < a.M && v_ok) ? *reinterpret_cast<const v4i*>(a.x + (int64_t)m * a.K + k_lane) : z;
            }
#pragma unroll
            for (int t = 0; t < TOK; ++t) {
                const int m = m0 + t;
                if (m >= a.M) break;  // uniform
                v4f h[2];
#pragma unroll
                for (int tt = 0; tt < 2; ++tt) {
                    h[tt] = v4f{0.f, 0.f, 0.f, 0.f};
                    h[tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hop[tt][0], __builtin_bit_cast(v8bf, xin[t]), h[tt], 0, 0, 0);
                }
                kronecker_levels<2>(h, g, kron);
                float y[8];
#pragma unroll
                for (int tt = 0; tt < 2; ++tt)
#pragma unroll
                    for (int v = 0; v < 4; ++v) y[4 * tt + v] = __fmaf_rn(h[tt][v], a.c_hi, h[tt][v] * a.c_lo);
                uint32_t out[1], sc[1];
                GQ::mx(y, out, sc);
                // lane (g, q) holds elements 8q .. 8q+7 of vector g = K-block g%4 of fragment g/4, row m
                const int pos = g * MP + m;
                sc_codes[pos * 4 + q] = out[0];
                if (q == 0) sc_scales[pos] = sc[0];
            }
        }
        // W fragments and scales of the chunk, asked for only now: holding them across the quantization above would cost the
        // registers that let eight waves per SIMD stay resident, and resident waves are what keeps HBM busy here
        // (the tail repeats the last fragment; its products are skipped below)
        v4i wf[U];
        uint32_t swv[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int kc = min(kc0 + u, k_end - 1);
            wf[u] = __builtin_nontemporal_load(wfrag + (int64_t)kc * 64);
            const uint32_t d = *(reinterpret_cast<const uint32_t*>(a.w_scales) + ((int64_t)rb * KS + (kc >> 2)) * 64 + lane);
            swv[u] = d >> (8 * (kc & 3));
        }
        // the chunk's activation fragments in B-operand order (same wave wrote them: LDS operations of a wave are in order)
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (kc0 + u < k_end) {
                // B-operand lane = K-block (lane / 16) of the fragment, row lane % 16
                const int row = lane & 15, pos = (u * 4 + (lane >> 4)) * MP + (row < MP ? row : 0);
                const v4i z = {0, 0, 0, 0};
                const v4i xf = row < MP ? *reinterpret_cast<const v4i*>(sc_codes + pos * 4) : z;
                const uint32_t sx = row < MP ? sc_scales[pos] : 0u;
                const v8i a8 = {wf[u][0], wf[u][1], wf[u][2], wf[u][3], 0, 0, 0, 0};
                const v8i b8 = {xf[0], xf[1], xf[2], xf[3], 0, 0, 0, 0};
                acc = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a8, b8, acc, 4, 4, 0, (int)swv[u], 0, (int)sx);
            }
        }
    }

    *reinterpret_cast<v4f*>(&partial[wave][lane * 4]) = acc;
    __syncthreads();
    for (int e = threadIdx.x; e < 256; e += kFusedWaves * 64) {
        const int l = e >> 2, v = e & 3;
        float s = 0.0f;
#pragma unroll
        for (int w = 0; w < kFusedWaves; ++w) s += partial[w][e];
        s *= a.alpha;
        const int m = l & 15;
        const int n = rb * 16 + (l >> 4) * 4 + v;
        if (m < a.M && n < a.N) {
            if constexpr (OUT_F32) static_cast<float*>(a.out)[(int64_t)m * a.N + n] = s;
            else static_cast<__bf16*>(a.out)[(int64_t)m * a.N + n] = (__bf16)s;
        }
    }
}


// ------------------------------------------------------------------------------------------------------
// Weight-only variant (W4A16) for a handful of tokens: out = bf16(X H_b) Q(W H_b)^T.  The paper's appendix on
// inference regimes recommends weight-only quantization where the layer is memory-bound: activation quantization
// buys no speed there and costs accuracy.  Same streaming of W, same rotation MFMA group per token and chunk; the
// rotated activations are rounded to bf16 instead of quantized, the E2M1 codes of W are decoded with their E8M0
// scale straight to bf16 (exact: two significant bits, bf16 has the exponent range of the scale) and the product runs
// on the bf16 MFMA, four K = 32 instructions per fragment.  The contraction index inside a fragment is permuted the
// same way for both operands (instruction j takes elements 32*kb + 8*j .. +8 of K-block kb), which a dot product
// does not see.
typedef __bf16 v2bf_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ v8bf decode8_bf16(uint32_t codes, float scale)
{
    const v2bf_t p0 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(codes, scale, 0);
    const v2bf_t p1 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(codes, scale, 1);
    const v2bf_t p2 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(codes, scale, 2);
    const v2bf_t p3 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(codes, scale, 3);
    const v8bf r = {p0[0], p0[1], p1[0], p1[1], p2[0], p2[1], p3[0], p3[1]};
    return r;
}

template <bool OUT_F32, int MP>
__global__ __launch_bounds__(kFusedWaves * 64) void gemm_w4a16_decode_kernel(FusedArgs a)
{
    constexpr int U = 4;    // fragments per chunk = 16 vectors of 32
    constexpr int TOK = 4;  // tokens whose loads are in flight together

    // staging: rotated activations in bf16, entry (vector v of the chunk, token m, part q) = 8 values = 16 bytes
    __shared__ __attribute__((aligned(16))) uint32_t st_y[kFusedWaves][16 * MP * 16];
    __shared__ float partial[kFusedWaves][256];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int g = lane & 15, q = lane >> 4;
    const int rb = blockIdx.x;
    const int KC = a.K >> 7, KS = (a.K + 511) >> 9;
    const int per = (KC + kFusedWaves - 1) / kFusedWaves;
    const int k_begin = min(wave * per, KC), k_end = min(k_begin + per, KC);

    v8bf hop[2][1];
    build_hadamard_operand<32>(hop, g, q, a.b < 32 ? a.b : 32);
    const int kron = a.b > 32 ? (a.b == 64 ? 1 : 2) : 0;

    uint32_t* const sy = st_y[wave];
    for (int i = lane; i < 16 * MP * 16; i += 64) sy[i] = 0u;  // rows that belong to no token stay zero

    const v4i* wfrag = reinterpret_cast<const v4i*>(a.w_codes + (int64_t)rb * KC * 1024) + lane;
    v4f acc = {0.f, 0.f, 0.f, 0.f};

    for (int kc0 = k_begin; kc0 < k_end; kc0 += U) {
        const bool v_ok = kc0 + (g >> 2) < k_end;
        const int64_t k_lane = (int64_t)kc0 * 128 + g * 32 + 8 * q;
        for (int m0 = 0; m0 < a.M; m0 += TOK) {
            v4i xin[TOK];
#pragma unroll
            for (int t = 0; t < TOK; ++t) {
                const v4i z = {0, 0, 0, 0};
                const int m = m0 + t;
                xin[t] = (m < a.M && v_ok) ? *reinterpret_cast<const v4i*>(a.x + (int64_t)m * a.K + k_lane) : z;
            }
#pragma unroll
            for (int t = 0; t < TOK; ++t) {
                const int m = m0 + t;
                if (m >= a.M) break;  // uniform
                v4f h[2];
#pragma unroll
                for (int tt = 0; tt < 2; ++tt) {
                    h[tt] = v4f{0.f, 0.f, 0.f, 0.f};
                    h[tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hop[tt][0], __builtin_bit_cast(v8bf, xin[t]), h[tt], 0, 0, 0);
                }
                kronecker_levels<2>(h, g, kron);
                v8bf yb;
#pragma unroll
                for (int tt = 0; tt < 2; ++tt)
#pragma unroll
                    for (int v = 0; v < 4; ++v) yb[4 * tt + v] = (__bf16)__fmaf_rn(h[tt][v], a.c_hi, h[tt][v] * a.c_lo);
                // lane (g, q) holds elements 8q .. 8q+7 of vector g, token m
                *reinterpret_cast<v8bf*>(sy + ((g * MP + m) * 4 + q) * 4) = yb;
            }
        }
        // W fragments and scales of the chunk, asked for only now (registers: see the quantizing kernel above)
        v4i wf[U];
        uint32_t swv[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int kc = min(kc0 + u, k_end - 1);
            wf[u] = __builtin_nontemporal_load(wfrag + (int64_t)kc * 64);
            const uint32_t d = *(reinterpret_cast<const uint32_t*>(a.w_scales) + ((int64_t)rb * KS + (kc >> 2)) * 64 + lane);
            swv[u] = (d >> (8 * (kc & 3))) & 0xffu;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (kc0 + u < k_end) {
                const float wscale = __uint_as_float(swv[u] << 23);  // E8M0 byte as the exponent field of a binary32
                const int row = lane & 15, kb = lane >> 4;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    // lane (row n, kb) of W holds elements 32 kb .. +32 of its row: dword j = elements 32 kb + 8 j .. +8
                    const v8bf w8 = decode8_bf16((uint32_t)wf[u][j], wscale);
                    const v8bf z = {(__bf16)0.f, (__bf16)0.f, (__bf16)0.f, (__bf16)0.f, (__bf16)0.f, (__bf16)0.f, (__bf16)0.f, (__bf16)0.f};
                    // lane (token row, kb) of X: the same elements 32 kb + 8 j .. +8 = part j of vector 4u + kb
                    const v8bf x8 = row < MP ? *reinterpret_cast<const v8bf*>(sy + (((u * 4 + kb) * MP + row) * 4 + j) * 4) : z;
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w8, x8, acc, 0, 0, 0);
                }
            }
        }
    }

    *reinterpret_cast<v4f*>(&partial[wave][lane * 4]) = acc;
    __syncthreads();
    for (int e = threadIdx.x; e < 256; e += kFusedWaves * 64) {
        const int l = e >> 2, v = e & 3;
        float s = 0.0f;
#pragma unroll
        for (int w = 0; w < kFusedWaves; ++w) s += partial[w][e];
        s *= a.alpha;
        const int m = l & 15;
        const int n = rb * 16 + (l >> 4) * 4 + v;
        if (m < a.M && n < a.N) {
            if constexpr (OUT_F32) static_cast<float*>(a.out)[(int64_t)m * a.N + n] = s;
            else static_cast<__bf16*>(a.out)[(int64_t)m * a.N + n] = (__bf16)s;
        }
    }
}

}  // namespace

hipError_t launch_fused_decode(const void* x, int64_t M, int64_t K, int b, const void* w_codes, const void* w_scales,
                               int64_t N, void* out, bool out_f32, bool weight_only, float alpha, hipStream_t st)
{
    FusedArgs a{};
    a.x = static_cast<const uint16_t*>(x);
    a.w_codes = static_cast<const uint8_t*>(w_codes);
    a.w_scales = static_cast<const uint8_t*>(w_scales);
    a.out = out;
    a.M = (int)M;
    a.N = (int)N;
    a.K = (int)K;
    a.b = b;
    const double c = 1.0 / sqrt((double)b);
    a.c_hi = (float)c;
    a.c_lo = (float)(c - (double)a.c_hi);
    a.alpha = alpha;
    const dim3 grid((unsigned)((N + 15) / 16)), block(kFusedWaves * 64);
    if (weight_only) {
        if (M <= 4) {
            if (out_f32) hipLaunchKernelGGL((gemm_w4a16_decode_kernel<true, 4>), grid, block, 0, st, a);
            else hipLaunchKernelGGL((gemm_w4a16_decode_kernel<false, 4>), grid, block, 0, st, a);
        } else {
            if (out_f32) hipLaunchKernelGGL((gemm_w4a16_decode_kernel<true, 16>), grid, block, 0, st, a);
            else hipLaunchKernelGGL((gemm_w4a16_decode_kernel<false, 16>), grid, block, 0, st, a);
        }
    } else if (M <= 4) {
        if (out_f32) hipLaunchKernelGGL((gemm_fused_decode_kernel<true, 4>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((gemm_fused_decode_kernel<false, 4>), grid, block, 0, st, a);
    } else {
        if (out_f32) hipLaunchKernelGGL((gemm_fused_decode_kernel<true, 16>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((gemm_fused_decode_kernel<false, 16>), grid, block, 0, st, a);
    }
    return hipGetLastError();
}

}  // namespace fp4mr
