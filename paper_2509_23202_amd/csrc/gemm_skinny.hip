// W4A4 GEMM for few tokens (M <= 64): the weight-streaming regime (arXiv 2509.23202, appendix on inference regimes:
// at small batch the layer is memory-bound).  out[m,n] = sum_k Ahat[m,k] * What[n,k], both formats.
//
// The weights are read exactly once, straight from global memory into registers: a workgroup owns one 16-column
// block of the output (one row-block of W, whose fragments are contiguous along K in GEMM layout), its 8 waves split K,
// and every wave issues one coalesced 1 KB load per fragment with several fragments in flight.  X (a few KB per K-step)
// comes from L2.  Each W fragment is multiplied against up to four 16-row X fragments (MT), so M <= 64 streams W once.
// Partial sums of the 8 waves meet in LDS and are added in a fixed order (deterministic), then written as bf16/fp32.
// No split-K workspace, no atomics, one launch.
#include "device_util.hpp"
#include "internal.hpp"
#include "layout.hpp"
#include "nv_dequant.hpp"

namespace fp4mr {
namespace {

constexpr int kSkinnyWaves = 8;

struct SkinnyArgs {
    const uint8_t* a_codes;
    const uint8_t* a_scales;
    const uint8_t* w_codes;
    const uint8_t* w_scales;
    const float* a_ts;
    const float* w_ts;
    void* out;
    int M, N, K;
    float alpha;  // MXFP4: factor on the result (powers of 4/3 for operands whose scales carry the tensor-level 4/3), else 1
};

template <int FMT, int MT, bool OUT_F32>
__global__ __launch_bounds__(kSkinnyWaves * 64) void gemm_skinny_kernel(SkinnyArgs g)
{
    constexpr int U = 4;  // fragments in flight per wave
    __shared__ float partial[kSkinnyWaves][MT][256];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int rb = blockIdx.x;  // row-block of W = 16 output columns
    const int KC = g.K >> 7, KS = (g.K + 511) >> 9;
    const int per = (KC + kSkinnyWaves - 1) / kSkinnyWaves;
    const int k_begin = min(wave * per, KC), k_end = min(k_begin + per, KC);

    const v4i* wfrag = reinterpret_cast<const v4i*>(g.w_codes + (int64_t)rb * KC * 1024) + lane;
    const v4i* xfrag = reinterpret_cast<const v4i*>(g.a_codes) + lane;
    const int a_rbs = (g.M + 15) >> 4;

    v4f acc[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) acc[t] = v4f{0.f, 0.f, 0.f, 0.f};

    for (int kc0 = k_begin; kc0 < k_end; kc0 += U) {
        v4i wf[U], xf[U][MT];
        uint32_t swv[U], sxv[U][MT];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int kc = min(kc0 + u, k_end - 1);  // the tail repeats the last fragment; its products are skipped below
            wf[u] = __builtin_nontemporal_load(wfrag + (int64_t)kc * 64);
            if constexpr (FMT == 0) {
                const uint32_t d = *(reinterpret_cast<const uint32_t*>(g.w_scales) + ((int64_t)rb * KS + (kc >> 2)) * 64 + lane);
                swv[u] = d >> (8 * (kc & 3));
            } else {
                swv[u] = *(reinterpret_cast<const uint16_t*>(g.w_scales) + ((int64_t)rb * KC + kc) * 64 + lane);
            }
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                const int mrb = min(t, a_rbs - 1);
                xf[u][t] = xfrag[((int64_t)mrb * KC + kc) * 64];
                if constexpr (FMT == 0) {
                    const uint32_t d = *(reinterpret_cast<const uint32_t*>(g.a_scales) + ((int64_t)mrb * KS + (kc >> 2)) * 64 + lane);
                    sxv[u][t] = d >> (8 * (kc & 3));
                } else {
                    sxv[u][t] = *(reinterpret_cast<const uint16_t*>(g.a_scales) + ((int64_t)mrb * KC + kc) * 64 + lane);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (kc0 + u < k_end) {
                if constexpr (FMT == 0) {
                    const v8i a8 = {wf[u][0], wf[u][1], wf[u][2], wf[u][3], 0, 0, 0, 0};
#pragma unroll
                    for (int t = 0; t < MT; ++t) {
                        const v8i b8 = {xf[u][t][0], xf[u][t][1], xf[u][t][2], xf[u][t][3], 0, 0, 0, 0};
                        acc[t] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a8, b8, acc[t], 4, 4, 0, (int)swv[u], 0, (int)sxv[u][t]);
                    }
                } else {
                    const NvFrag16 w16 = nv_dequant_frag(wf[u], swv[u]);
#pragma unroll
                    for (int t = 0; t < MT; ++t) {
                        const NvFrag16 x16 = nv_dequant_frag(xf[u][t], sxv[u][t]);
#pragma unroll
                        for (int s = 0; s < 4; ++s)
                            acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(w16.s[s], x16.s[s], acc[t], 0, 0, 0);
                    }
                }
            }
        }
    }

#pragma unroll
    for (int t = 0; t < MT; ++t)
        *reinterpret_cast<v4f*>(&partial[wave][t][lane * 4]) = acc[t];
    __syncthreads();

    float ts = g.alpha;
    if constexpr (FMT == 1) ts = (*g.a_ts) * (*g.w_ts);
    for (int e = threadIdx.x; e < MT * 256; e += kSkinnyWaves * 64) {
        const int t = e >> 8, r = e & 255, l = r >> 2, v = r & 3;
        float s = 0.0f;
#pragma unroll
        for (int w = 0; w < kSkinnyWaves; ++w) s += partial[w][t][r];
        s *= ts;
        const int m = t * 16 + (l & 15);
        const int n = rb * 16 + (l >> 4) * 4 + v;
        if (m < g.M && n < g.N) {
            if constexpr (OUT_F32) static_cast<float*>(g.out)[(int64_t)m * g.N + n] = s;
            else static_cast<__bf16*>(g.out)[(int64_t)m * g.N + n] = (__bf16)s;
        }
    }
}

template <int FMT, int MT>
hipError_t launch_mt(const SkinnyArgs& g, bool out_f32, hipStream_t st)
{
    const dim3 grid((unsigned)((g.N + 15) / 16)), block(kSkinnyWaves * 64);
    if (out_f32) hipLaunchKernelGGL((gemm_skinny_kernel<FMT, MT, true>), grid, block, 0, st, g);
    else hipLaunchKernelGGL((gemm_skinny_kernel<FMT, MT, false>), grid, block, 0, st, g);
    return hipGetLastError();
}

template <int FMT>
hipError_t launch_fmt(const SkinnyArgs& g, bool out_f32, hipStream_t st)
{
    const int mt = (g.M + 15) / 16;
    switch (mt) {
        case 1: return launch_mt<FMT, 1>(g, out_f32, st);
        case 2: return launch_mt<FMT, 2>(g, out_f32, st);
        case 3: return launch_mt<FMT, 3>(g, out_f32, st);
        case 4: return launch_mt<FMT, 4>(g, out_f32, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

hipError_t launch_gemm_skinny(const void* a_codes, const void* a_scales, const float* a_ts, const void* w_codes,
                              const void* w_scales, const float* w_ts, int64_t M, int64_t N, int64_t K, int fmt, void* out,
                              bool out_f32, float alpha, hipStream_t st)
{
    SkinnyArgs g{};
    g.alpha = alpha;
    g.a_codes = static_cast<const uint8_t*>(a_codes);
    g.a_scales = static_cast<const uint8_t*>(a_scales);
    g.w_codes = static_cast<const uint8_t*>(w_codes);
    g.w_scales = static_cast<const uint8_t*>(w_scales);
    g.a_ts = a_ts;
    g.w_ts = w_ts;
    g.out = out;
    g.M = (int)M;
    g.N = (int)N;
    g.K = (int)K;
    return fmt == 0 ? launch_fmt<0>(g, out_f32, st) : launch_fmt<1>(g, out_f32, st);
}

}  // namespace fp4mr
