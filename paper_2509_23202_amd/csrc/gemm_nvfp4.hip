// NVFP4 W4A4 GEMM (arXiv 2509.23202, Section 2 "The NVFP4 Format", Section 4.1 "Ingredient 1":
// Xhat = s_T * s_G * Q(.), groups of 16 with E4M3 scales plus one fp32 tensor scale per operand).
//
//   out[m,n] = sT_a * sT_w * sum_k (sa[m,k/16] * a[m,k]) * (sw[n,k/16] * w[n,k])
//
// CDNA4's block-scaled MFMA applies one power-of-two scale per 32 elements, so it cannot consume E4M3 scales on
// 16-element groups.  Here each fragment is dequantized in registers to fp16 -- exact: an E2M1 value times an
// E4M3 value has at most 6 significant bits and lies in [2^-10, 2688] -- and multiplied on the fp16 MFMA
// (v_mfma_f32_16x16x32_f16) with fp32 accumulation; the two tensor scales are applied once in the epilogue.
// Codes keep the 4.5-bit memory footprint all the way into the registers, so the weight-streaming (small M)
// regime gets the full bandwidth saving; the large-M regime is bounded by the fp16 MFMA rate, not the FP4 one.
//
// Data movement is the same as in the MXFP4 kernel: 1 KB code fragments and 128-byte scale blocks (two E4M3
// bytes per lane, copied by half a wave as dwords) go global -> LDS with direct-to-LDS loads into a ring, one
// barrier per K-step of 128.
// The contraction index inside a fragment is permuted (lane q, dword s, element e <-> k = 32q + 8s + e for both
// operands alike), which a dot product does not see.
#include "device_util.hpp"
#include "internal.hpp"
#include "layout.hpp"
#include "nv_dequant.hpp"

namespace fp4mr {
namespace {

struct NvGemmArgs {
    const uint8_t* a_codes;
    const uint8_t* a_scales;
    const uint8_t* w_codes;
    const uint8_t* w_scales;
    const float* a_ts;
    const float* w_ts;
    void* out;
    int64_t M, N, K;
    int tiles_m, tiles_n;
};

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0f70);
}

__device__ __forceinline__ void block_barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void global_void;

template <int BM, int BN, int WM, int WN, int STAGES, bool OUT_F32>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64) void gemm_nv_kernel(NvGemmArgs g)
{
    constexpr int NWM = BM / WM, NWN = BN / WN, NW = NWM * NWN;
    constexpr int FX = BM / 16, FW = BN / 16, F = FX + FW;
    constexpr int LPW = (F + NW - 1) / NW;
    constexpr int TM = WM / 16, TN = WN / 16;
    constexpr int STAGE_BYTES = F * (1024 + 128);  // codes then scales
    constexpr int SCALE_OFF = F * 1024;

    extern __shared__ __attribute__((aligned(1024))) char smem[];

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int wm = wave % NWM, wn = wave / NWM;
    const int tm = blockIdx.x % g.tiles_m, tn = blockIdx.x / g.tiles_m;

    const int64_t KC = g.K >> 7;
    const int KT = (int)KC;
    const int64_t rbx_max = (g.M + 15) / 16 - 1, rbw_max = (g.N + 15) / 16 - 1;

    const uint8_t* gsrc[LPW];
    const uint8_t* ssrc[LPW];
    int foff[LPW];
#pragma unroll
    for (int i = 0; i < LPW; ++i) {
        const int f = min(wave + i * NW, F - 1);
        int64_t rb;
        const uint8_t *cbase, *sbase;
        if (f < FX) {
            rb = (int64_t)tm * FX + f;
            rb = rb > rbx_max ? rbx_max : rb;
            cbase = g.a_codes;
            sbase = g.a_scales;
        } else {
            rb = (int64_t)tn * FW + (f - FX);
            rb = rb > rbw_max ? rbw_max : rb;
            cbase = g.w_codes;
            sbase = g.w_scales;
        }
        gsrc[i] = cbase + rb * KC * 1024 + lane * 16;
        ssrc[i] = sbase + rb * KC * 128 + (lane & 31) * 4;
        foff[i] = f;
    }

    v4f acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j) acc[i][j] = v4f{0.f, 0.f, 0.f, 0.f};

    auto issue = [&](int kt) {
        char* base = smem + (kt % STAGES) * STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            __builtin_amdgcn_global_load_lds((global_void*)(gsrc[i] + (int64_t)kt * 1024), (lds_void*)(base + foff[i] * 1024), 16, 0, 0);
            // direct-to-LDS loads place lane l's data at 4*l whatever the access size is below a dword, so the
            // 128-byte scale block is copied as 32 lanes x 4 bytes (the upper half-wave is masked off)
            if (lane < 32)
                __builtin_amdgcn_global_load_lds((global_void*)(ssrc[i] + (int64_t)kt * 128), (lds_void*)(base + SCALE_OFF + foff[i] * 128), 4, 0, 0);
        }
    };

#pragma unroll
    for (int s = 0; s < STAGES - 1; ++s)
        if (s < KT) issue(s);

    for (int kt = 0; kt < KT; ++kt) {
        if (kt + STAGES - 2 < KT) wait_vmcnt<(STAGES - 2) * 2 * LPW>(); else wait_vmcnt<0>();
        block_barrier();
        if (kt + STAGES - 1 < KT) issue(kt + STAGES - 1);

        const char* base = smem + (kt % STAGES) * STAGE_BYTES;
        NvFrag16 xf[TM];
#pragma unroll
        for (int j = 0; j < TM; ++j) {
            const int f = wm * TM + j;
            const v4i c = *(reinterpret_cast<const v4i*>(base + f * 1024) + lane);
            const uint32_t sc = *(reinterpret_cast<const uint16_t*>(base + SCALE_OFF + f * 128) + lane);
            xf[j] = nv_dequant_frag(c, sc);
        }
#pragma unroll
        for (int i = 0; i < TN; ++i) {
            const int f = FX + wn * TN + i;
            const v4i c = *(reinterpret_cast<const v4i*>(base + f * 1024) + lane);
            const uint32_t sc = *(reinterpret_cast<const uint16_t*>(base + SCALE_OFF + f * 128) + lane);
            const NvFrag16 wf = nv_dequant_frag(c, sc);
#pragma unroll
            for (int j = 0; j < TM; ++j)
#pragma unroll
                for (int s = 0; s < 4; ++s)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(wf.s[s], xf[j].s[s], acc[i][j], 0, 0, 0);
        }
    }

    const float ts = (*g.a_ts) * (*g.w_ts);
    const int64_t m_base = (int64_t)tm * BM + wm * WM + (lane & 15);
    const int64_t n_base = (int64_t)tn * BN + wn * WN + (lane >> 4) * 4;
#pragma unroll
    for (int j = 0; j < TM; ++j) {
        const int64_t m = m_base + 16 * j;
        if (m >= g.M) continue;
#pragma unroll
        for (int i = 0; i < TN; ++i) {
            const int64_t n = n_base + 16 * i;
            if (n >= g.N) continue;
            v4f v = acc[i][j];
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] *= ts;
            if constexpr (OUT_F32) {
                float* o = static_cast<float*>(g.out) + m * g.N + n;
                if (n + 3 < g.N && (g.N & 3) == 0) {
                    *reinterpret_cast<float4*>(o) = make_float4(v[0], v[1], v[2], v[3]);
                } else {
                    for (int e = 0; e < 4; ++e)
                        if (n + e < g.N) o[e] = v[e];
                }
            } else {
                __bf16* o = static_cast<__bf16*>(g.out) + m * g.N + n;
                typedef __bf16 v4bf __attribute__((ext_vector_type(4)));
                if (n + 3 < g.N && (g.N & 3) == 0) {
                    v4bf p = {(__bf16)v[0], (__bf16)v[1], (__bf16)v[2], (__bf16)v[3]};
                    *reinterpret_cast<v4bf*>(o) = p;
                } else {
                    for (int e = 0; e < 4; ++e)
                        if (n + e < g.N) o[e] = (__bf16)v[e];
                }
            }
        }
    }
}

template <int BM, int BN, int WM, int WN, int STAGES>
hipError_t launch_variant(const NvGemmArgs& g0, bool out_f32, hipStream_t st)
{
    NvGemmArgs g = g0;
    g.tiles_m = (int)((g.M + BM - 1) / BM);
    g.tiles_n = (int)((g.N + BN - 1) / BN);
    constexpr int threads = (BM / WM) * (BN / WN) * 64;
    constexpr size_t lds = (size_t)STAGES * (BM + BN) / 16 * (1024 + 128);
    const dim3 grid((unsigned)(g.tiles_m * g.tiles_n));
    hipError_t e;
    if (out_f32) {
        auto k = gemm_nv_kernel<BM, BN, WM, WN, STAGES, true>;
        if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)) != hipSuccess) return e;
        hipLaunchKernelGGL(k, grid, dim3(threads), lds, st, g);
    } else {
        auto k = gemm_nv_kernel<BM, BN, WM, WN, STAGES, false>;
        if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)) != hipSuccess) return e;
        hipLaunchKernelGGL(k, grid, dim3(threads), lds, st, g);
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm_nvfp4(const void* a_codes, const void* a_scales, const float* a_ts, const void* w_codes,
                             const void* w_scales, const float* w_ts, int64_t M, int64_t N, int64_t K, void* out,
                             bool out_f32, int variant, hipStream_t st)
{
    NvGemmArgs g{};
    g.a_codes = static_cast<const uint8_t*>(a_codes);
    g.a_scales = static_cast<const uint8_t*>(a_scales);
    g.w_codes = static_cast<const uint8_t*>(w_codes);
    g.w_scales = static_cast<const uint8_t*>(w_scales);
    g.a_ts = a_ts;
    g.w_ts = w_ts;
    g.out = out;
    g.M = M;
    g.N = N;
    g.K = K;
    if (variant == 0) variant = (M <= 16) ? 2 : 1;
    switch (variant) {
        case 1: return launch_variant<128, 128, 64, 64, 4>(g, out_f32, st);
        case 2: return launch_variant<16, 256, 16, 64, 4>(g, out_f32, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace fp4mr
