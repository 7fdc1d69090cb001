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

#include <algorithm>
#include <cmath>

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
    int tn0, tn_count;  // this launch covers the tile columns tn0 .. tn0 + tn_count - 1 (tn_count = 0: all of them)
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
    // the wave index is uniform across the wavefront: telling the compiler keeps every fragment's position in scalar
    // registers, so that the loads below cost no vector address arithmetic (the vector ALU is what bounds this kernel)
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int wm = wave % NWM, wn = wave / NWM;
    const int tm = blockIdx.x % g.tiles_m, tn = g.tn0 + blockIdx.x / g.tiles_m;

    const int64_t KC = g.K >> 7;
    const int KT = (int)KC;
    // Operands are addressed through buffer resources based at the tile's first row-block: one VGPR (16 or 4 times the
    // lane) is the only per-lane address, every fragment's position is a scalar offset.  Row-blocks past the end of an
    // operand (last tile) are clamped to its last row-block: the duplicates only feed outputs that are never stored.
    const int a_rbs = (int)((g.M + 15) / 16), w_rbs = (int)((g.N + 15) / 16);
    const int a_rb0 = min(tm * FX, a_rbs - 1), w_rb0 = min(tn * FW, w_rbs - 1);
    const int a_rb_last = a_rbs - 1 - a_rb0, w_rb_last = w_rbs - 1 - w_rb0;
    auto make_rsrc = [](const uint8_t* base, int64_t bytes) {
        const uint32_t n = bytes > 0xffffffffll ? 0xffffffffu : (uint32_t)bytes;
        return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(base), 0, (int)n, 0x00020000);
    };
    const __amdgpu_buffer_rsrc_t rs_ac = make_rsrc(g.a_codes + (int64_t)a_rb0 * KC * 1024, (int64_t)(a_rbs - a_rb0) * KC * 1024);
    const __amdgpu_buffer_rsrc_t rs_wc = make_rsrc(g.w_codes + (int64_t)w_rb0 * KC * 1024, (int64_t)(w_rbs - w_rb0) * KC * 1024);
    const __amdgpu_buffer_rsrc_t rs_as = make_rsrc(g.a_scales + (int64_t)a_rb0 * KC * 128, (int64_t)(a_rbs - a_rb0) * KC * 128);
    const __amdgpu_buffer_rsrc_t rs_ws = make_rsrc(g.w_scales + (int64_t)w_rb0 * KC * 128, (int64_t)(w_rbs - w_rb0) * KC * 128);
    const uint32_t lane16 = (uint32_t)lane * 16u, lane4 = (uint32_t)(lane & 31) * 4u;
    const int kc_bytes = (int)KC * 1024, ks_bytes = (int)KC * 128;

    v4f acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j) acc[i][j] = v4f{0.f, 0.f, 0.f, 0.f};

    auto issue = [&](int kt) {
        char* base = smem + (kt % STAGES) * STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            const int f = min(wave + i * NW, F - 1);  // spare slots re-copy the last fragment (same bytes to the same place)
            const bool is_x = (FX % NW == 0) ? (i < FX / NW) : (f < FX);
            if (is_x) __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_ac, (lds_void*)(base + f * 1024), 16, lane16, min(f, a_rb_last) * kc_bytes + kt * 1024, 0, 0);
            else __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_wc, (lds_void*)(base + f * 1024), 16, lane16, min(f - FX, w_rb_last) * kc_bytes + kt * 1024, 0, 0);
        }
        // direct-to-LDS loads place lane l's data at 4*l whatever the access size is below a dword, so a 128-byte scale
        // block is copied as 32 lanes x 4 bytes (the upper half-wave is masked off; one branch for all the blocks)
        if (lane < 32) {
#pragma unroll
            for (int i = 0; i < LPW; ++i) {
                const int f = min(wave + i * NW, F - 1);
                const bool is_x = (FX % NW == 0) ? (i < FX / NW) : (f < FX);
                if (is_x) __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_as, (lds_void*)(base + SCALE_OFF + f * 128), 4, lane4, min(f, a_rb_last) * ks_bytes + kt * 128, 0, 0);
                else __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_ws, (lds_void*)(base + SCALE_OFF + f * 128), 4, lane4, min(f - FX, w_rb_last) * ks_bytes + kt * 128, 0, 0);
            }
        }
    };

#pragma unroll
    for (int s = 0; s < STAGES - 1; ++s)
        if (s < KT) issue(s);

    // The X fragments of a step are read from LDS (as codes) at the end of the step before, so that their latency runs
    // under that step's last MFMAs instead of stalling both waves of a SIMD at the top of the step; that needs stage
    // kt + 1 in LDS when step kt starts, so one stage (not two) may be in flight at the top of a step.
    static_assert(STAGES >= 4, "one stage in flight, one being read ahead, one being consumed, one being refilled");
    v4i xcode[TM];
    uint32_t xscale[TM];
    auto read_x = [&](int kt) {
        const char* base = smem + (kt % STAGES) * STAGE_BYTES;
#pragma unroll
        for (int j = 0; j < TM; ++j) {
            const int f = wm * TM + j;
            xcode[j] = *(reinterpret_cast<const v4i*>(base + f * 1024) + lane);
            xscale[j] = *(reinterpret_cast<const uint16_t*>(base + SCALE_OFF + f * 128) + lane);
        }
    };
    // stage 0: with all STAGES - 1 stages of the prologue issued, the STAGES - 2 behind it may still be in flight
    if (KT >= STAGES - 1) wait_vmcnt<(STAGES - 2) * 2 * LPW>(); else wait_vmcnt<0>();
    block_barrier();
    read_x(0);

    for (int kt = 0; kt < KT; ++kt) {
        if (kt + STAGES - 2 < KT) wait_vmcnt<(STAGES - 3) * 2 * LPW>(); else wait_vmcnt<0>();  // stage kt + 1 has landed
        block_barrier();
        if (kt + STAGES - 1 < KT) issue(kt + STAGES - 1);

        const char* base = smem + (kt % STAGES) * STAGE_BYTES;
        NvFrag16 xf[TM];
#pragma unroll
        for (int j = 0; j < TM; ++j) xf[j] = nv_dequant_frag(xcode[j], xscale[j]);
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
        read_x(kt + 1);  // (past the last step: stale bytes of the ring that nothing consumes)
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
    const int cols = g.tn_count > 0 ? std::min(g.tn_count, g.tiles_n - g.tn0) : g.tiles_n - g.tn0;
    if (cols <= 0) return hipSuccess;
    const dim3 grid((unsigned)(g.tiles_m * cols));
    hipError_t e;
    static LdsAttrOnce raised[2];  // the dynamic-LDS limit of a kernel is raised once per device, not on every launch
    if (out_f32) {
        auto k = gemm_nv_kernel<BM, BN, WM, WN, STAGES, true>;
        if ((e = raised[1].ensure(reinterpret_cast<const void*>(k), (int)lds)) != hipSuccess) return e;
        hipLaunchKernelGGL(k, grid, dim3(threads), lds, st, g);
    } else {
        auto k = gemm_nv_kernel<BM, BN, WM, WN, STAGES, false>;
        if ((e = raised[0].ensure(reinterpret_cast<const void*>(k), (int)lds)) != hipSuccess) return e;
        hipLaunchKernelGGL(k, grid, dim3(threads), lds, st, g);
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm_nvfp4(const void* a_codes, const void* a_scales, const float* a_ts, const void* w_codes,
                             const void* w_scales, const float* w_ts, int64_t M, int64_t N, int64_t K, void* out,
                             bool out_f32, int variant, void* workspace, void* partial, hipStream_t st)
{
    // By default many-token products go to the kernel that takes its activations as fp16 (gemm_nv16.hip); the tile
    // kernels of this file, which dequantize both operands inside the product, remain as forced configurations.
    if (variant == 0) return launch_gemm_nv16(a_codes, a_scales, a_ts, w_codes, w_scales, w_ts, M, N, K, out, out_f32, workspace, partial, st);
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
    switch (variant) {
        case 1: return launch_variant<128, 128, 64, 64, 4>(g, out_f32, st);
        case 2: return launch_variant<16, 256, 16, 64, 4>(g, out_f32, st);
        case 3: return launch_variant<256, 256, 64, 128, 4>(g, out_f32, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace fp4mr
