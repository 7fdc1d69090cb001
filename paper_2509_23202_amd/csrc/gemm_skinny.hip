// W4A4 GEMM for few tokens (M <= 64, and up to 128 on narrow MXFP4 layers): the weight-streaming regime (arXiv 2509.23202, appendix on inference regimes:
// at small batch the layer is memory-bound).  out[m,n] = sum_k Ahat[m,k] * What[n,k], both formats.
//
// The weights are read exactly once, straight from global memory into registers: a workgroup owns one 16-column
// block of the output (one row-block of W, whose fragments are contiguous along K in GEMM layout), its 8 waves split K,
// and every wave issues one coalesced 1 KB load per fragment with several fragments in flight.  X (a few KB per K-step)
// comes from L2.  Each W fragment is multiplied against up to four 16-row X fragments (MT), so M <= 64 streams W once.
// Partial sums of the 8 waves meet in LDS and are added in a fixed order (deterministic), then written as bf16/fp32.
// No split-K workspace, no atomics, one launch.
//
// Three kernels share that scheme.  gemm_skinny_kernel launches one workgroup per row-block; its loads drain before the
// reduction, so each workgroup pays one memory latency with nothing in flight.  gemm_stream_kernel (MXFP4) keeps one
// workgroup per compute unit resident, walks the row-blocks with a stride, holds the activations in registers for the
// whole launch and two or three register batches of W per wave in rotation, so the loads of the next batches are in flight
// while the current one is multiplied and its row-block's partial sums meet in LDS.  gemm_skinny_nt_kernel (NVFP4; MXFP4
// where the activations do not fit the registers) gives a workgroup two row-blocks so that each X fragment serves two W
// fragments.  All add the eight partials in wave order: bit-identical results.
#include "device_util.hpp"
#include "internal.hpp"
#include "layout.hpp"
#include "nv_dequant.hpp"

#include <algorithm>
#include <type_traits>

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
    int parts;    // persistent kernel: > 1 = the token blocks are shared out between that many sets of workgroups, else 0 or 1
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

// ------------------------------------------------------------------------------------------------------
// NVFP4, up to 16 tokens.  The in-register dequantization (16 conversions, 16 packed multiplies and two scale decodes per
// fragment and operand) is what bounds the kernel above in this format: about 100 vector instructions per 1 KB of W, half
// of them spent on the X fragment, which is the same for every row-block.  Here a workgroup owns NT adjacent row-blocks
// and a wave multiplies each dequantized X fragment against the NT W fragments of its K position, so the X share of the
// arithmetic drops to 1/NT.  Same K split over the waves, same order of additions per output: bit-identical to the
// kernel above.  Row-blocks past the end of W (odd counts) re-read the last one and are not stored.
// MT = 16-token blocks of X (M <= 16 MT): every W fragment meets MT dequantized X fragments, each of them shared by the NT
// row-blocks (the arithmetic per KB of W is 48 (1 + MT / NT) instructions instead of 48 (1 + MT)).
// FMT 0 (MXFP4, two to four token blocks): no dequantization there, but the X fragments come from L2 once per W fragment in
// the kernel above and once per NT of them here.
template <int FMT, int NT, int MT, bool OUT_F32, bool PF = false>
__global__ __launch_bounds__(kSkinnyWaves * 64) void gemm_skinny_nt_kernel(SkinnyArgs g)
{
    constexpr int U = MT == 1 ? 4 : 2;  // K positions in flight per wave (NT W fragments and MT X fragments each)
    __shared__ float partial[kSkinnyWaves][NT * MT][256];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int n_rb = (g.N + 15) >> 4;
    const int a_rbs = (g.M + 15) >> 4;
    const int rb0 = blockIdx.x * NT;
    const int KC = g.K >> 7, KS = (g.K + 511) >> 9;
    const int per = (KC + kSkinnyWaves - 1) / kSkinnyWaves;
    const int k_begin = min(wave * per, KC), k_end = min(k_begin + per, KC);

    // scale of fragment kc of a row-block: NVFP4 two bytes per lane and fragment; MXFP4 one dword per lane and four
    // fragments, the fragment's byte shifted down to bits 7:0 (where the MFMA's op_sel 0 reads it)
    auto load_scale = [&](const uint8_t* row_block_scales, int kc) -> uint32_t {
        if constexpr (FMT == 1) return *(reinterpret_cast<const uint16_t*>(row_block_scales) + (int64_t)kc * 64 + lane);
        else return *(reinterpret_cast<const uint32_t*>(row_block_scales) + (int64_t)(kc >> 2) * 64 + lane) >> (8 * (kc & 3));
    };
    const int64_t sc_rb_bytes = FMT == 1 ? (int64_t)KC * 128 : (int64_t)KS * 256;

    const v4i* xfrag[MT];
    const uint8_t* xsc[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        const int mrb = min(t, a_rbs - 1);  // (token blocks past the end re-read the last one and are not stored)
        xfrag[t] = reinterpret_cast<const v4i*>(g.a_codes + (int64_t)mrb * KC * 1024) + lane;
        xsc[t] = g.a_scales + mrb * sc_rb_bytes;
    }
    const v4i* wfrag[NT];
    const uint8_t* wsc[NT];
#pragma unroll
    for (int r = 0; r < NT; ++r) {
        const int rb = min(rb0 + r, n_rb - 1);
        wfrag[r] = reinterpret_cast<const v4i*>(g.w_codes + (int64_t)rb * KC * 1024) + lane;
        wsc[r] = g.w_scales + rb * sc_rb_bytes;
    }

    v4f acc[NT][MT];
#pragma unroll
    for (int r = 0; r < NT; ++r)
#pragma unroll
        for (int t = 0; t < MT; ++t) acc[r][t] = v4f{0.f, 0.f, 0.f, 0.f};

    struct Fetch {
        v4i wf[U][NT], xf[U][MT];
        uint32_t swv[U][NT], sxv[U][MT];
    };
    // (a position past the wave's share repeats the last fragment -- valid memory, from L2 -- and its products are skipped)
    auto fetch = [&](Fetch& f, int kc0) {
        auto& wf = f.wf;
        auto& xf = f.xf;
        auto& swv = f.swv;
        auto& sxv = f.sxv;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int kc = min(kc0 + u, k_end - 1);  // the tail repeats the last fragment; its products are skipped below
#pragma unroll
            for (int r = 0; r < NT; ++r) {
                wf[u][r] = __builtin_nontemporal_load(wfrag[r] + (int64_t)kc * 64);
                swv[u][r] = load_scale(wsc[r], kc);
            }
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                xf[u][t] = xfrag[t][(int64_t)kc * 64];
                sxv[u][t] = load_scale(xsc[t], kc);
            }
        }
    };
    auto multiply = [&](const Fetch& f, int kc0) {
        const auto& wf = f.wf;
        const auto& xf = f.xf;
        const auto& swv = f.swv;
        const auto& sxv = f.sxv;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (kc0 + u < k_end) {
                if constexpr (FMT == 0) {
#pragma unroll
                    for (int t = 0; t < MT; ++t) {
                        const v8i b8 = {xf[u][t][0], xf[u][t][1], xf[u][t][2], xf[u][t][3], 0, 0, 0, 0};
#pragma unroll
                        for (int r = 0; r < NT; ++r) {
                            const v8i a8 = {wf[u][r][0], wf[u][r][1], wf[u][r][2], wf[u][r][3], 0, 0, 0, 0};
                            acc[r][t] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a8, b8, acc[r][t], 4, 4, 0, (int)swv[u][r], 0, (int)sxv[u][t]);
                        }
                    }
                } else if constexpr (MT == 1) {
                    // one X fragment: dequantize it once, then one W fragment at a time (fewest live registers)
                    const NvFrag16 x16 = nv_dequant_frag(xf[u][0], sxv[u][0]);
#pragma unroll
                    for (int r = 0; r < NT; ++r) {
                        const NvFrag16 w16 = nv_dequant_frag(wf[u][r], swv[u][r]);
#pragma unroll
                        for (int s = 0; s < 4; ++s)
                            acc[r][0] = __builtin_amdgcn_mfma_f32_16x16x32_f16(w16.s[s], x16.s[s], acc[r][0], 0, 0, 0);
                    }
                } else {
                    NvFrag16 w16[NT];
#pragma unroll
                    for (int r = 0; r < NT; ++r) w16[r] = nv_dequant_frag(wf[u][r], swv[u][r]);
#pragma unroll
                    for (int t = 0; t < MT; ++t) {
                        const NvFrag16 x16 = nv_dequant_frag(xf[u][t], sxv[u][t]);
#pragma unroll
                        for (int r = 0; r < NT; ++r)
#pragma unroll
                            for (int s = 0; s < 4; ++s)
                                acc[r][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(w16[r].s[s], x16.s[s], acc[r][t], 0, 0, 0);
                    }
                }
            }
        }
    };
    if constexpr (PF) {
        // Two register sets: the loads of the next U positions are issued -- unconditionally, so that the compiler's wait
        // in front of the current products leaves them in flight -- before the current ones are multiplied.  For launches
        // with at most one workgroup per compute unit, where no other workgroup's loads hide this one's latency.
        Fetch a, b;
        if (k_begin < k_end) {
            fetch(a, k_begin);
            for (int kc0 = k_begin;; kc0 += 2 * U) {
                fetch(b, kc0 + U);
                multiply(a, kc0);
                if (kc0 + U >= k_end) break;
                fetch(a, kc0 + 2 * U);
                multiply(b, kc0 + U);
                if (kc0 + 2 * U >= k_end) break;
            }
        }
    } else {
        for (int kc0 = k_begin; kc0 < k_end; kc0 += U) {
            Fetch f;
            fetch(f, kc0);
            multiply(f, kc0);
        }
    }

#pragma unroll
    for (int r = 0; r < NT; ++r)
#pragma unroll
        for (int t = 0; t < MT; ++t)
            *reinterpret_cast<v4f*>(&partial[wave][r * MT + t][lane * 4]) = acc[r][t];
    __syncthreads();

    float ts = g.alpha;
    if constexpr (FMT == 1) ts = (*g.a_ts) * (*g.w_ts);
    for (int e = threadIdx.x; e < NT * MT * 256; e += kSkinnyWaves * 64) {
        const int rt = e >> 8, r = rt / MT, t = rt - r * MT, q = e & 255, l = q >> 2, v = q & 3;
        float s = 0.0f;
#pragma unroll
        for (int w = 0; w < kSkinnyWaves; ++w) s += partial[w][rt][q];
        s *= ts;
        const int m = t * 16 + (l & 15);
        const int n = (rb0 + r) * 16 + (l >> 4) * 4 + v;
        if (m < g.M && n < g.N) {
            if constexpr (OUT_F32) static_cast<float*>(g.out)[(int64_t)m * g.N + n] = s;
            else static_cast<__bf16*>(g.out)[(int64_t)m * g.N + n] = (__bf16)s;
        }
    }
}

// ------------------------------------------------------------------------------------------------------
// The same decomposition as above -- a workgroup per 16-column block of the output, its 8 waves splitting K, partial sums
// added through LDS in a fixed order -- but the workgroups are PERSISTENT: one per compute unit, each walking the row-blocks
// of W with a stride of the grid.  A one-shot workgroup streams 32 KB (K = 4096) and spends most of its life on its own
// start-up, its load latency and its reduction, none of which overlap; here the loads of the next batches of fragments (of
// this row-block or the next) are in flight while the current batch is multiplied and while the row-block's partial sums
// are reduced and stored, so HBM sees a continuous stream.  Register buffers of U fragments each (W codes and scales); the
// barrier per row-block is a bare s_barrier (no vmcnt drain) and the partial sums are double-buffered in LDS, so one
// barrier per row-block suffices.  Bit-identical to the one-shot kernel (same K split, same order of additions).
// XRES: the wave's share of K is at most NB batches of U fragments, and since that share is the same for every row-block
// its X fragments -- of MT 16-token blocks -- are loaded once and stay in registers: a batch is W only, a W fragment meets
// all MT blocks, and nothing of X is read again for the rest of the launch (the one-shot kernels fetch MT X fragments from
// L2 per W fragment).  !XRES (MT = 1, any K): the X fragments travel with W in the batches, two buffers.
template <int FMT, bool OUT_F32, int U, bool XRES, int MT = 1, int NB = 1>
__global__ __launch_bounds__(kSkinnyWaves * 64) void gemm_stream_kernel(SkinnyArgs g)
{
    static_assert(MT == 1 || XRES, "several token blocks only with the X fragments resident");
    static_assert(NB == 1 || XRES, "a static number of batches per row-block only with the X fragments resident");
    static_assert(FMT == 0 || !XRES || MT == 1, "NVFP4 keeps one token block resident (as fp16: 16 registers per fragment)");
    __shared__ float partial[2][kSkinnyWaves][MT][256];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int KC = g.K >> 7, KS = (g.K + 511) >> 9;
    const int per = (KC + kSkinnyWaves - 1) / kSkinnyWaves;
    const int k_begin = min(wave * per, KC), k_end = min(k_begin + per, KC);
    const int nb = (k_end - k_begin + U - 1) / U;       // batches per row-block for this wave (0 for a wave without a K share)
    const int n_rb = (g.N + 15) >> 4;
    // Several sets of workgroups (g.parts = P > 1), each with its own MT token blocks: workgroups 8 P j .. 8 P j + 7 are
    // walkers 8 j .. 8 j + 7 of the first set, the next eight the same walkers of the second set, and so on, so the
    // workgroups that stream the same row-block of W start on the same XCD (workgroups go to the eight XCDs in turn) a
    // dispatch apart: all but the first find the fragments in that XCD's L2.
    int walker = (int)blockIdx.x, G = (int)gridDim.x, tb0 = 0;
    if (g.parts > 1) {
        const int group = (int)(blockIdx.x >> 3);
        walker = (group / g.parts) * 8 + (int)(blockIdx.x & 7);
        G = (int)gridDim.x / g.parts;
        tb0 = (group % g.parts) * MT;
    }

    // Buffer resources: the only per-lane addresses are 16 / 4 / 2 times the lane id, every fragment's position is a scalar
    // offset (64-bit per-load addresses in vector registers would cost the occupancy this kernel lives on).
    auto make_rsrc = [](const uint8_t* base, int64_t bytes) {
        const uint32_t n = bytes > 0xffffffffll ? 0xffffffffu : (uint32_t)bytes;
        return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(base), 0, (int)n, 0x00020000);
    };
    constexpr int SCB = FMT == 0 ? 256 : 128;            // scale bytes per (row-block, MXFP4: four fragments / NVFP4: fragment)
    const int sc_per_rb = FMT == 0 ? KS : KC;
    const int a_rbs = (g.M + 15) >> 4;
    const __amdgpu_buffer_rsrc_t rs_x = make_rsrc(g.a_codes, (int64_t)a_rbs * KC * 1024);
    const __amdgpu_buffer_rsrc_t rs_xs = make_rsrc(g.a_scales, (int64_t)a_rbs * sc_per_rb * SCB);
    const int lane16 = lane * 16, lane_sc = FMT == 0 ? lane * 4 : lane * 2;
    auto load_scale = [&](__amdgpu_buffer_rsrc_t rs, int kc, int rb_off = 0) -> uint32_t {
        if constexpr (FMT == 0) return __builtin_amdgcn_raw_buffer_load_b32(rs, lane_sc, rb_off + (kc >> 2) * 256, 0);
        else return (uint32_t)__builtin_amdgcn_raw_buffer_load_b16(rs, lane_sc, rb_off + kc * 128, 0);
    };

    struct Batch {
        v4i wf[U], xf[XRES ? 1 : U];
        uint32_t sw[U], sx[XRES ? 1 : U];
    };
    // Every batch is requested UNCONDITIONALLY: a batch that does not exist (past the last row-block, or of a wave without a
    // share of K) is requested through buffer resources of zero size, whose loads return zeros without touching memory.
    // The compiler waits for loaded registers by counting the memory operations issued behind them, and at a merge of
    // control flow it assumes the fewest: a prefetch issued under a condition counts as not issued, and the wait in front of
    // the current batch's first product then also waits for the batch just requested -- the prefetch would overlap nothing.
    const __amdgpu_buffer_rsrc_t rs_none = make_rsrc(g.a_codes, 0);
    auto load_batch = [&](Batch& b, int rb, int kc0, bool valid) {
        const int rbv = valid ? rb : 0;
        const __amdgpu_buffer_rsrc_t rs_w = make_rsrc(g.w_codes + (int64_t)rbv * KC * 1024, valid ? (int64_t)KC * 1024 : 0);
        const __amdgpu_buffer_rsrc_t rs_ws = make_rsrc(g.w_scales + (int64_t)rbv * sc_per_rb * SCB, valid ? (int64_t)sc_per_rb * SCB : 0);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int kc = max(min(kc0 + u, k_end - 1), 0);  // the tail repeats the last fragment; its product is skipped
            b.wf[u] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(rs_w, lane16, kc * 1024, 2));  // streamed once
            b.sw[u] = load_scale(rs_ws, kc);
            if constexpr (!XRES) {
                b.xf[u] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(valid ? rs_x : rs_none, lane16, kc * 1024, 0));
                b.sx[u] = load_scale(valid ? rs_xs : rs_none, kc);
            }
        }
    };
    constexpr int XF = XRES ? NB * U : 1;  // resident X fragments per token block: the wave's whole share of K
    // MXFP4: codes and scale dwords as loaded.  NVFP4: DEQUANTIZED once, as fp16 -- the per-fragment dequantization of X,
    // half of the vector arithmetic that bounds the one-shot NVFP4 kernels, is then paid once per workgroup
    v4i xres[FMT == 0 ? MT : 1][FMT == 0 ? XF : 1];
    uint32_t sxres[FMT == 0 ? MT : 1][FMT == 0 ? XF : 1];
    NvFrag16 xres16[FMT == 1 ? XF : 1];
    const bool mine = nb > 0;  // this wave has a share of K
    if constexpr (XRES) {
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            const int mrb = min(tb0 + t, a_rbs - 1);  // (a token block past the end re-reads the last one and is not stored)
#pragma unroll
            for (int j = 0; j < XF; ++j) {
                const bool has = k_begin + j < k_end;  // (fragments past the wave's share: zero-size loads, never multiplied)
                const int kc = has ? k_begin + j : 0;
                const v4i xf = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(has ? rs_x : rs_none, lane16, mrb * KC * 1024 + kc * 1024, 0));
                const uint32_t sx = load_scale(has ? rs_xs : rs_none, kc, mrb * sc_per_rb * SCB);
                if constexpr (FMT == 0) {
                    xres[t][j] = xf;
                    sxres[t][j] = sx;
                } else {
                    xres16[j] = nv_dequant_frag(xf, sx);
                }
            }
        }
    }
    // x0: index of the batch's first fragment among the resident ones (a compile-time constant at every call)
    auto consume = [&](const Batch& b, int kc0, v4f (&acc)[MT], auto x0) {
        constexpr int X0 = XRES ? decltype(x0)::value : 0;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (kc0 + u < k_end) {
                if constexpr (FMT == 0) {
                    const int kc = kc0 + u;
                    const v8i a8 = {b.wf[u][0], b.wf[u][1], b.wf[u][2], b.wf[u][3], 0, 0, 0, 0};
#pragma unroll
                    for (int t = 0; t < MT; ++t) {
                        const v4i xf = XRES ? xres[t][XRES && FMT == 0 ? X0 + u : 0] : b.xf[XRES ? 0 : u];
                        const uint32_t sx = XRES ? sxres[t][XRES && FMT == 0 ? X0 + u : 0] : b.sx[XRES ? 0 : u];
                        const v8i b8 = {xf[0], xf[1], xf[2], xf[3], 0, 0, 0, 0};
                        acc[t] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a8, b8, acc[t], 4, 4, 0, (int)(b.sw[u] >> (8 * (kc & 3))), 0,
                                                                                (int)(sx >> (8 * (kc & 3))));
                    }
                } else {
                    const NvFrag16 w16 = nv_dequant_frag(b.wf[u], b.sw[u]);
#pragma unroll
                    for (int t = 0; t < MT; ++t) {
                        NvFrag16 x16;
                        if constexpr (XRES) x16 = xres16[XRES && FMT == 1 ? X0 + u : 0];
                        else x16 = nv_dequant_frag(b.xf[XRES ? 0 : u], b.sx[XRES ? 0 : u]);
#pragma unroll
                        for (int s = 0; s < 4; ++s) acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(w16.s[s], x16.s[s], acc[t], 0, 0, 0);
                    }
                }
            }
        }
    };

    float ts = g.alpha;
    if constexpr (FMT == 1) ts = (*g.a_ts) * (*g.w_ts);

    // partial sums meet in LDS (two buffers, alternating: a buffer is written again two row-blocks later, behind the next
    // row-block's barrier, when every wave has long finished reading it)
    auto reduce_store = [&](const v4f (&acc)[MT], int rb, int it) {
#pragma unroll
        for (int t = 0; t < MT; ++t) *reinterpret_cast<v4f*>(&partial[it & 1][wave][t][lane * 4]) = acc[t];
        __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): the LDS writes have landed
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        // every wave reduces 32 of the 256 outputs of each token block, lanes 0..31 one each, adding the eight partials in
        // wave order (the order of additions of the one-shot kernel)
        const int r = wave * 32 + (lane & 31);
        const int l = r >> 2, v = r & 3;
        const int n = rb * 16 + (l >> 4) * 4 + v;
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            float sum = 0.0f;
#pragma unroll
            for (int w = 0; w < kSkinnyWaves; ++w) sum += partial[it & 1][w][t][r];
            sum *= ts;
            const int m = (tb0 + t) * 16 + (l & 15);
            if (lane < 32 && m < g.M && n < g.N) {
                if constexpr (OUT_F32) static_cast<float*>(g.out)[(int64_t)m * g.N + n] = sum;
                else static_cast<__bf16*>(g.out)[(int64_t)m * g.N + n] = (__bf16)sum;
            }
        }
    };

    // The batch buffers are addressed with compile-time indices only (a run-time index would put them in scratch memory).
    // No explicit vmcnt waits: the compiler's own, in front of the first use of each loaded register, are exact here
    // because every load of the loop is unconditional (output stores sit under conditions and count as not issued, which
    // makes a wait a few operations stricter than necessary).
    if constexpr (XRES) {
        // A row-block is NB batches per wave (a compile-time count: the resident X fragments are addressed statically; a
        // wave whose share of K is shorter requests its missing batches with zero size).  The batches of all the walker's
        // row-blocks form one sequence, NBUF - 1 of them in flight ahead of the one being multiplied, through NBUF
        // buffers in rotation; the loop body is NB * NBUF steps with every index a constant, left by `break` so that no
        // control flow merges back into it.
        constexpr int NBUF = MT * NB >= 7 ? 2 : 3;
        constexpr int P = NB * NBUF;
        static_assert(P <= 12, "the loop body below spells out twelve steps");
        Batch buf[NBUF];
        int rb = walker, it = 0;
        auto request = [&](Batch& b, int rbq, int batch) { load_batch(b, rbq, k_begin + batch * U, mine && rbq < n_rb && batch < nb); };
        request(buf[0], rb, 0);
        if constexpr (NBUF == 3) request(buf[1], rb + (1 / NB) * G, 1 % NB);
        v4f acc[MT];
#pragma unroll
        for (int t = 0; t < MT; ++t) acc[t] = v4f{0.f, 0.f, 0.f, 0.f};
        // step q of the body: request the batch NBUF - 1 ahead into the buffer multiplied last, multiply batch q % NB of the
        // current row-block, and behind a row-block's last batch reduce and store; true = that was the last row-block
        auto step = [&](auto qc) -> bool {
            constexpr int q = decltype(qc)::value, batch = q % NB, ahead = batch + NBUF - 1;
            request(buf[(q + NBUF - 1) % NBUF], rb + (ahead / NB) * G, ahead % NB);
            consume(buf[q % NBUF], k_begin + batch * U, acc, std::integral_constant<int, batch * U>{});
            if constexpr (batch == NB - 1) {
                reduce_store(acc, rb, it);
#pragma unroll
                for (int t = 0; t < MT; ++t) acc[t] = v4f{0.f, 0.f, 0.f, 0.f};
                ++it;
                rb += G;
                return rb >= n_rb;
            }
            return false;
        };
#define FP4MR_STEP(q) if constexpr (P > q) { if (step(std::integral_constant<int, q>{})) break; }
        if (rb < n_rb) {
            for (;;) {
                FP4MR_STEP(0) FP4MR_STEP(1) FP4MR_STEP(2) FP4MR_STEP(3) FP4MR_STEP(4) FP4MR_STEP(5)
                FP4MR_STEP(6) FP4MR_STEP(7) FP4MR_STEP(8) FP4MR_STEP(9) FP4MR_STEP(10) FP4MR_STEP(11)
            }
        }
#undef FP4MR_STEP
    } else {
        // Several batches per row-block: they alternate between two buffers, two per trip of the inner loop, and a
        // row-block with an odd number of batches hands the next one the other buffer first (`first`, uniform).
        Batch buf0, buf1;
        int first = 0;
        int rb = walker;
        load_batch(buf0, rb, k_begin, mine && rb < n_rb);
        for (int it = 0; rb < n_rb; ++it, rb += G) {
            v4f acc[MT];
#pragma unroll
            for (int t = 0; t < MT; ++t) acc[t] = v4f{0.f, 0.f, 0.f, 0.f};
            // one batch: request the one after it (of this row-block, else the first of the next) into `nxt`, multiply `cur`
            auto step = [&](Batch& cur, Batch& nxt, int b) {
                const bool more_here = b + 1 < nb;
                load_batch(nxt, more_here ? rb : rb + G, more_here ? k_begin + (b + 1) * U : k_begin, mine && (more_here || rb + G < n_rb));
                consume(cur, k_begin + b * U, acc, std::integral_constant<int, 0>{});
            };
            if (first == 0) {
                for (int b = 0; b < nb; b += 2) {
                    step(buf0, buf1, b);
                    if (b + 1 < nb) step(buf1, buf0, b + 1);
                }
            } else {
                for (int b = 0; b < nb; b += 2) {
                    step(buf1, buf0, b);
                    if (b + 1 < nb) step(buf0, buf1, b + 1);
                }
            }
            first ^= nb & 1;
            reduce_store(acc, rb, it);
        }
    }
}

// compute units of the current device
int stream_cus()
{
    return compute_units();
}

// Grid of the persistent kernels: one workgroup per compute unit, also where the registers would let two or three be
// resident -- fewer, longer walks measured faster at every shape (K = 4096, cold weights, 256 against 512 workgroups:
// M = 16, N = 6144 4.9 us against 5.5, N = 14336 7.7 against 8.5, N = 28672 12.1 against 12.7; M = 32, N = 6144 6.1 against 7.1).
int stream_walkers()
{
    int cap = stream_cus();
    // (the grid-cap option, a testing aid: a small grid makes every workgroup walk many row-blocks)
    if (options().gemm_grid > 0 && options().gemm_grid < cap) cap = options().gemm_grid;
    return cap;
}

// Workgroups of a persistent launch: one per compute unit, or, with several sets (parts > 1), as many walkers per set as
// share the row-blocks evenly -- as many rounds as the resident workgroups need, then the fewest walkers (whole groups of
// eight, all sets resident at once) that do it in that many rounds.
unsigned stream_grid(int N, int parts)
{
    const int n_rb = (N + 15) / 16, cap = stream_walkers();
    if (parts <= 1) return (unsigned)std::min(n_rb, cap);
    const int per_part = std::max(cap / parts / 8 * 8, 8);
    const int rounds = (n_rb + per_part - 1) / per_part;
    const int walkers = std::min(per_part, ((n_rb + rounds - 1) / rounds + 7) / 8 * 8);
    return (unsigned)(parts * walkers);
}

// MXFP4 with the activations resident in registers: MT 16-token blocks, a wave's share of K in NB batches of four fragments
// (K <= 4096 NB).  parts > 1: that many sets of workgroups, each with its own MT token blocks; W passes through every
// XCD's L2 once and is read from there once per set.
template <int MT, int NB>
hipError_t launch_stream_resident(SkinnyArgs g, bool out_f32, int parts, hipStream_t st)
{
    g.parts = parts;
    const dim3 grid(stream_grid(g.N, parts)), block(kSkinnyWaves * 64);
    if (out_f32) hipLaunchKernelGGL((gemm_stream_kernel<0, true, 4, true, MT, NB>), grid, block, 0, st, g);
    else hipLaunchKernelGGL((gemm_stream_kernel<0, false, 4, true, MT, NB>), grid, block, 0, st, g);
    return hipGetLastError();
}

// NVFP4, up to 16 tokens, K <= 8192: the activations resident as fp16 (a wave's share of K in NB batches of two fragments)
template <int NB>
hipError_t launch_stream_resident_nv(SkinnyArgs g, bool out_f32, int parts, hipStream_t st)
{
    g.parts = parts;
    const dim3 grid(stream_grid(g.N, parts)), block(kSkinnyWaves * 64);
    if (out_f32) hipLaunchKernelGGL((gemm_stream_kernel<1, true, 2, true, 1, NB>), grid, block, 0, st, g);
    else hipLaunchKernelGGL((gemm_stream_kernel<1, false, 2, true, 1, NB>), grid, block, 0, st, g);
    return hipGetLastError();
}

hipError_t launch_stream_nv(const SkinnyArgs& g, bool out_f32, int per, int parts, hipStream_t st)
{
    switch ((per + 1) / 2) {
        case 1: return launch_stream_resident_nv<1>(g, out_f32, parts, st);
        case 2: return launch_stream_resident_nv<2>(g, out_f32, parts, st);
        case 3: return launch_stream_resident_nv<3>(g, out_f32, parts, st);
        default: return launch_stream_resident_nv<4>(g, out_f32, parts, st);
    }
}

// largest number of batches per row-block for which MT token blocks of X fit the registers (MT * NB * 20 for X: up to
// 235 in all, no spills; three blocks with three batches would spill)
constexpr int stream_max_batches(int mt)
{
    return mt <= 2 ? 4 : 2;
}

// false (nothing launched): the wave's share of K (`per` fragments) does not fit
template <int MT>
bool try_stream_resident(const SkinnyArgs& g, bool out_f32, int per, int parts, hipStream_t st, hipError_t* err)
{
    const int nbk = (per + 3) / 4;
    if (nbk > stream_max_batches(MT)) return false;
    switch (nbk) {
        case 1: *err = launch_stream_resident<MT, 1>(g, out_f32, parts, st); break;
        case 2:
            if constexpr (stream_max_batches(MT) >= 2) *err = launch_stream_resident<MT, 2>(g, out_f32, parts, st);
            break;
        case 3:
            if constexpr (stream_max_batches(MT) >= 3) *err = launch_stream_resident<MT, 3>(g, out_f32, parts, st);
            break;
        default:
            if constexpr (stream_max_batches(MT) >= 4) *err = launch_stream_resident<MT, 4>(g, out_f32, parts, st);
            break;
    }
    return true;
}

// MXFP4, up to 16 tokens, a share of K too long to keep X resident (K > 16384): the X fragments travel with W, two buffers.
template <int FMT, int U>
hipError_t launch_stream_travelling(const SkinnyArgs& g, bool out_f32, hipStream_t st)
{
    const int n_rb = (g.N + 15) / 16;
    const dim3 grid((unsigned)std::min(n_rb, stream_walkers())), block(kSkinnyWaves * 64);
    if (out_f32) hipLaunchKernelGGL((gemm_stream_kernel<FMT, true, U, false>), grid, block, 0, st, g);
    else hipLaunchKernelGGL((gemm_stream_kernel<FMT, false, U, false>), grid, block, 0, st, g);
    return hipGetLastError();
}

template <int FMT, int MT>
hipError_t launch_mt(const SkinnyArgs& g, bool out_f32, hipStream_t st)
{
    const int n_rb = (g.N + 15) / 16;
    const dim3 grid((unsigned)n_rb), block(kSkinnyWaves * 64);
    // At most one workgroup per compute unit and several batches of K per wave: no other workgroup's loads hide this one's
    // latency, so the instantiation that requests the next batch before it multiplies the current one (NVFP4, N = 4096,
    // K = 14336 ...).  Same K split, same order of additions.
    const int per = ((g.K >> 7) + kSkinnyWaves - 1) / kSkinnyWaves;
    if (n_rb <= stream_cus() && per > (MT == 1 ? 4 : 2)) {
        if (out_f32) hipLaunchKernelGGL((gemm_skinny_nt_kernel<FMT, 1, MT, true, true>), grid, block, 0, st, g);
        else hipLaunchKernelGGL((gemm_skinny_nt_kernel<FMT, 1, MT, false, true>), grid, block, 0, st, g);
        return hipGetLastError();
    }
    if (out_f32) hipLaunchKernelGGL((gemm_skinny_kernel<FMT, MT, true>), grid, block, 0, st, g);
    else hipLaunchKernelGGL((gemm_skinny_kernel<FMT, MT, false>), grid, block, 0, st, g);
    return hipGetLastError();
}

// Two row-blocks per workgroup.  NVFP4: halves the X share of the dequantization; MXFP4 with two to four token blocks:
// halves the reads of the X fragments from L2.  Below about 0.6 workgroups per compute unit the halved grid costs more
// than that saves (NVFP4, K = 14336, N = 4096, M <= 16: 14.1 us against 11.2).  Returns false (nothing launched) when the
// one-row-block kernel is the better choice.
template <int FMT, int MT>
bool try_two_row_blocks(const SkinnyArgs& g, bool out_f32, hipStream_t st, hipError_t* err)
{
    const int n_rb = (g.N + 15) / 16, wgs = (n_rb + 1) / 2;
    if (5 * wgs < 3 * stream_cus()) return false;
    const dim3 grid((unsigned)wgs), block(kSkinnyWaves * 64);
    // at most one workgroup per compute unit and several batches of K per wave: the instantiation that prefetches
    const int per = ((g.K >> 7) + kSkinnyWaves - 1) / kSkinnyWaves;
    if (FMT == 1 && wgs <= stream_cus() && per > (MT == 1 ? 4 : 2)) {
        if (out_f32) hipLaunchKernelGGL((gemm_skinny_nt_kernel<FMT, 2, MT, true, true>), grid, block, 0, st, g);
        else hipLaunchKernelGGL((gemm_skinny_nt_kernel<FMT, 2, MT, false, true>), grid, block, 0, st, g);
        *err = hipGetLastError();
        return true;
    }
    if (out_f32) hipLaunchKernelGGL((gemm_skinny_nt_kernel<FMT, 2, MT, true>), grid, block, 0, st, g);
    else hipLaunchKernelGGL((gemm_skinny_nt_kernel<FMT, 2, MT, false>), grid, block, 0, st, g);
    *err = hipGetLastError();
    return true;
}

template <int FMT, int MT>
hipError_t launch_tokens(const SkinnyArgs& g, bool out_f32, hipStream_t st)
{
    if constexpr (FMT == 0 && MT >= 2) {
        // the persistent kernel with all MT token blocks of X in registers, where the wave's share of K fits: nothing of X is
        // read again after the first microsecond (the one-shot kernels fetch MT X fragments from L2 per W fragment)
        const int per = ((g.K >> 7) + kSkinnyWaves - 1) / kSkinnyWaves;
        hipError_t e = hipSuccess;
        if (try_stream_resident<MT>(g, out_f32, per, 1, st, &e)) return e;
    }
    // (MXFP4 with two token blocks measured level with the one-row-block kernel, with three and four 5-11 % faster:
    // N = 6144, K = 4096, M = 64: 8.5 us against 9.6; N = K = 8192: 14.4 against 16.1)
    if constexpr (FMT == 1 || MT >= 3) {
        hipError_t e = hipSuccess;
        if (try_two_row_blocks<FMT, MT>(g, out_f32, st, &e)) return e;
    }
    return launch_mt<FMT, MT>(g, out_f32, st);
}

// MXFP4, more token blocks than one set of workgroups can keep resident for this K: the fewest sets, then the fewest token
// blocks per set, that cover them (K <= 8192: up to four blocks per set, K <= 16384: two).  false: K too long.
bool try_stream_sets(const SkinnyArgs& g, bool out_f32, int mt, int per, hipStream_t st, hipError_t* err)
{
    const int nbk = (per + 3) / 4;
    const int mt_max = nbk <= stream_max_batches(4) ? 4 : nbk <= stream_max_batches(2) ? 2 : 0;
    if (mt_max == 0) return false;
    const int parts = (mt + mt_max - 1) / mt_max;
    switch ((mt + parts - 1) / parts) {
        case 1: return try_stream_resident<1>(g, out_f32, per, parts, st, err);
        case 2: return try_stream_resident<2>(g, out_f32, per, parts, st, err);
        case 3: return try_stream_resident<3>(g, out_f32, per, parts, st, err);
        default: return try_stream_resident<4>(g, out_f32, per, parts, st, err);
    }
}

template <int FMT>
hipError_t launch_fmt(const SkinnyArgs& g, bool out_f32, hipStream_t st)
{
    const int mt = (g.M + 15) / 16;
    const int per = ((g.K >> 7) + kSkinnyWaves - 1) / kSkinnyWaves;  // fragments of K per wave
    if constexpr (FMT == 0) {
        // more token blocks than fit one set of resident registers at this K
        const int nbk = (per + 3) / 4;
        const bool one_set = mt <= 4 && nbk <= stream_max_batches(mt);
        hipError_t e = hipSuccess;
        if (mt >= 2 && !one_set && try_stream_sets(g, out_f32, mt, per, st, &e)) return e;
    }
    switch (mt) {
        case 1:
            if constexpr (FMT == 0) {
                // The persistent kernels win by keeping loads in flight across batches and row-blocks, which needs several
                // batches per row-block or more row-blocks than workgroups: a layer of at most one row-block per compute unit
                // and one batch (N <= 4096, K <= 4096) is launch-bound and 0.1-0.4 us faster with the one-shot kernel's
                // occupancy.  (NVFP4 stays with the one-shot kernels: its in-register dequantization needs the registers of
                // the second batch buffer -- 68 us against 54 on N = 57344, K = 8192.)
                // ... and so is any layer with K <= 1024 (one fragment per wave: N = 8192, K = 1024, 3.7 us against 4.6)
                const bool one_shot = per <= 1 || (per <= 4 && (g.N + 15) / 16 <= stream_walkers());
                hipError_t e = hipSuccess;
                if (!one_shot) {
                    if (try_stream_resident<1>(g, out_f32, per, 1, st, &e)) return e;
                    return launch_stream_travelling<0, 4>(g, out_f32, st);
                }
            }
            if constexpr (FMT == 1) {
                // K <= 8192: the persistent kernel with the activations resident as fp16 (70B qkv, M = 16, cold weights: 15.3 ->
                // 11.3 us; gate_up 49 -> 43.5 us = 6.2 TB/s; N = 28672, K = 4096: 16.6 -> 13.0), bit-identical to the kernels below
                if (per <= 8) return launch_stream_nv(g, out_f32, per, 1, st);
            }
            return launch_tokens<FMT, 1>(g, out_f32, st);
        case 2:
        case 3:
        case 4:
            if constexpr (FMT == 1) {
                // 17 to 64 tokens on a narrow layer: one set of such workgroups per token block (every set dequantizes W again,
                // which the two-row-block kernels below share between token blocks: N = 10240, K = 8192, M = 32 / 64: 18.7 /
                // 29.5 -> 15.5 / 24.5 us; N = 16384: level; N = 57344: 59 / 100 -> 67 / 113, not taken)
                // (not with a single fragment per wave: N = 8192, K = 1024, M = 64: 5.4 us against 7.2)
                if (per >= 2 && per <= 8 && g.N <= 12288) return launch_stream_nv(g, out_f32, per, mt, st);
            }
            return mt == 2 ? launch_tokens<FMT, 2>(g, out_f32, st) : mt == 3 ? launch_tokens<FMT, 3>(g, out_f32, st) : launch_tokens<FMT, 4>(g, out_f32, st);
        default:
            if constexpr (FMT == 1) {
                if (mt <= 32 && per <= 8) return launch_stream_nv(g, out_f32, per, mt, st);
            }
            return hipErrorInvalidValue;
    }
}

}  // namespace

// More than 64 tokens: MXFP4 with K <= 8192 as several sets of persistent workgroups (up to four resident token blocks
// each), on layers narrow enough that the tile kernels' cost per launch (12-14 us at K = 4096, 15-25 at K = 8192, whatever
// the token count) exceeds what the persistent kernel spends per row-block and set.  Measured, cold weights, tiles -> sets:
// M = 96 (two sets), K = 4096: N = 4096 12.6 -> 6.4 us, 8192 12.9 -> 8.6, 14336 14.3 -> 12.2, 28672 17.9 -> 20.4 (not taken);
// K = 8192: N = 4096 16.0 -> 9.3, 8192 17.8 -> 12.6, 14336 25.1 -> 18.9; K = 2048: N = 4096 8.1 -> 6.0, 8192 9.4 -> 8.7,
// 14336 10.1 -> 12.6 (not taken); K = 1024: level or slower (not taken).  M = 256 (four sets), K = 4096: N = 4096 13.6 -> 9.3,
// 6144 14.2 -> 11.2, 8192 14.5 -> 13.3, 14336 16.8 -> 20.9 (not taken); K = 8192: N = 4096 23.8 -> 12.7, 8192 24.5 -> 19.7.
// M = 512 (eight sets): N = 4096 13.8 -> 12.8 (K = 4096), 24.0 -> 18.5 (K = 8192); N = 6144 15.1 -> 17.4 (not taken).
// So: sets x N up to 28672 (N = 16384, K = 6144, M = 128: 17.9 -> 21.3, not taken).  K = 14336 (sets of two blocks): level with the split-K tiles at N = 4096, slower beyond (not taken).
bool gemm_skinny_takes(int64_t M, int64_t N, int64_t K, int fmt)
{
    if (M <= 64) return true;
    const int64_t per = ((K >> 7) + kSkinnyWaves - 1) / kSkinnyWaves;  // fragments of K per wave
    // NVFP4, 65 to 256 tokens: one set of fp16-resident persistent workgroups per 16-token block where the layer is small
    // enough that dequantizing W once per set costs less than the many-token kernel's launch (which multiplies whole
    // 128-token tiles on a few compute units).  Measured, cold weights, tiles -> sets: N = K = 4096, M = 80 / 128 / 256:
    // 20.7 / 26.1 / 25.3 -> 10.3 / 12.5 / 21.6 us; N = K = 2048: 13.8 / 15.4 / 18.8 -> 4.8 / 5.7 / 8.5; N = 12288, K = 4096,
    // M = 80 / 128: 28.4 / 32.3 -> 21.2 / 30.3; N = 10240, K = 8192, M = 96 / 128: 38.2 / 41.6 -> 36.8 / 44.7 (128: not taken).
    // (257 to 512 tokens -- up to 32 sets -- on the smallest layers only: N = K = 2048, M = 512: 25 -> 15 us)
    if (fmt == 1) {
        if (per > 8 || N > 12288) return false;
        const int64_t work = (M + 15) / 16 * N * K;
        // (one fragment per wave, K <= 1024: a set's row-block is mostly its barrier and reduction -- N = 8192, K = 1024:
        // M = 80 / 128: 16 -> 9.0 / 11.9 us, M = 192: 17 -> 19.9, not taken)
        if (per == 1) return M <= 256 && work <= (int64_t)1 << 26;
        return M <= 512 && work <= (int64_t)1 << (M <= 256 ? 29 : 28);
    }
    if (fmt != 0 || M > 512) return false;
    // (up to four sets at K <= 4096: N = 4096, M = 384 / 512 measured 11.5 / 11.7 us on tiles against 12.3 / 13.5; with a longer
    // K the tiles cost more and up to eight sets pay: N = 4096, K = 8192, M = 512: 24.0 -> 18.5)
    const int64_t sets = (M + 63) / 64;
    if (per >= 4 && per <= 8) return sets * N <= 28672 && (per > 4 || sets <= 4);
    if (per == 2 || per == 3) return M <= 128 && N <= 8192;
    return false;
}

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
