// NVFP4 W4A4 GEMM for many tokens (arXiv 2509.23202, Section 2 "The NVFP4 Format", Section 4.1 "Ingredient 1":
// Xhat = s_T * s_G * Q(.), groups of 16 with E4M3 scales plus one fp32 tensor scale per operand).
//
//   out[m,n] = sT_a * sT_w * sum_k (sa[m,k/16] * a[m,k]) * (sw[n,k/16] * w[n,k])
//
// E4M3 scales on 16-element groups cannot go through CDNA4's block-scaled MFMA (one power-of-two scale per 32
// elements), so the product runs on the fp16 MFMA (v_mfma_f32_16x16x32_f16) over exactly dequantized operands: an E2M1
// value times an E4M3 value has at most 6 significant bits and lies in [2^-10, 2688].  What bounds such a kernel is the
// vector-ALU work of the dequantization, which grows with (tile rows + tile columns) while the MFMAs grow with their
// product.  Two things keep it below the MFMA time here:
//   * the activations are dequantized ONCE, by a pre-pass that writes them as fp16 in the MFMA's operand order into the
//     caller's workspace (2 bytes per element; every tile column of the product re-reads them from L2 instead of
//     re-converting them);
//   * only W is converted inside the product, and a wave's tile is 128 rows of X by 64 (or 32) rows of W: four (two)
//     half-fragment conversions per 64 (32) MFMAs.
// Block tile 128 x 256 (or 128 x 128 for a remainder of the tile grid), four waves side by side along N, K-step 64,
// three-stage LDS ring fed by direct-to-LDS loads, one barrier per K-step.  75 KB of LDS and 256 registers per wave: two
// workgroups share a compute unit, and one's barrier and fragment loads hide under the other's MFMAs.
//
// Operand order of one K-step of 64 (16 rows): the MFMA takes 8 halves per lane and call (lane = row r + 16 q); lane (r, q)
// owns the 16 elements k = 16 q .. 16 q + 15 -- exactly one NVFP4 group, one E4M3 scale -- and two MFMAs (s = 0, 1) consume
// its elements 8 s .. 8 s + 7; X and W use the same assignment, which a dot product does not see.
//   X (fp16, workspace): [row-block][K-step][plane s][lane][16 bytes]
//   W (codes, GEMM layout): the K-step is half a fragment, 512 contiguous bytes; lane (r, q) reads 8 bytes.
#include "device_util.hpp"
#include "internal.hpp"
#include "layout.hpp"
#include "nv_dequant.hpp"

#include <algorithm>

namespace fp4mr {
namespace {

struct Nv16Args {
    const uint8_t* x16;
    const uint8_t* w_codes;
    const uint8_t* w_scales;
    const float* a_ts;
    const float* w_ts;
    void* out;
    int64_t M, N, K;
    int tiles_m;
    int n_first;   // first output column of this launch (a multiple of 256)
    int n_cols;    // number of output columns this launch covers (to the end of N when the tile grid is ragged)
    int split_steps;  // split-K launches: K-steps of 64 per split (a multiple of 8); blockIdx.y is the split, out the fp32 partials
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

// ---------------------------------------------------------------------------------------------------------------
// Pre-pass: NVFP4 activations (GEMM layout) -> exact fp16 values code * s_G in the operand order above.  One wave per
// fragment (16 rows x 128 K): 1 KB of codes and 128 scale bytes in, two K-steps of 2 KB out.
__global__ __launch_bounds__(256) void nv_x16_kernel(const uint8_t* __restrict__ codes, const uint8_t* __restrict__ scales,
                                                     uint8_t* __restrict__ x16, int64_t n_frags)
{
    const int lane = threadIdx.x & 63;
    const int64_t f = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (f >= n_frags) return;
    const v4i c = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(codes + f * 1024) + lane);
    const uint32_t sc = *(reinterpret_cast<const uint16_t*>(scales + f * 128) + lane);
    const NvFrag16 v = nv_dequant_frag(c, sc);
    // lane (r, Q) holds k = 32 Q .. 32 Q + 31 of the fragment: K-step Q / 2, lanes q = 2 (Q % 2) + t of that step for its
    // elements 16 t .. 16 t + 15, plane s for elements 8 s .. 8 s + 7 of those
    const int r = lane & 15, Q = lane >> 4;
    uint8_t* dst = x16 + (f * 2 + (Q >> 1)) * 2048;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int s = 0; s < 2; ++s)
            *reinterpret_cast<v8h*>(dst + s * 1024 + ((2 * (Q & 1) + t) * 16 + r) * 16) = v.s[2 * t + s];
}

// ---------------------------------------------------------------------------------------------------------------
// SPLITK: the workgroup multiplies K-steps blockIdx.y * split_steps .. only and writes its fp32 partial tile, without the
// tensor scales, to slice blockIdx.y of the output; nv16_reduce_kernel adds the slices in split order.
template <int BN, bool OUT_F32, int STAGES = 3, bool SPLITK = false>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void gemm_nv16_kernel(Nv16Args g)
{
    static_assert(!SPLITK || OUT_F32, "split-K workgroups write fp32 partials");
    constexpr int BM = 128, NW = 4;
    constexpr int WN = BN / NW;            // 64 or 32 columns per wave
    constexpr int TM = BM / 16, TN = WN / 16;
    constexpr int FX = BM / 16, FW = BN / 16;
    constexpr int WS_SLOT = 256;           // scale bytes one full-wave copy writes: four row-blocks' worth per wave
    constexpr int X_BYTES = FX * 2048, WC_BYTES = FW * 512, WS_BYTES = NW * WS_SLOT;
    constexpr int STAGE_BYTES = X_BYTES + WC_BYTES + WS_BYTES;
    constexpr int XPW = FX * 2 / NW, WPW = FW / NW;      // 1 KB X chunks and W half-fragments a wave copies per stage
    constexpr int OPS = XPW + WPW / 2 + 1;                // vector-memory operations per wave and stage
    static_assert(FX * 2 % NW == 0 && FW % NW == 0, "the copies are dealt evenly to the waves");

    extern __shared__ __attribute__((aligned(1024))) char smem[];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int tm = blockIdx.x % g.tiles_m, tn = blockIdx.x / g.tiles_m;   // consecutive workgroups share a W column band
    const int64_t n_tile0 = (int64_t)g.n_first + (int64_t)tn * BN;

    const int KH_all = (int)(g.K >> 6), KC = (int)(g.K >> 7);   // K-steps of 64 / fragments of 128 per row-block in memory
    const int kh0 = SPLITK ? (int)blockIdx.y * g.split_steps : 0;  // (even: a split starts on a fragment)
    const int KH = SPLITK ? min(g.split_steps, KH_all - kh0) : KH_all;
    const int a_rbs = (int)((g.M + 15) / 16), w_rbs = (int)((g.N + 15) / 16);
    const int a_rb0 = min(tm * FX, a_rbs - 1), w_rb0 = min((int)(n_tile0 / 16), w_rbs - 1);
    const int a_rb_last = a_rbs - 1 - a_rb0, w_rb_last = w_rbs - 1 - w_rb0;
    auto make_rsrc = [](const uint8_t* base, int64_t bytes) {
        const uint32_t n = bytes > 0xffffffffll ? 0xffffffffu : (uint32_t)bytes;
        return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(base), 0, (int)n, 0x00020000);
    };
    const int64_t x0 = (int64_t)kh0 * 2048, c0 = (int64_t)(kh0 >> 1) * 1024, s0 = (int64_t)(kh0 >> 1) * 128;  // (0 unless SPLITK)
    const __amdgpu_buffer_rsrc_t rs_x = make_rsrc(g.x16 + (int64_t)a_rb0 * KH_all * 2048 + x0, (int64_t)(a_rbs - a_rb0) * KH_all * 2048 - x0);
    const __amdgpu_buffer_rsrc_t rs_wc = make_rsrc(g.w_codes + (int64_t)w_rb0 * KC * 1024 + c0, (int64_t)(w_rbs - w_rb0) * KC * 1024 - c0);
    const __amdgpu_buffer_rsrc_t rs_ws = make_rsrc(g.w_scales + (int64_t)w_rb0 * KC * 128 + s0, (int64_t)(w_rbs - w_rb0) * KC * 128 - s0);
    const uint32_t lane16 = (uint32_t)lane * 16u;
    const int x_rb_bytes = KH_all * 2048, wc_rb_bytes = KC * 1024, ws_rb_bytes = KC * 128;

    // Row-blocks past the end of an operand (last tile) are clamped to its last row-block: the duplicates only feed
    // outputs that are never stored.  A stage's copies are issued in three pieces (X, W codes, W scales) at three points of
    // the K-step.  Every copy is a full-wave instruction (no lane predicate, hence no branch inside the K-step):
    //   X: 1 KB chunks, 16 bytes per lane;
    //   W codes: a K-step of a fragment is 512 contiguous bytes -- one instruction copies the halves of TWO row-blocks,
    //     lanes 0-31 from one and lanes 32-63 from the next, into adjacent LDS slots (direct-to-LDS loads place lane l's
    //     data at 16 l behind the base whatever address the lane reads from);
    //   W scales: 64 bytes per row-block and K-step -- one instruction copies those of FOUR row-blocks, 16 lanes each.
    static_assert(WPW % 2 == 0 && (WPW == 4 || WPW == 2), "W halves are copied in pairs, scales in fours (or twos)");
    constexpr int WCI = WPW / 2;          // W code instructions per wave and stage
    const uint32_t wc_voff0 = (uint32_t)((lane & 31) * 16 + min(wave * WPW + (lane >> 5), w_rb_last) * wc_rb_bytes);
    const uint32_t wc_voff1 = (uint32_t)((lane & 31) * 16 + min(wave * WPW + 2 + (lane >> 5), w_rb_last) * wc_rb_bytes);   // (WCI = 2 only)
    // (a wave that owns two row-blocks only fills the rest of its 256-byte slot with the scales of the two behind them)
    const uint32_t ws_voff = (uint32_t)((lane & 15) * 4 + min(wave * WPW + (lane >> 4), w_rb_last) * ws_rb_bytes);
    auto issue_x = [&](int kl, char* base) {
#pragma unroll
        for (int i = 0; i < XPW; ++i) {
            const int c = wave * XPW + i;                 // chunk = (row-block, plane)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_x, (lds_void*)(base + c * 1024), 16, lane16,
                                                     min(c >> 1, a_rb_last) * x_rb_bytes + kl * 2048 + (c & 1) * 1024, 0, 0);
        }
    };
    auto issue_wc = [&](int kl, char* base) {
#pragma unroll
        for (int i = 0; i < WCI; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_wc, (lds_void*)(base + X_BYTES + (wave * WPW + 2 * i) * 512), 16, i == 0 ? wc_voff0 : wc_voff1,
                                                     (kl >> 1) * 1024 + (kl & 1) * 512, 0, 0);
    };
    auto issue_ws = [&](int kl, char* base) {
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_ws, (lds_void*)(base + X_BYTES + WC_BYTES + wave * WS_SLOT), 4, ws_voff,
                                                 (kl >> 1) * 128 + (kl & 1) * 64, 0, 0);
    };
    // stage k goes to ring slot k % STAGES; past the last stage the copies repeat it into a slot nobody reads any more, so
    // that every K-step issues the same operations (no branch, uniform vmcnt bookkeeping)
    auto issue = [&](int k) {
        const int kl = min(k, KH - 1);
        char* base = smem + (k % STAGES) * STAGE_BYTES;
        issue_x(kl, base);
        issue_wc(kl, base);
        issue_ws(kl, base);
    };

    v4f acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j) acc[i][j] = v4f{0.f, 0.f, 0.f, 0.f};

#pragma unroll
    for (int s = 0; s < STAGES - 1; ++s) issue(s);

    // where lane (r, q) finds its 8 code bytes and its scale byte inside a W half-fragment
    const int r = lane & 15, q = lane >> 4;
    const int w_code_off = ((q >> 1) * 16 + r) * 16 + (q & 1) * 8;
    const int w_scale_off = ((q >> 1) * 16 + r) * 2 + (q & 1);

    // A W half-fragment in three states: raw (8 code bytes + the scale byte), its scale as packed halves, and the 16
    // dequantized halves.  The conversion is cut into eight micro-steps (one byte of codes = two values each: a convert and
    // a packed multiply) that the K-step places between the MFMAs of the column-tile before: a wave issues in order, so
    // vector-ALU work overlaps MFMA execution only where the two alternate in the instruction stream.
    struct WRaw {
        v2i codes;
        uint32_t scale;
    };
    struct WHalf {
        v2h h[8];   // h[4 s + b] = elements 8 s + 2 b, 8 s + 2 b + 1
    };
    auto read_w = [&](const char* base, int i) {
        const int f = wave * TN + i;
        WRaw w;
        w.codes = *reinterpret_cast<const v2i*>(base + X_BYTES + f * 512 + w_code_off);
        w.scale = *reinterpret_cast<const uint8_t*>(base + X_BYTES + WC_BYTES + wave * WS_SLOT + i * 64 + w_scale_off);
        return w;
    };
    auto scale2 = [&](const WRaw& w) {
        const _Float16 sh = (_Float16)e4m3_decode<true>(w.scale);
        return v2h{sh, sh};
    };
    auto micro = [&](const WRaw& w, v2h s2, WHalf& out, int u) {   // u = 0..7, a compile-time constant after unrolling
        const uint32_t c = (uint32_t)w.codes[u >> 2];
        v2h p;
        switch (u & 3) {
            case 0: p = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(c, 1.0f, 0); break;
            case 1: p = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(c, 1.0f, 1); break;
            case 2: p = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(c, 1.0f, 2); break;
            default: p = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(c, 1.0f, 3); break;
        }
        out.h[u] = p * s2;
    };
    auto operand = [&](const WHalf& w, int s) {
        const v8h v = {w.h[4 * s][0], w.h[4 * s][1], w.h[4 * s + 1][0], w.h[4 * s + 1][1],
                       w.h[4 * s + 2][0], w.h[4 * s + 2][1], w.h[4 * s + 3][0], w.h[4 * s + 3][1]};
        return v;
    };

    for (int kh = 0; kh < KH; ++kh) {
        // stage kh has landed (this wave's copies: vmcnt; everybody's: barrier); the barrier also says that every wave is
        // done with stage kh - 1, whose slot stage kh + STAGES - 1 is about to refill
        wait_vmcnt<(STAGES - 2) * OPS>();
        block_barrier();
        const int kn = kh + STAGES - 1, kl = min(kn, KH - 1);
        char* const fill = smem + (kn % STAGES) * STAGE_BYTES;

        const char* base = smem + (kh % STAGES) * STAGE_BYTES;
        v8h xf[TM][2];
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int s = 0; s < 2; ++s) xf[j][s] = *(reinterpret_cast<const v8h*>(base + (j * 2 + s) * 1024) + lane);
        WRaw wraw[TN];
#pragma unroll
        for (int i = 0; i < TN; ++i) wraw[i] = read_w(base, i);
        WHalf wcur, wnext;
        {
            const v2h s2 = scale2(wraw[0]);
#pragma unroll
            for (int u = 0; u < 8; ++u) micro(wraw[0], s2, wcur, u);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < TN; ++i) {
            v2h s2 = {0, 0};
            if (i + 1 < TN) s2 = scale2(wraw[i + 1]);
            const v8h a0 = operand(wcur, 0), a1 = operand(wcur, 1);
#pragma unroll
            for (int t = 0; t < 2 * TM; ++t) {
                const int j = t % TM, s = t / TM;
                acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(s == 0 ? a0 : a1, xf[j][s], acc[i][j], 0, 0, 0);
                if (i + 1 < TN && t < 8) micro(wraw[i + 1], s2, wnext, t);
                __builtin_amdgcn_sched_barrier(0);
            }
            // the refill of the slot everybody left at this step's barrier, a third of it behind each of the first three
            // column-tiles (TN = 2: X behind the first, both W pieces behind the second)
            if (i == 0) issue_x(kl, fill);
            if (i == 1) issue_wc(kl, fill);
            if (i == (TN == 2 ? 1 : 2)) issue_ws(kl, fill);
            __builtin_amdgcn_sched_barrier(0);
            if (i + 1 < TN) wcur = wnext;
        }
    }
    wait_vmcnt<0>();   // (the repeated copies of the last steps: nothing may be in flight into LDS when the workgroup ends)

    // A lane owns out[m][n .. n+3] with m = m0 + 16 j + lane % 16, n = n0 + 16 i + 4 (lane / 16).
    const float ts = SPLITK ? 1.0f : (*g.a_ts) * (*g.w_ts);
    const int64_t n_lim = (int64_t)g.n_first + g.n_cols;
    const int64_t n_end = n_lim < g.N ? n_lim : g.N;
    const int64_t m_base = (int64_t)tm * BM + (lane & 15);
    const int64_t n_base = n_tile0 + wave * WN + (lane >> 4) * 4;
#pragma unroll
    for (int j = 0; j < TM; ++j) {
        const int64_t m = m_base + 16 * j;
        if (m >= g.M) continue;
#pragma unroll
        for (int i = 0; i < TN; ++i) {
            const int64_t n = n_base + 16 * i;
            if (n >= n_end) continue;
            v4f v = acc[i][j];
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] *= ts;
            if constexpr (OUT_F32) {
                float* o = static_cast<float*>(g.out) + (SPLITK ? (int64_t)blockIdx.y * g.M * g.N : 0) + m * g.N + n;
                if (n + 3 < n_end && (g.N & 3) == 0) {
                    *reinterpret_cast<float4*>(o) = make_float4(v[0], v[1], v[2], v[3]);
                } else {
                    for (int e = 0; e < 4; ++e)
                        if (n + e < n_end) o[e] = v[e];
                }
            } else {
                __bf16* o = static_cast<__bf16*>(g.out) + m * g.N + n;
                typedef __bf16 v4bf __attribute__((ext_vector_type(4)));
                if (n + 3 < n_end && (g.N & 3) == 0) {
                    const v4bf p = {(__bf16)v[0], (__bf16)v[1], (__bf16)v[2], (__bf16)v[3]};
                    __builtin_nontemporal_store(p, reinterpret_cast<v4bf*>(o));
                } else {
                    for (int e = 0; e < 4; ++e)
                        if (n + e < n_end) o[e] = (__bf16)v[e];
                }
            }
        }
    }
}

// out[i] = s_T(A) s_T(W) (partial[0][i] + partial[1][i] + ...), the splits added in their order, as bf16 or fp32
template <bool OUT_F32>
__global__ __launch_bounds__(256) void nv16_reduce_kernel(const float* __restrict__ partial, int splits, int64_t mn, const float* a_ts,
                                                          const float* w_ts, void* out)
{
    const float ts = (*a_ts) * (*w_ts);
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < mn; i += (int64_t)gridDim.x * 256) {
        float s = partial[i];
        for (int p = 1; p < splits; ++p) s += partial[(int64_t)p * mn + i];
        s *= ts;
        if constexpr (OUT_F32) static_cast<float*>(out)[i] = s;
        else static_cast<__bf16*>(out)[i] = (__bf16)s;
    }
}

// Split-K plan (see the MXFP4 kernels' plan: few tiles and a long K leave the launch bound by the latency of a handful of
// compute units' loads; here M = 128, N = 8192, K = 28672 is 32 tiles and 411 us, slower than a bf16 GEMM).  128 x 256
// (or 128 x 128) tiles, two workgroups per compute unit, at least 8 K-steps of 64 per part, at most sixteen parts.  A K-step takes about
// 0.93 us in a workgroup that has its compute unit to itself and half as much again when two share one; a 128 x 128 tile's
// takes 0.58 us.  The number of parts minimises the estimate (microseconds)
//     10 + K-steps per part x step time + (split only) 3 + splits x M x N x 8 bytes of partials at 8 TB/s
// (the partials are written and read back within microseconds: most of them never leave the last-level cache)
// and the product is split only for an estimated gain of at least 10 % over the unsplit launch (which uses the narrow
// tiles when the wide ones are at most a round and a quarter: see launch_gemm_nv16).
bool nv16_narrow_tiles(int64_t tiles_w, int cus)
{
    return 4 * tiles_w <= 5 * (int64_t)cus;
}

void plan_split_k_nv16(int64_t M, int64_t N, int64_t K, int cus, int* splits, int* steps, bool* narrow)
{
    *splits = 1;
    *steps = 0;
    *narrow = false;
    const int64_t tiles_m = (M + 127) / 128;
    const int64_t tiles_w = tiles_m * ((N + 255) / 256), tiles_n = tiles_m * ((N + 127) / 128);
    const int64_t slots = 2 * (int64_t)cus;
    const int kh = (int)(K >> 6);
    // every part is as slow as the slowest compute unit's, and that one runs two workgroups as soon as there are more
    // workgroups than compute units
    auto shared = [&](int64_t wgs) { return wgs <= cus ? 1.0 : 1.47; };
    double unsplit = 10.0 + kh * 0.93 * shared(tiles_w);
    if (nv16_narrow_tiles(tiles_w, cus)) unsplit = 10.0 + kh * 0.58 * shared(tiles_n);
    double best = 0.9 * unsplit;
    // parts of at least eight K-steps (whole multiples of eight), up to sixteen of them, of wide or of narrow tiles, on at most
    // two workgroups per compute unit
    for (int nar = 0; nar < 2; ++nar) {
        const int64_t tiles = nar ? tiles_n : tiles_w;
        const double step = nar ? 0.58 : 0.93;
        const int64_t s_max = std::min<int64_t>(std::min<int64_t>(slots / tiles, kh / 8), 16);
        for (int64_t s = 2; s <= s_max; ++s) {
            const int st = (int)(((kh + s - 1) / s + 7) / 8 * 8);
            const int64_t n = (kh + st - 1) / st;
            if (n < 2) continue;
            const double t = 10.0 + st * step * shared(n * tiles) + 3.0 + (double)n * (double)M * (double)N * 8.0 / 8.0e6;
            if (t < best) {
                best = t;
                *splits = (int)n;
                *steps = st;
                *narrow = nar != 0;
            }
        }
    }
}

int device_cus()
{
    return compute_units();
}

template <int BN, int STAGES>
hipError_t launch_tiles_ring(const Nv16Args& g, bool out_f32, hipStream_t st, int splits)
{
    constexpr size_t lds = STAGES * (size_t)(8 * 2048 + (BN / 16) * 512 + 4 * 256);
    const int tiles_n = (g.n_cols + BN - 1) / BN;
    if (splits > 1) {
        static LdsAttrOnce raised_s;
        auto k = gemm_nv16_kernel<BN, true, STAGES, true>;
        hipError_t es;
        if ((es = raised_s.ensure(reinterpret_cast<const void*>(k), (int)lds)) != hipSuccess) return es;
        hipLaunchKernelGGL(k, dim3((unsigned)(g.tiles_m * tiles_n), (unsigned)splits), dim3(256), lds, st, g);
        return hipGetLastError();
    }
    const dim3 grid((unsigned)(g.tiles_m * tiles_n));
    hipError_t e;
    static LdsAttrOnce raised[2];
    if (out_f32) {
        auto k = gemm_nv16_kernel<BN, true, STAGES>;
        if ((e = raised[1].ensure(reinterpret_cast<const void*>(k), (int)lds)) != hipSuccess) return e;
        hipLaunchKernelGGL(k, grid, dim3(256), lds, st, g);
    } else {
        auto k = gemm_nv16_kernel<BN, false, STAGES>;
        if ((e = raised[0].ensure(reinterpret_cast<const void*>(k), (int)lds)) != hipSuccess) return e;
        hipLaunchKernelGGL(k, grid, dim3(256), lds, st, g);
    }
    return hipGetLastError();
}

// Three stages (75 KB of LDS with 256 columns, two workgroups per compute unit).  (A ring of six or seven stages for launches
// with at most one workgroup per compute unit measured the same: N = K = 4096, M = 80: 43.1 against 43.5 us -- a K-step of
// such a launch is bound by the tile's own 64 MFMAs per wave, not by its loads.)
template <int BN>
hipError_t launch_tiles(const Nv16Args& g, bool out_f32, hipStream_t st, int splits = 1)
{
    if (g.n_cols <= 0) return hipSuccess;
    return launch_tiles_ring<BN, 3>(g, out_f32, st, splits);
}

}  // namespace

size_t nv16_workspace_bytes(int64_t M, int64_t K)
{
    return (size_t)(round_up(M, 16) * K * 2);
}

// bytes of fp32 partials a split-K run of this product needs (0: the product is not split)
size_t nv16_split_k_bytes(int64_t M, int64_t N, int64_t K)
{
    int splits, steps;
    bool narrow;
    plan_split_k_nv16(M, N, K, device_cus(), &splits, &steps, &narrow);
    return splits > 1 ? (size_t)splits * (size_t)M * (size_t)N * 4 : 0;
}

hipError_t launch_gemm_nv16(const void* a_codes, const void* a_scales, const float* a_ts, const void* w_codes,
                            const void* w_scales, const float* w_ts, int64_t M, int64_t N, int64_t K, void* out,
                            bool out_f32, void* workspace, void* partial, hipStream_t st)
{
    // 1. activations -> fp16 in operand order (workspace)
    const int64_t n_frags = round_up(M, 16) / 16 * (K / 128);
    hipLaunchKernelGGL(nv_x16_kernel, dim3((unsigned)((n_frags + 3) / 4)), dim3(256), 0, st, static_cast<const uint8_t*>(a_codes),
                       static_cast<const uint8_t*>(a_scales), static_cast<uint8_t*>(workspace), n_frags);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;

    // 2. the product.  Two workgroups per compute unit: a round of the chip is 2 * CUs tiles.  The tile columns that fill
    // whole rounds run as 128 x 256 tiles; what is left over runs as 128 x 128 tiles in a second launch when that fits it
    // into fewer rounds-worth of time (N = 10240 at M = 4096: 1280 wide tiles are two and a half rounds; 1024 of them
    // plus 512 narrow ones are two and a half rounds' worth of work in two and a half rounds' time).
    Nv16Args g{};
    g.x16 = static_cast<const uint8_t*>(workspace);
    g.w_codes = static_cast<const uint8_t*>(w_codes);
    g.w_scales = static_cast<const uint8_t*>(w_scales);
    g.a_ts = a_ts;
    g.w_ts = w_ts;
    g.out = out;
    g.M = M;
    g.N = N;
    g.K = K;
    g.tiles_m = (int)((M + 127) / 128);
    const int cus = device_cus();
    if (partial) {
        // few tiles, long K: every tile's K range shared by several workgroups, partial results added by a second kernel
        int splits, steps;
        bool narrow;
        plan_split_k_nv16(M, N, K, cus, &splits, &steps, &narrow);
        if (splits > 1) {
            g.out = partial;
            g.n_first = 0;
            g.n_cols = (int)N;
            g.split_steps = steps;
            if ((e = narrow ? launch_tiles<128>(g, true, st, splits) : launch_tiles<256>(g, true, st, splits)) != hipSuccess) return e;
            const int64_t mn = M * N;
            const unsigned rblocks = (unsigned)std::min<int64_t>((mn + 255) / 256, 256 * 16);
            if (out_f32) hipLaunchKernelGGL(nv16_reduce_kernel<true>, dim3(rblocks), dim3(256), 0, st, static_cast<const float*>(partial), splits, mn, a_ts, w_ts, out);
            else hipLaunchKernelGGL(nv16_reduce_kernel<false>, dim3(rblocks), dim3(256), 0, st, static_cast<const float*>(partial), splits, mn, a_ts, w_ts, out);
            return hipGetLastError();
        }
    }
    const int64_t slots = 2 * (int64_t)cus;
    const int64_t cols_w = (N + 255) / 256;                         // wide tile columns
    const int64_t tiles_w = cols_w * g.tiles_m;
    const int64_t full_cols = tiles_w / slots * slots / g.tiles_m;  // wide tile columns inside whole rounds
    const int64_t rest_cols = N - full_cols * 256;                  // output columns left over
    if (full_cols > 0 && full_cols < cols_w) {
        const int64_t narrow = (rest_cols + 127) / 128 * g.tiles_m;
        // time in units of a wide tile: ceil-rounds of wide tiles, against whole rounds + narrow tiles at half a unit each
        const double t_wide = (double)((tiles_w + slots - 1) / slots);
        const double t_split = (double)(full_cols * g.tiles_m / slots) + 0.5 * (double)((narrow + slots - 1) / slots);
        if (t_split < t_wide) {
            g.n_first = 0;
            g.n_cols = (int)(full_cols * 256);
            if ((e = launch_tiles<256>(g, out_f32, st)) != hipSuccess) return e;
            g.n_first = (int)(full_cols * 256);
            g.n_cols = (int)rest_cols;
            return launch_tiles<128>(g, out_f32, st);
        }
    }
    g.n_first = 0;
    g.n_cols = (int)N;
    // less than a round and a quarter of wide tiles (one per compute unit and a few doubled up, or compute units left
    // idle): 128 x 128 tiles spread the same work twice as finely (N = 10240, K = 8192 at M = 512: 136 -> 119 us;
    // N = 8192, K = 28672 at M = 512 without the split-K workspace: 412 -> 280 us)
    if (nv16_narrow_tiles(tiles_w, cus)) return launch_tiles<128>(g, out_f32, st);
    return launch_tiles<256>(g, out_f32, st);
}

}  // namespace fp4mr
