// Fused block-Hadamard rotation + FP4 microscaling quantization (arXiv 2509.23202, Section 4.2 item 1:
// online rotation X H_k with k in {16,32,64,128}, quantization and scale computation fused behind it).
//
// Design for gfx950.  The rotation is a small dense contraction y = x H_b over blocks of b elements; it runs
// on the bf16 MFMA (v_mfma_f32_16x16x32_bf16) with the +-1 Hadamard matrix held in registers as the A operand
// and 16 independent b-element vectors of the input as the B operand, loaded straight from global memory
// with one 16-byte load per lane (lane l: vector l%16, elements 8*(l/16)..+8 of a 32-element K-step).  The
// products are exact (+-x), accumulation is fp32.  Rows of the A operand are permuted so that every lane ends
// up with b'/4 CONSECUTIVE outputs of its vector, i.e. whole dwords of packed codes.  What remains for the
// vector ALU is |max|, two multiplies and the hardware FP4 pack per element, which keeps the kernel bound by
// HBM and not by VALU issue (a butterfly in registers costs about 10 VALU operations per element).
//
//   b' = operand width.  b = 16 uses b' = 32 with the block-diagonal matrix diag(H_16, H_16); Hadamard blocks of 64
//   and 128 also use b' = 32 and finish with butterfly levels across lanes (kronecker_levels) wherever the 16 vectors
//   of an MFMA group are consecutive along K; b' = 64 / 128 operands remain for caller-supplied dense rotations
//   and for small GEMM-order calls.
//   lane (g = l%16, q = l/16) of a "supertile" owns outputs [q*b'/4, (q+1)*b'/4) of vector g.
//
// Throughput is bound by the bytes in flight per compute unit: kernels keep registers low (many resident waves), ask
// for all of a wave's input before doing anything else and, for the built-in Hadamard, run one work item per wave /
// workgroup and leave load balancing to the hardware dispatcher.
//
// Normalisation 1/sqrt(b) is applied in fp32 after the contraction as y = fma(h, c_hi, h*c_lo) with
// c_hi + c_lo = 1/sqrt(b) to ~48 bits, so y is (almost always) the correctly rounded product.
#include "device_util.hpp"
#include "internal.hpp"
#include "layout.hpp"
#include "rq_core.hpp"

#include <type_traits>

namespace fp4mr {
namespace {

constexpr int kThreads = 256;
constexpr int kWavesPerBlock = kThreads / kWave;
constexpr int kAmaxPassBlocks = 1024;  // grid cap of the NVFP4 abs-max pass and of the tensor-scale fit pass (4096 partials)
constexpr int kFitRounds = 3;          // alternations of the tensor-scale fit
constexpr int kRangePassBlocks = 512;  // grid cap of the range pre-pass (two partials per wave: the same 4096 slots)

// Tensor-scale fit (Section 4.1 "Ingredient 1": alternating optimisation over the block scales and the per-tensor scale).
// With codes and group scales fixed the quantized tensor is s_T * v, v_i = s_G * E2M1(code_i), and the minimiser of
// sum (s_T v_i - x_i)^2 is sum x v / sum v v.  A lane adds its values' terms in fp64: v has at most 6 significant bits
// and x is binary32, so every product is exact and only the additions round.
template <int NO, int ND, int NG, bool HW>
__device__ __forceinline__ void fit_accumulate(const float (&y)[NO], const uint32_t (&out)[ND], const uint32_t (&sc)[NG], double& num, double& den)
{
    typedef float v2f_t __attribute__((ext_vector_type(2)));
    constexpr int DPG = ND / NG;  // code dwords per group
#pragma unroll
    for (int gi = 0; gi < NG; ++gi) {
        const float s_G = e4m3_decode<HW>(sc[gi]);
#pragma unroll
        for (int d = 0; d < DPG; ++d) {
            const uint32_t p = out[gi * DPG + d];
            const v2f_t q0 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(p, 1.0f, 0);
            const v2f_t q1 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(p, 1.0f, 1);
            const v2f_t q2 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(p, 1.0f, 2);
            const v2f_t q3 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(p, 1.0f, 3);
            const float q[8] = {q0[0], q0[1], q1[0], q1[1], q2[0], q2[1], q3[0], q3[1]};
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const double v = (double)(q[i] * s_G);  // exact in binary32
                num = fma((double)y[(gi * DPG + d) * 8 + i], v, num);
                den = fma(v, v, den);
            }
        }
    }
}

// the wave's two sums -> its slot of the partials (one slot per wave, no atomics: fixed order, deterministic)
__device__ __forceinline__ void fit_store_partial(double num, double den, double* partial, int64_t wave, int lane)
{
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) {
        num += __shfl_xor(num, m);
        den += __shfl_xor(den, m);
    }
    if (lane == 0) {
        partial[2 * wave] = num;
        partial[2 * wave + 1] = den;
    }
}

struct RqArgs {
    const void* x;
    uint8_t* codes;
    uint8_t* scales;
    float* tensor_scale;   // NVFP4: s_T (written by the quantize pass unless static); fitted scale range: alpha, beta, 256 scale values
    uint32_t* amax_bits;   // NVFP4 dynamic: bit pattern of max |y| over the tensor (workspace)
    uint32_t* amax_partial;  // NVFP4 dynamic: one partial maximum per wave of the abs-max pass (workspace); range pass: max and min per wave
    int n_partials;          // > 0: the quantize pass reduces that many partials itself (small calls: no finalize launch)
    double* fit_partial;     // tensor-scale fit: per wave of the fit pass, sum x v and sum v v (workspace)
    int64_t rows, K;
    int64_t n_items;
    int b;                 // rotation block (1 = none)
    const uint16_t* rot;   // dense rotation: bf16 [b, b] row-major, y = x . rot (null: normalised Hadamard)
    float c_hi, c_lo;      // 1/sqrt(b) split in two floats (1 and 0 for a dense rotation)
    int static_scale;
};

// Fitted scale range (appendix on MXFP scale fitting): what the quantize pass needs of (alpha, beta), read from the
// buffer that the range pre-pass (or the caller) filled: [0] alpha, [1] beta, [2 .. 257] the 256 scale values.
constexpr float kLog2Of6 = 2.5849625007211562f;
struct FitRange {
    float lmin, inv;
    const float* table;
};
__device__ __forceinline__ FitRange load_fit_range(const RqArgs& a)
{
    const float alpha = a.tensor_scale[0], beta = a.tensor_scale[1];
    FitRange f;
    f.lmin = beta + kLog2Of6;
    f.inv = alpha > 0.0f ? __fdiv_rn(1.0f, alpha) : 0.0f;
    f.table = a.tensor_scale + 2;
    return f;
}

// range pre-pass: the wave's largest group abs-max and its smallest non-zero one -> its two slots of the partials
__device__ __forceinline__ void range_store_partial(float rmax, float rmin, uint32_t* partial, int64_t wave, int lane)
{
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) {
        rmax = fmaxf(rmax, __shfl_xor(rmax, m));
        rmin = fminf(rmin, __shfl_xor(rmin, m));
    }
    if (lane == 0) {
        partial[2 * wave] = __float_as_uint(rmax);
        partial[2 * wave + 1] = __float_as_uint(rmin);  // +inf: the wave saw no non-zero group
    }
}

// NVFP4 tensor scale as the quantize pass sees it: caller-supplied, or abs-max / 2688 with the abs-max taken from the
// finalized word or -- small calls -- reduced here from the abs-max pass's per-wave partials (every wave computes the
// same maximum: order-independent).  Non-negative floats order like their bit patterns.
__device__ __forceinline__ float load_tensor_scale(const RqArgs& a, int lane)
{
    if (a.static_scale) return *a.tensor_scale;
    uint32_t m;
    if (a.n_partials > 0) {
        m = 0;
        for (int i = lane; i < a.n_partials; i += 64) m = max(m, a.amax_partial[i]);
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) m = max(m, (uint32_t)__shfl_xor((int)m, d));
    } else {
        m = *a.amax_bits;
    }
    return __fdiv_rn(__uint_as_float(m), 2688.0f);
}

template <int LAYOUT>
__device__ __forceinline__ int64_t codes_offset_gemm(int64_t row, int64_t k, int64_t KC)
{
    return ((row >> 4) * KC + (k >> 7)) * 1024 + ((((k & 127) >> 5) * 16 + (row & 15)) << 4) + ((k & 31) >> 1);
}

__device__ __forceinline__ int64_t mx_scale_offset_gemm(int64_t row, int64_t kg, int64_t KS)
{
    return ((((row >> 4) * KS + (kg >> 4)) * 64 + ((kg & 3) * 16 + (row & 15))) << 2) + ((kg >> 2) & 3);
}

__device__ __forceinline__ int64_t nv_scale_offset_gemm(int64_t row, int64_t g16, int64_t KC)
{
    return ((((row >> 4) * KC + (g16 >> 3)) * 64 + (((g16 & 7) >> 1) * 16 + (row & 15))) << 1) + (g16 & 1);
}

template <int ND>
__device__ __forceinline__ void store_codes(uint8_t* p, const uint32_t (&w)[ND])
{
    if constexpr (ND == 1) {
        __builtin_nontemporal_store(w[0], reinterpret_cast<uint32_t*>(p));
    } else if constexpr (ND == 2) {
        const v2i v = {(int)w[0], (int)w[1]};
        __builtin_nontemporal_store(v, reinterpret_cast<v2i*>(p));
    } else {
        const v4i v = {(int)w[0], (int)w[1], (int)w[2], (int)w[3]};
        __builtin_nontemporal_store(v, reinterpret_cast<v4i*>(p));
    }
}

// The same operand for a caller-supplied rotation (arXiv 2509.23202, Section 4.2 item 1: below k = 256 a dense
// k x k transform stays memory-bound, so any rotation costs what the Hadamard costs): A[i][k] = R[32s + k][c(t,i)]
// taken from the bf16 matrix R [b, b] in global memory (16-byte aligned), block-diagonal when b < BP.
// A lane's eight operand elements run down a COLUMN of R, so the workgroup first writes the b' x b' matrix transposed
// into LDS (rows read with 16-byte loads, lanes along the rows of R: the 2-byte LDS writes of a wave fall into
// consecutive addresses), then every lane fetches its BP*BP/64 elements with 16-byte LDS reads.  Row stride b' + 8
// elements keeps those reads 16-byte aligned.  All threads of the workgroup must call this (it has a barrier).
template <int BP>
constexpr int kDenseLdsBytes = BP * (BP + 8) * 2;

template <int BP>
__device__ __forceinline__ void build_dense_operand(v8bf (&hop)[BP / 16][BP / 32], int g, int q, int b, const uint16_t* __restrict__ rot,
                                                    unsigned char* lds)
{
    constexpr int S = BP / 32, T = BP / 16, NO = BP / 4, STRIDE = BP + 8;
    uint16_t* const rt = reinterpret_cast<uint16_t*>(lds);
    const unsigned bm = (unsigned)b - 1u;
    for (int idx = (int)threadIdx.x; idx < BP * BP / 8; idx += (int)blockDim.x) {
        const unsigned r = (unsigned)idx % BP, c0 = 8u * ((unsigned)idx / BP);
        const bool same = (r & ~bm) == (c0 & ~bm);  // b >= 16: a chunk of eight columns stays inside one diagonal block
        v4i v = {0, 0, 0, 0};
        if (same) v = *reinterpret_cast<const v4i*>(rot + (size_t)(r & bm) * (unsigned)b + (c0 & bm));
#pragma unroll
        for (unsigned e = 0; e < 8; ++e) rt[(c0 + e) * STRIDE + r] = (uint16_t)((uint32_t)v[e >> 1] >> (16 * (e & 1)));
    }
    __syncthreads();
#pragma unroll
    for (int t = 0; t < T; ++t) {
        const int c = (g >> 2) * NO + 4 * t + (g & 3);
#pragma unroll
        for (int s = 0; s < S; ++s) hop[t][s] = *reinterpret_cast<const v8bf*>(rt + c * STRIDE + 32 * s + 8 * q);
    }
}

// ------------------------------------------------------------------------------------------------------
// MFMA rotation kernel.  BP = b' in {32,64,128}; G = 32 (MXFP4) or 16 (NVFP4); LAYOUT 0 canonical / 1 GEMM;
// PASS 0 = quantize, 1 = tensor abs-max only (NVFP4 pre-pass), 2 = sums of the tensor-scale fit, 3 = largest and smallest
// non-zero group abs-max (pre-pass of the fitted scale range).  POL = scale policy (GroupQuant::run; 3 = fitted range).
//
// Work item = FR * (128/BP) supertiles = FR * 2048 elements.
//   canonical: supertiles are consecutive runs of 16 vectors in flat (row-major) order;
//   GEMM:      an item is FR fragments (16 rows x 128 K); supertile u covers K-offset u*BP of all 16 rows.
template <int BP, int G, int LAYOUT, int PASS, bool HW, int FR, int POL>
__global__ __launch_bounds__(kThreads) void rq_mfma_kernel(RqArgs a)
{
    constexpr int S = BP / 32;           // K-steps of the contraction
    constexpr int T = BP / 16;           // output tiles
    constexpr int NO = BP / 4;           // outputs per lane
    constexpr int NST = FR * (128 / BP); // supertiles per item
    using GQ = GroupQuant<G, NO, 16, HW>;

    extern __shared__ __attribute__((aligned(16))) unsigned char rq_dyn_lds[];  // dense rotations: kDenseLdsBytes<BP>

    const int lane = threadIdx.x & 63;
    const int g = lane & 15, q = lane >> 4;
    const int64_t wave = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
    const int64_t n_waves = (int64_t)gridDim.x * kWavesPerBlock;

    v8bf hop[T][S];
    if (a.rot) build_dense_operand<BP>(hop, g, q, a.b, a.rot, rq_dyn_lds);  // (uniform branch: every thread takes it)
    else build_hadamard_operand<BP>(hop, g, q, a.b < BP ? a.b : BP);
    // Hadamard blocks wider than the operand: finished by butterfly levels across the lanes of a quad
    const int kron = (!a.rot && a.b > BP) ? (a.b == 2 * BP ? 1 : 2) : 0;

    // vectors in the tensor; the last one may be half a vector (16-element blocks and groups: rows * K = 16 * odd), its
    // missing half loads as zeros and is neither stored nor scaled
    const int64_t total = a.rows * a.K;
    const int64_t NV = (total + BP - 1) / BP;
    const int64_t KC = a.K >> 7;
    const int64_t KS = (a.K + 511) >> 9;
    const uint16_t* __restrict__ x = static_cast<const uint16_t*>(a.x);

    float s_T = 0.0f;
    if constexpr (G == 16 && PASS != 1) {
        s_T = load_tensor_scale(a, (int)(threadIdx.x & 63));
        if (!a.static_scale && blockIdx.x == 0 && threadIdx.x == 0) *a.tensor_scale = s_T;
    }
    float hmax = 0.0f;
    double fit_num = 0.0, fit_den = 0.0;
    float rmax = 0.0f, rmin = __builtin_inff();
    FitRange fr{0.0f, 0.0f, nullptr};
    if constexpr (POL == 3 && PASS == 0) fr = load_fit_range(a);

    for (int64_t item = wave; item < a.n_items; item += n_waves) {
        int64_t ebase[NST];
        int64_t row[NST], k0[NST];
        bool valid[NST], frag_ok[NST];
        v4i xin[NST][S];
#pragma unroll
        for (int u = 0; u < NST; ++u) {
            if constexpr (LAYOUT == 0) {
                const int64_t v = (item * NST + u) * 16 + g;
                valid[u] = v < NV;
                frag_ok[u] = true;
                ebase[u] = v * BP;
                row[u] = 0;
                k0[u] = 0;
            } else {
                const int64_t f = item * FR + u / (128 / BP);
                const int64_t rb = f / KC, kc = f - rb * KC;
                row[u] = rb * 16 + g;
                k0[u] = kc * 128 + (u % (128 / BP)) * BP;
                valid[u] = row[u] < a.rows;
                frag_ok[u] = rb * 16 < a.rows;  // (the last item may hold fewer than FR fragments)
                ebase[u] = row[u] * a.K + k0[u];
            }
#pragma unroll
            for (int s = 0; s < S; ++s) {
                v4i z = {0, 0, 0, 0};
                if constexpr (LAYOUT == 0 && S == 1) {
                    // streamed once, whole cache lines per instruction: keep it out of the caches
                    const bool ok = valid[u] && ebase[u] + 8 * q + 8 <= total;
                    xin[u][s] = ok ? __builtin_nontemporal_load(reinterpret_cast<const v4i*>(x + ebase[u] + 32 * s + 8 * q)) : z;
                } else {
                    xin[u][s] = valid[u] ? *reinterpret_cast<const v4i*>(x + ebase[u] + 32 * s + 8 * q) : z;
                }
            }
        }
#pragma unroll
        for (int u = 0; u < NST; ++u) {
            v4f acc[T];
#pragma unroll
            for (int t = 0; t < T; ++t) {
                acc[t] = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < S; ++s)
                    acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hop[t][s], __builtin_bit_cast(v8bf, xin[u][s]), acc[t], 0, 0, 0);
            }
            if constexpr (LAYOUT == 0) kronecker_levels<T>(acc, g, kron);  // the launcher sends wider blocks here only in canonical order
            if constexpr (PASS == 1) {
#pragma unroll
                for (int t = 0; t < T; ++t)
#pragma unroll
                    for (int v = 0; v < 4; ++v) hmax = fabs_max(hmax, acc[t][v]);
                continue;
            }
            float y[NO];
#pragma unroll
            for (int t = 0; t < T; ++t)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float h = acc[t][v];
                    y[4 * t + v] = __fmaf_rn(h, a.c_hi, h * a.c_lo);
                }
            if constexpr (PASS == 3) {
                // (vectors past the end were loaded as zeros: an all-zero group takes no part)
#pragma unroll
                for (int gi = 0; gi < GQ::NG; ++gi) {
                    const float am = GQ::group_amax(y, gi);
                    rmax = fmaxf(rmax, am);
                    if (am > 0.0f) rmin = fminf(rmin, am);
                }
                continue;
            }
            uint32_t out[GQ::ND], sc[GQ::NG];
            if constexpr (POL == 3) GQ::mx_fit(y, fr.lmin, fr.inv, fr.table, out, sc);
            else GQ::template run<POL>(y, s_T, out, sc);
            if constexpr (PASS == 2) {
                // (vectors past the end were loaded as zeros: they add nothing)
                if constexpr (G == 16) fit_accumulate<NO, GQ::ND, GQ::NG, HW>(y, out, sc, fit_num, fit_den);
                continue;
            }

            if constexpr (LAYOUT == 0) {
                const int64_t e0 = ebase[u] + q * NO;
                if (valid[u] && e0 + NO <= total) {
                    store_codes<GQ::ND>(a.codes + (e0 >> 1), out);
                    if ((q % GQ::LG) == 0) {
#pragma unroll
                        for (int gi = 0; gi < GQ::NG; ++gi) a.scales[e0 / G + gi] = (uint8_t)sc[gi];
                    }
                }
            } else {
                // padded rows are written too (zeros come out of zero inputs), the buffers include the padding
                if (!frag_ok[u]) continue;
                const int64_t kk = k0[u] + q * NO;
                store_codes<GQ::ND>(a.codes + codes_offset_gemm<1>(row[u], kk, KC), out);
                if ((q % GQ::LG) == 0) {
#pragma unroll
                    for (int gi = 0; gi < GQ::NG; ++gi) {
                        if constexpr (G == 32) a.scales[mx_scale_offset_gemm(row[u], (kk >> 5) + gi, KS)] = (uint8_t)sc[gi];
                        else a.scales[nv_scale_offset_gemm(row[u], (kk >> 4) + gi, KC)] = (uint8_t)sc[gi];
                    }
                }
            }
        }
    }
    if constexpr (PASS == 1) {
        // wave max -> one slot per wave (no atomics: thousands of waves finish together and would queue on one address)
#pragma unroll
        for (int m = 1; m < 64; m <<= 1) hmax = fmaxf(hmax, __shfl_xor(hmax, m));
        if (lane == 0) {
            const float ymax = __fmaf_rn(hmax, a.c_hi, hmax * a.c_lo);  // monotone: max|y| = y(max|h|)
            a.amax_partial[wave] = __float_as_uint(ymax);  // one slot per wave, reduced by amax_finalize_kernel
        }
    }
    if constexpr (PASS == 2) fit_store_partial(fit_num, fit_den, a.fit_partial, wave, lane);
    if constexpr (PASS == 3) range_store_partial(rmax, rmin, a.amax_partial, wave, lane);
}

// ------------------------------------------------------------------------------------------------------
// GEMM-layout writer for b' in {32, 64} (the hot path in front of the GEMM).  Same arithmetic as rq_mfma_kernel,
// different data movement, shaped for HBM:
//   * a work item is 16 rows x (KI * 16 * b') K = NF = KI * b'/8 fragments of one row-block (1024 K either way), and
//     it belongs to one workgroup: each of the four waves takes four of the rows.  The 16 vectors of one MFMA group
//     are 16 consecutive vectors of ONE row, so a load instruction reads 32 * b' contiguous bytes (1 KB for b' = 32)
//     and a wave has all its loads (4 KB for b' = 32) in flight at once (few registers: many resident waves);
//   * packed codes are staged through NF KB of LDS per workgroup and leave as one 16-byte-per-lane store per fragment
//     (1 KB contiguous, the fragment itself; the item's fragments are adjacent in memory), NF/4 fragments per wave;
//   * scale bytes are staged likewise and leave as whole dwords (MXFP4: four fragments complete each lane's dword;
//     NVFP4: 128 bytes per fragment).
// One item per workgroup, no grid-stride loop: the dispatcher balances the load.  Input loads and all stores are
// non-temporal: every byte is touched exactly once.
template <int BP, int G, bool HW, int KI, int POL>
__global__ __launch_bounds__(kThreads) void rq_frag_kernel(RqArgs a)
{
    constexpr int S = BP / 32, T = BP / 16, NO = BP / 4;
    constexpr int NF = KI * BP / 8;      // fragments per item
    constexpr int IK = KI * 16 * BP;     // K-elements per item: KI groups of 16 vectors per row
    constexpr int RPW = 16 / kWavesPerBlock;  // rows per wave
    constexpr int FPW = NF / kWavesPerBlock;  // fragments stored per wave
    constexpr int SC_BYTES = (G == 32) ? (NF / 4) * 256 : NF * 128;
    static_assert(kWavesPerBlock == 4 && NF % kWavesPerBlock == 0 && NF / 4 <= kWavesPerBlock, "rows and fragments are dealt to four waves");
    using GQ = GroupQuant<G, NO, 16, HW>;

    __shared__ __attribute__((aligned(16))) uint32_t sc_codes[NF * 256];
    __shared__ __attribute__((aligned(16))) uint8_t sc_scales[SC_BYTES];

    const int lane = threadIdx.x & 63;
    const int wib = threadIdx.x >> 6;
    const int g = lane & 15, q = lane >> 4;

    const int KC = (int)(a.K >> 7), KS = (int)((a.K + 511) >> 9);
    // grid: x = the item's position along K, (y, z) = row-block -- no division anywhere on the way to the first load
    const int ik = (int)blockIdx.x;
    const int64_t rb = (int64_t)blockIdx.z * gridDim.y + blockIdx.y;
    if (rb * 16 >= a.rows) return;  // whole workgroup (the last z-slice may be ragged)
    const uint16_t* __restrict__ x = static_cast<const uint16_t*>(a.x);

    // Loads first: the operand set-up below runs under their latency.  What bounds this kernel is the number of bytes
    // in flight per compute unit (resident waves x bytes per wave), so a wave asks for all RPW * KI * S KB at once.
    const int64_t k_lane = (int64_t)ik * IK + g * BP + 8 * q;   // first of this lane's input elements (group 0)
    v4i xin[RPW][KI][S];
#pragma unroll
    for (int u = 0; u < RPW; ++u) {
        const int64_t row = rb * 16 + wib * RPW + u;
#pragma unroll
        for (int kk = 0; kk < KI; ++kk) {
            // the whole vector exists or not (K is a multiple of b')
            const bool ok = row < a.rows && (int64_t)ik * IK + kk * 16 * BP + g * BP < a.K;
#pragma unroll
            for (int s = 0; s < S; ++s) {
                v4i z = {0, 0, 0, 0};
                const v4i* p = reinterpret_cast<const v4i*>(x + row * a.K + k_lane + kk * 16 * BP + 32 * s);
                xin[u][kk][s] = ok ? __builtin_nontemporal_load(p) : z;
            }
        }
    }

    v8bf hop[T][S];
    build_hadamard_operand<BP>(hop, g, q, a.b < BP ? a.b : BP);  // (the launcher sends dense rotations to rq_mfma_kernel)
    // Hadamard blocks wider than the operand: finished by butterfly levels across the lanes of a quad
    const int kron = a.b > BP ? (a.b == 2 * BP ? 1 : 2) : 0;

    float s_T = 0.0f;
    if constexpr (G == 16) {
        s_T = load_tensor_scale(a, (int)(threadIdx.x & 63));
        if (!a.static_scale && blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0 && threadIdx.x == 0) *a.tensor_scale = s_T;
    }

    FitRange fr{0.0f, 0.0f, nullptr};
    if constexpr (POL == 3) fr = load_fit_range(a);

    // this lane's NO outputs of a vector of group kk start at element kk*16*BP + e_grp of the item's K range
    const int e_grp = g * BP + q * NO;

#pragma unroll
    for (int u = 0; u < RPW; ++u) {
#pragma unroll
        for (int kk = 0; kk < KI; ++kk) {
            v4f acc[T];
#pragma unroll
            for (int t = 0; t < T; ++t) {
                acc[t] = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < S; ++s)
                    acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hop[t][s], __builtin_bit_cast(v8bf, xin[u][kk][s]), acc[t], 0, 0, 0);
            }
            kronecker_levels<T>(acc, g, kron);
            float y[NO];
#pragma unroll
            for (int t = 0; t < T; ++t)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float h = acc[t][v];
                    y[4 * t + v] = __fmaf_rn(h, a.c_hi, h * a.c_lo);
                }
            uint32_t out[GQ::ND], sc[GQ::NG];
            if constexpr (POL == 3) GQ::mx_fit(y, fr.lmin, fr.inv, fr.table, out, sc);
            else GQ::template run<POL>(y, s_T, out, sc);
            const int rr = wib * RPW + u;  // row inside the row-block
            const int fr = kk * (BP / 8) + (e_grp >> 7), e0 = e_grp & 127;  // fragment of the item, offset inside it
            const int d = fr * 256 + ((((e0 >> 5) * 16 + rr) << 2) + ((e0 & 31) >> 3));
            if constexpr (GQ::ND == 1) sc_codes[d] = out[0];
            else *reinterpret_cast<uint2*>(sc_codes + d) = make_uint2(out[0], out[1]);
            if ((q % GQ::LG) == 0) {
                if constexpr (G == 32) {
                    sc_scales[(fr >> 2) * 256 + ((((e0 >> 5) * 16 + rr) << 2) + (fr & 3))] = (uint8_t)sc[0];
                } else {
#pragma unroll
                    for (int gi = 0; gi < GQ::NG; ++gi) {
                        const int g16 = (e0 >> 4) + gi;
                        sc_scales[fr * 128 + (((g16 >> 1) * 16 + rr) << 1) + (g16 & 1)] = (uint8_t)sc[gi];
                    }
                }
            }
        }
    }
    __syncthreads();

    // the item's fragments leave in one piece each (fragments past the end of K do not exist)
#pragma unroll
    for (int i = 0; i < FPW; ++i) {
        const int f = wib * FPW + i;
        const int kc = ik * NF + f;
        if (kc < KC) {
            const v4i frag = *reinterpret_cast<const v4i*>(sc_codes + f * 256 + lane * 4);
            __builtin_nontemporal_store(frag, reinterpret_cast<v4i*>(a.codes + ((rb * KC + kc) * 1024 + lane * 16)));
            if constexpr (G == 16) {
                if (lane < 32) {
                    const uint32_t w = *reinterpret_cast<const uint32_t*>(sc_scales + f * 128 + lane * 4);
                    __builtin_nontemporal_store(w, reinterpret_cast<uint32_t*>(a.scales + ((rb * KC + kc) * 128 + lane * 4)));
                }
            }
        }
    }
    if constexpr (G == 32) {
        // bytes of fragments past the end of K (K/128 not a multiple of 4) are padding: never read
        if (wib < NF / 4) {
            const int ks = ik * (NF / 4) + wib;
            if (ks < KS) {
                const uint32_t w = *reinterpret_cast<const uint32_t*>(sc_scales + wib * 256 + lane * 4);
                __builtin_nontemporal_store(w, reinterpret_cast<uint32_t*>(a.scales + ((rb * KS + ks) * 256 + lane * 4)));
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------------
// No-rotation kernel (had_block = 1), bf16 or fp32 input.  Lane handles 8 consecutive elements; a group of G
// spans G/8 adjacent lanes.  Work item = 2048 elements (256 lane-pieces, 4 per lane).
//   canonical: flat;   GEMM: item = fragment, piece p = j*64+lane: row = p/16, K-offset 8*(p%16).
template <typename TIN, int G, int LAYOUT, int PASS, bool HW, int POL>
__global__ __launch_bounds__(kThreads) void q_direct_kernel(RqArgs a)
{
    using GQ = GroupQuant<G, 8, 1, HW>;
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
    const int64_t n_waves = (int64_t)gridDim.x * kWavesPerBlock;
    const int64_t total = a.rows * a.K;
    const int64_t KC = a.K >> 7;
    const int64_t KS = (a.K + 511) >> 9;
    const TIN* __restrict__ x = static_cast<const TIN*>(a.x);

    float s_T = 0.0f;
    if constexpr (G == 16 && PASS != 1) {
        s_T = load_tensor_scale(a, (int)(threadIdx.x & 63));
        if (!a.static_scale && blockIdx.x == 0 && threadIdx.x == 0) *a.tensor_scale = s_T;
    }
    float hmax = 0.0f;
    double fit_num = 0.0, fit_den = 0.0;
    float rmax = 0.0f, rmin = __builtin_inff();
    FitRange fr{0.0f, 0.0f, nullptr};
    if constexpr (POL == 3 && PASS == 0) fr = load_fit_range(a);

    for (int64_t item = wave; item < a.n_items; item += n_waves) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int p = j * 64 + lane;
            int64_t e0, row = 0, kk = 0;
            bool valid;
            if constexpr (LAYOUT == 0) {
                e0 = item * 2048 + (int64_t)p * 8;
                valid = e0 < total;
            } else {
                const int64_t rb = item / KC, kc = item - rb * KC;
                row = rb * 16 + (p >> 4);
                kk = kc * 128 + (p & 15) * 8;
                valid = row < a.rows;
                e0 = row * a.K + kk;
            }
            float y[8];
            if (valid) {
                if constexpr (sizeof(TIN) == 2) {
                    const uint4 w = *reinterpret_cast<const uint4*>(x + e0);
                    const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        y[2 * i] = __uint_as_float(ww[i] << 16);
                        y[2 * i + 1] = __uint_as_float(ww[i] & 0xffff0000u);
                    }
                } else {
                    const float4 f0 = *reinterpret_cast<const float4*>(x + e0);
                    const float4 f1 = *reinterpret_cast<const float4*>(x + e0 + 4);
                    y[0] = f0.x; y[1] = f0.y; y[2] = f0.z; y[3] = f0.w;
                    y[4] = f1.x; y[5] = f1.y; y[6] = f1.z; y[7] = f1.w;
                }
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) y[i] = 0.0f;
            }
            if constexpr (PASS == 1) {
#pragma unroll
                for (int i = 0; i < 8; ++i) hmax = fabs_max(hmax, y[i]);
                continue;
            }
            if constexpr (PASS == 3) {
                const float am = GQ::group_amax(y, 0);
                rmax = fmaxf(rmax, am);
                if (am > 0.0f) rmin = fminf(rmin, am);
                continue;
            }
            uint32_t out[1], sc[1];
            if constexpr (POL == 3) GQ::mx_fit(y, fr.lmin, fr.inv, fr.table, out, sc);
            else GQ::template run<POL>(y, s_T, out, sc);
            if constexpr (PASS == 2) {
                if constexpr (G == 16) fit_accumulate<8, 1, 1, HW>(y, out, sc, fit_num, fit_den);
                continue;
            }
            if constexpr (LAYOUT == 0) {
                if (valid) {
                    *reinterpret_cast<uint32_t*>(a.codes + (e0 >> 1)) = out[0];
                    if ((lane % GQ::LG) == 0) a.scales[e0 / G] = (uint8_t)sc[0];
                }
            } else {
                *reinterpret_cast<uint32_t*>(a.codes + codes_offset_gemm<1>(row, kk, KC)) = out[0];
                if ((lane % GQ::LG) == 0) {
                    if constexpr (G == 32) a.scales[mx_scale_offset_gemm(row, kk >> 5, KS)] = (uint8_t)sc[0];
                    else a.scales[nv_scale_offset_gemm(row, kk >> 4, KC)] = (uint8_t)sc[0];
                }
            }
        }
    }
    if constexpr (PASS == 1) {
#pragma unroll
        for (int m = 1; m < 64; m <<= 1) hmax = fmaxf(hmax, __shfl_xor(hmax, m));
        if (lane == 0) a.amax_partial[wave] = __float_as_uint(hmax);
    }
    if constexpr (PASS == 2) fit_store_partial(fit_num, fit_den, a.fit_partial, wave, lane);
    if constexpr (PASS == 3) range_store_partial(rmax, rmin, a.amax_partial, wave, lane);
}

// max over the per-wave partials of the abs-max pass (non-negative floats order like their bit patterns)
__global__ __launch_bounds__(1024) void amax_finalize_kernel(const uint32_t* partial, int n, uint32_t* out)
{
    __shared__ uint32_t red[16];
    uint32_t m = 0;
    for (int i = threadIdx.x; i < n; i += 1024) m = max(m, partial[i]);
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) m = max(m, (uint32_t)__shfl_xor((int)m, d));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 16; ++w) m = max(m, red[w]);
        *out = m;
    }
}

// s_T = amax / 2688 from the reduced abs-max (the tensor-scale fit starts from the abs-max tensor scale)
__global__ void tensor_scale_from_amax_kernel(const uint32_t* amax_bits, float* tensor_scale)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) *tensor_scale = __fdiv_rn(__uint_as_float(*amax_bits), 2688.0f);
}

// tensor step of the fit: the partial sums are added in a fixed order (thread t takes slots t, t + 256, ...; then a
// tree over the 256 threads), s_T = sum x v / sum v v rounded once to binary32; kept as it is when a sum is not positive
__global__ __launch_bounds__(256) void fit_finalize_kernel(const double* partial, int n_waves, float* tensor_scale)
{
    __shared__ double red[2][256];
    double num = 0.0, den = 0.0;
    for (int i = threadIdx.x; i < n_waves; i += 256) {
        num += partial[2 * i];
        den += partial[2 * i + 1];
    }
    red[0][threadIdx.x] = num;
    red[1][threadIdx.x] = den;
    __syncthreads();
    for (int w = 128; w >= 1; w >>= 1) {
        if ((int)threadIdx.x < w) {
            red[0][threadIdx.x] += red[0][threadIdx.x + w];
            red[1][threadIdx.x] += red[1][threadIdx.x + w];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0 && red[1][0] > 0.0 && red[0][0] > 0.0) *tensor_scale = (float)(red[0][0] / red[1][0]);
}

// Fitted scale range: (alpha, beta) from the per-wave extremes of the range pre-pass (n_waves > 0) or as the caller left
// them in out[0..1] (n_waves == 0), then the 256 scale values 2^(alpha q + beta), one per thread.
//     alpha = (log2 amax_max - log2 amax_min) / 255,   beta = log2 amax_min - log2 6      (binary32, v_log_f32 / v_exp_f32)
// No non-zero group at all: alpha = beta = 0.
__global__ __launch_bounds__(256) void range_finalize_kernel(const uint32_t* partial, int n_waves, float* out)
{
    __shared__ uint32_t red[2][256];
    __shared__ float ab[2];
    if (n_waves > 0) {
        uint32_t hi = 0, lo = 0x7f800000u;  // non-negative floats order like their bit patterns
        for (int i = threadIdx.x; i < n_waves; i += 256) {
            hi = max(hi, partial[2 * i]);
            lo = min(lo, partial[2 * i + 1]);
        }
        red[0][threadIdx.x] = hi;
        red[1][threadIdx.x] = lo;
        __syncthreads();
        for (int w = 128; w >= 1; w >>= 1) {
            if ((int)threadIdx.x < w) {
                red[0][threadIdx.x] = max(red[0][threadIdx.x], red[0][threadIdx.x + w]);
                red[1][threadIdx.x] = min(red[1][threadIdx.x], red[1][threadIdx.x + w]);
            }
            __syncthreads();
        }
        if (threadIdx.x == 0) {
            const float amax = __uint_as_float(red[0][0]), amin = __uint_as_float(red[1][0]);
            float alpha = 0.0f, beta = 0.0f;
            if (amax > 0.0f) {
                const float lmin = __log2f(amin), lmax = __log2f(amax);
                alpha = __fdiv_rn(lmax - lmin, 255.0f);
                beta = lmin - kLog2Of6;
            }
            ab[0] = alpha;
            ab[1] = beta;
            out[0] = alpha;
            out[1] = beta;
        }
    } else if (threadIdx.x == 0) {
        ab[0] = out[0];
        ab[1] = out[1];
    }
    __syncthreads();
    out[2 + threadIdx.x] = exp2f(__fmaf_rn(ab[0], (float)threadIdx.x, ab[1]));
}

// ------------------------------------------------------------------------------------------------------
template <int BP, int G, bool HW, int POL>
hipError_t launch_frag(const RqArgs& a0, int grid_cap, hipStream_t st, int* blocks_out)
{
    RqArgs a = a0;
    // One group of 16 vectors per row and item.  Twice that for b' = 32 (8 KB of loads per wave instead of 4) measured
    // 3-8 % slower at every size tried: the smaller workgroups keep more waves resident and drain more evenly.
    constexpr int KI = 1;
    constexpr int IK = KI * 16 * BP;
    (void)grid_cap;
    // one item per workgroup: x = items along K, (y, z) = row-blocks
    const int64_t rbs = round_up(a.rows, 16) / 16, ipr = (a.K + IK - 1) / IK;
    a.n_items = rbs * ipr;
    const int64_t gy = rbs < 32768 ? rbs : 32768, gz = (rbs + gy - 1) / gy;
    if (rbs < 1 || gz > 65535 || ipr > 0x7fffffffll) return hipErrorInvalidValue;
    if (blocks_out) *blocks_out = (int)(ipr * gy * gz);
    hipLaunchKernelGGL((rq_frag_kernel<BP, G, HW, KI, POL>), dim3((unsigned)ipr, (unsigned)gy, (unsigned)gz), dim3(kThreads), 0, st, a);
    return hipGetLastError();
}

// The fragment-shaped kernel is for big calls with the built-in Hadamard (a few-token call has too few of its items
// to fill the GPU; a dense rotation gathers its operand per wave and wants several items per wave).
inline bool frag_kernel_eligible(const RqArgs& a)
{
    return round_up(a.rows, 16) / 16 * ((a.K + 511) / 512) >= 1024 && !a.rot;
}

template <int BP, int G, int LAYOUT, int PASS, bool HW, int POL>
hipError_t launch_mfma(const RqArgs& a0, int grid_cap, hipStream_t st, int* blocks_out)
{
    if constexpr (LAYOUT == 1 && PASS == 0 && BP <= 64) {
        // The fragment-shaped kernel walks 16 rows x 512 K per wave, which is what HBM likes for big tensors; a
        // few-token call has too few of those items to fill the GPU, so it keeps the one-fragment-per-wave kernel.
        if (frag_kernel_eligible(a0)) return launch_frag<BP, G, HW, POL>(a0, grid_cap, st, blocks_out);
    }
    // two fragments' worth of loads in flight per wave for the widest block (its operand takes half the registers,
    // so few waves are resident); an item may run past the end and is masked per vector / per fragment
    constexpr int FR = (BP == 128) ? 2 : 1;
    RqArgs a = a0;
    if (LAYOUT == 0) {
        const int64_t nv = (a.rows * a.K + BP - 1) / BP;  // (a trailing half vector counts)
        const int64_t nst = (nv + 15) / 16;
        a.n_items = (nst + FR * (128 / BP) - 1) / (FR * (128 / BP));
    } else {
        const int64_t nf = round_up(a.rows, 16) / 16 * (a.K / 128);
        a.n_items = (nf + FR - 1) / FR;
    }
    int64_t blocks = (a.n_items + kWavesPerBlock - 1) / kWavesPerBlock;
    if (blocks > grid_cap) blocks = grid_cap;
    if (blocks < 1) blocks = 1;
    if (blocks_out) *blocks_out = (int)blocks;
    const size_t lds = a.rot ? (size_t)kDenseLdsBytes<BP> : 0;  // staging of the transposed rotation matrix
    hipLaunchKernelGGL((rq_mfma_kernel<BP, G, LAYOUT, PASS, HW, FR, POL>), dim3((unsigned)blocks), dim3(kThreads), lds, st, a);
    return hipGetLastError();
}

template <typename TIN, int G, int LAYOUT, int PASS, bool HW, int POL>
hipError_t launch_direct(const RqArgs& a0, int grid_cap, hipStream_t st, int* blocks_out)
{
    RqArgs a = a0;
    if (LAYOUT == 0) a.n_items = (a.rows * a.K + 2047) / 2048;
    else a.n_items = round_up(a.rows, 16) / 16 * (a.K / 128);
    int64_t blocks = (a.n_items + kWavesPerBlock - 1) / kWavesPerBlock;
    if (blocks > grid_cap) blocks = grid_cap;
    if (blocks < 1) blocks = 1;
    if (blocks_out) *blocks_out = (int)blocks;
    hipLaunchKernelGGL((q_direct_kernel<TIN, G, LAYOUT, PASS, HW, POL>), dim3((unsigned)blocks), dim3(kThreads), 0, st, a);
    return hipGetLastError();
}

template <int G, int LAYOUT, int PASS, bool HW, int POL>
hipError_t dispatch_block(const RqArgs& a, bool in_f32, int grid_cap, hipStream_t st, int* blocks_out)
{
    if (a.b == 1) {
        if (in_f32) return launch_direct<float, G, LAYOUT, PASS, HW, POL>(a, grid_cap, st, blocks_out);
        return launch_direct<uint16_t, G, LAYOUT, PASS, HW, POL>(a, grid_cap, st, blocks_out);
    }
    if (a.b <= 32) return launch_mfma<32, G, LAYOUT, PASS, HW, POL>(a, grid_cap, st, blocks_out);
    // Hadamard blocks of 64 and 128 run on the 32-wide kernels plus butterfly levels across lanes wherever the
    // vectors of an MFMA group are consecutive along K: canonical order, and the big-call GEMM-order kernel.
    const bool k_consecutive = LAYOUT == 0 || frag_kernel_eligible(a);
    if (!a.rot && k_consecutive) return launch_mfma<32, G, LAYOUT, PASS, HW, POL>(a, grid_cap, st, blocks_out);
    if (a.b == 64) return launch_mfma<64, G, LAYOUT, PASS, HW, POL>(a, grid_cap, st, blocks_out);
    return launch_mfma<128, G, LAYOUT, PASS, HW, POL>(a, grid_cap, st, blocks_out);
}

template <int G, bool HW, int POL = 0>
hipError_t dispatch_layout_pass(const RqArgs& a, bool in_f32, int layout, int pass, int grid_cap, hipStream_t st, int* blocks_out = nullptr)
{
    if (pass == 1) return dispatch_block<G, 0, 1, HW, 0>(a, in_f32, grid_cap, st, blocks_out);  // layout and scale policy do not matter for the abs-max pass
    if constexpr (G == 32 && HW) {
        if (pass == 3) return dispatch_block<G, 0, 3, HW, 0>(a, in_f32, grid_cap, st, blocks_out);  // range pre-pass: extremes only
    }
    if constexpr (G == 16 && HW && POL == 1) {
        if (pass == 2) return dispatch_block<G, 0, 2, HW, 1>(a, in_f32, grid_cap, st, blocks_out);  // tensor-scale fit: sums only
    }
    if (layout == 0) return dispatch_block<G, 0, 0, HW, POL>(a, in_f32, grid_cap, st, blocks_out);
    return dispatch_block<G, 1, 0, HW, POL>(a, in_f32, grid_cap, st, blocks_out);
}

}  // namespace

hipError_t launch_rotate_quantize(const void* x, int64_t rows, int64_t K, int b, const void* rot, int fmt, bool in_f32,
                                  int layout_gemm, bool static_scale, int policy, void* codes, void* scales,
                                  float* tensor_scale, void* workspace, bool hw_codec, hipStream_t st)
{
    RqArgs a{};
    a.x = x;
    a.codes = static_cast<uint8_t*>(codes);
    a.scales = static_cast<uint8_t*>(scales);
    a.tensor_scale = tensor_scale;
    a.amax_bits = static_cast<uint32_t*>(workspace);
    a.rows = rows;
    a.K = K;
    a.b = b;
    a.rot = static_cast<const uint16_t*>(rot);
    const double c = rot ? 1.0 : 1.0 / sqrt((double)b);  // a dense rotation carries its own normalisation
    a.c_hi = (float)c;
    a.c_lo = (float)(c - (double)a.c_hi);
    a.static_scale = static_scale ? 1 : 0;
    // One work item per wave: the hardware's workgroup dispatcher balances the load better than a grid-stride loop
    // over resident waves does (measured on [16384, 8192]: 53 us against 59 us), and the per-wave set-up is cheap.
    // A dense rotation stages its operand through LDS once per workgroup: there the grid is capped at the workgroups
    // that are resident at once (b = 128: the operand takes 128 registers, two workgroups per compute unit; else eight)
    // and each wave walks several items.
    const int grid_cap = rot ? (b > 64 ? 256 * 2 : 256 * 8) : 1 << 20;

    hipError_t e;
    if (fmt == 1 && !static_scale) {
        // dynamic tensor scale: abs-max pass (one partial per wave) -> finalize -> quantize pass
        a.amax_partial = a.amax_bits + 64;
        const int pass_cap = kAmaxPassBlocks;
        int pass_blocks = 0;
        e = hw_codec ? dispatch_layout_pass<16, true>(a, in_f32, 0, 1, pass_cap, st, &pass_blocks)
                     : dispatch_layout_pass<16, false>(a, in_f32, 0, 1, pass_cap, st, &pass_blocks);
        if (e != hipSuccess) return e;
        // blocks that had no item still wrote their (zero) partial: every wave of the grid stores one
        const int n_partials = pass_blocks * kWavesPerBlock;
        if (n_partials <= 256 && policy != 3) {
            a.n_partials = n_partials;  // few-token calls: one launch less, the quantize pass reduces the partials itself
        } else {
            hipLaunchKernelGGL(amax_finalize_kernel, dim3(1), dim3(1024), 0, st, a.amax_partial, n_partials, a.amax_bits);
            if ((e = hipGetLastError()) != hipSuccess) return e;
        }
    }
    if (policy == 3) {
        // Alternating optimisation of the group scales and the tensor scale (Section 4.1 "Ingredient 1"): from the abs-max
        // tensor scale, kFitRounds times { group search with s_T fixed -> sums of x v and v v -> least-squares s_T }, then
        // the quantize pass proper with the final s_T.  Every pass reads *tensor_scale (written on the stream before it).
        if (fmt != 1 || static_scale) return hipErrorInvalidValue;
        hipLaunchKernelGGL(tensor_scale_from_amax_kernel, dim3(1), dim3(64), 0, st, a.amax_bits, a.tensor_scale);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        a.static_scale = 1;
        a.n_partials = 0;
        a.fit_partial = reinterpret_cast<double*>(static_cast<char*>(workspace) + 256 + 4096 * 4);
        for (int r = 0; r < kFitRounds; ++r) {
            int fit_blocks = 0;
            if ((e = dispatch_layout_pass<16, true, 1>(a, in_f32, 0, 2, kAmaxPassBlocks, st, &fit_blocks)) != hipSuccess) return e;
            hipLaunchKernelGGL(fit_finalize_kernel, dim3(1), dim3(256), 0, st, a.fit_partial, fit_blocks * kWavesPerBlock, a.tensor_scale);
            if ((e = hipGetLastError()) != hipSuccess) return e;
        }
        return dispatch_layout_pass<16, true, 1>(a, in_f32, layout_gemm, 0, grid_cap, st);
    }
    if (policy == 4) {
        // Scale byte fitted to the tensor's range of scales (appendix on MXFP scale fitting).  Dynamic: range pre-pass (one
        // pair of extremes per wave) -> (alpha, beta) and the 256 scale values -> quantize pass.  Static: the caller's
        // (alpha, beta) are in tensor_scale[0..1]; only the scale values are computed.
        if (fmt != 0 || !tensor_scale) return hipErrorInvalidValue;
        int range_blocks = 0;
        if (!static_scale) {
            a.amax_partial = a.amax_bits + 64;
            if ((e = dispatch_layout_pass<32, true>(a, in_f32, 0, 3, kRangePassBlocks, st, &range_blocks)) != hipSuccess) return e;
        }
        hipLaunchKernelGGL(range_finalize_kernel, dim3(1), dim3(256), 0, st, a.amax_partial, range_blocks * kWavesPerBlock, a.tensor_scale);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        return dispatch_layout_pass<32, true, 3>(a, in_f32, layout_gemm, 0, grid_cap, st);
    }
    if (policy == 1) {
        // the scale search is written with the hardware converts only
        return fmt == 0 ? dispatch_layout_pass<32, true, 1>(a, in_f32, layout_gemm, 0, grid_cap, st)
                        : dispatch_layout_pass<16, true, 1>(a, in_f32, layout_gemm, 0, grid_cap, st);
    }
    if (policy == 2) {
        if (fmt != 0) return hipErrorInvalidValue;
        return hw_codec ? dispatch_layout_pass<32, true, 2>(a, in_f32, layout_gemm, 0, grid_cap, st)
                        : dispatch_layout_pass<32, false, 2>(a, in_f32, layout_gemm, 0, grid_cap, st);
    }
    if (fmt == 0)
        return hw_codec ? dispatch_layout_pass<32, true>(a, in_f32, layout_gemm, 0, grid_cap, st)
                        : dispatch_layout_pass<32, false>(a, in_f32, layout_gemm, 0, grid_cap, st);
    return hw_codec ? dispatch_layout_pass<16, true>(a, in_f32, layout_gemm, 0, grid_cap, st)
                    : dispatch_layout_pass<16, false>(a, in_f32, layout_gemm, 0, grid_cap, st);
}

}  // namespace fp4mr
