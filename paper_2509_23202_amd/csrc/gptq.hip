// MR-GPTQ weight quantizer, the part that runs over the weight matrix (arXiv 2509.23202, Section 4: GPTQ quantizes
// all rows in one fixed column order and, after rounding a column, moves the columns not yet rounded by the
// optimal-brain update; Section 4.1: on rotated weights, with the scales fixed beforehand in the original column
// order and the columns visited in a static activation order).
//
// Given U, the upper-triangular factor of the damped inverse Hessian in visiting order (U^T U = Hinv), column j costs
//     q = Q(w_j / s),   e = (w_j - q s) / U[j,j],   w_k -= e U[j,k]  for every later column k.
// Rows never interact, so the sweep is data-parallel over the N rows and strictly sequential along K.  It is blocked
// 64 columns at a time: four lanes share a row and keep the block's 64 working weights in registers while the 64 x 64
// triangle of U is read from LDS; the block's 64 errors per row then update the later columns of the same 512-column
// outer block in a rank-64 product -- both by the wave that owns the 16 rows, one launch per outer block (outer
// kernel) -- and a finished outer block updates everything behind it in one rank-512 product (update kernel).  Working weights live in visiting order in an fp32 scratch matrix, codes in a
// byte-per-code scratch matrix, and a last kernel packs them back to the original column positions.
#include "device_util.hpp"
#include "internal.hpp"

#include <algorithm>
#include <cmath>

namespace fp4mr {
namespace {

constexpr int kB = 64;       // columns per block of the sequential sweep
constexpr int kOuter = 512;  // columns per outer block: later columns receive its errors in one rank-512 update

struct GptqArgs {
    const uint16_t* w;      // [N,K] bf16
    const float* U;         // [K,K] fp32, upper triangle used
    const int* perm;        // [K] or null
    int* iperm;             // [K] scratch
    float* wp;              // [N,K] scratch: working weights, visiting order
    uint8_t* q;             // [N,K] scratch: one code per byte, visiting order
    float* err;             // [N,kOuter] scratch: the errors of the current outer block
    const uint8_t* scales;  // [N,K/G] canonical
    const float* s_T;       // NVFP4 tensor scale (device), else null
    const float* table;     // 256 scale values indexed by the scale byte (fitted scale range), else null
    uint8_t* codes;         // [N,K/2] canonical
    int N, K, b, G;
    float c_hi, c_lo;       // 1/sqrt(b) in two floats
    float factor;           // 4/3 for scales that leave that factor out, else 1
};

__device__ __forceinline__ int visit_col(const GptqArgs& a, int j)
{
    // an entry outside [0, K) (not a permutation: caller error) is clamped, so that no access leaves the buffers
    const int c = a.perm ? a.perm[j] : j;
    return min(max(c, 0), a.K - 1);
}

__global__ void gptq_iperm_fill_kernel(GptqArgs a)
{
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j < a.K) a.iperm[j] = j;
}

__global__ void gptq_iperm_kernel(GptqArgs a)
{
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j < a.K) a.iperm[visit_col(a, j)] = j;
}

// wp[n, j] = (W H_b)[n, perm[j]]: the rotated weight of the column visited j-th.  One workgroup per row: the row is
// copied to LDS and rotated there in natural column order (sums of up to 128 bf16 values in fp32 -- exact unless their exponents spread
// over more than 16 bits -- then one multiplication by 1/sqrt(b) carried in two floats; neighbouring threads read the
// same block, so the loads are broadcasts), and read back from LDS in visiting order for coalesced stores.
__global__ __launch_bounds__(256) void gptq_rotate_gather_kernel(GptqArgs a)
{
    extern __shared__ float rowbuf[];  // K floats (the rotated row), then K bf16 (the row as read)
    uint16_t* const xs = reinterpret_cast<uint16_t*>(rowbuf + a.K);
    const int n = blockIdx.x;
    const uint32_t* x2 = reinterpret_cast<const uint32_t*>(a.w + (int64_t)n * a.K);
    for (int i = threadIdx.x; i < a.K / 2; i += 256) reinterpret_cast<uint32_t*>(xs)[i] = x2[i];
    __syncthreads();
    for (int col = threadIdx.x; col < a.K; col += 256) {
        const int j0 = col & ~(a.b - 1), c = col - j0;
        float sum = 0.0f;
#pragma unroll 8
        for (int r = 0; r < a.b; ++r) {
            const float v = __uint_as_float((uint32_t)xs[j0 + r] << 16);
            sum += (__popc((unsigned)(r & c)) & 1) ? -v : v;
        }
        rowbuf[col] = (a.b == 1) ? sum : __fmaf_rn(sum, a.c_hi, sum * a.c_lo);
    }
    __syncthreads();
    for (int j = threadIdx.x; j < a.K; j += 256) a.wp[(int64_t)n * a.K + j] = rowbuf[visit_col(a, j)];
}

template <int FMT>
__device__ __forceinline__ float decode_scale(uint32_t byte, float s_T, float factor)
{
    if constexpr (FMT == 0) {
        // 2^(byte - 127); byte 0 is 2^-127 (a subnormal in binary32, formed exactly)
        const float p = byte ? __uint_as_float(byte << 23) : __uint_as_float(0x00400000u);
        return p * factor;
    } else {
        return e4m3_decode<false>(byte) * s_T;
    }
}

// 64 columns b0 .. b0+63 (visiting order) of 16 rows per wave: four neighbouring lanes share a row, lane part p keeping
// the working weights of the block's columns 16p .. 16p+15 in registers.  At column j the lane that owns it rounds it
// and computes the error, the error is broadcast inside the quad, and every lane updates its 16 registers with row j
// of the block's triangle of U, read from LDS (zero below the diagonal, so columns already visited need no masking: they
// are touched but never read again).
template <int OWNER>
__device__ __forceinline__ float quad_owner_value(float v)
{
    constexpr int ctrl = OWNER * 0x55;  // quad_perm: every lane of the quad reads lane OWNER
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), ctrl, 0xf, 0xf, true));
}

typedef float v2f_t __attribute__((ext_vector_type(2)));

// Columns 16 P .. 16 P + 15 of the block.  The rounding uses the converting instructions (round-to-nearest-even onto
// E2M1, saturating; decode back to fp32); the two divisions of the definition are multiplications by reciprocals
// formed once per block (exact for power-of-two scales and a unit diagonal).  The owner lanes keep their errors and
// codes in registers (ek, ck) and store them once at the end.
template <int P>
__device__ __forceinline__ void sweep_part(float (&w)[16], float (&ek)[16], uint32_t (&ck)[4], const float* Us, const float* Ru,
                                           const v2f_t* Sc, int row, int part)
{
    const bool mine = part == P;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int j = P * 16 + i;
        const v2f_t sc = Sc[j * 16 + row];  // scale, 1 / scale (0 for a zero scale)
        const float wj = w[i];              // meaningful in the lanes with part == P
        const float t = wj * sc[1];
        const uint32_t pk = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(0u, t, t, 1.0f, 0);
        const uint32_t code = (sc[0] > 0.0f) ? (pk & 15u) : 0u;
        const v2f_t qv = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(code, 1.0f, 0);
        const float dq = qv[0] * sc[0];
        const float e_own = (wj - dq) * Ru[j];
        ek[i] = mine ? e_own : ek[i];
        ck[i / 4] = mine ? (ck[i / 4] | (code << (8 * (i & 3)))) : ck[i / 4];
        const float e = quad_owner_value<P>(e_own);
        const float4* u4 = reinterpret_cast<const float4*>(Us + j * kB + part * 16);
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const float4 u = u4[v];
            w[4 * v] = __fmaf_rn(-e, u.x, w[4 * v]);
            w[4 * v + 1] = __fmaf_rn(-e, u.y, w[4 * v + 1]);
            w[4 * v + 2] = __fmaf_rn(-e, u.z, w[4 * v + 2]);
            w[4 * v + 3] = __fmaf_rn(-e, u.w, w[4 * v + 3]);
        }
    }
}

// One outer block (columns o .. oe-1 in visiting order) of 16 rows, one wave, no other wave involved: rows never
// interact, so the wave walks the outer block's 64-column blocks by itself -- sweep a block, then push that block's 64
// errors onto the rest of the outer block for its own rows -- and the whole outer block is a single launch.
//   * sweep: sweep_part above (four lanes per row);
//   * push: wp[rows, c] -= sum_j e[rows, j] U[b0 + j, c] for b0 + 64 <= c < oe, a [16 x 64] x [64 x 16] product per 16
//     columns on the fp32 MFMA (v_mfma_f32_16x16x4_f32): the negated errors go through LDS into the A operand once per
//     block, the rows of U come straight from global memory as the B operand (64 bytes per row per load), and the
//     accumulator starts as the working weights;
//   * the next block's columns were just written by other lanes of this wave: a workgroup-scope fence orders the stores
//     before the loads (one compute unit, one vector cache).
// The errors also go to err[N, kOuter] for the rank-512 update of everything behind the outer block.
template <int FMT>
__global__ __launch_bounds__(64) void gptq_outer_kernel(GptqArgs a, int o, int oe)
{
    // the block's triangle of U, 1 / U[j,j] and the columns' original positions: two buffers, the next block's set is
    // fetched into registers before the push and stored after it (its latency hides behind the push)
    __shared__ __attribute__((aligned(16))) float Us2[2][kB * kB];
    __shared__ float Ru2[2][kB];
    __shared__ int cols2[2][kB];
    __shared__ __attribute__((aligned(8))) v2f_t Sc[kB * 16];   // [column][row of the wave]: scale and its reciprocal
    __shared__ __attribute__((aligned(16))) float Es[16][kB + 4];  // negated errors of the block: [row][term]
    const int lane = threadIdx.x;
    const int row = lane >> 2, part = lane & 3;  // sweep: four lanes per row
    const int l16 = lane & 15, q = lane >> 4;    // push: MFMA operand coordinates
    const int n_raw = blockIdx.x * 16 + row;
    const bool live = n_raw < a.N;
    const int n = live ? n_raw : a.N - 1;  // idle lanes shadow the last row and store nothing
    const float s_T = (FMT == 1) ? *a.s_T : 1.0f;
    const uint8_t* srow = a.scales + (int64_t)n * (a.K / a.G);
    const int gshift = (a.G == 32) ? 5 : 4;
    const float* __restrict__ Ug = a.U;
    float up[kB * kB / 64];  // a block's triangle on its way to LDS: element (it, lane) = row it, column lane
    float rup;
    int cup;
    auto fetch_block = [&](int bb) {  // (unrolled: all 64 loads in flight together)
#pragma unroll
        for (int it = 0; it < kB * kB / 64; ++it) up[it] = (lane >= it) ? Ug[(int64_t)(bb + it) * a.K + bb + lane] : 0.0f;
        rup = Ug[(int64_t)(bb + lane) * a.K + bb + lane];
        cup = visit_col(a, bb + lane);
    };
    auto stash_block = [&](int buf) {
#pragma unroll
        for (int it = 0; it < kB * kB / 64; ++it) Us2[buf][it * 64 + lane] = up[it];
        Ru2[buf][lane] = 1.0f / rup;
        cols2[buf][lane] = cup;
    };
    fetch_block(o);
    stash_block(0);
    __syncthreads();
    for (int b0 = o; b0 < oe; b0 += kB) {
        const int cur = ((b0 - o) / kB) & 1;
        const float* Us = Us2[cur];
        const float* Ru = Ru2[cur];
        const int* cols = cols2[cur];

        float w[16];
        const float4* src = reinterpret_cast<const float4*>(a.wp + (int64_t)n * a.K + b0 + part * 16);
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const float4 t = src[v];
            w[4 * v] = t.x;
            w[4 * v + 1] = t.y;
            w[4 * v + 2] = t.z;
            w[4 * v + 3] = t.w;
        }
        uint32_t sbyte[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) sbyte[i] = srow[cols[part * 16 + i] >> gshift];  // sixteen independent loads in flight
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int j = part * 16 + i;
            const float sv = a.table ? a.table[sbyte[i]] : decode_scale<FMT>(sbyte[i], s_T, a.factor);
            Sc[j * 16 + row] = v2f_t{sv, sv > 0.0f ? 1.0f / sv : 0.0f};
        }
        __syncthreads();  // the scale of a column is read by every lane of its row's quad
        float ek[16];
        uint32_t ck[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int i = 0; i < 16; ++i) ek[i] = 0.0f;
        sweep_part<0>(w, ek, ck, Us, Ru, Sc, row, part);
        sweep_part<1>(w, ek, ck, Us, Ru, Sc, row, part);
        sweep_part<2>(w, ek, ck, Us, Ru, Sc, row, part);
        sweep_part<3>(w, ek, ck, Us, Ru, Sc, row, part);
        if (live) {
            float4* ed = reinterpret_cast<float4*>(a.err + (int64_t)n * kOuter + (b0 - o) + part * 16);
#pragma unroll
            for (int v = 0; v < 4; ++v) ed[v] = make_float4(ek[4 * v], ek[4 * v + 1], ek[4 * v + 2], ek[4 * v + 3]);
            *reinterpret_cast<uint4*>(a.q + (int64_t)n * a.K + b0 + part * 16) = make_uint4(ck[0], ck[1], ck[2], ck[3]);
        }
        if (b0 + kB >= oe) break;

        fetch_block(b0 + kB);  // lands while the push below runs
        // push the block's errors onto the rest of the outer block
#pragma unroll
        for (int v = 0; v < 4; ++v)
            *reinterpret_cast<float4*>(&Es[row][part * 16 + 4 * v]) = make_float4(-ek[4 * v], -ek[4 * v + 1], -ek[4 * v + 2], -ek[4 * v + 3]);
        __syncthreads();
        float ea[16];  // A operand of the 16 MFMAs of a column tile: row l16, terms 4 ks + q
#pragma unroll
        for (int ks = 0; ks < 16; ++ks) ea[ks] = Es[l16][ks * 4 + q];
        // a lane holds rows 4q .. 4q+3 of column l16 of the output tile
        int64_t wrow[4];
        bool wlive[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int nn = blockIdx.x * 16 + 4 * q + v;
            wlive[v] = nn < a.N;
            wrow[v] = (int64_t)min(nn, a.N - 1) * a.K;
        }
        const float* __restrict__ ub = Ug + (int64_t)(b0 + q) * a.K + l16;  // + 4 ks K + c0
        // 64 columns (four tiles) per trip, the next trip's operands loaded before this trip's MFMAs: a single wave has
        // nothing else to cover the loads' latency with
        v4f acc[4], accn[4];
        float u[4][16], un[4][16];
        auto fetch = [&](int c0, v4f (&ac)[4], float (&uu)[4][16]) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
#pragma unroll
                for (int v = 0; v < 4; ++v) ac[t][v] = a.wp[wrow[v] + c0 + 16 * t + l16];
#pragma unroll
                for (int ks = 0; ks < 16; ++ks) uu[t][ks] = ub[(int64_t)ks * 4 * a.K + c0 + 16 * t];
            }
        };
        fetch(b0 + kB, acc, u);
        for (int c0 = b0 + kB; c0 < oe; c0 += 2 * kB) {  // two trips per iteration so that the buffers swap statically
            const bool second = c0 + kB < oe;
            if (second) fetch(c0 + kB, accn, un);
#pragma unroll
            for (int ks = 0; ks < 16; ++ks)
#pragma unroll
                for (int t = 0; t < 4; ++t) acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(ea[ks], u[t][ks], acc[t], 0, 0, 0);
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (wlive[v]) a.wp[wrow[v] + c0 + 16 * t + l16] = acc[t][v];
            if (!second) break;
            if (c0 + 2 * kB < oe) fetch(c0 + 2 * kB, acc, u);
#pragma unroll
            for (int ks = 0; ks < 16; ++ks)
#pragma unroll
                for (int t = 0; t < 4; ++t) accn[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(ea[ks], un[t][ks], accn[t], 0, 0, 0);
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (wlive[v]) a.wp[wrow[v] + c0 + kB + 16 * t + l16] = accn[t][v];
        }
        stash_block(cur ^ 1);
        __threadfence_block();  // the next block's working weights were written by other lanes of this wave
        __syncthreads();
    }
}

// wp[n, c] -= sum_{j < rank} err[n, e0 + j] * U[u0 + j, c] for the columns c_begin <= c < c_end (visiting order): a dense
// fp32 contraction, on the fp32 MFMA (v_mfma_f32_16x16x4_f32; the terms enter four at a time in ascending order, where the
// column-by-column definition applies them singly -- the same sum up to fp32 rounding order).  128 x 128 output tile per
// workgroup, a 64 x 64 quarter per wave (16 MFMA tiles whose accumulators start as the working weights), the negated
// errors and the rows of U staged through LDS 32 terms at a time, the next 32 fetched while the current ones multiply.
__global__ __launch_bounds__(256) void gptq_update_kernel(GptqArgs a, int u0, int e0, int rank, int c_begin, int c_end)
{
    constexpr int T = 128, KC = 32, LD = T + 20, NT = 4, NL = KC * T / 256;
    __shared__ float Et[KC][LD];  // [term][row], negated
    __shared__ float Ut[KC][LD];  // [term][column]
    const int c0 = c_begin + blockIdx.x * T;
    const int n0 = blockIdx.y * T;
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, l16 = lane & 15, q = lane >> 4;
    const int wr = (wave >> 1) * 64, wc = (wave & 1) * 64;
    // a lane holds rows 4q .. 4q+3 of column l16 of every 16 x 16 tile; c_end and the tile start are multiples of 64, so
    // a wave's 64 columns are in or out together
    const bool in = c0 + wc < c_end;
    v4f acc[NT][NT];
#pragma unroll
    for (int i = 0; i < NT; ++i)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int n = min(n0 + wr + i * 16 + 4 * q + v, a.N - 1);
            const float* src = a.wp + (int64_t)n * a.K + c0 + wc + l16;
#pragma unroll
            for (int j = 0; j < NT; ++j) acc[i][j][v] = in ? src[j * 16] : 0.0f;
        }
    float re[NL], ru[NL];
    auto fetch = [&](int r0) {
#pragma unroll
        for (int it = 0; it < NL; ++it) {
            const int idx = it * 256 + tid;
            // both reads run along the contiguous index: the errors of a row are consecutive over the terms, a row of U over
            // the columns
            const int te = idx % KC, xe = idx / KC;
            const int n = min(n0 + xe, a.N - 1);
            re[it] = -a.err[(int64_t)n * kOuter + e0 + r0 + te];
            const int x = idx % T, t = idx / T;
            ru[it] = (c0 + x < c_end) ? a.U[(int64_t)(u0 + r0 + t) * a.K + c0 + x] : 0.0f;
        }
    };
    fetch(0);
    for (int r0 = 0; r0 < rank; r0 += KC) {
        __syncthreads();
#pragma unroll
        for (int it = 0; it < NL; ++it) {
            const int idx = it * 256 + tid;
            Et[idx % KC][idx / KC] = re[it];
            Ut[idx / T][idx % T] = ru[it];
        }
        __syncthreads();
        if (r0 + KC < rank) fetch(r0 + KC);
#pragma unroll
        for (int ks = 0; ks < KC / 4; ++ks) {
            float e[NT], u[NT];
#pragma unroll
            for (int i = 0; i < NT; ++i) e[i] = Et[ks * 4 + q][wr + i * 16 + l16];
#pragma unroll
            for (int j = 0; j < NT; ++j) u[j] = Ut[ks * 4 + q][wc + j * 16 + l16];
#pragma unroll
            for (int i = 0; i < NT; ++i)
#pragma unroll
                for (int j = 0; j < NT; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(e[i], u[j], acc[i][j], 0, 0, 0);
        }
    }
    if (!in) return;
#pragma unroll
    for (int i = 0; i < NT; ++i)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int n = n0 + wr + i * 16 + 4 * q + v;
            if (n >= a.N) continue;
            float* dst = a.wp + (int64_t)n * a.K + c0 + wc + l16;
#pragma unroll
            for (int j = 0; j < NT; ++j) dst[j * 16] = acc[i][j][v];
        }
}

// codes[n, kb] = code of column 2 kb | code of column 2 kb + 1 << 4, fetched from their visiting positions
__global__ __launch_bounds__(256) void gptq_pack_kernel(GptqArgs a)
{
    const int n = blockIdx.x;
    const uint8_t* qr = a.q + (int64_t)n * a.K;
    for (int kb = threadIdx.x; kb < a.K / 2; kb += 256) {
        const uint32_t lo = qr[a.iperm[2 * kb]] & 15u, hi = qr[a.iperm[2 * kb + 1]] & 15u;
        a.codes[(int64_t)n * (a.K / 2) + kb] = (uint8_t)(lo | (hi << 4));
    }
}

inline size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }

}  // namespace

size_t gptq_workspace_bytes(int64_t N, int64_t K)
{
    return align256((size_t)N * K * 4) + align256((size_t)N * K) + align256((size_t)N * kOuter * 4) + align256((size_t)K * 4);
}

// out[t, :] = x[t, :] H_b in fp32, natural column order (the calibration rows a Hessian is accumulated from)
hipError_t launch_gptq_rotate_rows(const void* x, int64_t T, int64_t K, int b, float* out, hipStream_t st)
{
    GptqArgs a{};
    a.w = static_cast<const uint16_t*>(x);
    a.perm = nullptr;
    a.wp = out;
    a.N = (int)T;
    a.K = (int)K;
    a.b = b;
    const double c = 1.0 / sqrt((double)b);
    a.c_hi = (float)c;
    a.c_lo = (float)(c - (double)a.c_hi);
    if (K <= 0 || T <= 0 || K > 24576) return hipErrorInvalidValue;
    const size_t row_lds = (size_t)K * 6;
    if (row_lds > 48 * 1024) {
        const hipError_t le = hipFuncSetAttribute(reinterpret_cast<const void*>(gptq_rotate_gather_kernel),
                                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)row_lds);
        if (le != hipSuccess) return le;
    }
    hipLaunchKernelGGL(gptq_rotate_gather_kernel, dim3((unsigned)T), dim3(256), row_lds, st, a);
    return hipGetLastError();
}

hipError_t launch_gptq_sweep(const void* w, int64_t N, int64_t K, int b, int fmt, const float* U, const int* perm,
                             const void* scales, const float* s_T, const float* table, float factor, void* codes, void* workspace, hipStream_t st)
{
    GptqArgs a{};
    a.w = static_cast<const uint16_t*>(w);
    a.U = U;
    a.perm = perm;
    char* ws = static_cast<char*>(workspace);
    a.wp = reinterpret_cast<float*>(ws);
    ws += align256((size_t)N * K * 4);
    a.q = reinterpret_cast<uint8_t*>(ws);
    ws += align256((size_t)N * K);
    a.err = reinterpret_cast<float*>(ws);
    ws += align256((size_t)N * kOuter * 4);
    a.iperm = reinterpret_cast<int*>(ws);
    a.scales = static_cast<const uint8_t*>(scales);
    a.s_T = s_T;
    a.table = table;
    a.codes = static_cast<uint8_t*>(codes);
    a.N = (int)N;
    a.K = (int)K;
    a.b = b;
    a.G = fmt == 0 ? 32 : 16;
    const double c = 1.0 / sqrt((double)b);
    a.c_hi = (float)c;
    a.c_lo = (float)(c - (double)a.c_hi);
    a.factor = factor;
    if (K % kB != 0 || N <= 0 || K > 24576) return hipErrorInvalidValue;  // (a row is staged in LDS twice, as read and rotated: 6 K bytes)

    const unsigned kblocks = (unsigned)((K + 255) / 256);
    hipLaunchKernelGGL(gptq_iperm_fill_kernel, dim3(kblocks), dim3(256), 0, st, a);
    hipLaunchKernelGGL(gptq_iperm_kernel, dim3(kblocks), dim3(256), 0, st, a);
    const size_t row_lds = (size_t)K * 6;
    if (row_lds > 48 * 1024) {
        const hipError_t le = hipFuncSetAttribute(reinterpret_cast<const void*>(gptq_rotate_gather_kernel),
                                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)row_lds);
        if (le != hipSuccess) return le;
    }
    hipLaunchKernelGGL(gptq_rotate_gather_kernel, dim3((unsigned)N), dim3(256), row_lds, st, a);
    const unsigned row128 = (unsigned)((N + 127) / 128), row16 = (unsigned)((N + 15) / 16);
    auto update = [&](int u0, int e0, int rank, int c_begin, int c_end) {
        const unsigned tiles = (unsigned)((c_end - c_begin + 127) / 128);
        hipLaunchKernelGGL(gptq_update_kernel, dim3(tiles, row128), dim3(256), 0, st, a, u0, e0, rank, c_begin, c_end);
    };
    for (int o = 0; o < (int)K; o += kOuter) {
        const int oe = std::min(o + kOuter, (int)K);
        // the outer block itself: every wave sweeps its 16 rows through the block's columns, pushing each 64-column
        // block's errors onto the rest of the outer block as it goes ...
        if (fmt == 0) hipLaunchKernelGGL(gptq_outer_kernel<0>, dim3(row16), dim3(64), 0, st, a, o, oe);
        else hipLaunchKernelGGL(gptq_outer_kernel<1>, dim3(row16), dim3(64), 0, st, a, o, oe);
        // ... everything behind the outer block sees all of its errors in one pass
        if (oe < (int)K) update(o, 0, oe - o, oe, (int)K);
    }
    hipLaunchKernelGGL(gptq_pack_kernel, dim3((unsigned)N), dim3(256), 0, st, a);
    return hipGetLastError();
}

}  // namespace fp4mr
