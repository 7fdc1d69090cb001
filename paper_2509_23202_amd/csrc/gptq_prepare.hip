// From a layer's Hessian to what the MR-GPTQ sweep consumes (arXiv 2509.23202, Section 4 "Standard GPTQ" and Section
// 4.1 "Ingredient 2"; Section 5 "Algorithms": dampening 1e-2): the static activation order (columns by descending
// Hessian diagonal), the dampened, re-ordered Hessian A = H[perm][:,perm] + lambda mean(diag H) I, and the upper
// triangular U with U^T U = A^-1 whose row j drives the update after column j.
//
// U is obtained without forming A^-1: factor A = R R^T with R UPPER triangular; then A^-1 = R^-T R^-1 and U = R^-1.
// With J the index reversal, J A J = L L^T is an ordinary (lower) Cholesky factorization and R = J L J, so the work is
//   1. gather  At[i][j] = A[K-1-i][K-1-j]                       (one pass, applies order and dampening)
//   2. blocked Cholesky of At in place, 64 columns at a time:   diagonal block factored (and inverted) by one wave,
//      panel  L21 = A21 L11^-T  as a product with that inverse, trailing update  A22 -= L21 L21^T
//   3. V = L^-1 by recursive doubling over the diagonal blocks: [L11 0; L21 L22]^-1 = [V11 0; -V22 L21 V11, V22]
//   4. U[i][j] = V[K-1-i][K-1-j]
// All in fp32; the products run on one tiled kernel on the fp32 MFMA.
#include "device_util.hpp"
#include "internal.hpp"

#include <algorithm>
#include <cmath>

namespace fp4mr {
namespace {

constexpr int NB = 64;  // block size of the factorization

// ---------------------------------------------------------------- ordering and gather

// rank of column i in the order "descending diagonal, ties by ascending index"; perm[rank] = i.  (A diagonal with
// NaNs does not rank into a permutation; perm is pre-filled with the identity so that every entry is at least valid.)
__global__ __launch_bounds__(256) void order_kernel(const float* diag, int K, int use_order, int* perm)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= K) return;
    const float di = diag[i];
    int rank = i;
    if (use_order) {
        rank = 0;
        for (int j = 0; j < K; ++j) {
            const float dj = diag[j];
            rank += (dj > di) || (dj == di && j < i);
        }
    }
    perm[min(rank, K - 1)] = i;
}

__global__ __launch_bounds__(256) void identity_kernel(int K, int* perm)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < K) perm[i] = i;
}

// the diagonal as a contiguous array, and its mean (summed in double, one workgroup)
__global__ __launch_bounds__(256) void mean_diag_kernel(const float* H, int K, float* diag, float* out)
{
    __shared__ double part[256];
    double s = 0.0;
    for (int i = threadIdx.x; i < K; i += 256) {
        const float d = H[(int64_t)i * K + i];
        diag[i] = d;
        s += (double)d;
    }
    part[threadIdx.x] = s;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) *out = (float)(part[0] / (double)K);
}

// At[i][j] = H[perm[K-1-i]][perm[K-1-j]] + (i == j) damp * mean;  V = 0
__global__ __launch_bounds__(256) void gather_kernel(const float* H, const int* perm, const float* mean, float damp, int K,
                                                     float* At, float* V)
{
    const int j = blockIdx.x * 256 + threadIdx.x;
    const int i = blockIdx.y;
    if (j >= K) return;
    const int pi = min(max(perm[K - 1 - i], 0), K - 1), pj = min(max(perm[K - 1 - j], 0), K - 1);
    float v = H[(int64_t)pi * K + pj];
    if (i == j) v += damp * (*mean);
    At[(int64_t)i * K + j] = v;
    V[(int64_t)i * K + j] = 0.0f;
}

// ---------------------------------------------------------------- diagonal block: Cholesky and inverse, one wave

// A[k0:k0+nb, k0:k0+nb] (nb <= 64) -> L11 in place (lower), its inverse into V's diagonal block (lower) and into
// Linv (dense 64 x 64 scratch, row-major, zero above the diagonal and beyond nb).  One wave; lane r keeps row r of the
// block in registers, and what a step needs from another lane's row comes through v_readlane with a constant lane
// index (both loops are fully unrolled), so the factorization itself touches no memory.  Rows beyond nb are rows of
// the identity.  Entries right of the diagonal in a lane's registers are scratch: updated, never used.
__device__ __forceinline__ float lane_value(float v, int lane)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}

__global__ __launch_bounds__(64) void diag_block_kernel(float* A, float* V, float* Linv, int K, int k0, int nb)
{
    __shared__ float t[NB][NB + 1];
    __shared__ float xs[NB][NB + 1];
    const int r = threadIdx.x;
    // memory is walked a row per step with the lane as the column (coalesced); LDS transposes to a row per lane
#pragma unroll 16
    for (int rr = 0; rr < NB; ++rr)
        t[rr][r] = (rr < nb && r < nb && r <= rr) ? A[(int64_t)(k0 + rr) * K + k0 + r] : (rr == r ? 1.0f : 0.0f);
    __syncthreads();
    float row[NB];
#pragma unroll
    for (int c = 0; c < NB; ++c) row[c] = t[r][c];
    // right-looking Cholesky: after step j, row[j] holds L[r][j] for the lanes r >= j
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        const float d = sqrtf(lane_value(row[j], j));
        row[j] = (r == j) ? d : row[j] / d;
#pragma unroll
        for (int c = j + 1; c < NB; ++c) row[c] = fmaf(-row[j], lane_value(row[j], c), row[c]);
        __builtin_amdgcn_sched_barrier(0);  // (keeps the scheduler's regions, and the compile time, small)
    }
    // L goes to LDS (row per lane -> row-major) for the coalesced store and for the inversion
    __syncthreads();
#pragma unroll
    for (int c = 0; c < NB; ++c) t[r][c] = row[c];
    __syncthreads();
#pragma unroll 16
    for (int rr = 0; rr < NB; ++rr)
        if (rr < nb && r < nb && r <= rr) A[(int64_t)(k0 + rr) * K + k0 + r] = t[rr][r];
    // inverse, column by column: lane c solves L x = e_c by forward substitution, its x in LDS column c.  Eight rows at a
    // time: their sums over the rows already solved are eight independent chains fed by one read of x and two 16-byte
    // broadcast reads of a transposed copy of L; then the 8 x 8 triangle in registers.  The loops over row groups and
    // solved rows stay rolled: unrolled like the factorization they cost minutes of compile time.
    __shared__ __attribute__((aligned(16))) float tT[NB][NB + 4];  // tT[u][i] = L[i][u]
#pragma unroll
    for (int c = 0; c < NB; ++c) tT[c][r] = row[c];
    __syncthreads();
    {
        const int c = r;
        for (int i0 = 0; i0 < NB; i0 += 8) {
            float sum[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) sum[k] = (i0 + k == c) ? 1.0f : 0.0f;
#pragma unroll 4
            for (int u = 0; u < i0; ++u) {
                const float xv = xs[u][c];
                const float4 la = *reinterpret_cast<const float4*>(&tT[u][i0]);
                const float4 lb = *reinterpret_cast<const float4*>(&tT[u][i0 + 4]);
                sum[0] = fmaf(-la.x, xv, sum[0]);
                sum[1] = fmaf(-la.y, xv, sum[1]);
                sum[2] = fmaf(-la.z, xv, sum[2]);
                sum[3] = fmaf(-la.w, xv, sum[3]);
                sum[4] = fmaf(-lb.x, xv, sum[4]);
                sum[5] = fmaf(-lb.y, xv, sum[5]);
                sum[6] = fmaf(-lb.z, xv, sum[6]);
                sum[7] = fmaf(-lb.w, xv, sum[7]);
            }
            float x[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
#pragma unroll
                for (int k2 = 0; k2 < k; ++k2) sum[k] = fmaf(-tT[i0 + k2][i0 + k], x[k2], sum[k]);
                x[k] = (i0 + k >= c) ? sum[k] / tT[i0 + k][i0 + k] : 0.0f;
                xs[i0 + k][c] = x[k];
            }
        }
    }
    __syncthreads();
#pragma unroll 16
    for (int rr = 0; rr < NB; ++rr) {
        const float v = (rr < nb && r < nb && r <= rr) ? xs[rr][r] : 0.0f;
        if (rr < nb && r < nb) V[(int64_t)(k0 + rr) * K + k0 + r] = v;
        Linv[rr * NB + r] = v;
    }
}

// ---------------------------------------------------------------- plain fp32 product
// C[m x n] = beta C + alpha op(A) op(B),  op(A) = A[m x k] or A^T with A stored [k x m], op(B) = B[k x n] or B^T with
// B stored [n x k]; row-major with leading dimensions.  A dense fp32 contraction, so it runs on the fp32 MFMA
// (v_mfma_f32_16x16x4_f32: true fp32 products and sums): T x T tile per workgroup (T = 64, or 128 for big products),
// one quarter of it per wave as (T/32)^2 MFMA tiles, k in chunks of 16 (32 for the wide tile) through LDS with the next chunk prefetched into registers; results are written after all
// inputs of the tile have been read (a tile may overwrite its own A rows when n fits one tile).
// Batches along blockIdx.z: pointers advance by the given strides.  ragged > 0 (the pairs of the triangular
// inversion): batch z covers rows [z 2s + s, z 2s + 2s) of a matrix with `total` rows, s = ragged; its row count is
// clipped to what exists, and so is k when k_is_rows is set.  lower_only skips tiles strictly above the diagonal.
struct GemmF32 {
    float* C;
    const float* A;
    const float* B;
    int64_t ldc, lda, ldb;
    int64_t sC, sA, sB;
    int m, n, k;
    float alpha, beta;
    int transB, ragged, total, k_is_rows, lower_only;
    int transA;  // A stored [k x m] (the product is A^T op(B))
};

template <int T>
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmF32 g)
{
    constexpr int KC = (T == 128) ? 32 : 16;  // k per chunk
    // row pitch = 20 mod 64 banks: the fills along k (16 k-rows x 4 rows per wave store) hit 64 different banks, and the
    // four k-rows of an MFMA operand read (16 consecutive floats each) overlap in 12 banks only
    constexpr int LD = T + 20;
    constexpr int WT = T / 2, NT = WT / 16;  // wave tile and its MFMA tiles per side
    __shared__ float As[KC][LD];  // [k][row]
    __shared__ float Bs[KC][LD];  // [k][col]
    const int z = blockIdx.z;
    int m = g.m, k = g.k;
    if (g.ragged > 0) {
        const int rows = min(g.ragged, g.total - (z * 2 * g.ragged + g.ragged));
        if (rows <= 0) return;
        m = rows;
        if (g.k_is_rows) k = rows;
    }
    const int r0 = blockIdx.y * T, c0 = blockIdx.x * T;
    if (r0 >= m || c0 >= g.n) return;
    if (g.lower_only && c0 > r0 + T - 1) return;
    const float* A = g.A + (int64_t)z * g.sA;
    const float* B = g.B + (int64_t)z * g.sB;
    float* C = g.C + (int64_t)z * g.sC;
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, l16 = lane & 15, q = lane >> 4;
    const int wr = (wave >> 1) * WT, wc = (wave & 1) * WT;  // this wave's corner inside the tile
    v4f acc[NT][NT];
#pragma unroll
    for (int i = 0; i < NT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j) acc[i][j] = v4f{0.f, 0.f, 0.f, 0.f};
    // the next chunk's elements travel from global memory into registers while the MFMAs of the current chunk run
    constexpr int NL = KC * T / 256;
    float ra[NL], rb[NL];
    auto fetch = [&](int kk) {
#pragma unroll
        for (int it = 0; it < NL; ++it) {
            const int idx = it * 256 + tid;
            if (g.transA) {  // A stored [k x m]: consecutive threads along the row index (contiguous in memory)
                const int rr = idx % T, kx = idx / T;
                const int row = r0 + rr, kc = kk + kx;
                ra[it] = (row < m && kc < k) ? A[(int64_t)kc * g.lda + row] : 0.0f;
            } else {         // A stored [m x k]: consecutive threads along k
                const int kx = idx % KC, rr = idx / KC;
                const int row = r0 + rr, kc = kk + kx;
                ra[it] = (row < m && kc < k) ? A[(int64_t)row * g.lda + kc] : 0.0f;
            }
            if (g.transB) {  // B stored [n x k]
                const int kx = idx % KC, cc = idx / KC;
                const int col = c0 + cc, kc = kk + kx;
                rb[it] = (col < g.n && kc < k) ? B[(int64_t)col * g.ldb + kc] : 0.0f;
            } else {         // B stored [k x n]
                const int cc = idx % T, kx = idx / T;
                const int col = c0 + cc, kc = kk + kx;
                rb[it] = (col < g.n && kc < k) ? B[(int64_t)kc * g.ldb + col] : 0.0f;
            }
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int it = 0; it < NL; ++it) {
            const int idx = it * 256 + tid;
            if (g.transA) As[idx / T][idx % T] = ra[it]; else As[idx % KC][idx / KC] = ra[it];
            if (g.transB) Bs[idx % KC][idx / KC] = rb[it]; else Bs[idx / T][idx % T] = rb[it];
        }
    };
    fetch(0);
    for (int kk = 0; kk < k; kk += KC) {
        __syncthreads();  // the previous chunk's MFMA operands have been read
        stash();
        __syncthreads();
        if (kk + KC < k) fetch(kk + KC);
        // one MFMA = 16 x 16 outputs over 4 k: lane (l16, q) supplies op(A)[row l16][k q] and op(B)[k q][col l16]
#pragma unroll
        for (int ks = 0; ks < KC / 4; ++ks) {
            float a[NT], b[NT];
#pragma unroll
            for (int i = 0; i < NT; ++i) a[i] = As[ks * 4 + q][wr + i * 16 + l16];
#pragma unroll
            for (int j = 0; j < NT; ++j) b[j] = Bs[ks * 4 + q][wc + j * 16 + l16];
#pragma unroll
            for (int i = 0; i < NT; ++i)
#pragma unroll
                for (int j = 0; j < NT; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[i], b[j], acc[i][j], 0, 0, 0);
        }
    }
    __syncthreads();  // every thread of the tile has read its inputs
    // a lane holds rows 4q .. 4q+3 of column l16 of every MFMA tile
#pragma unroll
    for (int i = 0; i < NT; ++i) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int row = r0 + wr + i * 16 + 4 * q + v;
            if (row >= m) continue;
#pragma unroll
            for (int j = 0; j < NT; ++j) {
                const int col = c0 + wc + j * 16 + l16;
                if (col >= g.n) continue;
                float* p = C + (int64_t)row * g.ldc + col;
                *p = (g.beta == 0.0f) ? g.alpha * acc[i][j][v] : g.beta * (*p) + g.alpha * acc[i][j][v];
            }
        }
    }
}

hipError_t gemm_f32(const GemmF32& g, int batches, hipStream_t st)
{
    if (g.m <= 0 || g.n <= 0 || batches <= 0) return hipSuccess;
    // the wide tile for products with enough tiles of it to fill the chip and enough k to pay for its larger fills (never
    // the in-place panel, whose n is one narrow tile, nor the rank-64 trailing updates, which want many small tiles)
    if (g.m >= 1024 && g.n >= 1024 && g.k >= 256) {
        const dim3 grid((unsigned)((g.n + 127) / 128), (unsigned)((g.m + 127) / 128), (unsigned)batches);
        hipLaunchKernelGGL(gemm_f32_kernel<128>, grid, dim3(256), 0, st, g);
    } else {
        const dim3 grid((unsigned)((g.n + 63) / 64), (unsigned)((g.m + 63) / 64), (unsigned)batches);
        hipLaunchKernelGGL(gemm_f32_kernel<64>, grid, dim3(256), 0, st, g);
    }
    return hipGetLastError();
}

// U[i][j] = V[K-1-i][K-1-j] on and above the diagonal, 0 below
__global__ __launch_bounds__(256) void reverse_kernel(const float* V, int K, float* U)
{
    const int j = blockIdx.x * 256 + threadIdx.x;
    const int i = blockIdx.y;
    if (j >= K) return;
    U[(int64_t)i * K + j] = (j >= i) ? V[(int64_t)(K - 1 - i) * K + (K - 1 - j)] : 0.0f;
}

inline size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }

}  // namespace

size_t gptq_prepare_workspace_bytes(int64_t K)
{
    // At, V: K x K each; T: K x K / 2; the diagonal block's inverse; the diagonal; the mean
    return 2 * align256((size_t)K * K * 4) + align256((size_t)K * K * 2) + align256((size_t)NB * NB * 4) + align256((size_t)K * 4) + 256;
}

// H = (accumulate ? H : 0) + Xr^T Xr for rotated calibration rows Xr [T, K] (fp32, row-major)
hipError_t launch_gptq_hessian_product(const float* Xr, int64_t T, int64_t K, float* H, bool accumulate, hipStream_t st)
{
    GemmF32 g{};
    g.C = H;
    g.A = Xr;
    g.B = Xr;
    g.ldc = g.lda = g.ldb = K;
    g.m = (int)K;
    g.n = (int)K;
    g.k = (int)T;
    g.alpha = 1.0f;
    g.beta = accumulate ? 1.0f : 0.0f;
    g.transA = 1;
    return gemm_f32(g, 1, st);
}

hipError_t launch_gptq_prepare(const float* H, int64_t K64, float damp, bool use_order, int* perm, float* U, void* workspace,
                               hipStream_t st)
{
    const int K = (int)K64;
    if (K <= 0 || K > 65535) return hipErrorInvalidValue;  // (rows ride on grid.y)
    char* ws = static_cast<char*>(workspace);
    float* At = reinterpret_cast<float*>(ws);
    ws += align256((size_t)K * K * 4);
    float* V = reinterpret_cast<float*>(ws);
    ws += align256((size_t)K * K * 4);
    float* T = reinterpret_cast<float*>(ws);
    ws += align256((size_t)K * K * 2);
    float* Linv = reinterpret_cast<float*>(ws);
    ws += align256((size_t)NB * NB * 4);
    float* diag = reinterpret_cast<float*>(ws);
    ws += align256((size_t)K * 4);
    float* mean = reinterpret_cast<float*>(ws);

    const unsigned kb = (unsigned)((K + 255) / 256);
    hipLaunchKernelGGL(mean_diag_kernel, dim3(1), dim3(256), 0, st, H, K, diag, mean);
    hipLaunchKernelGGL(identity_kernel, dim3(kb), dim3(256), 0, st, K, perm);
    hipLaunchKernelGGL(order_kernel, dim3(kb), dim3(256), 0, st, (const float*)diag, K, use_order ? 1 : 0, perm);
    hipLaunchKernelGGL(gather_kernel, dim3(kb, (unsigned)K), dim3(256), 0, st, H, (const int*)perm, (const float*)mean, damp, K, At, V);

    hipError_t e;
    // 2. blocked Cholesky
    for (int k0 = 0; k0 < K; k0 += NB) {
        const int nb = std::min(NB, K - k0);
        hipLaunchKernelGGL(diag_block_kernel, dim3(1), dim3(64), 0, st, At, V, Linv, K, k0, nb);
        const int rest = K - k0 - nb;
        if (rest <= 0) break;
        GemmF32 p{};  // panel: L21 = A21 Linv^T  (in place; one tile wide, so a tile reads all it overwrites first)
        p.C = At + (int64_t)(k0 + nb) * K + k0;
        p.A = p.C;
        p.B = Linv;
        p.ldc = p.lda = K;
        p.ldb = NB;
        p.m = rest;
        p.n = nb;
        p.k = nb;
        p.alpha = 1.0f;
        p.beta = 0.0f;
        p.transB = 1;
        if ((e = gemm_f32(p, 1, st)) != hipSuccess) return e;
        GemmF32 u{};  // trailing update: A22 -= L21 L21^T (lower tiles)
        u.C = At + (int64_t)(k0 + nb) * K + (k0 + nb);
        u.A = At + (int64_t)(k0 + nb) * K + k0;
        u.B = u.A;
        u.ldc = u.lda = u.ldb = K;
        u.m = rest;
        u.n = rest;
        u.k = nb;
        u.alpha = -1.0f;
        u.beta = 1.0f;
        u.transB = 1;
        u.lower_only = 1;
        if ((e = gemm_f32(u, 1, st)) != hipSuccess) return e;
    }
    // 3. V = L^-1: the diagonal blocks are in place; double the inverted block size until it spans the matrix
    for (int s = NB; s < K; s *= 2) {
        const int pairs = (K + 2 * s - 1) / (2 * s);
        GemmF32 t{};  // T_z = L21 V11
        t.C = T;
        t.A = At + (int64_t)s * K;
        t.B = V;
        t.ldc = s;
        t.lda = t.ldb = K;
        t.sC = (int64_t)s * s;
        t.sA = t.sB = (int64_t)2 * s * K + 2 * s;
        t.m = s;
        t.n = s;
        t.k = s;
        t.alpha = 1.0f;
        t.beta = 0.0f;
        t.ragged = s;
        t.total = K;
        if ((e = gemm_f32(t, pairs, st)) != hipSuccess) return e;
        GemmF32 v{};  // V21_z = -V22 T_z
        v.C = V + (int64_t)s * K;
        v.A = V + (int64_t)s * K + s;
        v.B = T;
        v.ldc = v.lda = K;
        v.ldb = s;
        v.sC = v.sA = (int64_t)2 * s * K + 2 * s;
        v.sB = (int64_t)s * s;
        v.m = s;
        v.n = s;
        v.k = s;
        v.alpha = -1.0f;
        v.beta = 0.0f;
        v.ragged = s;
        v.total = K;
        v.k_is_rows = 1;
        if ((e = gemm_f32(v, pairs, st)) != hipSuccess) return e;
    }
    hipLaunchKernelGGL(reverse_kernel, dim3(kb, (unsigned)K), dim3(256), 0, st, (const float*)V, K, U);
    return hipGetLastError();
}

}  // namespace fp4mr
