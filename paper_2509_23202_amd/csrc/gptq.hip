// MR-GPTQ weight quantizer, the part that runs over the weight matrix (arXiv 2509.23202, Section 4: GPTQ quantizes
// all rows in one fixed column order and, after rounding a column, moves the columns not yet rounded by the
// optimal-brain update; Section 4.1: on rotated weights, with the scales fixed beforehand in the original column
// order and the columns visited in a static activation order).
//
// Given U, the upper-triangular factor of the damped inverse Hessian in visiting order (U^T U = Hinv), column j costs
//     q = Q(w_j / s),   e = (w_j - q s) / U[j,j],   w_k -= e U[j,k]  for every later column k.
// Rows never interact, so the sweep is data-parallel over the N rows and strictly sequential along K.  It is blocked
// 64 columns at a time: four lanes share a row and keep the block's 64 working weights in registers while the 64 x 64
// triangle of U is read from LDS (block kernel); the block's 64 errors per row then update the later columns of the
// same 512-column outer block in a rank-64 product, and a finished outer block updates everything behind it in one
// rank-512 product (update kernel).  Working weights live in visiting order in an fp32 scratch matrix, codes in a
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

// wp[n, j] = (W H_b)[n, perm[j]]: the rotated weight of the column visited j-th.  Sums of up to 128 bf16 values in fp32
// (exact unless their exponents spread over more than 16 bits), then one multiplication by 1/sqrt(b) carried in two
// floats.
__global__ void gptq_rotate_gather_kernel(GptqArgs a)
{
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    const int n = blockIdx.y;
    if (j >= a.K) return;
    const int col = visit_col(a, j);
    const int j0 = col & ~(a.b - 1), c = col - j0;
    const uint16_t* x = a.w + (int64_t)n * a.K + j0;
    float sum = 0.0f;
    for (int r = 0; r < a.b; ++r) {
        const float v = __uint_as_float((uint32_t)x[r] << 16);
        sum += (__popc((unsigned)(r & c)) & 1) ? -v : v;
    }
    a.wp[(int64_t)n * a.K + j] = (a.b == 1) ? sum : __fmaf_rn(sum, a.c_hi, sum * a.c_lo);
}

// nearest E2M1 code (ties to the even code, saturating), sign in bit 3
__device__ __forceinline__ uint32_t e2m1_code(float t)
{
    const float m = fabsf(t);
    uint32_t c = 0;
    c += m > 0.25f;
    c += m >= 0.75f;
    c += m > 1.25f;
    c += m >= 1.75f;
    c += m > 2.5f;
    c += m >= 3.5f;
    c += m > 5.0f;
    return c | ((__float_as_uint(t) >> 31) << 3);
}

__device__ __forceinline__ float e2m1_value(uint32_t code)
{
    const uint32_t m = code & 7u, e = m >> 1, man = m & 1u;
    const float mag = (e == 0) ? 0.5f * (float)man : __uint_as_float((126u + e) << 23) * (1.0f + 0.5f * (float)man);
    return (code & 8u) ? -mag : mag;
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

template <int FMT, int P>
__device__ __forceinline__ void sweep_part(float (&w)[16], const float* Us, const float* Ss, int row, int part, bool live,
                                           float* erow, uint8_t* qrow)
{
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        constexpr int base = P * 16;
        const int j = base + i;
        const float s = Ss[j * 16 + row];
        const float wj = w[i];  // meaningful in the lanes with part == P
        const uint32_t code = (s > 0.0f) ? e2m1_code(wj / s) : 0u;
        const float dq = e2m1_value(code) * s;
        const float e_own = (wj - dq) / Us[j * kB + j];
        if (live && part == P) {
            erow[j] = e_own;
            qrow[j] = (uint8_t)code;
        }
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

template <int FMT>
__global__ __launch_bounds__(64) void gptq_block_kernel(GptqArgs a, int b0, int e0)
{
    __shared__ __attribute__((aligned(16))) float Us[kB * kB];
    __shared__ float Ss[kB * 16];  // [column][row of the wave]
    __shared__ int cols[kB];
    const int lane = threadIdx.x;
    for (int i = lane; i < kB * kB; i += 64) {
        const int r = i / kB, c = i % kB;
        Us[i] = (c >= r) ? a.U[(int64_t)(b0 + r) * a.K + b0 + c] : 0.0f;
    }
    cols[lane] = visit_col(a, b0 + lane);
    __syncthreads();

    const int row = lane >> 2, part = lane & 3;
    const int n_raw = blockIdx.x * 16 + row;
    const bool live = n_raw < a.N;
    const int n = live ? n_raw : a.N - 1;  // idle lanes shadow the last row and store nothing
    const float s_T = (FMT == 1) ? *a.s_T : 1.0f;
    const uint8_t* srow = a.scales + (int64_t)n * (a.K / a.G);
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
    for (int i = 0; i < 16; ++i) {
        const int j = part * 16 + i;
        Ss[j * 16 + row] = decode_scale<FMT>(srow[cols[j] / a.G], s_T, a.factor);
    }
    __syncthreads();  // the scale of a column is read by every lane of its row's quad
    float* const erow = a.err + (int64_t)n * kOuter + e0;
    uint8_t* const qrow = a.q + (int64_t)n * a.K + b0;
    sweep_part<FMT, 0>(w, Us, Ss, row, part, live, erow, qrow);
    sweep_part<FMT, 1>(w, Us, Ss, row, part, live, erow, qrow);
    sweep_part<FMT, 2>(w, Us, Ss, row, part, live, erow, qrow);
    sweep_part<FMT, 3>(w, Us, Ss, row, part, live, erow, qrow);
}

// wp[n, c] -= sum_{j < rank} err[n, e0 + j] * U[u0 + j, c] for the columns c_begin <= c < c_end (visiting order), the
// terms applied one j at a time in ascending order like the column-by-column definition.  128 x 128 output tile per
// workgroup, 8 x 8 per thread, the errors and the rows of U staged through LDS 32 terms at a time.
__global__ __launch_bounds__(256) void gptq_update_kernel(GptqArgs a, int u0, int e0, int rank, int c_begin, int c_end)
{
    constexpr int T = 128, KC = 32;
    __shared__ __attribute__((aligned(16))) float Et[KC][T];  // [term][row]
    __shared__ __attribute__((aligned(16))) float Ut[KC][T];  // [term][column]
    const int c0 = c_begin + blockIdx.x * T;
    const int n0 = blockIdx.y * T;
    const int tid = threadIdx.x;
    const int ty = tid / 16, tx = tid % 16;
    float acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int n = min(n0 + ty * 8 + i, a.N - 1);
        const float* src = a.wp + (int64_t)n * a.K + c0 + tx * 8;
        const bool in = c0 + tx * 8 < c_end;  // c_end and the tile start are multiples of 64: 8 columns are in or out together
        const float4 lo = in ? *reinterpret_cast<const float4*>(src) : make_float4(0.f, 0.f, 0.f, 0.f);
        const float4 hi = in ? *reinterpret_cast<const float4*>(src + 4) : make_float4(0.f, 0.f, 0.f, 0.f);
        acc[i][0] = lo.x; acc[i][1] = lo.y; acc[i][2] = lo.z; acc[i][3] = lo.w;
        acc[i][4] = hi.x; acc[i][5] = hi.y; acc[i][6] = hi.z; acc[i][7] = hi.w;
    }
    for (int r0 = 0; r0 < rank; r0 += KC) {
        __syncthreads();
        for (int idx = tid; idx < KC * T; idx += 256) {
            const int x = idx % T, t = idx / T;
            const int n = min(n0 + x, a.N - 1);
            Et[t][x] = a.err[(int64_t)n * kOuter + e0 + r0 + t];
            Ut[t][x] = (c0 + x < c_end) ? a.U[(int64_t)(u0 + r0 + t) * a.K + c0 + x] : 0.0f;
        }
        __syncthreads();
#pragma unroll 4
        for (int t = 0; t < KC; ++t) {
            const float4 e0v = *reinterpret_cast<const float4*>(&Et[t][ty * 8]);
            const float4 e1v = *reinterpret_cast<const float4*>(&Et[t][ty * 8 + 4]);
            const float4 u0v = *reinterpret_cast<const float4*>(&Ut[t][tx * 8]);
            const float4 u1v = *reinterpret_cast<const float4*>(&Ut[t][tx * 8 + 4]);
            const float e[8] = {e0v.x, e0v.y, e0v.z, e0v.w, e1v.x, e1v.y, e1v.z, e1v.w};
            const float u[8] = {u0v.x, u0v.y, u0v.z, u0v.w, u1v.x, u1v.y, u1v.z, u1v.w};
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int k = 0; k < 8; ++k) acc[i][k] = __fmaf_rn(-e[i], u[k], acc[i][k]);
        }
    }
    if (c0 + tx * 8 >= c_end) return;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int n = n0 + ty * 8 + i;
        if (n >= a.N) continue;
        float* dst = a.wp + (int64_t)n * a.K + c0 + tx * 8;
        *reinterpret_cast<float4*>(dst) = make_float4(acc[i][0], acc[i][1], acc[i][2], acc[i][3]);
        *reinterpret_cast<float4*>(dst + 4) = make_float4(acc[i][4], acc[i][5], acc[i][6], acc[i][7]);
    }
}

// The same update for the 64 errors of one block onto the few hundred remaining columns of its outer block: 64 x 64
// tiles, 4 x 4 per thread -- many small workgroups, since there is little work and it sits on the critical path
// between two sequential block kernels.
__global__ __launch_bounds__(256) void gptq_update_inner_kernel(GptqArgs a, int u0, int e0, int c_begin, int c_end)
{
    __shared__ float Es[kB][kB + 1];  // [row][term]
    __shared__ float Ut[kB][kB];      // [term][column]
    const int c0 = c_begin + blockIdx.x * kB;
    const int n0 = blockIdx.y * kB;
    const int tid = threadIdx.x;
    for (int i = tid; i < kB * kB; i += 256) {
        const int r = i / kB, c = i % kB;
        const int n = min(n0 + r, a.N - 1);
        Es[r][c] = a.err[(int64_t)n * kOuter + e0 + c];
        Ut[r][c] = (c0 + c < c_end) ? a.U[(int64_t)(u0 + r) * a.K + c0 + c] : 0.0f;
    }
    __syncthreads();
    const int ty = tid / 16, tx = tid % 16;
    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int n = min(n0 + ty * 4 + i, a.N - 1);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int c = c0 + tx * 4 + k;
            acc[i][k] = (c < c_end) ? a.wp[(int64_t)n * a.K + c] : 0.0f;
        }
    }
    for (int j = 0; j < kB; ++j) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float e = Es[ty * 4 + i][j];
#pragma unroll
            for (int k = 0; k < 4; ++k) acc[i][k] = __fmaf_rn(-e, Ut[j][tx * 4 + k], acc[i][k]);
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int n = n0 + ty * 4 + i;
        if (n >= a.N) continue;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int c = c0 + tx * 4 + k;
            if (c < c_end) a.wp[(int64_t)n * a.K + c] = acc[i][k];
        }
    }
}

// codes[n, kb] = code of column 2 kb | code of column 2 kb + 1 << 4, fetched from their visiting positions
__global__ void gptq_pack_kernel(GptqArgs a)
{
    const int kb = blockIdx.x * blockDim.x + threadIdx.x;
    const int n = blockIdx.y;
    if (kb >= a.K / 2) return;
    const uint8_t* qr = a.q + (int64_t)n * a.K;
    const uint32_t lo = qr[a.iperm[2 * kb]] & 15u, hi = qr[a.iperm[2 * kb + 1]] & 15u;
    a.codes[(int64_t)n * (a.K / 2) + kb] = (uint8_t)(lo | (hi << 4));
}

inline size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }

}  // namespace

size_t gptq_workspace_bytes(int64_t N, int64_t K)
{
    return align256((size_t)N * K * 4) + align256((size_t)N * K) + align256((size_t)N * kOuter * 4) + align256((size_t)K * 4);
}

hipError_t launch_gptq_sweep(const void* w, int64_t N, int64_t K, int b, int fmt, const float* U, const int* perm,
                             const void* scales, const float* s_T, float factor, void* codes, void* workspace, hipStream_t st)
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
    a.codes = static_cast<uint8_t*>(codes);
    a.N = (int)N;
    a.K = (int)K;
    a.b = b;
    a.G = fmt == 0 ? 32 : 16;
    const double c = 1.0 / sqrt((double)b);
    a.c_hi = (float)c;
    a.c_lo = (float)(c - (double)a.c_hi);
    a.factor = factor;
    if (K % kB != 0 || N <= 0) return hipErrorInvalidValue;

    const unsigned kblocks = (unsigned)((K + 255) / 256);
    hipLaunchKernelGGL(gptq_iperm_fill_kernel, dim3(kblocks), dim3(256), 0, st, a);
    hipLaunchKernelGGL(gptq_iperm_kernel, dim3(kblocks), dim3(256), 0, st, a);
    hipLaunchKernelGGL(gptq_rotate_gather_kernel, dim3(kblocks, (unsigned)N), dim3(256), 0, st, a);
    const unsigned row128 = (unsigned)((N + 127) / 128), row16 = (unsigned)((N + 15) / 16);
    auto update = [&](int u0, int e0, int rank, int c_begin, int c_end) {
        const unsigned tiles = (unsigned)((c_end - c_begin + 127) / 128);
        hipLaunchKernelGGL(gptq_update_kernel, dim3(tiles, row128), dim3(256), 0, st, a, u0, e0, rank, c_begin, c_end);
    };
    for (int o = 0; o < (int)K; o += kOuter) {
        const int oe = std::min(o + kOuter, (int)K);
        for (int b0 = o; b0 < oe; b0 += kB) {
            if (fmt == 0) hipLaunchKernelGGL(gptq_block_kernel<0>, dim3(row16), dim3(64), 0, st, a, b0, b0 - o);
            else hipLaunchKernelGGL(gptq_block_kernel<1>, dim3(row16), dim3(64), 0, st, a, b0, b0 - o);
            // the rest of the outer block sees this block's errors at once ...
            if (b0 + kB < oe)
                hipLaunchKernelGGL(gptq_update_inner_kernel, dim3((unsigned)((oe - b0 - kB) / kB), (unsigned)((N + 63) / 64)), dim3(256), 0,
                                   st, a, b0, b0 - o, b0 + kB, oe);
        }
        // ... everything behind the outer block sees all of its errors in one pass
        if (oe < (int)K) update(o, 0, oe - o, oe, (int)K);
    }
    hipLaunchKernelGGL(gptq_pack_kernel, dim3((unsigned)((K / 2 + 255) / 256), (unsigned)N), dim3(256), 0, st, a);
    return hipGetLastError();
}

}  // namespace fp4mr
