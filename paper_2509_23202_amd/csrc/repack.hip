// Canonical (row-major) -> GEMM layout copy of one quantized operand.  Only used when fp4_gemm is handed an
// operand in canonical layout (parity tests, interop); the quantize kernels write GEMM layout directly.
#include "device_util.hpp"
#include "internal.hpp"
#include "layout.hpp"

namespace fp4mr {
namespace {

__global__ void repack_codes_kernel(const uint8_t* __restrict__ src, uint8_t* __restrict__ dst, int64_t rows, int64_t K, int64_t n_chunks)
{
    const int64_t KC = K >> 7;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < n_chunks; idx += (int64_t)gridDim.x * blockDim.x) {
        const int64_t f = idx >> 6;
        const int l = (int)(idx & 63);
        const int64_t rb = f / KC, kc = f - rb * KC;
        const int64_t row = rb * 16 + (l & 15);
        uint4 v = make_uint4(0, 0, 0, 0);
        if (row < rows) v = *reinterpret_cast<const uint4*>(src + row * (K >> 1) + kc * 64 + (l >> 4) * 16);
        *reinterpret_cast<uint4*>(dst + idx * 16) = v;
    }
}

// fmt 0: MXFP4 (dword per lane per 4 fragments); fmt 1: NVFP4 (2 bytes per lane per fragment)
__global__ void repack_scales_kernel(const uint8_t* __restrict__ src, uint8_t* __restrict__ dst, int64_t rows, int64_t K, int fmt, int64_t n_bytes)
{
    const int64_t KC = K >> 7, KS = (K + 511) >> 9;
    for (int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; o < n_bytes; o += (int64_t)gridDim.x * blockDim.x) {
        uint8_t v;
        if (fmt == 0) {
            const int64_t blk = o >> 8;
            const int w = (int)(o & 255);
            const int64_t rb = blk / KS, ss = blk - rb * KS;
            const int lane = w >> 2, kcq = w & 3;
            const int64_t row = rb * 16 + (lane & 15);
            const int64_t kg = ss * 16 + kcq * 4 + (lane >> 4);
            v = (row < rows && kg < (K >> 5)) ? src[row * (K >> 5) + kg] : (uint8_t)127;
        } else {
            const int64_t blk = o >> 7;
            const int w = (int)(o & 127);
            const int64_t rb = blk / KC, kc = blk - rb * KC;
            const int lane = w >> 1, h = w & 1;
            const int64_t row = rb * 16 + (lane & 15);
            const int64_t g16 = kc * 8 + (lane >> 4) * 2 + h;
            v = (row < rows) ? src[row * (K >> 4) + g16] : (uint8_t)0;
        }
        dst[o] = v;
    }
}

}  // namespace

hipError_t launch_repack_to_gemm(const void* codes, const void* scales, int64_t rows, int64_t K, int fmt,
                                 void* codes_gemm, void* scales_gemm, hipStream_t st)
{
    const int64_t n_chunks = gemm_codes_bytes(rows, K) / 16;
    const int64_t n_sbytes = gemm_scales_bytes(rows, K, fmt);
    int64_t b1 = (n_chunks + 255) / 256, b2 = (n_sbytes + 255) / 256;
    if (b1 > 8192) b1 = 8192;
    if (b2 > 8192) b2 = 8192;
    hipLaunchKernelGGL(repack_codes_kernel, dim3((unsigned)b1), dim3(256), 0, st, static_cast<const uint8_t*>(codes),
                       static_cast<uint8_t*>(codes_gemm), rows, K, n_chunks);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(repack_scales_kernel, dim3((unsigned)b2), dim3(256), 0, st, static_cast<const uint8_t*>(scales),
                       static_cast<uint8_t*>(scales_gemm), rows, K, fmt, n_sbytes);
    return hipGetLastError();
}

}  // namespace fp4mr
