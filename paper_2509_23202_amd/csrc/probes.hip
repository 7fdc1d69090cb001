// Measured ceilings of the machine the library runs on, for the denominators of a roofline report (the datasheet
// peaks assume the nominal 2.4 GHz clock, which the chip does not hold under matrix load):
//   * a register-resident issue loop of the block-scaled FP4 MFMA the MXFP4 GEMM is built on, and of the fp16 MFMA
//     the NVFP4 GEMM is built on -- eight waves per compute unit (two per SIMD, as in the GEMM kernels), sixteen
//     independent accumulators per wave, no memory traffic at all: what the matrix pipes deliver when nothing else
//     is in the way;
//   * a streaming copy and a streaming read of a large buffer, 16 bytes per lane, non-temporal: what HBM delivers to
//     the access pattern the rotate+quantize kernel uses.
// The host times the launches with events.  The issue loops also record the raw differences of the two shader-readable
// counters; their tick rates are machine-dependent, so no rate is derived from them here.
#include "device_util.hpp"
#include "internal.hpp"

namespace fp4mr {
namespace {

struct ProbeOut {
    uint64_t shader_clocks;  // s_memtime ticks over the loop
    uint64_t ref_ticks;      // s_memrealtime ticks over the loop
    uint64_t checksum;       // keeps the accumulators alive
};

template <bool FP4>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2))) void mfma_issue_kernel(ProbeOut* out, int iters)
{
    v4f acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = v4f{0.f, 0.f, 0.f, 0.f};
    // operands: every code pattern occurs (the data path toggles as it does on quantized data)
    const uint32_t seed = 0x9e3779b9u * (uint32_t)(blockIdx.x * 512 + threadIdx.x + 1);
    const v4i a = {(int)seed, (int)(seed * 3u), (int)(seed * 5u), (int)(seed * 7u)};
    const v4i b = {(int)(seed * 11u), (int)(seed * 13u), (int)(seed * 17u), (int)(seed * 19u)};
    const uint32_t scale = 0x7f7f7f7fu;  // E8M0 127 = 2^0 in every byte
    const uint64_t t0 = __builtin_amdgcn_s_memtime();
    const uint64_t r0 = __builtin_amdgcn_s_memrealtime();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int rep = 0; rep < 2; ++rep) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                if constexpr (FP4) {
                    const v8i a8 = {a[0], a[1], a[2], a[3], 0, 0, 0, 0};
                    const v8i b8 = {b[0], b[1], b[2], b[3], 0, 0, 0, 0};
                    acc[i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a8, b8, acc[i], 4, 4, 0, (int)scale, 0, (int)scale);
                } else {
                    // fp16 operands with finite values: sign and mantissa kept, exponent field forced to 2^-1
                    auto h = [](int w) { return (int)(((uint32_t)w & 0x83ff83ffu) | 0x38003800u); };
                    const v4i ah = {h(a[0]), h(a[1]), h(a[2]), h(a[3])};
                    const v4i bh = {h(b[0]), h(b[1]), h(b[2]), h(b[3])};
                    acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(v8h, ah), __builtin_bit_cast(v8h, bh), acc[i], 0, 0, 0);
                }
            }
        }
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
    const uint64_t t1 = __builtin_amdgcn_s_memtime();
    const uint64_t r1 = __builtin_amdgcn_s_memrealtime();
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) s += __shfl_xor(s, d);
    if (threadIdx.x == 0) {
        out[blockIdx.x].shader_clocks = t1 - t0;
        out[blockIdx.x].ref_ticks = r1 - r0;
        out[blockIdx.x].checksum = (uint64_t)__float_as_uint(s);
    }
}

// dst[i] = src[i] over n 16-byte words (COPY), or a checksum of src (read only)
template <bool COPY>
__global__ __launch_bounds__(256) void stream_kernel(const v4i* __restrict__ src, v4i* __restrict__ dst, int64_t n, uint32_t* sink)
{
    const int64_t stride = (int64_t)gridDim.x * 256 * 4;
    int acc = 0;
    for (int64_t i = (int64_t)blockIdx.x * 1024 + threadIdx.x; i < n; i += stride) {
        v4i v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t j = i + u * 256;
            v[u] = j < n ? __builtin_nontemporal_load(src + j) : v4i{0, 0, 0, 0};
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t j = i + u * 256;
            if constexpr (COPY) {
                if (j < n) __builtin_nontemporal_store(v[u], dst + j);
            } else {
                acc ^= v[u][0] ^ v[u][1] ^ v[u][2] ^ v[u][3];
            }
        }
    }
    if constexpr (!COPY) {
        if (acc == 0x5a5a5a5a) *sink = (uint32_t)acc;  // (practically never: the loads must still be performed)
    }
}

}  // namespace

hipError_t launch_probe(int which, void* buf, size_t bytes, int iters, hipStream_t st)
{
    int cus = 256, dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
    if (which == 0 || which == 1) {
        if (bytes < (size_t)cus * sizeof(ProbeOut) || iters <= 0) return hipErrorInvalidValue;
        if (which == 0) hipLaunchKernelGGL(mfma_issue_kernel<true>, dim3((unsigned)cus), dim3(512), 0, st, static_cast<ProbeOut*>(buf), iters);
        else hipLaunchKernelGGL(mfma_issue_kernel<false>, dim3((unsigned)cus), dim3(512), 0, st, static_cast<ProbeOut*>(buf), iters);
        return hipGetLastError();
    }
    if (which == 2 || which == 3) {
        const int64_t half = (int64_t)(bytes / 32);  // 16-byte words per half of the buffer
        if (half < 1) return hipErrorInvalidValue;
        const v4i* src = static_cast<const v4i*>(buf);
        v4i* dst = static_cast<v4i*>(buf) + half;
        // one pass of 1024 words per workgroup-iteration; enough workgroups to fill the chip many times over
        int64_t blocks = (half + 1023) / 1024;
        if (blocks > (int64_t)cus * 64) blocks = (int64_t)cus * 64;
        if (which == 2) hipLaunchKernelGGL(stream_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, st, src, dst, half, nullptr);
        else hipLaunchKernelGGL(stream_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, st, src, dst, half, reinterpret_cast<uint32_t*>(dst));
        return hipGetLastError();
    }
    return hipErrorInvalidValue;
}

}  // namespace fp4mr
