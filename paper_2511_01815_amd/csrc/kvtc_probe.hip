// Achievable-ceiling probes for gfx950 (declared in include/kvtc_probe.h): streaming read / write /
// copy of a device buffer and a register-only loop of bf16 matrix-core operations.  They give the
// numbers the coder's roofline fractions are quoted beside; the coder never calls them.
#include <hip/hip_runtime.h>
#include "../../include/kvtc_probe.h"

namespace kvtc {

typedef __bf16 bf16x8p __attribute__((ext_vector_type(8)));
typedef float f32x16p __attribute__((ext_vector_type(16)));

constexpr int kProbeThreads = 256;
constexpr int kProbeUnroll = 4;      // 16-byte pieces in flight per lane and trip

template <int MODE>
__global__ void __launch_bounds__(kProbeThreads) probe_stream_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
    const size_t stride = (size_t)gridDim.x * kProbeThreads;
    size_t i = (size_t)blockIdx.x * kProbeThreads + threadIdx.x;
    uint4 acc = make_uint4(0u, 0u, 0u, 0u);
    const uint4 fill = make_uint4(0x3c003c00u, 0x3c003c00u, 0x3c003c00u, 0x3c003c00u);
    for (; i + (kProbeUnroll - 1) * stride < n16; i += kProbeUnroll * stride) {
        uint4 v[kProbeUnroll];
        if (MODE != KVTC_PROBE_WRITE) {
#pragma unroll
            for (int k = 0; k < kProbeUnroll; ++k) v[k] = src[i + k * stride];
        }
#pragma unroll
        for (int k = 0; k < kProbeUnroll; ++k) {
            if (MODE == KVTC_PROBE_READ) { acc.x ^= v[k].x; acc.y ^= v[k].y; acc.z ^= v[k].z; acc.w ^= v[k].w; }
            else if (MODE == KVTC_PROBE_WRITE) dst[i + k * stride] = fill;
            else dst[i + k * stride] = v[k];
        }
    }
    for (; i < n16; i += stride) {
        if (MODE == KVTC_PROBE_READ) { const uint4 v = src[i]; acc.x ^= v.x; acc.y ^= v.y; acc.z ^= v.z; acc.w ^= v.w; }
        else if (MODE == KVTC_PROBE_WRITE) dst[i] = fill;
        else dst[i] = src[i];
    }
    if (MODE == KVTC_PROBE_READ && (acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u && acc.x == 0x7f4a7c15u && acc.y == 0xf39cc060u)
        reinterpret_cast<uint32_t*>(dst)[0] = acc.w;       // keeps the loads alive; practically never taken
}

// RANDOM = 0: operands take eight small values (little switching in the multipliers); 1: every operand
// register holds pseudo-random bf16 values of both signs with exponents spread over 2^-4 .. 2^3, and
// successive instructions see different operands -- what the coder's products look like to the matrix cores.
template <int RANDOM>
__global__ void __launch_bounds__(kProbeThreads) probe_mfma_kernel(int iters, float* sink) {
    const int lane = threadIdx.x & 63;
    bf16x8p a[4], b[2];
    if (RANDOM) {
        uint32_t st = 0x9e3779b9u * (uint32_t)(blockIdx.x * kProbeThreads + threadIdx.x + 1);
        auto next_pair = [&]() {                   // two bf16 values: random sign and mantissa, exponent 123..130
            st = st * 1664525u + 1013904223u;
            const uint32_t r = st >> 4;
            const uint32_t lo = ((r & 0x8000u) | ((123u + ((r >> 7) & 7u)) << 7) | (r & 0x7fu)) & 0xffffu;
            const uint32_t r2 = st >> 14;
            const uint32_t hi = ((r2 & 0x8000u) | ((123u + ((r2 >> 7) & 7u)) << 7) | (r2 & 0x7fu)) & 0xffffu;
            return lo | (hi << 16);
        };
        for (int k = 0; k < 4; ++k) a[k] = __builtin_bit_cast(bf16x8p, make_uint4(next_pair(), next_pair(), next_pair(), next_pair()));
        for (int k = 0; k < 2; ++k) b[k] = __builtin_bit_cast(bf16x8p, make_uint4(next_pair(), next_pair(), next_pair(), next_pair()));
    } else {
        bf16x8p a0, b0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            a0[e] = (__bf16)(0.001f * (float)((lane + e) & 7));
            b0[e] = (__bf16)(0.002f * (float)((lane * 3 + e) & 7));
        }
        for (int k = 0; k < 4; ++k) a[k] = a0;
        for (int k = 0; k < 2; ++k) b[k] = b0;
    }
    f32x16p acc[8];
#pragma unroll
    for (int k = 0; k < 8; ++k)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[k][e] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int k = 0; k < 8; ++k) acc[k] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[k & 3], b[k >> 2], acc[k], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int k = 0; k < 8; ++k)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[k][e];
    if (s != s) *sink = s;
}

}  // namespace kvtc

using namespace kvtc;

extern "C" {

kvtc_status kvtc_probe_stream(kvtc_probe_mode mode, const void* src_dev, void* dst_dev, size_t bytes, kvtc_stream stream) {
    if (mode < KVTC_PROBE_READ || mode > KVTC_PROBE_COPY) return KVTC_E_ARG;
    if (!dst_dev || (mode != KVTC_PROBE_WRITE && !src_dev)) return KVTC_E_ARG;
    if ((bytes & 15u) || (reinterpret_cast<uintptr_t>(src_dev) & 15u) || (reinterpret_cast<uintptr_t>(dst_dev) & 15u)) return KVTC_E_ARG;
    if (bytes == 0) return KVTC_OK;
    int dev = 0, cus = 256;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
        cus = prop.multiProcessorCount;
    const size_t n16 = bytes / 16;
    size_t want = (n16 + (size_t)kProbeThreads * kProbeUnroll - 1) / ((size_t)kProbeThreads * kProbeUnroll);
    const int grid = (int)(want < (size_t)cus * 8 ? want : (size_t)cus * 8);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint4* s = static_cast<const uint4*>(src_dev);
    uint4* d = static_cast<uint4*>(dst_dev);
    if (mode == KVTC_PROBE_READ) hipLaunchKernelGGL(probe_stream_kernel<KVTC_PROBE_READ>, dim3(grid), dim3(kProbeThreads), 0, st, s, d, n16);
    else if (mode == KVTC_PROBE_WRITE) hipLaunchKernelGGL(probe_stream_kernel<KVTC_PROBE_WRITE>, dim3(grid), dim3(kProbeThreads), 0, st, s, d, n16);
    else hipLaunchKernelGGL(probe_stream_kernel<KVTC_PROBE_COPY>, dim3(grid), dim3(kProbeThreads), 0, st, s, d, n16);
    return hipGetLastError() == hipSuccess ? KVTC_OK : KVTC_E_HIP;
}

kvtc_status kvtc_probe_mfma_bf16(int iters, int random_operands, void* sink_dev, double* flops_host, kvtc_stream stream) {
    if (iters < 1 || !sink_dev || !flops_host || random_operands < 0 || random_operands > 1) return KVTC_E_ARG;
    int dev = 0, cus = 256;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
        cus = prop.multiProcessorCount;
    const int grid = cus * 2;                      // two 4-wave workgroups per compute unit: two waves per SIMD
    if (random_operands)
        hipLaunchKernelGGL(probe_mfma_kernel<1>, dim3(grid), dim3(kProbeThreads), 0, static_cast<hipStream_t>(stream), iters,
                           static_cast<float*>(sink_dev));
    else
        hipLaunchKernelGGL(probe_mfma_kernel<0>, dim3(grid), dim3(kProbeThreads), 0, static_cast<hipStream_t>(stream), iters,
                           static_cast<float*>(sink_dev));
    if (hipGetLastError() != hipSuccess) return KVTC_E_HIP;
    *flops_host = (double)grid * (kProbeThreads / 64) * (double)iters * 8.0 * 2.0 * 32.0 * 32.0 * 16.0;
    return KVTC_OK;
}

}  // extern "C"
