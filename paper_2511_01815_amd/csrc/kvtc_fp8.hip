// FP8 storage of the sink tokens and the stream offsets of an incremental append, for gfx950.
// (Paper, Section "Sliding Windows and Sink Tokens": the s oldest tokens are not transform-coded;
// Appendix "Compression ratio with sliding window": they are kept in FP8.  Section "Experimental
// setup": the coder runs again every c new tokens.)
//
// FP8 here is OCP E4M3: 1 sign, 4 exponent bits (bias 7), 3 mantissa bits, no infinities, the
// all-ones exponent with all-ones mantissa is NaN, largest finite magnitude 448.  Conversion is a
// plain cast of each value: round to nearest, ties to even mantissa, magnitudes from 448 up
// saturate to 448, NaN gives 0x7f.  Done in integer arithmetic so that every step is defined here
// and not by a conversion instruction's mode bits.  The work is a few KB per tensor: no tuning.
#include <hip/hip_runtime.h>
#include "kvtc_dev.h"

namespace kvtc {

__device__ __forceinline__ uint32_t e4m3_from_f32(float f) {
    const uint32_t u = __float_as_uint(f);
    const uint32_t sign = (u >> 24) & 0x80u;
    const uint32_t a = u & 0x7fffffffu;
    if (a > 0x7f800000u) return 0x7fu;                              // NaN
    if (a >= 0x43e00000u) return sign | 0x7eu;                      // |f| >= 448 (and infinity): saturate
    if (a < 0x3c800000u) {                                          // |f| < 2^-6: the subnormal grid, spacing 2^-9
        const float q = __builtin_rintf(__uint_as_float(a) * 512.0f);   // exact product, round half to even; 8 = smallest normal
        return sign | (uint32_t)q;
    }
    // normal: keep 3 of the 23 mantissa bits, round half to even (a carry runs into the exponent as it should)
    const uint32_t r = a + 0x7ffffu + ((a >> 20) & 1u);
    return sign | ((r >> 20) - (120u << 3));                        // exponent bias 127 -> 7
}

__device__ __forceinline__ float f32_from_e4m3(uint32_t c) {
    const uint32_t sign = (c & 0x80u) << 24;
    const uint32_t e = (c >> 3) & 0xfu, m = c & 7u;
    if (e == 0u) return __uint_as_float(sign | __float_as_uint((float)m * 0.001953125f));   // m * 2^-9
    if ((c & 0x7fu) == 0x7fu) return __uint_as_float(0x7fc00000u);
    return __uint_as_float(sign | ((e + 120u) << 23) | (m << 20));
}

__device__ __forceinline__ float load_elem(const uint16_t* p) { return __uint_as_float((uint32_t)*p << 16); }
__device__ __forceinline__ float load_elem(const float* p) { return *p; }
__device__ __forceinline__ void store_elem(uint16_t* p, float v) { *p = (uint16_t)(__float_as_uint(v) >> 16); }   // E4M3 values are exact in bf16
__device__ __forceinline__ void store_elem(float* p, float v) { *p = v; }

// x [n_tokens][ld_x] -> out [n_tokens][p] bytes; fp32 inputs are first rounded to bf16 (nearest even), as
// the coder does with them, so that both parts of a cache see the same values
template <typename XT>
__global__ void __launch_bounds__(256) fp8_pack_kernel(const XT* x, int64_t n_tokens, int p, int64_t ld_x, uint8_t* out) {
    const int64_t total = n_tokens * p;
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t t = i / p;
        const int f = (int)(i - t * p);
        float v = load_elem(x + t * ld_x + f);
        if (sizeof(XT) == 4) {
            const uint32_t u = __float_as_uint(v);
            if ((u & 0x7fffffffu) <= 0x7f800000u) v = __uint_as_float((u + 0x7fffu + ((u >> 16) & 1u)) & 0xffff0000u);
        }
        out[i] = (uint8_t)e4m3_from_f32(v);
    }
}

template <typename XT>
__global__ void __launch_bounds__(256) fp8_unpack_kernel(const uint8_t* in, int64_t n_tokens, int p, int64_t ld_x, XT* x) {
    const int64_t total = n_tokens * p;
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t t = i / p;
        const int f = (int)(i - t * p);
        store_elem(x + t * ld_x + f, f32_from_e4m3(in[i]));
    }
}

// offsets[j] = region[j] + n_coded[j] * R(plan of job j): where the records of job j's new tokens go when
// job j's stream lives in its own region of the buffer and already holds n_coded[j] records.  A job
// whose new records would run past the start of the next region gets the offset ~0, which the encode
// launch reports as a job that does not fit.  offsets[n_jobs] = region[n_jobs].
__global__ void __launch_bounds__(256) offsets_append_kernel(const uint32_t* rec_dwords, int n_plans, const kvtc_job* jobs, int n_jobs,
                                                            const uint64_t* region, const int64_t* n_coded, uint64_t* offsets) {
    for (int j = blockIdx.x * blockDim.x + threadIdx.x; j <= n_jobs; j += gridDim.x * blockDim.x) {
        if (j == n_jobs) { offsets[j] = region[j]; continue; }
        const kvtc_job jb = jobs[j];
        uint64_t off = ~0ull;
        if (jb.plan >= 0 && jb.plan < n_plans && jb.n_tokens >= 0 && n_coded[j] >= 0 && region[j + 1] >= region[j]) {
            const uint64_t R = (uint64_t)rec_dwords[jb.plan] * 4ull;
            const uint64_t room = region[j + 1] - region[j];
            const uint64_t have = (uint64_t)n_coded[j], add = (uint64_t)jb.n_tokens;
            if (have <= room / R && add <= room / R - have) off = region[j] + have * R;
        }
        offsets[j] = off;
    }
}

hipError_t launch_fp8_pack(const void* x, kvtc_dtype dtype, int64_t n_tokens, int p, int64_t ld_x, void* out, hipStream_t stream) {
    const int64_t total = n_tokens * p;
    const int grid = (int)((total + 255) / 256 < 4096 ? (total + 255) / 256 : 4096);
    if (dtype == KVTC_BF16)
        hipLaunchKernelGGL(fp8_pack_kernel<uint16_t>, dim3(grid), dim3(256), 0, stream, static_cast<const uint16_t*>(x), n_tokens, p, ld_x, static_cast<uint8_t*>(out));
    else
        hipLaunchKernelGGL(fp8_pack_kernel<float>, dim3(grid), dim3(256), 0, stream, static_cast<const float*>(x), n_tokens, p, ld_x, static_cast<uint8_t*>(out));
    return hipGetLastError();
}

hipError_t launch_fp8_unpack(const void* in, int64_t n_tokens, int p, void* x, kvtc_dtype dtype, int64_t ld_x, hipStream_t stream) {
    const int64_t total = n_tokens * p;
    const int grid = (int)((total + 255) / 256 < 4096 ? (total + 255) / 256 : 4096);
    if (dtype == KVTC_BF16)
        hipLaunchKernelGGL(fp8_unpack_kernel<uint16_t>, dim3(grid), dim3(256), 0, stream, static_cast<const uint8_t*>(in), n_tokens, p, ld_x, static_cast<uint16_t*>(x));
    else
        hipLaunchKernelGGL(fp8_unpack_kernel<float>, dim3(grid), dim3(256), 0, stream, static_cast<const uint8_t*>(in), n_tokens, p, ld_x, static_cast<float*>(x));
    return hipGetLastError();
}

hipError_t launch_offsets_append(const uint32_t* rec_dwords, int n_plans, const kvtc_job* jobs, int n_jobs, const uint64_t* region,
                                 const int64_t* n_coded, uint64_t* offsets, hipStream_t stream) {
    hipLaunchKernelGGL(offsets_append_kernel, dim3((n_jobs + 256) / 256), dim3(256), 0, stream, rec_dwords, n_plans, jobs, n_jobs, region,
                       n_coded, offsets);
    return hipGetLastError();
}

}  // namespace kvtc
