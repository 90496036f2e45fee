// Calibration on the GPU, the data-heavy part of the bit allocation (declared in include/kvtc.h,
// "Calibration"): the table of block errors that the dynamic programme reads.  (Paper, Section
// "Quantization" and appendix "Dynamic programming algorithm": for every candidate block of subsequent
// PCA coordinates and every quantiser type, the block of calibration coefficients is quantised as the
// coder would quantise it, and the squared error is compared with dropping the block.)
//
// One workgroup per candidate block, so every sum has a fixed order and the table is reproducible.
// A group of L = 16 or 64 lanes owns a token (L = 16 for blocks of fewer than 64 coordinates): the
// token's coefficients of the block sit in registers, the group's min and max come from shuffles, and
// every width is evaluated from the same registers with the coder's own scalar numerics (fp16 shift
// rounded down, scale rounded up, code by subtract, multiply by the rounded reciprocal, round to
// even, clamp).  Errors are accumulated in double from exactly representable terms.
//
// Also here: the first and second moments of the calibration tokens (sum of x and sum of x x^T, in
// double), the one pass over the calibration data that the PCA needs (paper, Section "Feature
// decorrelation", eq. 2: mean and SVD of the centred matrix; its right singular vectors are the
// eigenvectors of the centred second-moment matrix, which the caller forms and decomposes on the host).
#include <hip/hip_runtime.h>

#include "kvtc_dev.h"
#include "kvtc_numeric.h"

namespace kvtc {
kvtc_status set_error(kvtc_status st, const char* fmt, ...);
}
using namespace kvtc;

namespace {

constexpr int kCalibMaxBits = 8;
constexpr int kCalibMaxN = 1024;
constexpr int kCalibThreads = 256;

template <int L>
__device__ __forceinline__ float group_min(float v) {
#pragma unroll
    for (int d = L / 2; d > 0; d >>= 1) v = fminf(v, __shfl_xor(v, d, 64));
    return v;
}
template <int L>
__device__ __forceinline__ float group_max(float v) {
#pragma unroll
    for (int d = L / 2; d > 0; d >>= 1) v = fmaxf(v, __shfl_xor(v, d, 64));
    return v;
}

// PER = coordinates per lane (n <= L * PER)
template <int L, int PER>
__device__ __forceinline__ void block_errors(const float* coef, int64_t n_tokens, int64_t ld, int start, int n, int max_bits, double* acc /*[kCalibMaxBits + 1]*/) {
    const int tid = threadIdx.x;
    const int grp = tid / L, gl = tid % L, n_grp = kCalibThreads / L;
    for (int64_t t0 = 0; t0 < n_tokens; t0 += n_grp) {          // every lane runs the same trips: the shuffles need whole waves
        const int64_t t = t0 + grp;
        const bool live = t < n_tokens;
        float d[PER];
        float lo = __builtin_inff(), hi = -__builtin_inff();
#pragma unroll
        for (int k = 0; k < PER; ++k) {
            const int j = gl + k * L;
            const bool in = live && j < n;
            d[k] = in ? coef[t * ld + start + j] : 0.0f;
            if (in) { lo = fminf(lo, d[k]); hi = fmaxf(hi, d[k]); }
        }
        lo = group_min<L>(lo);
        hi = group_max<L>(hi);
        if (!live) continue;
        double energy = 0.0;
#pragma unroll
        for (int k = 0; k < PER; ++k)
            if (gl + k * L < n) energy += (double)d[k] * (double)d[k];
        acc[0] += energy;
#pragma unroll
        for (int b = 1; b <= kCalibMaxBits; ++b) {          // (unrolled: the accumulators stay in registers)
            if (b > max_bits) break;
            const GroupQ q = group_header(lo, hi, b);
            const float qmax = (float)((1u << b) - 1u);
            const double shift = (double)q.shift, scale = (double)f16_bits_to_f32(q.scale16);
            double e = 0.0;
#pragma unroll
            for (int k = 0; k < PER; ++k)
                if (gl + k * L < n) {
                    const double dh = shift + (double)code_of(d[k], q.shift, q.inv, qmax) * scale;
                    const double r = (double)d[k] - dh;
                    e += r * r;
                }
            acc[b] += e;
        }
    }
}

// change[block][b - 1] = sum over tokens and the block's coordinates of (d - d_hat)^2 - d^2
__global__ void __launch_bounds__(kCalibThreads) calib_block_errors_kernel(const float* coef, int64_t n_tokens, int64_t ld, const kvtc_calib_block* blocks,
                                                                          int max_bits, double* change) {
    __shared__ double red[kCalibThreads];
    const kvtc_calib_block blk = blocks[blockIdx.x];
    const int start = blk.start, n = blk.n;
    // the list lives on the device, out of the host's sight: a block outside a row (or longer than a lane group holds) gets NaN
    if (n < 1 || n > kCalibMaxN || start < 0 || (int64_t)start + n > ld) {
        if ((int)threadIdx.x < max_bits) change[(size_t)blockIdx.x * max_bits + threadIdx.x] = __builtin_nan("");
        return;
    }
    double acc[kCalibMaxBits + 1];
#pragma unroll
    for (int b = 0; b <= kCalibMaxBits; ++b) acc[b] = 0.0;
    if (n < 64) block_errors<16, 4>(coef, n_tokens, ld, start, n, max_bits, acc);
    else if (n <= 256) block_errors<64, 4>(coef, n_tokens, ld, start, n, max_bits, acc);
    else block_errors<64, 16>(coef, n_tokens, ld, start, n, max_bits, acc);
    // fixed-order reduction over the workgroup, one width at a time
    double energy = 0.0;
#pragma unroll
    for (int b = 0; b <= kCalibMaxBits; ++b) {
        if (b > max_bits) break;
        red[threadIdx.x] = acc[b];
        __syncthreads();
        for (int d = kCalibThreads / 2; d > 0; d >>= 1) {
            if ((int)threadIdx.x < d) red[threadIdx.x] += red[threadIdx.x + d];
            __syncthreads();
        }
        if (b == 0) energy = red[0];
        else if (threadIdx.x == 0) change[(size_t)blockIdx.x * max_bits + (b - 1)] = red[0] - energy;
        __syncthreads();
    }
}


// ---- moments ------------------------------------------------------------------------------------
constexpr int kGramTile = 64;      // a workgroup owns a 64 x 64 tile of the second-moment matrix, a thread 4 x 4 of it
constexpr int kGramTokens = 32;    // tokens staged per step

template <typename XT> __device__ __forceinline__ double load_as_double(const XT* p);
template <> __device__ __forceinline__ double load_as_double<uint16_t>(const uint16_t* p) { return (double)bits_f32((uint32_t)*p << 16); }
template <> __device__ __forceinline__ double load_as_double<float>(const float* p) { return (double)*p; }

// element offset of feature f inside a token (blocks of 2^blk_log2 features lie blk_jump elements apart; 0 = contiguous)
__device__ __forceinline__ int64_t feature_offset(int f, int blk_log2, int64_t blk_jump) {
    return (int64_t)f + (blk_log2 ? (int64_t)(f >> blk_log2) * blk_jump : (int64_t)0);
}

template <typename XT>
__global__ void __launch_bounds__(256) calib_sum_kernel(const XT* x, int64_t n_tokens, int p, int64_t ld, int blk_log2, int64_t blk_jump, double* sum) {
    const int f = blockIdx.x * 256 + threadIdx.x;
    if (f >= p) return;
    const XT* col = x + feature_offset(f, blk_log2, blk_jump);
    double s = 0.0;
    for (int64_t t = 0; t < n_tokens; ++t) s += load_as_double<XT>(col + t * ld);       // token order: a fixed sum
    sum[f] = s;
}

template <typename XT>
__global__ void __launch_bounds__(256) calib_gram_kernel(const XT* x, int64_t n_tokens, int p, int64_t ld, int blk_log2, int64_t blk_jump, double* gram) {
    __shared__ double a[kGramTokens][kGramTile], b[kGramTokens][kGramTile];
    const int tid = threadIdx.x, ty = tid >> 4, tx = tid & 15;
    const int i0 = blockIdx.y * kGramTile, j0 = blockIdx.x * kGramTile;
    double acc[4][4];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[r][c] = 0.0;
    for (int64_t t0 = 0; t0 < n_tokens; t0 += kGramTokens) {
#pragma unroll
        for (int k = 0; k < kGramTokens * kGramTile / 256; ++k) {
            const int e = tid + k * 256, tt = e / kGramTile, ff = e % kGramTile;
            const int64_t t = t0 + tt;
            const bool in = t < n_tokens;
            a[tt][ff] = in ? load_as_double<XT>(x + t * ld + feature_offset(i0 + ff, blk_log2, blk_jump)) : 0.0;
            b[tt][ff] = in ? load_as_double<XT>(x + t * ld + feature_offset(j0 + ff, blk_log2, blk_jump)) : 0.0;
        }
        __syncthreads();
#pragma unroll 4
        for (int tt = 0; tt < kGramTokens; ++tt) {
            double ra[4], rb[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) { ra[r] = a[tt][ty * 4 + r]; rb[r] = b[tt][tx * 4 + r]; }
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[r][c] = __builtin_fma(ra[r], rb[c], acc[r][c]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c) gram[(size_t)(i0 + ty * 4 + r) * p + (j0 + tx * 4 + c)] = acc[r][c];
}

}  // namespace

namespace kvtc {
// x: n_tokens tokens of p features (p a multiple of 64) at the given layout; sum [p], gram [p][p]
hipError_t launch_calib_moments(const void* x, kvtc_dtype dtype, int64_t n_tokens, int p, int64_t ld, int blk_log2, int64_t blk_jump,
                                double* sum, double* gram, hipStream_t stream) {
    const dim3 gs((unsigned)((p + 255) / 256)), gg((unsigned)(p / kGramTile), (unsigned)(p / kGramTile));
    if (dtype == KVTC_BF16) {
        hipLaunchKernelGGL(calib_sum_kernel<uint16_t>, gs, dim3(256), 0, stream, static_cast<const uint16_t*>(x), n_tokens, p, ld, blk_log2, blk_jump, sum);
        hipLaunchKernelGGL(calib_gram_kernel<uint16_t>, gg, dim3(256), 0, stream, static_cast<const uint16_t*>(x), n_tokens, p, ld, blk_log2, blk_jump, gram);
    } else {
        hipLaunchKernelGGL(calib_sum_kernel<float>, gs, dim3(256), 0, stream, static_cast<const float*>(x), n_tokens, p, ld, blk_log2, blk_jump, sum);
        hipLaunchKernelGGL(calib_gram_kernel<float>, gg, dim3(256), 0, stream, static_cast<const float*>(x), n_tokens, p, ld, blk_log2, blk_jump, gram);
    }
    return hipGetLastError();
}
}  // namespace kvtc

namespace {
}  // namespace

extern "C" {

kvtc_status kvtc_calib_block_errors(const float* coef_dev, int64_t n_tokens, int64_t ld, const kvtc_calib_block* blocks_dev, int n_blocks,
                                    int max_bits, double* change_dev, kvtc_stream stream) {
    if (n_blocks < 0 || n_tokens < 0) return set_error(KVTC_E_ARG, "kvtc_calib_block_errors: n_blocks=%d, n_tokens=%lld", n_blocks, (long long)n_tokens);
    if (max_bits < 1 || max_bits > kCalibMaxBits) return set_error(KVTC_E_ARG, "kvtc_calib_block_errors: max_bits=%d outside 1..%d", max_bits, kCalibMaxBits);
    if (n_blocks == 0) return KVTC_OK;
    if (!coef_dev || !blocks_dev || !change_dev) return set_error(KVTC_E_ARG, "kvtc_calib_block_errors: null argument");
    if (ld < 1) return set_error(KVTC_E_ARG, "kvtc_calib_block_errors: ld=%lld", (long long)ld);
    if ((reinterpret_cast<uintptr_t>(coef_dev) & 3u) || (reinterpret_cast<uintptr_t>(change_dev) & 7u) || (reinterpret_cast<uintptr_t>(blocks_dev) & 3u))
        return set_error(KVTC_E_ARG, "kvtc_calib_block_errors: misaligned buffer");
    hipLaunchKernelGGL(calib_block_errors_kernel, dim3((unsigned)n_blocks), dim3(kCalibThreads), 0, static_cast<hipStream_t>(stream), coef_dev, n_tokens, ld,
                       blocks_dev, max_bits, change_dev);
    const hipError_t err = hipGetLastError();
    if (err != hipSuccess) return set_error(KVTC_E_HIP, "kvtc_calib_block_errors: launch failed: %s", hipGetErrorString(err));
    return KVTC_OK;
}

}  // extern "C"
