// Rotary positional embedding of keys, undone before they are coded and redone after they are
// decoded, for gfx950.  (Paper, Section "Feature decorrelation": the positional rotation hides the
// low-rank structure of keys, so it is removed before the transform and compression works on keys
// as they were before the rotation; decoded keys are rotated again before attention reads them.)
//
// The rotation is RoFormer's: inside every head, features are paired, and the pair (a, b) of the
// token at position m is turned by m * theta_j, theta_j = base^(-2j / d_head):
//     a' = a cos - b sin,  b' = a sin + b cos        (undoing it: the opposite angle).
// Pair j is (j, j + d_head/2) ("half", the rotate-half form) or (2j, 2j+1) ("interleaved").
//
// A streaming kernel, in place: 2 x element size bytes of traffic per value.  Angles, sines,
// cosines, products and sums are all double precision -- an angle reaches 10^5 radians, where a
// float has lost the sine -- and the result is rounded once to the tensor's type, so it equals a
// float64 reference rounded the same way.  A lane owns one pair index of its token in every head:
// one sincos serves all heads, and neighbouring lanes touch neighbouring elements.  The
// frequencies theta_j are computed on the host and travel as kernel arguments.
#include <hip/hip_runtime.h>
#include "kvtc_dev.h"

namespace kvtc {

constexpr int kRopeMaxHalf = 128;      // d_head / 2 at most (the frequency table is a kernel argument)

struct RopeArgs {
    void* x;
    int64_t n_tokens, token_stride, head_stride;     // strides in elements
    const int32_t* positions;                        // device, [n_tokens], or nullptr: position0 + token
    int64_t position0;
    int32_t n_heads, d_head, inverse;
    double theta[kRopeMaxHalf];                      // [d_head / 2]
};

__device__ __forceinline__ double load_val(const uint16_t* p) { return (double)__uint_as_float((uint32_t)*p << 16); }
__device__ __forceinline__ double load_val(const float* p) { return (double)*p; }
__device__ __forceinline__ void store_val(uint16_t* p, double v) {
    // double -> float -> bf16, both to nearest even (the float step can move a result only if it lies within 2^-29
    // relative of a bf16 rounding boundary)
    const uint32_t u = __float_as_uint((float)v);
    if ((u & 0x7fffffffu) > 0x7f800000u) { *p = (uint16_t)((u >> 16) | 0x40u); return; }      // NaN stays NaN
    *p = (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}
__device__ __forceinline__ void store_val(float* p, double v) { *p = (float)v; }

// INTERLEAVED = 0: pair j = (j, j + half); 1: pair j = (2j, 2j + 1)
template <typename T, int INTERLEAVED>
__global__ void __launch_bounds__(256) rope_kernel(const RopeArgs a) {
    const int half = a.d_head / 2;
    const int64_t n_items = a.n_tokens * (int64_t)half;          // one item = one (token, pair index)
    T* x = static_cast<T*>(a.x);
    for (int64_t item = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; item < n_items; item += (int64_t)gridDim.x * blockDim.x) {
        const int64_t t = item / half;
        const int j = (int)(item - t * half);
        const int64_t pos = a.positions ? (int64_t)a.positions[t] : a.position0 + t;
        double s, c;
        sincos((double)pos * a.theta[j], &s, &c);
        if (a.inverse) s = -s;
        T* row = x + t * a.token_stride;
        const int ia = INTERLEAVED ? 2 * j : j, ib = INTERLEAVED ? 2 * j + 1 : j + half;
        for (int h = 0; h < a.n_heads; ++h) {
            T* head = row + (int64_t)h * a.head_stride;
            const double va = load_val(head + ia), vb = load_val(head + ib);
            store_val(head + ia, __dsub_rn(__dmul_rn(va, c), __dmul_rn(vb, s)));
            store_val(head + ib, __dadd_rn(__dmul_rn(va, s), __dmul_rn(vb, c)));
        }
    }
}

hipError_t launch_rope(const RopeArgs& a, kvtc_dtype dtype, int interleaved, int grid, hipStream_t stream) {
    if (dtype == KVTC_BF16) {
        if (interleaved) hipLaunchKernelGGL((rope_kernel<uint16_t, 1>), dim3(grid), dim3(256), 0, stream, a);
        else hipLaunchKernelGGL((rope_kernel<uint16_t, 0>), dim3(grid), dim3(256), 0, stream, a);
    } else {
        if (interleaved) hipLaunchKernelGGL((rope_kernel<float, 1>), dim3(grid), dim3(256), 0, stream, a);
        else hipLaunchKernelGGL((rope_kernel<float, 0>), dim3(grid), dim3(256), 0, stream, a);
    }
    return hipGetLastError();
}

}  // namespace kvtc
