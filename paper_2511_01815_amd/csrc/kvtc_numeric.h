// Scalar numerics of the quantiser, shared by the gfx950 kernels and the host-side
// test helpers of the library (one definition, compiled for both).
//
// The paper (Section "Quantization") fixes "16-bit shift and scaling factors" per
// group and uniform min-max quantisation; the concrete choices are:
// IEEE fp16, shift rounded toward -inf, scale toward +inf (so the stored range
// always covers [lo, hi] and no entry clips), saturation at +-65504, and the code
// decided by round-half-even((d - shift) * (1/scale)) in fp32.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#include <hip/hip_runtime.h>
#define KVTC_HD __host__ __device__ __forceinline__
#else
#define KVTC_HD inline
#endif

namespace kvtc {

KVTC_HD uint32_t f32_bits(float x) { return __builtin_bit_cast(uint32_t, x); }
KVTC_HD float bits_f32(uint32_t u) { return __builtin_bit_cast(float, u); }

// fp32 -> fp16 bit pattern with directed rounding, pure integer arithmetic.
// up = true: toward +inf, false: toward -inf.  Magnitudes above 65504 (and NaN)
// saturate to +-65504.
KVTC_HD uint16_t f16_round_dir(float x, bool up) {
    const uint32_t u = f32_bits(x);
    const uint32_t sign = u >> 31;
    uint32_t a = u & 0x7fffffffu;
    if (a > 0x477fe000u) a = 0x477fe000u;              // 65504.0f
    const uint32_t e = a >> 23;
    const uint32_t m = a & 0x7fffffu;
    uint32_t h, rem;
    if (e >= 113u) {                                     // fp16 normal
        h = ((e - 112u) << 10) | (m >> 13);
        rem = m & 0x1fffu;
    } else if (e >= 102u) {                              // fp16 subnormal
        const uint32_t mant = m | 0x800000u;
        const uint32_t sh = 126u - e;                    // 14 .. 24
        h = mant >> sh;
        rem = mant & ((1u << sh) - 1u);
    } else {                                             // below half the smallest subnormal
        h = 0u;
        rem = a;
    }
    const bool away = up ? (sign == 0u) : (sign != 0u);  // round the magnitude away from zero?
    if (rem != 0u && away) h += 1u;
    return (uint16_t)((sign << 15) | h);
}

KVTC_HD float f16_bits_to_f32(uint16_t hbits) {
    const uint32_t sign = (uint32_t)(hbits >> 15) << 31;
    const uint32_t e = (hbits >> 10) & 0x1fu;
    const uint32_t m = hbits & 0x3ffu;
    if (e == 0u) {                                       // zero / subnormal: m * 2^-24, exact in fp32
        const float v = (float)m * 5.9604644775390625e-08f;
        return bits_f32(f32_bits(v) | sign);
    }
    if (e == 31u) return bits_f32(sign | 0x7f800000u | (m << 13));
    return bits_f32(sign | ((e + 112u) << 23) | (m << 13));
}

struct GroupQ {
    uint16_t shift16, scale16;
    float shift, inv;        // fp32 values used for the code decision
};

KVTC_HD float div_rn(float a, float b) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __fdiv_rn(a, b);
#else
    return a / b;
#endif
}

// Header of one (token, group) from the group's fp32 min and max.
KVTC_HD GroupQ group_header(float lo, float hi, int bits) {
    GroupQ g;
    g.shift16 = f16_round_dir(lo, false);
    g.shift = f16_bits_to_f32(g.shift16);
    const float qmax = (float)((1u << bits) - 1u);
    const float range = hi - g.shift;                    // one fp32 subtraction
    g.scale16 = f16_round_dir(div_rn(range, qmax), true);
    const float sc = f16_bits_to_f32(g.scale16);
    g.inv = sc > 0.0f ? div_rn(1.0f, sc) : 0.0f;
    return g;
}

// The code of one coefficient from its group's decoded header: two fp32 operations (subtract the
// shift, multiply by the rounded reciprocal of the scale), round half to even, clamp to
// [0, qmax = 2^bits - 1].  inv == 0 (zero scale) gives 0.
KVTC_HD float code_of(float d, float shift, float inv, float qmax) {
#if defined(__HIP_DEVICE_COMPILE__)
    const float q = __fmul_rn(__fsub_rn(d, shift), inv);
    return __builtin_amdgcn_fmed3f(__builtin_rintf(q), 0.0f, qmax);
#else
    volatile float t = d - shift;            // kept apart: the host compiler must not fuse them
    volatile float q = t * inv;
    float rq = __builtin_nearbyintf(q);
    if (!(rq >= 0.0f)) rq = 0.0f;
    if (rq > qmax) rq = qmax;
    return rq;
#endif
}

}  // namespace kvtc
