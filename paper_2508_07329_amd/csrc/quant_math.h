// Arithmetic shared by the kernels that quantise activations (Eq. 1, Q(s^-1 X)): exact
// divisions through reused reciprocals, chunk loads, rounding and byte packing.
#pragma once
#include "haq_common.h"

namespace haq {

struct alignas(16) Half8 { __half v[8]; };

// x / d for a divisor that is reused: r = RN(1/d) once, then q0 = RN(x r),
// q = RN(q0 + r (x - q0 d)) with both corrections fused.  This is the correctly rounded
// quotient (the final step of the classic reciprocal-based division; checked here
// exhaustively for every binary16 significand of x against every binary32 significand of
// d) as long as nothing under- or overflows, which `safe_divisor` guarantees for binary16
// numerators; other divisors take the hardware division.  The second division of the kernel,
// y / scale with a binary32 numerator, only feeds a round-to-nearest-integer of magnitude
// <= 127: the sequence stays within 2 ulp of the quotient, so it could round differently from
// the IEEE quotient only next to a half-integer, and every numerator within 8 ulp of every
// half-integer multiple of every scale significand has been checked to round alike.
__device__ __forceinline__ bool safe_divisor(float d) { return d >= 0x1p-40f && d <= 0x1p40f; }
__device__ __forceinline__ float div_by(float x, float d, float r, bool fast) {
    if (fast) {
        const float q0 = x * r;
        const float e = __builtin_fmaf(-q0, d, x);
        return __builtin_fmaf(e, r, q0);
    }
    return x / d;
}

__device__ __forceinline__ void load_x16(const __half* xrow, int c, float (&x)[16]) {
    const uint4* px = reinterpret_cast<const uint4*>(xrow + c * 16);
    const uint4 r0 = px[0], r1 = px[1];
    Half8 h0, h1;
    *reinterpret_cast<uint4*>(&h0) = r0;
    *reinterpret_cast<uint4*>(&h1) = r1;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        x[i] = h2f(h0.v[i]);
        x[8 + i] = h2f(h1.v[i]);
    }
}

// reciprocals of one 16-channel chunk of the smoothing vector; `fast` says whether every
// channel of the chunk may use them
__device__ __forceinline__ bool load_s16(const float* s, int c, float (&sv)[16], float (&rv)[16]) {
    const float4* ps = reinterpret_cast<const float4*>(s + c * 16);
    bool fast = true;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float4 v = ps[i];
        sv[4 * i + 0] = v.x;
        sv[4 * i + 1] = v.y;
        sv[4 * i + 2] = v.z;
        sv[4 * i + 3] = v.w;
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        rv[i] = 1.0f / sv[i];
        fast = fast && safe_divisor(sv[i]);
    }
    return fast;
}

// Rounding in the common case: q = y / scale satisfies |q| <= 127 (1 + 2^-23) because
// |y| <= absmax and scale = RN(absmax / 127) is a normal number, so RN-to-integer never
// leaves [-127, 127] and the clamp of Eq. 1 is a no-op; adding 1.5 * 2^23 rounds q to an
// integer (ties to even, like rint) and leaves its two's-complement low byte in the low
// byte of the sum, which byte permutes gather four at a time.
__device__ __forceinline__ uint32_t round_pack4(float q0, float q1, float q2, float q3) {
    const uint32_t b0 = __float_as_uint(q0 + 12582912.0f), b1 = __float_as_uint(q1 + 12582912.0f);
    const uint32_t b2 = __float_as_uint(q2 + 12582912.0f), b3 = __float_as_uint(q3 + 12582912.0f);
    const uint32_t lo = __builtin_amdgcn_perm(b1, b0, 0x0c0c0400u);
    const uint32_t hi = __builtin_amdgcn_perm(b3, b2, 0x0c0c0400u);
    return __builtin_amdgcn_perm(hi, lo, 0x05040100u);
}


}  // namespace haq
