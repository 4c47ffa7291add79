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
        fast = fast & safe_divisor(sv[i]);  // no short circuit: branch-free
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

// One row of Q(s^-1 x) by a whole work-group of NT threads (NCH 16-channel chunks per thread, so up
// to NT * NCH chunks): raw halves stay in registers between the absmax reduction and the rounding.
// `red` is LDS scratch of NT / 64 floats; `store(chunk, codes)` receives each finished chunk.  Every
// thread of the work-group must call it; returns the row scale absmax / 127.
template <int NT, int NCH, class Store>
__device__ __forceinline__ float quantise_row(const __half* xrow, const float* s, int nchunk, float* red, Store&& store) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint4 raw[NCH][2];
    float sv[NCH][16], rv[NCH][16];
    bool fast[NCH];
    float x[16];
    float amax = 0.0f;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const int c = tid + i * NT;
        fast[i] = true;
        raw[i][0] = raw[i][1] = make_uint4(0, 0, 0, 0);
        if (c < nchunk) {
            const uint4* px = reinterpret_cast<const uint4*>(xrow + c * 16);
            raw[i][0] = px[0];
            raw[i][1] = px[1];
            if (s) fast[i] = load_s16(s, c, sv[i], rv[i]);
        }
    }
    auto unpack = [&](int i) {
        Half8 h0, h1;
        *reinterpret_cast<uint4*>(&h0) = raw[i][0];
        *reinterpret_cast<uint4*>(&h1) = raw[i][1];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            x[k] = h2f(h0.v[k]);
            x[8 + k] = h2f(h1.v[k]);
        }
    };
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        if (tid + i * NT < nchunk) {
            unpack(i);
            if (!s) {
#pragma unroll
                for (int k = 0; k < 16; ++k) amax = fmaxf(amax, fabsf(x[k]));
            } else if (fast[i]) {
#pragma unroll
                for (int k = 0; k < 16; ++k) amax = fmaxf(amax, fabsf(div_by(x[k], sv[i][k], rv[i][k], true)));
            } else {
#pragma unroll
                for (int k = 0; k < 16; ++k) amax = fmaxf(amax, fabsf(x[k] / sv[i][k]));
            }
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) amax = fmaxf(amax, __shfl_xor(amax, o));
    __syncthreads();  // an earlier use of `red` is over
    if (lane == 0) red[wave] = amax;
    __syncthreads();
    float m = 0.0f;
#pragma unroll
    for (int w = 0; w < NT / 64; ++w) m = fmaxf(m, red[w]);
    const float scale = m / 127.0f;
    const float rscale = 1.0f / scale;
    const bool sfast = scale >= 0x1p-100f && scale <= 0x1p100f;
    // keeps the compiler from recomputing (and holding) the quotients of the first pass
#pragma unroll
    for (int i = 0; i < NCH; ++i)
#pragma unroll
        for (int h = 0; h < 2; ++h)
            asm volatile("" : "+v"(raw[i][h].x), "+v"(raw[i][h].y), "+v"(raw[i][h].z), "+v"(raw[i][h].w));
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const int c = tid + i * NT;
        if (c < nchunk) {
            uint32_t w[4] = {0, 0, 0, 0};
            if (m != 0.0f) {
                unpack(i);
                if (fast[i] && sfast) {
                    float q[16];
#pragma unroll
                    for (int k = 0; k < 16; ++k) {
                        const float y = s ? div_by(x[k], sv[i][k], rv[i][k], true) : x[k];
                        q[k] = div_by(y, scale, rscale, true);
                    }
#pragma unroll
                    for (int k = 0; k < 4; ++k) w[k] = round_pack4(q[4 * k], q[4 * k + 1], q[4 * k + 2], q[4 * k + 3]);
                } else {
#pragma unroll
                    for (int k = 0; k < 16; ++k) {
                        const float y = s ? x[k] / sv[i][k] : x[k];
                        w[k / 4] |= (uint32_t)(code_of(y, scale) & 0xff) << (8 * (k % 4));
                    }
                }
            }
            store(c, make_uint4(w[0], w[1], w[2], w[3]));
        }
    }
    return scale;
}

// One 16-channel chunk of the requantised intermediate: codes of (h / s_mid) / scale with the
// row's absmax m already known (scale = m / 127, rscale = 1 / scale, sfast: the reciprocal path
// is valid for this scale).
__device__ __forceinline__ uint4 requant_chunk(uint4 r0, uint4 r1, const float (&sv)[16], float m, float scale, float rscale,
                                               bool sfast) {
    uint32_t w[4] = {0, 0, 0, 0};
    if (m != 0.0f) {
        const __half* h0 = reinterpret_cast<const __half*>(&r0);
        const __half* h1 = reinterpret_cast<const __half*>(&r1);
        if (sfast) {
            float q[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float y = h2f(i < 8 ? h0[i] : h1[i - 8]) / sv[i];
                q[i] = div_by(y, scale, rscale, true);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) w[i] = round_pack4(q[4 * i], q[4 * i + 1], q[4 * i + 2], q[4 * i + 3]);
        } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float y = h2f(i < 8 ? h0[i] : h1[i - 8]) / sv[i];
                w[i / 4] |= (uint32_t)(code_of(y, scale) & 0xff) << (8 * (i % 4));
            }
        }
    }
    return make_uint4(w[0], w[1], w[2], w[3]);
}

}  // namespace haq
