// CPU check for the second division of the activation-quantisation kernel, y / scale with an
// arbitrary binary32 numerator, where only the integer rne(y / scale) is used (|code| <= 255:
// 127 for symmetric codes, 255 for asymmetric ones).
// The reciprocal sequence q1 = fma(fma(-q0, d, y), r, q0), q0 = RN(y r), r = RN(1/d), stays
// within 2 ulp of the true quotient, and so does the IEEE quotient; the two can therefore round
// to different integers only if y / scale lies within a few ulp of a half-integer k + 1/2.
// This program visits, for every binary32 significand of the scale and every k in 0..255, all
// numerators within +-8 ulp of (k + 1/2) * scale and compares the two roundings.  (Exponents only
// shift both sides; negative numerators mirror the positive ones.)
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <omp.h>
static inline float mk(uint32_t b) { float f; memcpy(&f, &b, 4); return f; }
static inline uint32_t bits(float f) { uint32_t b; memcpy(&b, &f, 4); return b; }
int main() {
    long long bad = 0, quot_differs = 0;
#pragma omp parallel for schedule(dynamic, 4096) reduction(+ : bad, quot_differs)
    for (uint32_t ms = 0; ms < (1u << 23); ++ms) {
        const float d = mk(0x3f800000u | ms);  // scale in [1, 2)
        const float r = 1.0f / d;
        for (int k = 0; k < 256; ++k) {
            const float centre = ((float)k + 0.5f) * d;
            const uint32_t cb = bits(centre);
            for (int j = -8; j <= 8; ++j) {
                const float y = mk(cb + j);
                const float q0 = y * r;
                const float e = fmaf(-q0, d, y);
                const float q1 = fmaf(e, r, q0);
                const float q = y / d;
                if (q1 != q) ++quot_differs;
                if (rintf(q1) != rintf(q)) ++bad;
            }
        }
    }
    printf("rounding mismatches %lld (quotients that differ in the last place: %lld)\n", bad, quot_differs);
    return bad != 0;
}
