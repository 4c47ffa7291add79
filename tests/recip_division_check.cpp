// CPU check of the division shortcut used by the activation-quantisation kernel: with
// r = RN(1/s) and q0 = RN(x*r), q1 = fma(fma(-q0, s, x), r, q0) equals the IEEE quotient
// RN(x/s).  Exhaustive over every binary16 significand of x and every binary32
// significand of s (exponents only shift both sides as long as nothing under/overflows).
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <omp.h>
static inline float mk(uint32_t b) { float f; memcpy(&f, &b, 4); return f; }
int main() {
    long long bad = 0, allones_bad = 0;
#pragma omp parallel for schedule(dynamic, 1024) reduction(+ : bad, allones_bad)
    for (uint32_t ms = 0; ms < (1u << 23); ++ms) {
        const float s = mk(0x3f800000u | ms);  // [1, 2)
        const float r = 1.0f / s;
        for (uint32_t mx = 0; mx < 1024; ++mx) {
            const float x = mk(0x3f800000u | (mx << 13));
            const float q0 = x * r;
            const float e = fmaf(-q0, s, x);
            const float q1 = fmaf(e, r, q0);
            if (q1 != x / s) { ++bad; if (ms == 0x7fffff) ++allones_bad; }
        }
    }
    printf("mismatches %lld (with all-ones significand of s: %lld)\n", bad, allones_bad);
    return bad != 0;
}
