// CPU oracle for the smoothed W8A8 expert-FFN path of HAQ (arXiv 2508.07329).
//
// THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, loop-level
// statement of what the path computes, written from the paper's definitions and
// used only by the tests, by the smoke check and as the timed CPU baseline of the
// benchmark.  It shares no code with the HIP library and the HIP library never
// calls it.
//
// Arithmetic: IEEE binary32 with one rounding per written operation (build with
// -fno-fast-math -ffp-contract=off; fused multiply-adds appear only where fmaf is
// written), int32 accumulation, round-half-to-even everywhere.
//
// Orientation: the paper writes Y = W X with W [C_o x C_i] and X [C_i x tokens]
// (Section III.B.1, Eq. 1).  Here activations are X [T x K] (one token per row)
// and weights are W [K x N] (input channel major), i.e. the same operator
// transposed: Y = X W.
//
// Parity pins: every function below is pinned by tests/test_oracle_*.py
// (closed forms, brute force, invariants, numpy/fp64 cross-checks); none is
// "parity unpinned".
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>

#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

// ---------------------------------------------------------------- binary16
// IEEE binary16 <-> binary32 by bit manipulation (no compiler half type needed).

float half_to_float(uint16_t h) {
    const uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    const uint32_t exp = (h >> 10) & 0x1fu;
    const uint32_t man = h & 0x3ffu;
    uint32_t bits;
    if (exp == 0) {
        // zero or subnormal: value = man * 2^-24, exact in binary32
        float v = (float)man * 5.9604644775390625e-8f;  // 2^-24
        std::memcpy(&bits, &v, 4);
        bits |= sign;
    } else if (exp == 31) {
        bits = sign | 0x7f800000u | (man << 13);
    } else {
        bits = sign | ((exp + 112u) << 23) | (man << 13);
    }
    float f;
    std::memcpy(&f, &bits, 4);
    return f;
}

// Round-to-nearest-even; overflow goes to infinity (values >= 65520 in magnitude).
uint16_t float_to_half(float f) {
    uint32_t x;
    std::memcpy(&x, &f, 4);
    const uint16_t sign = (uint16_t)((x >> 16) & 0x8000u);
    x &= 0x7fffffffu;
    if (x >= 0x7f800000u) {  // inf / nan
        return (uint16_t)(sign | 0x7c00u | ((x > 0x7f800000u) ? 0x200u : 0u));
    }
    if (x >= 0x477ff000u) {  // >= 65520 rounds to infinity
        return (uint16_t)(sign | 0x7c00u);
    }
    if (x < 0x38800000u) {  // below 2^-14: result is a binary16 subnormal (or zero)
        float a;
        std::memcpy(&a, &x, 4);
        // a * 2^24 is exact; rintf rounds half to even in the default rounding mode
        const float m = std::rint(a * 16777216.0f);
        return (uint16_t)(sign | (uint16_t)m);  // m == 1024 is the smallest normal
    }
    const uint32_t man = x & 0x7fffffu;
    const uint32_t exp = (x >> 23) - 112u;
    uint32_t h = (exp << 10) | (man >> 13);
    const uint32_t rest = man & 0x1fffu;
    if (rest > 0x1000u || (rest == 0x1000u && (h & 1u))) h += 1;  // carry may bump the exponent
    return (uint16_t)(sign | h);
}

// ---------------------------------------------------------------- exp used by SiLU / softmax
// The path needs e^t in binary32 inside SiLU and the router softmax.  So that the
// int8 codes and gate weights that depend on it are decided by the same sequence
// of roundings on every implementation, e^t is DEFINED here as the following
// fixed sequence of IEEE operations (argument reduction by ln 2 in two parts,
// degree-7 Taylor polynomial in Horner form with fused multiply-adds, exact
// scaling by 2^n).  It is within 1 ulp of the true exponential on [-87, 88]; t is
// clamped to that interval (e^-87 < 2^-125 is absorbed by the "1 +" of SiLU and is
// far below one ulp of any softmax sum).
float exp_spec(float t) {
    t = std::fmin(std::fmax(t, -87.0f), 88.0f);
    const float n = std::rint(t * 1.44269502162933349609375f);        // log2(e) rounded to binary32
    float r = std::fmaf(n, -0.693145751953125f, t);                   // high part of ln 2 (exact product)
    r = std::fmaf(n, -1.42860682030941723212e-6f, r);  // low part of ln 2
    float p = 1.0f / 5040.0f;
    p = std::fmaf(p, r, 1.0f / 720.0f);
    p = std::fmaf(p, r, 1.0f / 120.0f);
    p = std::fmaf(p, r, 1.0f / 24.0f);
    p = std::fmaf(p, r, 1.0f / 6.0f);
    p = std::fmaf(p, r, 0.5f);
    p = std::fmaf(p, r, 1.0f);
    p = std::fmaf(p, r, 1.0f);
    const uint32_t sbits = (uint32_t)((int32_t)n + 127) << 23;  // 2^n, n in [-126, 127]
    float scale;
    std::memcpy(&scale, &sbits, 4);
    return p * scale;
}

inline float silu(float g) { return g / (1.0f + exp_spec(-g)); }

inline int8_t code_of(float y, float scale) {
    // y / scale in binary32, round half to even, saturate to the symmetric range
    float c = std::rint(y / scale);
    c = std::fmin(std::fmax(c, -127.0f), 127.0f);
    return (int8_t)c;
}

// One row of Eq. 1's Q(s^-1 X) with the scale on the token dimension
// (Section III.B.1, last paragraph): x/s per channel, scale = absmax/127,
// codes = rne((x/s)/scale) in [-127,127].  A zero row gives scale 0 and zero codes.
void quant_row(const float* xrow, const float* s, int K, int8_t* q, float* scale_out,
               std::vector<float>& y) {
    float a = 0.0f;
    for (int k = 0; k < K; ++k) {
        y[k] = s ? xrow[k] / s[k] : xrow[k];
        a = std::fmax(a, std::fabs(y[k]));
    }
    const float sc = a / 127.0f;
    *scale_out = sc;
    if (a == 0.0f) {
        for (int k = 0; k < K; ++k) q[k] = 0;
        return;
    }
    for (int k = 0; k < K; ++k) q[k] = code_of(y[k], sc);
}

// acc[n] = sum_k q[k] * Wq[k][n]  for one row; Wq is [K x N] row-major.
void int8_row_gemm(const int8_t* q, const int8_t* Wq, int K, int N, int32_t* acc) {
    for (int n = 0; n < N; ++n) acc[n] = 0;
    for (int k = 0; k < K; ++k) {
        const int32_t a = q[k];
        const int8_t* w = Wq + (size_t)k * N;
        for (int n = 0; n < N; ++n) acc[n] += a * (int32_t)w[n];
    }
}

inline float dequant(int32_t acc, float sx, float sw) { return ((float)acc * sx) * sw; }

}  // namespace

extern "C" {

int oracle_num_threads() {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_half_to_float(const uint16_t* h, int64_t n, float* f) {
    for (int64_t i = 0; i < n; ++i) f[i] = half_to_float(h[i]);
}
void oracle_float_to_half(const float* f, int64_t n, uint16_t* h) {
    for (int64_t i = 0; i < n; ++i) h[i] = float_to_half(f[i]);
}
void oracle_exp_spec(const float* t, int64_t n, float* out) {
    for (int64_t i = 0; i < n; ++i) out[i] = exp_spec(t[i]);
}

// Per-channel activation magnitude s_X (Eq. 3): ax[k] = max_t |X[t][k]|.
void oracle_col_absmax_f16(const uint16_t* X, int64_t ldx, int T, int K, float* ax) {
    for (int k = 0; k < K; ++k) ax[k] = 0.0f;
    for (int t = 0; t < T; ++t)
        for (int k = 0; k < K; ++k)
            ax[k] = std::fmax(ax[k], std::fabs(half_to_float(X[(size_t)t * ldx + k])));
}

// Per-input-channel weight magnitude: aw[k] = max_n |W[k][n]|; accumulates into aw
// (callers zero it) so several matrices that share one input can be folded in.
void oracle_row_absmax_f32(const float* W, int K, int N, float* aw) {
    for (int k = 0; k < K; ++k) {
        float a = aw[k];
        for (int n = 0; n < N; ++n) a = std::fmax(a, std::fabs(W[(size_t)k * N + n]));
        aw[k] = a;
    }
}

// Smoothing vector for a fixed exponent alpha (Eq. 3 with e = alpha; the weight
// term in the denominator is the SmoothQuant form the workloads prescribe):
// s_k = ax_k^alpha / aw_k^(1-alpha), evaluated in binary64, rounded once to
// binary32, clamped to [1e-5, 1e5]; s_k = 1 where either magnitude is zero.
// use_weight == 0 gives the paper's activation-only form s_k = ax_k^alpha.
void oracle_smoothing_vector(const float* ax, const float* aw, int K, double alpha, int use_weight, float* s) {
    for (int k = 0; k < K; ++k) {
        const double a = ax[k], w = use_weight ? (double)aw[k] : 1.0;
        if (a == 0.0 || w == 0.0) {
            s[k] = 1.0f;
            continue;
        }
        double v = std::pow(a, alpha) / std::pow(w, 1.0 - alpha);
        v = std::min(std::max(v, 1e-5), 1e5);
        s[k] = (float)v;
    }
}

// Q(s^-1 X), per-token scale (Eq. 1, activation operand).  s may be null (all ones).
void oracle_smooth_quant_act(const uint16_t* X, int64_t ldx, const float* s, int T, int K,
                             int8_t* q, int64_t ldq, float* row_scale) {
#pragma omp parallel
    {
        std::vector<float> xr(K), y(K);
#pragma omp for schedule(static)
        for (int t = 0; t < T; ++t) {
            for (int k = 0; k < K; ++k) xr[k] = half_to_float(X[(size_t)t * ldx + k]);
            quant_row(xr.data(), s, K, q + (size_t)t * ldq, &row_scale[t], y);
        }
    }
}

// Q(W s), per-output-channel scale (Eq. 1, weight operand; Algorithm 1 step 1
// folds s into the weight).  W fp32 [K x N]; s may be null.  A zero column gives
// scale 0 and zero codes.
void oracle_quant_weight(const float* W, const float* s, int K, int N, int8_t* Wq, float* col_scale) {
    std::vector<float> a(N, 0.0f);
    for (int k = 0; k < K; ++k) {
        const float sk = s ? s[k] : 1.0f;
        for (int n = 0; n < N; ++n) a[n] = std::fmax(a[n], std::fabs(sk * W[(size_t)k * N + n]));
    }
    for (int n = 0; n < N; ++n) col_scale[n] = a[n] / 127.0f;
#pragma omp parallel for schedule(static)
    for (int k = 0; k < K; ++k) {
        const float sk = s ? s[k] : 1.0f;
        for (int n = 0; n < N; ++n) {
            const float w = sk * W[(size_t)k * N + n];
            Wq[(size_t)k * N + n] = (a[n] == 0.0f) ? (int8_t)0 : code_of(w, col_scale[n]);
        }
    }
}

// acc[t][n] = sum_k q[t][k] * Wq[k][n], int32.
void oracle_gemm_i8(const int8_t* q, int64_t ldq, const int8_t* Wq, int T, int K, int N, int32_t* acc) {
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) int8_row_gemm(q + (size_t)t * ldq, Wq, K, N, acc + (size_t)t * N);
}

// Dequantise with the two outer-dimension scales, optional ReLU, round to binary16.
// act: 0 none, 1 ReLU.
void oracle_epilogue(const int32_t* acc, const float* sx, const float* sw, int T, int N, int act,
                     uint16_t* Y, int64_t ldy) {
    for (int t = 0; t < T; ++t)
        for (int n = 0; n < N; ++n) {
            float r = dequant(acc[(size_t)t * N + n], sx[t], sw[n]);
            if (act == 1) r = std::fmax(r, 0.0f);
            Y[(size_t)t * ldy + n] = float_to_half(r);
        }
}

// Router: top-2 experts by logit (lowest index wins ties) and their gate weights:
// softmax over all E experts with max subtraction, then renormalised over the two.
void oracle_route_top2(const uint16_t* logits, int64_t ldl, int T, int E, int32_t* idx, float* gw) {
    std::vector<float> l(E), p(E);
    for (int t = 0; t < T; ++t) {
        for (int e = 0; e < E; ++e) l[e] = half_to_float(logits[(size_t)t * ldl + e]);
        int i0 = 0;
        for (int e = 1; e < E; ++e)
            if (l[e] > l[i0]) i0 = e;
        int i1 = (i0 == 0) ? 1 : 0;
        for (int e = 0; e < E; ++e)
            if (e != i0 && l[e] > l[i1]) i1 = e;
        float z = 0.0f;
        for (int e = 0; e < E; ++e) {
            p[e] = exp_spec(l[e] - l[i0]);
            z += p[e];
        }
        const float p0 = p[i0] / z, p1 = p[i1] / z;
        const float d = p0 + p1;
        idx[2 * t] = i0;
        idx[2 * t + 1] = i1;
        gw[2 * t] = p0 / d;
        gw[2 * t + 1] = p1 / d;
    }
}

// Token permutation: pair r = 2t+k goes to expert idx[r]; counts per expert,
// exclusive offsets [E+1], perm = pair ids ordered by (expert, pair id), inv its inverse.
void oracle_permute(const int32_t* idx, int T, int E, int32_t* counts, int32_t* offsets, int32_t* perm,
                    int32_t* inv) {
    const int P = 2 * T;
    for (int e = 0; e < E; ++e) counts[e] = 0;
    for (int r = 0; r < P; ++r) counts[idx[r]]++;
    offsets[0] = 0;
    for (int e = 0; e < E; ++e) offsets[e + 1] = offsets[e] + counts[e];
    std::vector<int32_t> cursor(offsets, offsets + E);
    for (int r = 0; r < P; ++r) {
        const int pos = cursor[idx[r]]++;
        perm[pos] = r;
        inv[r] = pos;
    }
}

struct OracleExpert {
    const int8_t* w1;  // [H x I] int8, input channel major
    const int8_t* w3;  // [H x I]
    const int8_t* w2;  // [I x H]
    const float* sw1;  // [I]
    const float* sw3;  // [I]
    const float* sw2;  // [H]
    const float* s_mid;  // [I] smoothing vector of the down projection
};

// Top-2 routed SwiGLU expert FFN for the tokens listed in `tokens` (n_tok of them;
// null = all T tokens in order).  Per token: quantise once with s_in; per selected
// expert: gate/up int8 GEMMs, dequantise, h = fp16(silu(g) * u); requantise h with
// the expert's s_mid; down int8 GEMM, dequantise, y = fp16; out = fp16(g0*y0 + g1*y1).
// out is [n_tok x H] (row i belongs to tokens[i]).  Optional dumps (null to skip):
// mid [n_tok*2 x I] fp16, hq [n_tok*2 x I] int8, sh [n_tok*2], y [n_tok*2 x H] fp16,
// rows ordered by (token position in `tokens`, slot k).
void oracle_moe_ffn(const uint16_t* X, int64_t ldx, const int32_t* idx, const float* gw, const float* s_in,
                    const OracleExpert* experts, int T, int H, int I, const int32_t* tokens, int n_tok,
                    uint16_t* out, uint16_t* mid_dump, int8_t* hq_dump, float* sh_dump, uint16_t* y_dump) {
    (void)T;
#pragma omp parallel
    {
        std::vector<float> xr(H), ybuf(std::max(H, I)), hrow(I);
        std::vector<int8_t> q(H), hq(I);
        std::vector<int32_t> a1(I), a3(I), a2(H);
        std::vector<uint16_t> yh(2 * (size_t)H);
#pragma omp for schedule(dynamic, 1)
        for (int i = 0; i < n_tok; ++i) {
            const int t = tokens ? tokens[i] : i;
            for (int k = 0; k < H; ++k) xr[k] = half_to_float(X[(size_t)t * ldx + k]);
            float sx;
            quant_row(xr.data(), s_in, H, q.data(), &sx, ybuf);
            for (int k2 = 0; k2 < 2; ++k2) {
                const OracleExpert& ex = experts[idx[2 * t + k2]];
                int8_row_gemm(q.data(), ex.w1, H, I, a1.data());
                int8_row_gemm(q.data(), ex.w3, H, I, a3.data());
                for (int j = 0; j < I; ++j) {
                    const float g = dequant(a1[j], sx, ex.sw1[j]);
                    const float u = dequant(a3[j], sx, ex.sw3[j]);
                    const uint16_t hh = float_to_half(silu(g) * u);
                    if (mid_dump) mid_dump[((size_t)2 * i + k2) * I + j] = hh;
                    hrow[j] = half_to_float(hh);
                }
                float sh;
                quant_row(hrow.data(), ex.s_mid, I, hq.data(), &sh, ybuf);
                if (hq_dump) std::memcpy(hq_dump + ((size_t)2 * i + k2) * I, hq.data(), I);
                if (sh_dump) sh_dump[2 * i + k2] = sh;
                int8_row_gemm(hq.data(), ex.w2, I, H, a2.data());
                for (int n = 0; n < H; ++n) {
                    yh[(size_t)k2 * H + n] = float_to_half(dequant(a2[n], sh, ex.sw2[n]));
                    if (y_dump) y_dump[((size_t)2 * i + k2) * H + n] = yh[(size_t)k2 * H + n];
                }
            }
            const float g0 = gw[2 * t], g1 = gw[2 * t + 1];
            for (int n = 0; n < H; ++n) {
                const float v = g0 * half_to_float(yh[n]) + g1 * half_to_float(yh[(size_t)H + n]);
                out[(size_t)i * H + n] = float_to_half(v);
            }
        }
    }
}

// Per-expert activation magnitude of the down projection's input, used offline to
// build s_mid (Algorithm 1 step 1 collects the activations each layer sees): for
// each pair routed to expert e, h = fp16(silu(g) * u) from the quantised gate/up
// projections; ax_mid[e][j] = max over those pairs of |h_j|.
void oracle_moe_mid_absmax(const uint16_t* X, int64_t ldx, const int32_t* idx, const float* s_in,
                           const OracleExpert* experts, int T, int H, int I, int E, float* ax_mid) {
    for (size_t i = 0; i < (size_t)E * I; ++i) ax_mid[i] = 0.0f;
#pragma omp parallel
    {
        std::vector<float> xr(H), ybuf(H), mine((size_t)E * I, 0.0f);
        std::vector<int8_t> q(H);
        std::vector<int32_t> a1(I), a3(I);
#pragma omp for schedule(dynamic, 1)
        for (int t = 0; t < T; ++t) {
            for (int k = 0; k < H; ++k) xr[k] = half_to_float(X[(size_t)t * ldx + k]);
            float sx;
            quant_row(xr.data(), s_in, H, q.data(), &sx, ybuf);
            for (int k2 = 0; k2 < 2; ++k2) {
                const int e = idx[2 * t + k2];
                const OracleExpert& ex = experts[e];
                int8_row_gemm(q.data(), ex.w1, H, I, a1.data());
                int8_row_gemm(q.data(), ex.w3, H, I, a3.data());
                for (int j = 0; j < I; ++j) {
                    const float g = dequant(a1[j], sx, ex.sw1[j]);
                    const float u = dequant(a3[j], sx, ex.sw3[j]);
                    const float h = half_to_float(float_to_half(silu(g) * u));
                    float& m = mine[(size_t)e * I + j];
                    m = std::fmax(m, std::fabs(h));
                }
            }
        }
#pragma omp critical
        for (size_t i = 0; i < (size_t)E * I; ++i) ax_mid[i] = std::fmax(ax_mid[i], mine[i]);
    }
}

// ---- adaptive smoothing (Algorithm 1 step 1, Eq. 3) ---------------------------------------
// Full-precision product the quantised layer is compared with: Yref = X W with the binary16
// activations and binary32 weights taken as exact numbers, products and sums in binary64
// (k ascending).  X [T x K], W [K x N], Yref [T x N].
void oracle_matmul_f64(const uint16_t* X, int64_t ldx, const float* W, int T, int K, int N, double* Yref) {
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        double* y = Yref + (size_t)t * N;
        for (int n = 0; n < N; ++n) y[n] = 0.0;
        for (int k = 0; k < K; ++k) {
            const double x = (double)half_to_float(X[(size_t)t * ldx + k]);
            const float* w = W + (size_t)k * N;
            for (int n = 0; n < N; ++n) y[n] += x * (double)w[n];
        }
    }
}

// Quantisation loss of one candidate: mean over all T*N outputs of (Y - Yref)^2, the binary16
// outputs of the quantised layer against the full-precision product, in binary64 (row sums
// first, then the rows in order).
double oracle_mse_f64(const uint16_t* Y, int64_t ldy, const double* Yref, int T, int N) {
    double total = 0.0;
    for (int t = 0; t < T; ++t) {
        double row = 0.0;
        for (int n = 0; n < N; ++n) {
            const double d = (double)half_to_float(Y[(size_t)t * ldy + n]) - Yref[(size_t)t * N + n];
            row += d * d;
        }
        total += row;
    }
    return total / ((double)T * (double)N);
}

// ---- Hessian-aware weight quantisation (Section III.B.2, Eq. 4-6; Algorithm 1 step 2) ---------
// Everything here is binary64 and every sum has a stated order, so that an implementation
// that performs the same operations gets the same bits.
//
// H = 2 Xs^T Xs over the calibration rows, Xs = X / s (the smoothed activations the layer
// will see; the division is the binary32 one of the activation path), sums over the tokens
// in ascending order with one fused multiply-add per term.  A channel that never fires
// (H_jj = 0) gets H_jj = 1.  Damping: percdamp times the mean of the diagonal (summed in
// index order) is added to the diagonal, the usual safeguard for the inversion.
void oracle_hessian(const uint16_t* X, int64_t ldx, const float* s, int T, int K, double percdamp, double* H) {
    std::vector<double> xs((size_t)T * K);
    for (int t = 0; t < T; ++t)
        for (int k = 0; k < K; ++k) {
            const float x = half_to_float(X[(size_t)t * ldx + k]);
            xs[(size_t)t * K + k] = (double)(s ? x / s[k] : x);
        }
#pragma omp parallel for schedule(dynamic, 8)
    for (int j = 0; j < K; ++j)
        for (int l = 0; l < K; ++l) {
            double acc = 0.0;
            for (int t = 0; t < T; ++t) acc = std::fma(xs[(size_t)t * K + j], xs[(size_t)t * K + l], acc);
            H[(size_t)j * K + l] = 2.0 * acc;
        }
    for (int j = 0; j < K; ++j)
        if (H[(size_t)j * K + j] == 0.0) H[(size_t)j * K + j] = 1.0;
    double tr = 0.0;
    for (int j = 0; j < K; ++j) tr += H[(size_t)j * K + j];
    const double damp = percdamp * (tr / (double)K);
    for (int j = 0; j < K; ++j) H[(size_t)j * K + j] += damp;
}

// U upper triangular with H^-1 = U^T U (the Cholesky reformulation: row i of U is, up to the
// factor U_ii, row i of the inverse Hessian of the channels not yet quantised, i.e. what
// Eq. 5-6 need at step i).  Route: flip H (reverse both index orders), Cholesky-factorise
// the flipped matrix, A = L L^T, invert the triangle, M = L^-1, and flip back: U = flip(M).
//   L_jj = sqrt(a_jj - sum_{k<j} L_jk^2),  L_ij = (a_ij - sum_{k<j} L_ik L_jk) / L_jj,
//   M_jj = 1 / L_jj,  M_ij = -(sum_{j<=k<i} L_ik M_kj) / L_ii,
// every sum accumulated from the leading term with one fused multiply-add per k ascending.
// Returns 0, or j + 1 if the pivot of column j is not positive.
int oracle_inverse_cholesky_upper(const double* H, int K, double* U) {
    std::vector<double> L((size_t)K * K, 0.0), M((size_t)K * K, 0.0);
    auto A = [&](int i, int j) { return H[(size_t)(K - 1 - i) * K + (K - 1 - j)]; };
    for (int j = 0; j < K; ++j) {
        double d = A(j, j);
        for (int k = 0; k < j; ++k) d = std::fma(-L[(size_t)j * K + k], L[(size_t)j * K + k], d);
        if (!(d > 0.0)) return j + 1;
        const double ljj = std::sqrt(d);
        L[(size_t)j * K + j] = ljj;
#pragma omp parallel for schedule(static)
        for (int i = j + 1; i < K; ++i) {
            double v = A(i, j);
            for (int k = 0; k < j; ++k) v = std::fma(-L[(size_t)i * K + k], L[(size_t)j * K + k], v);
            L[(size_t)i * K + j] = v / ljj;
        }
    }
#pragma omp parallel for schedule(dynamic, 8)
    for (int j = 0; j < K; ++j) {
        M[(size_t)j * K + j] = 1.0 / L[(size_t)j * K + j];
        for (int i = j + 1; i < K; ++i) {
            double v = 0.0;
            for (int k = j; k < i; ++k) v = std::fma(-L[(size_t)i * K + k], M[(size_t)k * K + j], v);
            M[(size_t)i * K + j] = v / L[(size_t)i * K + i];
        }
    }
    for (int a = 0; a < K; ++a)
        for (int b = 0; b < K; ++b) U[(size_t)a * K + b] = M[(size_t)(K - 1 - a) * K + (K - 1 - b)];
    return 0;
}

// Input channels in order (Section III.B.2 steps 1-3).  The per-output-channel grid is the
// one of plain rounding, scale_n = max_k |s_k W_kn| / 127 in binary32; the working copy of
// the folded weight is binary64.  Channel i: code = clamp(rne(w_in / scale_n)), the error
// e_n = (w_in - code * scale_n) / U_ii, and every later channel j > i is compensated,
// w_jn <- w_jn - e_n U_ij (one fused multiply-add): Eq. 6 with row i of the remaining
// inverse Hessian written through U.  Output channels are independent of each other.
void oracle_gptq(const float* W, const float* s, const double* U, int K, int N, int8_t* Wq, float* col_scale) {
    std::vector<float> a(N, 0.0f);
    for (int k = 0; k < K; ++k) {
        const float sk = s ? s[k] : 1.0f;
        for (int n = 0; n < N; ++n) a[n] = std::fmax(a[n], std::fabs(sk * W[(size_t)k * N + n]));
    }
    for (int n = 0; n < N; ++n) col_scale[n] = a[n] / 127.0f;
#pragma omp parallel
    {
        std::vector<double> w(K);
#pragma omp for schedule(static)
        for (int n = 0; n < N; ++n) {
            for (int k = 0; k < K; ++k) w[k] = (double)((s ? s[k] : 1.0f) * W[(size_t)k * N + n]);
            const double scale = (double)col_scale[n];
            for (int i = 0; i < K; ++i) {
                double code = 0.0;
                if (a[n] != 0.0f) {
                    code = std::nearbyint(w[i] / scale);
                    code = std::fmin(std::fmax(code, -127.0), 127.0);
                }
                Wq[(size_t)i * N + n] = (int8_t)code;
                const double err = (w[i] - code * scale) / U[(size_t)i * K + i];
                for (int j = i + 1; j < K; ++j) w[j] = std::fma(-err, U[(size_t)i * K + j], w[j]);
            }
        }
    }
}

// ---- asymmetric activations (Section IV.A names asymmetric quantisation as the default) --------
// Per token: y = x / s, the range [mn, mx] of the row widened to contain 0, scale = (mx - mn) / 255,
// zero point zp = clamp(rne(-mn / scale), 0, 255), codes q = clamp(rne(y / scale) + zp, 0, 255),
// all in binary32; y is represented by (q - zp) * scale.  A row with mx = mn (= 0) gives scale 0,
// zp 0 and zero codes.  The weight operand stays symmetric per output channel.
void oracle_asym_quant_act(const uint16_t* X, int64_t ldx, const float* s, int T, int K, uint8_t* q, int64_t ldq,
                           float* row_scale, int32_t* row_zp) {
#pragma omp parallel
    {
        std::vector<float> y(K);
#pragma omp for schedule(static)
        for (int t = 0; t < T; ++t) {
            float mn = 0.0f, mx = 0.0f;
            for (int k = 0; k < K; ++k) {
                const float x = half_to_float(X[(size_t)t * ldx + k]);
                y[k] = s ? x / s[k] : x;
                mn = std::fmin(mn, y[k]);
                mx = std::fmax(mx, y[k]);
            }
            const float range = mx - mn;
            uint8_t* qr = q + (size_t)t * ldq;
            if (range == 0.0f) {
                row_scale[t] = 0.0f;
                row_zp[t] = 0;
                for (int k = 0; k < K; ++k) qr[k] = 0;
                continue;
            }
            const float sc = range / 255.0f;
            float z = std::rint(-mn / sc);
            z = std::fmin(std::fmax(z, 0.0f), 255.0f);
            row_scale[t] = sc;
            row_zp[t] = (int32_t)z;
            for (int k = 0; k < K; ++k) {
                float c = std::rint(y[k] / sc) + z;
                c = std::fmin(std::fmax(c, 0.0f), 255.0f);
                qr[k] = (uint8_t)c;
            }
        }
    }
}

// acc[t][n] = sum_k (q[t][k] - zp[t]) * Wq[k][n], int32.
void oracle_asym_gemm(const uint8_t* q, int64_t ldq, const int32_t* zp, const int8_t* Wq, int T, int K, int N, int32_t* acc) {
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        int32_t* a = acc + (size_t)t * N;
        for (int n = 0; n < N; ++n) a[n] = 0;
        for (int k = 0; k < K; ++k) {
            const int32_t v = (int32_t)q[(size_t)t * ldq + k] - zp[t];
            const int8_t* w = Wq + (size_t)k * N;
            for (int n = 0; n < N; ++n) a[n] += v * (int32_t)w[n];
        }
    }
}


// ---- asymmetric activation codes inside the routed expert FFN ---------------------------------
// One row of the asymmetric quantiser above (same arithmetic), on binary32 inputs.
static void asym_quant_row(const float* xrow, const float* s, int K, uint8_t* q, float* scale_out, int32_t* zp_out,
                           std::vector<float>& y) {
    float mn = 0.0f, mx = 0.0f;
    for (int k = 0; k < K; ++k) {
        y[k] = s ? xrow[k] / s[k] : xrow[k];
        mn = std::fmin(mn, y[k]);
        mx = std::fmax(mx, y[k]);
    }
    const float range = mx - mn;
    if (range == 0.0f) {
        *scale_out = 0.0f;
        *zp_out = 0;
        for (int k = 0; k < K; ++k) q[k] = 0;
        return;
    }
    const float sc = range / 255.0f;
    float z = std::rint(-mn / sc);
    z = std::fmin(std::fmax(z, 0.0f), 255.0f);
    *scale_out = sc;
    *zp_out = (int32_t)z;
    for (int k = 0; k < K; ++k) {
        float c = std::rint(y[k] / sc) + z;
        c = std::fmin(std::fmax(c, 0.0f), 255.0f);
        q[k] = (uint8_t)c;
    }
}

// acc[n] = sum_k (q[k] - zp) * Wq[k][n] for one row.
static void asym_row_gemm(const uint8_t* q, int32_t zp, const int8_t* Wq, int K, int N, int32_t* acc) {
    for (int n = 0; n < N; ++n) acc[n] = 0;
    for (int k = 0; k < K; ++k) {
        const int32_t a = (int32_t)q[k] - zp;
        const int8_t* w = Wq + (size_t)k * N;
        for (int n = 0; n < N; ++n) acc[n] += a * (int32_t)w[n];
    }
}

// The routed expert FFN of oracle_moe_ffn with asymmetric activation codes (Section IV.A names
// asymmetric quantisation as the default of the experiments): the token is quantised once with
// s_in to (q, scale, zero point); per selected expert the gate/up accumulators are sums of
// (q - zp) * w, h = fp16(silu(g) * u) as before, h is requantised asymmetrically with the
// expert's s_mid, the down accumulator is the sum of (hq - zh) * w2, and everything after the
// accumulators (dequantisation with the outer-dimension scales, fp16 rounding, combination) is
// unchanged.  Weights stay symmetric per output channel.  Dumps as in oracle_moe_ffn, plus the
// zero points of the requantised intermediate.
void oracle_moe_ffn_asym(const uint16_t* X, int64_t ldx, const int32_t* idx, const float* gw, const float* s_in,
                         const OracleExpert* experts, int T, int H, int I, const int32_t* tokens, int n_tok,
                         uint16_t* out, uint16_t* mid_dump, uint8_t* hq_dump, float* sh_dump, int32_t* zh_dump,
                         uint16_t* y_dump) {
    (void)T;
#pragma omp parallel
    {
        std::vector<float> xr(H), ybuf(std::max(H, I)), hrow(I);
        std::vector<uint8_t> q(H), hq(I);
        std::vector<int32_t> a1(I), a3(I), a2(H);
        std::vector<uint16_t> yh(2 * (size_t)H);
#pragma omp for schedule(dynamic, 1)
        for (int i = 0; i < n_tok; ++i) {
            const int t = tokens ? tokens[i] : i;
            for (int k = 0; k < H; ++k) xr[k] = half_to_float(X[(size_t)t * ldx + k]);
            float sx;
            int32_t zx;
            asym_quant_row(xr.data(), s_in, H, q.data(), &sx, &zx, ybuf);
            for (int k2 = 0; k2 < 2; ++k2) {
                const OracleExpert& ex = experts[idx[2 * t + k2]];
                asym_row_gemm(q.data(), zx, ex.w1, H, I, a1.data());
                asym_row_gemm(q.data(), zx, ex.w3, H, I, a3.data());
                for (int j = 0; j < I; ++j) {
                    const float g = dequant(a1[j], sx, ex.sw1[j]);
                    const float u = dequant(a3[j], sx, ex.sw3[j]);
                    const uint16_t hh = float_to_half(silu(g) * u);
                    if (mid_dump) mid_dump[((size_t)2 * i + k2) * I + j] = hh;
                    hrow[j] = half_to_float(hh);
                }
                float sh;
                int32_t zh;
                asym_quant_row(hrow.data(), ex.s_mid, I, hq.data(), &sh, &zh, ybuf);
                if (hq_dump) std::memcpy(hq_dump + ((size_t)2 * i + k2) * I, hq.data(), I);
                if (sh_dump) sh_dump[2 * i + k2] = sh;
                if (zh_dump) zh_dump[2 * i + k2] = zh;
                asym_row_gemm(hq.data(), zh, ex.w2, I, H, a2.data());
                for (int n = 0; n < H; ++n) {
                    yh[(size_t)k2 * H + n] = float_to_half(dequant(a2[n], sh, ex.sw2[n]));
                    if (y_dump) y_dump[((size_t)2 * i + k2) * H + n] = yh[(size_t)k2 * H + n];
                }
            }
            const float g0 = gw[2 * t], g1 = gw[2 * t + 1];
            for (int n = 0; n < H; ++n) {
                const float v = g0 * half_to_float(yh[n]) + g1 * half_to_float(yh[(size_t)H + n]);
                out[(size_t)i * H + n] = float_to_half(v);
            }
        }
    }
}

// ---- the CPU side of the heterogeneous deployment (Section III.B.3; Algorithm 1 step 3, CPU
// branch; Section III.C.1a, option A) ---------------------------------------------------------
// On the CPU an expert's int8 weights are dequantised once, when the model is loaded, to a
// floating-point copy that stays cached in host memory; an expert that the offload policy
// decides to compute on the CPU then runs in floating point on that copy, and only its output
// rows travel to the GPU.  Reading taken here: the cached copy is binary32,
// Wf[k][n] = float(code[k][n]) * scale[n] (one multiplication); the activations are not
// quantised on this side but carry the same smoothing, xs = x / s (binary32 division); every
// inner product is one binary32 accumulator started at 0 that takes the terms in ascending k
// with one fused multiply-add each; SiLU and the binary16 roundings of the intermediate and of
// the output are those of the int8 path.
void oracle_dequant_weight(const int8_t* Wq, const float* col_scale, int K, int N, float* Wf) {
    for (int k = 0; k < K; ++k)
        for (int n = 0; n < N; ++n) Wf[(size_t)k * N + n] = (float)Wq[(size_t)k * N + n] * col_scale[n];
}

// Y[t][n] = sum_k (X[t][k] / s[k]) * Wf[k][n], binary32, k ascending, fused multiply-adds.
// X is binary32 here (the caller converts binary16 exactly); s may be null.
void oracle_fp_linear(const float* X, int64_t ldx, const float* s, const float* Wf, int T, int K, int N, float* Y) {
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        float* y = Y + (size_t)t * N;
        for (int n = 0; n < N; ++n) y[n] = 0.0f;
        for (int k = 0; k < K; ++k) {
            const float x = X[(size_t)t * ldx + k];
            const float xs = s ? x / s[k] : x;
            const float* w = Wf + (size_t)k * N;
            for (int n = 0; n < N; ++n) y[n] = std::fmaf(xs, w[n], y[n]);
        }
    }
}

// One SwiGLU expert on the CPU's floating-point copy for n_rows token rows (fp16 in, fp16 out):
// g = (x / s_in) W1f, u = (x / s_in) W3f, h = fp16(silu(g) * u), y = fp16((h / s_mid) W2f).
// Optional dump of h (null to skip).
void oracle_cpu_expert_ffn(const uint16_t* X, int64_t ldx, const float* s_in, const float* W1f, const float* W3f,
                           const float* W2f, const float* s_mid, int n_rows, int H, int I, uint16_t* Y, int64_t ldy,
                           uint16_t* mid_dump) {
    std::vector<float> xf((size_t)n_rows * H), g((size_t)n_rows * I), u((size_t)n_rows * I), hf((size_t)n_rows * I),
        y((size_t)n_rows * H);
    for (int t = 0; t < n_rows; ++t)
        for (int k = 0; k < H; ++k) xf[(size_t)t * H + k] = half_to_float(X[(size_t)t * ldx + k]);
    oracle_fp_linear(xf.data(), H, s_in, W1f, n_rows, H, I, g.data());
    oracle_fp_linear(xf.data(), H, s_in, W3f, n_rows, H, I, u.data());
    for (size_t i = 0; i < (size_t)n_rows * I; ++i) {
        const uint16_t hh = float_to_half(silu(g[i]) * u[i]);
        if (mid_dump) mid_dump[i] = hh;
        hf[i] = half_to_float(hh);
    }
    oracle_fp_linear(hf.data(), I, s_mid, W2f, n_rows, I, H, y.data());
    for (int t = 0; t < n_rows; ++t)
        for (int n = 0; n < H; ++n) Y[(size_t)t * ldy + n] = float_to_half(y[(size_t)t * H + n]);
}

// out[t] = fp16(g0 * y[2t] + g1 * y[2t+1]): the weighted combination at the end of the expert
// FFN as a step of its own (y holds the two expert outputs of every token, pair order).
void oracle_combine(const uint16_t* y, const float* gw, int T, int H, uint16_t* out) {
    for (int t = 0; t < T; ++t)
        for (int n = 0; n < H; ++n) {
            const float v = gw[2 * t] * half_to_float(y[((size_t)2 * t) * H + n]) +
                            gw[2 * t + 1] * half_to_float(y[((size_t)2 * t + 1) * H + n]);
            out[(size_t)t * H + n] = float_to_half(v);
        }
}

}  // extern "C"
