// The CPU side of the heterogeneous deployment (Section III.B.3; Algorithm 1 step 3, CPU branch;
// Section III.C.1a, option A).  An expert that lives in host memory keeps, next to its int8 codes,
// a floating-point copy that is produced once when the expert is loaded: Wf = float(code) * scale.
// (A second storage mode keeps only the codes and forms the very same Wf inside the inner loop: the
// expert is bound by host memory bandwidth, and the codes are a quarter of the bytes.)
// When the offload policy decides that moving the expert to the GPU does not pay (Eq. 7-8), its
// token rows are computed here, in floating point on that copy, and only the output rows travel
// to the GPU.  This is host code: nothing in this file touches the device.
//
// Arithmetic (what the path is defined to compute, so that it is reproducible bit for bit):
//   xs = x / s_in (binary32);  g = xs W1f, u = xs W3f;  h = fp16(silu(g) * u);
//   y = fp16((h / s_mid) W2f);
// every inner product is one binary32 accumulator that starts at 0 and takes its terms in
// ascending input-channel order, one fused multiply-add each; silu and e^t are those of the
// int8 path.  Outputs are independent of the thread count: threads split the output channels.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include <system_error>
#include <thread>
#include <vector>

#include "haq_common.h"
#if defined(__x86_64__) && defined(__AVX2__) && defined(__FMA__) && !defined(__HIP_DEVICE_COMPILE__)
#include <immintrin.h>
#define HAQ_CPU_AVX2 1
#endif

struct haq_cpu_expert {
    int H = 0, I = 0;
    bool codes = false;                       // false: binary32 copies below; true: the int8 codes and their scales
    std::vector<float> w1f, w3f, w2f, s_mid;  // [H x I], [H x I], [I x H], [I]
    std::vector<int8_t> w1q, w3q, w2q;
    std::vector<float> sw1, sw3, sw2;
};

namespace haq {
namespace {

// binary16 -> binary32 (exact): re-bias the exponent; subnormals are normalised by a multiplication
float h2f_host(uint16_t h) {
    const uint32_t sign = (uint32_t)(h >> 15) << 31, em = h & 0x7fffu;
    uint32_t bits;
    float f;
    if (em >= 0x7c00u) {
        bits = sign | 0x7f800000u | ((em & 0x3ffu) << 13);
    } else if (em >= 0x0400u) {
        bits = sign | ((em << 13) + (112u << 23));
    } else {
        const float v = (float)em * 0x1p-24f;
        memcpy(&bits, &v, 4);
        bits |= sign;
    }
    memcpy(&f, &bits, 4);
    return f;
}

// binary32 -> binary16, round to nearest even; magnitudes from 65520 on become infinity
uint16_t f2h_host(float f) {
    uint32_t x;
    memcpy(&x, &f, 4);
    const uint16_t sign = (uint16_t)((x >> 16) & 0x8000u);
    const uint32_t a = x & 0x7fffffffu;
    if (a > 0x7f800000u) return (uint16_t)(sign | 0x7e00u);
    if (a >= 0x477ff000u) return (uint16_t)(sign | 0x7c00u);  // 65520 and beyond (and infinity)
    float m;
    memcpy(&m, &a, 4);
    if (a < 0x38800000u) {  // below 2^-14: a multiple of 2^-24 (binary16 subnormal, or zero)
        const float r = m * 0x1p24f;               // exact
        const float k = std::nearbyint(r);         // ties to even
        return (uint16_t)(sign | (uint16_t)k);     // 1024 is the smallest normal
    }
    const uint32_t e = (a >> 23) - 112u, man = a & 0x7fffffu;
    uint32_t h = (e << 10) | (man >> 13);
    const uint32_t rest = man & 0x1fffu;
    h += (rest > 0x1000u) | ((rest == 0x1000u) & (h & 1u));
    return (uint16_t)(sign | h);
}

// e^t by the fixed binary32 sequence that defines it on this path (clamp, n = rne(t log2 e), two-part
// ln 2 reduction, degree-7 Horner with fused multiply-adds, exact scaling by 2^n)
float exp_host(float t) {
    t = std::fmin(std::fmax(t, -87.0f), 88.0f);
    const float n = std::nearbyint(t * 1.44269502162933349609375f);
    float r = std::fmaf(n, -0.693145751953125f, t);
    r = std::fmaf(n, -1.42860682030941723212e-6f, r);
    const float c[7] = {1.0f / 720.0f, 1.0f / 120.0f, 1.0f / 24.0f, 1.0f / 6.0f, 0.5f, 1.0f, 1.0f};
    float p = 1.0f / 5040.0f;
    for (float ci : c) p = std::fmaf(p, r, ci);
    const uint32_t sb = (uint32_t)((int32_t)n + 127) << 23;
    float scale;
    memcpy(&scale, &sb, 4);
    return p * scale;
}

// y[r][n] = sum_k xs[r][k] W[k][n] for the output channels [n0, n1): k ascending, one fused
// multiply-add per term; up to RB rows share one pass over the weight slice
constexpr int RB = 4;
void linear_slice(const float* xs, int R, int K, const float* W, int N, int n0, int n1, float* y) {
    for (int r0 = 0; r0 < R; r0 += RB) {
        const int rb = std::min(RB, R - r0);
        for (int r = 0; r < rb; ++r) std::fill(y + (size_t)(r0 + r) * N + n0, y + (size_t)(r0 + r) * N + n1, 0.0f);
        for (int k = 0; k < K; ++k) {
            const float* w = W + (size_t)k * N;
            for (int r = 0; r < rb; ++r) {
                const float x = xs[(size_t)(r0 + r) * K + k];
                float* yr = y + (size_t)(r0 + r) * N;
                for (int n = n0; n < n1; ++n) yr[n] = std::fmaf(x, w[n], yr[n]);
            }
        }
    }
}

// Codes mode.  The codes are kept in blocks of eight output channels, [N/8][K][8], so that a thread that owns a
// range of channel blocks reads one contiguous stream.  y[r][n] = sum_k xs[r][k] * (float(code[k][n]) * sc[n]):
// the weight is formed on the spot exactly as in the binary32 copy (the conversion is exact, the product rounds
// once), and every output keeps its own accumulator with k ascending and one fused multiply-add per term, so the
// values are those of linear_slice.  NB channel blocks and up to RB rows are in flight together.
template <int RBK, int NB>
void blocked_tile(const float* xs, int K, const int8_t* Qb, const float* sc, int N, int nb, float* y) {
#ifdef HAQ_CPU_AVX2
    __m256 acc[RBK][NB], scv[NB];
    const int8_t* q[NB];
    for (int b = 0; b < NB; ++b) {
        scv[b] = _mm256_loadu_ps(sc + (size_t)(nb + b) * 8);
        q[b] = Qb + (size_t)(nb + b) * K * 8;
        for (int r = 0; r < RBK; ++r) acc[r][b] = _mm256_setzero_ps();
    }
    for (int k = 0; k < K; ++k) {
        __m256 w[NB];
        for (int b = 0; b < NB; ++b)
            w[b] = _mm256_mul_ps(_mm256_cvtepi32_ps(_mm256_cvtepi8_epi32(_mm_loadl_epi64(reinterpret_cast<const __m128i*>(q[b] + (size_t)k * 8)))), scv[b]);
        for (int r = 0; r < RBK; ++r) {
            const __m256 xv = _mm256_broadcast_ss(xs + (size_t)r * K + k);
            for (int b = 0; b < NB; ++b) acc[r][b] = _mm256_fmadd_ps(xv, w[b], acc[r][b]);
        }
    }
    for (int r = 0; r < RBK; ++r)
        for (int b = 0; b < NB; ++b) _mm256_storeu_ps(y + (size_t)r * N + (size_t)(nb + b) * 8, acc[r][b]);
#else
    for (int b = 0; b < NB; ++b) {
        const int8_t* q = Qb + (size_t)(nb + b) * K * 8;
        for (int r = 0; r < RBK; ++r) {
            float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
            for (int k = 0; k < K; ++k) {
                const float x = xs[(size_t)r * K + k];
                for (int j = 0; j < 8; ++j) acc[j] = std::fmaf(x, (float)q[(size_t)k * 8 + j] * sc[(size_t)(nb + b) * 8 + j], acc[j]);
            }
            for (int j = 0; j < 8; ++j) y[(size_t)r * N + (size_t)(nb + b) * 8 + j] = acc[j];
        }
    }
#endif
}

template <int RBK>
void blocked_rows(const float* xs, int K, const int8_t* Qb, const float* sc, int N, int nb0, int nb1, float* y) {
    constexpr int NB = RBK == 1 ? 4 : 2;
    int nb = nb0;
    for (; nb + NB <= nb1; nb += NB) blocked_tile<RBK, NB>(xs, K, Qb, sc, N, nb, y);
    for (; nb < nb1; ++nb) blocked_tile<RBK, 1>(xs, K, Qb, sc, N, nb, y);
}

// channel blocks [nb0, nb1) of y = xs W for R rows
void linear_slice_codes(const float* xs, int R, int K, const int8_t* Qb, const float* sc, int N, int nb0, int nb1, float* y) {
    for (int r0 = 0; r0 < R; r0 += RB) {
        const int rb = std::min(RB, R - r0);
        const float* x = xs + (size_t)r0 * K;
        float* yr = y + (size_t)r0 * N;
        switch (rb) {
            case 1: blocked_rows<1>(x, K, Qb, sc, N, nb0, nb1, yr); break;
            case 2: blocked_rows<2>(x, K, Qb, sc, N, nb0, nb1, yr); break;
            case 3: blocked_rows<3>(x, K, Qb, sc, N, nb0, nb1, yr); break;
            default: blocked_rows<4>(x, K, Qb, sc, N, nb0, nb1, yr); break;
        }
    }
}

// W: binary32 weights [K x N], or null with the blocked codes Qb and their scales sc
void linear_mt(const float* xs, int R, int K, const float* W, const int8_t* Qb, const float* sc, int N, float* y, int n_threads) {
    const int nt = std::max(1, std::min(n_threads, N / 64));
    auto slice = [=](int n0, int n1) {
        if (W)
            linear_slice(xs, R, K, W, N, n0, n1, y);
        else
            linear_slice_codes(xs, R, K, Qb, sc, N, n0 / 8, n1 / 8, y);
    };
    if (nt == 1) {
        slice(0, N);
        return;
    }
    std::vector<std::thread> th;
    th.reserve((size_t)nt);
    const int per = ((N + nt - 1) / nt + 15) / 16 * 16;
    try {
        for (int t = 0; t < nt; ++t) {
            const int n0 = std::min(N, t * per), n1 = std::min(N, n0 + per);
            if (n0 < n1) th.emplace_back(slice, n0, n1);
        }
    } catch (...) {  // a worker could not be started: finish the ones that were, then report
        for (auto& t : th) t.join();
        throw;
    }
    for (auto& t : th) t.join();
}

}  // namespace
}  // namespace haq

using namespace haq;

extern "C" {

int32_t haq_cpu_expert_create(const int8_t* w1q, const int8_t* w3q, const int8_t* w2q, const float* sw1, const float* sw3,
                              const float* sw2, const float* s_mid, int32_t H, int32_t I, int32_t keep_codes, haq_cpu_expert** out) {
    if (!out) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_cpu_expert_create: null output");
    *out = nullptr;
    if (H <= 0 || I <= 0) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_cpu_expert_create: H=%d I=%d", H, I);
    if (!w1q || !w3q || !w2q || !sw1 || !sw3 || !sw2 || !s_mid) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_cpu_expert_create: null buffer");
    haq_cpu_expert* e = nullptr;
    try {
        e = new haq_cpu_expert();
        e->H = H;
        e->I = I;
        e->codes = keep_codes != 0;
        e->s_mid.assign(s_mid, s_mid + I);
        if (e->codes) {
            if (H % 8 != 0 || I % 8 != 0) {
                delete e;
                HAQ_FAIL(HAQ_ERR_UNSUPPORTED, "haq_cpu_expert_create: keep_codes needs H=%d and I=%d to be multiples of 8", H, I);
            }
            // [K x N] row-major -> blocks of eight output channels [N/8][K][8]
            auto block = [](const int8_t* q, int K, int N, std::vector<int8_t>& out) {
                out.resize((size_t)K * N);
                for (int nb = 0; nb < N / 8; ++nb)
                    for (int k = 0; k < K; ++k) memcpy(out.data() + ((size_t)nb * K + k) * 8, q + (size_t)k * N + (size_t)nb * 8, 8);
            };
            block(w1q, H, I, e->w1q);
            block(w3q, H, I, e->w3q);
            block(w2q, I, H, e->w2q);
            e->sw1.assign(sw1, sw1 + I);
            e->sw3.assign(sw3, sw3 + I);
            e->sw2.assign(sw2, sw2 + H);
        } else {
            e->w1f.resize((size_t)H * I);
            e->w3f.resize((size_t)H * I);
            e->w2f.resize((size_t)I * H);
        }
    } catch (const std::bad_alloc&) {
        delete e;
        HAQ_FAIL(HAQ_ERR_HIP, "haq_cpu_expert_create: out of host memory");
    }
    if (e->codes) {
        *out = e;
        return HAQ_OK;
    }
    // the one-time dequantisation: float(code) * scale of the output channel
    auto deq = [](const int8_t* q, const float* sc, int K, int N, float* f) {
        for (int k = 0; k < K; ++k)
            for (int n = 0; n < N; ++n) f[(size_t)k * N + n] = (float)q[(size_t)k * N + n] * sc[n];
    };
    deq(w1q, sw1, H, I, e->w1f.data());
    deq(w3q, sw3, H, I, e->w3f.data());
    deq(w2q, sw2, I, H, e->w2f.data());
    *out = e;
    return HAQ_OK;
}

int32_t haq_cpu_expert_destroy(haq_cpu_expert* e) {
    delete e;
    return HAQ_OK;
}

int32_t haq_cpu_expert_ffn(const haq_cpu_expert* e, const void* x_fp16, int64_t ldx, const float* s_in, int32_t n_rows,
                           void* y_fp16, int64_t ldy, int32_t n_threads) {
    if (!e) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_cpu_expert_ffn: null expert");
    if (n_rows < 0 || ldx < e->H || ldy < e->H) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_cpu_expert_ffn: n_rows=%d ldx=%lld ldy=%lld", n_rows, (long long)ldx, (long long)ldy);
    if (n_rows == 0) return HAQ_OK;
    if (!x_fp16 || !y_fp16) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_cpu_expert_ffn: null buffer");
    const int H = e->H, I = e->I;
    int nt = n_threads > 0 ? n_threads : (int)std::thread::hardware_concurrency();
    nt = std::max(1, std::min(nt, 64));
    try {
        std::vector<float> xs((size_t)n_rows * H), g((size_t)n_rows * I), u((size_t)n_rows * I), y((size_t)n_rows * H);
        const uint16_t* X = (const uint16_t*)x_fp16;
        for (int r = 0; r < n_rows; ++r)
            for (int k = 0; k < H; ++k) {
                const float x = h2f_host(X[(size_t)r * ldx + k]);
                xs[(size_t)r * H + k] = s_in ? x / s_in[k] : x;
            }
        const bool c = e->codes;
        linear_mt(xs.data(), n_rows, H, c ? nullptr : e->w1f.data(), e->w1q.data(), e->sw1.data(), I, g.data(), nt);
        linear_mt(xs.data(), n_rows, H, c ? nullptr : e->w3f.data(), e->w3q.data(), e->sw3.data(), I, u.data(), nt);
        // h = fp16(silu(g) * u), then the smoothed operand of the down projection, in place in g
        for (int r = 0; r < n_rows; ++r)
            for (int j = 0; j < I; ++j) {
                const size_t i = (size_t)r * I + j;
                const float gv = g[i];
                const float sl = gv / (1.0f + exp_host(-gv));
                g[i] = h2f_host(f2h_host(sl * u[i])) / e->s_mid[j];
            }
        linear_mt(g.data(), n_rows, I, c ? nullptr : e->w2f.data(), e->w2q.data(), e->sw2.data(), H, y.data(), nt);
        uint16_t* Y = (uint16_t*)y_fp16;
        for (int r = 0; r < n_rows; ++r)
            for (int n = 0; n < H; ++n) Y[(size_t)r * ldy + n] = f2h_host(y[(size_t)r * H + n]);
    } catch (const std::bad_alloc&) {
        HAQ_FAIL(HAQ_ERR_HIP, "haq_cpu_expert_ffn: out of host memory");
    } catch (const std::system_error&) {
        HAQ_FAIL(HAQ_ERR_HIP, "haq_cpu_expert_ffn: could not start a worker thread");
    }
    return HAQ_OK;
}

}  // extern "C"
