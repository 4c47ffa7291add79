// The CPU side of the heterogeneous deployment (Section III.B.3; Algorithm 1 step 3, CPU branch;
// Section III.C.1a, option A).  An expert that lives in host memory keeps, next to its int8 codes,
// a floating-point copy that is produced once when the expert is loaded: Wf = float(code) * scale.
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

struct haq_cpu_expert {
    int H = 0, I = 0;
    std::vector<float> w1f, w3f, w2f, s_mid;  // [H x I], [H x I], [I x H], [I]
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

void linear_mt(const float* xs, int R, int K, const float* W, int N, float* y, int n_threads) {
    const int nt = std::max(1, std::min(n_threads, N / 64));
    if (nt == 1) {
        linear_slice(xs, R, K, W, N, 0, N, y);
        return;
    }
    std::vector<std::thread> th;
    th.reserve((size_t)nt);
    const int per = ((N + nt - 1) / nt + 15) / 16 * 16;
    try {
        for (int t = 0; t < nt; ++t) {
            const int n0 = std::min(N, t * per), n1 = std::min(N, n0 + per);
            if (n0 < n1) th.emplace_back(linear_slice, xs, R, K, W, N, n0, n1, y);
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
                              const float* sw2, const float* s_mid, int32_t H, int32_t I, haq_cpu_expert** out) {
    if (!out) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_cpu_expert_create: null output");
    *out = nullptr;
    if (H <= 0 || I <= 0) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_cpu_expert_create: H=%d I=%d", H, I);
    if (!w1q || !w3q || !w2q || !sw1 || !sw3 || !sw2 || !s_mid) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_cpu_expert_create: null buffer");
    haq_cpu_expert* e = nullptr;
    try {
        e = new haq_cpu_expert();
        e->H = H;
        e->I = I;
        e->w1f.resize((size_t)H * I);
        e->w3f.resize((size_t)H * I);
        e->w2f.resize((size_t)I * H);
        e->s_mid.assign(s_mid, s_mid + I);
    } catch (const std::bad_alloc&) {
        delete e;
        HAQ_FAIL(HAQ_ERR_HIP, "haq_cpu_expert_create: out of host memory");
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
        linear_mt(xs.data(), n_rows, H, e->w1f.data(), I, g.data(), nt);
        linear_mt(xs.data(), n_rows, H, e->w3f.data(), I, u.data(), nt);
        // h = fp16(silu(g) * u), then the smoothed operand of the down projection, in place in g
        for (int r = 0; r < n_rows; ++r)
            for (int j = 0; j < I; ++j) {
                const size_t i = (size_t)r * I + j;
                const float gv = g[i];
                const float sl = gv / (1.0f + exp_host(-gv));
                g[i] = h2f_host(f2h_host(sl * u[i])) / e->s_mid[j];
            }
        linear_mt(g.data(), n_rows, I, e->w2f.data(), H, y.data(), nt);
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
