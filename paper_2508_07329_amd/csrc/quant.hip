// Activation quantisation (Eq. 1, Q(s^-1 X), scale on the token dimension) and
// the offline weight-side kernels (Q(W s), per-channel magnitudes, packing).
#include "haq_common.h"

namespace haq {

namespace {

constexpr int QROWS = 8;      // rows per block
constexpr int QTHREADS = 256;
constexpr int QGROUPS = QTHREADS / QROWS;  // 16-element chunks handled side by side per row

struct alignas(16) Half8 { __half v[8]; };

__device__ __forceinline__ void load_y16(const __half* xrow, const float* s, int c, float (&y)[16]) {
    const uint4* px = reinterpret_cast<const uint4*>(xrow + c * 16);
    uint4 r0 = px[0], r1 = px[1];
    Half8 h0, h1;
    *reinterpret_cast<uint4*>(&h0) = r0;
    *reinterpret_cast<uint4*>(&h1) = r1;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        y[i] = h2f(h0.v[i]);
        y[8 + i] = h2f(h1.v[i]);
    }
    if (s) {
        const float4* ps = reinterpret_cast<const float4*>(s + c * 16);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float4 sv = ps[i];
            y[4 * i + 0] = y[4 * i + 0] / sv.x;
            y[4 * i + 1] = y[4 * i + 1] / sv.y;
            y[4 * i + 2] = y[4 * i + 2] / sv.z;
            y[4 * i + 3] = y[4 * i + 3] / sv.w;
        }
    }
}

// Block = 8 rows x 32 chunk lanes: thread (row = tid % 8, g = tid / 8) owns chunks
// g, g + 32, ...  Eight neighbouring lanes of a row read 256 contiguous bytes of X
// and, in the chunk-major output, eight neighbouring rows of one chunk fill one
// 128-byte line.  Pass 1 reduces the row absmax (lane shuffles, then 4 waves via
// LDS); pass 2 re-reads the row (L2 resident) and rounds.
__global__ __launch_bounds__(QTHREADS) void smooth_quant_kernel(QuantArgs a) {
    __shared__ float red[QTHREADS / 64][QROWS];
    const int tid = threadIdx.x;
    const int rib = tid % QROWS, g = tid / QROWS;
    const int t = blockIdx.x * QROWS + rib;
    const bool live = t < a.T;
    const int nchunk = a.K / 16;
    const __half* xrow = a.x + (size_t)(live ? t : 0) * a.ldx;
    const float* s = a.s;
    if (a.tab) {  // smoothing vector of the expert that owns this sorted row
        int e = 0;
        while (e + 1 < a.E && t >= a.offsets[e + 1]) ++e;
        s = a.tab[e].s_mid;
    }
    float amax = 0.0f;
    float y[16];
    if (live) {
        for (int c = g; c < nchunk; c += QGROUPS) {
            load_y16(xrow, s, c, y);
#pragma unroll
            for (int i = 0; i < 16; ++i) amax = fmaxf(amax, fabsf(y[i]));
        }
    }
    amax = fmaxf(amax, __shfl_xor(amax, 8));
    amax = fmaxf(amax, __shfl_xor(amax, 16));
    amax = fmaxf(amax, __shfl_xor(amax, 32));
    if ((tid & 63) < QROWS) red[tid >> 6][rib] = amax;
    __syncthreads();
    amax = fmaxf(fmaxf(red[0][rib], red[1][rib]), fmaxf(red[2][rib], red[3][rib]));
    if (!live) return;
    const float scale = amax / 127.0f;
    int64_t d0 = t, d1 = -1;
    if (a.dest) {
        d0 = a.dest[2 * t];
        d1 = a.dest[2 * t + 1];
    }
    if (g == 0) {
        if (a.scale) a.scale[t] = scale;
        if (a.scale_dest) {
            a.scale_dest[d0] = scale;
            if (d1 >= 0) a.scale_dest[d1] = scale;
        }
    }
    for (int c = g; c < nchunk; c += QGROUPS) {
        uint32_t w[4] = {0, 0, 0, 0};
        if (amax != 0.0f) {
            load_y16(xrow, s, c, y);
#pragma unroll
            for (int i = 0; i < 16; ++i) w[i / 4] |= (uint32_t)(code_of(y[i], scale) & 0xff) << (8 * (i % 4));
        }
        const uint4 v = make_uint4(w[0], w[1], w[2], w[3]);
        if (a.q_rm) *reinterpret_cast<uint4*>(a.q_rm + (size_t)t * a.ldq + c * 16) = v;
        if (a.q_cm) {
            *reinterpret_cast<uint4*>(a.q_cm + ((size_t)c * a.R + d0) * 16) = v;
            if (d1 >= 0) *reinterpret_cast<uint4*>(a.q_cm + ((size_t)c * a.R + d1) * 16) = v;
        }
    }
}

// ---- offline: per-channel magnitudes ----------------------------------------
__global__ void channel_absmax_f16_kernel(const __half* x, int64_t ldx, int T, int K, float* ax) {
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= K) return;
    float m = 0.0f;
    for (int t = blockIdx.y; t < T; t += gridDim.y) m = fmaxf(m, fabsf(h2f(x[(size_t)t * ldx + k])));
    // non-negative floats order like their bit patterns
    atomicMax(reinterpret_cast<unsigned int*>(ax) + k, __float_as_uint(m));
}

__global__ void weight_row_absmax_kernel(const float* w, int K, int N, float* aw) {
    __shared__ float red[256];
    const int k = blockIdx.x;
    float m = 0.0f;
    for (int n = threadIdx.x; n < N; n += blockDim.x) m = fmaxf(m, fabsf(w[(size_t)k * N + n]));
    red[threadIdx.x] = m;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) red[threadIdx.x] = fmaxf(red[threadIdx.x], red[threadIdx.x + o]);
        __syncthreads();
    }
    if (threadIdx.x == 0) aw[k] = fmaxf(aw[k], red[0]);
}

// ---- offline: Q(W s), scale per output channel -------------------------------
__global__ void weight_col_absmax_kernel(const float* w, const float* s, int K, int N, float* colmax) {
    const int n = blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= N) return;
    float m = 0.0f;
    for (int k = blockIdx.y; k < K; k += gridDim.y) {
        const float sk = s ? s[k] : 1.0f;
        m = fmaxf(m, fabsf(sk * w[(size_t)k * N + n]));
    }
    atomicMax(reinterpret_cast<unsigned int*>(colmax) + n, __float_as_uint(m));
}

__global__ void weight_codes_kernel(const float* w, const float* s, int K, int N, const float* colmax, int8_t* wq) {
    const int n = blockIdx.x * blockDim.x + threadIdx.x;
    const int k = blockIdx.y;
    if (n >= N) return;
    const float a = colmax[n];
    const float sk = s ? s[k] : 1.0f;
    int c = 0;
    if (a != 0.0f) c = code_of(sk * w[(size_t)k * N + n], a / 127.0f);
    wq[(size_t)k * N + n] = (int8_t)c;
}

__global__ void absmax_to_scale_kernel(float* v, int N) {
    const int n = blockIdx.x * blockDim.x + threadIdx.x;
    if (n < N) v[n] = v[n] / 127.0f;
}

__global__ void fill_zero_kernel(uint32_t* p, size_t n) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

// ---- offline: packing ---------------------------------------------------------
// out[(kc * Npad + n) * 16 + j] = src(kc * 16 + j, n); columns n >= N are zero.
// With w3 != null the output channel n of the packed matrix maps to blocks of 32:
// even blocks come from w1, odd blocks from w3 (gate / up side by side).
__global__ void pack_kernel(const int8_t* w1, const int8_t* w3, int K, int Nsrc, int Nout, int Npad, int8_t* out) {
    const int n = blockIdx.x * blockDim.x + threadIdx.x;
    const int kc = blockIdx.y;
    if (n >= Npad) return;
    uint32_t wv[4] = {0, 0, 0, 0};
    if (n < Nout) {
        const int8_t* src = w1;
        int col = n;
        if (w3) {
            const int blk = n / 32;
            col = (blk / 2) * 32 + (n % 32);
            src = (blk & 1) ? w3 : w1;
        }
#pragma unroll
        for (int j = 0; j < 16; ++j)
            wv[j / 4] |= (uint32_t)(uint8_t)src[(size_t)(kc * 16 + j) * Nsrc + col] << (8 * (j % 4));
    }
    *reinterpret_cast<uint4*>(out + ((size_t)kc * Npad + n) * 16) = make_uint4(wv[0], wv[1], wv[2], wv[3]);
}

}  // namespace

int launch_quant(const QuantArgs& a, hipStream_t st) {
    if (a.T <= 0) return HAQ_OK;
    hipLaunchKernelGGL(smooth_quant_kernel, dim3(cdiv(a.T, QROWS)), dim3(QTHREADS), 0, st, a);
    HAQ_CHECK_HIP(hipGetLastError());
    return HAQ_OK;
}

}  // namespace haq

using namespace haq;

extern "C" {

int32_t haq_smooth_quant_act(const void* x_fp16, int64_t ldx, const float* s, int32_t T, int32_t K, int8_t* q,
                             int64_t ldq, float* row_scale, void* stream) {
    if (T < 0 || K <= 0) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_smooth_quant_act: T=%d K=%d", T, K);
    if (K % 64 != 0 || K > 65536) HAQ_FAIL(HAQ_ERR_UNSUPPORTED, "haq_smooth_quant_act: K=%d must be a multiple of 64, <= 65536", K);
    if (T == 0) return HAQ_OK;
    if (!x_fp16 || !q || !row_scale) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_smooth_quant_act: null buffer");
    if (ldx < K || ldq < K || ldx % 8 != 0 || ldq % 16 != 0)
        HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_smooth_quant_act: ldx=%lld (>=K, %%8) ldq=%lld (>=K, %%16)", (long long)ldx, (long long)ldq);
    if (!aligned16(x_fp16) || !aligned16(q) || (s && !aligned16(s)))
        HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_smooth_quant_act: pointers must be 16-byte aligned");
    QuantArgs a{};
    a.x = (const __half*)x_fp16;
    a.ldx = ldx;
    a.s = s;
    a.T = T;
    a.K = K;
    a.q_rm = q;
    a.ldq = ldq;
    a.scale = row_scale;
    return launch_quant(a, (hipStream_t)stream);
}

int32_t haq_channel_absmax_f16(const void* x_fp16, int64_t ldx, int32_t T, int32_t K, float* ax, void* stream) {
    if (T < 0 || K <= 0 || ldx < K) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_channel_absmax_f16: T=%d K=%d ldx=%lld", T, K, (long long)ldx);
    if (T == 0) return HAQ_OK;
    if (!x_fp16 || !ax) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_channel_absmax_f16: null buffer");
    const int ty = T < 64 ? T : 64;
    hipLaunchKernelGGL(channel_absmax_f16_kernel, dim3(cdiv(K, 256), ty), dim3(256), 0, (hipStream_t)stream,
                       (const __half*)x_fp16, ldx, T, K, ax);
    HAQ_CHECK_HIP(hipGetLastError());
    return HAQ_OK;
}

int32_t haq_weight_row_absmax(const float* w, int32_t K, int32_t N, float* aw, void* stream) {
    if (K <= 0 || N <= 0) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_weight_row_absmax: K=%d N=%d", K, N);
    if (!w || !aw) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_weight_row_absmax: null buffer");
    hipLaunchKernelGGL(weight_row_absmax_kernel, dim3(K), dim3(256), 0, (hipStream_t)stream, w, K, N, aw);
    HAQ_CHECK_HIP(hipGetLastError());
    return HAQ_OK;
}

int32_t haq_quant_weight(const float* w, const float* s, int32_t K, int32_t N, int8_t* wq, float* w_scale, void* stream) {
    if (K <= 0 || N <= 0 || K > 65535) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_quant_weight: K=%d N=%d", K, N);
    if (!w || !wq || !w_scale) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_quant_weight: null buffer");
    hipStream_t st = (hipStream_t)stream;
    // w_scale first holds the column absmax, then is turned into the scale in place
    hipLaunchKernelGGL(fill_zero_kernel, dim3(cdiv(N, 256)), dim3(256), 0, st, (uint32_t*)w_scale, (size_t)N);
    const int ky = K < 64 ? K : 64;
    hipLaunchKernelGGL(weight_col_absmax_kernel, dim3(cdiv(N, 256), ky), dim3(256), 0, st, w, s, K, N, w_scale);
    hipLaunchKernelGGL(weight_codes_kernel, dim3(cdiv(N, 256), K), dim3(256), 0, st, w, s, K, N, (const float*)w_scale, wq);
    hipLaunchKernelGGL(absmax_to_scale_kernel, dim3(cdiv(N, 256)), dim3(256), 0, st, w_scale, N);
    HAQ_CHECK_HIP(hipGetLastError());
    return HAQ_OK;
}

size_t haq_packed_bytes(int32_t K, int32_t N) {
    if (K <= 0 || N <= 0) return 0;
    return (size_t)K * (size_t)round_up(N, NPAD);
}

int32_t haq_pack_weight(const int8_t* wq, int32_t K, int32_t N, int8_t* packed, void* stream) {
    if (K <= 0 || N <= 0) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_pack_weight: K=%d N=%d", K, N);
    if (K % 64 != 0 || K / 16 > 65535) HAQ_FAIL(HAQ_ERR_UNSUPPORTED, "haq_pack_weight: K=%d must be a multiple of 64", K);
    if (!wq || !packed || !aligned16(packed)) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_pack_weight: null or misaligned buffer");
    const int Npad = (int)round_up(N, NPAD);
    hipLaunchKernelGGL(pack_kernel, dim3(Npad / 256, K / 16), dim3(256), 0, (hipStream_t)stream, wq,
                       (const int8_t*)nullptr, K, N, N, Npad, packed);
    HAQ_CHECK_HIP(hipGetLastError());
    return HAQ_OK;
}

int32_t haq_pack_gate_up(const int8_t* w1q, const int8_t* w3q, int32_t K, int32_t N, int8_t* packed, void* stream) {
    if (K <= 0 || N <= 0) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_pack_gate_up: K=%d N=%d", K, N);
    if (K % 64 != 0 || K / 16 > 65535 || N % 32 != 0)
        HAQ_FAIL(HAQ_ERR_UNSUPPORTED, "haq_pack_gate_up: K=%d must be a multiple of 64 and N=%d of 32", K, N);
    if (!w1q || !w3q || !packed || !aligned16(packed)) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_pack_gate_up: null or misaligned buffer");
    const int Npad = (int)round_up(2 * (int64_t)N, NPAD);
    hipLaunchKernelGGL(pack_kernel, dim3(Npad / 256, K / 16), dim3(256), 0, (hipStream_t)stream, w1q, w3q, K, N, 2 * N,
                       Npad, packed);
    HAQ_CHECK_HIP(hipGetLastError());
    return HAQ_OK;
}

}  // extern "C"
