// Adaptive activation smoothing (Algorithm 1 step 1, Eq. 3): grid search of the exponent e
// of s = ax^e for one linear layer.  Every candidate goes through the library's own offline
// quantiser and its run-time W8A8 linear; what this file adds is the full-precision product
// the candidates are measured against, the loss reduction, and the search loop around them.
#include "haq_common.h"

#include <cmath>
#include <limits>
#include <vector>

namespace haq {

namespace {

// ---- Yref = X W in binary64 ---------------------------------------------------------------
// One binary64 accumulator per output, k ascending, one fused multiply-add per term.  The
// product of a binary16 and a binary32 number is exact in binary64, so the FMA rounds exactly
// where "multiply, then add" would: the result does not depend on the tiling.
// 64 x 64 outputs per work-group, 4 x 4 per thread, K in steps of 16 through LDS.
constexpr int RT = 64, RK = 16;
__global__ __launch_bounds__(256) void ref_gemm_f64_kernel(const __half* x, int64_t ldx, const float* w, int T, int K,
                                                           int N, double* yref) {
    __shared__ double xs[RK][RT + 1];  // [k][row]
    __shared__ double ws[RK][RT];      // [k][col]
    const int tid = threadIdx.x;
    const int tx = tid % 16, ty = tid / 16;  // thread's 4 columns / 4 rows inside the tile
    const int row0 = blockIdx.y * RT, col0 = blockIdx.x * RT;
    double acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.0;
    for (int k0 = 0; k0 < K; k0 += RK) {
        // X tile: 64 rows x 16 k; thread loads 4 consecutive k of one row
        {
            const int r = tid / 4, kk = (tid % 4) * 4;
            const int row = row0 + r;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int k = k0 + kk + i;
                xs[kk + i][r] = (row < T && k < K) ? (double)h2f(x[(size_t)row * ldx + k]) : 0.0;
            }
        }
        // W tile: 16 k x 64 columns; thread loads 4 consecutive columns of one k
        {
            const int kk = tid / 16, c = (tid % 16) * 4;
            const int k = k0 + kk;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int col = col0 + c + i;
                ws[kk][c + i] = (k < K && col < N) ? (double)w[(size_t)k * N + col] : 0.0;
            }
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < RK; ++kk) {
            double xv[4], wv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) xv[i] = xs[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) wv[j] = ws[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_fma(xv[i], wv[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = row0 + ty * 4 + i;
        if (row >= T) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int col = col0 + tx * 4 + j;
            if (col < N) yref[(size_t)row * N + col] = acc[i][j];
        }
    }
}

// ---- loss = mean (Y - Yref)^2 in binary64 ------------------------------------------------------
// Row sums run over the columns in order (one sequential chain per row, as the definition is
// written), so the value does not depend on the launch shape: a work-group owns 64 rows, stages
// 64 x 64 tiles of the differences' squares through LDS with coalesced loads, and thread r adds
// the 64 values of row r in column order.  A single thread then adds the rows in order.
__global__ __launch_bounds__(256) void row_sq_err_kernel(const __half* y, int64_t ldy, const double* yref, int T, int N,
                                                         double* row_sum) {
    __shared__ double sq[64][65];
    const int tid = threadIdx.x;
    const int row0 = blockIdx.x * 64;
    double run = 0.0;
    for (int c0 = 0; c0 < N; c0 += 64) {
        for (int i = tid; i < 64 * 64; i += 256) {
            const int r = i / 64, c = i % 64;
            const int row = row0 + r, col = c0 + c;
            double v = 0.0;
            if (row < T && col < N) {
                const double d = (double)h2f(y[(size_t)row * ldy + col]) - yref[(size_t)row * N + col];
                v = d * d;
            }
            sq[r][c] = v;
        }
        __syncthreads();
        if (tid < 64) {
            const int lim = min(64, N - c0);
            for (int c = 0; c < lim; ++c) run += sq[tid][c];
        }
        __syncthreads();
    }
    if (tid < 64 && row0 + tid < T) row_sum[row0 + tid] = run;
}

__global__ void total_loss_kernel(const double* row_sum, int T, int N, double* loss) {
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        double total = 0.0;
        for (int t = 0; t < T; ++t) total += row_sum[t];
        *loss = total / ((double)T * (double)N);
    }
}

struct SearchWs {
    float *ax, *aw, *s_all, *sw;
    double *yref, *row_sum, *losses;
    int8_t *wq, *packed;
    __half* y;
    void* lin;
    size_t lin_bytes, bytes;
};

SearchWs carve_search(void* ws, int T, int K, int N, int n_e) {
    uint8_t* base = (uint8_t*)ws;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        void* p = base ? base + off : nullptr;
        off += (size_t)round_up((int64_t)bytes, 256);
        return p;
    };
    SearchWs w;
    w.ax = (float*)take((size_t)K * 4);
    w.aw = (float*)take((size_t)K * 4);
    w.s_all = (float*)take((size_t)n_e * K * 4);
    w.sw = (float*)take((size_t)N * 4);
    w.yref = (double*)take((size_t)T * N * 8);
    w.row_sum = (double*)take((size_t)T * 8);
    w.losses = (double*)take((size_t)n_e * 8);
    w.wq = (int8_t*)take((size_t)K * N);
    w.packed = (int8_t*)take(haq_packed_bytes(K, N));
    w.y = (__half*)take((size_t)T * N * 2);
    w.lin_bytes = haq_linear_workspace_bytes(T, K, N);
    w.lin = take(w.lin_bytes);
    w.bytes = off;
    return w;
}

}  // namespace

}  // namespace haq

using namespace haq;

extern "C" {

size_t haq_smoothing_search_workspace_bytes(int32_t T, int32_t K, int32_t N, int32_t n_e) {
    if (T <= 0 || K <= 0 || N <= 0 || n_e <= 0) return 0;
    return carve_search(nullptr, T, K, N, n_e).bytes;
}

int32_t haq_reference_matmul_f64(const void* x_fp16, int64_t ldx, const float* w, int32_t T, int32_t K, int32_t N,
                                 double* yref, void* stream) {
    if (T <= 0 || K <= 0 || N <= 0) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_reference_matmul_f64: T=%d K=%d N=%d", T, K, N);
    if (!x_fp16 || !w || !yref || ldx < K) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_reference_matmul_f64: null buffer or ldx=%lld", (long long)ldx);
    hipLaunchKernelGGL(ref_gemm_f64_kernel, dim3(cdiv(N, RT), cdiv(T, RT)), dim3(256), 0, (hipStream_t)stream,
                       (const __half*)x_fp16, ldx, w, T, K, N, yref);
    HAQ_CHECK_HIP(hipGetLastError());
    return HAQ_OK;
}

int32_t haq_quant_loss_f64(const void* y_fp16, int64_t ldy, const double* yref, int32_t T, int32_t N, double* row_scratch,
                           double* loss, void* stream) {
    if (T <= 0 || N <= 0) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_quant_loss_f64: T=%d N=%d", T, N);
    if (!y_fp16 || !yref || !row_scratch || !loss || ldy < N) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_quant_loss_f64: null buffer or ldy=%lld", (long long)ldy);
    hipStream_t st = (hipStream_t)stream;
    hipLaunchKernelGGL(row_sq_err_kernel, dim3(cdiv(T, 64)), dim3(256), 0, st, (const __half*)y_fp16, ldy, yref, T, N, row_scratch);
    hipLaunchKernelGGL(total_loss_kernel, dim3(1), dim3(64), 0, st, (const double*)row_scratch, T, N, loss);
    HAQ_CHECK_HIP(hipGetLastError());
    return HAQ_OK;
}

int32_t haq_smoothing_search(const void* x_fp16, int64_t ldx, const float* w, int32_t T, int32_t K, int32_t N,
                             const double* exponents, int32_t n_e, int32_t use_weight, double* losses, int32_t* best,
                             float* s_best, void* workspace, size_t workspace_bytes, void* stream) {
    if (T <= 0 || K <= 0 || N <= 0) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_smoothing_search: T=%d K=%d N=%d", T, K, N);
    if (K % 64 != 0 || K > 65535 || N % 16 != 0)
        HAQ_FAIL(HAQ_ERR_UNSUPPORTED, "haq_smoothing_search: K=%d must be a multiple of 64 (< 65536), N=%d of 16", K, N);
    if (n_e <= 0 || n_e > 256 || !exponents) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_smoothing_search: n_e=%d outside [1, 256] or no grid", n_e);
    for (int i = 0; i < n_e; ++i)
        if (!(exponents[i] >= 0.0 && exponents[i] <= 1.0))
            HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_smoothing_search: exponent %d = %g outside [0, 1]", i, exponents[i]);
    if (!x_fp16 || !w || !losses || !best || !s_best) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_smoothing_search: null buffer");
    if (ldx < K || ldx % 8 != 0 || !aligned16(x_fp16) || !aligned16(s_best))
        HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_smoothing_search: ldx=%lld (>= K, multiple of 8), 16-byte aligned x and s_best", (long long)ldx);
    const size_t need = carve_search(nullptr, T, K, N, n_e).bytes;
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255u))
        HAQ_FAIL(HAQ_ERR_WORKSPACE, "haq_smoothing_search: workspace of %zu bytes (256-byte aligned) needed, got %zu", need, workspace_bytes);
    hipStream_t st = (hipStream_t)stream;
    SearchWs ws = carve_search(workspace, T, K, N, n_e);
    int rc;

    // channel magnitudes of the calibration activations (and of the weight rows), to the host
    HAQ_CHECK_HIP(hipMemsetAsync(ws.ax, 0, (size_t)K * 4, st));
    HAQ_CHECK_HIP(hipMemsetAsync(ws.aw, 0, (size_t)K * 4, st));
    if ((rc = haq_channel_absmax_f16(x_fp16, ldx, T, K, ws.ax, stream)) != HAQ_OK) return rc;
    if (use_weight && (rc = haq_weight_row_absmax(w, K, N, ws.aw, stream)) != HAQ_OK) return rc;
    std::vector<float> ax((size_t)K), aw((size_t)K), s_all((size_t)n_e * K);
    HAQ_CHECK_HIP(hipMemcpyAsync(ax.data(), ws.ax, (size_t)K * 4, hipMemcpyDeviceToHost, st));
    HAQ_CHECK_HIP(hipMemcpyAsync(aw.data(), ws.aw, (size_t)K * 4, hipMemcpyDeviceToHost, st));
    HAQ_CHECK_HIP(hipStreamSynchronize(st));
    for (int i = 0; i < n_e; ++i)
        if ((rc = haq_smoothing_vector(ax.data(), use_weight ? aw.data() : nullptr, K, exponents[i], s_all.data() + (size_t)i * K)) != HAQ_OK)
            return rc;
    HAQ_CHECK_HIP(hipMemcpyAsync(ws.s_all, s_all.data(), s_all.size() * 4, hipMemcpyHostToDevice, st));

    if ((rc = haq_reference_matmul_f64(x_fp16, ldx, w, T, K, N, ws.yref, stream)) != HAQ_OK) return rc;
    for (int i = 0; i < n_e; ++i) {
        const float* s = ws.s_all + (size_t)i * K;
        if ((rc = haq_quant_weight(w, s, K, N, ws.wq, ws.sw, stream)) != HAQ_OK) return rc;
        if ((rc = haq_pack_weight(ws.wq, K, N, ws.packed, stream)) != HAQ_OK) return rc;
        if ((rc = haq_w8a8_linear(x_fp16, ldx, s, ws.packed, ws.sw, T, K, N, HAQ_ACT_NONE, ws.y, N, nullptr, nullptr, nullptr,
                                  ws.lin, ws.lin_bytes, stream)) != HAQ_OK)
            return rc;
        if ((rc = haq_quant_loss_f64(ws.y, N, ws.yref, T, N, ws.row_sum, ws.losses + i, stream)) != HAQ_OK) return rc;
    }
    HAQ_CHECK_HIP(hipMemcpyAsync(losses, ws.losses, (size_t)n_e * 8, hipMemcpyDeviceToHost, st));
    HAQ_CHECK_HIP(hipStreamSynchronize(st));  // also keeps s_all alive until its copy has landed

    // a candidate replaces the incumbent only if its loss is strictly smaller
    int b = -1;
    double best_loss = std::numeric_limits<double>::infinity();
    for (int i = 0; i < n_e; ++i) {
        if (losses[i] < best_loss) {
            best_loss = losses[i];
            b = i;
        }
    }
    if (b < 0) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_smoothing_search: no candidate has a finite loss");
    *best = b;
    HAQ_CHECK_HIP(hipMemcpyAsync(s_best, ws.s_all + (size_t)b * K, (size_t)K * 4, hipMemcpyDeviceToDevice, st));
    HAQ_CHECK_HIP(hipStreamSynchronize(st));
    return HAQ_OK;
}

}  // extern "C"
