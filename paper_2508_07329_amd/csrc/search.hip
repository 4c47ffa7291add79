// Adaptive activation smoothing (Algorithm 1 step 1, Eq. 3): grid search of the exponent e
// of s = ax^e for one linear layer.  Every candidate goes through the library's own offline
// quantiser and its run-time W8A8 linear; what this file adds is the full-precision product
// the candidates are measured against, the loss reduction, and the search loop around them.
#include "haq_common.h"

#include <cmath>
#include <limits>
#include <new>
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
// written), so the value does not depend on the launch shape.  A work-group owns 16 rows and
// walks over tiles of 256 columns: all threads fetch the next tile (coalesced) and square the
// differences while thread r < 16 adds the 256 values of row r of the current tile, in column
// order, from LDS (two buffers, one barrier per tile).  A last small kernel adds the rows in
// order.
constexpr int LR = 16, LC = 256;
__global__ __launch_bounds__(256) void row_sq_err_kernel(const __half* y, int64_t ldy, const double* yref, int T, int N,
                                                         double* row_sum) {
    __shared__ double sq[2][LR][LC + 2];
    const int tid = threadIdx.x;
    const int row0 = blockIdx.x * LR;
    const int ntile = (N + LC - 1) / LC;
    double v[LR];
    auto fetch = [&](int tile) {  // thread = one column of the tile, all 16 rows
        const int col = tile * LC + tid;
        const int colc = min(col, N - 1);  // loads stay unconditional (clamped), masked afterwards
        __half yv[LR];
        double rv[LR];
#pragma unroll
        for (int r = 0; r < LR; ++r) {
            const int rowc = min(row0 + r, T - 1);
            yv[r] = y[(size_t)rowc * ldy + colc];
            rv[r] = yref[(size_t)rowc * N + colc];
        }
#pragma unroll
        for (int r = 0; r < LR; ++r) {
            const double d = (double)h2f(yv[r]) - rv[r];
            v[r] = (row0 + r < T && col < N) ? d * d : 0.0;
        }
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int r = 0; r < LR; ++r) sq[buf][r][tid] = v[r];
    };
    fetch(0);
    stage(0);
    __syncthreads();
    double run = 0.0;
    for (int tile = 0; tile < ntile; ++tile) {
        const int buf = tile & 1;
        if (tile + 1 < ntile) fetch(tile + 1);  // in flight while the chain below runs
        if (tid < LR) {
            const int lim = min(LC, N - tile * LC);
            const double* p = sq[buf][tid];
            int c = 0;
            for (; c + 16 <= lim; c += 16) {  // 16 loads ahead of the dependent additions
                double t[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) t[i] = p[c + i];
#pragma unroll
                for (int i = 0; i < 16; ++i) run += t[i];
            }
            for (; c < lim; ++c) run += p[c];
        }
        if (tile + 1 < ntile) stage(buf ^ 1);
        __syncthreads();
    }
    if (tid < LR && row0 + tid < T) row_sum[row0 + tid] = run;
}

__global__ __launch_bounds__(256) void total_loss_kernel(const double* row_sum, int T, int N, double* loss) {
    __shared__ double part[1024];
    double total = 0.0;
    for (int t0 = 0; t0 < T; t0 += 1024) {  // rows in order, 1024 at a time through LDS
        for (int i = threadIdx.x; i < 1024; i += 256) part[i] = t0 + i < T ? row_sum[t0 + i] : 0.0;
        __syncthreads();
        if (threadIdx.x == 0) {
            const int lim = min(1024, T - t0);
            for (int i = 0; i < lim; ++i) total += part[i];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) *loss = total / ((double)T * (double)N);
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
    hipLaunchKernelGGL(row_sq_err_kernel, dim3(cdiv(T, LR)), dim3(256), 0, st, (const __half*)y_fp16, ldy, yref, T, N, row_scratch);
    hipLaunchKernelGGL(total_loss_kernel, dim3(1), dim3(256), 0, st, (const double*)row_scratch, T, N, loss);
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
    std::vector<float> ax, aw, s_all;  // host staging; no asynchronous copy outlives this function
    try {
        ax.resize((size_t)K);
        aw.resize((size_t)K);
        s_all.resize((size_t)n_e * K);
    } catch (const std::bad_alloc&) {
        HAQ_FAIL(HAQ_ERR_HIP, "haq_smoothing_search: out of host memory");
    }
    HAQ_CHECK_HIP(hipMemcpyAsync(ax.data(), ws.ax, (size_t)K * 4, hipMemcpyDeviceToHost, st));
    HAQ_CHECK_HIP(hipMemcpyAsync(aw.data(), ws.aw, (size_t)K * 4, hipMemcpyDeviceToHost, st));
    HAQ_CHECK_HIP(hipStreamSynchronize(st));
    for (int i = 0; i < n_e; ++i)
        if ((rc = haq_smoothing_vector(ax.data(), use_weight ? aw.data() : nullptr, K, exponents[i], s_all.data() + (size_t)i * K)) != HAQ_OK)
            return rc;
    HAQ_CHECK_HIP(hipMemcpyAsync(ws.s_all, s_all.data(), s_all.size() * 4, hipMemcpyHostToDevice, st));
    HAQ_CHECK_HIP(hipStreamSynchronize(st));  // s_all is pageable host memory: the copy has landed before any return below

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
    HAQ_CHECK_HIP(hipStreamSynchronize(st));

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
