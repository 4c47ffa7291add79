// Hessian-aware weight quantisation (Section III.B.2, Eq. 4-6; Algorithm 1 step 2), offline.
//
// Everything is binary64 and every accumulation is a chain of fused multiply-adds in a stated
// order (tokens ascending for the Hessian, eliminated columns ascending for the factorisation,
// quantised input channels ascending for the compensation).  Blocking only regroups which
// work-item applies a link of a chain and when; it never reorders a chain, so the bits do not
// depend on the tile sizes below.
//
//   H  = 2 Xs^T Xs + damping                       hessian_kernel, hessian_finish_kernel
//   A  = flip(H) = L L^T                           chol_panel_kernel, chol_trail_kernel
//   M  = L^-1 (lower)                              tri_inverse_block_kernel
//   U  = flip(M): upper, H^-1 = U^T U              flip_kernel
//   channels i ascending: code, error, compensate  gptq_block_kernel, gptq_update_kernel
#include "haq_common.h"

namespace haq {

namespace {

constexpr int HT = 64, HK = 16;  // Hessian tile (outputs) and token step
constexpr int PB = 32;           // Cholesky panel width
constexpr int GB = 64;           // input channels quantised per compensation block

// ---- H = 2 Xs^T Xs -------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void hessian_kernel(const __half* x, int64_t ldx, const float* s, int T, int K, double* H) {
    __shared__ double xa[HK][HT + 1];
    __shared__ double xb[HK][HT + 1];
    const int tid = threadIdx.x;
    const int tx = tid % 16, ty = tid / 16;
    const int j0 = blockIdx.y * HT, l0 = blockIdx.x * HT;
    double acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.0;
    for (int t0 = 0; t0 < T; t0 += HK) {
        const int tt = tid / 16, c = (tid % 16) * 4;
        const int t = t0 + tt;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int ja = j0 + c + i, lb = l0 + c + i;
            double va = 0.0, vb = 0.0;
            if (t < T && ja < K) {
                const float v = h2f(x[(size_t)t * ldx + ja]);
                va = (double)(s ? v / s[ja] : v);
            }
            if (t < T && lb < K) {
                const float v = h2f(x[(size_t)t * ldx + lb]);
                vb = (double)(s ? v / s[lb] : v);
            }
            xa[tt][c + i] = va;
            xb[tt][c + i] = vb;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < HK; ++kk) {
            double av[4], bv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) av[i] = xa[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) bv[j] = xb[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_fma(av[i], bv[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int j = j0 + ty * 4 + i;
        if (j >= K) continue;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            const int l = l0 + tx * 4 + jj;
            if (l < K) H[(size_t)j * K + l] = 2.0 * acc[i][jj];
        }
    }
}

// Dead channels get a unit diagonal; damping = percdamp * mean(diag), the diagonal summed in index order.
__global__ __launch_bounds__(256) void hessian_finish_kernel(double* H, int K, double percdamp) {
    __shared__ double part[1024];
    __shared__ double damp_s;
    double tr = 0.0;
    for (int j0 = 0; j0 < K; j0 += 1024) {
        for (int i = threadIdx.x; i < 1024; i += 256) {
            const int j = j0 + i;
            double d = 0.0;
            if (j < K) {
                d = H[(size_t)j * K + j];
                if (d == 0.0) {
                    d = 1.0;
                    H[(size_t)j * K + j] = 1.0;
                }
            }
            part[i] = d;
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            const int lim = min(1024, K - j0);
            for (int i = 0; i < lim; ++i) tr += part[i];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) damp_s = percdamp * (tr / (double)K);
    __syncthreads();
    const double damp = damp_s;
    for (int j = threadIdx.x; j < K; j += 256) H[(size_t)j * K + j] += damp;
}

// A(i, j) = H(K-1-i, K-1-j); also used to turn M into U.
__global__ void flip_kernel(const double* src, int K, double* dst) {
    const int j = blockIdx.x * blockDim.x + threadIdx.x, i = blockIdx.y;
    if (j < K) dst[(size_t)i * K + j] = src[(size_t)(K - 1 - i) * K + (K - 1 - j)];
}

// ---- Cholesky, right-looking in panels of PB columns ------------------------------------------
// Panel kernel: every work-group first factorises the PB x PB diagonal block in LDS (redundantly:
// it is tiny), then its threads each take one row below the block and solve it against the block,
// column by column: v = A_ic; v -= L_ik L_ck for the panel's earlier columns k ascending; L_ic = v / L_cc.
// Work-group 0 leaves the factorised diagonal block in `dblock` (it cannot go to A here: the other
// work-groups may still be reading the unfactorised block); chol_store_diag_kernel moves it afterwards.
// status: first non-positive pivot + 1.
__global__ __launch_bounds__(256) void chol_panel_kernel(double* A, int K, int j0, double* dblock, int* status) {
    __shared__ double D[PB][PB + 1];
    const int tid = threadIdx.x;
    const int pb = min(PB, K - j0);
    for (int i = tid; i < PB * PB; i += 256) {
        const int r = i / PB, c = i % PB;
        D[r][c] = (r < pb && c <= r) ? A[(size_t)(j0 + r) * K + j0 + c] : 0.0;
    }
    __syncthreads();
    for (int c = 0; c < pb; ++c) {
        // column c of the block: rows r >= c, each by one thread (the chain over k < c is sequential)
        if (tid >= c && tid < pb) {
            const int r = tid;
            double v = D[r][c];
            for (int k = 0; k < c; ++k) v = __builtin_fma(-D[r][k], D[c][k], v);
            D[r][c] = v;  // not yet divided
        }
        __syncthreads();
        if (tid == c) {
            const double d = D[c][c];
            if (!(d > 0.0) && blockIdx.x == 0) atomicCAS(status, 0, j0 + c + 1);
            D[c][c] = sqrt(d);
        }
        __syncthreads();
        if (tid > c && tid < pb) D[tid][c] = D[tid][c] / D[c][c];
        __syncthreads();
    }
    if (blockIdx.x == 0)
        for (int i = tid; i < PB * PB; i += 256) dblock[i] = D[i / PB][i % PB];
    // rows below the diagonal block
    const int i = j0 + pb + blockIdx.x * 256 + tid;
    if (i < K) {
        double row[PB];
#pragma unroll
        for (int c = 0; c < PB; ++c) row[c] = c < pb ? A[(size_t)i * K + j0 + c] : 0.0;
#pragma unroll
        for (int c = 0; c < PB; ++c) {
            if (c < pb) {
                double v = row[c];
#pragma unroll
                for (int k = 0; k < PB; ++k)
                    if (k < c) v = __builtin_fma(-row[k], D[c][k], v);
                row[c] = v / D[c][c];
            }
        }
#pragma unroll
        for (int c = 0; c < PB; ++c)
            if (c < pb) A[(size_t)i * K + j0 + c] = row[c];
    }
}

__global__ __launch_bounds__(256) void chol_store_diag_kernel(double* A, int K, int j0, const double* dblock) {
    const int pb = min(PB, K - j0);
    for (int i = threadIdx.x; i < PB * PB; i += 256) {
        const int r = i / PB, c = i % PB;
        if (r < pb && c <= r) A[(size_t)(j0 + r) * K + j0 + c] = dblock[i];
    }
}

// Trailing update after a panel: for i >= l >= j0 + PB: A_il -= L_ik L_lk, k over the panel ascending.
// 64 x 64 tiles of the lower triangle, 4 x 4 elements per thread.
__global__ __launch_bounds__(256) void chol_trail_kernel(double* A, int K, int j0) {
    const int base = j0 + PB;
    const int ti = blockIdx.y, tl = blockIdx.x;
    if (tl > ti) return;  // only tiles that touch the lower triangle
    __shared__ double Li[64][PB + 1];
    __shared__ double Ll[64][PB + 1];
    const int tid = threadIdx.x;
    const int i0 = base + ti * 64, l0 = base + tl * 64;
    for (int e = tid; e < 64 * PB; e += 256) {
        const int r = e / PB, c = e % PB;
        Li[r][c] = (i0 + r < K) ? A[(size_t)(i0 + r) * K + j0 + c] : 0.0;
        Ll[r][c] = (l0 + r < K) ? A[(size_t)(l0 + r) * K + j0 + c] : 0.0;
    }
    __syncthreads();
    const int tx = tid % 16, ty = tid / 16;
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const int i = i0 + ty * 4 + a;
        if (i >= K) continue;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int l = l0 + tx * 4 + b;
            if (l > i || l >= K) continue;
            double v = A[(size_t)i * K + l];
#pragma unroll
            for (int k = 0; k < PB; ++k) v = __builtin_fma(-Li[ty * 4 + a][k], Ll[tx * 4 + b][k], v);
            A[(size_t)i * K + l] = v;
        }
    }
}

// ---- M = L^-1, blocks of TR rows ---------------------------------------------------------------
// M_jj = 1 / L_jj; M_ij = -(sum_{j <= k < i} L_ik M_kj) / L_ii, the sum a chain over k ascending.
// A launch handles rows i0 .. i0 + TR - 1 (the launches run in row order); a work-group owns 64
// columns.  First the links k < i0 of every chain (M_kj from earlier launches): wave w carries the
// chains of rows 8w .. 8w + 7 for the 64 columns, the same k for all lanes (lanes whose column
// starts later are masked), L tile and M chunk through LDS.  Then wave 0 adds the links inside the
// block, row by row, with the M_kj it has just produced.  M must be zero on entry (the part above
// the diagonal is never written).
constexpr int TR = 32, TW = 4, RPW = TR / TW;
__global__ __launch_bounds__(64 * TW) void tri_inverse_block_kernel(const double* L, int K, int i0, double* M) {
    __shared__ double Lt[TR][64 + 1];  // [row][k in chunk]; later the diagonal block
    __shared__ double Ms[64][64];      // [k in chunk][column]
    __shared__ double Acc[TR][64];     // chains after the links k < i0
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int jmin = blockIdx.x * 64, j = jmin + lane;
    const int rows = min(TR, K - i0);
    if (jmin >= i0 + rows) return;  // uniform: the whole work-group lies right of the diagonal block
    const bool on = j < i0 + rows;
    double acc[RPW];
#pragma unroll
    for (int r = 0; r < RPW; ++r) acc[r] = 0.0;
    for (int k0 = jmin; k0 < i0; k0 += 64) {
        const int lim = min(64, i0 - k0);
        __syncthreads();
        for (int e = tid; e < TR * 64; e += 64 * TW) {
            const int r = e / 64, c = e % 64;
            Lt[r][c] = (r < rows && c < lim) ? L[(size_t)(i0 + r) * K + k0 + c] : 0.0;
        }
        for (int e = tid; e < 64 * 64; e += 64 * TW) {  // coalesced over the columns
            const int kk = e / 64, c = e % 64;
            const int k = k0 + kk, col = jmin + c;
            Ms[kk][c] = (kk < lim && col < i0 + rows && k >= col) ? M[(size_t)k * K + col] : 0.0;
        }
        __syncthreads();
        if (on) {
            // Ms is zero where k < j or past the chunk's end, and a link with M_kj = 0 leaves the chain
            // as it is (v - L * 0 = v exactly; a chain never holds -0 because it starts from +0), so the
            // loop needs no per-lane condition and unrolls
#pragma unroll 8
            for (int e = 0; e < 64; ++e) {
                const double m = Ms[e][lane];
#pragma unroll
                for (int r = 0; r < RPW; ++r) acc[r] = __builtin_fma(-Lt[wave * RPW + r][e], m, acc[r]);
            }
        }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < RPW; ++r) Acc[wave * RPW + r][lane] = acc[r];
    for (int e = tid; e < TR * TR; e += 64 * TW) {
        const int r = e / TR, c = e % TR;
        Lt[r][c] = (r < rows && c <= r) ? L[(size_t)(i0 + r) * K + i0 + c] : 0.0;
    }
    __syncthreads();
    if (wave != 0 || !on) return;
    double mloc[TR];
#pragma unroll
    for (int r = 0; r < TR; ++r) {
        mloc[r] = 0.0;
        if (r < rows) {
            const int i = i0 + r;
            if (i == j) {
                mloc[r] = 1.0 / Lt[r][r];
                M[(size_t)i * K + j] = mloc[r];
            } else if (i > j) {
                double v = Acc[r][lane];
#pragma unroll
                for (int c = 0; c < TR; ++c)
                    if (c < r && i0 + c >= j) v = __builtin_fma(-Lt[r][c], mloc[c], v);
                mloc[r] = v / Lt[r][r];
                M[(size_t)i * K + j] = mloc[r];
            }
        }
    }
}

// ---- the quantise-and-compensate sweep ------------------------------------------------------------
__global__ void fold_weight_kernel(const float* w, const float* s, int K, int N, double* w64) {
    const int n = blockIdx.x * blockDim.x + threadIdx.x, k = blockIdx.y;
    if (n < N) w64[(size_t)k * N + n] = (double)((s ? s[k] : 1.0f) * w[(size_t)k * N + n]);
}

// Channels b0 .. b0 + GB - 1, one thread per output channel n: code, error, compensation of the
// block's later channels; the errors go to err [GB x N] for the rows below the block.
__global__ __launch_bounds__(64) void gptq_block_kernel(double* w64, const double* U, const float* scale, int K, int N, int b0,
                                                        int8_t* wq, double* err) {
    __shared__ double Ub[GB][GB + 1];
    const int gb = min(GB, K - b0);
    for (int e = threadIdx.x; e < GB * GB; e += 64) {
        const int r = e / GB, c = e % GB;
        Ub[r][c] = (r < gb && c < gb) ? U[(size_t)(b0 + r) * K + b0 + c] : 0.0;
    }
    __syncthreads();
    const int n = blockIdx.x * 64 + threadIdx.x;
    if (n >= N) return;
    const float sc_f = scale[n];
    const double sc = (double)sc_f;
    double w[GB];
#pragma unroll
    for (int i = 0; i < GB; ++i) w[i] = i < gb ? w64[(size_t)(b0 + i) * N + n] : 0.0;
#pragma unroll
    for (int i = 0; i < GB; ++i) {
        if (i < gb) {
            double code = 0.0;
            if (sc_f != 0.0f) {
                code = __builtin_rint(w[i] / sc);
                code = fmin(fmax(code, -127.0), 127.0);
            }
            wq[(size_t)(b0 + i) * N + n] = (int8_t)code;
            const double e = (w[i] - code * sc) / Ub[i][i];
            err[(size_t)i * N + n] = e;
#pragma unroll
            for (int j = 0; j < GB; ++j)
                if (j > i && j < gb) w[j] = __builtin_fma(-e, Ub[i][j], w[j]);
        }
    }
}

// Rows j >= b0 + GB: w_jn -= err_in U_ij for the block's channels i ascending.  64 rows x 64
// output channels per work-group, 4 x 4 per thread held in registers; the block's channels come
// through LDS 32 at a time (in order).
__global__ __launch_bounds__(256) void gptq_update_kernel(double* w64, const double* U, const double* err, int K, int N, int b0) {
    constexpr int GH = 32;
    __shared__ double Es[GH][64 + 1];  // [i][n]
    __shared__ double Us[GH][64 + 1];  // [i][j]
    const int tid = threadIdx.x;
    const int r0 = b0 + GB + blockIdx.y * 64, n0 = blockIdx.x * 64;
    const int tx = tid % 16, ty = tid / 16;
    const bool full_cols = n0 + tx * 4 + 3 < N && (N % 2 == 0);
    double v[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const int j = r0 + ty * 4 + a;
        const double* p = w64 + (size_t)j * N + n0 + tx * 4;
        if (j < K && full_cols) {  // 32 contiguous bytes per thread, two 16-byte accesses
            const double2 lo = *reinterpret_cast<const double2*>(p), hi = *reinterpret_cast<const double2*>(p + 2);
            v[a][0] = lo.x; v[a][1] = lo.y; v[a][2] = hi.x; v[a][3] = hi.y;
        } else {
#pragma unroll
            for (int b = 0; b < 4; ++b) v[a][b] = (j < K && n0 + tx * 4 + b < N) ? p[b] : 0.0;
        }
    }
    for (int h = 0; h < GB; h += GH) {
        __syncthreads();
        for (int e = tid; e < GH * 64; e += 256) {
            const int i = e / 64, c = e % 64;
            Es[i][c] = (n0 + c < N) ? err[(size_t)(h + i) * N + n0 + c] : 0.0;
            Us[i][c] = (r0 + c < K) ? U[(size_t)(b0 + h + i) * K + r0 + c] : 0.0;
        }
        __syncthreads();
#pragma unroll 8
        for (int i = 0; i < GH; ++i) {
            double ev[4], uv[4];
#pragma unroll
            for (int b = 0; b < 4; ++b) ev[b] = Es[i][tx * 4 + b];
#pragma unroll
            for (int a = 0; a < 4; ++a) uv[a] = Us[i][ty * 4 + a];
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b) v[a][b] = __builtin_fma(-ev[b], uv[a], v[a][b]);
        }
    }
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const int j = r0 + ty * 4 + a;
        if (j >= K) continue;
        double* p = w64 + (size_t)j * N + n0 + tx * 4;
        if (full_cols) {
            *reinterpret_cast<double2*>(p) = make_double2(v[a][0], v[a][1]);
            *reinterpret_cast<double2*>(p + 2) = make_double2(v[a][2], v[a][3]);
        } else {
#pragma unroll
            for (int b = 0; b < 4; ++b)
                if (n0 + tx * 4 + b < N) p[b] = v[a][b];
        }
    }
}

struct HessWs {
    double *H, *A, *M, *w64, *err;
    int* status;
    size_t bytes;
};

HessWs carve_hess(void* ws, int K, int N) {
    uint8_t* base = (uint8_t*)ws;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        void* p = base ? base + off : nullptr;
        off += (size_t)round_up((int64_t)bytes, 256);
        return p;
    };
    HessWs w;
    w.H = (double*)take((size_t)K * K * 8);
    w.A = (double*)take((size_t)K * K * 8);
    w.M = (double*)take((size_t)K * K * 8);
    w.w64 = (double*)take((size_t)K * N * 8);
    w.err = (double*)take((size_t)GB * N * 8);
    w.status = (int*)take(64 + PB * PB * 8);
    w.bytes = off;
    return w;
}

}  // namespace

}  // namespace haq

using namespace haq;

extern "C" {

int32_t haq_hessian_f64(const void* x_fp16, int64_t ldx, const float* s, int32_t T, int32_t K, double percdamp, double* H,
                        void* stream) {
    if (T <= 0 || K <= 0 || !(percdamp >= 0.0)) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_hessian_f64: T=%d K=%d percdamp=%g", T, K, percdamp);
    if (!x_fp16 || !H || ldx < K) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_hessian_f64: null buffer or ldx=%lld", (long long)ldx);
    hipStream_t st = (hipStream_t)stream;
    hipLaunchKernelGGL(hessian_kernel, dim3(cdiv(K, HT), cdiv(K, HT)), dim3(256), 0, st, (const __half*)x_fp16, ldx, s, T, K, H);
    hipLaunchKernelGGL(hessian_finish_kernel, dim3(1), dim3(256), 0, st, H, K, percdamp);
    HAQ_CHECK_HIP(hipGetLastError());
    return HAQ_OK;
}

size_t haq_inverse_cholesky_workspace_bytes(int32_t K) {
    if (K <= 0) return 0;
    return 2 * (size_t)round_up((int64_t)K * K * 8, 256) + 64 + PB * PB * 8;
}

// H may alias U: H is read once, into A, before anything else runs.
static int32_t inverse_cholesky_upper(const double* H, int K, double* U, double* A, double* M, int* status, hipStream_t st) {
    double* dblock = reinterpret_cast<double*>(status) + 8;  // PB x PB doubles behind the status word
    HAQ_CHECK_HIP(hipMemsetAsync(status, 0, sizeof(int), st));
    hipLaunchKernelGGL(flip_kernel, dim3(cdiv(K, 256), K), dim3(256), 0, st, H, K, A);
    for (int j0 = 0; j0 < K; j0 += PB) {
        const int pb = K - j0 < PB ? K - j0 : PB;
        const int below = K - j0 - pb;
        hipLaunchKernelGGL(chol_panel_kernel, dim3(below > 0 ? cdiv(below, 256) : 1), dim3(256), 0, st, A, K, j0, dblock, status);
        hipLaunchKernelGGL(chol_store_diag_kernel, dim3(1), dim3(256), 0, st, A, K, j0, (const double*)dblock);
        if (below > 0) {
            const int nt = cdiv(below, 64);
            hipLaunchKernelGGL(chol_trail_kernel, dim3(nt, nt), dim3(256), 0, st, A, K, j0);
        }
    }
    HAQ_CHECK_HIP(hipMemsetAsync(M, 0, (size_t)K * K * sizeof(double), st));
    for (int i0 = 0; i0 < K; i0 += TR)
        hipLaunchKernelGGL(tri_inverse_block_kernel, dim3(cdiv(i0 + TR < K ? i0 + TR : K, 64)), dim3(64 * TW), 0, st, (const double*)A, K, i0, M);
    hipLaunchKernelGGL(flip_kernel, dim3(cdiv(K, 256), K), dim3(256), 0, st, (const double*)M, K, U);
    HAQ_CHECK_HIP(hipGetLastError());
    int host_status = 0;
    HAQ_CHECK_HIP(hipMemcpyAsync(&host_status, status, sizeof(int), hipMemcpyDeviceToHost, st));
    HAQ_CHECK_HIP(hipStreamSynchronize(st));
    if (host_status != 0)
        HAQ_FAIL(HAQ_ERR_INVALID_ARG, "the Hessian is not positive definite (pivot %d of the flipped matrix)", host_status - 1);
    return HAQ_OK;
}

int32_t haq_inverse_cholesky_upper_f64(const double* H, int32_t K, double* U, void* workspace, size_t workspace_bytes,
                                       void* stream) {
    if (K <= 0 || K > 65535 || !H || !U) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_inverse_cholesky_upper_f64: K=%d or null buffer", K);
    if (!workspace || workspace_bytes < haq_inverse_cholesky_workspace_bytes(K) || ((uintptr_t)workspace & 255u))
        HAQ_FAIL(HAQ_ERR_WORKSPACE, "haq_inverse_cholesky_upper_f64: workspace of %zu bytes (256-byte aligned) needed, got %zu",
                 haq_inverse_cholesky_workspace_bytes(K), workspace_bytes);
    const size_t mat = (size_t)round_up((int64_t)K * K * 8, 256);
    return inverse_cholesky_upper(H, K, U, (double*)workspace, (double*)((uint8_t*)workspace + mat),
                                  (int*)((uint8_t*)workspace + 2 * mat), (hipStream_t)stream);
}

size_t haq_hessian_quant_workspace_bytes(int32_t K, int32_t N) {
    if (K <= 0 || N <= 0) return 0;
    return carve_hess(nullptr, K, N).bytes;
}

int32_t haq_hessian_quant_weight(const void* x_fp16, int64_t ldx, int32_t T, const float* w, const float* s, int32_t K,
                                 int32_t N, double percdamp, int8_t* wq, float* w_scale, void* workspace,
                                 size_t workspace_bytes, void* stream) {
    if (T <= 0 || K <= 0 || N <= 0 || K > 65535) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_hessian_quant_weight: T=%d K=%d N=%d", T, K, N);
    if (!x_fp16 || !w || !wq || !w_scale || ldx < K) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_hessian_quant_weight: null buffer or ldx=%lld", (long long)ldx);
    const size_t need = carve_hess(nullptr, K, N).bytes;
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255u))
        HAQ_FAIL(HAQ_ERR_WORKSPACE, "haq_hessian_quant_weight: workspace of %zu bytes (256-byte aligned) needed, got %zu", need, workspace_bytes);
    hipStream_t st = (hipStream_t)stream;
    HessWs ws = carve_hess(workspace, K, N);
    int rc;
    // the per-output-channel grid is the one of plain rounding (its codes are overwritten below)
    if ((rc = haq_quant_weight(w, s, K, N, wq, w_scale, stream)) != HAQ_OK) return rc;
    if ((rc = haq_hessian_f64(x_fp16, ldx, s, T, K, percdamp, ws.H, stream)) != HAQ_OK) return rc;
    if ((rc = inverse_cholesky_upper(ws.H, K, ws.H, ws.A, ws.M, ws.status, st)) != HAQ_OK) return rc;  // U replaces H
    const double* U = ws.H;
    hipLaunchKernelGGL(fold_weight_kernel, dim3(cdiv(N, 256), K), dim3(256), 0, st, w, s, K, N, ws.w64);
    for (int b0 = 0; b0 < K; b0 += GB) {
        hipLaunchKernelGGL(gptq_block_kernel, dim3(cdiv(N, 64)), dim3(64), 0, st, ws.w64, U, (const float*)w_scale, K, N, b0, wq, ws.err);
        const int below = K - b0 - GB;
        if (below > 0)
            hipLaunchKernelGGL(gptq_update_kernel, dim3(cdiv(N, 64), cdiv(below, 64)), dim3(256), 0, st, ws.w64, U,
                               (const double*)ws.err, K, N, b0);
    }
    HAQ_CHECK_HIP(hipGetLastError());
    return HAQ_OK;
}

size_t haq_quantize_layer_workspace_bytes(int32_t T, int32_t K, int32_t N, int32_t n_e) {
    const size_t a = haq_smoothing_search_workspace_bytes(T, K, N, n_e), b = haq_hessian_quant_workspace_bytes(K, N);
    return a > b ? a : b;
}

int32_t haq_quantize_layer(const void* x_fp16, int64_t ldx, int32_t T, const float* w, int32_t K, int32_t N,
                           const double* exponents, int32_t n_e, int32_t use_weight, double percdamp, float* s,
                           int8_t* wq, float* w_scale, double* losses, int32_t* best, void* workspace,
                           size_t workspace_bytes, void* stream) {
    if (!s || !wq || !w_scale) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_quantize_layer: null output");
    if (T <= 0 || K <= 0 || N <= 0 || n_e <= 0) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_quantize_layer: T=%d K=%d N=%d n_e=%d", T, K, N, n_e);
    if (workspace_bytes < haq_quantize_layer_workspace_bytes(T, K, N, n_e))
        HAQ_FAIL(HAQ_ERR_WORKSPACE, "haq_quantize_layer: workspace of %zu bytes needed, got %zu", haq_quantize_layer_workspace_bytes(T, K, N, n_e),
                 workspace_bytes);
    // step 1: smoothing vector by grid search; step 2: Hessian-aware quantisation of the folded weight;
    // step 3 on this device is to keep the int8 codes (the caller packs them for the MFMA kernels)
    int rc = haq_smoothing_search(x_fp16, ldx, w, T, K, N, exponents, n_e, use_weight, losses, best, s, workspace, workspace_bytes, stream);
    if (rc != HAQ_OK) return rc;
    return haq_hessian_quant_weight(x_fp16, ldx, T, w, s, K, N, percdamp, wq, w_scale, workspace, workspace_bytes, stream);
}

}  // extern "C"
