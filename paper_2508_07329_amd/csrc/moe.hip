// Routing side of the top-2 expert FFN: router softmax/top-2, the stable token
// permutation that groups (token, expert) pairs by expert, and the weighted
// combination of the two expert outputs of each token.
#include "haq_common.h"
#include "moe.h"

namespace haq {

namespace {

// Top-2 by logit (lowest index wins ties); gate weights are the softmax over all experts,
// renormalised over the two.  The sum runs over the experts in index order so that every
// implementation rounds alike.
__device__ __forceinline__ void route_token(const __half* l, int E, int32_t* idx, float* gw) {
    int i0 = 0;
    float l0 = h2f(l[0]);
    for (int e = 1; e < E; ++e) {
        const float v = h2f(l[e]);
        if (v > l0) {
            l0 = v;
            i0 = e;
        }
    }
    int i1 = (i0 == 0) ? 1 : 0;
    float l1 = h2f(l[i1]);
    for (int e = 0; e < E; ++e) {
        const float v = h2f(l[e]);
        if (e != i0 && v > l1) {
            l1 = v;
            i1 = e;
        }
    }
    float z = 0.0f;
    for (int e = 0; e < E; ++e) z += exp_spec(h2f(l[e]) - l0);
    const float p0 = exp_spec(l0 - l0) / z;
    const float p1 = exp_spec(l1 - l0) / z;
    const float d = p0 + p1;
    idx[0] = i0;
    idx[1] = i1;
    gw[0] = p0 / d;
    gw[1] = p1 / d;
}

struct TabAll {
    ExpertTab e[32];
};

// One work-group does the whole routing side: router top-2 for every token, then a stable
// counting sort of the P = 2T pairs by expert (thread i owns a contiguous run of pair ids, so
// ranks inside an expert follow pair id), and it drops the expert table into device memory
// for the kernels that follow.
constexpr int PERM_THREADS = 256;
__global__ __launch_bounds__(PERM_THREADS) void route_permute_kernel(const __half* logits, int64_t ldl, int T, int E,
                                                                     TabAll tab, ExpertTab* tab_dev, int32_t* idx,
                                                                     float* gw, int32_t* counts, int32_t* offsets,
                                                                     int32_t* perm, int32_t* inv) {
    extern __shared__ int32_t sm[];  // cnt[E][PERM_THREADS], then off[E + 1]
    int32_t* cnt = sm;
    int32_t* off = sm + E * PERM_THREADS;
    const int tid = threadIdx.x;
    const int P = 2 * T;
    if (tid < E) tab_dev[tid] = tab.e[tid];
    for (int t = tid; t < T; t += PERM_THREADS) route_token(logits + (size_t)t * ldl, E, idx + 2 * t, gw + 2 * t);
    __syncthreads();  // idx is re-read below by other threads (global memory, same work-group)
    const int seg = (P + PERM_THREADS - 1) / PERM_THREADS;
    const int lo = min(P, tid * seg), hi = min(P, lo + seg);
    for (int e = 0; e < E; ++e) cnt[e * PERM_THREADS + tid] = 0;
    for (int r = lo; r < hi; ++r) cnt[idx[r] * PERM_THREADS + tid] += 1;
    __syncthreads();
    // exclusive scan over the 256 per-thread counts of each expert: one wave per expert at a
    // time, four counts per lane, lane sums scanned with shuffles
    {
        const int lane = tid & 63, wave = tid >> 6;
        for (int e = wave; e < E; e += PERM_THREADS / 64) {
            int32_t* row = cnt + e * PERM_THREADS + 4 * lane;
            const int c0 = row[0], c1 = row[1], c2 = row[2], c3 = row[3];
            const int sum = c0 + c1 + c2 + c3;
            int incl = sum;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const int v = __shfl_up(incl, o);
                if (lane >= o) incl += v;
            }
            const int excl = incl - sum;
            row[0] = excl;
            row[1] = excl + c0;
            row[2] = excl + c0 + c1;
            row[3] = excl + c0 + c1 + c2;
            if (lane == 63) {
                counts[e] = incl;
                off[e] = incl;  // count for now
            }
        }
    }
    __syncthreads();
    if (tid == 0) {
        int run = 0;
        for (int e = 0; e < E; ++e) {
            const int c = off[e];
            off[e] = run;
            offsets[e] = run;
            run += c;
        }
        off[E] = run;
        offsets[E] = run;
    }
    __syncthreads();
    for (int r = lo; r < hi; ++r) {
        const int e = idx[r];
        const int pos = off[e] + cnt[e * PERM_THREADS + tid]++;
        perm[pos] = r;
        inv[r] = pos;
    }
}

// out[t] = fp16(g0 * y[inv[2t]] + g1 * y[inv[2t+1]]), 8 channels per thread.
__global__ void combine_kernel(const __half* y, int64_t ldy, const int32_t* inv, const float* gw, int T, int H,
                               __half* out, int64_t ldo) {
    const int t = blockIdx.x;
    const float g0 = gw[2 * t], g1 = gw[2 * t + 1];
    const __half* y0 = y + (size_t)inv[2 * t] * ldy;
    const __half* y1 = y + (size_t)inv[2 * t + 1] * ldy;
    for (int c = threadIdx.x * 8; c < H; c += blockDim.x * 8) {
        const uint4 a = *reinterpret_cast<const uint4*>(y0 + c);
        const uint4 b = *reinterpret_cast<const uint4*>(y1 + c);
        const __half* ha = reinterpret_cast<const __half*>(&a);
        const __half* hb = reinterpret_cast<const __half*>(&b);
        uint4 o;
        __half* ho = reinterpret_cast<__half*>(&o);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float v0 = g0 * h2f(ha[i]);
            const float v1 = g1 * h2f(hb[i]);
            ho[i] = f2h(v0 + v1);
        }
        *reinterpret_cast<uint4*>(out + (size_t)t * ldo + c) = o;
    }
}

}  // namespace

int launch_route_permute(const __half* logits, int64_t ldl, int T, int E, const ExpertTab* tab_host, ExpertTab* tab_dev,
                         int32_t* idx, float* gw, int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv,
                         hipStream_t st) {
    TabAll tab{};
    for (int e = 0; e < E; ++e) tab.e[e] = tab_host[e];
    const size_t sm = ((size_t)E * PERM_THREADS + E + 1) * sizeof(int32_t);
    hipLaunchKernelGGL(route_permute_kernel, dim3(1), dim3(PERM_THREADS), sm, st, logits, ldl, T, E, tab, tab_dev, idx, gw,
                       counts, offsets, perm, inv);
    HAQ_CHECK_HIP(hipGetLastError());
    return HAQ_OK;
}

int launch_combine(const __half* y, int64_t ldy, const int32_t* inv, const float* gw, int T, int H, __half* out,
                   int64_t ldo, hipStream_t st) {
    hipLaunchKernelGGL(combine_kernel, dim3(T), dim3(256), 0, st, y, ldy, inv, gw, T, H, out, ldo);
    HAQ_CHECK_HIP(hipGetLastError());
    return HAQ_OK;
}

}  // namespace haq
