// Routing side of the top-2 expert FFN: router softmax/top-2, the stable token
// permutation that groups (token, expert) pairs by expert, and the weighted
// combination of the two expert outputs of each token.
#include "haq_common.h"
#include "moe.h"
#include "quant_math.h"
#include "routing.h"

namespace haq {

namespace {

struct ColsumAll {
    ColsumTab e[32];
};

// One work-group does the whole routing side: router top-2 for every token, then a stable
// counting sort of the P = 2T pairs by expert (thread i owns a contiguous run of pair ids, so
// ranks inside an expert follow pair id), and it drops the expert table into device memory
// for the kernels that follow.
constexpr int PERM_THREADS = 256;
constexpr int ROUTE_SINGLE_MAX = 256;  // longer batches take the multi-work-group kernels
__global__ __launch_bounds__(PERM_THREADS) void route_permute_kernel(const __half* logits, int64_t ldl, int T, int E,
                                                                     TabAll tab, ExpertTab* tab_dev, int32_t* idx,
                                                                     float* gw, int32_t* counts, int32_t* offsets,
                                                                     int32_t* perm, int32_t* inv, ColsumAll cs, ColsumTab* cs_dev) {
    extern __shared__ int32_t sm[];  // cnt[E][PERM_THREADS], then off[E + 1]
    int32_t* cnt = sm;
    int32_t* off = sm + E * PERM_THREADS;
    const int tid = threadIdx.x;
    const int P = 2 * T;
    if (tid < E) {
        tab_dev[tid] = tab.e[tid];
        if (cs_dev) cs_dev[tid] = cs.e[tid];  // asymmetric codes: the experts' column-sum table travels the same way
    }
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


// ---- the same result with many work-groups (long token batches) -------------------------
// Kernel 1: one thread per token routes it; the work-group leaves its expert histogram.
// Kernel 2: every work-group sums the histograms of the work-groups before it (that is the
// rank base of its pairs inside each expert), ranks its own pairs with wave ballots -- a
// token holds at most one pair per expert, so the rank of a pair among equal experts is the
// number of earlier tokens that use that expert -- and scatters perm / inv.
constexpr int RT_THREADS = 256;
__global__ __launch_bounds__(RT_THREADS) void route_count_kernel(const __half* logits, int64_t ldl, int T, int E,
                                                                 int32_t* idx, float* gw, int32_t* blk_counts) {
    __shared__ int32_t hist[32];
    const int tid = threadIdx.x, t = blockIdx.x * RT_THREADS + tid;
    if (tid < 32) hist[tid] = 0;
    __syncthreads();
    if (t < T) {
        int32_t id2[2];
        float g2[2];
        route_token(logits + (size_t)t * ldl, E, id2, g2);
        idx[2 * t] = id2[0];
        idx[2 * t + 1] = id2[1];
        gw[2 * t] = g2[0];
        gw[2 * t + 1] = g2[1];
        atomicAdd(&hist[id2[0]], 1);  // integer counts: the order of the additions is immaterial
        atomicAdd(&hist[id2[1]], 1);
    }
    __syncthreads();
    if (tid < E) blk_counts[blockIdx.x * E + tid] = hist[tid];
}

__global__ __launch_bounds__(RT_THREADS) void permute_kernel(int T, int E, TabAll tab, ExpertTab* tab_dev,
                                                             const int32_t* idx, const int32_t* blk_counts, int nblk,
                                                             int32_t* counts, int32_t* offsets, int32_t* perm,
                                                             int32_t* inv, ColsumAll cs, ColsumTab* cs_dev) {
    __shared__ int32_t total[32], before[32], base[32];
    __shared__ int32_t wave_cnt[RT_THREADS / 64][32];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid < E) {
        int bef = 0, tot = 0;
        for (int b = 0; b < nblk; ++b) {
            const int c = blk_counts[b * E + tid];
            if (b < (int)blockIdx.x) bef += c;
            tot += c;
        }
        total[tid] = tot;
        before[tid] = bef;
        if (blockIdx.x == 0) {
            tab_dev[tid] = tab.e[tid];
            if (cs_dev) cs_dev[tid] = cs.e[tid];
            counts[tid] = tot;
        }
    }
    __syncthreads();
    if (tid == 0) {
        int run = 0;
        for (int e = 0; e < E; ++e) {
            base[e] = run + before[e];
            if (blockIdx.x == 0) offsets[e] = run;
            run += total[e];
        }
        if (blockIdx.x == 0) offsets[E] = run;
    }
    const int t = blockIdx.x * RT_THREADS + tid;
    const bool valid = t < T;
    const int e0 = valid ? idx[2 * t] : -1, e1 = valid ? idx[2 * t + 1] : -1;
    int r0 = 0, r1 = 0;
    for (int e = 0; e < E; ++e) {
        const unsigned long long mask = __ballot(e0 == e || e1 == e);
        const int below = __popcll(mask & ((1ull << lane) - 1ull));
        if (lane == 0) wave_cnt[wave][e] = __popcll(mask);
        if (e0 == e) r0 = below;
        if (e1 == e) r1 = below;
    }
    __syncthreads();
    if (valid) {
        for (int w = 0; w < wave; ++w) {
            r0 += wave_cnt[w][e0];
            r1 += wave_cnt[w][e1];
        }
        const int p0 = base[e0] + r0, p1 = base[e1] + r1;
        perm[p0] = 2 * t;
        inv[2 * t] = p0;
        perm[p1] = 2 * t + 1;
        inv[2 * t + 1] = p1;
    }
}

// Rewrites the device copy of the expert table (the staging slot of a streamed expert is only
// known once the routing histogram is back on the host).
__global__ void set_tab_kernel(TabAll tab, int E, ExpertTab* tab_dev) {
    if ((int)threadIdx.x < E) tab_dev[threadIdx.x] = tab.e[threadIdx.x];
}


// ---- decode prologue: routing, permutation and token quantisation in one launch ------------------
// For at most 64 tokens.  Work-group p produces sorted row p (one (token, expert) pair): every
// work-group repeats the routing of all tokens and the stable counting sort in LDS (a few hundred
// operations), finds the pair that lands on its row, and quantises that token with the shared
// smoothing vector (same arithmetic as the activation-quantisation kernels).  Work-group 0 also
// writes the routing results and the expert table.  NCH = 16-channel chunks per thread.
struct PrologueArgs {
    const __half* logits;
    int64_t ldl;
    int T, E;
    ExpertTab* tab_dev;
    int32_t *idx, *counts, *offsets, *perm, *inv;
    float* gw;
    const __half* x;
    int64_t ldx;
    const float* s;
    int H;
    int8_t* q_cm;
    int64_t R;
    int8_t* q_rm;      // optional dense [T x H]
    int64_t ldq;
    float* sx_tok;     // optional [T]
    float* sx_sorted;  // [2T]
};

constexpr int PRO_THREADS = 256, PRO_MAXP = ROUTE_LDS_MAXP;
template <int NCH>
__global__ __launch_bounds__(PRO_THREADS) void decode_prologue_kernel(PrologueArgs a, TabAll tab) {
    __shared__ RouteLds r;
    __shared__ float s_red[PRO_THREADS / 64];
    const int tid = threadIdx.x;
    const int P = 2 * a.T;
    route_in_lds(a.logits, a.ldl, a.T, a.E, r, blockIdx.x == 0);  // only work-group 0 writes the gate weights
    if (blockIdx.x == 0) {
        if (tid < a.E) {
            a.tab_dev[tid] = tab.e[tid];
            a.counts[tid] = r.cnt[tid];
        }
        if (tid <= a.E) a.offsets[tid] = r.off[tid];
        if (tid < P) {
            a.idx[tid] = r.idx[tid];
            a.gw[tid] = r.gw[tid];
            a.perm[r.pos[tid]] = tid;
            a.inv[tid] = r.pos[tid];
        }
    }
    // ---- quantise the token of this row
    const int p = blockIdx.x, t = r.src[p] >> 1;
    const float scale = quantise_row<PRO_THREADS, NCH>(a.x + (size_t)t * a.ldx, a.s, a.H / 16, s_red, [&](int c, uint4 v) {
        if (a.q_rm) *reinterpret_cast<uint4*>(a.q_rm + (size_t)t * a.ldq + c * 16) = v;
        *reinterpret_cast<uint4*>(a.q_cm + ((size_t)c * a.R + p) * 16) = v;
    });
    if (tid == 0) {
        a.sx_sorted[p] = scale;
        if (a.sx_tok) a.sx_tok[t] = scale;
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

int route_blocks(int T) { return T > ROUTE_SINGLE_MAX ? cdiv(T, RT_THREADS) : 0; }

int launch_route_permute(const __half* logits, int64_t ldl, int T, int E, const ExpertTab* tab_host, ExpertTab* tab_dev,
                         int32_t* idx, float* gw, int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv,
                         int32_t* blk_counts, hipStream_t st, const ColsumTab* cs_host, ColsumTab* cs_dev) {
    TabAll tab{};
    for (int e = 0; e < E; ++e) tab.e[e] = tab_host[e];
    ColsumAll cs{};
    if (cs_host && cs_dev)
        for (int e = 0; e < E; ++e) cs.e[e] = cs_host[e];
    else
        cs_dev = nullptr;
    if (const int nblk = route_blocks(T)) {
        hipLaunchKernelGGL(route_count_kernel, dim3(nblk), dim3(RT_THREADS), 0, st, logits, ldl, T, E, idx, gw, blk_counts);
        hipLaunchKernelGGL(permute_kernel, dim3(nblk), dim3(RT_THREADS), 0, st, T, E, tab, tab_dev, (const int32_t*)idx,
                           (const int32_t*)blk_counts, nblk, counts, offsets, perm, inv, cs, cs_dev);
        HAQ_CHECK_HIP(hipGetLastError());
        return HAQ_OK;
    }
    const size_t sm = ((size_t)E * PERM_THREADS + E + 1) * sizeof(int32_t);
    hipLaunchKernelGGL(route_permute_kernel, dim3(1), dim3(PERM_THREADS), sm, st, logits, ldl, T, E, tab, tab_dev, idx, gw,
                       counts, offsets, perm, inv, cs, cs_dev);
    HAQ_CHECK_HIP(hipGetLastError());
    return HAQ_OK;
}

bool decode_prologue_supported(int T, int H) { return T >= 1 && 2 * T <= PRO_MAXP && H % 16 == 0 && H / 16 <= 2 * PRO_THREADS; }

int launch_decode_prologue(const __half* logits, int64_t ldl, int T, int E, const ExpertTab* tab_host, ExpertTab* tab_dev,
                           int32_t* idx, float* gw, int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv,
                           const __half* x, int64_t ldx, const float* s, int H, int8_t* q_cm, int64_t R, int8_t* q_rm,
                           float* sx_tok, float* sx_sorted, hipStream_t st) {
    TabAll tab{};
    for (int e = 0; e < E; ++e) tab.e[e] = tab_host[e];
    PrologueArgs a{logits, ldl, T, E, tab_dev, idx, counts, offsets, perm, inv, gw, x, ldx, s, H, q_cm, R, q_rm, H, sx_tok, sx_sorted};
    if (H / 16 <= PRO_THREADS)
        hipLaunchKernelGGL(decode_prologue_kernel<1>, dim3(2 * T), dim3(PRO_THREADS), 0, st, a, tab);
    else
        hipLaunchKernelGGL(decode_prologue_kernel<2>, dim3(2 * T), dim3(PRO_THREADS), 0, st, a, tab);
    HAQ_CHECK_HIP(hipGetLastError());
    return HAQ_OK;
}

int launch_set_tab(const ExpertTab* tab_host, int E, ExpertTab* tab_dev, hipStream_t st) {
    TabAll tab{};
    for (int e = 0; e < E; ++e) tab.e[e] = tab_host[e];
    hipLaunchKernelGGL(set_tab_kernel, dim3(1), dim3(64), 0, st, tab, E, tab_dev);
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
