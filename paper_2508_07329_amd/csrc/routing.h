// Router arithmetic and the in-LDS routing of short batches, shared by the kernels that route
// inside a larger launch (top-2 softmax gating, then the stable grouping of pairs by expert).
#pragma once
#include "haq_common.h"

namespace haq {

struct TabAll {  // the expert table as a kernel argument
    ExpertTab e[32];
};

#ifdef __HIPCC__
// Top-2 by logit (lowest index wins ties); gate weights are the softmax over all experts,
// renormalised over the two.  The sum runs over the experts in index order so that every
// implementation rounds alike.  All logits of the token (E <= 32) are fetched into registers with
// independent loads first, so the serial comparisons and the sum wait for memory once.
__device__ __forceinline__ void route_token(const __half* l, int E, int32_t* idx, float* gw, bool need_gw = true) {
    float v[32];
#pragma unroll
    for (int e = 0; e < 32; ++e) v[e] = h2f(l[e < E ? e : E - 1]);
    int i0 = 0;
    float l0 = v[0];
#pragma unroll
    for (int e = 1; e < 32; ++e) {
        if (e < E && v[e] > l0) {
            l0 = v[e];
            i0 = e;
        }
    }
    int i1 = (i0 == 0) ? 1 : 0;
    float l1 = (i0 == 0) ? v[1] : v[0];
#pragma unroll
    for (int e = 0; e < 32; ++e) {
        if (e < E && e != i0 && v[e] > l1) {
            l1 = v[e];
            i1 = e;
        }
    }
    idx[0] = i0;
    idx[1] = i1;
    if (!need_gw) return;  // the caller only needs to know which experts
    float z = 0.0f;
#pragma unroll
    for (int e = 0; e < 32; ++e)
        if (e < E) z += exp_spec(v[e] - l0);
    const float p0 = exp_spec(l0 - l0) / z;
    const float p1 = exp_spec(l1 - l0) / z;
    const float d = p0 + p1;
    gw[0] = p0 / d;
    gw[1] = p1 / d;
}

// Routing of T <= 64 tokens and the stable counting sort of their P = 2T pairs by expert, done by
// one work-group of at least 128 threads entirely in LDS (cheap enough for every work-group of a
// launch to repeat): idx/gw by pair id, cnt/off by expert, pos = sorted row of a pair, src = pair
// of a sorted row (gw only if need_gw: the softmax is the longest dependent chain of the routing and
// most callers inside a larger launch only need the grouping).  Thread p holds pair p; its rank among the pairs of the same expert is the
// number of lower lanes of its wave that vote for that expert, plus all of wave 0's for a pair of
// wave 1.  Ends with a barrier.
constexpr int ROUTE_LDS_MAXP = 128;
struct RouteLds {
    int32_t idx[ROUTE_LDS_MAXP], pos[ROUTE_LDS_MAXP], src[ROUTE_LDS_MAXP], cnt[33], off[33], wcnt[2][32];
    float gw[ROUTE_LDS_MAXP];
};
__device__ __forceinline__ void route_in_lds(const __half* logits, int64_t ldl, int T, int E, RouteLds& r, bool need_gw = true) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int P = 2 * T;
    if (tid < T) {
        int32_t id2[2];
        float g2[2] = {0.0f, 0.0f};
        route_token(logits + (size_t)tid * ldl, E, id2, g2, need_gw);
        r.idx[2 * tid] = id2[0];
        r.idx[2 * tid + 1] = id2[1];
        r.gw[2 * tid] = g2[0];
        r.gw[2 * tid + 1] = g2[1];
    }
    __syncthreads();
    const int my_e = tid < P ? r.idx[tid] : -1;
    int my_rank = 0;
    for (int e = 0; e < E; ++e) {
        const unsigned long long votes = __ballot(my_e == e);
        if (my_e == e) my_rank = __popcll(votes & ((1ull << lane) - 1ull));
        if (lane == 0 && wave < 2) r.wcnt[wave][e] = __popcll(votes);
    }
    __syncthreads();
    if (tid <= E) {  // thread e: count of expert e and the sum of the counts before it
        int run = 0;
        for (int e = 0; e < tid; ++e) run += r.wcnt[0][e] + r.wcnt[1][e];
        r.off[tid] = run;
        if (tid < E) r.cnt[tid] = r.wcnt[0][tid] + r.wcnt[1][tid];
    }
    __syncthreads();
    if (tid < P) {
        const int pos = r.off[my_e] + my_rank + (wave == 1 ? r.wcnt[0][my_e] : 0);
        r.pos[tid] = pos;
        r.src[pos] = tid;
    }
    __syncthreads();
}
#endif

}  // namespace haq
