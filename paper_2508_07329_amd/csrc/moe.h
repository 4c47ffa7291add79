// Launchers of the routing-side kernels (router, permutation, combine).
#pragma once
#include "haq_common.h"

namespace haq {
int launch_route_permute(const __half* logits, int64_t ldl, int T, int E, const ExpertTab* tab_host, ExpertTab* tab_dev,
                         int32_t* idx, float* gw, int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv,
                         int32_t* blk_counts, hipStream_t st, const ColsumTab* cs_host = nullptr, ColsumTab* cs_dev = nullptr);
// work-groups of the multi-work-group routing path for T tokens (0: the single work-group
// kernel is used); blk_counts holds route_blocks(T) * E entries
int route_blocks(int T);
// One launch for routing, permutation and token quantisation (at most 64 tokens, H <= 8192).
bool decode_prologue_supported(int T, int H);
int launch_decode_prologue(const __half* logits, int64_t ldl, int T, int E, const ExpertTab* tab_host, ExpertTab* tab_dev,
                           int32_t* idx, float* gw, int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv,
                           const __half* x, int64_t ldx, const float* s, int H, int8_t* q_cm, int64_t R, int8_t* q_rm,
                           float* sx_tok, float* sx_sorted, hipStream_t st);
int launch_set_tab(const ExpertTab* tab_host, int E, ExpertTab* tab_dev, hipStream_t st);
int launch_combine(const __half* y, int64_t ldy, const int32_t* inv, const float* gw, int T, int H, __half* out,
                   int64_t ldo, hipStream_t st);
}  // namespace haq
