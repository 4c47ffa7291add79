// Decode path of the routed expert FFN: at most 64 rows per expert, so every
// activated expert's int8 weights are streamed from HBM exactly once and the
// work is bound by that stream (Section III.B.3: experts stay int8 on the GPU to
// relieve memory bandwidth).
//
// Weight fragments go straight from global memory into MFMA operand registers
// (no LDS, and non-temporal loads: nothing is reused): with the chunk-major layout a lane's 16 bytes are
// one output channel's 16 consecutive k, lanes 0-31 cover 32 neighbouring
// channels (512 contiguous bytes) and lanes 32-63 the next k chunk.  The weights
// are the first MFMA operand, the (few) token rows the second, so a lane ends up
// with 16 output channels of one token.  The K range of a unit of output
// channels is split across the waves of a work-group and the exact int32
// partial sums are added through LDS.
#include "haq_common.h"
#include "moe.h"
#include "quant_math.h"
#include "routing.h"

namespace haq {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef const __attribute__((address_space(1))) v4i* gptr_v4i;
__device__ __forceinline__ v4i gload16(const int8_t* p) { return *(gptr_v4i)(uintptr_t)p; }
// weights are read once: streamed past the caches so that the token rows every work-group re-reads stay in L2
__device__ __forceinline__ v4i gload16_stream(const int8_t* p) { return __builtin_nontemporal_load((gptr_v4i)(uintptr_t)p); }

constexpr int GU_WAVES = 4;    // gate/up: 64 packed channels (32 gate + 32 up) per work-group
constexpr int DN_WAVES = 8;    // down with one or two tokens: 32 channels per work-group, K split 8 ways, one work-group per CU
constexpr int DNG_WAVES = 4;   // down, 3..64 tokens: three smaller work-groups per CU, so that one's epilogue and
constexpr int DNG_WGS = 3;     // start-up overlap the others' streaming
constexpr int DNG_DEPTH = 14, DNG_DEPTH2 = 9;
constexpr int GU_DEPTH = 8;    // k-steps of weight fragments in flight per wave (two operands each)
constexpr int DN_DEPTH = 14;
constexpr int GU_DEPTH2 = 5;   // the same with two row blocks per work-group (twice the token fragments)
constexpr int GU_DEPTH_TINY = 5;  // one or two tokens: four work-groups per CU (128 registers), so that the units of two
                                  // experts (896 work-groups at the Mixtral shape) are all resident at once

// blockIdx.y enumerates the experts that hold rows, in index order (the grid has min(E, 2T) of
// them: with one token only two experts can be active, and work-groups that find nothing to do
// would still cost dispatch slots).  Returns -1 past the last active expert.
__device__ __forceinline__ int nth_active_expert(const int32_t* offsets, int E, int j) {
    for (int e = 0; e < E; ++e) {
        if (offsets[e + 1] > offsets[e]) {
            if (j == 0) return e;
            --j;
        }
    }
    return -1;
}

// ---- gate / up projections + SwiGLU + per-unit row maxima of h / s_mid ---------------
// Work-group (unit, j): unit of 64 packed channels of the j-th active expert, all its rows: NRB = 1
// for up to 32 rows, NRB = 2 for 33..64 (two blocks of 32 rows against the same weight fragments, so
// that the weights of every activated expert are streamed exactly once).
//
// XLDS: the token codes and their scales do not come from memory but from LDS (rows of H bytes at
// xl, scales at sxl), where `prep` -- called once the first weight fragments are in flight --
// leaves them; lanes past the last row read the last row (their results are dropped).
//
// ASYM: the token codes are unsigned with a zero point per row (the operand holds code - 128): the
// accumulators are corrected by (128 - zero point) x column sum of the expert's weights before the
// scales are applied, and no partial row maxima are left (the asymmetric requantisation needs the
// row's minimum and maximum and finds them itself).
template <int NRB, int DEPTH, bool XLDS, bool ASYM, class Prep>
__device__ __forceinline__ void gate_up_body(const DecodeArgs& a, const ExpertTab& t, int lo, int m, int unit,
                                             int (*part)[2][16][64], float (*wmax)[32], const int8_t* xl, const float* sxl,
                                             Prep&& prep, const ColsumTab* cs = nullptr) {
    static_assert(!XLDS || NRB == 1, "the LDS variant carries one row block");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hi = lane >> 5;
    const int nchunk = a.H / 16;
    const int cpw = nchunk / GU_WAVES;  // chunks per wave (even)
    const int c0 = wave * cpw + hi;     // this lane's first chunk; it advances by 2 per MFMA
    const int64_t npad = a.Npad13;
    // running pointers to the next k-step to fetch (gate fragment; the up fragment is 512 bytes further;
    // the token rows of the second row block are 32 rows = 512 bytes further)
    const int8_t* pw = t.w13 + ((size_t)c0 * npad + unit * 64 + l32) * 16;
    const size_t wstep = (size_t)2 * npad * 16;
    // lanes past the expert's last row re-read that row (their results are dropped): fewer distinct lines
    const int8_t* px = XLDS ? xl + (size_t)min(l32, m - 1) * a.H + c0 * 16 : a.q_cm + ((size_t)c0 * a.R + lo + min(l32, m - 1)) * 16;
    const int xb1 = (min(32 + l32, m - 1) - min(l32, m - 1)) * 16;  // second row block, relative to the first
    const size_t xstep = XLDS ? 32 : (size_t)2 * a.R * 16;

    v16i accg[NRB], accu[NRB];

    // rolling prefetch: DEPTH k-steps of fragments are always in flight.  Straight-line groups of
    // DEPTH steps (fill, steady state, drain), then a plain loop for what is left.
    const int nks = cpw / 2;
    const int ngroups = nks / DEPTH;
    struct Frag {
        v4i g, u, x[NRB];
    };
    auto fetch = [&](Frag& f) {
        f.g = gload16_stream(pw);
        f.u = gload16_stream(pw + 512);
        pw += wstep;
        if constexpr (!XLDS) {
#pragma unroll
            for (int b = 0; b < NRB; ++b) f.x[b] = gload16(px + xb1 * b);
            px += xstep;
        }
    };
    auto mac = [&](const Frag& f) {
        if constexpr (XLDS) {
            const v4i xv = *reinterpret_cast<const v4i*>(px);
            px += xstep;
            accg[0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f.g, xv, accg[0], 0, 0, 0);
            accu[0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f.u, xv, accu[0], 0, 0, 0);
        } else {
#pragma unroll
            for (int b = 0; b < NRB; ++b) {
                accg[b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f.g, f.x[b], accg[b], 0, 0, 0);
                accu[b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f.u, f.x[b], accu[b], 0, 0, 0);
            }
        }
    };
    Frag fr[DEPTH];
    if (ngroups > 0) {
#pragma unroll
        for (int i = 0; i < DEPTH; ++i) fetch(fr[i]);
    }
    prep();
#pragma unroll
    for (int b = 0; b < NRB; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) accg[b][r] = accu[b][r] = 0;
    if (ngroups > 0) {
        for (int grp = 0; grp + 1 < ngroups; ++grp) {
#pragma unroll
            for (int i = 0; i < DEPTH; ++i) {
                const Frag f = fr[i];
                fetch(fr[i]);
                mac(f);
            }
        }
#pragma unroll
        for (int i = 0; i < DEPTH; ++i) mac(fr[i]);
    }
    for (int k = ngroups * DEPTH; k < nks; ++k) {
        Frag f;
        fetch(f);
        mac(f);
    }
    if constexpr (XLDS) __syncthreads();  // the codes may share LDS with `part`
    // wave w finishes registers 4w..4w+3: channels 8w + 4*hi + 0..3 of the unit, token row l32 of a row block
    const int ch = unit * 32 + 8 * wave + 4 * hi;
    const float4 s1 = *reinterpret_cast<const float4*>(t.sw1 + ch);
    const float4 s3 = *reinterpret_cast<const float4*>(t.sw3 + ch);
    const float4 sm = *reinterpret_cast<const float4*>(t.s_mid + ch);
    const float s1v[4] = {s1.x, s1.y, s1.z, s1.w}, s3v[4] = {s3.x, s3.y, s3.z, s3.w}, smv[4] = {sm.x, sm.y, sm.z, sm.w};
    int c1v[4] = {0, 0, 0, 0}, c3v[4] = {0, 0, 0, 0};
    if constexpr (ASYM) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            c1v[q] = cs->cs1[ch + q];
            c3v[q] = cs->cs3[ch + q];
        }
    }
#pragma unroll
    for (int b = 0; b < NRB; ++b) {
        if (b > 0) __syncthreads();  // part and wmax are reused
        // exact int32 reduction over the K split
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            part[wave][0][r][lane] = accg[b][r];
            part[wave][1][r][lane] = accu[b][r];
        }
        __syncthreads();
        const int row = 32 * b + l32;
        const bool live = row < m;
        const float sx = live ? (XLDS ? sxl[row] : a.sx[lo + row]) : 0.0f;
        int zshift = 0;
        if constexpr (ASYM) zshift = live ? 128 - a.zx[lo + row] : 0;
        __half hv[4];
        float ymax = 0.0f;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            int g = 0, u = 0;
#pragma unroll
            for (int w = 0; w < GU_WAVES; ++w) {
                g += part[w][0][4 * wave + q][lane];
                u += part[w][1][4 * wave + q][lane];
            }
            if constexpr (ASYM) {
                g += zshift * c1v[q];
                u += zshift * c3v[q];
            }
            const float gf = dequant(g, sx, s1v[q]), uf = dequant(u, sx, s3v[q]);
            hv[q] = f2h(silu(gf) * uf);
            if constexpr (!ASYM) ymax = fmaxf(ymax, fabsf(h2f(hv[q]) / smv[q]));
        }
        if (live) *reinterpret_cast<uint2*>(a.mid + (size_t)(lo + row) * a.I + ch) = *reinterpret_cast<const uint2*>(hv);
        if constexpr (ASYM) continue;
        ymax = fmaxf(ymax, __shfl_xor(ymax, 32));
        if (hi == 0) wmax[wave][l32] = ymax;
        __syncthreads();
        // one partial row maximum of |h / s_mid| per (row, unit): reduced by the requantisation kernel
        if (tid < 32 && 32 * b + tid < m) {
            float v = 0.0f;
#pragma unroll
            for (int w = 0; w < GU_WAVES; ++w) v = fmaxf(v, wmax[w][tid]);
            a.pmax[(size_t)(lo + 32 * b + tid) * (a.I / 32) + unit] = v;
        }
    }
}

template <bool ASYM>
__global__ __launch_bounds__(GU_WAVES * 64, 3) void decode_gate_up_kernel(DecodeArgs a) {
    __shared__ int part[GU_WAVES][2][16][64];
    __shared__ float wmax[GU_WAVES][32];
    const int e = a.one_expert ? a.one_expert - 1 : nth_active_expert(a.offsets, a.E, blockIdx.y);
    if (e < 0) return;
    const int lo = a.offsets[e], m = a.offsets[e + 1] - lo;
    const ColsumTab* cs = ASYM ? a.cstab + e : nullptr;
    if (m > 32)  // uniform over the work-group
        gate_up_body<2, GU_DEPTH2, false, ASYM>(a, a.tab[e], lo, m, blockIdx.x, part, wmax, nullptr, nullptr, [] {}, cs);
    else
        gate_up_body<1, GU_DEPTH, false, ASYM>(a, a.tab[e], lo, m, blockIdx.x, part, wmax, nullptr, nullptr, [] {}, cs);
}

// One or two tokens: routing, the stable grouping of the pairs and the quantisation of the
// expert's token rows are repeated by every work-group (cheap next to the 256 KB of weights it
// streams, and hidden behind its first weight fragments), so the layer needs no launch before
// this one.  Work-group (0, 0) leaves the routing results for the kernels that follow.
struct TinyArgs {
    const __half* logits;
    int64_t ldl;
    const __half* x;
    int64_t ldx;
    const float* s;  // smoothing vector of the layer input (null: all ones)
    int T;
    int32_t *idx, *counts, *offsets, *perm, *inv;
    float* gw;
    ExpertTab* tab_dev;
};

template <int NCH>
__global__ __launch_bounds__(GU_WAVES * 64, 4) void decode_tiny_gate_up_kernel(DecodeArgs a, TinyArgs r, TabAll tab) {
    __shared__ int part[GU_WAVES][2][16][64];  // the token codes live here until the K loop is over
    __shared__ float wmax[GU_WAVES][32];
    __shared__ RouteLds rt;
    __shared__ float s_red[GU_WAVES], s_sx[2];
    const int tid = threadIdx.x;
    const int P = 2 * r.T;
    const bool writer = blockIdx.x == 0 && blockIdx.y == 0;  // leaves the routing results (gate weights included)
    route_in_lds(r.logits, r.ldl, r.T, a.E, rt, writer);
    if (writer) {
        if (tid < a.E) {
            r.tab_dev[tid] = tab.e[tid];
            r.counts[tid] = rt.cnt[tid];
        }
        if (tid <= a.E) r.offsets[tid] = rt.off[tid];
        if (tid < P) {
            r.idx[tid] = rt.idx[tid];
            r.gw[tid] = rt.gw[tid];
            r.perm[rt.pos[tid]] = tid;
            r.inv[tid] = rt.pos[tid];
        }
    }
    const int e = nth_active_expert(rt.off, a.E, blockIdx.y);
    if (e < 0) return;
    const int lo = rt.off[e], m = rt.cnt[e];  // m <= 2: one pair per token at most
    int8_t* xq = reinterpret_cast<int8_t*>(part);
    gate_up_body<1, GU_DEPTH_TINY, true, false>(a, tab.e[e], lo, m, blockIdx.x, part, wmax, xq, s_sx, [&] {
#pragma nounroll
        for (int row = 0; row < m; ++row) {
            const int tok = rt.src[lo + row] >> 1;
            const float scale = quantise_row<GU_WAVES * 64, NCH>(r.x + (size_t)tok * r.ldx, r.s, a.H / 16, s_red, [&](int c, uint4 v) {
                *reinterpret_cast<uint4*>(xq + (size_t)row * a.H + c * 16) = v;
            });
            if (tid == 0) s_sx[row] = scale;
        }
        __syncthreads();
    });
}

// ---- requantisation of the intermediate with known partial maxima ------------------------
// One work-group per sorted row, one thread per 16-channel chunk (as many threads as the row
// has chunks, up to 1024): reduce the row's partial maxima, then round h / s_mid / scale; the
// division by the row scale goes through its reciprocal (quant_math.h).
constexpr int RQ_THREADS = 1024;
__global__ __launch_bounds__(RQ_THREADS) void decode_requant_kernel(DecodeArgs a) {
    __shared__ float red[RQ_THREADS / 64];
    const int pos = a.row0 + blockIdx.x;
    int e = 0;
    while (e + 1 < a.E && pos >= a.offsets[e + 1]) ++e;
    const float* s = a.tab[e].s_mid;
    const int tid = threadIdx.x, nu = a.I / 32, nthr = blockDim.x, nwave = nthr >> 6;
    const __half* hrow = a.mid + (size_t)pos * a.I;
    // the row's halves and smoothing entries are fetched before the maximum is known
    const int nchunk = a.I / 16;
    uint4 r0 = make_uint4(0, 0, 0, 0), r1 = r0;
    float sv[16];
    const bool single = nchunk <= nthr;  // one chunk per thread: keep it in registers
    if (single && tid < nchunk) {
        const uint4* px = reinterpret_cast<const uint4*>(hrow + tid * 16);
        r0 = px[0];
        r1 = px[1];
        const float4* ps = reinterpret_cast<const float4*>(s + tid * 16);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float4 v = ps[i];
            sv[4 * i] = v.x;
            sv[4 * i + 1] = v.y;
            sv[4 * i + 2] = v.z;
            sv[4 * i + 3] = v.w;
        }
    }
    float m = 0.0f;
    for (int i = tid; i < nu; i += nthr) m = fmaxf(m, a.pmax[(size_t)pos * nu + i]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    if ((tid & 63) == 0) red[tid >> 6] = m;
    __syncthreads();
    m = 0.0f;
    for (int w = 0; w < nwave; ++w) m = fmaxf(m, red[w]);
    const float scale = m / 127.0f;
    const float rscale = 1.0f / scale;
    const bool sfast = scale >= 0x1p-100f && scale <= 0x1p100f;
    if (tid == 0) a.sh[pos] = scale;
    for (int c = tid; c < nchunk; c += nthr) {
        if (!single && m != 0.0f) {
            const uint4* px = reinterpret_cast<const uint4*>(hrow + c * 16);
            r0 = px[0];
            r1 = px[1];
#pragma unroll
            for (int i = 0; i < 16; ++i) sv[i] = s[c * 16 + i];
        }
        const uint4 v = requant_chunk(r0, r1, sv, m, scale, rscale, sfast);
        *reinterpret_cast<uint4*>(a.hq_cm + ((size_t)c * a.R + pos) * 16) = v;
        if (a.hq_rm) *reinterpret_cast<uint4*>(a.hq_rm + (size_t)pos * a.I + c * 16) = v;
    }
}

// ---- down projection ---------------------------------------------------------------------
// NW waves split K; wave w finishes 16 / NW of the 16 accumulator registers.
// `tid` is the thread's index among the NW * 64 threads that share the unit (threadIdx.x, unless a work-group
// holds several such groups); ylds, if given, also receives the fp16 outputs: ylds[row * 32 + channel of the unit].
// ASYM: codes of the intermediate with a zero point per row, corrected as in the gate/up kernel (cs2: column sums of w2).
template <int NW, int NRB, int DEPTH, bool XLDS, bool ASYM, class Prep>
__device__ __forceinline__ void down_body(const DecodeArgs& a, const ExpertTab& t, int lo, int m, int unit, int (*part)[16][64],
                                          const int8_t* xl, const float* shl, Prep&& prep, int tid, __half* ylds = nullptr,
                                          const int32_t* cs2 = nullptr) {
    static_assert(!XLDS || NRB == 1, "the LDS variant carries one row block");
    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hi = lane >> 5;
    const int nchunk = a.I / 16;
    const int cpw = nchunk / NW;
    const int c0 = wave * cpw + hi;
    const int64_t npad = a.Npad2;
    const int8_t* pw = t.w2 + ((size_t)c0 * npad + unit * 32 + l32) * 16;  // next k-step to fetch
    const size_t wstep = (size_t)2 * npad * 16;
    const int8_t* px = XLDS ? xl + (size_t)min(l32, m - 1) * a.I + c0 * 16 : a.hq_cm + ((size_t)c0 * a.R + lo + min(l32, m - 1)) * 16;
    const int xb1 = (min(32 + l32, m - 1) - min(l32, m - 1)) * 16;  // second row block, relative to the first
    const size_t xstep = XLDS ? 32 : (size_t)2 * a.R * 16;

    v16i acc[NRB];
#pragma unroll
    for (int b = 0; b < NRB; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[b][r] = 0;

    const int nks = cpw / 2;
    const int ngroups = nks / DEPTH;
    struct Frag {
        v4i w, x[NRB];
    };
    auto fetch = [&](Frag& f) {
        f.w = gload16_stream(pw);
        pw += wstep;
        if constexpr (!XLDS) {
#pragma unroll
            for (int b = 0; b < NRB; ++b) f.x[b] = gload16(px + xb1 * b);
            px += xstep;
        }
    };
    auto mac = [&](const Frag& f) {
        if constexpr (XLDS) {
            const v4i xv = *reinterpret_cast<const v4i*>(px);
            px += xstep;
            acc[0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f.w, xv, acc[0], 0, 0, 0);
        } else {
#pragma unroll
            for (int b = 0; b < NRB; ++b) acc[b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f.w, f.x[b], acc[b], 0, 0, 0);
        }
    };
    Frag fr[DEPTH];
    if (ngroups > 0) {
#pragma unroll
        for (int i = 0; i < DEPTH; ++i) fetch(fr[i]);
    }
    prep();
    if (ngroups > 0) {
        for (int grp = 0; grp + 1 < ngroups; ++grp) {
#pragma unroll
            for (int i = 0; i < DEPTH; ++i) {
                const Frag f = fr[i];
                fetch(fr[i]);
                mac(f);
            }
        }
#pragma unroll
        for (int i = 0; i < DEPTH; ++i) mac(fr[i]);
    }
    for (int k = ngroups * DEPTH; k < nks; ++k) {
        Frag f;
        fetch(f);
        mac(f);
    }
    if constexpr (XLDS) __syncthreads();  // the codes may share LDS with `part`
    // register r holds channel 8*(r/4) + 4*hi + r%4 of the unit; wave w finishes registers RPW*w .. RPW*w + RPW-1
    constexpr int RPW = 16 / NW;
    static_assert(RPW == 2 || RPW == 4, "4 or 8 waves");
    const int r0 = RPW * wave;
    const int ch = unit * 32 + 8 * (r0 / 4) + 4 * hi + (r0 % 4);
    float sw[RPW];
#pragma unroll
    for (int q = 0; q < RPW; ++q) sw[q] = t.sw2[ch + q];
    int cv[RPW];
#pragma unroll
    for (int q = 0; q < RPW; ++q) cv[q] = ASYM ? cs2[ch + q] : 0;
#pragma unroll
    for (int b = 0; b < NRB; ++b) {
        if (b > 0) __syncthreads();  // part is reused
#pragma unroll
        for (int r = 0; r < 16; ++r) part[wave][r][lane] = acc[b][r];
        __syncthreads();
        const int row = 32 * b + l32;
        const bool live = row < m;
        const float sh = live ? (XLDS ? shl[row] : a.sh[lo + row]) : 0.0f;
        int zshift = 0;
        if constexpr (ASYM) zshift = live ? 128 - a.zh[lo + row] : 0;
        __half hv[RPW];
#pragma unroll
        for (int q = 0; q < RPW; ++q) {
            int v = 0;
#pragma unroll
            for (int w = 0; w < NW; ++w) v += part[w][r0 + q][lane];
            if constexpr (ASYM) v += zshift * cv[q];
            hv[q] = f2h(dequant(v, sh, sw[q]));
        }
        if (live) {
            __half* dst = a.y + (size_t)(lo + row) * a.H + ch;
            if constexpr (RPW == 2)
                *reinterpret_cast<uint32_t*>(dst) = *reinterpret_cast<const uint32_t*>(hv);
            else
                *reinterpret_cast<uint2*>(dst) = *reinterpret_cast<const uint2*>(hv);
            if (ylds) {
#pragma unroll
                for (int q = 0; q < RPW; ++q) ylds[row * 32 + (ch - unit * 32) + q] = hv[q];
            }
        }
    }
}

template <bool ASYM>
__global__ __launch_bounds__(DNG_WAVES * 64, DNG_WGS) void decode_down_kernel(DecodeArgs a) {
    __shared__ int part[DNG_WAVES][16][64];
    const int e = a.one_expert ? a.one_expert - 1 : nth_active_expert(a.offsets, a.E, blockIdx.y);
    if (e < 0) return;
    const int lo = a.offsets[e], m = a.offsets[e + 1] - lo;
    const int32_t* cs2 = ASYM ? a.cstab[e].cs2 : nullptr;
    if (m > 32)  // uniform over the work-group
        down_body<DNG_WAVES, 2, DNG_DEPTH2, false, ASYM>(a, a.tab[e], lo, m, blockIdx.x, part, nullptr, nullptr, [] {}, threadIdx.x,
                                                         nullptr, cs2);
    else
        down_body<DNG_WAVES, 1, DNG_DEPTH, false, ASYM>(a, a.tab[e], lo, m, blockIdx.x, part, nullptr, nullptr, [] {}, threadIdx.x,
                                                        nullptr, cs2);
}

// One or two tokens: every work-group requantises the expert's one or two rows of the
// intermediate itself (partial row maxima from the gate/up kernel, the arithmetic of
// decode_requant_kernel) while its first weight fragments are in flight, so no launch sits
// between the two projections.
// Requantisation of the m rows of one expert's intermediate into LDS (xq: rows of I codes, s_sh: their
// scales) by the NT threads of a K-split group (partial row maxima from the gate/up kernel, the arithmetic of
// decode_requant_kernel).  Every thread of the work-group must reach the barriers inside; m is the same for
// all groups of a work-group.
template <int NT>
__device__ __forceinline__ void requant_rows_to_lds(const DecodeArgs& a, const ExpertTab& t, int lo, int m, int tid, int8_t* xq,
                                                    float* s_red, float* s_sh) {
    const int nu = a.I / 32, nchunk = a.I / 16;
    for (int row = 0; row < m; ++row) {
        const int pos = lo + row;
        float mx = 0.0f;
        for (int i = tid; i < nu; i += NT) mx = fmaxf(mx, a.pmax[(size_t)pos * nu + i]);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
        __syncthreads();  // an earlier use of s_red is over
        if ((tid & 63) == 0) s_red[tid >> 6] = mx;
        __syncthreads();
        mx = 0.0f;
#pragma unroll
        for (int w = 0; w < NT / 64; ++w) mx = fmaxf(mx, s_red[w]);
        const float scale = mx / 127.0f;
        const float rscale = 1.0f / scale;
        const bool sfast = scale >= 0x1p-100f && scale <= 0x1p100f;
        if (tid == 0) s_sh[row] = scale;
        const __half* hrow = a.mid + (size_t)pos * a.I;
        for (int c = tid; c < nchunk; c += NT) {
            uint4 r0 = make_uint4(0, 0, 0, 0), r1 = r0;
            float sv[16];
            if (mx != 0.0f) {
                const uint4* px = reinterpret_cast<const uint4*>(hrow + c * 16);
                r0 = px[0];
                r1 = px[1];
                const float4* ps = reinterpret_cast<const float4*>(t.s_mid + c * 16);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float4 v = ps[i];
                    sv[4 * i] = v.x;
                    sv[4 * i + 1] = v.y;
                    sv[4 * i + 2] = v.z;
                    sv[4 * i + 3] = v.w;
                }
            }
            *reinterpret_cast<uint4*>(xq + (size_t)row * a.I + c * 16) = requant_chunk(r0, r1, sv, mx, scale, rscale, sfast);
        }
    }
    __syncthreads();
}

__global__ __launch_bounds__(DN_WAVES * 64, 1) void decode_tiny_down_kernel(DecodeArgs a, TabAll tab) {
    __shared__ int part[DN_WAVES][16][64];  // the intermediate's codes live here until the K loop is over
    __shared__ float s_red[DN_WAVES], s_sh[2];
    const int e = nth_active_expert(a.offsets, a.E, blockIdx.y);
    if (e < 0) return;
    const int lo = a.offsets[e], m = a.offsets[e + 1] - lo;
    const ExpertTab& t = tab.e[e];
    int8_t* xq = reinterpret_cast<int8_t*>(part);
    down_body<DN_WAVES, 1, DN_DEPTH, true, false>(
        a, t, lo, m, blockIdx.x, part, xq, s_sh,
        [&] { requant_rows_to_lds<DN_WAVES * 64>(a, t, lo, m, threadIdx.x, xq, s_red, s_sh); }, threadIdx.x);
}

}  // namespace

bool decode_tiny_supported(int T, int H, int I) { return decode_supported(T, H, I) && T <= 2 && H <= 8192 && I <= 16384; }

int launch_decode_tiny(const DecodeArgs& a, const __half* logits, int64_t ldl, const __half* x, int64_t ldx, const float* s, int T,
                       const ExpertTab* tab_host, int32_t* idx, float* gw, int32_t* counts, int32_t* offsets, int32_t* perm,
                       int32_t* inv, ExpertTab* tab_dev, __half* out, bool* combined, hipStream_t st) {
    TabAll tab{};
    for (int e = 0; e < a.E; ++e) tab.e[e] = tab_host[e];
    const TinyArgs r{logits, ldl, x, ldx, s, T, idx, counts, offsets, perm, inv, gw, tab_dev};
    const int P = 2 * T;
    const int ne = a.E < P ? a.E : P;
    const dim3 g1(a.I / 32, ne), g2(a.H / 32, ne);
    if (a.H / 16 <= GU_WAVES * 64)
        hipLaunchKernelGGL(decode_tiny_gate_up_kernel<1>, g1, dim3(GU_WAVES * 64), 0, st, a, r, tab);
    else
        hipLaunchKernelGGL(decode_tiny_gate_up_kernel<2>, g1, dim3(GU_WAVES * 64), 0, st, a, r, tab);
    // Measured and left out (both bit-equal, both slower than three launches at 69.6 us per layer): both experts of a
    // single token in one work-group of 16 waves with the combination formed in LDS (76 us: 128 work-groups do not draw
    // the streaming rate that 256 do); 256 work-groups whose weight operand holds 16 channels of either expert, so that
    // both outputs of a channel meet in one work-group (73.2 us: every work-group then requantises both rows).
    *combined = false;
    (void)out;
    hipLaunchKernelGGL(decode_tiny_down_kernel, g2, dim3(DN_WAVES * 64), 0, st, a, tab);
    HAQ_CHECK_HIP(hipGetLastError());
    return HAQ_OK;
}

bool decode_supported(int T, int H, int I) { return T <= 64 && H % (GU_WAVES * 32) == 0 && I % (DN_WAVES * 32) == 0 && I % (DNG_WAVES * 32) == 0; }

int launch_decode(const DecodeArgs& a, int T, hipStream_t st) {
    const int P = 2 * T;
    const int ne = a.E < P ? a.E : P;  // at most 2T experts can hold rows
    const dim3 g1(a.I / 32, ne), g2(a.H / 32, ne);
    hipLaunchKernelGGL(decode_gate_up_kernel<false>, g1, dim3(GU_WAVES * 64), 0, st, a);
    {
        const int nchunk = a.I / 16;
        const int thr = nchunk >= RQ_THREADS ? RQ_THREADS : (int)round_up(nchunk, 64);
        hipLaunchKernelGGL(decode_requant_kernel, dim3(P), dim3(thr), 0, st, a);
    }
    hipLaunchKernelGGL(decode_down_kernel<false>, g2, dim3(DNG_WAVES * 64), 0, st, a);
    HAQ_CHECK_HIP(hipGetLastError());
    return HAQ_OK;
}

int launch_decode_one_expert(DecodeArgs a, int e, int row0, int m, hipEvent_t before_down, hipStream_t st) {
    if (e < 0 || e >= a.E || m < 1 || m > 64 || row0 < 0) return HAQ_ERR_INVALID_ARG;
    a.one_expert = e + 1;
    a.row0 = row0;
    hipLaunchKernelGGL(decode_gate_up_kernel<false>, dim3(a.I / 32, 1), dim3(GU_WAVES * 64), 0, st, a);
    const int nchunk = a.I / 16;
    const int thr = nchunk >= RQ_THREADS ? RQ_THREADS : (int)round_up(nchunk, 64);
    hipLaunchKernelGGL(decode_requant_kernel, dim3(m), dim3(thr), 0, st, a);
    if (before_down) HAQ_CHECK_HIP(hipStreamWaitEvent(st, before_down, 0));
    hipLaunchKernelGGL(decode_down_kernel<false>, dim3(a.H / 32, 1), dim3(DNG_WAVES * 64), 0, st, a);
    HAQ_CHECK_HIP(hipGetLastError());
    return HAQ_OK;
}

int launch_decode_gate_up_asym(const DecodeArgs& a, int T, hipStream_t st) {
    if (!a.zx || !a.cstab) return HAQ_ERR_INVALID_ARG;
    const int P = 2 * T;
    const int ne = a.E < P ? a.E : P;
    hipLaunchKernelGGL(decode_gate_up_kernel<true>, dim3(a.I / 32, ne), dim3(GU_WAVES * 64), 0, st, a);
    HAQ_CHECK_HIP(hipGetLastError());
    return HAQ_OK;
}

int launch_decode_down_asym(const DecodeArgs& a, int T, hipStream_t st) {
    if (!a.zh || !a.cstab) return HAQ_ERR_INVALID_ARG;
    const int P = 2 * T;
    const int ne = a.E < P ? a.E : P;
    hipLaunchKernelGGL(decode_down_kernel<true>, dim3(a.H / 32, ne), dim3(DNG_WAVES * 64), 0, st, a);
    HAQ_CHECK_HIP(hipGetLastError());
    return HAQ_OK;
}

}  // namespace haq
