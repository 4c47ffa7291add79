// Activation quantisation (Eq. 1, Q(s^-1 X), scale on the token dimension) and
// the offline weight-side kernels (Q(W s), per-channel magnitudes, packing).
#include "haq_common.h"
#include "quant_math.h"

#include <mutex>

namespace haq {

namespace {

constexpr int QMAX_THREADS = 1024;

// Two-pass kernel for rows longer than 16 * QMAX_THREADS channels.
// Work-group = 8 consecutive output rows of one expert group (or of the matrix).  Threads
// form G row groups x CL chunk lanes: thread (g, c) owns the 16-channel chunks c, c + CL, ...
// of RS = 8 / G rows, so the reciprocals of the smoothing vector are formed once per chunk
// for RS rows, a wave reads 2 KB contiguous per row, and the 8 rows of one chunk fill one
// 128-byte line of the chunk-major output from inside one work-group.  Pass 1 reduces the
// row absmax of y = x / s (lane shuffles, then across the waves of a row group through
// LDS); pass 2 re-reads the rows (L2 resident), rounds y / scale and writes 16 codes per
// chunk.  With `gather` the rows are read through a permutation (sorted pair -> token).
constexpr int QBLOCK_ROWS = 8;
template <int RS>
__global__ __launch_bounds__(QMAX_THREADS) void smooth_quant_kernel(QuantArgs a, int CL) {
    __shared__ float red[QMAX_THREADS / 64][RS];
    const int tid = threadIdx.x;
    const int c0 = tid % CL, g = tid / CL;
    const int waves_per_group = CL >> 6, wave = tid >> 6;
    const int nchunk = a.K / 16;
    // rows of this work-group: [row0, row_end), never straddling two expert groups
    int row0, row_end;
    const float* s = a.s;
    if (a.tab) {
        int b = blockIdx.x, i = 0, e = 0;
        row0 = row_end = 0;
        for (; i < a.n_sel; ++i) {
            e = a.sel[i];
            const int lo = a.offsets[e], hi = a.offsets[e + 1];
            const int nb = (hi - lo + QBLOCK_ROWS - 1) / QBLOCK_ROWS;
            if (b < nb) {
                row0 = lo + b * QBLOCK_ROWS;
                row_end = hi;
                break;
            }
            b -= nb;
        }
        if (i == a.n_sel) return;  // the grid is an upper bound
        s = a.tab[e].s_mid;
    } else {
        row0 = blockIdx.x * QBLOCK_ROWS;
        row_end = a.T;
    }
    row0 += g * RS;  // first row of this thread's row group
    const int nrow = min(RS, row_end - row0);  // may be <= 0
    const __half* xrow[RS];
#pragma unroll
    for (int r = 0; r < RS; ++r) {
        int src = row0 + (r < nrow ? r : 0);
        if (nrow <= 0) src = 0;
        if (a.gather) src = a.gather[src] >> 1;
        xrow[r] = a.x + (size_t)src * a.ldx;
    }

    float amax[RS];
#pragma unroll
    for (int r = 0; r < RS; ++r) amax[r] = 0.0f;
    float sv[16], rv[16], x[16];
    for (int c = c0; c < nchunk; c += CL) {
        bool fast = true;
        if (s) fast = load_s16(s, c, sv, rv);
#pragma unroll
        for (int r = 0; r < RS; ++r) {
            if (r < nrow) {
                load_x16(xrow[r], c, x);
                float m = amax[r];
                if (!s) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) m = fmaxf(m, fabsf(x[i]));
                } else if (fast) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) m = fmaxf(m, fabsf(div_by(x[i], sv[i], rv[i], true)));
                } else {
#pragma unroll
                    for (int i = 0; i < 16; ++i) m = fmaxf(m, fabsf(x[i] / sv[i]));
                }
                amax[r] = m;
            }
        }
    }
#pragma unroll
    for (int r = 0; r < RS; ++r) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) amax[r] = fmaxf(amax[r], __shfl_xor(amax[r], o));
    }
    if ((tid & 63) == 0) {
#pragma unroll
        for (int r = 0; r < RS; ++r) red[wave][r] = amax[r];
    }
    __syncthreads();
    float scale[RS], rscale[RS];
    bool sfast[RS];
#pragma unroll
    for (int r = 0; r < RS; ++r) {
        float m = 0.0f;
        for (int w = 0; w < waves_per_group; ++w) m = fmaxf(m, red[g * waves_per_group + w][r]);
        amax[r] = m;
        scale[r] = m / 127.0f;
        rscale[r] = 1.0f / scale[r];
        sfast[r] = scale[r] >= 0x1p-100f && scale[r] <= 0x1p100f;
    }
    if (c0 < nrow) {
        const int t = row0 + c0;
        float sc = 0.0f;
#pragma unroll
        for (int r = 0; r < RS; ++r)
            if (r == c0) sc = scale[r];
        if (a.scale_dest) a.scale_dest[t] = sc;
        if (a.scale) a.scale[a.gather ? (a.gather[t] >> 1) : t] = sc;
    }
    for (int c = c0; c < nchunk; c += CL) {
        bool fast = true;
        if (s) fast = load_s16(s, c, sv, rv);
#pragma unroll
        for (int r = 0; r < RS; ++r) {
            if (r < nrow) {
                const int t = row0 + r;
                uint32_t w[4] = {0, 0, 0, 0};
                if (amax[r] != 0.0f) {
                    load_x16(xrow[r], c, x);
                    if (fast && sfast[r]) {  // the common case: both divisions through reciprocals
#pragma unroll
                        for (int i = 0; i < 16; ++i) {
                            const float y = s ? div_by(x[i], sv[i], rv[i], true) : x[i];
                            float q = rintf(div_by(y, scale[r], rscale[r], true));
                            q = fminf(fmaxf(q, -127.0f), 127.0f);
                            w[i / 4] |= (uint32_t)((int)q & 0xff) << (8 * (i % 4));
                        }
                    } else {
#pragma unroll
                        for (int i = 0; i < 16; ++i) {
                            const float y = s ? x[i] / sv[i] : x[i];
                            float q = rintf(y / scale[r]);
                            q = fminf(fmaxf(q, -127.0f), 127.0f);
                            w[i / 4] |= (uint32_t)((int)q & 0xff) << (8 * (i % 4));
                        }
                    }
                }
                const uint4 v = make_uint4(w[0], w[1], w[2], w[3]);
                if (a.q_rm) {
                    const int tr = a.gather ? (a.gather[t] >> 1) : t;
                    *reinterpret_cast<uint4*>(a.q_rm + (size_t)tr * a.ldq + c * 16) = v;
                }
                if (a.q_cm) *reinterpret_cast<uint4*>(a.q_cm + ((size_t)c * a.R + t) * 16) = v;
            }
        }
    }
}

// Single-pass kernel for K <= 16 * QMAX_THREADS: thread (g, c) owns exactly one 16-channel
// chunk of RS rows and keeps the raw halves in registers between the absmax reduction and
// the rounding, so every row is read from memory once.
template <int RS>
__global__ __launch_bounds__(QMAX_THREADS) void smooth_quant_reg_kernel(QuantArgs a, int CL) {
    __shared__ float red[QMAX_THREADS / 64][RS];
    const int tid = threadIdx.x;
    const int c = tid % CL, g = tid / CL;
    const int brows = (blockDim.x / CL) * RS;  // rows per work-group
    const int waves_per_group = CL >> 6, wave = tid >> 6;
    const int nchunk = a.K / 16;
    int row0, row_end;
    const float* s = a.s;
    if (a.tab) {
        int b = blockIdx.x, i = 0, e = 0;
        row0 = row_end = 0;
        for (; i < a.n_sel; ++i) {
            e = a.sel[i];
            const int lo = a.offsets[e], hi = a.offsets[e + 1];
            const int nb = (hi - lo + brows - 1) / brows;
            if (b < nb) {
                row0 = lo + b * brows;
                row_end = hi;
                break;
            }
            b -= nb;
        }
        if (i == a.n_sel) return;  // the grid is an upper bound
        s = a.tab[e].s_mid;
    } else {
        row0 = blockIdx.x * brows;
        row_end = a.T;
    }
    row0 += g * RS;
    const int nrow = min(RS, row_end - row0);  // may be <= 0
    const bool active = c < nchunk;
    uint4 raw[RS][2];
#pragma unroll
    for (int r = 0; r < RS; ++r) {
        raw[r][0] = raw[r][1] = make_uint4(0, 0, 0, 0);
        if (active && r < nrow) {
            int src = row0 + r;
            if (a.gather) src = a.gather[src] >> 1;
            const uint4* px = reinterpret_cast<const uint4*>(a.x + (size_t)src * a.ldx + c * 16);
            raw[r][0] = px[0];
            raw[r][1] = px[1];
        }
    }
    float sv[16], rv[16];
    bool fast = true;
    if (s && active) fast = load_s16(s, c, sv, rv);
    auto unpack = [&](int r, float (&x)[16]) {
        Half8 h0, h1;
        *reinterpret_cast<uint4*>(&h0) = raw[r][0];
        *reinterpret_cast<uint4*>(&h1) = raw[r][1];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            x[i] = h2f(h0.v[i]);
            x[8 + i] = h2f(h1.v[i]);
        }
    };
    float amax[RS];
    float x[16];
#pragma unroll
    for (int r = 0; r < RS; ++r) {
        float m = 0.0f;
        unpack(r, x);
        if (!s) {
#pragma unroll
            for (int i = 0; i < 16; ++i) m = fmaxf(m, fabsf(x[i]));
        } else if (fast) {
#pragma unroll
            for (int i = 0; i < 16; ++i) m = fmaxf(m, fabsf(div_by(x[i], sv[i], rv[i], true)));
        } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) m = fmaxf(m, fabsf(x[i] / sv[i]));
        }
        amax[r] = m;
    }
#pragma unroll
    for (int r = 0; r < RS; ++r) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) amax[r] = fmaxf(amax[r], __shfl_xor(amax[r], o));
    }
    if ((tid & 63) == 0) {
#pragma unroll
        for (int r = 0; r < RS; ++r) red[wave][r] = amax[r];
    }
    __syncthreads();
    if (!active) return;
    // the rounding pass recomputes x / s from the raw halves; the empty asm keeps the
    // compiler from carrying the 16 * RS quotients of the first pass across the barrier
#pragma unroll
    for (int r = 0; r < RS; ++r) {
#pragma unroll
        for (int h = 0; h < 2; ++h)
            asm volatile("" : "+v"(raw[r][h].x), "+v"(raw[r][h].y), "+v"(raw[r][h].z), "+v"(raw[r][h].w));
    }
#pragma unroll
    for (int r = 0; r < RS; ++r) {
        if (r < nrow) {
            // every thread of the row group derives the row's scale from the per-wave maxima
            float m = 0.0f;
            for (int w = 0; w < waves_per_group; ++w) m = fmaxf(m, red[g * waves_per_group + w][r]);
            const float scale = m / 127.0f;
            const float rscale = 1.0f / scale;
            const bool sfast = scale >= 0x1p-100f && scale <= 0x1p100f;
            const int t = row0 + r;
            if (c == r) {
                if (a.scale_dest) a.scale_dest[t] = scale;
                if (a.scale) a.scale[a.gather ? (a.gather[t] >> 1) : t] = scale;
            }
            uint32_t w[4] = {0, 0, 0, 0};
            if (m != 0.0f) {
                unpack(r, x);
                if (fast && sfast) {  // the common case: both divisions through reciprocals
                    float q[16];
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const float y = s ? div_by(x[i], sv[i], rv[i], true) : x[i];
                        q[i] = div_by(y, scale, rscale, true);
                    }
#pragma unroll
                    for (int i = 0; i < 4; ++i) w[i] = round_pack4(q[4 * i], q[4 * i + 1], q[4 * i + 2], q[4 * i + 3]);
                } else {
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const float y = s ? x[i] / sv[i] : x[i];
                        float q = rintf(y / scale);
                        q = fminf(fmaxf(q, -127.0f), 127.0f);
                        w[i / 4] |= (uint32_t)((int)q & 0xff) << (8 * (i % 4));
                    }
                }
            }
            const uint4 v = make_uint4(w[0], w[1], w[2], w[3]);
            if (a.q_rm) {
                const int tr = a.gather ? (a.gather[t] >> 1) : t;
                *reinterpret_cast<uint4*>(a.q_rm + (size_t)tr * a.ldq + c * 16) = v;
            }
            if (a.q_cm) *reinterpret_cast<uint4*>(a.q_cm + ((size_t)c * a.R + t) * 16) = v;
        }
    }
}


// Pipelined single pass for K <= 16 * QMAX_THREADS.  Thread (g, c) owns one 16-channel chunk
// (reciprocals of the smoothing vector formed once per work-group) and walks over a run of
// slabs of RS rows per row group; the halves of the next slab are fetched into registers while
// the current slab is reduced and rounded.  Every row is read from memory once.
//
// The chunk-major output keeps the 16 bytes of consecutive rows of one chunk side by side, so a
// thread that stored its own codes would write 16 bytes per row, 64 different cache lines per store
// instruction (measured: a third of the kernel's time).  The codes of up to QSTAGE rows are therefore
// staged in LDS and written out transposed: eight neighbouring lanes write the 16-byte pieces of
// eight consecutive rows of one chunk, i.e. whole 128-byte lines when the rows are aligned.
constexpr int QSTAGE = 8;
__host__ __device__ inline int qstage_rows(int slab) { return slab > QSTAGE ? slab : QSTAGE; }
// row pitch of the staging area in bytes: 8 (mod 16) pieces of 16 bytes, so that the transposed
// reads of eight rows x eight chunks spread evenly over the banks
__host__ __device__ inline int qstage_pitch(int nchunk) { return (nchunk + ((24 - nchunk % 16) % 16)) * 16; }

//
// ASYM: unsigned codes with a zero point per row (range of the row widened to contain 0, scale = range / 255,
// zero point = rne(-min / scale)); the packed operand holds code - 128, the optional row-major output the codes.
template <int RS, bool ASYM>
__global__ __launch_bounds__(QMAX_THREADS) void smooth_quant_lds_kernel(QuantArgs a, int CL) {
    extern __shared__ __attribute__((aligned(1024))) uint8_t qlds[];
    const int nthr = blockDim.x;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = tid % CL, g = tid / CL;
    const int G = nthr / CL;
    const int waves_per_group = CL >> 6;
    const int nchunk = a.K / 16;
    const int slab = G * RS;
    const int srows = qstage_rows(slab), pitch = qstage_pitch(nchunk);
    float* red = reinterpret_cast<float*>(qlds + (size_t)srows * pitch);  // [2][QMAX_THREADS / 64][RS] maxima (ASYM: then minima)
    constexpr int RED_HALF = 2 * (QMAX_THREADS / 64) * RS;
    // Slabs per work-group: the grid is fixed (one work-group per CU); every group (expert)
    // is cut into runs of `nit` slabs, so no work-group does more than nit slabs whatever the
    // group sizes are, and sum_e ceil(slabs_e / nit) <= total / nit + groups <= grid.
    int nit;
    if (a.tab) {
        int total = 0;
        for (int i = 0; i < a.n_sel; ++i) {
            const int e = a.sel[i];
            total += (a.offsets[e + 1] - a.offsets[e] + slab - 1) / slab;
        }
        const int avail = max(1, (int)gridDim.x - a.n_sel);
        nit = max(1, (total + avail - 1) / avail);
    } else {
        const int total = (a.T + slab - 1) / slab;
        nit = (total + (int)gridDim.x - 1) / (int)gridDim.x;
    }
    const int brows = slab * nit;
    int row0, row_end;
    const float* s = a.s;
    if (a.tab) {
        int b = blockIdx.x, i = 0, e = 0;
        row0 = row_end = 0;
        for (; i < a.n_sel; ++i) {
            e = a.sel[i];
            const int lo = a.offsets[e], hi = a.offsets[e + 1];
            const int nb = (hi - lo + brows - 1) / brows;
            if (b < nb) {
                row0 = lo + b * brows;
                row_end = hi;
                break;
            }
            b -= nb;
        }
        if (i == a.n_sel) return;  // the grid is an upper bound
        s = a.tab[e].s_mid;
    } else {
        row0 = blockIdx.x * brows;
        row_end = a.T;
    }
    if (row0 >= row_end) return;  // uniform over the work-group
    const bool active = c < nchunk;
    float sv[16], rv[16];
    bool fast = true;
    if (s && active) fast = load_s16(s, c, sv, rv);

    // source row of slab `it`, row r of this thread (-1: none)
    auto source = [&](int it, int (&src)[RS]) {
#pragma unroll
        for (int r = 0; r < RS; ++r) {
            const int row = row0 + it * slab + g * RS + r;
            src[r] = -1;
            if (active && it < nit && row < row_end) src[r] = a.gather ? (a.gather[row] >> 1) : row;
        }
    };
    auto fetch = [&](const int (&src)[RS], uint4 (&raw)[RS][2]) {
#pragma unroll
        for (int r = 0; r < RS; ++r) {
            raw[r][0] = raw[r][1] = make_uint4(0, 0, 0, 0);
            if (src[r] >= 0) {
                const uint4* px = reinterpret_cast<const uint4*>(a.x + (size_t)src[r] * a.ldx + c * 16);
                raw[r][0] = px[0];
                raw[r][1] = px[1];
            }
        }
    };
    int src[RS], src_nxt[RS];
    uint4 raw[RS][2], raw_nxt[RS][2];
    source(0, src);
    fetch(src, raw);
    source(1, src_nxt);
    int staged = 0;          // rows in the staging area (uniform)
    int stage_t0 = row0;     // output row of its first row
    for (int it = 0; it < nit; ++it) {
        const int base = row0 + it * slab;
        if (base >= row_end) break;  // uniform over the work-group
        fetch(src_nxt, raw_nxt);  // arrives while this slab is reduced and rounded
        // quotients x / s of the slab stay in registers from the reduction to the rounding
        float y[RS][16];
        float amax[RS], amin[RS];
#pragma unroll
        for (int r = 0; r < RS; ++r) {
            float m = 0.0f, mlo = 0.0f;
#pragma unroll
            for (int i = 0; i < 16; ++i) y[r][i] = 0.0f;
            if (src[r] >= 0) {
                float x[16];
                Half8 h0, h1;
                *reinterpret_cast<uint4*>(&h0) = raw[r][0];
                *reinterpret_cast<uint4*>(&h1) = raw[r][1];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    x[i] = h2f(h0.v[i]);
                    x[8 + i] = h2f(h1.v[i]);
                }
                if (!s) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) y[r][i] = x[i];
                } else if (fast) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) y[r][i] = div_by(x[i], sv[i], rv[i], true);
                } else {
#pragma unroll
                    for (int i = 0; i < 16; ++i) y[r][i] = x[i] / sv[i];
                }
                if constexpr (ASYM) {  // the range always contains 0
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        m = fmaxf(m, y[r][i]);
                        mlo = fminf(mlo, y[r][i]);
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < 16; ++i) m = fmaxf(m, fabsf(y[r][i]));
                }
            }
            amax[r] = m;
            amin[r] = mlo;
        }
#pragma unroll
        for (int r = 0; r < RS; ++r) {
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) {
                amax[r] = fmaxf(amax[r], __shfl_xor(amax[r], o));
                if constexpr (ASYM) amin[r] = fminf(amin[r], __shfl_xor(amin[r], o));
            }
        }
        float* redp = red + (size_t)(it & 1) * (QMAX_THREADS / 64) * RS;
        if (lane == 0) {
#pragma unroll
            for (int r = 0; r < RS; ++r) {
                redp[wave * RS + r] = amax[r];
                if constexpr (ASYM) redp[RED_HALF + wave * RS + r] = amin[r];
            }
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < RS; ++r) {
            if (src[r] >= 0) {
                uint32_t w[4] = {0, 0, 0, 0};
                float m = 0.0f, mlo = 0.0f;
                for (int w2 = 0; w2 < waves_per_group; ++w2) {
                    m = fmaxf(m, redp[(g * waves_per_group + w2) * RS + r]);
                    if constexpr (ASYM) mlo = fminf(mlo, redp[RED_HALF + (g * waves_per_group + w2) * RS + r]);
                }
                float scale, z = 0.0f;
                if constexpr (ASYM) {
                    const float range = m - mlo;
                    scale = 0.0f;
                    if (range != 0.0f) {
                        scale = range / 255.0f;
                        z = fminf(fmaxf(rintf(-mlo / scale), 0.0f), 255.0f);
                        const float rscale = 1.0f / scale;
                        const bool sfast = scale >= 0x1p-100f && scale <= 0x1p100f;
                        float q[16];
#pragma unroll
                        for (int i = 0; i < 16; ++i) {
                            const float qv = sfast ? div_by(y[r][i], scale, rscale, true) : y[r][i] / scale;
                            q[i] = fminf(fmaxf(rintf(qv) + z, 0.0f), 255.0f);  // an integer in [0, 255]
                        }
#pragma unroll
                        for (int i = 0; i < 4; ++i) w[i] = round_pack4(q[4 * i], q[4 * i + 1], q[4 * i + 2], q[4 * i + 3]);
                    }
                } else {
                    scale = m / 127.0f;
                    const float rscale = 1.0f / scale;
                    const bool sfast = scale >= 0x1p-100f && scale <= 0x1p100f;
                    if (m != 0.0f) {
                        if (sfast) {  // the common case: the division through the reciprocal
                            float q[16];
#pragma unroll
                            for (int i = 0; i < 16; ++i) q[i] = div_by(y[r][i], scale, rscale, true);
#pragma unroll
                            for (int i = 0; i < 4; ++i) w[i] = round_pack4(q[4 * i], q[4 * i + 1], q[4 * i + 2], q[4 * i + 3]);
                        } else {
#pragma unroll
                            for (int i = 0; i < 16; ++i) w[i / 4] |= (uint32_t)(code_of(y[r][i], scale) & 0xff) << (8 * (i % 4));
                        }
                    }
                }
                const uint4 code = make_uint4(w[0], w[1], w[2], w[3]);
                const int t = base + g * RS + r;
                if (c == r) {
                    if (a.scale_dest) a.scale_dest[t] = scale;
                    if (a.scale) a.scale[src[r]] = scale;
                    if constexpr (ASYM) {
                        if (a.zp_dest) a.zp_dest[t] = (int32_t)z;
                        if (a.zp) a.zp[src[r]] = (int32_t)z;
                    }
                }
                if (a.q_rm) *reinterpret_cast<uint4*>(a.q_rm + (size_t)src[r] * a.ldq + c * 16) = code;
                // the operand of the signed matrix instruction: code - 128
                const uint4 packed = ASYM ? make_uint4(w[0] ^ 0x80808080u, w[1] ^ 0x80808080u, w[2] ^ 0x80808080u, w[3] ^ 0x80808080u) : code;
                *reinterpret_cast<uint4*>(qlds + (size_t)(staged + g * RS + r) * pitch + c * 16) = packed;
            }
        }
        staged += slab;
        const bool last = it + 1 == nit || base + slab >= row_end;
        if (staged + slab > srows || last) {
            __syncthreads();  // the staged codes are complete
            if (a.q_cm) {
                const int nrow = min(staged, row_end - stage_t0);
                // srows is a power of two (8 or 16): shifts instead of a division by a run-time value
                const int sh = srows == 8 ? 3 : 4;
                for (int i = tid; i < nchunk * srows; i += nthr) {
                    const int row = i & (srows - 1), ch = i >> sh;
                    if (row < nrow)
                        *reinterpret_cast<uint4*>(a.q_cm + ((size_t)ch * a.R + stage_t0 + row) * 16) =
                            *reinterpret_cast<const uint4*>(qlds + (size_t)row * pitch + ch * 16);
                }
            }
            stage_t0 += staged;
            staged = 0;
            if (!last) __syncthreads();  // the staging area may be overwritten
        }
#pragma unroll
        for (int r = 0; r < RS; ++r) {
            src[r] = src_nxt[r];
            raw[r][0] = raw_nxt[r][0];
            raw[r][1] = raw_nxt[r][1];
        }
        source(it + 2, src_nxt);
    }
}


// ---- asymmetric activation codes ---------------------------------------------------------------
// Per token: range [mn, mx] of y = x / s widened to contain 0, scale = (mx - mn) / 255, zero point
// zp = clamp(rne(-mn / scale), 0, 255), code = clamp(rne(y / scale) + zp, 0, 255).  The packed
// operand holds code - 128 (the MFMA operands are signed; the GEMM epilogue adds
// (128 - zp) * column sum back).  Same thread mapping as the register-resident symmetric kernel.
struct AsymQuantArgs {
    const __half* x;
    int64_t ldx;
    const float* s;
    int T, K;
    int8_t* q_cm;     // packed, code - 128
    int64_t R;
    uint8_t* q_rm;    // optional dense [T x K] codes
    int64_t ldq;
    float* scale;     // [T]
    int32_t* zp;      // [T]
};

template <int RS>
__global__ __launch_bounds__(QMAX_THREADS) void asym_quant_kernel(AsymQuantArgs a, int CL) {
    __shared__ float red_mn[QMAX_THREADS / 64][RS];
    __shared__ float red_mx[QMAX_THREADS / 64][RS];
    const int tid = threadIdx.x;
    const int c = tid % CL, g = tid / CL;
    const int brows = (blockDim.x / CL) * RS;
    const int waves_per_group = CL >> 6, wave = tid >> 6;
    const int nchunk = a.K / 16;
    const int row0 = blockIdx.x * brows + g * RS;
    const int nrow = min(RS, a.T - row0);
    const bool active = c < nchunk;
    uint4 raw[RS][2];
#pragma unroll
    for (int r = 0; r < RS; ++r) {
        raw[r][0] = raw[r][1] = make_uint4(0, 0, 0, 0);
        if (active && r < nrow) {
            const uint4* px = reinterpret_cast<const uint4*>(a.x + (size_t)(row0 + r) * a.ldx + c * 16);
            raw[r][0] = px[0];
            raw[r][1] = px[1];
        }
    }
    float sv[16], rv[16];
    bool fast = true;
    if (a.s && active) fast = load_s16(a.s, c, sv, rv);
    float x[16];
    auto smoothed = [&](int r) {  // y of this thread's chunk of row r into x[]
        Half8 h0, h1;
        *reinterpret_cast<uint4*>(&h0) = raw[r][0];
        *reinterpret_cast<uint4*>(&h1) = raw[r][1];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            x[i] = h2f(h0.v[i]);
            x[8 + i] = h2f(h1.v[i]);
        }
        if (a.s) {
            if (fast) {
#pragma unroll
                for (int i = 0; i < 16; ++i) x[i] = div_by(x[i], sv[i], rv[i], true);
            } else {
#pragma unroll
                for (int i = 0; i < 16; ++i) x[i] = x[i] / sv[i];
            }
        }
    };
    float mn[RS], mx[RS];
#pragma unroll
    for (int r = 0; r < RS; ++r) {
        mn[r] = mx[r] = 0.0f;  // the range always contains 0 (also covers inactive lanes and absent rows)
        if (active && r < nrow) {
            smoothed(r);
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                mn[r] = fminf(mn[r], x[i]);
                mx[r] = fmaxf(mx[r], x[i]);
            }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            mn[r] = fminf(mn[r], __shfl_xor(mn[r], o));
            mx[r] = fmaxf(mx[r], __shfl_xor(mx[r], o));
        }
    }
    if ((tid & 63) == 0) {
#pragma unroll
        for (int r = 0; r < RS; ++r) {
            red_mn[wave][r] = mn[r];
            red_mx[wave][r] = mx[r];
        }
    }
    __syncthreads();
    if (!active) return;
#pragma unroll
    for (int r = 0; r < RS; ++r) {
#pragma unroll
        for (int h = 0; h < 2; ++h)
            asm volatile("" : "+v"(raw[r][h].x), "+v"(raw[r][h].y), "+v"(raw[r][h].z), "+v"(raw[r][h].w));
    }
#pragma unroll
    for (int r = 0; r < RS; ++r) {
        if (r < nrow) {
            float lo = 0.0f, hi = 0.0f;
            for (int w = 0; w < waves_per_group; ++w) {
                lo = fminf(lo, red_mn[g * waves_per_group + w][r]);
                hi = fmaxf(hi, red_mx[g * waves_per_group + w][r]);
            }
            const float range = hi - lo;
            const int t = row0 + r;
            float scale = 0.0f, z = 0.0f;
            uint32_t w4[4] = {0x80808080u, 0x80808080u, 0x80808080u, 0x80808080u};  // code 0 -> -128
            uint32_t u4[4] = {0, 0, 0, 0};
            if (range != 0.0f) {
                scale = range / 255.0f;
                z = fminf(fmaxf(rintf(-lo / scale), 0.0f), 255.0f);
                const float rscale = 1.0f / scale;
                const bool sfast = scale >= 0x1p-100f && scale <= 0x1p100f;
                smoothed(r);
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const float qv = sfast ? div_by(x[i], scale, rscale, true) : x[i] / scale;
                    const float cf = fminf(fmaxf(rintf(qv) + z, 0.0f), 255.0f);
                    const uint32_t code = (uint32_t)(int)cf;
                    u4[i / 4] |= code << (8 * (i % 4));
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) w4[i] = u4[i] ^ 0x80808080u;  // code - 128 as a signed byte
            }
            if (c == r) {
                a.scale[t] = scale;
                a.zp[t] = (int32_t)z;
            }
            if (a.q_rm) *reinterpret_cast<uint4*>(a.q_rm + (size_t)t * a.ldq + c * 16) = make_uint4(u4[0], u4[1], u4[2], u4[3]);
            *reinterpret_cast<uint4*>(a.q_cm + ((size_t)c * a.R + t) * 16) = make_uint4(w4[0], w4[1], w4[2], w4[3]);
        }
    }
}

// The same codes one row per work-group (thread c owns chunk c of the row; K <= 16 * QMAX_THREADS), for the
// routed expert FFN: rows gathered through the permutation, or rows of the sorted intermediate with the
// smoothing vector of the expert whose group holds the row.
__global__ __launch_bounds__(QMAX_THREADS) void asym_quant_row_kernel(AsymRowArgs a) {
    __shared__ float red_mn[QMAX_THREADS / 64], red_mx[QMAX_THREADS / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nwave = blockDim.x >> 6;
    const int row = blockIdx.x;
    const int src = a.gather ? (a.gather[row] >> 1) : row;
    const float* s = a.s;
    if (a.tab) {
        int e = 0;
        while (e + 1 < a.E && row >= a.offsets[e + 1]) ++e;
        s = a.tab[e].s_mid;
    }
    const int nchunk = a.K / 16;
    const bool active = tid < nchunk;
    float y[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) y[i] = 0.0f;
    if (active) {
        load_x16(a.x + (size_t)src * a.ldx, tid, y);
        if (s) {
            float sv[16], rv[16];
            const bool fast = load_s16(s, tid, sv, rv);
            if (fast) {
#pragma unroll
                for (int i = 0; i < 16; ++i) y[i] = div_by(y[i], sv[i], rv[i], true);
            } else {
#pragma unroll
                for (int i = 0; i < 16; ++i) y[i] = y[i] / sv[i];
            }
        }
    }
    float mn = 0.0f, mx = 0.0f;  // the range always contains 0
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        mn = fminf(mn, y[i]);
        mx = fmaxf(mx, y[i]);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        mn = fminf(mn, __shfl_xor(mn, o));
        mx = fmaxf(mx, __shfl_xor(mx, o));
    }
    if (lane == 0) {
        red_mn[wave] = mn;
        red_mx[wave] = mx;
    }
    __syncthreads();
    float lo = 0.0f, hi = 0.0f;
    for (int w = 0; w < nwave; ++w) {
        lo = fminf(lo, red_mn[w]);
        hi = fmaxf(hi, red_mx[w]);
    }
    const float range = hi - lo;
    float scale = 0.0f, z = 0.0f;
    uint32_t w4[4] = {0x80808080u, 0x80808080u, 0x80808080u, 0x80808080u};  // code 0 -> -128
    uint32_t u4[4] = {0, 0, 0, 0};
    if (range != 0.0f) {
        scale = range / 255.0f;
        z = fminf(fmaxf(rintf(-lo / scale), 0.0f), 255.0f);
        const float rscale = 1.0f / scale;
        const bool sfast = scale >= 0x1p-100f && scale <= 0x1p100f;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float qv = sfast ? div_by(y[i], scale, rscale, true) : y[i] / scale;
            const float cf = fminf(fmaxf(rintf(qv) + z, 0.0f), 255.0f);
            u4[i / 4] |= (uint32_t)(int)cf << (8 * (i % 4));
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) w4[i] = u4[i] ^ 0x80808080u;
    }
    if (tid == 0) {
        a.scale_out[row] = scale;
        a.zp_out[row] = (int32_t)z;
        if (a.scale_in) a.scale_in[src] = scale;
        if (a.zp_in) a.zp_in[src] = (int32_t)z;
    }
    if (!active) return;
    if (a.q_rm) *reinterpret_cast<uint4*>(a.q_rm + (size_t)(a.gather ? src : row) * a.ldq + tid * 16) = make_uint4(u4[0], u4[1], u4[2], u4[3]);
    *reinterpret_cast<uint4*>(a.q_cm + ((size_t)tid * a.R + row) * 16) = make_uint4(w4[0], w4[1], w4[2], w4[3]);
}

__global__ void weight_colsum_kernel(const int8_t* wq, int K, int N, int32_t* colsum) {
    const int n = blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= N) return;
    int32_t acc = 0;
    for (int k = 0; k < K; ++k) acc += wq[(size_t)k * N + n];
    colsum[n] = acc;
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
    if (n < Nout && kc * 16 < K) {  // chunks past K (the pad up to a whole 64-byte k-step) stay zero
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
    const int nchunk = a.K / 16;
    int CL = (int)round_up(nchunk, 64);  // chunk lanes
    if (CL > QMAX_THREADS) CL = QMAX_THREADS;
    int G = QMAX_THREADS / CL;           // row groups: 1, 2, 4 or 8
    G = G >= 8 ? 8 : G >= 4 ? 4 : G >= 2 ? 2 : 1;
    const int threads = CL * G;
    // with per-expert groups every group may end in a partial block: T/8 + E is an upper bound
    const int blocks = a.tab ? a.max_rows / QBLOCK_ROWS + a.n_sel : cdiv(a.T, QBLOCK_ROWS);
    if (nchunk <= CL) {
        // one chunk per thread.  With enough rows to give every CU a slab, the pipelined kernel
        // (2 rows per row group per slab, next slab in flight, transposed write-out), one
        // work-group per CU
        constexpr int LRS = 2;
        const int rows = a.tab ? a.max_rows : a.T;
        static int n_cu = 0;
        if (n_cu == 0) {
            int devid = 0, v = 0;
            HAQ_CHECK_HIP(hipGetDevice(&devid));
            HAQ_CHECK_HIP(hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, devid));
            n_cu = v > 64 ? v : 256;
        }
        if (rows / (LRS * G) >= n_cu) {
            const size_t red_bytes = 4 * (QMAX_THREADS / 64) * LRS * sizeof(float);  // maxima and (asymmetric codes) minima
            const size_t lds = (size_t)qstage_rows(LRS * G) * qstage_pitch(nchunk) + red_bytes;
            static std::once_flag once;
            static hipError_t attr_err = hipSuccess;
            std::call_once(once, [&] {  // the largest case: one row group, QMAX_THREADS chunks
                const int most = QSTAGE * qstage_pitch(QMAX_THREADS) + (int)red_bytes;
                attr_err = hipFuncSetAttribute((const void*)smooth_quant_lds_kernel<LRS, false>, hipFuncAttributeMaxDynamicSharedMemorySize, most);
                if (attr_err == hipSuccess)
                    attr_err = hipFuncSetAttribute((const void*)smooth_quant_lds_kernel<LRS, true>, hipFuncAttributeMaxDynamicSharedMemorySize, most);
            });
            HAQ_CHECK_HIP(attr_err);
            if (a.zp_dest)
                hipLaunchKernelGGL((smooth_quant_lds_kernel<LRS, true>), dim3(n_cu), dim3(threads), lds, st, a, CL);
            else
                hipLaunchKernelGGL((smooth_quant_lds_kernel<LRS, false>), dim3(n_cu), dim3(threads), lds, st, a, CL);
            HAQ_CHECK_HIP(hipGetLastError());
            return HAQ_OK;
        }
        if (a.zp_dest) return HAQ_ERR_UNSUPPORTED;  // asymmetric codes: only the pipelined kernel; the caller has a row kernel
        // otherwise the register-resident single pass, at most 4 rows per thread
        const int RS = QBLOCK_ROWS / G > 4 ? 4 : QBLOCK_ROWS / G;
        const int brows = RS * G;
        const int nb = a.tab ? a.max_rows / brows + a.n_sel : cdiv(a.T, brows);
        switch (RS) {
            case 4: hipLaunchKernelGGL(smooth_quant_reg_kernel<4>, dim3(nb), dim3(threads), 0, st, a, CL); break;
            case 2: hipLaunchKernelGGL(smooth_quant_reg_kernel<2>, dim3(nb), dim3(threads), 0, st, a, CL); break;
            default: hipLaunchKernelGGL(smooth_quant_reg_kernel<1>, dim3(nb), dim3(threads), 0, st, a, CL); break;
        }
        HAQ_CHECK_HIP(hipGetLastError());
        return HAQ_OK;
    }
    if (a.zp_dest) return HAQ_ERR_UNSUPPORTED;
    switch (QBLOCK_ROWS / G) {
        case 8: hipLaunchKernelGGL(smooth_quant_kernel<8>, dim3(blocks), dim3(threads), 0, st, a, CL); break;
        case 4: hipLaunchKernelGGL(smooth_quant_kernel<4>, dim3(blocks), dim3(threads), 0, st, a, CL); break;
        case 2: hipLaunchKernelGGL(smooth_quant_kernel<2>, dim3(blocks), dim3(threads), 0, st, a, CL); break;
        default: hipLaunchKernelGGL(smooth_quant_kernel<1>, dim3(blocks), dim3(threads), 0, st, a, CL); break;
    }
    HAQ_CHECK_HIP(hipGetLastError());
    return HAQ_OK;
}

int launch_asym_quant(const __half* x, int64_t ldx, const float* s, int T, int K, int8_t* q_cm, int64_t R, uint8_t* q_rm,
                      int64_t ldq, float* scale, int32_t* zp, hipStream_t st) {
    if (T <= 0) return HAQ_OK;
    const int nchunk = K / 16;
    int CL = (int)round_up(nchunk, 64);
    if (CL > QMAX_THREADS) return HAQ_ERR_UNSUPPORTED;  // K > 16384: not built for the asymmetric variant
    int G = QMAX_THREADS / CL;
    G = G >= 8 ? 8 : G >= 4 ? 4 : G >= 2 ? 2 : 1;
    const int RS = QBLOCK_ROWS / G > 4 ? 4 : QBLOCK_ROWS / G;
    const int threads = CL * G, nb = cdiv(T, RS * G);
    AsymQuantArgs a{x, ldx, s, T, K, q_cm, R, q_rm, ldq, scale, zp};
    switch (RS) {
        case 4: hipLaunchKernelGGL(asym_quant_kernel<4>, dim3(nb), dim3(threads), 0, st, a, CL); break;
        case 2: hipLaunchKernelGGL(asym_quant_kernel<2>, dim3(nb), dim3(threads), 0, st, a, CL); break;
        default: hipLaunchKernelGGL(asym_quant_kernel<1>, dim3(nb), dim3(threads), 0, st, a, CL); break;
    }
    HAQ_CHECK_HIP(hipGetLastError());
    return HAQ_OK;
}

int launch_asym_quant_rows(const AsymRowArgs& a, hipStream_t st) {
    if (a.rows <= 0) return HAQ_OK;
    const int nchunk = a.K / 16;
    const int threads = (int)round_up(nchunk, 64);
    if (threads > QMAX_THREADS) return HAQ_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(asym_quant_row_kernel, dim3(a.rows), dim3(threads), 0, st, a);
    HAQ_CHECK_HIP(hipGetLastError());
    return HAQ_OK;
}

}  // namespace haq

using namespace haq;

extern "C" {

int32_t haq_smooth_quant_act(const void* x_fp16, int64_t ldx, const float* s, int32_t T, int32_t K, int8_t* q,
                             int64_t ldq, float* row_scale, void* stream) {
    if (T < 0 || K <= 0) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_smooth_quant_act: T=%d K=%d", T, K);
    if (K % 16 != 0 || K > 65536) HAQ_FAIL(HAQ_ERR_UNSUPPORTED, "haq_smooth_quant_act: K=%d must be a multiple of 16, <= 65536", K);
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

int32_t haq_weight_colsum(const int8_t* wq, int32_t K, int32_t N, int32_t* colsum, void* stream) {
    if (K <= 0 || N <= 0) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_weight_colsum: K=%d N=%d", K, N);
    if (!wq || !colsum) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_weight_colsum: null buffer");
    hipLaunchKernelGGL(weight_colsum_kernel, dim3(cdiv(N, 256)), dim3(256), 0, (hipStream_t)stream, wq, K, N, colsum);
    HAQ_CHECK_HIP(hipGetLastError());
    return HAQ_OK;
}

size_t haq_packed_bytes(int32_t K, int32_t N) {
    if (K <= 0 || N <= 0) return 0;
    return (size_t)round_up(K, 64) * (size_t)round_up(N, NPAD);
}

int32_t haq_pack_weight(const int8_t* wq, int32_t K, int32_t N, int8_t* packed, void* stream) {
    if (K <= 0 || N <= 0) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_pack_weight: K=%d N=%d", K, N);
    if (K % 16 != 0 || K / 16 > 65532) HAQ_FAIL(HAQ_ERR_UNSUPPORTED, "haq_pack_weight: K=%d must be a multiple of 16", K);
    if (!wq || !packed || !aligned16(packed)) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_pack_weight: null or misaligned buffer");
    const int Npad = (int)round_up(N, NPAD);
    hipLaunchKernelGGL(pack_kernel, dim3(Npad / 256, (unsigned)(round_up(K, 64) / 16)), dim3(256), 0, (hipStream_t)stream, wq,
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
