// int8 x int8 -> int32 GEMM on the gfx950 matrix cores with the dequantise /
// activation epilogue (Eq. 1 evaluated at run time: Q(s^-1 X) . Q(W s), scales on
// the token and output-channel dimensions), for one matrix or for a set of
// expert groups over rows sorted by expert.
//
// Both operands are chunk-major int8 ([K/16][rows][16]).  A workgroup of 256
// threads (4 waves, 2 x 2) owns a BM x BN output tile; each wave owns a
// (BM/2) x (BN/2) sub-tile as a grid of 32 x 32 accumulators fed by
// v_mfma_i32_32x32x32_i8 (16 bytes of k per lane per operand).  K advances 64
// bytes per stage through a double-buffered LDS tile.
#include "haq_common.h"

namespace haq {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef const __attribute__((address_space(1))) v4i* gptr_v4i;  // global (not generic) 16-byte loads

__device__ __forceinline__ v4i gload16(const int8_t* p) { return *(gptr_v4i)(uintptr_t)p; }

constexpr int BK = 64;           // bytes of k per stage
constexpr int KC = BK / 16;      // 16-byte chunks per stage
constexpr int GEMM_THREADS = 256;

struct TileCoord {
    int m0;       // first sorted row of the tile
    int m_end;    // one past the last valid row (group end)
    int n0;       // first packed output channel of the tile
    int e;        // expert (or 0)
    bool valid;
};

// Work-group id -> tile.  Ids are dealt round-robin to the 8 XCDs by the
// hardware; undo that so that each XCD (one L2) walks a contiguous range of
// tiles, M fastest, i.e. neighbouring work-groups on one XCD share B tiles and
// the A tiles stay L2 resident.
template <int BM, int BN>
__device__ __forceinline__ TileCoord decode_tile(const GemmArgs& a) {
    TileCoord tc;
    tc.valid = false;
    tc.e = 0;
    tc.m0 = tc.m_end = tc.n0 = 0;
    const int ntn = (a.N + BN - 1) / BN;
    int total_mt = 0;
    if (!a.offsets) {
        total_mt = (a.M + BM - 1) / BM;
    } else {
        for (int i = 0; i < a.n_sel; ++i) {
            const int e = a.sel[i];
            total_mt += (a.offsets[e + 1] - a.offsets[e] + BM - 1) / BM;
        }
    }
    const int total = total_mt * ntn;
    // the grid is a multiple of 8 and at least `total`: XCD x owns ids [x*per, (x+1)*per)
    const int per = (total + 7) / 8;
    const int xcd = blockIdx.x % 8, slot = blockIdx.x / 8;
    if (slot >= per) return tc;
    const int id = xcd * per + slot;
    if (id >= total) return tc;
    int mi = id % total_mt;
    tc.n0 = (id / total_mt) * BN;
    if (!a.offsets) {
        tc.m0 = mi * BM;
        tc.m_end = a.M;
        tc.valid = true;
        return tc;
    }
    // grouped: M tiles of the selected experts, one after another
    for (int i = 0; i < a.n_sel; ++i) {
        const int e = a.sel[i];
        const int lo = a.offsets[e], hi = a.offsets[e + 1];
        const int mt = (hi - lo + BM - 1) / BM;
        if (mi < mt) {
            tc.e = e;
            tc.m0 = lo + mi * BM;
            tc.m_end = hi;
            tc.valid = true;
            return tc;
        }
        mi -= mt;
    }
    return tc;
}

template <int BM, int BN, int EPI>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_i8_kernel(GemmArgs a) {
    constexpr int WM = BM / 2, WN = BN / 2;  // wave tile
    constexpr int MI = WM / 32, NI = WN / 32;
    constexpr int A_LOADS = KC * BM / GEMM_THREADS;  // 16-byte loads per thread per stage
    constexpr int B_LOADS = KC * BN / GEMM_THREADS;
    __shared__ __attribute__((aligned(16))) int8_t lds_a[2][KC * BM * 16];
    __shared__ __attribute__((aligned(16))) int8_t lds_b[2][KC * BN * 16];

    const TileCoord tc = decode_tile<BM, BN>(a);
    if (!tc.valid) return;

    const int8_t* Bmat = a.B;
    const float* sw_a = a.sw;
    const float* sw_b = nullptr;
    if (a.offsets) {
        const ExpertTab& t = a.tab[tc.e];
        if (a.which == 0) {
            Bmat = t.w13;
            sw_a = t.sw1;
            sw_b = t.sw3;
        } else {
            Bmat = t.w2;
            sw_a = t.sw2;
        }
    }

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int nkt = a.K / BK;

    // global source of this thread's stage loads: load i of a stage covers chunk
    // tid/BM + i*(256/BM), row tid%BM; a stage advances KC chunks
    const int8_t* ga = a.A + ((size_t)(tid / BM) * a.R + tc.m0 + (tid % BM)) * 16;
    const int8_t* gb = Bmat + ((size_t)(tid / BN) * a.Npad + tc.n0 + (tid % BN)) * 16;
    const size_t a_ld = (size_t)(GEMM_THREADS / BM) * a.R * 16, b_ld = (size_t)(GEMM_THREADS / BN) * a.Npad * 16;
    const size_t a_step = (size_t)KC * a.R * 16, b_step = (size_t)KC * a.Npad * 16;

    v16i acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    v4i ra[A_LOADS], rb[B_LOADS];
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i) ra[i] = gload16(ga + i * a_ld);
#pragma unroll
    for (int i = 0; i < B_LOADS; ++i) rb[i] = gload16(gb + i * b_ld);
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i) *reinterpret_cast<v4i*>(&lds_a[0][(tid + i * GEMM_THREADS) * 16]) = ra[i];
#pragma unroll
    for (int i = 0; i < B_LOADS; ++i) *reinterpret_cast<v4i*>(&lds_b[0][(tid + i * GEMM_THREADS) * 16]) = rb[i];
    __syncthreads();

    // fragment addresses inside a stage: chunk = 2*kk + lane/32, row = wave base + 32*i + lane%32
    const int frag_a = ((lane >> 5) * BM + wm * WM + (lane & 31)) * 16;
    const int frag_b = ((lane >> 5) * BN + wn * WN + (lane & 31)) * 16;

    for (int kt = 0; kt < nkt; ++kt) {
        const int cur = kt & 1;
        {   // prefetch the next stage into registers (the last iteration re-reads its own stage)
            const int kn = (kt + 1 < nkt) ? kt + 1 : kt;
#pragma unroll
            for (int i = 0; i < A_LOADS; ++i) ra[i] = gload16(ga + (size_t)kn * a_step + i * a_ld);
#pragma unroll
            for (int i = 0; i < B_LOADS; ++i) rb[i] = gload16(gb + (size_t)kn * b_step + i * b_ld);
        }
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            v4i fa[MI], fb[NI];
#pragma unroll
            for (int i = 0; i < MI; ++i)
                fa[i] = *reinterpret_cast<const v4i*>(&lds_a[cur][frag_a + (kk * 2 * BM + i * 32) * 16]);
#pragma unroll
            for (int j = 0; j < NI; ++j)
                fb[j] = *reinterpret_cast<const v4i*>(&lds_b[cur][frag_b + (kk * 2 * BN + j * 32) * 16]);
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < A_LOADS; ++i)
            *reinterpret_cast<v4i*>(&lds_a[cur ^ 1][(tid + i * GEMM_THREADS) * 16]) = ra[i];
#pragma unroll
        for (int i = 0; i < B_LOADS; ++i)
            *reinterpret_cast<v4i*>(&lds_b[cur ^ 1][(tid + i * GEMM_THREADS) * 16]) = rb[i];
        __syncthreads();
    }

    // ---- epilogue.  32x32 accumulator: register r of lane l holds
    // row 8*(r/4) + 4*(l/32) + r%4, column l%32.
    const int col_l = lane & 31;
    const int row_l = (lane >> 5) * 4;
#pragma unroll
    for (int i = 0; i < MI; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = tc.m0 + wm * WM + i * 32 + 8 * (r / 4) + row_l + (r % 4);
            if (row >= tc.m_end) continue;
            const float sx = a.sx[row];
            if (EPI == EPI_LINEAR) {
#pragma unroll
                for (int j = 0; j < NI; ++j) {
                    const int col = tc.n0 + wn * WN + j * 32 + col_l;
                    if (col >= a.N) continue;
                    const int v = acc[i][j][r];
                    if (a.acc_dbg) a.acc_dbg[(size_t)row * a.N + col] = v;
                    float f = dequant(v, sx, sw_a[col]);
                    if (a.act == HAQ_ACT_RELU) f = fmaxf(f, 0.0f);
                    a.Y[(size_t)row * a.ldy + col] = f2h(f);
                }
            } else {
#pragma unroll
                for (int j = 0; j < NI; j += 2) {
                    const int pc = tc.n0 + wn * WN + j * 32;  // packed column of the gate block
                    if (pc >= a.N) continue;
                    const int col = (pc / 64) * 32 + col_l;
                    const float g = dequant(acc[i][j][r], sx, sw_a[col]);
                    const float u = dequant(acc[i][j + 1][r], sx, sw_b[col]);
                    a.Y[(size_t)row * a.ldy + col] = f2h(silu(g) * u);
                }
            }
        }
    }
}

template <int BM, int BN>
int launch_tile(const GemmArgs& a, int epi, hipStream_t st) {
    const int ntn = cdiv(a.N, BN);
    int mt;
    if (!a.offsets) {
        mt = cdiv(a.M, BM);
    } else {
        // upper bound on the M tiles of the selected groups: rows/BM + one partial tile per group
        mt = a.max_rows / BM + a.n_sel;
    }
    if (mt <= 0 || ntn <= 0) return HAQ_OK;
    const dim3 grid((unsigned)round_up((int64_t)mt * ntn, 8));
    if (epi == EPI_LINEAR)
        hipLaunchKernelGGL((gemm_i8_kernel<BM, BN, EPI_LINEAR>), grid, dim3(GEMM_THREADS), 0, st, a);
    else
        hipLaunchKernelGGL((gemm_i8_kernel<BM, BN, EPI_SWIGLU>), grid, dim3(GEMM_THREADS), 0, st, a);
    HAQ_CHECK_HIP(hipGetLastError());
    return HAQ_OK;
}

}  // namespace

int launch_gemm(const GemmArgs& a, int epi, hipStream_t st) {
    return launch_tile<256, 256>(a, epi, st);
}

}  // namespace haq
