// int8 x int8 -> int32 GEMM kernel for the gfx950 matrix cores with the dequantise /
// activation epilogue (Eq. 1 evaluated at run time: Q(s^-1 X) . Q(W s), scales on the
// token and output-channel dimensions), for one matrix or for expert groups over rows
// sorted by expert.
//
// Data flow of a work-group (BM x BN output tile, WAVES_M x WAVES_N waves):
//   HBM/L2 --global_load_lds (16 B/lane, no VGPR staging)--> LDS ring of STAGES K-steps
//   (64 bytes of k each) --ds_read_b128--> fragment registers, one whole K-step ahead
//   --> v_mfma_i32_32x32x32_i8 (16 bytes of k per lane per operand).
// Both operands are chunk-major ([K/16][rows][16]), so a K-step of a tile is four
// contiguous row segments per operand, lands in LDS in fragment order and is read back
// without bank conflicts.  One raw s_barrier per K-step.  The product is formed
// transposed (weights as first operand) so that a lane owns four consecutive output
// channels; the epilogue dequantises, applies the activation, stages fp16 rows in LDS
// and writes 16 bytes per lane.
#pragma once
#include "haq_common.h"

namespace haq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// s_waitcnt immediates (gfx9 encoding): vmcnt in bits [3:0] and [15:14], lgkmcnt in [11:8]
#define HAQ_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 0xF) | (((n) >> 4) << 14) | (0x7 << 4) | (0xF << 8))
#define HAQ_WAIT_LGKM0() __builtin_amdgcn_s_waitcnt(0xF | (0x3 << 14) | (0x7 << 4) | (0x0 << 8))
#define HAQ_CFENCE() asm volatile("" ::: "memory")

struct TileCoord {
    int m0;     // first (sorted) row of the tile
    int m_end;  // one past the last valid row (end of the group)
    int n0;     // first packed output channel of the tile
    int e;      // expert (0 for a single matrix)
    bool valid;
};

// Work-group id -> tile.  The hardware deals work-group ids round-robin to the 8 XCDs;
// undo that so that each XCD (one L2) owns a contiguous range of tile ids, M fastest:
// neighbouring work-groups of an XCD share weight tiles and the activation tiles stay in
// its L2.  The grid is a multiple of 8 and at least the tile count.
#ifndef HAQ_TILE_BAND
#define HAQ_TILE_BAND 8
#endif
constexpr int TILE_BAND = HAQ_TILE_BAND;

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
    const int per = (total + 7) / 8;
    const int xcd = blockIdx.x % 8, slot = blockIdx.x / 8;
    if (slot >= per) return tc;
    const int id = xcd * per + slot;
    if (id >= total) return tc;
    // bands of TILE_BAND row tiles, channel tiles inside a band, rows fastest: the
    // work-groups resident on one XCD at a time then form a compact block of the tile grid
    // (a row tile's activations and a channel tile's weights are each shared by ~8 of them
    // in L2) instead of one channel tile across every row tile of every expert
    // (256-row tiles: bands of 4, the same 1024 rows; with one work-group per CU an XCD then holds 4 x 8 tiles)
    constexpr int BAND = BM >= 256 ? TILE_BAND / 2 : TILE_BAND;
    const int band = id / (BAND * ntn), rem = id % (BAND * ntn);
    const int band_rows = min(BAND, total_mt - band * BAND);
    int mi = band * BAND + rem % band_rows;
    tc.n0 = (rem / band_rows) * BN;
    if (!a.offsets) {
        tc.m0 = mi * BM;
        tc.m_end = a.M;
        tc.valid = true;
        return tc;
    }
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

template <int BM, int BN, int WAVES_M, int WAVES_N, int STAGES>
struct GemmShape {
    static constexpr int NW = WAVES_M * WAVES_N;
    static constexpr int THREADS = NW * 64;
    static constexpr int STAGE_BYTES = (BM + BN) * 64;
    static constexpr int SCALE_BYTES = (BM + 2 * BN) * 4;  // row scales, channel scales and (asymmetric codes) column sums of the tile
    static constexpr int LDS_BYTES = STAGES * STAGE_BYTES + SCALE_BYTES;
};

template <int BM, int BN, int WAVES_M, int WAVES_N, int STAGES, int MINB, int EPI, bool DBG>
__global__ __launch_bounds__(WAVES_M * WAVES_N * 64, MINB) void gemm_i8_kernel(GemmArgs a) {
    using S = GemmShape<BM, BN, WAVES_M, WAVES_N, STAGES>;
    constexpr int NW = S::NW;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;  // wave tile
    constexpr int MI = WM / 32, NI = WN / 32;
    constexpr int STAGE_BYTES = S::STAGE_BYTES;
    constexpr int GA = 4 * BM / 64, GB = 4 * BN / 64;  // 1 KB (64 rows x 16 B) load groups per K-step
    constexpr int LPW = (GA + GB) / NW;                // direct-to-LDS loads per wave per K-step
    static_assert((GA + GB) % NW == 0, "load groups must divide among the waves");
    // a tile's loads cover BM rows and BN channels whatever the problem size: the packed operands are padded for that
    static_assert(NPAD % BN == 0, "a channel tile must not reach past the padded width of the packed weights");
    static_assert(BM <= 256, "packed activations carry 256 rows of padding");
    constexpr bool SWIGLU = EPI == EPI_SWIGLU || EPI == EPI_SWIGLU_ASYM;
    constexpr bool ASYM = EPI == EPI_LINEAR_ASYM || EPI == EPI_SWIGLU_ASYM;
    static_assert(!SWIGLU || NI % 2 == 0, "gate/up blocks come in pairs");
    constexpr int OUT_WN = SWIGLU ? WN / 2 : WN;  // output channels per wave tile
    // staged fp16 row pitch in bytes: 2 (mod 64) dwords, so the 8-byte pieces that the 32 rows of a half-wave
    // write land in 32 different bank pairs (a pitch of 4 (mod 64) dwords costs 6 conflict cycles per write)
    constexpr int PITCH = OUT_WN * 2 + 8;
    static_assert(32 * PITCH * NW <= STAGES * STAGE_BYTES, "epilogue staging must fit in the ring");
    extern __shared__ __attribute__((aligned(1024))) int8_t lds[];
    float* sx_s = reinterpret_cast<float*>(lds + STAGES * STAGE_BYTES);  // [BM] row scales of the tile
    float* sw_s = sx_s + BM;                                             // [BN] channel scales, packed order
    int32_t* cs_s = reinterpret_cast<int32_t*>(sw_s + BN);               // [BN] column sums of the weight codes, packed order (ASYM)

    const TileCoord tc = decode_tile<BM, BN>(a);
    if (!tc.valid) return;

    const int8_t* Bmat = a.B;
    const float* sw_a = a.sw;
    const float* sw_b = nullptr;
    const int32_t* cs_a = a.colsum;  // column sums of the weight codes (asymmetric activation codes only)
    const int32_t* cs_b = nullptr;
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
        if (ASYM) {
            const ColsumTab& c = a.cstab[tc.e];
            cs_a = a.which == 0 ? c.cs1 : c.cs2;
            cs_b = c.cs3;
        }
    }

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int nkt = (a.K + 63) / 64;  // a last partial k-step reads chunks past K: the weight operand is zero there

    // tile scales into LDS (consumed only by the epilogue)
    for (int i = tid; i < BM; i += S::THREADS) {
        const int row = tc.m0 + i;
        sx_s[i] = row < tc.m_end ? a.sx[row] : 0.0f;
    }
    for (int i = tid; i < BN; i += S::THREADS) {
        const int pc = tc.n0 + i;
        float v = 0.0f;
        int cs = 0;
        if (pc < a.N) {
            if (SWIGLU) {
                const int col = (pc / 64) * 32 + (pc % 32);
                v = ((pc / 32) & 1) ? sw_b[col] : sw_a[col];
                if (ASYM) cs = ((pc / 32) & 1) ? cs_b[col] : cs_a[col];
            } else {
                v = sw_a[pc];
                if (ASYM) cs = cs_a[pc];
            }
        }
        sw_s[i] = v;
        if (ASYM) cs_s[i] = cs;
    }

    // direct-to-LDS load descriptors: group g = wave + i*NW covers 64 rows of one 16-byte chunk.  The base of a
    // group is the same for all lanes of the wave (scalar registers; the tile origin and the expert's matrix come
    // out of memory and are made wave-uniform explicitly), the lane adds 16 bytes per row: the loads then use the
    // scalar-base + 32-bit lane-offset form and their addresses cost no vector instructions in the K loop.
    auto uniform_ptr = [](const int8_t* p) {
        const uint64_t v = (uint64_t)(uintptr_t)p;
        const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
        return (const int8_t*)(uintptr_t)(((uint64_t)hi << 32) | lo);
    };
    const int m0u = __builtin_amdgcn_readfirstlane(tc.m0), n0u = __builtin_amdgcn_readfirstlane(tc.n0);
    const int8_t* Au = uniform_ptr(a.A);
    const int8_t* Bu = uniform_ptr(Bmat);
    const uint32_t lane_off = (uint32_t)lane * 16u;
    const int8_t* gsrc[LPW];
    size_t gstep[LPW];
#pragma unroll
    for (int i = 0; i < LPW; ++i) {
        const int g = wave + i * NW;
        if (g < GA) {
            const int c = g / (BM / 64), rg = g % (BM / 64);
            gsrc[i] = Au + ((size_t)c * a.R + m0u + rg * 64) * 16;
            gstep[i] = (size_t)4 * a.R * 16;
        } else {
            const int g2 = g - GA;
            const int c = g2 / (BN / 64), rg = g2 % (BN / 64);
            gsrc[i] = Bu + ((size_t)c * a.Npad + n0u + rg * 64) * 16;
            gstep[i] = (size_t)4 * a.Npad * 16;
        }
    }
    auto load_stage = [&](int buf, int kt) {
        // (the empty asm keeps the widening of the lane offset next to its use: hoisted out of the loop as a 64-bit
        // vector value it would turn every address back into a vector add)
        uint32_t lo = lane_off;
        asm volatile("" : "+v"(lo));
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            const int8_t* src = gsrc[i] + (size_t)kt * gstep[i] + lo;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(uintptr_t)src,
                                             (__attribute__((address_space(3))) void*)(lds + buf * STAGE_BYTES + (wave + i * NW) * 1024),
                                             16, 0, 0);
        }
    };

    v16i acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    // fragment address inside a stage: chunk = 2*half + lane/32, row = wave base + 32*tile + lane%32
    const int frag_a = ((lane >> 5) * BM + wm * WM + (lane & 31)) * 16;
    const int frag_b = BM * 64 + ((lane >> 5) * BN + wn * WN + (lane & 31)) * 16;
    v4i fa[2][2][MI], fb[2][2][NI];  // [register buffer][k half][tile]

    auto read_frags = [&](int buf, int kk, v4i(&xa)[MI], v4i(&xb)[NI]) {
        const int8_t* sb = lds + buf * STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < MI; ++i) xa[i] = *reinterpret_cast<const v4i*>(sb + frag_a + (kk * 2 * BM + i * 32) * 16);
#pragma unroll
        for (int j = 0; j < NI; ++j) xb[j] = *reinterpret_cast<const v4i*>(sb + frag_b + (kk * 2 * BN + j * 32) * 16);
    };
    auto mfmas = [&](v4i(&xa)[MI], v4i(&xb)[NI]) {
        // channel block outermost: consecutive MFMAs keep the weight fragment and change the (fewer)
        // token fragments -- measured 2.4 % faster than the other nesting on 64 x 128 wave tiles
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int i = 0; i < MI; ++i)
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(xb[j], xa[i], acc[i][j], 0, 0, 0);
    };
#ifndef HAQ_ILV
#define HAQ_ILV 0
#endif
    auto interleave = [&]() {
#if HAQ_ILV == 0
        // one LDS read behind each of the first MFMAs of the group
#pragma unroll
        for (int i = 0; i < MI + NI; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, MI * NI - (MI + NI), 0);
#elif HAQ_ILV == 1
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, MI + NI, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, MI * NI - 1, 0);
#elif HAQ_ILV == 2
        __builtin_amdgcn_sched_group_barrier(0x100, MI + NI, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, MI * NI, 0);
#elif HAQ_ILV == 3
        // two reads behind each of the first MFMAs
#pragma unroll
        for (int i = 0; i < (MI + NI) / 2; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, MI * NI - (MI + NI) / 2, 0);
#endif
    };

    // prologue: request every ring buffer (K-steps 0..STAGES-1); K-step 0 landed -> its fragments
#pragma unroll
    for (int s = 0; s < STAGES; ++s)
        if (s < nkt) load_stage(s, s);
    if (nkt >= STAGES) {
        HAQ_WAIT_VMCNT(LPW * (STAGES - 1));
    } else {
        HAQ_WAIT_VMCNT(0);
    }
    HAQ_CFENCE();
    __builtin_amdgcn_s_barrier();
    HAQ_CFENCE();
    read_frags(0, 0, fa[0][0], fb[0][0]);
    read_frags(0, 1, fa[0][1], fb[0][1]);

    // iteration kt: MFMAs on K-step kt (registers), LDS reads of K-step kt+1, global loads of
    // K-step kt+STAGES into the buffer K-step kt has vacated.
    auto body = [&](int kt, int cur, v4i(&ca)[2][MI], v4i(&cb)[2][NI], v4i(&na)[2][MI], v4i(&nb)[2][NI]) {
        int nxt = cur + 1;
        if (nxt >= STAGES) nxt -= STAGES;
        // K-step kt+1 has landed for this wave and its reads of K-step kt are complete; after
        // the barrier that holds for every wave, so the buffer of K-step kt may be overwritten.
        if (nkt - 2 - kt >= STAGES - 2) {
            HAQ_WAIT_VMCNT(LPW * (STAGES - 2));
        } else {
            HAQ_WAIT_VMCNT(0);
        }
        HAQ_WAIT_LGKM0();
        HAQ_CFENCE();
        __builtin_amdgcn_s_barrier();
        HAQ_CFENCE();
        __builtin_amdgcn_sched_barrier(0);
        if (kt + STAGES < nkt) load_stage(cur, kt + STAGES);
        read_frags(nxt, 0, na[0], nb[0]);  // past the last K-step this reads a stale buffer; unused
        mfmas(ca[0], cb[0]);
        interleave();
        __builtin_amdgcn_sched_barrier(0);
        read_frags(nxt, 1, na[1], nb[1]);
        mfmas(ca[1], cb[1]);
        interleave();
        __builtin_amdgcn_sched_barrier(0);
    };
    {
        int st = 0, kt = 0;
        for (; kt + 1 < nkt; kt += 2) {
            body(kt, st, fa[0], fb[0], fa[1], fb[1]);
            st = st + 1 >= STAGES ? 0 : st + 1;
            body(kt + 1, st, fa[1], fb[1], fa[0], fb[0]);
            st = st + 1 >= STAGES ? 0 : st + 1;
        }
        if (kt < nkt) body(kt, st, fa[0], fb[0], fa[1], fb[1]);
    }

    // ---- epilogue.  Lane l, register r of acc[i][j] holds token row i*32 + l%32 and packed
    // channel j*32 + 8*(r/4) + 4*(l/32) + r%4 of the wave tile.
    HAQ_WAIT_LGKM0();
    HAQ_CFENCE();
    __builtin_amdgcn_s_barrier();  // all reads of the ring are complete: it becomes the staging area
    HAQ_CFENCE();
    int8_t* stage = lds + wave * (32 * PITCH);  // private to the wave, 32 rows at a time
    const int m_l = lane & 31, n_l = (lane >> 5) * 4;
    constexpr int LANES_PER_ROW = OUT_WN * 2 / 16;
    constexpr int ROWS_PER_IT = 64 / LANES_PER_ROW;
    const int out_n = SWIGLU ? a.N / 2 : a.N;
    const int out_n0 = SWIGLU ? (tc.n0 + wn * WN) / 2 : tc.n0 + wn * WN;
#pragma unroll
    for (int i = 0; i < MI; ++i) {
        const int rloc = wm * WM + i * 32 + m_l;
        const float sx = sx_s[rloc];
        int zshift = 0;  // 128 - zero point of this lane's token row (asymmetric codes only)
        if (ASYM) zshift = (tc.m0 + rloc < tc.m_end) ? 128 - a.zp[tc.m0 + rloc] : 0;
        if (!SWIGLU) {
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int nloc = j * 32 + 8 * q + n_l;
                    const float4 sw = *reinterpret_cast<const float4*>(sw_s + wn * WN + nloc);
                    const float swv[4] = {sw.x, sw.y, sw.z, sw.w};
                    int csv[4] = {0, 0, 0, 0};
                    if (ASYM) {
                        const int4 c4 = *reinterpret_cast<const int4*>(cs_s + wn * WN + nloc);
                        csv[0] = c4.x, csv[1] = c4.y, csv[2] = c4.z, csv[3] = c4.w;
                    }
                    __half hv[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        int v = acc[i][j][4 * q + e];
                        if (ASYM) v += zshift * csv[e];  // channels past N hold column sum 0
                        if (DBG) {
                            const int row = tc.m0 + rloc, col = tc.n0 + wn * WN + nloc + e;
                            if (row < tc.m_end && col < a.N) a.acc_dbg[(size_t)row * a.N + col] = v;
                        }
                        float f = dequant(v, sx, swv[e]);
                        if (a.act == HAQ_ACT_RELU) f = fmaxf(f, 0.0f);
                        hv[e] = f2h(f);
                    }
                    *reinterpret_cast<uint2*>(stage + m_l * PITCH + nloc * 2) = *reinterpret_cast<const uint2*>(hv);
                }
        } else {
#pragma unroll
            for (int j = 0; j < NI; j += 2)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int nloc = j * 32 + 8 * q + n_l;  // packed channel of the gate value
                    const float4 s1 = *reinterpret_cast<const float4*>(sw_s + wn * WN + nloc);
                    const float4 s3 = *reinterpret_cast<const float4*>(sw_s + wn * WN + nloc + 32);
                    const float s1v[4] = {s1.x, s1.y, s1.z, s1.w}, s3v[4] = {s3.x, s3.y, s3.z, s3.w};
                    int c1v[4] = {0, 0, 0, 0}, c3v[4] = {0, 0, 0, 0};
                    if (ASYM) {
                        const int4 c1 = *reinterpret_cast<const int4*>(cs_s + wn * WN + nloc);
                        const int4 c3 = *reinterpret_cast<const int4*>(cs_s + wn * WN + nloc + 32);
                        c1v[0] = c1.x, c1v[1] = c1.y, c1v[2] = c1.z, c1v[3] = c1.w;
                        c3v[0] = c3.x, c3v[1] = c3.y, c3v[2] = c3.z, c3v[3] = c3.w;
                    }
                    __half hv[4];
                    const int oloc = (j / 2) * 32 + 8 * q + n_l;  // output channel inside the wave tile
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        int ag = acc[i][j][4 * q + e], au = acc[i][j + 1][4 * q + e];
                        if (ASYM) {
                            ag += zshift * c1v[e];
                            au += zshift * c3v[e];
                        }
                        const float g = dequant(ag, sx, s1v[e]);
                        const float u = dequant(au, sx, s3v[e]);
                        hv[e] = f2h(silu(g) * u);
                    }
                    *reinterpret_cast<uint2*>(stage + m_l * PITCH + oloc * 2) = *reinterpret_cast<const uint2*>(hv);
                }
        }
        // the staging area is private to the wave and LDS serves one wave's requests in order
        HAQ_CFENCE();
#pragma unroll
        for (int it = 0; it < 32 / ROWS_PER_IT; ++it) {
            const int r2 = it * ROWS_PER_IT + lane / LANES_PER_ROW;
            const int c8 = (lane % LANES_PER_ROW) * 8;
            const int orow = tc.m0 + wm * WM + i * 32 + r2, ocol = out_n0 + c8;
            const uint2 v0 = *reinterpret_cast<const uint2*>(stage + r2 * PITCH + c8 * 2);  // rows are 8-byte aligned
            const uint2 v1 = *reinterpret_cast<const uint2*>(stage + r2 * PITCH + c8 * 2 + 8);
            const uint4 v = make_uint4(v0.x, v0.y, v1.x, v1.y);
            if (orow < tc.m_end && ocol < out_n) *reinterpret_cast<uint4*>(a.Y + (size_t)orow * a.ldy + ocol) = v;
        }
        HAQ_CFENCE();
    }
}

}  // namespace haq
