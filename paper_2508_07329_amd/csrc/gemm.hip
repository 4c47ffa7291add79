// Launcher of the int8 MFMA GEMM kernel (gemm_kernel.h): picks the tile shape, sizes
// the grid and opts the kernel into its dynamic LDS size.
#include <mutex>

#include "gemm_kernel.h"

namespace haq {

namespace {

// 128 x 256 tiles, 4 waves (2 x 2, 64 x 128 each), 3-deep ring: 75 KB of LDS and at most
// 256 registers per lane, so two work-groups share a CU and fill each other's stalls.
// (The shape can be overridden at compile time to measure other tilings; the small-problem instantiation below is fixed.)
#ifndef HAQ_BM
#define HAQ_BM 128
#define HAQ_BN 256
#define HAQ_MINB 2
#define HAQ_STAGES 3
#endif
#ifndef HAQ_WAVES_M
#define HAQ_WAVES_M 2
#endif
#ifndef HAQ_WAVES_N
#define HAQ_WAVES_N 2
#endif
constexpr int BM = HAQ_BM, BN = HAQ_BN, WAVES_M = HAQ_WAVES_M, WAVES_N = HAQ_WAVES_N, STAGES = HAQ_STAGES, MINB = HAQ_MINB;
using Shape = GemmShape<BM, BN, WAVES_M, WAVES_N, STAGES>;

template <int EPI, bool DBG>
int launch_one(const GemmArgs& a, dim3 grid, hipStream_t st) {
    auto kern = gemm_i8_kernel<BM, BN, WAVES_M, WAVES_N, STAGES, MINB, EPI, DBG>;
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [&] {
        attr_err = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, Shape::LDS_BYTES);
    });
    HAQ_CHECK_HIP(attr_err);
    hipLaunchKernelGGL(kern, grid, dim3(Shape::THREADS), Shape::LDS_BYTES, st, a);
    HAQ_CHECK_HIP(hipGetLastError());
    return HAQ_OK;
}

// 128 x 128 tiles (wave tile 64 x 64) for problems whose 128 x 256 tiling would leave half of the
// work-group slots empty: twice the tiles, 49 KB of LDS, three work-groups per CU.
#ifndef HAQ_SMALL_TILE_LIMIT
#define HAQ_SMALL_TILE_LIMIT 256
#endif
constexpr int SMALL_TILE_LIMIT = HAQ_SMALL_TILE_LIMIT;  // 128 x 256 tiles that would not even give every CU one work-group
constexpr int BN_S = 128, MINB_S = 3;
using ShapeS = GemmShape<128, BN_S, 2, 2, 3>;
int launch_small(const GemmArgs& a, dim3 grid, hipStream_t st) {
    auto kern = gemm_i8_kernel<128, BN_S, 2, 2, 3, MINB_S, EPI_LINEAR, false>;
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [&] {
        attr_err = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, ShapeS::LDS_BYTES);
    });
    HAQ_CHECK_HIP(attr_err);
    hipLaunchKernelGGL(kern, grid, dim3(ShapeS::THREADS), ShapeS::LDS_BYTES, st, a);
    HAQ_CHECK_HIP(hipGetLastError());
    return HAQ_OK;
}

// 256 x 256 tiles, 8 waves (4 x 2, the same 64 x 128 wave tile and per-wave code as the main shape), one
// work-group per CU: a third fewer direct-to-LDS bytes per matrix instruction, which is what limits the K loop.
// For dense problems with at least two full rounds of such tiles (one per CU and round); measured +3 % on
// 2048..8192 x 4096 x 16384, -8 % on a single round, and slower on ragged expert groups (more padding rows).
constexpr int LARGE_TILE_MIN = 512;
using ShapeL = GemmShape<256, 256, 4, 2, 3>;
int launch_large(const GemmArgs& a, dim3 grid, hipStream_t st) {
    auto kern = gemm_i8_kernel<256, 256, 4, 2, 3, 1, EPI_LINEAR, false>;
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [&] {
        attr_err = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, ShapeL::LDS_BYTES);
    });
    HAQ_CHECK_HIP(attr_err);
    hipLaunchKernelGGL(kern, grid, dim3(ShapeL::THREADS), ShapeL::LDS_BYTES, st, a);
    HAQ_CHECK_HIP(hipGetLastError());
    return HAQ_OK;
}

// 256 x 128 tiles, 8 waves (4 x 2 of 64 x 64), one work-group per CU: for dense problems that this tiling covers in
// one round with most CUs busy (fc2 of the OPT-6.7B block: 8 x 32 tiles on 256 CUs).  A quarter fewer
// direct-to-LDS bytes per matrix instruction than the 128 x 128 shape such problems would otherwise take: -2 %.
using ShapeT = GemmShape<256, 128, 4, 2, 3>;
int launch_tall(const GemmArgs& a, dim3 grid, hipStream_t st) {
    auto kern = gemm_i8_kernel<256, 128, 4, 2, 3, 1, EPI_LINEAR, false>;
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [&] {
        attr_err = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, ShapeT::LDS_BYTES);
    });
    HAQ_CHECK_HIP(attr_err);
    hipLaunchKernelGGL(kern, grid, dim3(ShapeT::THREADS), ShapeT::LDS_BYTES, st, a);
    HAQ_CHECK_HIP(hipGetLastError());
    return HAQ_OK;
}

int cu_count() {
    static int n_cu = 0;
    if (n_cu == 0) {
        int devid = 0, v = 0;
        if (hipGetDevice(&devid) == hipSuccess && hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, devid) == hipSuccess && v > 0)
            n_cu = v;
        else
            n_cu = 256;
    }
    return n_cu;
}

}  // namespace

int launch_gemm(const GemmArgs& a, int epi, hipStream_t st) {
    const int ntn = cdiv(a.N, BN);
    // upper bound on the M tiles: exact for one matrix; rows/BM plus one partial tile per group otherwise
    const int mt = a.offsets ? a.max_rows / BM + a.n_sel : cdiv(a.M, BM);
    if (mt <= 0 || ntn <= 0) return HAQ_OK;
    if (!a.offsets && epi == EPI_LINEAR && !a.acc_dbg) {
        const int64_t tiles_l = (int64_t)cdiv(a.M, 256) * cdiv(a.N, 256);
        if (tiles_l >= LARGE_TILE_MIN) return launch_large(a, dim3((unsigned)round_up(tiles_l, 8)), st);
        const int64_t tiles_t = (int64_t)cdiv(a.M, 256) * cdiv(a.N, 128);
        const int n_cu = cu_count();
        if (tiles_t <= n_cu && 4 * tiles_t > 3 * n_cu) return launch_tall(a, dim3((unsigned)round_up(tiles_t, 8)), st);
    }
    if (!a.offsets && epi == EPI_LINEAR && !a.acc_dbg && mt * ntn <= SMALL_TILE_LIMIT) {
        const int ntn_s = cdiv(a.N, BN_S), mt_s = cdiv(a.M, 128);
        return launch_small(a, dim3((unsigned)round_up((int64_t)mt_s * ntn_s, 8)), st);
    }
    const dim3 grid((unsigned)round_up((int64_t)mt * ntn, 8));
    if (epi == EPI_SWIGLU) return launch_one<EPI_SWIGLU, false>(a, grid, st);
    if (epi == EPI_SWIGLU_ASYM) return launch_one<EPI_SWIGLU_ASYM, false>(a, grid, st);
    if (epi == EPI_LINEAR_ASYM) return a.acc_dbg ? launch_one<EPI_LINEAR_ASYM, true>(a, grid, st) : launch_one<EPI_LINEAR_ASYM, false>(a, grid, st);
    if (a.acc_dbg) return launch_one<EPI_LINEAR, true>(a, grid, st);
    return launch_one<EPI_LINEAR, false>(a, grid, st);
}

}  // namespace haq
