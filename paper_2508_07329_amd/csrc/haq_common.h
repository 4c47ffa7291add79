// Shared host/device helpers of the HAQ W8A8 library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "haq.h"

namespace haq {

// ---- error reporting -------------------------------------------------------
void set_error(const char* fmt, ...);  // thread-local text behind haq_last_error()

#define HAQ_FAIL(code, ...)        \
    do {                           \
        haq::set_error(__VA_ARGS__); \
        return (code);             \
    } while (0)

#define HAQ_CHECK_HIP(expr)                                                                 \
    do {                                                                                    \
        hipError_t e_ = (expr);                                                             \
        if (e_ != hipSuccess) HAQ_FAIL(HAQ_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }
inline int cdiv(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

// ---- layouts ---------------------------------------------------------------
// "Chunk-major" int8 operand layout shared by activations and packed weights:
// [K/16][R][16] - for each group of 16 consecutive k, all R rows side by side.
// A tile of BM rows x 64 k is then four contiguous segments of BM*16 bytes and
// lands in LDS in the order the MFMA fragments are read, without bank conflicts.
constexpr int KCHUNK = 16;
constexpr int NPAD = 256;  // packed weights pad the output-channel count to this

// ---- device arithmetic (every operation rounds once; no contraction) --------
#ifdef __HIPCC__
__device__ __forceinline__ float h2f(__half h) { return __half2float(h); }
// binary32 -> binary16, round to nearest even.  The empty asm keeps the compiler
// from folding the producing multiply/add into a mixed-precision instruction that
// rounds only once (v_fma_mixlo_f16): every binary32 result is rounded to binary32
// first, then to binary16.
__device__ __forceinline__ __half f2h(float f) {
    asm("" : "+v"(f));
    return __float2half_rn(f);
}

// e^t as a fixed binary32 sequence: clamp to [-87, 88], n = rne(t*log2 e),
// r = t - n*ln2 (two-part), degree-7 Taylor/Horner with FMAs, times 2^n.
__device__ __forceinline__ float exp_spec(float t) {
    t = fminf(fmaxf(t, -87.0f), 88.0f);
    const float n = rintf(t * 1.44269502162933349609375f);
    float r = __builtin_fmaf(n, -0.693145751953125f, t);
    r = __builtin_fmaf(n, -1.42860682030941723212e-6f, r);
    float p = 1.0f / 5040.0f;
    p = __builtin_fmaf(p, r, 1.0f / 720.0f);
    p = __builtin_fmaf(p, r, 1.0f / 120.0f);
    p = __builtin_fmaf(p, r, 1.0f / 24.0f);
    p = __builtin_fmaf(p, r, 1.0f / 6.0f);
    p = __builtin_fmaf(p, r, 0.5f);
    p = __builtin_fmaf(p, r, 1.0f);
    p = __builtin_fmaf(p, r, 1.0f);
    const float scale = __int_as_float(((int)n + 127) << 23);
    return p * scale;
}
__device__ __forceinline__ float silu(float g) { return g / (1.0f + exp_spec(-g)); }
__device__ __forceinline__ float dequant(int acc, float sx, float sw) { return ((float)acc * sx) * sw; }
__device__ __forceinline__ int code_of(float y, float scale) {
    float c = rintf(y / scale);
    c = fminf(fmaxf(c, -127.0f), 127.0f);
    return (int)c;
}
#endif

// ---- internal launchers (host) ----------------------------------------------
struct ExpertTab {  // device-side table entry
    const int8_t* w13;
    const int8_t* w2;
    const float* sw1;
    const float* sw3;
    const float* sw2;
    const float* s_mid;
};

struct QuantArgs {
    const __half* x;   // [T x K], row stride ldx
    int64_t ldx;
    const float* s;    // [K] or null (all ones); ignored when tab is set
    const struct ExpertTab* tab;  // null, or per-expert table: row r uses tab[e(r)].s_mid, e(r) from offsets
    const int32_t* offsets;       // [E+1] sorted-row offsets (with tab)
    int E;
    int T, K;
    int8_t* q_rm;      // optional row-major output, row stride ldq
    int64_t ldq;
    int8_t* q_cm;      // optional chunk-major output [K/16][R][16]
    int64_t R;
    const int32_t* gather;  // null: output row t reads input row t; else input row gather[t] >> 1
                            // (sorted pair -> token), and T counts output rows
    float* scale;      // optional, indexed by input row
    float* scale_dest; // optional, indexed by output row
    int n_sel;         // with tab: the experts whose row groups this launch covers
    int sel[32];
    int max_rows;      // with tab: upper bound of the rows of the selected groups (grid sizing)
    // Asymmetric codes (zp_dest set): zero points by output row and (optional) by input row; q_rm then holds the
    // unsigned codes and q_cm code - 128.  Only the pipelined kernel has this variant: launch_quant returns
    // HAQ_ERR_UNSUPPORTED (no error message) when the batch is too short for it or K > 16384.
    int32_t* zp_dest;
    int32_t* zp;
};
int launch_quant(const QuantArgs& a, hipStream_t st);

enum { EPI_LINEAR = 0, EPI_SWIGLU = 1, EPI_LINEAR_ASYM = 2, EPI_SWIGLU_ASYM = 3 };

struct ColsumTab {  // device-side table entry: column sums of an expert's weight codes (asymmetric activation codes)
    const int32_t* cs1;  // [I] gate
    const int32_t* cs3;  // [I] up
    const int32_t* cs2;  // [H] down
};

struct GemmArgs {
    const int8_t* A;   // chunk-major [K/16][R][16]
    int64_t R;
    const float* sx;   // [rows] per A row
    int K;
    int N;             // packed output channels (before SwiGLU halving)
    int64_t Npad;
    // single group (offsets == null): rows [0, M), weights B, scales sw
    int M;
    const int8_t* B;
    const float* sw;
    // grouped: offsets [E+1] on device, experts tab on device, selected experts
    const int32_t* offsets;
    const ExpertTab* tab;
    int which;         // 0: gate/up (w13, sw1/sw3), 1: down (w2, sw2)
    int n_sel;
    int sel[32];
    int max_rows;      // upper bound of rows over the selected groups (grid sizing)
    int act;
    __half* Y;
    int64_t ldy;
    int32_t* acc_dbg;  // optional dense [rows x N]
    // asymmetric activation codes (EPI_LINEAR_ASYM): A holds code - 128; the accumulator is corrected by
    // (128 - zp[row]) * colsum[channel] before it is dequantised
    const int32_t* zp;      // [rows]
    const int32_t* colsum;  // [N] column sums of the weight codes (single matrix)
    const ColsumTab* cstab; // grouped: per-expert column sums, on the device
};
int launch_gemm(const GemmArgs& a, int epi, hipStream_t st);
int launch_asym_quant(const __half* x, int64_t ldx, const float* s, int T, int K, int8_t* q_cm, int64_t R, uint8_t* q_rm,
                      int64_t ldq, float* scale, int32_t* zp, hipStream_t st);

// Asymmetric codes row by row (one work-group per output row, K <= 16384), for the routed expert FFN:
// output row r reads input row gather[r] >> 1 (or r), with the shared vector s or, when tab is set, the
// s_mid of the expert whose group (offsets) holds row r.
struct AsymRowArgs {
    const __half* x;
    int64_t ldx;
    const float* s;
    const ExpertTab* tab;
    const int32_t* offsets;
    int E;
    const int32_t* gather;
    int rows, K;
    int8_t* q_cm;      // chunk-major [K/16][R][16], code - 128, by output row
    int64_t R;
    uint8_t* q_rm;     // optional dense codes [.. x K]: by input row when gather is set, else by output row
    int64_t ldq;
    float* scale_out;  // [rows] by output row
    int32_t* zp_out;   // [rows] by output row
    float* scale_in;   // optional, by input row
    int32_t* zp_in;    // optional, by input row
};
int launch_asym_quant_rows(const AsymRowArgs& a, hipStream_t st);

// Decode path (at most 64 rows per expert): weight-streaming kernels.
struct DecodeArgs {
    const int8_t* q_cm;   // token codes, chunk-major [H/16][R][16], sorted-pair rows
    const float* sx;      // [P] sorted
    int64_t R;
    const int32_t* offsets;
    const ExpertTab* tab;
    int E, H, I;
    int64_t Npad13, Npad2;
    __half* mid;          // [P x I] sorted
    float* pmax;          // [P x I/32] partial row maxima of |h / s_mid|
    int8_t* hq_cm;        // [I/16][R][16]
    int8_t* hq_rm;        // optional dense [P x I]
    float* sh;            // [P]
    __half* y;            // [P x H] sorted
    // asymmetric codes only: zero points of the token rows and of the intermediate's rows (sorted), column sums per expert
    const int32_t* zx;
    const int32_t* zh;
    const ColsumTab* cstab;
    int one_expert;       // 1 + index of the only expert to process (its rows start at row0), 0: every expert that holds rows
    int row0;
};
bool decode_supported(int T, int H, int I);
int launch_decode(const DecodeArgs& a, int T, hipStream_t st);
// The two projections of launch_decode for asymmetric codes (zx / zh, cstab set); the caller quantises the
// intermediate between the two (no partial row maxima are produced).
// One expert with 1..64 rows (rows row0 .. row0 + m - 1 of the sorted order): the three launches of launch_decode
// for that expert alone; the launch stream waits for before_down (if given) ahead of the down projection.
int launch_decode_one_expert(DecodeArgs a, int e, int row0, int m, hipEvent_t before_down, hipStream_t st);
int launch_decode_gate_up_asym(const DecodeArgs& a, int T, hipStream_t st);
int launch_decode_down_asym(const DecodeArgs& a, int T, hipStream_t st);
// One or two tokens: two launches do routing, token quantisation, both projections and the
// requantisation between them (q_cm, sx, hq_cm, hq_rm and sh of `a` are not used); the routing
// results are written for the combination that follows.  With one token the second launch also
// forms the combination into `out` (*combined = true: the caller launches no combine kernel).
bool decode_tiny_supported(int T, int H, int I);
int launch_decode_tiny(const DecodeArgs& a, const __half* logits, int64_t ldl, const __half* x, int64_t ldx, const float* s, int T,
                       const ExpertTab* tab_host, int32_t* idx, float* gw, int32_t* counts, int32_t* offsets, int32_t* perm,
                       int32_t* inv, ExpertTab* tab_dev, __half* out, bool* combined, hipStream_t st);

}  // namespace haq
