// C ABI entry points: argument validation on the host, workspace carving and the
// launch sequence of the linear layer and of the routed expert FFN.
#include <cmath>
#include <cstdarg>
#include <mutex>
#include <new>
#include <vector>

#include "haq_common.h"
#include "moe.h"

namespace haq {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

namespace {

// Bump allocator over the caller's workspace (256-byte granules).
struct Carver {
    uint8_t* base;
    size_t off = 0;
    explicit Carver(void* p) : base((uint8_t*)p) {}
    template <typename T>
    T* take(size_t n) {
        T* r = base ? (T*)(base + off) : nullptr;
        off += (size_t)round_up((int64_t)(n * sizeof(T)), 256);
        return r;
    }
};

constexpr int TILE_M = 256;  // largest row tile of the GEMM: operands are padded by this many rows

inline int64_t padded_rows(int64_t rows) { return round_up(rows, 16) + TILE_M; }

struct LinearWs {
    int8_t* q_cm;
    float* sx;
    int64_t R;
    size_t bytes;
};
LinearWs carve_linear(void* ws, int T, int K) {
    Carver c(ws);
    LinearWs w;
    w.R = padded_rows(T);
    w.q_cm = c.take<int8_t>((size_t)round_up(K, 64) * w.R);  // whole 64-byte k-steps (the pad is never written, its weights are zero)
    w.sx = c.take<float>((size_t)T);
    w.bytes = c.off;
    return w;
}

struct FfnWs {
    int8_t *q1, *q2;
    float *sx1, *sx2;
    __half* h;
    size_t bytes;
};
FfnWs carve_ffn(void* ws, int T, int K, int F) {
    Carver c(ws);
    FfnWs w;
    const int64_t R = padded_rows(T);
    w.q1 = c.take<int8_t>((size_t)round_up(K, 64) * R);
    w.q2 = c.take<int8_t>((size_t)round_up(F, 64) * R);
    w.sx1 = c.take<float>((size_t)T);
    w.sx2 = c.take<float>((size_t)T);
    w.h = c.take<__half>((size_t)T * F);
    w.bytes = c.off;
    return w;
}

struct MoeWs {
    int32_t *idx, *counts, *offsets, *perm, *inv;
    float *gw, *sx, *sx_sorted, *sh;
    ExpertTab* tab;
    int32_t* blk_counts;
    int8_t *q_cm, *hq_cm;
    __half *mid, *y;
    float* pmax;
    int64_t R;
    size_t bytes;
};
MoeWs carve_moe(void* ws, int T, int H, int I, int E) {
    Carver c(ws);
    MoeWs w;
    const size_t P = 2 * (size_t)T;
    w.R = padded_rows((int64_t)P);
    w.idx = c.take<int32_t>(P);
    w.gw = c.take<float>(P);
    w.counts = c.take<int32_t>(E);
    w.offsets = c.take<int32_t>(E + 1);
    w.perm = c.take<int32_t>(P);
    w.inv = c.take<int32_t>(P);
    w.sx = c.take<float>(T);
    w.sx_sorted = c.take<float>(P);
    w.sh = c.take<float>(P);
    w.tab = c.take<ExpertTab>(E);
    w.blk_counts = c.take<int32_t>((size_t)route_blocks(T) * E + 1);
    w.q_cm = c.take<int8_t>((size_t)H * w.R);
    w.hq_cm = c.take<int8_t>((size_t)I * w.R);
    w.mid = c.take<__half>(P * (size_t)I);
    w.y = c.take<__half>(P * (size_t)H);
    w.pmax = c.take<float>(P * (size_t)(I / 32 + 1));
    w.bytes = c.off;
    return w;
}

int quant_packed(const void* x_fp16, int64_t ldx, const float* s, int T, int K, int8_t* q_cm, float* sx, int8_t* q_rm,
                 hipStream_t st) {
    QuantArgs qa{};
    qa.x = (const __half*)x_fp16;
    qa.ldx = ldx;
    qa.s = s;
    qa.T = T;
    qa.K = K;
    qa.q_rm = q_rm;
    qa.ldq = K;
    qa.q_cm = q_cm;
    qa.R = padded_rows(T);
    qa.scale_dest = sx;
    return launch_quant(qa, st);
}

int gemm_packed(const int8_t* q_cm, const float* sx, const int8_t* w_packed, const float* w_scale, int T, int K, int N,
                int act, void* y_fp16, int64_t ldy, int32_t* acc_dbg, hipStream_t st) {
    GemmArgs ga{};
    ga.A = q_cm;
    ga.R = padded_rows(T);
    ga.sx = sx;
    ga.K = K;
    ga.N = N;
    ga.Npad = round_up(N, NPAD);
    ga.M = T;
    ga.B = w_packed;
    ga.sw = w_scale;
    ga.act = act;
    ga.Y = (__half*)y_fp16;
    ga.ldy = ldy;
    ga.acc_dbg = acc_dbg;
    return launch_gemm(ga, EPI_LINEAR, st);
}

}  // namespace
}  // namespace haq

using namespace haq;

// Scratch memory of haq_moe_w8a8_ffn_static: one array per GPU, part of the loaded code object
// (it lives until the process ends).  In host code the name `scratch` is only a handle for the
// symbol; the array's device address is looked up once per device and kept in g_scratch_ptr.
#define HAQ_STATIC_SCRATCH_BYTES (16u << 20)
static __device__ __align__(256) unsigned char scratch[HAQ_STATIC_SCRATCH_BYTES];
static void* g_scratch_ptr[64] = {};
static std::mutex g_scratch_mutex;

static int static_scratch_address(void** out) {
    int dev = -1;
    HAQ_CHECK_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) HAQ_FAIL(HAQ_ERR_UNSUPPORTED, "haq_moe_w8a8_ffn_static: device ordinal %d outside [0, 64)", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        HAQ_CHECK_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) HAQ_FAIL(HAQ_ERR_HIP, "haq_moe_w8a8_ffn_static: the scratch array has no device address");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return HAQ_OK;
}

// Stage timing (haq_profile_*): events recorded at the stage boundaries of the block-level calls.
namespace {
constexpr int PROF_MAX = 16;
struct Profile {
    bool on = false;
    hipEvent_t ev[PROF_MAX + 1] = {};
    const char* name[PROF_MAX] = {};
    int n = -1;  // stages recorded by the last profiled call; -1: none yet
} g_prof;
inline void prof_begin(hipStream_t st) {
    if (!g_prof.on) return;
    g_prof.n = hipEventRecord(g_prof.ev[0], st) == hipSuccess ? 0 : -1;
}
inline void prof_mark(hipStream_t st, const char* name) {  // the stage `name` ends here
    if (!g_prof.on || g_prof.n < 0 || g_prof.n >= PROF_MAX) return;
    if (hipEventRecord(g_prof.ev[g_prof.n + 1], st) != hipSuccess) {
        g_prof.n = -1;
        return;
    }
    g_prof.name[g_prof.n++] = name;
}
}  // namespace

// Context of layers with host-resident experts: staging slots in HBM, the copy stream and the
// events that order copies against the GEMMs that read (and later overwrite) a slot.
struct haq_ctx {
    int H = 0, I = 0, n_slots = 0;
    size_t w13_bytes = 0, w2_bytes = 0;
    hipStream_t copy_stream = nullptr;
    int8_t* slot[32] = {};
    hipEvent_t copied13[32] = {}, copied[32] = {}, done[32] = {};  // gate/up weights landed; both landed; GEMMs over
    hipEvent_t routed = nullptr, call_done = nullptr;
    // timeline of the last call with host-resident experts (timing events): start of the call, first copy
    // issued, last copy landed, end of the call
    hipEvent_t t_start = nullptr, t_copy0 = nullptr, t_copy1 = nullptr, t_end = nullptr;
    bool timed = false, timed_copies = false;
    bool used = false;
    // Offload policy (Section III.C.1a-b): the cost model of Eq. 7-8 and the CPU copies of host-resident
    // experts it may choose; a third stream carries the small copies of the CPU experts' rows
    bool policy_on = false;
    double t_e = 0.0, latency_cpu = 0.0, latency_gpu = 0.0;
    int64_t n_critical = 0;
    int cpu_threads = 0, stage_rows = 0;
    bool has_s_in = false;
    std::vector<float> s_in_host;
    struct CpuReg {
        const void* key;
        const haq_cpu_expert* ex;
    };
    std::vector<CpuReg> cpu_experts;
    hipStream_t aux_stream = nullptr;
    hipEvent_t aux_done = nullptr;
    uint16_t *x_stage = nullptr, *y_stage = nullptr;  // pinned [stage_rows x H]
    int32_t* perm_stage = nullptr;                    // pinned [stage_rows]
    int n_dec = 0;
    int32_t dec_expert[32] = {}, dec_n[32] = {}, dec_what[32] = {};
    int32_t* counts_host = nullptr;  // pinned
    // the slots double as an expert cache with least-recently-used replacement: which host
    // expert (keyed by the address of its gate/up matrix) a slot holds, and when it was last used
    const void* slot_key[32] = {};
    uint64_t slot_tick[32] = {};
    uint64_t tick = 0;
    int64_t hits = 0, misses = 0, bytes_copied = 0;
};

extern "C" {

int32_t haq_version(void) { return 1; }
const char* haq_last_error(void) { return g_err; }

int32_t haq_smoothing_vector(const float* ax, const float* aw, int32_t K, double alpha, float* s) {
    if (K <= 0 || !ax || !s) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_smoothing_vector: K=%d or null buffer", K);
    if (!(alpha >= 0.0 && alpha <= 1.0)) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_smoothing_vector: alpha=%g outside [0,1]", alpha);
    for (int k = 0; k < K; ++k) {
        const double a = ax[k], w = aw ? (double)aw[k] : 1.0;
        double v = 1.0;
        if (a != 0.0 && w != 0.0) {
            v = std::pow(a, alpha) / std::pow(w, 1.0 - alpha);
            v = v < 1e-5 ? 1e-5 : (v > 1e5 ? 1e5 : v);
        }
        s[k] = (float)v;
    }
    return HAQ_OK;
}

size_t haq_linear_workspace_bytes(int32_t T, int32_t K, int32_t N) {
    (void)N;
    if (T < 0 || K <= 0) return 0;
    return carve_linear(nullptr, T, K).bytes;
}

int32_t haq_w8a8_linear(const void* x_fp16, int64_t ldx, const float* s, const int8_t* w_packed, const float* w_scale,
                        int32_t T, int32_t K, int32_t N, int32_t act, void* y_fp16, int64_t ldy, int32_t* acc_dbg,
                        int8_t* q_dbg, float* sx_dbg, void* workspace, size_t workspace_bytes, void* stream) {
    if (T < 0 || K <= 0 || N <= 0) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_w8a8_linear: T=%d K=%d N=%d", T, K, N);
    if (K % 16 != 0 || K > 65536 || N % 16 != 0)
        HAQ_FAIL(HAQ_ERR_UNSUPPORTED, "haq_w8a8_linear: K=%d must be a multiple of 16 (<= 65536), N=%d of 16", K, N);
    if (act != HAQ_ACT_NONE && act != HAQ_ACT_RELU) HAQ_FAIL(HAQ_ERR_UNSUPPORTED, "haq_w8a8_linear: act=%d", act);
    if (T == 0) return HAQ_OK;
    if (!x_fp16 || !w_packed || !w_scale || !y_fp16) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_w8a8_linear: null buffer");
    if (ldx < K || ldx % 8 != 0 || ldy < N || ldy % 8 != 0)
        HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_w8a8_linear: ldx=%lld ldy=%lld (multiples of 8)", (long long)ldx, (long long)ldy);
    if (!aligned16(x_fp16) || !aligned16(w_packed) || !aligned16(y_fp16) || (s && !aligned16(s)) || (q_dbg && !aligned16(q_dbg)))
        HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_w8a8_linear: pointers must be 16-byte aligned");
    const size_t need = carve_linear(nullptr, T, K).bytes;
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255u))
        HAQ_FAIL(HAQ_ERR_WORKSPACE, "haq_w8a8_linear: workspace of %zu bytes (256-byte aligned) needed, got %zu", need, workspace_bytes);
    hipStream_t st = (hipStream_t)stream;
    const LinearWs w = carve_linear(workspace, T, K);
    int rc = quant_packed(x_fp16, ldx, s, T, K, w.q_cm, w.sx, q_dbg, st);
    if (rc != HAQ_OK) return rc;
    if (sx_dbg) HAQ_CHECK_HIP(hipMemcpyAsync(sx_dbg, w.sx, (size_t)T * sizeof(float), hipMemcpyDeviceToDevice, st));
    return gemm_packed(w.q_cm, w.sx, w_packed, w_scale, T, K, N, act, y_fp16, ldy, acc_dbg, st);
}

size_t haq_linear_kn_workspace_bytes(int32_t T, int32_t K, int32_t N) {
    if (T < 0 || K <= 0 || N <= 0) return 0;
    return carve_linear(nullptr, T, K).bytes + (size_t)round_up((int64_t)haq_packed_bytes(K, N), 256);
}

int32_t haq_w8a8_linear_kn(const void* x_fp16, int64_t ldx, const float* s, const int8_t* wq_kn, const float* w_scale, int32_t T,
                           int32_t K, int32_t N, int32_t act, void* y_fp16, int64_t ldy, void* workspace, size_t workspace_bytes,
                           void* stream) {
    if (T < 0 || K <= 0 || N <= 0) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_w8a8_linear_kn: T=%d K=%d N=%d", T, K, N);
    if (K % 16 != 0 || K > 65536 || N % 16 != 0)
        HAQ_FAIL(HAQ_ERR_UNSUPPORTED, "haq_w8a8_linear_kn: K=%d must be a multiple of 16 (<= 65536), N=%d of 16", K, N);
    if (T == 0) return HAQ_OK;
    if (!wq_kn) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_w8a8_linear_kn: null buffer");
    const size_t lin = carve_linear(nullptr, T, K).bytes, need = haq_linear_kn_workspace_bytes(T, K, N);
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255u))
        HAQ_FAIL(HAQ_ERR_WORKSPACE, "haq_w8a8_linear_kn: workspace of %zu bytes (256-byte aligned) needed, got %zu", need, workspace_bytes);
    int8_t* packed = (int8_t*)workspace + lin;
    const int rc = haq_pack_weight(wq_kn, K, N, packed, stream);
    if (rc != HAQ_OK) return rc;
    return haq_w8a8_linear(x_fp16, ldx, s, packed, w_scale, T, K, N, act, y_fp16, ldy, nullptr, nullptr, nullptr, workspace, lin, stream);
}

size_t haq_linear_asym_workspace_bytes(int32_t T, int32_t K, int32_t N) {
    (void)N;
    if (T < 0 || K <= 0) return 0;
    return carve_linear(nullptr, T, K).bytes + (size_t)round_up((int64_t)(T > 0 ? T : 1) * 4, 256);
}

int32_t haq_w8a8_linear_asym(const void* x_fp16, int64_t ldx, const float* s, const int8_t* w_packed, const float* w_scale,
                             const int32_t* w_colsum, int32_t T, int32_t K, int32_t N, int32_t act, void* y_fp16,
                             int64_t ldy, int32_t* acc_dbg, uint8_t* q_dbg, float* sx_dbg, int32_t* zp_dbg, void* workspace,
                             size_t workspace_bytes, void* stream) {
    if (T < 0 || K <= 0 || N <= 0) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_w8a8_linear_asym: T=%d K=%d N=%d", T, K, N);
    if (K % 16 != 0 || K > 16384 || N % 16 != 0)
        HAQ_FAIL(HAQ_ERR_UNSUPPORTED, "haq_w8a8_linear_asym: K=%d must be a multiple of 16 (<= 16384), N=%d of 16", K, N);
    if (act != HAQ_ACT_NONE && act != HAQ_ACT_RELU) HAQ_FAIL(HAQ_ERR_UNSUPPORTED, "haq_w8a8_linear_asym: act=%d", act);
    if (T == 0) return HAQ_OK;
    if (!x_fp16 || !w_packed || !w_scale || !w_colsum || !y_fp16) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_w8a8_linear_asym: null buffer");
    if (ldx < K || ldx % 8 != 0 || ldy < N || ldy % 8 != 0)
        HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_w8a8_linear_asym: ldx=%lld ldy=%lld (multiples of 8)", (long long)ldx, (long long)ldy);
    if (!aligned16(x_fp16) || !aligned16(w_packed) || !aligned16(y_fp16) || (s && !aligned16(s)) || (q_dbg && !aligned16(q_dbg)))
        HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_w8a8_linear_asym: pointers must be 16-byte aligned");
    const size_t need = haq_linear_asym_workspace_bytes(T, K, N);
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255u))
        HAQ_FAIL(HAQ_ERR_WORKSPACE, "haq_w8a8_linear_asym: workspace of %zu bytes (256-byte aligned) needed, got %zu", need, workspace_bytes);
    hipStream_t st = (hipStream_t)stream;
    const LinearWs w = carve_linear(workspace, T, K);
    int32_t* zp = reinterpret_cast<int32_t*>((uint8_t*)workspace + w.bytes);
    // long batches: the pipelined quantiser; short ones: the register-resident kernel
    QuantArgs pa{};
    pa.x = (const __half*)x_fp16;
    pa.ldx = ldx;
    pa.s = s;
    pa.T = T;
    pa.K = K;
    pa.q_rm = (int8_t*)q_dbg;
    pa.ldq = K;
    pa.q_cm = w.q_cm;
    pa.R = w.R;
    pa.scale_dest = w.sx;
    pa.zp_dest = zp;
    int rc = launch_quant(pa, st);
    if (rc == HAQ_ERR_UNSUPPORTED) rc = launch_asym_quant((const __half*)x_fp16, ldx, s, T, K, w.q_cm, w.R, q_dbg, K, w.sx, zp, st);
    if (rc == HAQ_ERR_UNSUPPORTED) HAQ_FAIL(HAQ_ERR_UNSUPPORTED, "haq_w8a8_linear_asym: K=%d not supported", K);
    if (rc != HAQ_OK) return rc;
    if (sx_dbg) HAQ_CHECK_HIP(hipMemcpyAsync(sx_dbg, w.sx, (size_t)T * sizeof(float), hipMemcpyDeviceToDevice, st));
    if (zp_dbg) HAQ_CHECK_HIP(hipMemcpyAsync(zp_dbg, zp, (size_t)T * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
    GemmArgs ga{};
    ga.A = w.q_cm;
    ga.R = w.R;
    ga.sx = w.sx;
    ga.K = K;
    ga.N = N;
    ga.Npad = round_up(N, NPAD);
    ga.M = T;
    ga.B = w_packed;
    ga.sw = w_scale;
    ga.act = act;
    ga.Y = (__half*)y_fp16;
    ga.ldy = ldy;
    ga.acc_dbg = acc_dbg;
    ga.zp = zp;
    ga.colsum = w_colsum;
    return launch_gemm(ga, EPI_LINEAR_ASYM, st);
}

size_t haq_ffn_workspace_bytes(int32_t T, int32_t K, int32_t F, int32_t N) {
    (void)N;
    if (T < 0 || K <= 0 || F <= 0) return 0;
    return carve_ffn(nullptr, T, K, F).bytes;
}

int32_t haq_w8a8_ffn(const void* x_fp16, int64_t ldx, const float* s1, const int8_t* w1_packed, const float* w1_scale,
                     int32_t act, const float* s2, const int8_t* w2_packed, const float* w2_scale, int32_t T, int32_t K,
                     int32_t F, int32_t N, void* y_fp16, int64_t ldy, void* h_dbg_fp16, void* workspace,
                     size_t workspace_bytes, void* stream) {
    if (T < 0 || K <= 0 || F <= 0 || N <= 0) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_w8a8_ffn: T=%d K=%d F=%d N=%d", T, K, F, N);
    if (K % 16 != 0 || F % 16 != 0 || N % 16 != 0 || K > 65536 || F > 65536)
        HAQ_FAIL(HAQ_ERR_UNSUPPORTED, "haq_w8a8_ffn: K=%d and F=%d must be multiples of 16 (<= 65536), N=%d of 16", K, F, N);
    if (act != HAQ_ACT_NONE && act != HAQ_ACT_RELU) HAQ_FAIL(HAQ_ERR_UNSUPPORTED, "haq_w8a8_ffn: act=%d", act);
    if (T == 0) return HAQ_OK;
    if (!x_fp16 || !w1_packed || !w1_scale || !w2_packed || !w2_scale || !y_fp16) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_w8a8_ffn: null buffer");
    if (ldx < K || ldx % 8 != 0 || ldy < N || ldy % 8 != 0)
        HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_w8a8_ffn: ldx=%lld ldy=%lld (multiples of 8)", (long long)ldx, (long long)ldy);
    if (!aligned16(x_fp16) || !aligned16(w1_packed) || !aligned16(w2_packed) || !aligned16(y_fp16) || (s1 && !aligned16(s1)) ||
        (s2 && !aligned16(s2)) || (h_dbg_fp16 && !aligned16(h_dbg_fp16)))
        HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_w8a8_ffn: pointers must be 16-byte aligned");
    const size_t need = carve_ffn(nullptr, T, K, F).bytes;
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255u))
        HAQ_FAIL(HAQ_ERR_WORKSPACE, "haq_w8a8_ffn: workspace of %zu bytes (256-byte aligned) needed, got %zu", need, workspace_bytes);
    hipStream_t st = (hipStream_t)stream;
    const FfnWs w = carve_ffn(workspace, T, K, F);
    __half* h = h_dbg_fp16 ? (__half*)h_dbg_fp16 : w.h;
    prof_begin(st);
    int rc = quant_packed(x_fp16, ldx, s1, T, K, w.q1, w.sx1, nullptr, st);
    if (rc != HAQ_OK) return rc;
    prof_mark(st, "quantise X");
    if ((rc = gemm_packed(w.q1, w.sx1, w1_packed, w1_scale, T, K, F, act, h, F, nullptr, st)) != HAQ_OK) return rc;
    prof_mark(st, "GEMM 1 + activation");
    if ((rc = quant_packed(h, F, s2, T, F, w.q2, w.sx2, nullptr, st)) != HAQ_OK) return rc;
    prof_mark(st, "requantise H");
    rc = gemm_packed(w.q2, w.sx2, w2_packed, w2_scale, T, F, N, HAQ_ACT_NONE, y_fp16, ldy, nullptr, st);
    prof_mark(st, "GEMM 2");
    return rc;
}

int64_t haq_packed_act_rows(int32_t T) { return T < 0 ? 0 : padded_rows(T); }
size_t haq_packed_act_bytes(int32_t T, int32_t K) { return (T < 0 || K <= 0) ? 0 : (size_t)round_up(K, 64) * (size_t)padded_rows(T); }

int32_t haq_quant_act_packed(const void* x_fp16, int64_t ldx, const float* s, int32_t T, int32_t K, int8_t* q_packed,
                             float* row_scale, void* stream) {
    if (T < 0 || K <= 0) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_quant_act_packed: T=%d K=%d", T, K);
    if (K % 16 != 0 || K > 65536) HAQ_FAIL(HAQ_ERR_UNSUPPORTED, "haq_quant_act_packed: K=%d must be a multiple of 16, <= 65536", K);
    if (T == 0) return HAQ_OK;
    if (!x_fp16 || !q_packed || !row_scale) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_quant_act_packed: null buffer");
    if (ldx < K || ldx % 8 != 0) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_quant_act_packed: ldx=%lld", (long long)ldx);
    if (!aligned16(x_fp16) || !aligned16(q_packed) || (s && !aligned16(s)))
        HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_quant_act_packed: pointers must be 16-byte aligned");
    return quant_packed(x_fp16, ldx, s, T, K, q_packed, row_scale, nullptr, (hipStream_t)stream);
}

int32_t haq_gemm_w8a8_packed(const int8_t* q_packed, const float* row_scale, const int8_t* w_packed, const float* w_scale,
                             int32_t T, int32_t K, int32_t N, int32_t act, void* y_fp16, int64_t ldy, int32_t* acc_dbg,
                             void* stream) {
    if (T < 0 || K <= 0 || N <= 0) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_gemm_w8a8_packed: T=%d K=%d N=%d", T, K, N);
    if (K % 16 != 0 || N % 16 != 0) HAQ_FAIL(HAQ_ERR_UNSUPPORTED, "haq_gemm_w8a8_packed: K=%d must be a multiple of 16, N=%d of 16", K, N);
    if (act != HAQ_ACT_NONE && act != HAQ_ACT_RELU) HAQ_FAIL(HAQ_ERR_UNSUPPORTED, "haq_gemm_w8a8_packed: act=%d", act);
    if (T == 0) return HAQ_OK;
    if (!q_packed || !row_scale || !w_packed || !w_scale || !y_fp16) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_gemm_w8a8_packed: null buffer");
    if (ldy < N || ldy % 8 != 0) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_gemm_w8a8_packed: ldy=%lld (multiple of 8)", (long long)ldy);
    if (!aligned16(q_packed) || !aligned16(w_packed) || !aligned16(y_fp16)) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_gemm_w8a8_packed: pointers must be 16-byte aligned");
    return gemm_packed(q_packed, row_scale, w_packed, w_scale, T, K, N, act, y_fp16, ldy, acc_dbg, (hipStream_t)stream);
}

int32_t haq_ctx_create(int32_t H, int32_t I, int32_t n_slots, haq_ctx** out) {
    if (!out) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_ctx_create: null output");
    *out = nullptr;
    if (H <= 0 || I <= 0 || n_slots < 1 || n_slots > 32) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_ctx_create: H=%d I=%d n_slots=%d", H, I, n_slots);
    haq_ctx* c = new (std::nothrow) haq_ctx();
    if (!c) HAQ_FAIL(HAQ_ERR_HIP, "haq_ctx_create: out of host memory");
    c->H = H;
    c->I = I;
    c->n_slots = n_slots;
    c->w13_bytes = haq_packed_bytes(H, 2 * I);
    c->w2_bytes = haq_packed_bytes(I, H);
    hipError_t e = hipStreamCreateWithFlags(&c->copy_stream, hipStreamNonBlocking);  // default priority
    for (int i = 0; e == hipSuccess && i < n_slots; ++i) e = hipMalloc((void**)&c->slot[i], c->w13_bytes + c->w2_bytes);
    for (int i = 0; e == hipSuccess && i < 32; ++i) {
        e = hipEventCreateWithFlags(&c->copied[i], hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&c->copied13[i], hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&c->done[i], hipEventDisableTiming);
    }
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c->routed, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c->call_done, hipEventDisableTiming);
    for (hipEvent_t* t : {&c->t_start, &c->t_copy0, &c->t_copy1, &c->t_end})
        if (e == hipSuccess) e = hipEventCreate(t);
    if (e == hipSuccess) e = hipHostMalloc((void**)&c->counts_host, 32 * sizeof(int32_t), hipHostMallocDefault);
    if (e != hipSuccess) {
        set_error("haq_ctx_create: %s", hipGetErrorString(e));
        haq_ctx_destroy(c);
        return HAQ_ERR_HIP;
    }
    *out = c;
    return HAQ_OK;
}

int32_t haq_ctx_destroy(haq_ctx* c) {
    if (!c) return HAQ_OK;
    if (c->copy_stream) (void)hipStreamSynchronize(c->copy_stream);
    for (int i = 0; i < 32; ++i) {
        if (c->slot[i]) (void)hipFree(c->slot[i]);
        if (c->copied[i]) (void)hipEventDestroy(c->copied[i]);
        if (c->copied13[i]) (void)hipEventDestroy(c->copied13[i]);
        if (c->done[i]) (void)hipEventDestroy(c->done[i]);
    }
    if (c->routed) (void)hipEventDestroy(c->routed);
    if (c->call_done) (void)hipEventDestroy(c->call_done);
    for (hipEvent_t t : {c->t_start, c->t_copy0, c->t_copy1, c->t_end})
        if (t) (void)hipEventDestroy(t);
    if (c->counts_host) (void)hipHostFree(c->counts_host);
    if (c->aux_stream) (void)hipStreamSynchronize(c->aux_stream);
    if (c->x_stage) (void)hipHostFree(c->x_stage);
    if (c->y_stage) (void)hipHostFree(c->y_stage);
    if (c->perm_stage) (void)hipHostFree(c->perm_stage);
    if (c->aux_done) (void)hipEventDestroy(c->aux_done);
    if (c->aux_stream) (void)hipStreamDestroy(c->aux_stream);
    if (c->copy_stream) (void)hipStreamDestroy(c->copy_stream);
    delete c;
    return HAQ_OK;
}

int32_t haq_ctx_cache_stats(const haq_ctx* c, int64_t* hits, int64_t* misses, int64_t* bytes_copied, const void** slot_keys) {
    if (!c) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_ctx_cache_stats: null context");
    if (hits) *hits = c->hits;
    if (misses) *misses = c->misses;
    if (bytes_copied) *bytes_copied = c->bytes_copied;
    if (slot_keys)
        for (int i = 0; i < c->n_slots; ++i) slot_keys[i] = c->slot_key[i];
    return HAQ_OK;
}

int32_t haq_ctx_cache_invalidate(haq_ctx* c) {
    if (!c) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_ctx_cache_invalidate: null context");
    for (int i = 0; i < 32; ++i) {
        c->slot_key[i] = nullptr;
        c->slot_tick[i] = 0;
    }
    return HAQ_OK;
}

size_t haq_moe_workspace_bytes(int32_t T, int32_t H, int32_t I, int32_t E) {
    if (T < 0 || H <= 0 || I <= 0 || E <= 0) return 0;
    return carve_moe(nullptr, T, H, I, E).bytes;
}

int32_t haq_moe_w8a8_ffn(haq_ctx* ctx, const void* x_fp16, int64_t ldx, const void* logits_fp16, int64_t ldl,
                         const float* s_in, const haq_expert_desc* experts, int32_t T, int32_t H, int32_t I, int32_t E,
                         int32_t top_k, void* out_fp16, int64_t ldo, const haq_moe_debug* dbg, void* workspace,
                         size_t workspace_bytes, void* stream) {
    if (T < 0 || H <= 0 || I <= 0 || E <= 0) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_moe_w8a8_ffn: T=%d H=%d I=%d E=%d", T, H, I, E);
    if (top_k != 2) HAQ_FAIL(HAQ_ERR_UNSUPPORTED, "haq_moe_w8a8_ffn: top_k=%d (only 2)", top_k);
    if (E < 2 || E > 32) HAQ_FAIL(HAQ_ERR_UNSUPPORTED, "haq_moe_w8a8_ffn: E=%d outside [2, 32]", E);
    if (H % 64 != 0 || I % 64 != 0 || H > 65536 || I > 65536)
        HAQ_FAIL(HAQ_ERR_UNSUPPORTED, "haq_moe_w8a8_ffn: H=%d and I=%d must be multiples of 64 (both <= 65536)", H, I);
    if (T == 0) return HAQ_OK;
    if (!x_fp16 || !logits_fp16 || !experts || !out_fp16) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_moe_w8a8_ffn: null buffer");
    if (ldx < H || ldx % 8 != 0 || ldl < E || ldo < H || ldo % 8 != 0)
        HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_moe_w8a8_ffn: ldx=%lld ldl=%lld ldo=%lld", (long long)ldx, (long long)ldl, (long long)ldo);
    if (!aligned16(x_fp16) || !aligned16(out_fp16) || (s_in && !aligned16(s_in)))
        HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_moe_w8a8_ffn: pointers must be 16-byte aligned");
    if (dbg && ((dbg->q && !aligned16(dbg->q)) || (dbg->hq && !aligned16(dbg->hq)) || (dbg->mid_fp16 && !aligned16(dbg->mid_fp16)) ||
                (dbg->y_fp16 && !aligned16(dbg->y_fp16))))
        HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_moe_w8a8_ffn: debug buffers q, hq, mid_fp16 and y_fp16 must be 16-byte aligned");
    ExpertTab tab[32];
    int host_expert[32], n_host = 0;
    for (int e = 0; e < E; ++e) {
        const haq_expert_desc& d = experts[e];
        if (!d.w13 || !d.w2 || !d.sw1 || !d.sw3 || !d.sw2 || !d.s_mid)
            HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_moe_w8a8_ffn: expert %d has a null pointer", e);
        if (!aligned16(d.w13) || !aligned16(d.w2) || !aligned16(d.s_mid) || !aligned16(d.sw1) || !aligned16(d.sw3) || !aligned16(d.sw2))
            HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_moe_w8a8_ffn: expert %d pointers must be 16-byte aligned", e);
        tab[e] = ExpertTab{d.w13, d.w2, d.sw1, d.sw3, d.sw2, d.s_mid};
        if (d.location != HAQ_LOC_DEVICE) {
            if (d.location != HAQ_LOC_HOST_PINNED) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_moe_w8a8_ffn: expert %d location=%d", e, d.location);
            if (!ctx) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_moe_w8a8_ffn: expert %d is host resident but no context was given", e);
            if (ctx->H != H || ctx->I != I) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_moe_w8a8_ffn: context was created for H=%d I=%d", ctx->H, ctx->I);
            host_expert[n_host++] = e;  // its slot is chosen once the routing histogram is known
        }
    }
    const size_t need = carve_moe(nullptr, T, H, I, E).bytes;
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255u))
        HAQ_FAIL(HAQ_ERR_WORKSPACE, "haq_moe_w8a8_ffn: workspace of %zu bytes (256-byte aligned) needed, got %zu", need, workspace_bytes);

    hipStream_t st = (hipStream_t)stream;
    MoeWs w = carve_moe(workspace, T, H, I, E);
    const int P = 2 * T;
    haq_moe_debug d{};
    if (dbg) d = *dbg;
    // debug buffers with the same shape as a workspace buffer simply take its place
    int32_t* idx = d.topk_idx ? d.topk_idx : w.idx;
    float* gw = d.topk_w ? d.topk_w : w.gw;
    int32_t* counts = d.counts ? d.counts : w.counts;
    int32_t* offsets = d.offsets ? d.offsets : w.offsets;
    int32_t* perm = d.perm ? d.perm : w.perm;
    int32_t* inv = d.inv ? d.inv : w.inv;
    __half* mid = d.mid_fp16 ? (__half*)d.mid_fp16 : w.mid;
    __half* y = d.y_fp16 ? (__half*)d.y_fp16 : w.y;
    float* sh = d.sh ? d.sh : w.sh;

    int rc;
    prof_begin(st);
    const bool decode_path = n_host == 0 && decode_supported(T, H, I);
    // one or two tokens, and none of the intermediate outputs the fused kernels keep on chip is asked for
    const bool tiny_path = decode_path && decode_tiny_supported(T, H, I) && !d.q && !d.sx && !d.hq && !d.sh;
    if (tiny_path) {
        // routing and token quantisation happen inside the gate/up launch below
    } else if (decode_path && decode_prologue_supported(T, H)) {
        // few tokens: routing, permutation and token quantisation in one launch
        if ((rc = launch_decode_prologue((const __half*)logits_fp16, ldl, T, E, tab, w.tab, idx, gw, counts, offsets, perm, inv,
                                         (const __half*)x_fp16, ldx, s_in, H, w.q_cm, w.R, d.q, d.sx, w.sx_sorted, st)) != HAQ_OK)
            return rc;
    } else {
    if ((rc = launch_route_permute((const __half*)logits_fp16, ldl, T, E, tab, w.tab, idx, gw, counts, offsets, perm, inv,
                                   w.blk_counts, st)) != HAQ_OK)
        return rc;

    QuantArgs qa{};
    qa.x = (const __half*)x_fp16;
    qa.ldx = ldx;
    qa.s = s_in;
    qa.T = P;  // one output row per (token, expert) pair, in sorted order
    qa.K = H;
    qa.q_rm = d.q;
    qa.ldq = H;
    qa.q_cm = w.q_cm;
    qa.R = w.R;
    qa.gather = perm;
    qa.scale = d.sx;
    qa.scale_dest = w.sx_sorted;
    if ((rc = launch_quant(qa, st)) != HAQ_OK) return rc;
    }
    if (!tiny_path) prof_mark(st, "route + permute + quantise tokens");

    if (decode_path) {
        // few rows per expert: stream every activated expert's weights once
        DecodeArgs da{};
        da.q_cm = w.q_cm;
        da.sx = w.sx_sorted;
        da.R = w.R;
        da.offsets = offsets;
        da.tab = w.tab;
        da.E = E;
        da.H = H;
        da.I = I;
        da.Npad13 = round_up(2 * (int64_t)I, NPAD);
        da.Npad2 = round_up(H, NPAD);
        da.mid = mid;
        da.pmax = w.pmax;
        da.hq_cm = w.hq_cm;
        da.hq_rm = d.hq;
        da.sh = sh;
        da.y = y;
        bool combined = false;
        if (tiny_path)
            rc = launch_decode_tiny(da, (const __half*)logits_fp16, ldl, (const __half*)x_fp16, ldx, s_in, T, tab, idx, gw, counts,
                                    offsets, perm, inv, w.tab, (__half*)out_fp16, &combined, st);
        else
            rc = launch_decode(da, T, st);
        if (rc != HAQ_OK) return rc;
        prof_mark(st, combined ? "route + quantise + gate/up + requantise + down + combine (2 launches)"
                  : tiny_path ? "route + quantise + gate/up + requantise + down (2 launches)" : "gate/up + requantise + down (3 launches)");
        if (combined) return HAQ_OK;
        rc = launch_combine(y, H, inv, gw, T, H, (__half*)out_fp16, ldo, st);
        prof_mark(st, "combine");
        return rc;
    }

    // gate/up GEMM + SwiGLU, requantisation and down GEMM for a set of experts (rows of the others untouched)
    // (before_down: an event the launch stream waits for between the requantisation and the down GEMM)
    auto run_experts = [&](const int* sel, int n_sel, int max_rows, hipEvent_t before_down = nullptr) -> int {
        GemmArgs g1{};
        g1.A = w.q_cm;
        g1.R = w.R;
        g1.sx = w.sx_sorted;
        g1.K = H;
        g1.N = 2 * I;
        g1.Npad = round_up(2 * (int64_t)I, NPAD);
        g1.offsets = offsets;
        g1.tab = w.tab;
        g1.which = 0;
        g1.n_sel = n_sel;
        for (int i = 0; i < n_sel; ++i) g1.sel[i] = sel[i];
        g1.max_rows = max_rows;
        g1.Y = mid;
        g1.ldy = I;
        int r = launch_gemm(g1, EPI_SWIGLU, st);
        if (r != HAQ_OK) return r;
        if (n_host == 0) prof_mark(st, "grouped gate/up GEMM + SwiGLU");

        QuantArgs qb{};
        qb.x = mid;
        qb.ldx = I;
        qb.tab = w.tab;
        qb.offsets = offsets;
        qb.E = E;
        qb.T = P;
        qb.K = I;
        qb.q_rm = d.hq;
        qb.ldq = I;
        qb.q_cm = w.hq_cm;
        qb.R = w.R;
        qb.scale_dest = sh;
        qb.n_sel = n_sel;
        for (int i = 0; i < n_sel; ++i) qb.sel[i] = sel[i];
        qb.max_rows = max_rows;
        if ((r = launch_quant(qb, st)) != HAQ_OK) return r;
        if (n_host == 0) prof_mark(st, "requantise intermediate");
        if (before_down) HAQ_CHECK_HIP(hipStreamWaitEvent(st, before_down, 0));

        GemmArgs g2{};
        g2.A = w.hq_cm;
        g2.R = w.R;
        g2.sx = sh;
        g2.K = I;
        g2.N = H;
        g2.Npad = round_up(H, NPAD);
        g2.offsets = offsets;
        g2.tab = w.tab;
        g2.which = 1;
        g2.n_sel = n_sel;
        for (int i = 0; i < n_sel; ++i) g2.sel[i] = sel[i];
        g2.max_rows = max_rows;
        g2.act = HAQ_ACT_NONE;
        g2.Y = y;
        g2.ldy = H;
        return launch_gemm(g2, EPI_LINEAR, st);
    };

    if (n_host == 0) {
        int all[32];
        for (int e = 0; e < E; ++e) all[e] = e;
        if ((rc = run_experts(all, E, P)) != HAQ_OK) return rc;
        prof_mark(st, "grouped down GEMM");
        rc = launch_combine(y, H, inv, gw, T, H, (__half*)out_fp16, ldo, st);
        prof_mark(st, "combine");
        return rc;
    }

    // ---- some experts live in pinned host memory (Section III.C: experts are moved in their
    // low-bit form).  The routing result comes back to the host (one small blocking copy), the
    // activated host experts are copied into the staging slots on the copy stream, and the
    // device-resident experts compute meanwhile; each streamed expert computes as soon as its
    // copy has landed and frees its slot for the expert n_slots further down the list.
    ctx->timed = false;
    HAQ_CHECK_HIP(hipEventRecord(ctx->t_start, st));
    HAQ_CHECK_HIP(hipMemcpyAsync(ctx->counts_host, counts, (size_t)E * sizeof(int32_t), hipMemcpyDeviceToHost, st));
    HAQ_CHECK_HIP(hipEventRecord(ctx->routed, st));
    HAQ_CHECK_HIP(hipEventSynchronize(ctx->routed));
    int resident[32], n_res = 0, res_rows = 0;
    bool is_host[32] = {};
    for (int i = 0; i < n_host; ++i) is_host[host_expert[i]] = true;
    for (int e = 0; e < E; ++e)
        if (!is_host[e] && ctx->counts_host[e] > 0) {
            resident[n_res++] = e;
            res_rows += ctx->counts_host[e];
        }
    // Activated host experts in expert order go through the expert cache (Section III.C.1c): a
    // hit costs no transfer, a miss takes a free slot, else the least recently used one.  With
    // more activated host experts than slots the victim may be a slot handed out earlier in this
    // very call: the copy then waits for that expert's GEMMs.  The plan is made on copies of the
    // cache state; the context only takes it over once every copy and launch of the call is
    // enqueued, so a call that fails half way never leaves a slot labelled with weights that did
    // not arrive.
    // Decision per activated host expert (Section III.C.1b): one that the cache holds computes on the GPU;
    // otherwise, with a cost model set and a CPU copy registered, it is transferred only if its batch
    // exceeds the break-even size of Eq. 7-8 and computed on the CPU if not.
    int order[32], n_order = 0, cpu_list[32], n_cpu = 0;
    const haq_cpu_expert* cpu_of[32] = {};
    ctx->n_dec = 0;
    for (int i = 0; i < n_host; ++i) {
        const int e = host_expert[i], n = ctx->counts_host[e];
        if (n <= 0) continue;
        const void* key = experts[e].w13;
        bool cached = false;
        for (int c = 0; c < ctx->n_slots; ++c) cached = cached || ctx->slot_key[c] == key;
        int what = cached ? HAQ_DECISION_GPU_CACHED : HAQ_DECISION_TRANSFER;
        if (!cached && ctx->policy_on && (ctx->n_critical < 0 || n <= ctx->n_critical) && n <= ctx->stage_rows &&
            (!s_in || ctx->has_s_in)) {
            for (const auto& r : ctx->cpu_experts)
                if (r.key == key) cpu_of[e] = r.ex;
            if (cpu_of[e]) what = HAQ_DECISION_CPU;
        }
        ctx->dec_expert[ctx->n_dec] = e;
        ctx->dec_n[ctx->n_dec] = n;
        ctx->dec_what[ctx->n_dec++] = what;
        if (what == HAQ_DECISION_CPU)
            cpu_list[n_cpu++] = e;
        else
            order[n_order++] = e;
    }
    uint64_t keys_l[32], ticks_l[32], tick_l = ctx->tick, req[32];
    for (int c = 0; c < 32; ++c) {
        keys_l[c] = (uint64_t)(uintptr_t)ctx->slot_key[c];
        ticks_l[c] = ctx->slot_tick[c];
    }
    for (int k = 0; k < n_order; ++k) req[k] = (uint64_t)(uintptr_t)experts[order[k]].w13;
    int32_t slot_of[32], prev_user[32], hit[32];
    if (n_order > 0 && (rc = haq_lru_plan(ctx->n_slots, keys_l, ticks_l, &tick_l, req, n_order, slot_of, hit, prev_user)) != HAQ_OK)
        return rc;
    int n_hit = 0;
    for (int k = 0; k < n_order; ++k) {
        n_hit += hit[k] ? 1 : 0;
        tab[order[k]].w13 = ctx->slot[slot_of[k]];
        tab[order[k]].w2 = ctx->slot[slot_of[k]] + ctx->w13_bytes;
    }

    bool issued[32] = {};
    auto issue_copy = [&](int k) -> int {
        const int e = order[k];
        int8_t* slot = ctx->slot[slot_of[k]];
        HAQ_CHECK_HIP(hipMemcpyAsync(slot, experts[e].w13, ctx->w13_bytes, hipMemcpyHostToDevice, ctx->copy_stream));
        HAQ_CHECK_HIP(hipEventRecord(ctx->copied13[k], ctx->copy_stream));
        HAQ_CHECK_HIP(hipMemcpyAsync(slot + ctx->w13_bytes, experts[e].w2, ctx->w2_bytes, hipMemcpyHostToDevice, ctx->copy_stream));
        HAQ_CHECK_HIP(hipEventRecord(ctx->copied[k], ctx->copy_stream));
        issued[k] = true;
        return HAQ_OK;
    };
    int off_host[33] = {0};
    for (int e = 0; e < E; ++e) off_host[e + 1] = off_host[e] + ctx->counts_host[e];
    auto enqueue = [&]() -> int {
        int r;
        // slots may still be read by the previous call on another stream
        if (ctx->used) {
            HAQ_CHECK_HIP(hipStreamWaitEvent(ctx->copy_stream, ctx->call_done, 0));
            // and a cached expert was copied during an earlier call, possibly issued from another stream
            HAQ_CHECK_HIP(hipStreamWaitEvent(st, ctx->call_done, 0));
        }
        if ((r = launch_set_tab(tab, E, w.tab, st)) != HAQ_OK) return r;
        HAQ_CHECK_HIP(hipEventRecord(ctx->t_copy0, ctx->copy_stream));
        // misses whose slot is not in use by an earlier expert of this call are copied right away
        for (int k = 0; k < n_order; ++k)
            if (!hit[k] && prev_user[k] < 0 && (r = issue_copy(k)) != HAQ_OK) return r;
        // Device-resident experts, and cached ones whose slot nobody evicts later in this call, compute as
        // one grouped launch while the first copies are in flight.
        bool grouped[32] = {};
        for (int k = 0; k < n_order; ++k) {
            bool evicted_later = false;
            for (int k2 = k + 1; k2 < n_order; ++k2) evicted_later = evicted_later || prev_user[k2] == k;
            if (hit[k] && !evicted_later) {
                grouped[k] = true;
                resident[n_res++] = order[k];
                res_rows += ctx->counts_host[order[k]];
            }
        }
        if (n_res > 0 && (r = run_experts(resident, n_res, res_rows)) != HAQ_OK) return r;
        for (int k = 0; k < n_order; ++k) {
            const int e = order[k];
            if (grouped[k]) continue;
            // a streamed expert's gate/up projection starts when its gate/up weights have landed, under the copy of
            // its down weights; the down projection waits for those
            if (!hit[k]) {
                if (!issued[k]) HAQ_FAIL(HAQ_ERR_HIP, "haq_moe_w8a8_ffn: internal error, expert copy never issued");
                HAQ_CHECK_HIP(hipStreamWaitEvent(st, ctx->copied13[k], 0));
            }
            const int n_e = ctx->counts_host[e];
            hipEvent_t w2_landed = hit[k] ? nullptr : ctx->copied[k];
            if (n_e <= 64 && decode_supported(n_e, H, I)) {
                // few rows: stream the expert's weights once through the weight-streaming kernels instead of
                // running the tiled GEMMs on a handful of work-groups (same arithmetic, same bits)
                DecodeArgs da{};
                da.q_cm = w.q_cm;
                da.sx = w.sx_sorted;
                da.R = w.R;
                da.offsets = offsets;
                da.tab = w.tab;
                da.E = E;
                da.H = H;
                da.I = I;
                da.Npad13 = round_up(2 * (int64_t)I, NPAD);
                da.Npad2 = round_up(H, NPAD);
                da.mid = mid;
                da.pmax = w.pmax;
                da.hq_cm = w.hq_cm;
                da.hq_rm = d.hq;
                da.sh = sh;
                da.y = y;
                r = launch_decode_one_expert(da, e, off_host[e], n_e, w2_landed, st);
            } else {
                r = run_experts(&e, 1, n_e, w2_landed);
            }
            if (r != HAQ_OK) return r;
            HAQ_CHECK_HIP(hipEventRecord(ctx->done[k], st));
            // a later expert of this call that evicts this one may overwrite the slot after these GEMMs
            for (int k2 = k + 1; k2 < n_order; ++k2) {
                if (prev_user[k2] != k) continue;
                HAQ_CHECK_HIP(hipStreamWaitEvent(ctx->copy_stream, ctx->done[k], 0));
                if ((r = issue_copy(k2)) != HAQ_OK) return r;
                break;
            }
        }
        HAQ_CHECK_HIP(hipEventRecord(ctx->t_copy1, ctx->copy_stream));
        // Option A: the experts left to the CPU are computed here, on the host, while the GPU works through
        // what was enqueued above; their token rows come over on a third stream and their output rows go
        // back into the sorted per-pair outputs before the combination.
        if (n_cpu > 0) {
            HAQ_CHECK_HIP(hipStreamWaitEvent(ctx->aux_stream, ctx->routed, 0));
            for (int i = 0; i < n_cpu; ++i) {
                const int e = cpu_list[i], n = ctx->counts_host[e], lo = off_host[e];
                HAQ_CHECK_HIP(hipMemcpyAsync(ctx->perm_stage, perm + lo, (size_t)n * sizeof(int32_t), hipMemcpyDeviceToHost, ctx->aux_stream));
                HAQ_CHECK_HIP(hipStreamSynchronize(ctx->aux_stream));
                for (int q = 0; q < n; ++q)
                    HAQ_CHECK_HIP(hipMemcpyAsync(ctx->x_stage + (size_t)q * H, (const __half*)x_fp16 + (size_t)(ctx->perm_stage[q] >> 1) * ldx,
                                                 (size_t)H * 2, hipMemcpyDeviceToHost, ctx->aux_stream));
                HAQ_CHECK_HIP(hipStreamSynchronize(ctx->aux_stream));
                if ((r = haq_cpu_expert_ffn(cpu_of[e], ctx->x_stage, H, s_in ? ctx->s_in_host.data() : nullptr, n, ctx->y_stage, H,
                                            ctx->cpu_threads)) != HAQ_OK)
                    return r;
                HAQ_CHECK_HIP(hipMemcpyAsync(y + (size_t)lo * H, ctx->y_stage, (size_t)n * H * 2, hipMemcpyHostToDevice, ctx->aux_stream));
                HAQ_CHECK_HIP(hipStreamSynchronize(ctx->aux_stream));  // the staging rows are free again
            }
            HAQ_CHECK_HIP(hipEventRecord(ctx->aux_done, ctx->aux_stream));
            HAQ_CHECK_HIP(hipStreamWaitEvent(st, ctx->aux_done, 0));
        }
        if ((r = launch_combine(y, H, inv, gw, T, H, (__half*)out_fp16, ldo, st)) != HAQ_OK) return r;
        HAQ_CHECK_HIP(hipEventRecord(ctx->t_end, st));
        HAQ_CHECK_HIP(hipEventRecord(ctx->call_done, st));
        return HAQ_OK;
    };
    rc = enqueue();
    if (rc != HAQ_OK) {
        // Some copies may have been issued into the slots: nothing the cache says about them can be
        // trusted any more.  Forget every slot; the next call waits for whatever is still in flight.
        for (int c = 0; c < 32; ++c) {
            ctx->slot_key[c] = nullptr;
            ctx->slot_tick[c] = 0;
        }
        (void)hipEventRecord(ctx->call_done, st);
        ctx->used = true;
        return rc;
    }
    for (int c = 0; c < 32; ++c) {
        ctx->slot_key[c] = (const void*)(uintptr_t)keys_l[c];
        ctx->slot_tick[c] = ticks_l[c];
    }
    ctx->tick = tick_l;
    ctx->hits += n_hit;
    ctx->misses += n_order - n_hit;
    ctx->bytes_copied += (int64_t)(n_order - n_hit) * (int64_t)(ctx->w13_bytes + ctx->w2_bytes);
    ctx->used = true;
    ctx->timed = true;
    ctx->timed_copies = n_order - n_hit > 0;
    return HAQ_OK;
}

int32_t haq_ctx_set_offload_policy(haq_ctx* c, double t_e, double latency_cpu, double latency_gpu, const float* s_in_host,
                                   int32_t cpu_threads) {
    if (!c) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_ctx_set_offload_policy: null context");
    if (t_e < 0.0) {  // back to "always transfer"
        c->policy_on = false;
        return HAQ_OK;
    }
    int64_t nc = 0;
    const int rc = haq_offload_n_critical(t_e, latency_cpu, latency_gpu, &nc);
    if (rc != HAQ_OK) return rc;
    if (cpu_threads < 0) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_ctx_set_offload_policy: cpu_threads=%d", cpu_threads);
    // staging for the rows of one CPU expert: as many rows as the rule can ever send to the CPU, at most 1024
    const int rows = (int)(nc < 0 ? 1024 : (nc < 1 ? 1 : (nc > 1024 ? 1024 : nc)));
    if (rows > c->stage_rows) {
        if (c->aux_stream) HAQ_CHECK_HIP(hipStreamSynchronize(c->aux_stream));
        if (c->x_stage) (void)hipHostFree(c->x_stage);
        if (c->y_stage) (void)hipHostFree(c->y_stage);
        if (c->perm_stage) (void)hipHostFree(c->perm_stage);
        c->x_stage = c->y_stage = nullptr;
        c->perm_stage = nullptr;
        c->stage_rows = 0;
        HAQ_CHECK_HIP(hipHostMalloc((void**)&c->x_stage, (size_t)rows * c->H * 2, hipHostMallocDefault));
        HAQ_CHECK_HIP(hipHostMalloc((void**)&c->y_stage, (size_t)rows * c->H * 2, hipHostMallocDefault));
        HAQ_CHECK_HIP(hipHostMalloc((void**)&c->perm_stage, (size_t)rows * sizeof(int32_t), hipHostMallocDefault));
        c->stage_rows = rows;
    }
    if (!c->aux_stream) HAQ_CHECK_HIP(hipStreamCreateWithFlags(&c->aux_stream, hipStreamNonBlocking));  // default priority
    if (!c->aux_done) HAQ_CHECK_HIP(hipEventCreateWithFlags(&c->aux_done, hipEventDisableTiming));
    try {
        c->has_s_in = s_in_host != nullptr;
        if (s_in_host) c->s_in_host.assign(s_in_host, s_in_host + c->H);
    } catch (const std::bad_alloc&) {
        HAQ_FAIL(HAQ_ERR_HIP, "haq_ctx_set_offload_policy: out of host memory");
    }
    c->t_e = t_e;
    c->latency_cpu = latency_cpu;
    c->latency_gpu = latency_gpu;
    c->n_critical = nc;
    c->cpu_threads = cpu_threads;
    c->policy_on = true;
    return HAQ_OK;
}

int32_t haq_ctx_register_cpu_expert(haq_ctx* c, const void* key, const haq_cpu_expert* expert) {
    if (!c || !key) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_ctx_register_cpu_expert: null context or key");
    try {
        for (size_t i = 0; i < c->cpu_experts.size(); ++i)
            if (c->cpu_experts[i].key == key) {
                c->cpu_experts.erase(c->cpu_experts.begin() + (long)i);
                break;
            }
        if (expert) c->cpu_experts.push_back({key, expert});
    } catch (const std::bad_alloc&) {
        HAQ_FAIL(HAQ_ERR_HIP, "haq_ctx_register_cpu_expert: out of host memory");
    }
    return HAQ_OK;
}

int32_t haq_ctx_last_decisions(const haq_ctx* c, int32_t max_n, int32_t* n, int32_t* expert, int32_t* n_inputs, int32_t* decision,
                               int64_t* n_critical) {
    if (!c || !n || max_n < 0 || (max_n > 0 && (!expert || !n_inputs || !decision)))
        HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_ctx_last_decisions: null argument");
    const int k = c->n_dec < max_n ? c->n_dec : max_n;
    for (int i = 0; i < k; ++i) {
        expert[i] = c->dec_expert[i];
        n_inputs[i] = c->dec_n[i];
        decision[i] = c->dec_what[i];
    }
    *n = k;
    if (n_critical) *n_critical = c->policy_on ? c->n_critical : -2;
    return HAQ_OK;
}

int32_t haq_ctx_last_call_timing(haq_ctx* c, float* total_ms, float* copies_ms, float* after_last_copy_ms) {
    if (!c || !total_ms || !copies_ms || !after_last_copy_ms) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_ctx_last_call_timing: null argument");
    if (!c->timed) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_ctx_last_call_timing: no completed call with host-resident experts on this context");
    HAQ_CHECK_HIP(hipEventSynchronize(c->t_end));
    HAQ_CHECK_HIP(hipEventSynchronize(c->t_copy1));
    HAQ_CHECK_HIP(hipEventElapsedTime(total_ms, c->t_start, c->t_end));
    *copies_ms = 0.0f;
    *after_last_copy_ms = *total_ms;
    if (c->timed_copies) {
        HAQ_CHECK_HIP(hipEventElapsedTime(copies_ms, c->t_copy0, c->t_copy1));
        HAQ_CHECK_HIP(hipEventElapsedTime(after_last_copy_ms, c->t_copy1, c->t_end));
    }
    return HAQ_OK;
}

int32_t haq_moe_w8a8_ffn_static(const void* x_fp16, int64_t ldx, const void* logits_fp16, int64_t ldl, const float* s_in,
                                const haq_expert_desc* experts, int32_t T, int32_t H, int32_t I, int32_t E, int32_t top_k,
                                void* out_fp16, int64_t ldo, void* stream) {
    if (T < 0 || H <= 0 || I <= 0 || E <= 0) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_moe_w8a8_ffn_static: T=%d H=%d I=%d E=%d", T, H, I, E);
    const size_t need = haq_moe_workspace_bytes(T, H, I, E);
    if (need > HAQ_STATIC_SCRATCH_BYTES)
        HAQ_FAIL(HAQ_ERR_WORKSPACE,
                 "haq_moe_w8a8_ffn_static: T=%d H=%d I=%d E=%d needs %zu bytes of scratch, the built-in array holds %u; use "
                 "haq_moe_w8a8_ffn with a workspace",
                 T, H, I, E, need, (unsigned)HAQ_STATIC_SCRATCH_BYTES);
    if (experts)
        for (int e = 0; e < E && e < 32; ++e)
            if (experts[e].location != HAQ_LOC_DEVICE)
                HAQ_FAIL(HAQ_ERR_UNSUPPORTED, "haq_moe_w8a8_ffn_static: expert %d is not device resident", e);
    void* ws = nullptr;
    const int rc = static_scratch_address(&ws);
    if (rc != HAQ_OK) return rc;
    // every buffer carved from the scratch is written before it is read within the call: nothing has to be cleared
    return haq_moe_w8a8_ffn(nullptr, x_fp16, ldx, logits_fp16, ldl, s_in, experts, T, H, I, E, top_k, out_fp16, ldo, nullptr, ws,
                            HAQ_STATIC_SCRATCH_BYTES, stream);
}

size_t haq_moe_asym_workspace_bytes(int32_t T, int32_t H, int32_t I, int32_t E) {
    if (T < 0 || H <= 0 || I <= 0 || E <= 0) return 0;
    const size_t P = 2 * (size_t)T;
    return carve_moe(nullptr, T, H, I, E).bytes + 2 * (size_t)round_up((int64_t)(P > 0 ? P : 1) * 4, 256) +
           (size_t)round_up((int64_t)E * (int64_t)sizeof(ColsumTab), 256);
}

int32_t haq_moe_w8a8_ffn_asym(const void* x_fp16, int64_t ldx, const void* logits_fp16, int64_t ldl, const float* s_in,
                              const haq_expert_desc* experts, const haq_expert_colsum* colsums, int32_t T, int32_t H, int32_t I,
                              int32_t E, int32_t top_k, void* out_fp16, int64_t ldo, const haq_moe_debug_asym* dbg,
                              void* workspace, size_t workspace_bytes, void* stream) {
    if (T < 0 || H <= 0 || I <= 0 || E <= 0) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_moe_w8a8_ffn_asym: T=%d H=%d I=%d E=%d", T, H, I, E);
    if (top_k != 2) HAQ_FAIL(HAQ_ERR_UNSUPPORTED, "haq_moe_w8a8_ffn_asym: top_k=%d (only 2)", top_k);
    if (E < 2 || E > 32) HAQ_FAIL(HAQ_ERR_UNSUPPORTED, "haq_moe_w8a8_ffn_asym: E=%d outside [2, 32]", E);
    if (H % 64 != 0 || I % 64 != 0 || H > 16384 || I > 16384)
        HAQ_FAIL(HAQ_ERR_UNSUPPORTED, "haq_moe_w8a8_ffn_asym: H=%d and I=%d must be multiples of 64 (both <= 16384)", H, I);
    if (T == 0) return HAQ_OK;
    if (!x_fp16 || !logits_fp16 || !experts || !colsums || !out_fp16) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_moe_w8a8_ffn_asym: null buffer");
    if (ldx < H || ldx % 8 != 0 || ldl < E || ldo < H || ldo % 8 != 0)
        HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_moe_w8a8_ffn_asym: ldx=%lld ldl=%lld ldo=%lld", (long long)ldx, (long long)ldl, (long long)ldo);
    if (!aligned16(x_fp16) || !aligned16(out_fp16) || (s_in && !aligned16(s_in)))
        HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_moe_w8a8_ffn_asym: pointers must be 16-byte aligned");
    haq_moe_debug_asym d{};
    if (dbg) d = *dbg;
    if ((d.base.q && !aligned16(d.base.q)) || (d.base.hq && !aligned16(d.base.hq)) || (d.base.mid_fp16 && !aligned16(d.base.mid_fp16)) ||
        (d.base.y_fp16 && !aligned16(d.base.y_fp16)))
        HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_moe_w8a8_ffn_asym: debug buffers q, hq, mid_fp16 and y_fp16 must be 16-byte aligned");
    ExpertTab tab[32];
    ColsumTab cst[32];
    for (int e = 0; e < E; ++e) {
        const haq_expert_desc& x = experts[e];
        const haq_expert_colsum& c = colsums[e];
        if (!x.w13 || !x.w2 || !x.sw1 || !x.sw3 || !x.sw2 || !x.s_mid || !c.cs1 || !c.cs3 || !c.cs2)
            HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_moe_w8a8_ffn_asym: expert %d has a null pointer", e);
        if (!aligned16(x.w13) || !aligned16(x.w2) || !aligned16(x.s_mid) || !aligned16(x.sw1) || !aligned16(x.sw3) || !aligned16(x.sw2))
            HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_moe_w8a8_ffn_asym: expert %d pointers must be 16-byte aligned", e);
        if (x.location != HAQ_LOC_DEVICE) HAQ_FAIL(HAQ_ERR_UNSUPPORTED, "haq_moe_w8a8_ffn_asym: expert %d is not device resident", e);
        tab[e] = ExpertTab{x.w13, x.w2, x.sw1, x.sw3, x.sw2, x.s_mid};
        cst[e] = ColsumTab{c.cs1, c.cs3, c.cs2};
    }
    const size_t need = haq_moe_asym_workspace_bytes(T, H, I, E);
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255u))
        HAQ_FAIL(HAQ_ERR_WORKSPACE, "haq_moe_w8a8_ffn_asym: workspace of %zu bytes (256-byte aligned) needed, got %zu", need, workspace_bytes);
    hipStream_t st = (hipStream_t)stream;
    MoeWs w = carve_moe(workspace, T, H, I, E);
    const int P = 2 * T;
    Carver extra((uint8_t*)workspace + w.bytes);
    int32_t* zx_sorted = extra.take<int32_t>((size_t)P);
    int32_t* zh_ws = extra.take<int32_t>((size_t)P);
    ColsumTab* cstab = extra.take<ColsumTab>((size_t)E);
    const haq_moe_debug& b = d.base;
    int32_t* idx = b.topk_idx ? b.topk_idx : w.idx;
    float* gw = b.topk_w ? b.topk_w : w.gw;
    int32_t* counts = b.counts ? b.counts : w.counts;
    int32_t* offsets = b.offsets ? b.offsets : w.offsets;
    int32_t* perm = b.perm ? b.perm : w.perm;
    int32_t* inv = b.inv ? b.inv : w.inv;
    __half* mid = b.mid_fp16 ? (__half*)b.mid_fp16 : w.mid;
    __half* y = b.y_fp16 ? (__half*)b.y_fp16 : w.y;
    float* sh = b.sh ? b.sh : w.sh;
    int32_t* zh = d.zh ? d.zh : zh_ws;

    int rc;
    if ((rc = launch_route_permute((const __half*)logits_fp16, ldl, T, E, tab, w.tab, idx, gw, counts, offsets, perm, inv, w.blk_counts,
                                   st, cst, cstab)) != HAQ_OK)
        return rc;
    // tokens: one row of codes per (token, expert) pair in sorted order, zero point and scale with it
    AsymRowArgs qa{};
    qa.x = (const __half*)x_fp16;
    qa.ldx = ldx;
    qa.s = s_in;
    qa.gather = perm;
    qa.rows = P;
    qa.K = H;
    qa.q_cm = w.q_cm;
    qa.R = w.R;
    qa.q_rm = (uint8_t*)b.q;
    qa.ldq = H;
    qa.scale_out = w.sx_sorted;
    qa.zp_out = zx_sorted;
    qa.scale_in = b.sx;
    qa.zp_in = d.zx;
    // long batches take the pipelined quantiser (its asymmetric instantiation), short ones the row kernel
    QuantArgs pa{};
    pa.x = (const __half*)x_fp16;
    pa.ldx = ldx;
    pa.s = s_in;
    pa.T = P;
    pa.K = H;
    pa.q_rm = b.q;
    pa.ldq = H;
    pa.q_cm = w.q_cm;
    pa.R = w.R;
    pa.gather = perm;
    pa.scale = b.sx;
    pa.scale_dest = w.sx_sorted;
    pa.zp = d.zx;
    pa.zp_dest = zx_sorted;
    rc = launch_quant(pa, st);
    if (rc == HAQ_ERR_UNSUPPORTED) rc = launch_asym_quant_rows(qa, st);
    if (rc != HAQ_OK) return rc;

    // At most 64 tokens: every activated expert's weights are streamed once by the weight-streaming kernels
    // (their asymmetric instantiations); longer batches take the grouped tiled GEMM.
    const bool decode_path = decode_supported(T, H, I);
    DecodeArgs da{};
    da.q_cm = w.q_cm;
    da.sx = w.sx_sorted;
    da.R = w.R;
    da.offsets = offsets;
    da.tab = w.tab;
    da.E = E;
    da.H = H;
    da.I = I;
    da.Npad13 = round_up(2 * (int64_t)I, NPAD);
    da.Npad2 = round_up(H, NPAD);
    da.mid = mid;
    da.hq_cm = w.hq_cm;
    da.sh = sh;
    da.y = y;
    da.zx = zx_sorted;
    da.zh = zh;
    da.cstab = cstab;

    GemmArgs g1{};
    g1.A = w.q_cm;
    g1.R = w.R;
    g1.sx = w.sx_sorted;
    g1.K = H;
    g1.N = 2 * I;
    g1.Npad = round_up(2 * (int64_t)I, NPAD);
    g1.offsets = offsets;
    g1.tab = w.tab;
    g1.which = 0;
    g1.n_sel = E;
    for (int e = 0; e < E; ++e) g1.sel[e] = e;
    g1.max_rows = P;
    g1.Y = mid;
    g1.ldy = I;
    g1.zp = zx_sorted;
    g1.cstab = cstab;
    if ((rc = decode_path ? launch_decode_gate_up_asym(da, T, st) : launch_gemm(g1, EPI_SWIGLU_ASYM, st)) != HAQ_OK) return rc;

    AsymRowArgs qb{};
    qb.x = mid;
    qb.ldx = I;
    qb.tab = w.tab;
    qb.offsets = offsets;
    qb.E = E;
    qb.rows = P;
    qb.K = I;
    qb.q_cm = w.hq_cm;
    qb.R = w.R;
    qb.q_rm = (uint8_t*)b.hq;
    qb.ldq = I;
    qb.scale_out = sh;
    qb.zp_out = zh;
    QuantArgs pb{};
    pb.x = mid;
    pb.ldx = I;
    pb.tab = w.tab;
    pb.offsets = offsets;
    pb.E = E;
    pb.T = P;
    pb.K = I;
    pb.q_rm = b.hq;
    pb.ldq = I;
    pb.q_cm = w.hq_cm;
    pb.R = w.R;
    pb.scale_dest = sh;
    pb.zp_dest = zh;
    pb.n_sel = E;
    for (int e = 0; e < E; ++e) pb.sel[e] = e;
    pb.max_rows = P;
    rc = launch_quant(pb, st);
    if (rc == HAQ_ERR_UNSUPPORTED) rc = launch_asym_quant_rows(qb, st);
    if (rc != HAQ_OK) return rc;

    GemmArgs g2{};
    g2.A = w.hq_cm;
    g2.R = w.R;
    g2.sx = sh;
    g2.K = I;
    g2.N = H;
    g2.Npad = round_up(H, NPAD);
    g2.offsets = offsets;
    g2.tab = w.tab;
    g2.which = 1;
    g2.n_sel = E;
    for (int e = 0; e < E; ++e) g2.sel[e] = e;
    g2.max_rows = P;
    g2.act = HAQ_ACT_NONE;
    g2.Y = y;
    g2.ldy = H;
    g2.zp = zh;
    g2.cstab = cstab;
    if ((rc = decode_path ? launch_decode_down_asym(da, T, st) : launch_gemm(g2, EPI_LINEAR_ASYM, st)) != HAQ_OK) return rc;
    return launch_combine(y, H, inv, gw, T, H, (__half*)out_fp16, ldo, st);
}

int32_t haq_profile_enable(int32_t on) {
    if (on && !g_prof.on) {
        for (int i = 0; i <= PROF_MAX; ++i) HAQ_CHECK_HIP(hipEventCreate(&g_prof.ev[i]));
        g_prof.on = true;
        g_prof.n = -1;
    } else if (!on && g_prof.on) {
        g_prof.on = false;
        for (int i = 0; i <= PROF_MAX; ++i) {
            if (g_prof.ev[i]) (void)hipEventDestroy(g_prof.ev[i]);
            g_prof.ev[i] = nullptr;
        }
    }
    return HAQ_OK;
}

int32_t haq_profile_read(int32_t max_stages, int32_t* n_stages, const char** names, float* ms) {
    if (!n_stages || max_stages < 0 || (max_stages > 0 && (!names || !ms))) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_profile_read: null buffer");
    if (!g_prof.on || g_prof.n < 0) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_profile_read: no profiled call (haq_profile_enable(1), then a block-level call)");
    const int n = g_prof.n < max_stages ? g_prof.n : max_stages;
    HAQ_CHECK_HIP(hipEventSynchronize(g_prof.ev[g_prof.n]));
    for (int i = 0; i < n; ++i) {
        names[i] = g_prof.name[i];
        HAQ_CHECK_HIP(hipEventElapsedTime(&ms[i], g_prof.ev[i], g_prof.ev[i + 1]));
    }
    *n_stages = n;
    return HAQ_OK;
}

int32_t haq_lru_plan(int32_t n_slots, uint64_t* slot_keys, uint64_t* slot_ticks, uint64_t* tick, const uint64_t* keys,
                     int32_t n_keys, int32_t* slot_of, int32_t* hit, int32_t* prev_user) {
    if (n_slots < 1 || n_slots > 32 || n_keys < 0 || n_keys > 32) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_lru_plan: n_slots=%d n_keys=%d (both at most 32)", n_slots, n_keys);
    if (!slot_keys || !slot_ticks || !tick || (n_keys > 0 && (!keys || !slot_of || !hit || !prev_user)))
        HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_lru_plan: null buffer");
    for (int k = 0; k < n_keys; ++k) {
        if (keys[k] == 0) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_lru_plan: key %d is 0 (0 marks an empty slot)", k);
        for (int j = 0; j < k; ++j)
            if (keys[j] == keys[k]) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_lru_plan: keys %d and %d are equal", j, k);
    }
    int user[32];  // request of this call that last took each slot
    for (int c = 0; c < n_slots; ++c) user[c] = -1;
    for (int k = 0; k < n_keys; ++k) {
        int sl = -1;
        for (int c = 0; c < n_slots && sl < 0; ++c)
            if (slot_keys[c] == keys[k]) sl = c;
        hit[k] = sl >= 0;
        for (int c = 0; c < n_slots && sl < 0; ++c)  // miss: a free slot ...
            if (slot_keys[c] == 0) sl = c;
        if (sl < 0) {                                // ... else the one used longest ago
            sl = 0;
            for (int c = 1; c < n_slots; ++c)
                if (slot_ticks[c] < slot_ticks[sl]) sl = c;
        }
        slot_of[k] = sl;
        prev_user[k] = hit[k] ? -1 : user[sl];
        user[sl] = k;
        slot_keys[sl] = keys[k];
        slot_ticks[sl] = ++*tick;
    }
    return HAQ_OK;
}

}  // extern "C"
