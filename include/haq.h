/*
 * haq.h - C ABI of the MI355X (gfx950) library for the smoothed W8A8 expert FFN
 * of HAQ (arXiv 2508.07329, Section III.B).
 *
 * Operator (Section III.B.1, Eq. 1):  Y = Q(W s) Q(s^-1 X).  Here activations
 * are X [T x K] (one token per row) and weights W [K x N] (input channel major),
 * the transpose of the paper's W X.  Quantisation scales sit on the outer
 * dimensions only (Section III.B.1, last paragraph): one scale per token for the
 * activations, one per output channel for the weights.  Both operands are
 * symmetric int8 in [-127, 127].
 *
 * Conventions for every entry point
 *  - Every pointer is a DEVICE pointer unless its comment says "host".
 *  - Buffers are owned by the caller.  Work is enqueued on `stream` (a
 *    hipStream_t passed as void*; NULL = the default stream) and the call
 *    returns without synchronising; buffers must stay alive until the stream
 *    has drained.  The library allocates nothing on these calls: scratch comes
 *    from the caller's workspace, sized by the matching *_workspace_bytes query.
 *  - Arguments are validated on the host before any HIP call.  Return value:
 *    HAQ_OK or a negative HAQ_ERR_*; haq_last_error() gives a thread-local text.
 *  - Device pointers must be 16-byte aligned; leading dimensions are in
 *    elements; the contracted dimension K must be a multiple of 16 for the dense
 *    calls (the packed layouts round it up to whole 64-byte k-steps and keep the
 *    pad of the weights at zero) and of 64 for the expert FFN and the offline
 *    search / Hessian tools.
 *  - Arithmetic is IEEE binary32 with one rounding per operation, int32
 *    accumulation, round-half-to-even; results do not depend on launch shape.
 */
#ifndef HAQ_H
#define HAQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HAQ_OK 0
#define HAQ_ERR_INVALID_ARG (-1) /* null / negative / misaligned argument */
#define HAQ_ERR_UNSUPPORTED (-2) /* shape or enum the kernels do not cover */
#define HAQ_ERR_WORKSPACE (-3)   /* workspace missing or too small */
#define HAQ_ERR_HIP (-4)         /* a HIP call failed */

#define HAQ_ACT_NONE 0
#define HAQ_ACT_RELU 1

#define HAQ_LOC_DEVICE 0      /* expert weights live in HBM */
#define HAQ_LOC_HOST_PINNED 1 /* expert weights live in pinned host memory and are streamed in */

int32_t haq_version(void);
const char* haq_last_error(void); /* host string, valid until the thread's next failing call */

/* ------------------------------------------------------------------------
 * Activation operand of Eq. 1, Q(s^-1 X), scale on the token dimension.
 *   y = x / s_k (binary32 divide);  scale_t = max_k |y| / 127;
 *   q = clamp(rne(y / scale_t), -127, 127).   A zero row gives scale 0, codes 0.
 * x_fp16 [T x K] row-major (row stride ldx), s [K] (> 0, finite) or NULL for all
 * ones.  Outputs q int8 [T x K] (row stride ldq) and row_scale [T].
 * T >= 0 (T == 0 is a no-op), K % 16 == 0, K <= 65536.
 */
int32_t haq_smooth_quant_act(const void* x_fp16, int64_t ldx, const float* s, int32_t T, int32_t K,
                             int8_t* q, int64_t ldq, float* row_scale, void* stream);

/* ------------------------------------------------------------------------
 * Offline side of Eq. 1 / Algorithm 1 step 1 for a fixed exponent (the values
 * the hot path consumes are produced once, outside the timed path).
 *
 * haq_channel_absmax_f16: ax[k] = max(ax[k], max_t |X[t][k]|)  - the per-channel
 *   activation magnitude s_X of Eq. 3.  Folds into ax (caller zeroes it first).
 * haq_weight_row_absmax: aw[k] = max(aw[k], max_n |W[k][n]|), W fp32 [K x N].
 * haq_smoothing_vector (HOST pointers): s_k = ax_k^alpha / aw_k^(1-alpha) in
 *   binary64, rounded to binary32, clamped to [1e-5, 1e5]; 1 where ax_k or aw_k
 *   is 0.  aw == NULL gives Eq. 3's activation-only form s_k = ax_k^alpha.
 * haq_quant_weight: Q(W s) with one scale per output channel.  W fp32 [K x N],
 *   s [K] or NULL; outputs wq int8 [K x N] (canonical layout) and w_scale [N].
 */
int32_t haq_channel_absmax_f16(const void* x_fp16, int64_t ldx, int32_t T, int32_t K, float* ax, void* stream);
int32_t haq_weight_row_absmax(const float* w, int32_t K, int32_t N, float* aw, void* stream);
int32_t haq_smoothing_vector(const float* ax_host, const float* aw_host, int32_t K, double alpha, float* s_host);
int32_t haq_quant_weight(const float* w, const float* s, int32_t K, int32_t N, int8_t* wq, float* w_scale,
                         void* stream);

/* ------------------------------------------------------------------------
 * Weight layout for the MFMA kernels (offline, Algorithm 1 step 3 keeps int8
 * weights on the GPU in the form its kernels consume).
 *
 * Packed layout of a [K x N] int8 matrix: [Kpad/16][Npad][16] - for each group of
 * 16 consecutive input channels, all output channels side by side, each with its
 * 16 bytes.  Npad = N rounded up to a multiple of 256, Kpad = K rounded up to a
 * multiple of 64; padding is zero.  K % 16 == 0 (haq_pack_gate_up: K % 64 == 0).
 * haq_packed_bytes(K, N) gives the size.  haq_pack_weight converts the canonical
 * row-major [K x N] matrix.  haq_pack_gate_up interleaves the gate (w1) and up
 * (w3) matrices of a SwiGLU expert, both [K x N], into one packed [K x 2N]
 * matrix whose output channels alternate in blocks of 32: 32 of w1, the same 32
 * of w3, and so on (N % 32 == 0).
 */
size_t haq_packed_bytes(int32_t K, int32_t N);
int32_t haq_pack_weight(const int8_t* wq, int32_t K, int32_t N, int8_t* packed, void* stream);
int32_t haq_pack_gate_up(const int8_t* w1q, const int8_t* w3q, int32_t K, int32_t N, int8_t* packed, void* stream);

/* ------------------------------------------------------------------------
 * One smoothed W8A8 linear layer (Eq. 1 evaluated at run time):
 *   q, sx = Q(s^-1 X);  acc = q Wq (int32);  r = (float(acc) * sx_t) * sw_n;
 *   act;  Y = fp16(r).
 * x_fp16 [T x K], s [K] or NULL, w_packed from haq_pack_weight, w_scale [N].
 * Y fp16 [T x N] (row stride ldy).  Optional outputs (NULL to skip): acc_dbg
 * int32 [T x N] dense, q_dbg int8 [T x K] dense, sx_dbg [T].
 * T >= 0, K % 16 == 0, N % 16 == 0.
 */
size_t haq_linear_workspace_bytes(int32_t T, int32_t K, int32_t N);

/* The two stages of haq_w8a8_linear as calls of their own (same kernels, same
 * results), for callers that keep activations in int8 between layers or time the
 * stages separately.  The packed activation layout is that of the weights:
 * [Kpad/16][R][16] with R = haq_packed_act_rows(T) rows (T rounded up to 16, plus
 * one 256-row tile of slack that the GEMM may read but never uses) and Kpad = K
 * rounded up to 64 (chunks past K are never written; the weights are zero there);
 * its size is haq_packed_act_bytes(T, K) = Kpad * R.
 * haq_quant_act_packed: Q(s^-1 X) as in haq_smooth_quant_act, codes written in
 *   the packed layout.  haq_gemm_w8a8_packed: int8 GEMM + dequantise + activation
 *   on such codes; row_scale [T], y fp16 [T x N]; acc_dbg optional.            */
int64_t haq_packed_act_rows(int32_t T);
size_t haq_packed_act_bytes(int32_t T, int32_t K);
int32_t haq_quant_act_packed(const void* x_fp16, int64_t ldx, const float* s, int32_t T, int32_t K,
                             int8_t* q_packed, float* row_scale, void* stream);
int32_t haq_gemm_w8a8_packed(const int8_t* q_packed, const float* row_scale, const int8_t* w_packed,
                             const float* w_scale, int32_t T, int32_t K, int32_t N, int32_t act, void* y_fp16,
                             int64_t ldy, int32_t* acc_dbg, void* stream);
int32_t haq_w8a8_linear(const void* x_fp16, int64_t ldx, const float* s, const int8_t* w_packed,
                        const float* w_scale, int32_t T, int32_t K, int32_t N, int32_t act, void* y_fp16,
                        int64_t ldy, int32_t* acc_dbg, int8_t* q_dbg, float* sx_dbg, void* workspace,
                        size_t workspace_bytes, void* stream);

/* The same layer on weights in the canonical layout of Eq. 1's weight operand as the offline
 * quantiser emits it: wq_kn int8 [K x N] row-major (input channel major).  The call packs the
 * matrix into its workspace first (one extra pass over the weights per call: the run-time
 * path proper takes pre-packed weights), then runs haq_w8a8_linear; same results.            */
size_t haq_linear_kn_workspace_bytes(int32_t T, int32_t K, int32_t N);
int32_t haq_w8a8_linear_kn(const void* x_fp16, int64_t ldx, const float* s, const int8_t* wq_kn, const float* w_scale,
                           int32_t T, int32_t K, int32_t N, int32_t act, void* y_fp16, int64_t ldy, void* workspace,
                           size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------
 * The linear layer with ASYMMETRIC activation codes (the quantisation mode the
 * paper's experimental setup, Section IV.A, names as its default); the weight
 * operand stays symmetric per output channel.  Per token t, with y = x / s:
 *   mn = min(0, min_k y), mx = max(0, max_k y), scale_t = (mx - mn) / 255,
 *   zp_t = clamp(rne(-mn / scale_t), 0, 255), q = clamp(rne(y / scale_t) + zp_t, 0, 255)
 * (binary32, IEEE division, round half to even; a row with mx = mn gives scale 0,
 * zp 0, q 0), acc[t][n] = sum_k (q[t][k] - zp_t) Wq[k][n] (int32, exact), then the
 * same epilogue as haq_w8a8_linear with scale_t in place of sx_t.
 * The packed activation operand holds q - 128 and the GEMM epilogue adds
 * (128 - zp_t) * colsum[n] to the accumulator, colsum[n] = sum_k Wq[k][n] from
 * haq_weight_colsum (offline, int32 [N], device).
 * Optional outputs: acc_dbg int32 [T x N] (corrected accumulators), q_dbg uint8
 * [T x K] dense codes, sx_dbg [T], zp_dbg int32 [T].  K % 16 == 0, K <= 16384,
 * N % 16 == 0.                                                                */
int32_t haq_weight_colsum(const int8_t* wq, int32_t K, int32_t N, int32_t* colsum, void* stream);
size_t haq_linear_asym_workspace_bytes(int32_t T, int32_t K, int32_t N);
int32_t haq_w8a8_linear_asym(const void* x_fp16, int64_t ldx, const float* s, const int8_t* w_packed,
                             const float* w_scale, const int32_t* w_colsum, int32_t T, int32_t K, int32_t N,
                             int32_t act, void* y_fp16, int64_t ldy, int32_t* acc_dbg, uint8_t* q_dbg,
                             float* sx_dbg, int32_t* zp_dbg, void* workspace, size_t workspace_bytes,
                             void* stream);

/* ------------------------------------------------------------------------
 * Two chained smoothed W8A8 linears (a dense FFN block, e.g. OPT: fc1, ReLU, fc2):
 *   H = fp16(act(deq(Q(s1^-1 X) W1q)));   Y = fp16(deq(Q(s2^-1 H) W2q)).
 * Results are identical to two haq_w8a8_linear calls; the block call keeps H and
 * both sets of int8 codes in one workspace.  X [T x K], W1 packed
 * [K x F], W2 packed [F x N]; h_dbg optional fp16 [T x F] dense copy of H.
 * K % 16 == 0, F % 16 == 0, N % 16 == 0.                                     */
size_t haq_ffn_workspace_bytes(int32_t T, int32_t K, int32_t F, int32_t N);
int32_t haq_w8a8_ffn(const void* x_fp16, int64_t ldx, const float* s1, const int8_t* w1_packed, const float* w1_scale,
                     int32_t act, const float* s2, const int8_t* w2_packed, const float* w2_scale, int32_t T,
                     int32_t K, int32_t F, int32_t N, void* y_fp16, int64_t ldy, void* h_dbg_fp16, void* workspace,
                     size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------
 * Adaptive activation smoothing (Algorithm 1 step 1; Eq. 3): grid search of the
 * exponent e in [0, 1] of the smoothing vector for one linear layer, on
 * calibration activations X (fp16 [T x K], device) and the layer's weight W
 * (fp32 [K x N], device, input-channel major).
 *
 * For every exponent of the grid, in order:
 *   s = ax^e  (ax_k = max_t |X_tk|; Eq. 3 -- with use_weight != 0 the balanced
 *   form ax^e / aw^(1-e), aw_k = max_n |W_kn|; both as haq_smoothing_vector
 *   evaluates them), the weight is folded and quantised, Q(W s), the calibration
 *   activations go through the quantised layer exactly as haq_w8a8_linear runs
 *   it, and the loss is the mean over all T*N outputs of (Y - Yref)^2, where
 *   Yref = X W in binary64 (the norm of Eq. 1 read as a mean squared error).
 * A candidate replaces the incumbent only if its loss is strictly smaller: the
 * first of equal minima wins.
 *
 * exponents: host [n_e], 1 <= n_e <= 256, each in [0, 1].  Outputs: losses host
 * [n_e] (binary64), *best host (index into the grid), s_best device [K].
 * The call synchronises the stream (the decision is taken on the host) and is
 * meant for the offline quantiser, not for a serving loop.  K % 64 == 0,
 * K < 65536, N % 16 == 0.  Workspace (256-byte aligned, device) of
 * haq_smoothing_search_workspace_bytes(T, K, N, n_e) bytes: it holds Yref
 * (8 T N bytes), one candidate's weights and outputs, and the grid's vectors.
 *
 * The two building blocks are callable on their own:
 * haq_reference_matmul_f64: Yref [T x N] binary64 (device) = X W, one binary64
 *   accumulator per output, input channels in ascending order.
 * haq_quant_loss_f64: *loss (device) = mean (Y - Yref)^2 for Y fp16 [T x N] (row
 *   stride ldy); row sums run over the columns in order, then the rows in
 *   order, so the value does not depend on the launch shape; row_scratch is T
 *   doubles of device memory.
 */
size_t haq_smoothing_search_workspace_bytes(int32_t T, int32_t K, int32_t N, int32_t n_e);
int32_t haq_reference_matmul_f64(const void* x_fp16, int64_t ldx, const float* w, int32_t T, int32_t K, int32_t N,
                                 double* yref, void* stream);
int32_t haq_quant_loss_f64(const void* y_fp16, int64_t ldy, const double* yref, int32_t T, int32_t N, double* row_scratch,
                           double* loss, void* stream);
int32_t haq_smoothing_search(const void* x_fp16, int64_t ldx, const float* w, int32_t T, int32_t K, int32_t N,
                             const double* exponents, int32_t n_e, int32_t use_weight, double* losses, int32_t* best,
                             float* s_best, void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------
 * Hessian-aware weight quantisation (Section III.B.2, Eq. 4-6; Algorithm 1 step
 * 2), offline: Q(W s) with the rounding error of every input channel pushed onto
 * the channels not yet quantised, so that the layer's output on the calibration
 * activations, not the weight itself, is preserved (Eq. 4).
 *
 *   H = 2 Xs^T Xs over the T calibration rows, Xs = X / s (binary32 division as
 *   on the activation path; s NULL = ones); a channel with H_jj = 0 gets H_jj =
 *   1; percdamp * mean(diag H) is added to the diagonal.
 *   U = upper triangular with H^-1 = U^T U: row i of U is, up to U_ii, row i of
 *   the inverse Hessian of the channels i, i+1, ... (what Eq. 5-6 need at step
 *   i; the Cholesky reformulation the paper mentions).
 *   Grid: scale_n = max_k |s_k W_kn| / 127 as haq_quant_weight.  Input channels
 *   i = 0 .. K-1 in order: code = clamp(rne(w_in / scale_n)), e_n = (w_in -
 *   code scale_n) / U_ii, and w_jn -= e_n U_ij for every j > i (Eq. 6).
 * All arithmetic is binary64 with one fused multiply-add per term and sums in
 * ascending order of the token / eliminated column / quantised channel, so the
 * result is defined bit for bit.
 *
 * x_fp16 [T x K] device, w fp32 [K x N] device, s [K] device or NULL.  Outputs
 * wq int8 [K x N] dense and w_scale [N] (device), to be packed with
 * haq_pack_weight.  K < 65536.  The calls synchronise the stream once (the
 * factorisation reports a non-positive pivot as HAQ_ERR_INVALID_ARG).
 * Workspace: haq_hessian_quant_workspace_bytes(K, N) bytes, 256-byte aligned
 * (three K x K and one K x N binary64 matrices).
 * Building blocks: haq_hessian_f64 (H [K x K] device), and
 * haq_inverse_cholesky_upper_f64 (U [K x K] device from H; U may alias H).     */
size_t haq_hessian_quant_workspace_bytes(int32_t K, int32_t N);
size_t haq_inverse_cholesky_workspace_bytes(int32_t K);
int32_t haq_hessian_f64(const void* x_fp16, int64_t ldx, const float* s, int32_t T, int32_t K, double percdamp,
                        double* H, void* stream);
int32_t haq_inverse_cholesky_upper_f64(const double* H, int32_t K, double* U, void* workspace,
                                       size_t workspace_bytes, void* stream);
int32_t haq_hessian_quant_weight(const void* x_fp16, int64_t ldx, int32_t T, const float* w, const float* s,
                                 int32_t K, int32_t N, double percdamp, int8_t* wq, float* w_scale,
                                 void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------
 * Algorithm 1 for one linear layer, on this device: step 1 (haq_smoothing_search:
 * the smoothing vector s by grid search on the calibration activations), step 2
 * (haq_hessian_quant_weight on the weight folded with that s), step 3 (the GPU
 * keeps the int8 codes: pack them with haq_pack_weight).  Outputs: s [K] device,
 * wq int8 [K x N] device, w_scale [N] device, losses [n_e] host, *best host.
 * Same constraints as the two calls it chains; synchronises the stream.
 * losses and best must not be NULL.                                          */
size_t haq_quantize_layer_workspace_bytes(int32_t T, int32_t K, int32_t N, int32_t n_e);
int32_t haq_quantize_layer(const void* x_fp16, int64_t ldx, int32_t T, const float* w, int32_t K, int32_t N,
                           const double* exponents, int32_t n_e, int32_t use_weight, double percdamp, float* s,
                           int8_t* wq, float* w_scale, double* losses, int32_t* best, void* workspace,
                           size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------
 * Top-2 routed SwiGLU expert FFN with W8A8 experts: Eq. 1 (Section III.B.1)
 * applied to every linear of an expert, experts kept in int8 on the GPU (Section
 * III.B.3), "the gating network selects" which experts a token visits (Section
 * III.C.1b), two per layer (an activation path holds 2 experts per layer: Section
 * III.C.2, stage 1 of the proposed strategy), and host-resident experts move to
 * the GPU in their low-bit form through an expert cache (Section III.C.1c).  The
 * paper names neither the gate normalisation nor the expert's activation; they
 * are those of the Mixtral-style layers its experiments run on.
 *
 * Per token t: top-2 experts by router logit (lowest index wins ties); gate
 * weights = softmax over all E logits, renormalised over the two.  The token is
 * quantised once with s_in (shared by the gate/up projections of all experts,
 * which all see the same X).  Per (token, expert) pair:
 *   g = deq(q w1), u = deq(q w3), h = fp16(silu(g) * u);
 *   hq, sh = Q(s_mid^-1 h);  y = fp16(deq(hq w2));
 * out[t] = fp16(g0 * y0 + g1 * y1).  silu(g) = g / (1 + e^-g) with e^t evaluated
 * by a fixed binary32 sequence (two-part ln 2 reduction, degree-7 Horner with
 * FMAs), so that codes and outputs are reproducible bit for bit.
 *
 * Pairs are processed grouped by expert: pair id r = 2t + k, sorted by
 * (expert, r) (stable), which is what the debug arrays expose.
 */
typedef struct haq_expert_desc {
    const int8_t* w13;  /* packed gate/up [H x 2I] from haq_pack_gate_up; device, or pinned HOST if location says so */
    const int8_t* w2;   /* packed down [I x H] from haq_pack_weight; same location as w13 */
    const float* sw1;   /* [I] device */
    const float* sw3;   /* [I] device */
    const float* sw2;   /* [H] device */
    const float* s_mid; /* [I] device, smoothing vector of the down projection */
    int32_t location;   /* HAQ_LOC_DEVICE or HAQ_LOC_HOST_PINNED */
    int32_t reserved;
} haq_expert_desc;

typedef struct haq_moe_debug { /* every field optional (NULL to skip); all device pointers */
    int32_t* topk_idx; /* [T x 2] */
    float* topk_w;     /* [T x 2] */
    int32_t* counts;   /* [E] */
    int32_t* offsets;  /* [E + 1] */
    int32_t* perm;     /* [2T] pair id at each sorted position */
    int32_t* inv;      /* [2T] sorted position of each pair id */
    int8_t* q;         /* [T x H] dense, codes of the tokens */
    float* sx;         /* [T] */
    void* mid_fp16;    /* [2T x I] dense, sorted order */
    int8_t* hq;        /* [2T x I] dense, sorted order */
    float* sh;         /* [2T] sorted order */
    void* y_fp16;      /* [2T x H] dense, sorted order */
} haq_moe_debug;

/* Context for layers with host-resident experts: owns a side stream, events and
 * `n_slots` HBM slots, each large enough for one expert of the given geometry.
 * Creating and destroying it allocates / frees; the FFN call does not.
 *
 * The slots are the GPU expert cache of Section III.C.1(c): a host-resident
 * expert that a call activates is first looked up in the slots (a hit costs no
 * transfer); on a miss it is copied into a free slot, else into the least
 * recently used one.  The cache persists across calls on the same context and
 * is keyed by the host address of the expert's gate/up matrix: after changing
 * the bytes behind an address call haq_ctx_cache_invalidate.  Calls that share
 * a context must not overlap.
 * haq_ctx_cache_stats: totals since creation (any output may be NULL);
 * slot_keys [n_slots] receives the address cached in each slot (NULL: empty). */
typedef struct haq_ctx haq_ctx;
int32_t haq_ctx_create(int32_t H, int32_t I, int32_t n_slots, haq_ctx** out_host);
int32_t haq_ctx_destroy(haq_ctx* ctx);
int32_t haq_ctx_cache_stats(const haq_ctx* ctx, int64_t* hits, int64_t* misses, int64_t* bytes_copied,
                            const void** slot_keys);
int32_t haq_ctx_cache_invalidate(haq_ctx* ctx);
/* Timeline of the context's last call that had host-resident experts, from events the call
 * records on its two streams (waits for that call): *total_ms from its first launch to the end
 * of the combination; *copies_ms from the first expert copy being issued to the last one having
 * landed (0 when every activated expert was cached); *after_last_copy_ms from there to the end
 * of the call, i.e. the part of the call that no copy overlaps (= *total_ms without copies).   */
int32_t haq_ctx_last_call_timing(haq_ctx* ctx, float* total_ms, float* copies_ms, float* after_last_copy_ms);

/* ------------------------------------------------------------------------
 * Host-side planning of the offload runtime (no device work).
 *
 * haq_offload_n_critical (Eq. 7-8): computing a host-resident expert on the CPU
 * costs T_CPU = n * latency_cpu; transferring it costs T_sum = t_e + n *
 * latency_gpu.  *n_critical = the largest batch n for which the CPU is not
 * slower; the expert is worth transferring when n_inputs > *n_critical.
 * *n_critical = -1 when latency_cpu <= latency_gpu (never transfer).
 * haq_moe_w8a8_ffn applies the rule once a context has been given the three
 * figures (haq_ctx_set_offload_policy below); without them it always transfers.
 *
 * haq_select_experts (Algorithm 2): which experts of every layer to keep
 * resident.  Layer l owns the paths path_offsets[l] .. path_offsets[l+1]-1;
 * path p lists path_len experts of that layer (path_experts [n_paths x
 * path_len], the layer's slice of one activation path) with frequency
 * path_freq[p]; expert_freq is [num_layers x experts_per_layer].  Stage I
 * takes the experts of the layer's paths from the most frequent path down
 * until top_k (>= 1) are selected; stage II adds the layer's most frequently
 * activated experts until top_k + supplement_k are.  Equal frequencies keep
 * input (index) order.  selected is [num_layers x (top_k + supplement_k)] in
 * order of selection, padded with -1; n_selected [num_layers].  All host.    */
int32_t haq_offload_n_critical(double t_e, double latency_cpu, double latency_gpu, int64_t* n_critical);
/* haq_lru_plan (Section III.C.1c, cache fill and LRU replacement): one call's look-ups in an
 * expert cache of n_slots slots, on the caller's copy of the cache state.  slot_keys [n_slots]
 * (in/out) is the key held by each slot, 0 for an empty one; slot_ticks [n_slots] (in/out) the
 * time each slot was last used; *tick (in/out) the clock.  keys [n_keys] are the requests in
 * order (non-zero, distinct).  For request k: hit[k] = 1 if a slot holds the key (no transfer);
 * else it takes the first empty slot, else the least recently used one.  slot_of[k] is its slot;
 * prev_user[k] is the earlier request of this same batch whose slot it takes over, or -1.
 * haq_moe_w8a8_ffn plans with this function and takes the new state over only after every copy
 * and launch of the call has been enqueued.  All host; n_slots, n_keys <= 32.                */
int32_t haq_lru_plan(int32_t n_slots, uint64_t* slot_keys, uint64_t* slot_ticks, uint64_t* tick, const uint64_t* keys,
                     int32_t n_keys, int32_t* slot_of, int32_t* hit, int32_t* prev_user);
int32_t haq_select_experts(int32_t num_layers, int32_t experts_per_layer, int32_t top_k, int32_t supplement_k,
                           const int32_t* path_offsets, const int32_t* path_experts, int32_t path_len,
                           const double* path_freq, const double* expert_freq, int32_t* selected,
                           int32_t* n_selected);

/* ------------------------------------------------------------------------
 * The CPU side of the heterogeneous deployment (Section III.B.3; Algorithm 1
 * step 3, CPU branch; Section III.C.1a, option A).  All pointers HOST.
 *
 * haq_cpu_expert_create dequantises an expert once, at load time, into a
 * floating-point copy that stays cached in host memory: Wf = float(code) *
 * scale of the output channel, binary32.  Inputs are the canonical row-major
 * int8 matrices of haq_quant_weight (w1q, w3q [H x I], w2q [I x H]), their
 * scales and the expert's s_mid [I]; the copy takes 12 H I bytes.  With
 * keep_codes != 0 the handle keeps the int8 codes and the scales instead (3 H I
 * bytes) and forms the same Wf = float(code) * scale inside the inner loop:
 * identical results, a quarter of the host memory traffic per token row.
 * haq_cpu_expert_ffn computes the expert for n_rows token rows in floating
 * point on that copy (the activations are not quantised on this side):
 *   xs = x / s_in;  g = xs W1f, u = xs W3f;  h = fp16(silu(g) * u);
 *   y = fp16((h / s_mid) W2f)
 * with one binary32 accumulator per inner product, input channels in ascending
 * order, one fused multiply-add per term (silu and e^t as in haq_moe_w8a8_ffn),
 * so the result does not depend on n_threads (0 = all hardware threads, at most
 * 64; threads split the output channels).  x fp16 [n_rows x H] (row stride ldx),
 * s_in [H] or NULL, y fp16 [n_rows x H] (row stride ldy).
 *
 * haq_ctx_set_offload_policy gives a context the cost model of Eq. 7-8 (t_e,
 * latency_cpu, latency_gpu in one unit of time, calibrated by the caller) and a
 * host copy of s_in (NULL if the layer has none); haq_ctx_register_cpu_expert
 * tells it which host-resident expert (key = the w13 pointer its descriptor
 * carries) has a CPU copy (expert = NULL removes the entry).  From then on
 * haq_moe_w8a8_ffn decides per activated host-resident expert (Section
 * III.C.1b): held by the GPU cache -> computed there; else n_inputs >
 * n_critical -> transferred (through the cache, as before); else -> computed by
 * haq_cpu_expert_ffn on the host while the GPU works on the other experts, and
 * only its output rows are copied to the GPU.  Experts without a CPU copy, or
 * with more rows than the staging area (min(n_critical, 1024) rows), are
 * transferred.  t_e < 0 switches the rule off again (always transfer, the
 * default).  The calls allocate (pinned staging, a stream): set-up, not serving.
 * haq_ctx_last_decisions: for the last call, per activated host-resident expert
 * in expert order: its index, its batch n_inputs and the decision; *n_critical
 * (optional) receives the break-even batch in force (-1: the CPU is never
 * slower; -2: no cost model set).                                            */
#define HAQ_DECISION_GPU_CACHED 0
#define HAQ_DECISION_TRANSFER 1
#define HAQ_DECISION_CPU 2
typedef struct haq_cpu_expert haq_cpu_expert;
int32_t haq_cpu_expert_create(const int8_t* w1q, const int8_t* w3q, const int8_t* w2q, const float* sw1, const float* sw3,
                              const float* sw2, const float* s_mid, int32_t H, int32_t I, int32_t keep_codes,
                              haq_cpu_expert** out);
int32_t haq_cpu_expert_destroy(haq_cpu_expert* expert);
int32_t haq_cpu_expert_ffn(const haq_cpu_expert* expert, const void* x_fp16, int64_t ldx, const float* s_in, int32_t n_rows,
                           void* y_fp16, int64_t ldy, int32_t n_threads);
int32_t haq_ctx_set_offload_policy(haq_ctx* ctx, double t_e, double latency_cpu, double latency_gpu, const float* s_in_host,
                                   int32_t cpu_threads);
int32_t haq_ctx_register_cpu_expert(haq_ctx* ctx, const void* key, const haq_cpu_expert* expert);
int32_t haq_ctx_last_decisions(const haq_ctx* ctx, int32_t max_n, int32_t* n, int32_t* expert, int32_t* n_inputs,
                               int32_t* decision, int64_t* n_critical);

size_t haq_moe_workspace_bytes(int32_t T, int32_t H, int32_t I, int32_t E);

/* experts: HOST array of E descriptors (read during the call only).  ctx may be
 * NULL when every expert is device resident.  2 <= E <= 32, top_k must be 2,
 * H % 64 == 0, I % 64 == 0.  Host-resident experts that the call activates and
 * the context's cache does not hold are copied into its slots with
 * hipMemcpyAsync on its side stream while resident experts compute; results
 * are identical to the all-resident call.  With host-resident experts the call
 * is NOT asynchronous: it waits on the host for the routing histogram (which
 * experts are activated decides what is copied; one small device-to-host copy),
 * and, when the offload policy sends experts to the CPU, for their computation;
 * everything else of the call is enqueued as usual.
 * Launch shapes (same results on every path): more than 64 tokens or any
 * host-resident expert -> grouped tiled GEMMs (a streamed expert with at most 64
 * rows runs on the weight-streaming kernels when H and I allow); up to 64 tokens, all experts
 * resident, H % 128 == 0 and I % 256 == 0 -> weight-streaming kernels (five
 * launches); one or two tokens with H <= 8192, I <= 16384 and none of q, sx, hq,
 * sh asked for in dbg -> three launches (those four stay on chip on that path). */
int32_t haq_moe_w8a8_ffn(haq_ctx* ctx, const void* x_fp16, int64_t ldx, const void* logits_fp16, int64_t ldl,
                         const float* s_in, const haq_expert_desc* experts_host, int32_t T, int32_t H, int32_t I,
                         int32_t E, int32_t top_k, void* out_fp16, int64_t ldo, const haq_moe_debug* dbg_host,
                         void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------
 * The routed expert FFN with ASYMMETRIC activation codes (Section IV.A: asymmetric
 * quantisation is the default of the paper's experiments), for the tokens and for
 * the requantised intermediate; expert weights stay symmetric per output channel.
 * Routing, grouping by expert and the combination are those of haq_moe_w8a8_ffn
 * (top-2 softmax gating; pairs sorted by (expert, pair id)).  Per token, with
 * y = x / s_in: scale, zero point zx and codes q in [0, 255] exactly as in
 * haq_w8a8_linear_asym.  Per (token, expert) pair:
 *   g = deq(sum_k (q - zx) w1), u = deq(sum_k (q - zx) w3), h = fp16(silu(g) * u);
 *   hq, sh, zh = asymmetric codes of h / s_mid;  y = fp16(deq(sum_j (hq - zh) w2));
 * out[t] = fp16(g0 * y0 + g1 * y1).  The packed operands hold code - 128 and the
 * GEMM epilogues add (128 - zero point) * column sum of the expert's weight codes:
 * colsums_host [E] (HOST array) points at int32 device vectors cs1 [I], cs3 [I]
 * (of the w1 and w3 codes) and cs2 [H] (of the w2 codes) from haq_weight_colsum.
 * Every expert must be device resident.  More than 64 tokens -> grouped tiled
 * GEMMs; up to 64 tokens with H % 128 == 0 and I % 256 == 0 -> the
 * weight-streaming kernels for the two projections.  2 <= E <= 32, top_k = 2, H % 64 == 0, I % 64 == 0, both <= 16384.
 * dbg: the fields of haq_moe_debug (q and hq receive the uint8 codes) plus the zero
 * points zx [T] and zh [2T] (sorted order); every field optional.               */
typedef struct haq_expert_colsum {
    const int32_t* cs1; /* [I] device */
    const int32_t* cs3; /* [I] device */
    const int32_t* cs2; /* [H] device */
} haq_expert_colsum;
typedef struct haq_moe_debug_asym {
    haq_moe_debug base;
    int32_t* zx; /* [T] */
    int32_t* zh; /* [2T] sorted order */
} haq_moe_debug_asym;
size_t haq_moe_asym_workspace_bytes(int32_t T, int32_t H, int32_t I, int32_t E);
int32_t haq_moe_w8a8_ffn_asym(const void* x_fp16, int64_t ldx, const void* logits_fp16, int64_t ldl, const float* s_in,
                              const haq_expert_desc* experts_host, const haq_expert_colsum* colsums_host, int32_t T,
                              int32_t H, int32_t I, int32_t E, int32_t top_k, void* out_fp16, int64_t ldo,
                              const haq_moe_debug_asym* dbg_host, void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------
 * Measurement aids (no part of the method; used by the benchmark).
 *
 * haq_profile_enable(1) creates events (allocates; call it outside timed regions
 * and graph capture); from then on haq_w8a8_ffn and haq_moe_w8a8_ffn (all experts
 * resident) record one at every stage boundary of each call.  haq_profile_read
 * waits for the last profiled call and returns the stage names (host strings owned
 * by the library) and durations in milliseconds, at most max_stages of them.  The
 * state is process wide and not thread safe; haq_profile_enable(0) frees it.
 *
 * haq_probe_mfma_i8: a launch of `work_groups` work-groups of four waves that
 * issue nothing but v_mfma_i32_32x32x32_i8 on operands held in registers: every
 * wave reads 4 operand sets of 6 fragments (2 token, 4 weight fragments, the
 * register tile of the GEMM kernel; lane l of fragment f of set s = the 16 bytes
 * at data[((s * 6 + f) * 64 + l) * 16], 24 KiB in all) and accumulates
 * acc[i][j] += W(s, j) . X(s, i) over the sets, `iters` times: 2 * 32^3 * 32 *
 * iters operations per wave.  What a GPU sustains on this loop for operands with
 * the statistics of a workload is the ceiling a GEMM on such operands can reach.
 * out: int32 [256 * 128] device, the accumulators of work-group 0 (thread t,
 * tile (i, j), register r at ((t * 8 + i * 4 + j) * 16 + r), int32 wrap-around).
 *
 * haq_probe_kloop_i8: the same operands, register tile, work-group shape, `out`
 * and accumulators as haq_probe_mfma_i8, with the ingredients of the GEMM
 * kernel's K loop added one level at a time: 1 = the operand fragments are
 * re-read from LDS for every K-step; 2 = plus one work-group barrier per K-step;
 * 3 = plus the direct-to-LDS loads that refill the ring (six 1 KiB loads per
 * wave and K-step, all work-groups from the same 24 KiB); 4 = as 3 with the
 * refill through registers (vector loads, LDS writes a K-step later).  One iteration is two
 * K-steps (32 matrix instructions per wave).  The rate lost from one level to the
 * next is what that ingredient costs the matrix pipes.
 *
 * haq_probe_clock: one wave spins for ticks_100mhz periods of the constant 100 MHz
 * counter; out[0] = shader clock cycles elapsed, out[1] = 100 MHz periods elapsed
 * (uint64, device).  Launched on a second stream it reads the shader clock while
 * the kernels of another stream run.                                          */
int32_t haq_profile_enable(int32_t on);
int32_t haq_profile_read(int32_t max_stages, int32_t* n_stages, const char** names, float* ms);
int32_t haq_probe_mfma_i8(const int8_t* data, int32_t iters, int32_t work_groups, int32_t* out, void* stream);
int32_t haq_probe_kloop_i8(const int8_t* data, int32_t level, int32_t iters, int32_t work_groups, int32_t* out, void* stream);
int32_t haq_probe_clock(uint64_t* out, int64_t ticks_100mhz, void* stream);

/* ------------------------------------------------------------------------
 * haq_moe_w8a8_ffn for callers that cannot allocate device memory and have no
 * workspace to hand over: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, kernels and results as
 * haq_moe_w8a8_ffn with ctx = NULL and dbg = NULL (every expert device resident),
 * but the scratch memory is an array of 16 MiB built into the library (one per
 * GPU, held until the process ends) instead of a caller workspace.  The call
 * allocates nothing (no hipMalloc / hipFree, no allocating library routine).
 * Limit: haq_moe_workspace_bytes(T, H, I, E) <= 16 MiB (the Mixtral geometry, H =
 * 4096, I = 14336, 8 experts: up to 104 tokens); larger problems return HAQ_ERR_WORKSPACE and
 * say how much was needed.  The first call on a device looks the array's address
 * up (make that call outside graph capture); call with the stream's device current.
 * All calls on one GPU share the array: calls that overlap on one GPU (two streams, or two host
 * threads) race; calls on one stream are ordered and safe.  Nothing in the array
 * has to be cleared between calls: every buffer carved from it is written before
 * it is read within a call.                                                    */
int32_t haq_moe_w8a8_ffn_static(const void* x_fp16, int64_t ldx, const void* logits_fp16, int64_t ldl,
                                const float* s_in, const haq_expert_desc* experts_host, int32_t T, int32_t H,
                                int32_t I, int32_t E, int32_t top_k, void* out_fp16, int64_t ldo, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* HAQ_H */
