"""GPU-vs-oracle parity through the C ABI (ctypes binding), element by element.

Bars: bit-exact for int8 codes, scales derived by IEEE operations, int32
accumulators, routing indices and permutations; fp16 outputs within
|gpu - cpu| <= 1e-3 |cpu| + 1e-3 rms(cpu row) (they are in fact expected to be
bit-identical, because both sides round every binary32 operation once and use the
same defined e^t sequence; the tests report that too).
"""
import numpy as np
import pytest
import torch

import haq_inputs as hi
import oracle
import paper_2508_07329_amd as haq
from tests import offline
from tests.gpu_util import bits_equal, dev, diff_report, fp16_close, host, mixtral_layer, upload_experts

pytestmark = pytest.mark.gpu
F32 = np.float32


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    haq.lib()


# ------------------------------------------------------------------ A1
@pytest.mark.parametrize("T,K,with_s", [(16, 768, True), (2048, 4096, True), (37, 14336, True), (1, 64, False),
                                         (9, 16384, True), (300, 832, False), (11, 32768, True), (3, 65536, False),
                                         (2101, 16384, True), (8203, 4096, True), (16390, 832, False)])
def test_smooth_quant_act_bit_exact(T, K, with_s):
    X, _, _ = hi.hidden_states(100 + T, T, K, n_outlier=max(1, K // 200))
    if T > 4:
        X[3] = 0  # a zero row
    s = np.exp(np.random.default_rng(T).normal(0, 1, K)).astype(F32) if with_s else None
    q_ref, sx_ref = oracle.smooth_quant_act(X, s)
    q, sx = haq.haq_smooth_quant_act(dev(X), None if s is None else dev(s))
    assert bits_equal(host(sx), sx_ref)
    assert bits_equal(host(q), q_ref)


def test_smooth_quant_act_divisors_outside_reciprocal_range():
    """Smoothing entries and row scales beyond the range in which the kernel divides through
    reciprocals: those chunks and rows must take true divisions and still match bit for bit."""
    T, K = 21, 1024
    X, _, _ = hi.hidden_states(77, T, K, n_outlier=5)
    rng = np.random.default_rng(78)
    s = np.exp(rng.normal(0, 1, K)).astype(F32)
    s[rng.integers(0, K, 40)] = F32(1e-20)
    s[rng.integers(0, K, 40)] = F32(1e20)
    X[5] = np.float16(6e-8)  # subnormal halves: a tiny row scale
    X[6, :] = 0
    X[6, 17] = np.float16(-3.0)
    for sv in (s, np.full(K, 1e25, F32), np.full(K, 1e-13, F32)):
        q_ref, sx_ref = oracle.smooth_quant_act(X, sv)
        assert np.isfinite(sx_ref).all()
        q, sx = haq.haq_smooth_quant_act(dev(X), dev(sv))
        assert bits_equal(host(sx), sx_ref)
        assert bits_equal(host(q), q_ref)


def test_smooth_quant_act_strided_input_and_empty():
    X, _, _ = hi.hidden_states(5, 20, 256)
    big = torch.zeros((20, 512), dtype=torch.float16, device="cuda:0")
    big[:, :256] = dev(X)
    q, sx = haq.haq_smooth_quant_act(big[:, :256], None)
    q_ref, sx_ref = oracle.smooth_quant_act(X, None)
    assert bits_equal(host(q), q_ref) and bits_equal(host(sx), sx_ref)
    q0, sx0 = haq.haq_smooth_quant_act(torch.empty((0, 256), dtype=torch.float16, device="cuda:0"), None)
    assert q0.shape == (0, 256) and sx0.shape == (0,)


# ------------------------------------------------------------------ offline side
def test_offline_quantiser_bit_exact():
    X, _, _ = hi.hidden_states(6, 70, 320, 4, 50.0)
    W = hi.gaussian_weight(6, 0, 320, 200)
    W[:, 7] = 0  # a zero output channel
    ax = host(haq.haq_channel_absmax_f16(dev(X)))
    aw = host(haq.haq_weight_row_absmax(dev(W)))
    assert bits_equal(ax, oracle.col_absmax_f16(X)) and bits_equal(aw, oracle.row_absmax_f32(W))
    s = haq.haq_smoothing_vector(dev(ax), dev(aw), 0.5)
    s_ref = oracle.smoothing_vector(ax, aw, 0.5)
    assert bits_equal(host(s), s_ref)
    wq, sw = haq.haq_quant_weight(dev(W), s)
    wq_ref, sw_ref = oracle.quant_weight(W, s_ref)
    assert bits_equal(host(sw), sw_ref) and bits_equal(host(wq), wq_ref)
    wq1, sw1 = haq.haq_quant_weight(dev(W), None)
    wq1_ref, sw1_ref = oracle.quant_weight(W, None)
    assert bits_equal(host(sw1), sw1_ref) and bits_equal(host(wq1), wq1_ref)


def test_pack_layouts():
    rng = np.random.default_rng(7)
    K, N = 128, 96
    w1 = rng.integers(-127, 128, (K, N)).astype(np.int8)
    w3 = rng.integers(-127, 128, (K, N)).astype(np.int8)
    p = host(haq.haq_pack_weight(dev(w1))).reshape(K // 16, 256, 16)
    ref = np.zeros((K // 16, 256, 16), np.int8)
    ref[:, :N, :] = w1.reshape(K // 16, 16, N).transpose(0, 2, 1)
    assert np.array_equal(p, ref)
    g = host(haq.haq_pack_gate_up(dev(w1), dev(w3))).reshape(K // 16, 256, 16)
    inter = np.zeros((K, 2 * N), np.int8)
    for b in range(N // 32):
        inter[:, 64 * b:64 * b + 32] = w1[:, 32 * b:32 * b + 32]
        inter[:, 64 * b + 32:64 * b + 64] = w3[:, 32 * b:32 * b + 32]
    ref = np.zeros((K // 16, 256, 16), np.int8)
    ref[:, :2 * N, :] = inter.reshape(K // 16, 16, 2 * N).transpose(0, 2, 1)
    assert np.array_equal(g, ref)


# ------------------------------------------------------------------ A1+A2+A3 linear
def _linear_case(X, W, act):
    s, Wq, sw = offline.quantize_linear(X, W)
    Y_ref, acc_ref, q_ref, sx_ref = oracle.w8a8_linear(X, s, Wq, sw, act, full=True)
    wp = haq.haq_pack_weight(dev(Wq))
    y, acc, q, sx = haq.haq_w8a8_linear(dev(X), dev(s), wp, dev(sw), W.shape[1], oracle.ACT[act], debug=True)
    assert bits_equal(host(q), q_ref) and bits_equal(host(sx), sx_ref)
    assert bits_equal(host(acc), acc_ref)
    assert fp16_close(host(y), Y_ref)
    assert bits_equal(host(y), Y_ref)
    y2 = haq.haq_w8a8_linear(dev(X), dev(s), wp, dev(sw), W.shape[1], oracle.ACT[act])
    assert bits_equal(host(y2), Y_ref)


def test_linear_opt125m_config():
    wl = hi.OPT125M_LINEAR
    X, _, _ = hi.hidden_states(wl.seed, wl.T, wl.K, wl.n_outlier, wl.mult)
    _linear_case(X, hi.gaussian_weight(wl.seed, 0, wl.K, wl.N), wl.act)


@pytest.mark.parametrize("T,K,N,act", [(300, 832, 1040, "relu"), (1, 64, 16, "none"), (257, 1024, 272, "none"),
                                        (513, 2048, 768, "relu"), (5, 32768, 48, "none"), (130, 65536, 16, "relu"),
                                        (4101, 128, 32, "relu"), (2051, 4096, 64, "none"),
                                        (4100, 128, 7696, "relu"), (8200, 64, 4112, "none"),
                                        (2000, 64, 3984, "relu"), (1600, 128, 4000, "none")])
def test_linear_ragged_shapes(T, K, N, act):
    """Two are long enough for the pipelined quantisation kernel (its transposed write-out of the packed codes ends
    in a partial block of rows); two have at least 512 tiles of 256 x 256 and take the large-tile instantiation of
    the GEMM, the last two fill one round of 256 x 128 tiles and take that instantiation (ragged last row and
    channel tiles), each on the call without debug outputs."""
    X, _, _ = hi.hidden_states(T + K, T, K, n_outlier=3)
    _linear_case(X, hi.gaussian_weight(T + K, 0, K, N), act)


@pytest.mark.parametrize("T,K,N,act", [(37, 80, 48, "relu"), (300, 1040, 272, "none"), (5, 16, 16, "none"), (2051, 4112, 64, "relu")])
def test_linear_input_widths_that_are_not_whole_k_steps(T, K, N, act):
    """K a multiple of 16 but not of 64: the packed operands round K up, the pad of the weights is zero and whatever the
    activation buffer holds there drops out.  The workspace is filled with a non-zero pattern first."""
    X, _, _ = hi.hidden_states(T + K, T, K, n_outlier=2)
    W = hi.gaussian_weight(T + K, 0, K, N)
    s, Wq, sw = offline.quantize_linear(X, W)
    Y_ref, acc_ref, q_ref, sx_ref = oracle.w8a8_linear(X, s, Wq, sw, act, full=True)
    ws = torch.full((haq.haq_linear_workspace_bytes(T, K, N),), 0x5B, dtype=torch.uint8, device="cuda:0")
    y, acc, q, sx = haq.haq_w8a8_linear(dev(X), dev(s), haq.haq_pack_weight(dev(Wq)), dev(sw), N, oracle.ACT[act], workspace=ws, debug=True)
    assert bits_equal(host(q), q_ref) and bits_equal(host(sx), sx_ref) and bits_equal(host(acc), acc_ref)
    assert bits_equal(host(y), Y_ref)
    # the call that takes the canonical [K x N] layout of the weight operand
    ws2 = torch.full((haq.haq_linear_kn_workspace_bytes(T, K, N),), 0x5B, dtype=torch.uint8, device="cuda:0")
    assert bits_equal(host(haq.haq_w8a8_linear_kn(dev(X), dev(s), dev(Wq), dev(sw), oracle.ACT[act], workspace=ws2)), Y_ref)
    q2, sx2 = haq.haq_smooth_quant_act(dev(X), dev(s))
    assert bits_equal(host(q2), q_ref) and bits_equal(host(sx2), sx_ref)


def test_ffn_widths_that_are_not_whole_k_steps():
    T, K, F, N = 130, 208, 304, 80
    X, _, _ = hi.hidden_states(9, T, K, n_outlier=2)
    W1, W2 = hi.gaussian_weight(9, 0, K, F), hi.gaussian_weight(9, 1, F, N)
    (s1, W1q, sw1), (s2, W2q, sw2) = offline.quantize_ffn(X, W1, W2)
    h_ref = oracle.w8a8_linear(X, s1, W1q, sw1, "relu")
    y_ref = oracle.w8a8_linear(h_ref, s2, W2q, sw2, "none")
    y, h = haq.haq_w8a8_ffn(dev(X), dev(s1), haq.haq_pack_weight(dev(W1q)), dev(sw1), F, haq.HAQ_ACT_RELU, dev(s2),
                            haq.haq_pack_weight(dev(W2q)), dev(sw2), N, debug=True)
    assert bits_equal(host(h), h_ref) and bits_equal(host(y), y_ref)


def test_linear_extreme_accumulators():
    K = 16384
    X = np.full((3, K), 127, np.float16)
    X[1] = -127
    X[2, ::2] = -127
    Wq = np.full((K, 16), 127, np.int8)
    Wq[:, 1] = -127
    sw = np.full(16, 1e-6, F32)
    y, acc, q, sx = haq.haq_w8a8_linear(dev(X), None, haq.haq_pack_weight(dev(Wq)), dev(sw), 16, debug=True)
    Y_ref, acc_ref, _, _ = oracle.w8a8_linear(X, None, Wq, sw, "none", full=True)
    assert acc_ref[0, 0] == 127 * 127 * K
    assert bits_equal(host(acc), acc_ref) and bits_equal(host(y), Y_ref)


def test_ffn_opt67b_full_size_every_row():
    """OPT-6.7B FFN block at full size; the oracle computes all 2048 token rows end to end."""
    wl = hi.OPT67B_FFN
    X, _, _ = hi.hidden_states(wl.seed, wl.T, wl.H, wl.n_outlier, wl.mult)
    W1 = hi.gaussian_weight(wl.seed, 0, wl.H, wl.F)
    W2 = hi.gaussian_weight(wl.seed, 1, wl.F, wl.H)
    rows = np.arange(wl.T)
    (s1, W1q, sw1), (s2, W2q, sw2) = offline.quantize_ffn(X, W1, W2)
    del W1, W2
    w1p, w2p = haq.haq_pack_weight(dev(W1q)), haq.haq_pack_weight(dev(W2q))
    h = haq.haq_w8a8_linear(dev(X), dev(s1), w1p, dev(sw1), wl.F, haq.HAQ_ACT_RELU)
    y = haq.haq_w8a8_linear(h, dev(s2), w2p, dev(sw2), wl.H, haq.HAQ_ACT_NONE)
    yf, hf = haq.haq_w8a8_ffn(dev(X), dev(s1), w1p, dev(sw1), wl.F, haq.HAQ_ACT_RELU, dev(s2), w2p, dev(sw2), wl.H, debug=True)
    assert bits_equal(host(hf), host(h)) and bits_equal(host(yf), host(y))
    h_ref = oracle.w8a8_linear(X[rows], s1, W1q, sw1, "relu")
    y_ref = oracle.w8a8_linear(h_ref, s2, W2q, sw2, "none")
    assert bits_equal(host(h)[rows], h_ref)
    assert fp16_close(host(y)[rows], y_ref)
    assert bits_equal(host(y)[rows], y_ref)


@pytest.mark.parametrize("T,K,F,N,act", [(300, 256, 1088, 272, "relu"), (1, 64, 64, 16, "none"), (513, 832, 768, 1040, "relu")])
def test_fused_ffn_equals_oracle_chain(T, K, F, N, act):
    X, _, _ = hi.hidden_states(T + F, T, K, n_outlier=3)
    W1, W2 = hi.gaussian_weight(T + F, 0, K, F), hi.gaussian_weight(T + F, 1, F, N)
    if act == "none":  # the offline helper calibrates the second layer on a ReLU intermediate: do it by hand here
        s1, W1q, sw1 = offline.quantize_linear(X, W1)
        s2, W2q, sw2 = offline.quantize_linear(oracle.w8a8_linear(X, s1, W1q, sw1, act), W2)
    else:
        (s1, W1q, sw1), (s2, W2q, sw2) = offline.quantize_ffn(X, W1, W2)
    h_ref = oracle.w8a8_linear(X, s1, W1q, sw1, act)
    y_ref = oracle.w8a8_linear(h_ref, s2, W2q, sw2, "none")
    y, h = haq.haq_w8a8_ffn(dev(X), dev(s1), haq.haq_pack_weight(dev(W1q)), dev(sw1), F, oracle.ACT[act], dev(s2),
                            haq.haq_pack_weight(dev(W2q)), dev(sw2), N, debug=True)
    assert bits_equal(host(h), h_ref), diff_report(host(h), h_ref)
    assert fp16_close(host(y), y_ref)
    assert bits_equal(host(y), y_ref), diff_report(host(y), y_ref)
    y2 = haq.haq_w8a8_ffn(dev(X), dev(s1), haq.haq_pack_weight(dev(W1q)), dev(sw1), F, oracle.ACT[act], None,
                          haq.haq_pack_weight(dev(oracle.quant_weight(W2, None)[0])), dev(oracle.quant_weight(W2, None)[1]), N)
    y2_ref = oracle.w8a8_linear(h_ref, None, *oracle.quant_weight(W2, None), "none")
    assert bits_equal(host(y2), y2_ref)


# ------------------------------------------------------------------ MoE, small shapes, everything compared
def _check_moe(m, dev_experts=None, tokens=None, ctx=None):
    X, logits, s_in, experts = m["X"], m["logits"], m["s_in"], m["experts"]
    T, H = X.shape
    I = experts[0].w1.shape[1]
    E = len(experts)
    if dev_experts is None:
        dev_experts = upload_experts(experts)
    out, d = haq.haq_moe_w8a8_ffn(dev(X), dev(logits), dev(s_in), dev_experts, I, ctx=ctx, debug=True)
    torch.cuda.synchronize()
    idx_ref, gw_ref = oracle.route_top2(logits)
    counts, offsets, perm, inv = oracle.permute(idx_ref, E)
    assert bits_equal(host(d.topk_idx), idx_ref)
    assert bits_equal(host(d.topk_w), gw_ref)
    assert bits_equal(host(d.counts), counts) and bits_equal(host(d.offsets), offsets)
    assert bits_equal(host(d.perm), perm) and bits_equal(host(d.inv), inv)
    q_ref, sx_ref = oracle.smooth_quant_act(X, s_in)
    assert bits_equal(host(d.q), q_ref) and bits_equal(host(d.sx), sx_ref)
    tok = np.arange(T, dtype=np.int32) if tokens is None else np.asarray(tokens, np.int32)
    out_ref, mid_ref, hq_ref, sh_ref, y_ref = oracle.moe_ffn(X, idx_ref, gw_ref, s_in, experts, tokens=tok, dumps=True)
    pos = inv[(2 * tok[:, None] + np.arange(2)[None, :]).ravel()]  # sorted positions of the sampled pairs
    assert fp16_close(host(d.mid_fp16)[pos], mid_ref)
    assert fp16_close(host(d.y_fp16)[pos], y_ref)
    assert fp16_close(host(out)[tok], out_ref)
    for name, g, c in (("mid", host(d.mid_fp16)[pos], mid_ref), ("hq", host(d.hq)[pos], hq_ref),
                       ("sh", host(d.sh)[pos], sh_ref), ("y", host(d.y_fp16)[pos], y_ref), ("out", host(out)[tok], out_ref)):
        assert bits_equal(g, c), f"{name}: {diff_report(g, c)}"
    out2 = haq.haq_moe_w8a8_ffn(dev(X), dev(logits), dev(s_in), dev_experts, I, ctx=ctx)
    assert bits_equal(host(out2), host(out))
    return counts


@pytest.mark.parametrize("T,H,I,E", [(37, 128, 320, 8), (1, 128, 192, 8), (300, 256, 576, 8), (9, 128, 192, 2),
                                      (530, 192, 448, 4), (257, 128, 192, 8), (700, 128, 192, 32), (2100, 128, 256, 8)])
def test_moe_small_everything_bit_exact(T, H, I, E):
    """(The 2100-token case is long enough for the pipelined quantisation kernel on both the gathered token
    rows and the per-expert requantisation, with expert groups that start at unaligned rows.)"""
    _check_moe(offline.small_moe(seed=20 + T, T=T, H=H, I=I, E=E))


@pytest.mark.parametrize("T,H,I,E", [(37, 128, 512, 8), (1, 128, 512, 8), (64, 256, 1024, 4), (33, 384, 512, 8),
                                      (5, 128, 512, 2)])
def test_moe_small_decode_path_bit_exact(T, H, I, E):
    """Shapes that take the weight-streaming (at most 64 tokens) kernels."""
    _check_moe(offline.small_moe(seed=40 + T, T=T, H=H, I=I, E=E))


@pytest.mark.parametrize("T,H,I,E,same_experts", [(1, 128, 512, 8, False), (2, 128, 512, 8, False), (2, 256, 768, 4, True),
                                                   (2, 4352, 512, 8, False), (1, 4224, 256, 2, False)])
def test_moe_one_or_two_tokens_fused_launches(T, H, I, E, same_experts):
    """One or two tokens without the on-chip intermediates asked for: routing and token quantisation run
    inside the gate/up launch and the requantisation inside the down launch.  Everything this path still
    writes (routing results, h, per-pair y, output) must equal the oracle bit for bit; H > 4096 takes
    the two-chunks-per-thread variant of the in-kernel token quantisation."""
    m = offline.small_moe(seed=70 + T + H, T=T, H=H, I=I, E=E)
    if same_experts:  # both tokens to the same two experts: two rows per expert
        m["logits"][:, 1] = 30
        m["logits"][:, 2] = 20
    X, logits, s_in, experts = m["X"], m["logits"], m["s_in"], m["experts"]
    dev_experts = upload_experts(experts)
    want = ("topk_idx", "topk_w", "counts", "offsets", "perm", "inv", "mid_fp16", "y_fp16")
    idx_ref, gw_ref = oracle.route_top2(logits)
    counts, offsets, perm, inv = oracle.permute(idx_ref, E)
    if same_experts:
        assert counts[1] == 2 and counts[2] == 2
    out_ref, mid_ref, _, _, y_ref = oracle.moe_ffn(X, idx_ref, gw_ref, s_in, experts, tokens=np.arange(T, dtype=np.int32), dumps=True)
    pos = inv[(2 * np.arange(T)[:, None] + np.arange(2)[None, :]).ravel()]
    for rep in range(2):  # the second call finds the workspace and caches as the first left them
        out, d = haq.haq_moe_w8a8_ffn(dev(X), dev(logits), dev(s_in), dev_experts, I, debug=want)
        torch.cuda.synchronize()
        assert d.q is None and d.hq is None
        assert bits_equal(host(d.topk_idx), idx_ref) and bits_equal(host(d.topk_w), gw_ref)
        assert bits_equal(host(d.counts), counts) and bits_equal(host(d.offsets), offsets)
        assert bits_equal(host(d.perm), perm) and bits_equal(host(d.inv), inv)
        for name, g, c in (("mid", host(d.mid_fp16)[pos], mid_ref), ("y", host(d.y_fp16)[pos], y_ref), ("out", host(out), out_ref)):
            assert bits_equal(g, c), f"{name} (call {rep}): {diff_report(g, c)}"
    plain = haq.haq_moe_w8a8_ffn(dev(X), dev(logits), None if s_in is None else dev(s_in), dev_experts, I)
    assert bits_equal(host(plain), out_ref)


def test_moe_one_or_two_tokens_fused_launches_agree_with_the_five_launch_path():
    """Many random small layers (expert counts 2..32, tied logits included): the three-launch path for one or
    two tokens must give the bits of the five-launch path, which the other tests pin to the oracle."""
    rng = np.random.default_rng(77)
    for case in range(40):
        T = int(rng.integers(1, 3))
        E = int(rng.choice([2, 3, 8, 17, 32]))
        H = int(rng.choice([128, 256, 640]))
        I = int(rng.choice([256, 512, 1280]))
        X = dev((rng.standard_normal((T, H)) * rng.choice([0.01, 1.0, 30.0])).astype(np.float16))
        logits_h = rng.standard_normal((T, E)).astype(np.float16)
        if case % 4 == 0:
            logits_h[:] = logits_h[:, :1]  # every expert tied: the lowest indices win
        logits = dev(logits_h)
        s_in = dev(np.exp(rng.normal(0, 1, H)).astype(F32))
        g = torch.Generator(device="cuda:0").manual_seed(case)
        r8 = lambda n: torch.randint(-127, 128, (n,), dtype=torch.int8, device="cuda:0", generator=g)
        rf = lambda n, lo, hi: torch.rand(n, device="cuda:0", generator=g) * (hi - lo) + lo
        experts = [haq.ExpertWeights(r8(haq.haq_packed_bytes(H, 2 * I)), r8(haq.haq_packed_bytes(I, H)), rf(I, 1e-3, 2e-3),
                                     rf(I, 1e-3, 2e-3), rf(H, 1e-3, 2e-3), rf(I, 0.5, 2.0)) for _ in range(E)]
        fused = haq.haq_moe_w8a8_ffn(X, logits, s_in, experts, I)
        general, d = haq.haq_moe_w8a8_ffn(X, logits, s_in, experts, I, debug=True)
        torch.cuda.synchronize()
        assert torch.equal(fused.view(torch.int16), general.view(torch.int16)), f"case {case}: T={T} E={E} H={H} I={I}"
        if case % 4 == 0:
            assert host(d.topk_idx).tolist() == [[0, 1]] * T


def test_moe_decode_path_experts_with_more_than_32_rows():
    """Weight-streaming path with skewed routing: expert 0 takes every token (64 rows: two row blocks in
    one pass), another one more than 32, the rest few or none."""
    m = offline.small_moe(seed=44, T=64, H=256, I=512, E=8, routing="popularity")
    m["logits"][:, 0] = 50                      # everybody's first choice
    m["logits"][:40, 3] = 40                    # 40 tokens' second choice
    m["logits"][:, 6] = -100                    # nobody's
    counts = _check_moe(m)
    assert counts[0] == 64 and 40 <= counts[3] <= 64 and counts[6] == 0 and 0 < counts[1] <= 32


def test_moe_small_skewed_routing_and_empty_expert():
    m = offline.small_moe(seed=31, T=64, H=128, I=192, E=8, routing="popularity")
    m["logits"][:, 5] = -100  # nobody picks expert 5
    counts = _check_moe(m)
    assert counts[5] == 0 and counts.max() > 2 * np.median(counts)


# ------------------------------------------------------------------ experts streamed from pinned host memory
def _offload(dev_experts, host_ids):
    """Copies of the experts in `host_ids` moved to pinned host memory (the others stay as they are)."""
    out = []
    for e, ex in enumerate(dev_experts):
        if e in host_ids:
            w13 = torch.empty(ex.w13.shape, dtype=torch.int8, pin_memory=True).copy_(ex.w13)
            w2 = torch.empty(ex.w2.shape, dtype=torch.int8, pin_memory=True).copy_(ex.w2)
            out.append(haq.ExpertWeights(w13, w2, ex.sw1, ex.sw3, ex.sw2, ex.s_mid, haq.HAQ_LOC_HOST_PINNED))
        else:
            out.append(ex)
    torch.cuda.synchronize()
    return out


@pytest.mark.parametrize("H,I", [(128, 320), (256, 512)])   # the second shape lets streamed experts with at most 64 rows
@pytest.mark.parametrize("n_slots,host_ids", [(2, (4, 5, 6, 7)), (1, (0, 3, 5)), (3, (1, 2, 3, 4, 5, 6, 7))])   # take the weight-streaming kernels
def test_moe_offload_small_matches_resident_and_oracle(n_slots, host_ids, H, I):
    m = offline.small_moe(seed=50 + n_slots, T=90, H=H, I=I, E=8, routing="popularity")
    if n_slots == 1:
        m["logits"][:, 3] = -100  # a host-resident expert nobody selects: never copied
    dev_experts = upload_experts(m["experts"])
    X, logits, s_in = dev(m["X"]), dev(m["logits"]), dev(m["s_in"])
    ref = haq.haq_moe_w8a8_ffn(X, logits, s_in, dev_experts, I)
    ctx = haq.haq_ctx_create(H, I, n_slots)
    try:
        mixed = _offload(dev_experts, host_ids)
        _check_moe(m, mixed, ctx=ctx)
        for _ in range(2):  # slots are reused across calls
            out = haq.haq_moe_w8a8_ffn(X, logits, s_in, mixed, I, ctx=ctx)
            assert bits_equal(host(out), host(ref))
    finally:
        torch.cuda.synchronize()
        haq.haq_ctx_destroy(ctx)


def test_moe_offload_needs_context():
    m = offline.small_moe(seed=53, T=8, H=128, I=320, E=8)
    mixed = _offload(upload_experts(m["experts"]), (2,))
    with pytest.raises(haq.HaqError):
        haq.haq_moe_w8a8_ffn(dev(m["X"]), dev(m["logits"]), dev(m["s_in"]), mixed, 320)


# ------------------------------------------------------------------ MoE at the Mixtral shape (every token)
@pytest.fixture(scope="module")
def layer():
    return mixtral_layer()


def _mixtral_case(wl, layer):
    X = hi.moe_hidden_states(wl)
    logits = hi.moe_logits(wl, X)
    return dict(X=X, logits=logits, s_in=layer["s_in"], experts=layer["experts"])


@pytest.mark.parametrize("b", [1, 8, 64])
def test_moe_mixtral_decode(layer, b):
    wl = {w.T: w for w in hi.MIXTRAL_DECODE}[b]
    _check_moe(_mixtral_case(wl, layer), layer["dev_experts"], np.arange(b))  # every token


@pytest.mark.parametrize("b", [1, 8])
def test_moe_mixtral_decode_graph_replay(layer, b):
    """The launch configuration bench.py times for decode: the call captured once into a graph and
    replayed.  Every replay (with eager work on other inputs in between, which dirties the shared
    workspace) must give the oracle's output."""
    wl = {w.T: w for w in hi.MIXTRAL_DECODE}[b]
    case = _mixtral_case(wl, layer)
    other = _mixtral_case({w.T: w for w in hi.MIXTRAL_DECODE}[64], layer)
    idx, gw = oracle.route_top2(case["logits"])
    ref = oracle.moe_ffn(case["X"], idx, gw, case["s_in"], case["experts"])
    X, logits = dev(case["X"]), dev(case["logits"])
    Xo, Lo = dev(other["X"]), dev(other["logits"])
    ws = torch.empty(haq.haq_moe_workspace_bytes(64, wl.H, wl.I, wl.E), dtype=torch.uint8, device="cuda:0")
    out = torch.empty((b, wl.H), dtype=torch.float16, device="cuda:0")
    haq.haq_moe_w8a8_ffn(X, logits, layer["dev_s_in"], layer["dev_experts"], wl.I, out=out, workspace=ws)  # warm-up
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        haq.haq_moe_w8a8_ffn(X, logits, layer["dev_s_in"], layer["dev_experts"], wl.I, out=out, workspace=ws)
    for rep in range(4):
        out.zero_()
        haq.haq_moe_w8a8_ffn(Xo, Lo, layer["dev_s_in"], layer["dev_experts"], wl.I, workspace=ws)  # eager, same workspace
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert bits_equal(host(out), ref), f"replay {rep}: {diff_report(host(out), ref)}"


def test_moe_mixtral_offload_four_of_eight_resident(layer):
    """256 tokens, experts 4-7 in pinned host memory and streamed through 2 staging slots."""
    wl = hi.MIXTRAL_OFFLOAD
    case = _mixtral_case(wl, layer)
    mixed = _offload(layer["dev_experts"], set(range(wl.E)) - set(wl.resident))
    ctx = haq.haq_ctx_create(wl.H, wl.I, 2)
    try:
        counts = _check_moe(case, mixed, np.arange(wl.T), ctx=ctx)  # every token
        assert np.all(counts > 0)
        ref = haq.haq_moe_w8a8_ffn(dev(case["X"]), dev(case["logits"]), layer["dev_s_in"], layer["dev_experts"], wl.I)
        out = haq.haq_moe_w8a8_ffn(dev(case["X"]), dev(case["logits"]), layer["dev_s_in"], mixed, wl.I, ctx=ctx)
        assert bits_equal(host(out), host(ref))
    finally:
        torch.cuda.synchronize()
        haq.haq_ctx_destroy(ctx)


def test_moe_mixtral_prefill_zipf(layer):
    """All 4096 tokens (8192 pairs: every row tile of every expert group) against the oracle."""
    wl = hi.MIXTRAL_PREFILL
    counts = _check_moe(_mixtral_case(wl, layer), layer["dev_experts"], np.arange(wl.T))
    share = counts / counts.sum()
    assert np.max(np.abs(share - hi.zipf_shares(8))) < 0.02


# ------------------------------------------------------------------ adaptive smoothing grid search (Algorithm 1 step 1)
def _search_case(name):
    if name == "small_ragged":
        X, _, _ = hi.hidden_states(61, 37, 128, 3, 40.0)
        return X, hi.gaussian_weight(61, 0, 128, 48)
    if name == "tiles_and_tails":
        X, _, _ = hi.hidden_states(62, 203, 320, 4, 50.0)
        return X, hi.gaussian_weight(62, 0, 320, 208)
    l = hi.OPT125M_LINEAR
    X, _, _ = hi.hidden_states(l.seed, l.T, l.K, l.n_outlier, l.mult)
    return X, hi.gaussian_weight(l.seed, 0, l.K, l.N)


@pytest.mark.parametrize("name", ["small_ragged", "tiles_and_tails", "opt125m_linear"])
def test_reference_product_and_loss_bit_exact(name):
    """One binary64 accumulator per output with ascending k, and sequential row sums: both
    sides perform the same binary64 operations in the same order, so the bits agree."""
    X, W = _search_case(name)
    yref = haq.haq_reference_matmul_f64(dev(X), dev(W))
    ref = oracle.matmul_f64(X, W)
    assert bits_equal(host(yref), ref)
    s, Wq, sw = offline.quantize_linear(X, W)
    Y = oracle.w8a8_linear(X, s, Wq, sw)
    loss = haq.haq_quant_loss_f64(dev(Y), yref)
    assert float(host(loss)[0]) == oracle.mse_f64(Y, ref)


@pytest.mark.parametrize("name,use_weight", [("small_ragged", False), ("small_ragged", True), ("tiles_and_tails", False),
                                             ("opt125m_linear", False), ("opt125m_linear", True)])
def test_smoothing_search_matches_oracle(name, use_weight):
    X, W = _search_case(name)
    grid = [i / 10 for i in range(11)]
    losses_ref, best_ref, s_ref = oracle.smoothing_search(X, W, grid, use_weight)
    losses, best, s = haq.haq_smoothing_search(dev(X), dev(W), grid, use_weight)
    assert np.array_equal(np.asarray(losses), losses_ref), diff_report(np.asarray(losses), losses_ref)
    assert best == best_ref
    assert bits_equal(host(s), s_ref)


def test_smoothing_search_ties_and_single_candidate():
    rng = np.random.default_rng(63)
    T, K, N = 24, 128, 48
    X = rng.uniform(-3.9, 3.9, (T, K)).astype(np.float16)
    X[rng.integers(0, T, K), np.arange(K)] = np.float16(4.0)
    W = rng.uniform(-0.24, 0.24, (K, N)).astype(F32)
    losses, best, s = haq.haq_smoothing_search(dev(X), dev(W), [1.0, 0.0, 0.5])
    assert losses[0] == losses[1] == losses[2] and best == 0      # s = 4, 1, 2: identical outputs, first kept
    assert bits_equal(host(s), np.full(K, 4.0, F32))
    l1, b1, s1 = haq.haq_smoothing_search(dev(X), dev(W), [0.3])
    lr, br, sr = oracle.smoothing_search(X, W, [0.3])
    assert b1 == 0 and l1[0] == lr[0] and bits_equal(host(s1), sr)
    with pytest.raises(haq.HaqError):
        haq.haq_smoothing_search(dev(X), dev(W), [0.5, 1.5])


def test_smoothing_search_full_size_fc1():
    """fc1 of the OPT-6.7B-shaped block, the shape bench.py's smooth_search workload times."""
    wl = hi.OPT67B_FFN
    X, _, _ = hi.hidden_states(wl.seed, wl.T, wl.H, wl.n_outlier, wl.mult)
    W = hi.gaussian_weight(wl.seed, 0, wl.H, wl.F)
    grid = [0.0, 0.5, 0.8]
    losses_ref, best_ref, s_ref = oracle.smoothing_search(X, W, grid)
    losses, best, s = haq.haq_smoothing_search(dev(X), dev(W), grid)
    assert np.array_equal(np.asarray(losses), losses_ref)
    assert best == best_ref == 1
    assert bits_equal(host(s), s_ref)


# ------------------------------------------------------------------ LRU expert cache across calls (Section III.C.1c)
def test_expert_cache_follows_lru_across_calls():
    """Calls whose routing activates chosen subsets of the host-resident experts: hits, misses and the
    final slot contents must follow a plain LRU cache, and every output must equal the all-resident one."""
    E, H, I, n_slots = 8, 128, 320, 3
    m = offline.small_moe(seed=71, T=40, H=H, I=I, E=E)
    dev_experts = upload_experts(m["experts"])
    host_ids = (2, 3, 4, 5, 6, 7)
    mixed = _offload(dev_experts, host_ids)
    X, s_in = dev(m["X"]), dev(m["s_in"])
    # each call allows only a subset of experts (the others get a logit nobody can pick)
    subsets = [(0, 2, 3), (2, 4), (0, 1), (5, 2), (3, 6, 7, 4), (2, 1), (7, 6, 5, 4, 3, 2), (2, 3)]
    ctx = haq.haq_ctx_create(H, I, n_slots)
    try:
        trace, hits_total = [], 0
        for sub in subsets:
            logits = m["logits"].copy()
            mask = np.ones(E, bool)
            mask[list(sub)] = False
            logits[:, mask] = -100
            ref = haq.haq_moe_w8a8_ffn(X, dev(logits), s_in, dev_experts, I)
            out, dbg = haq.haq_moe_w8a8_ffn(X, dev(logits), s_in, mixed, I, ctx=ctx, debug=True)
            assert bits_equal(host(out), host(ref)), f"subset {sub}"
            counts = host(dbg.counts)
            trace += [e for e in range(E) if e in host_ids and counts[e] > 0]   # activated host experts, expert order
        hit_flags, cache = oracle.lru_trace(trace, n_slots)
        hits, misses, nbytes, keys = haq.haq_ctx_cache_stats(ctx)
        assert hits == sum(hit_flags) and misses == len(trace) - sum(hit_flags) and hits > 0
        per_expert = haq.haq_packed_bytes(H, 2 * I) + haq.haq_packed_bytes(I, H)
        assert nbytes == misses * per_expert
        cached = {k for k in keys[:n_slots] if k}
        assert cached == {mixed[e].w13.data_ptr() for e in cache}
        # after invalidation the next call misses again and still computes the same result
        haq.haq_ctx_cache_invalidate(ctx)
        logits = m["logits"].copy()
        logits[:, [0, 1, 4, 5, 6, 7]] = -100
        out = haq.haq_moe_w8a8_ffn(X, dev(logits), s_in, mixed, I, ctx=ctx)
        assert bits_equal(host(out), host(haq.haq_moe_w8a8_ffn(X, dev(logits), s_in, dev_experts, I)))
        h2, m2, _, _ = haq.haq_ctx_cache_stats(ctx)
        assert (h2, m2) == (hits, misses + 2)
    finally:
        torch.cuda.synchronize()
        haq.haq_ctx_destroy(ctx)


# ------------------------------------------------------------------ Hessian-aware weight quantisation (Algorithm 1 step 2)
def _correlated(seed, T, K, rank):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((T, rank)) @ rng.standard_normal((rank, K)) + 0.1 * rng.standard_normal((T, K))).astype(np.float16)


@pytest.mark.parametrize("T,K,N,with_s", [(200, 64, 48, True), (203, 320, 208, True), (90, 96, 16, False), (512, 768, 3072, True)])
def test_hessian_quantiser_bit_exact(T, K, N, with_s):
    """Binary64 chains in the same order on both sides: Hessian, factor of its inverse, codes and scales."""
    X = _correlated(80 + K, T, K, max(4, K // 16))
    if K > 64:
        X[:, 5] = 0  # a channel that never fires
    W = hi.gaussian_weight(80 + K, 0, K, N)
    s = oracle.smoothing_vector(oracle.col_absmax_f16(X), oracle.row_absmax_f32(W), 0.5) if with_s else None
    H_ref = oracle.hessian(X, s, 0.01)
    H = haq.haq_hessian_f64(dev(X), None if s is None else dev(s), 0.01)
    assert bits_equal(host(H), H_ref), diff_report(host(H), H_ref)
    U_ref = oracle.inverse_cholesky_upper(H_ref)
    U = haq.haq_inverse_cholesky_upper_f64(H)
    assert bits_equal(host(U), U_ref), diff_report(host(U), U_ref)
    Wq_ref, sw_ref = oracle.gptq(W, s, U_ref)
    Wq, sw = haq.haq_hessian_quant_weight(dev(X), dev(W), None if s is None else dev(s), 0.01)
    assert bits_equal(host(sw), sw_ref)
    assert bits_equal(host(Wq), Wq_ref), diff_report(host(Wq), Wq_ref)
    # and the result is what the method is for: a lower output error than plain rounding
    Wr, _ = oracle.quant_weight(W, s)
    Xs = (X.astype(F32) / (s if s is not None else F32(1))).astype(np.float64)
    Ws = ((s[:, None] if s is not None else F32(1)) * W).astype(np.float64)
    err = lambda q: np.sum((Xs @ Ws - Xs @ (q * sw_ref.astype(np.float64))) ** 2)
    assert err(host(Wq)) < err(Wr)


def test_hessian_quantiser_rejects_an_indefinite_matrix():
    H = torch.tensor([[1.0, 2.0], [2.0, 1.0]], dtype=torch.float64, device="cuda:0")
    with pytest.raises(haq.HaqError):
        haq.haq_inverse_cholesky_upper_f64(H)


# ------------------------------------------------------------------ asymmetric activation codes (dense linear)
@pytest.mark.parametrize("T,K,N,act,relu_in", [(16, 768, 3072, "relu", False), (203, 320, 208, "none", True),
                                                (1, 64, 16, "none", False), (2048, 4096, 1024, "relu", True),
                                                (4101, 128, 32, "relu", False), (2051, 4096, 64, "none", False)])
def test_linear_asym_bit_exact(T, K, N, act, relu_in):
    X, _, _ = hi.hidden_states(90 + T, T, K, n_outlier=max(1, K // 200))
    if relu_in:
        X = np.maximum(X, 0).astype(np.float16)   # one-sided rows: zero point 0
    if T > 4:
        X[3] = 0
    if T > 8:
        X[5] = -np.abs(X[5])                       # all negative: zero point 255
        X[7] = np.float16(0.75)                    # a constant row
    W = hi.gaussian_weight(90 + T, 0, K, N)
    s, Wq, sw = offline.quantize_linear(X, W)
    y_ref, acc_ref, q_ref, sx_ref, zp_ref = oracle.w8a8_linear_asym(X, s, Wq, sw, act, full=True)
    wq_d = dev(Wq)
    y, acc, q, sx, zp = haq.haq_w8a8_linear_asym(dev(X), dev(s), haq.haq_pack_weight(wq_d), dev(sw), haq.haq_weight_colsum(wq_d),
                                                 N, haq.HAQ_ACT_RELU if act == "relu" else haq.HAQ_ACT_NONE, debug=True)
    assert bits_equal(host(haq.haq_weight_colsum(wq_d)), Wq.astype(np.int32).sum(axis=0, dtype=np.int32))
    assert bits_equal(host(sx), sx_ref) and bits_equal(host(zp), zp_ref)
    assert bits_equal(host(q), q_ref), diff_report(host(q), q_ref)
    assert bits_equal(host(acc), acc_ref), diff_report(host(acc), acc_ref)
    assert bits_equal(host(y), y_ref)
    y2 = haq.haq_w8a8_linear_asym(dev(X), dev(s), haq.haq_pack_weight(wq_d), dev(sw), haq.haq_weight_colsum(wq_d), N,
                                  haq.HAQ_ACT_RELU if act == "relu" else haq.HAQ_ACT_NONE)
    assert bits_equal(host(y2), y_ref)   # the launch without the debug dump


# ------------------------------------------------------------------ Algorithm 1 for one layer (search, then Hessian-aware codes)
@pytest.mark.parametrize("name", ["tiles_and_tails", "opt125m_linear"])
def test_quantize_layer_matches_oracle_composition(name):
    X, W = _search_case(name)
    if name == "opt125m_linear":
        X = np.concatenate([X, _correlated(95, 496, X.shape[1], 24)])   # more rows than the 16 of the config
    grid = [0.0, 0.25, 0.5, 0.75, 1.0]
    losses_ref, best_ref, s_ref = oracle.smoothing_search(X, W, grid)
    Wq_ref, sw_ref = oracle.hessian_quant_weight(X, W, s_ref, 0.01)
    s, wq, sw, losses, best = haq.haq_quantize_layer(dev(X), dev(W), grid)
    assert best == best_ref and np.array_equal(np.asarray(losses), losses_ref)
    assert bits_equal(host(s), s_ref) and bits_equal(host(sw), sw_ref)
    assert bits_equal(host(wq), Wq_ref), diff_report(host(wq), Wq_ref)
    # and the layer it produces runs on the hot path as the oracle's does
    y = haq.haq_w8a8_linear(dev(X), s, haq.haq_pack_weight(wq), sw, W.shape[1])
    assert bits_equal(host(y), oracle.w8a8_linear(X, s_ref, Wq_ref, sw_ref))


# ------------------------------------------------------------------ measurement aids
def test_mfma_probe_computes_the_stated_dot_products():
    """The pure-MFMA loop behind the benchmark's sustained ceiling is a correct computation: its accumulators
    equal the int8 dot products of the operand fragments it was given, times the iteration count."""
    rng = np.random.default_rng(5)
    data = rng.integers(-127, 128, 24576).astype(np.int8)
    iters = 3
    out = host(haq.haq_probe_mfma_i8(dev(data), iters, 3))          # [256 threads, 8 tiles, 16 registers]
    frag = data.reshape(4, 6, 64, 16).astype(np.int64)
    rows = np.concatenate([frag[:, :, :32, :], frag[:, :, 32:, :]], axis=3)   # [set, fragment, row 32, k 32]
    X, W = rows[:, :2], rows[:, 2:]
    prod = np.einsum("sjwk,sixk->ijwx", W, X) * iters                # [i, j, weight row, token row]
    ref = np.empty((256, 8, 16), np.int64)
    for t in range(256):
        l = t % 64
        for r in range(16):
            wrow = 8 * (r // 4) + 4 * (l // 32) + r % 4
            ref[t, :, r] = prod[:, :, wrow, l % 32].reshape(8)
    assert np.array_equal(out.astype(np.int64), ref)
    # the K-loop probes (fragments re-read from LDS; + barrier; + direct-to-LDS refills) compute the same sums
    for level in (1, 2, 3, 4):
        got = host(haq.haq_probe_kloop_i8(dev(data), level, iters, 5))
        assert np.array_equal(got.astype(np.int64), ref), f"level {level}"


def test_stage_profile_and_clock_probe_report():
    m = offline.small_moe(seed=33, T=300, H=128, I=320, E=8)
    experts = upload_experts(m["experts"])
    haq.haq_profile_enable(True)
    try:
        haq.haq_moe_w8a8_ffn(dev(m["X"]), dev(m["logits"]), dev(m["s_in"]), experts, 320)
        stages = haq.haq_profile_read()
    finally:
        haq.haq_profile_enable(False)
    names = [n for n, _ in stages]
    assert names == ["route + permute + quantise tokens", "grouped gate/up GEMM + SwiGLU", "requantise intermediate",
                     "grouped down GEMM", "combine"]
    assert all(0.0 < ms < 50.0 for _, ms in stages)
    clk = haq.haq_probe_clock(20000)
    torch.cuda.synchronize()
    cycles, ticks = (int(v) for v in clk.tolist())
    assert ticks >= 20000 and 100.0 < cycles / ticks * 100.0 < 3000.0     # MHz


# ------------------------------------------------------------------ asymmetric codes inside the routed expert FFN
def _colsums(dev_experts_src):
    """Per expert (cs1, cs3, cs2) from the library's own column-sum kernel on the canonical int8 matrices."""
    return [(haq.haq_weight_colsum(dev(ex.w1)), haq.haq_weight_colsum(dev(ex.w3)), haq.haq_weight_colsum(dev(ex.w2)))
            for ex in dev_experts_src]


def _check_moe_asym(m, dev_experts=None, colsums=None, tokens=None):
    X, logits, s_in, experts = m["X"], m["logits"], m["s_in"], m["experts"]
    T, H = X.shape
    I = experts[0].w1.shape[1]
    E = len(experts)
    if dev_experts is None:
        dev_experts = upload_experts(experts)
    if colsums is None:
        colsums = _colsums(experts)
    out, d, zx, zh = haq.haq_moe_w8a8_ffn_asym(dev(X), dev(logits), dev(s_in), dev_experts, colsums, I, debug=True)
    torch.cuda.synchronize()
    idx_ref, gw_ref = oracle.route_top2(logits)
    counts, offsets, perm, inv = oracle.permute(idx_ref, E)
    assert bits_equal(host(d.topk_idx), idx_ref) and bits_equal(host(d.topk_w), gw_ref)
    assert bits_equal(host(d.counts), counts) and bits_equal(host(d.offsets), offsets)
    assert bits_equal(host(d.perm), perm) and bits_equal(host(d.inv), inv)
    q_ref, sx_ref, zx_ref = oracle.asym_quant_act(X, s_in)
    assert bits_equal(host(d.sx), sx_ref) and bits_equal(host(zx), zx_ref)
    assert bits_equal(host(d.q), q_ref), diff_report(host(d.q), q_ref)
    tok = np.arange(T, dtype=np.int32) if tokens is None else np.asarray(tokens, np.int32)
    out_ref, mid_ref, hq_ref, sh_ref, zh_ref, y_ref = oracle.moe_ffn_asym(X, idx_ref, gw_ref, s_in, experts, tokens=tok, dumps=True)
    pos = inv[(2 * tok[:, None] + np.arange(2)[None, :]).ravel()]
    assert fp16_close(host(out)[tok], out_ref)
    for name, g, c in (("mid", host(d.mid_fp16)[pos], mid_ref), ("hq", host(d.hq)[pos], hq_ref), ("sh", host(d.sh)[pos], sh_ref),
                       ("zh", host(zh)[pos], zh_ref), ("y", host(d.y_fp16)[pos], y_ref), ("out", host(out)[tok], out_ref)):
        assert bits_equal(g, c), f"{name}: {diff_report(g, c)}"
    out2 = haq.haq_moe_w8a8_ffn_asym(dev(X), dev(logits), dev(s_in), dev_experts, colsums, I)
    assert bits_equal(host(out2), host(out))
    return counts


@pytest.mark.parametrize("T,H,I,E", [(37, 128, 320, 8), (1, 128, 192, 8), (300, 256, 576, 8), (9, 128, 192, 2), (530, 192, 448, 4),
                                      (700, 128, 192, 32), (64, 256, 1024, 4), (2100, 128, 256, 8),
                                      # at most 64 tokens with I a multiple of 256: the weight-streaming kernels
                                      (1, 128, 256, 8), (2, 256, 512, 8), (33, 128, 512, 2), (64, 128, 256, 2), (17, 256, 768, 8),
                                      (64, 128, 256, 32)])
def test_moe_asym_small_everything_bit_exact(T, H, I, E):
    _check_moe_asym(offline.small_moe(seed=220 + T, T=T, H=H, I=I, E=E))


def test_moe_asym_skewed_routing_empty_expert_and_one_sided_tokens():
    m = offline.small_moe(seed=231, T=64, H=128, I=192, E=8, routing="popularity")
    m["logits"][:, 5] = -100                     # nobody picks expert 5
    m["X"][:20] = np.abs(m["X"][:20])            # one-sided rows: zero point 0
    m["X"][7] = 0                                # a zero row: scale 0, zero point 0, codes 0
    counts = _check_moe_asym(m)
    assert counts[5] == 0


def test_moe_asym_identical_experts_equal_the_dense_asymmetric_linear_chain():
    """All experts the same: every pair's y is the dense chain (asymmetric gate/up linears, SwiGLU, asymmetric down
    linear) that haq_w8a8_linear_asym computes for the down stage."""
    m = offline.small_moe(seed=232, T=40, H=128, I=320, E=4)
    ex0 = m["experts"][0]
    same = [ex0] * 4
    m2 = dict(m, experts=same)
    _check_moe_asym(m2)
    out, d, zx, zh = haq.haq_moe_w8a8_ffn_asym(dev(m["X"]), dev(m["logits"]), dev(m["s_in"]), upload_experts(same), _colsums(same),
                                               320, debug=True)
    w2_d = dev(ex0.w2)
    y_lin = haq.haq_w8a8_linear_asym(d.mid_fp16, dev(ex0.s_mid), haq.haq_pack_weight(w2_d), dev(ex0.sw2), haq.haq_weight_colsum(w2_d), 128)
    assert bits_equal(host(y_lin), host(d.y_fp16))


def test_moe_asym_streaming_kernels_skewed_routing_and_empty_expert():
    m = offline.small_moe(seed=233, T=60, H=256, I=512, E=8, routing="popularity")
    m["logits"][:, 2] = -100                     # nobody picks expert 2
    m["X"][:10] = np.abs(m["X"][:10])
    m["X"][11] = 0
    counts = _check_moe_asym(m)
    assert counts[2] == 0 and counts.max() > 32  # both row-block code paths in one launch


@pytest.mark.parametrize("name", ["decode_b1", "decode_b8", "decode_b64", "prefill"])
def test_moe_asym_mixtral(layer, name):
    """The Mixtral-shaped layer with asymmetric codes: 1, 8 and 64 tokens (weight-streaming kernels), and the
    4096-token Zipf prefill batch (every token against the oracle)."""
    wl = hi.MIXTRAL_PREFILL if name == "prefill" else {w.T: w for w in hi.MIXTRAL_DECODE}[int(name.split("_b")[1])]
    if "colsums" not in layer:
        layer["colsums"] = _colsums(layer["experts"])
    _check_moe_asym(_mixtral_case(wl, layer), layer["dev_experts"], layer["colsums"], np.arange(wl.T))


def test_zero_token_calls_return_empty_outputs_on_every_block_level_entry_point():
    """T = 0 is a valid batch: every call returns an empty output and launches nothing."""
    m = offline.small_moe(seed=240, T=4, H=128, I=256, E=4)
    ex = upload_experts(m["experts"])
    X0 = torch.empty((0, 128), dtype=torch.float16, device="cuda:0")
    L0 = torch.empty((0, 4), dtype=torch.float16, device="cuda:0")
    s_in = dev(m["s_in"])
    assert haq.haq_moe_w8a8_ffn(X0, L0, s_in, ex, 256).shape == (0, 128)
    assert haq.haq_moe_w8a8_ffn_asym(X0, L0, s_in, ex, _colsums(m["experts"]), 256).shape == (0, 128)
    out0 = torch.empty((0, 128), dtype=torch.float16, device="cuda:0")
    assert haq.haq_moe_w8a8_ffn_static(X0, L0, s_in, ex, 256, out=out0).shape == (0, 128)
    e0 = m["experts"][0]
    w1, sw1 = dev(e0.w1), dev(e0.sw1)
    assert haq.haq_w8a8_linear(X0, s_in, haq.haq_pack_weight(w1), sw1, 256).shape == (0, 256)
    assert haq.haq_w8a8_linear_kn(X0, s_in, w1, sw1).shape == (0, 256)
    assert haq.haq_w8a8_linear_asym(X0, s_in, haq.haq_pack_weight(w1), sw1, haq.haq_weight_colsum(w1), 256).shape == (0, 256)
    assert haq.haq_w8a8_ffn(X0, s_in, haq.haq_pack_weight(w1), sw1, 256, haq.HAQ_ACT_RELU, dev(e0.s_mid), haq.haq_pack_weight(dev(e0.w2)),
                            dev(e0.sw2), 128).shape == (0, 128)
    torch.cuda.synchronize()


# ------------------------------------------------------------------ offload policy: Eq. 7-8 decision and CPU experts
def _cpu_handles(experts, ids):
    """CPU copies of the experts, alternately as binary32 copies and as kept int8 codes (same results)."""
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a))
    return {e: haq.haq_cpu_expert_create(t(experts[e].w1), t(experts[e].w3), t(experts[e].w2), t(experts[e].sw1), t(experts[e].sw3),
                                         t(experts[e].sw2), t(experts[e].s_mid), keep_codes=bool(e & 1)) for e in ids}


@pytest.mark.parametrize("t_e,lat_cpu,lat_gpu", [(10.0, 1.0, 0.5), (3.0, 1.0, 0.9), (0.4, 1.0, 0.1), (5.0, 0.2, 0.5)])
def test_offload_policy_decides_by_the_break_even_batch_and_cpu_experts_match_the_oracle(t_e, lat_cpu, lat_gpu):
    """Host-resident experts with CPU copies: per activated expert the call must take the decision of Eq. 7-8
    (n_inputs > n_critical -> transfer, else CPU; a cached expert stays on the GPU), and the layer output must be
    the oracle's hybrid layer for exactly those experts, bit for bit."""
    E, H, I = 8, 128, 320
    m = offline.small_moe(seed=140, T=48, H=H, I=I, E=E, routing="popularity")
    host_ids = (2, 3, 4, 5, 6, 7)
    dev_experts = upload_experts(m["experts"])
    mixed = _offload(dev_experts, host_ids)
    handles = _cpu_handles(m["experts"], host_ids[:-1])       # expert 7 has no CPU copy: always transferred
    ctx = haq.haq_ctx_create(H, I, 2)
    try:
        haq.haq_ctx_set_offload_policy(ctx, t_e, lat_cpu, lat_gpu, torch.from_numpy(m["s_in"]), 3)
        for e, h in handles.items():
            haq.haq_ctx_register_cpu_expert(ctx, mixed[e], h)
        n_crit = oracle.n_critical(t_e, lat_cpu, lat_gpu)
        X, logits, s_in = dev(m["X"]), dev(m["logits"]), dev(m["s_in"])
        idx, gw = oracle.route_top2(m["logits"])
        counts = np.bincount(idx.ravel(), minlength=E)
        cached = set()
        for call in range(2):
            out = haq.haq_moe_w8a8_ffn(X, logits, s_in, mixed, I, ctx=ctx)
            torch.cuda.synchronize()
            dec, nc = haq.haq_ctx_last_decisions(ctx)
            assert nc == (-1 if n_crit is None else n_crit)
            want, on_cpu = [], []
            for e in host_ids:
                if counts[e] == 0:
                    continue
                if e in cached:
                    what = haq.HAQ_DECISION_GPU_CACHED
                elif e in handles and (n_crit is None or counts[e] <= n_crit):
                    what = haq.HAQ_DECISION_CPU
                    on_cpu.append(e)
                else:
                    what = haq.HAQ_DECISION_TRANSFER
                want.append((e, int(counts[e]), what))
            assert dec == want, (call, dec, want)
            ref, _ = oracle.moe_ffn_hybrid(m["X"], idx, gw, m["s_in"], m["experts"], on_cpu)
            assert bits_equal(host(out), ref), f"call {call}: {diff_report(host(out), ref)}"
            _, _, _, keys = haq.haq_ctx_cache_stats(ctx)
            cached = {e for e in host_ids if mixed[e].w13.data_ptr() in keys[:2]}
        # the rule switched off: everything is transferred again and the result is the all-GPU one
        haq.haq_ctx_set_offload_policy(ctx, -1.0, 0.0, 0.0)
        out = haq.haq_moe_w8a8_ffn(X, logits, s_in, mixed, I, ctx=ctx)
        assert bits_equal(host(out), host(haq.haq_moe_w8a8_ffn(X, logits, s_in, dev_experts, I)))
        assert all(d[2] != haq.HAQ_DECISION_CPU for d in haq.haq_ctx_last_decisions(ctx)[0])
    finally:
        torch.cuda.synchronize()
        haq.haq_ctx_destroy(ctx)
        for h in handles.values():
            haq.haq_cpu_expert_destroy(h)
