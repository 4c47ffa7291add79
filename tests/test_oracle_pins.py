"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests calls the HIP library.  Each one is chosen so that a plausible
mistake in the oracle (dropped term, wrong sign / axis / index, transposed operand,
wrong rounding mode) fails it.  The paper prints no worked numerical example of the
operator, so the pins are closed forms, invariants, brute force on tiny inputs,
special cases that reduce to numpy routines and the a-priori quantisation error
bound of Eq. 1's operator.
"""
import itertools

import numpy as np
import pytest

import haq_inputs as hi
import oracle
from tests import offline

F32 = np.float32


# ----------------------------------------------------------------- binary16 / exp
def test_half_to_float_exhaustive():
    h = np.arange(65536, dtype=np.uint16)
    got = oracle.half_to_float(h)
    ref = h.view(np.float16).astype(np.float32)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got.view(np.uint32)[~nan], ref.view(np.uint32)[~nan])


def test_float_to_half_rne_against_numpy():
    rng = np.random.default_rng(0)
    x = rng.standard_normal(1_000_000).astype(F32) * F32(10.0) ** rng.integers(-9, 5, 1_000_000).astype(F32)
    # exact halfway points between neighbouring halves, and the overflow boundary
    h = np.arange(0, 0x7bff, dtype=np.uint16)
    lo = h.view(np.float16).astype(np.float64)
    hi_ = (h + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    mid = ((lo + hi_) / 2).astype(F32)
    edge = np.array([65504, 65519.996, 65520, 65536, 1e30, 2.0 ** -24, 2.0 ** -25, 2.0 ** -25 * 1.0001,
                     2.0 ** -14, 2.0 ** -14 * 0.99999, 0.0, -0.0, np.inf, -np.inf], dtype=F32)
    allx = np.concatenate([x, -x, mid, -mid, np.nextafter(mid, F32(0)), np.nextafter(mid, F32(1e9)), edge])
    with np.errstate(over="ignore"):
        ref = allx.astype(np.float16)
    got = oracle.float_to_half(allx)
    assert np.array_equal(got.view(np.uint16), ref.view(np.uint16))


def test_exp_spec_within_one_ulp_of_exp():
    t = np.concatenate([np.linspace(-87, 88, 1_500_001), np.linspace(-1, 1, 500_001)]).astype(F32)
    got = oracle.exp_spec(t).astype(np.float64)
    ref = np.exp(t.astype(np.float64))
    ulp = np.spacing(ref.astype(F32)).astype(np.float64)
    assert np.max(np.abs(got - ref) / ulp) < 1.0
    assert oracle.exp_spec(np.array([0.0], F32))[0] == 1.0
    # clamped outside [-87, 88]
    lo, hi_ = oracle.exp_spec(np.array([-87, 88], F32))
    assert np.array_equal(oracle.exp_spec(np.array([-1e4, -np.inf, 1e4], F32)), np.array([lo, lo, hi_], F32))
    # monotone on a coarse grid (catches a sign error in the reduction)
    g = oracle.exp_spec(np.linspace(-80, 80, 1601).astype(F32))
    assert np.all(np.diff(g) > 0)


# ----------------------------------------------------------------- O1 activation quantisation
def _acts(seed=0, T=33, K=200, **kw):
    return hi.hidden_states(seed, T, K, **kw)[0]


def test_act_quant_rounding_mode_and_scale():
    # absmax 127 and s = 1 -> scale exactly 1 -> codes are rne(x): ties go to even
    x = np.array([[127, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.5, 126.5, -126.5, 0.49, 0.51]], np.float16)
    q, sx = oracle.smooth_quant_act(x, None)
    assert sx[0] == 1.0
    assert q[0].tolist() == [127, 0, 2, 2, 0, -2, -2, 4, 126, -126, 0, 1]


def test_act_quant_integer_identity_and_zero_row():
    rng = np.random.default_rng(1)
    X = rng.integers(-127, 128, size=(9, 64)).astype(np.float16)
    X[:, 0] = 127
    X[4] = 0
    q, sx = oracle.smooth_quant_act(X, None)
    keep = np.arange(9) != 4
    assert np.array_equal(q[keep], X[keep].astype(np.int8)) and np.all(sx[keep] == 1.0)
    assert np.all(q[4] == 0) and sx[4] == 0.0


def test_act_quant_divides_by_s_per_channel():
    # x/s = [127, 100] -> scale 1; a multiply, or s indexed by token, gives other codes
    X = np.array([[254, 100], [-127, 200]], np.float16)
    s = np.array([2, 1], F32)
    q, sx = oracle.smooth_quant_act(X, s)
    assert q.tolist() == [[127, 100], [-40, 127]]  # row 1: y = [-63.5, 200], scale 200/127
    assert sx[0] == 1.0 and sx[1] == F32(200) / F32(127)
    assert q[1, 0] == int(np.rint(F32(-63.5) / sx[1]))


def test_act_quant_power_of_two_s_equals_prescaled_input():
    X = _acts(2, 17, 96)
    e = np.random.default_rng(2).integers(-3, 4, 96)
    s = (2.0 ** e).astype(F32)
    q1, sx1 = oracle.smooth_quant_act(X, s)
    Xs = (X.astype(F32) / s).astype(np.float16)  # exact: power-of-two scaling, no overflow/underflow here
    assert np.array_equal(Xs.astype(F32), X.astype(F32) / s)
    q2, sx2 = oracle.smooth_quant_act(Xs, None)
    assert np.array_equal(q1, q2) and np.array_equal(sx1, sx2)


def test_act_quant_error_bound_and_range():
    X = _acts(3, 64, 512, n_outlier=4)
    s = np.exp(np.random.default_rng(3).normal(0, 1, 512)).astype(F32)
    q, sx = oracle.smooth_quant_act(X, s)
    y = (X.astype(F32) / s)  # numpy binary32 division is IEEE
    assert q.min() >= -127 and q.max() <= 127
    err = np.abs(y.astype(np.float64) - q.astype(np.float64) * sx[:, None].astype(np.float64))
    assert np.all(err <= sx[:, None].astype(np.float64) / 2 * (1 + 2.0 ** -21))
    # every non-zero row reaches +-127 at its absmax, and the scale is absmax/127 in binary32
    a = np.abs(y).max(axis=1)
    assert np.array_equal(sx, a / F32(127))
    j = np.abs(y).argmax(axis=1)
    assert np.all(np.abs(q[np.arange(64), j]) == 127)


def test_act_quant_matches_numpy_binary32_recomputation():
    X = _acts(4, 40, 300)
    s = np.exp(np.random.default_rng(4).normal(0, 1, 300)).astype(F32)
    q, sx = oracle.smooth_quant_act(X, s)
    y = X.astype(F32) / s
    sc = np.abs(y).max(axis=1) / F32(127)
    ref = np.clip(np.rint(y / sc[:, None]), -127, 127).astype(np.int8)
    assert np.array_equal(q, ref) and np.array_equal(sx, sc)


# ----------------------------------------------------------------- O0 / O2 offline side
def test_smoothing_vector_closed_forms():
    ax = np.array([4, 16, 9, 0, 5, 1e12, 1e-12], F32)
    aw = np.array([1, 4, 0.25, 3, 0, 1e-12, 1e12], F32)
    s = oracle.smoothing_vector(ax, aw, 0.5)
    assert s.tolist() == [2.0, 2.0, 6.0, 1.0, 1.0, F32(1e5), F32(1e-5)]
    assert np.array_equal(oracle.smoothing_vector(ax[:3], aw[:3], 1.0), ax[:3])          # e = 1: s = s_X
    assert np.array_equal(oracle.smoothing_vector(ax[:3], aw[:3], 0.0), 1 / aw[:3])      # e = 0: weight only
    assert np.array_equal(oracle.smoothing_vector(ax[:3], None, 0.5), np.array([2, 4, 3], F32))  # Eq. 3 form
    # general exponent against binary64 pow
    rng = np.random.default_rng(5)
    ax, aw = rng.uniform(0.1, 300, 100).astype(F32), rng.uniform(0.01, 1, 100).astype(F32)
    ref = (ax.astype(np.float64) ** 0.3 / aw.astype(np.float64) ** 0.7).astype(F32)
    assert np.array_equal(oracle.smoothing_vector(ax, aw, 0.3), ref)


def test_absmax_reductions_axes():
    X = np.array([[1, -7, 2], [-3, 4, 0.5]], np.float16)
    assert oracle.col_absmax_f16(X).tolist() == [3, 7, 2]          # over tokens, per channel
    W = np.array([[1, -9], [0.5, 0.25], [-2, 1]], F32)
    assert oracle.row_absmax_f32(W).tolist() == [9, 0.5, 2]        # over outputs, per input channel
    assert oracle.row_absmax_f32(W, np.array([1, 1, 1], F32)).tolist() == [9, 1, 2]  # folds into running max


def test_weight_quant_scale_axis_and_smoothing_multiplies():
    # column 0 has absmax 127 after smoothing, column 1 absmax 12.7: scales on the OUTPUT channel
    W = np.array([[63.5, 1.0], [-100, 12.7]], F32)
    s = np.array([2, 1], F32)  # W' = diag(s) W = [[127, 2], [-100, 12.7]]
    Wq, sw = oracle.quant_weight(W, s)
    assert sw[0] == 1.0 and sw[1] == F32(12.7) / F32(127)
    assert Wq[:, 0].tolist() == [127, -100]
    assert Wq[:, 1].tolist() == [20, 127]
    # zero column
    Wq, sw = oracle.quant_weight(np.array([[1, 0], [2, 0]], F32), None)
    assert sw[1] == 0 and Wq[:, 1].tolist() == [0, 0] and Wq[:, 0].tolist() == [64, 127]


def test_weight_quant_error_bound():
    W = hi.gaussian_weight(6, 0, 300, 70)
    s = np.exp(np.random.default_rng(6).normal(0, 1, 300)).astype(F32)
    Wq, sw = oracle.quant_weight(W, s)
    Ws = (s[:, None] * W)
    err = np.abs(Ws.astype(np.float64) - Wq.astype(np.float64) * sw[None, :].astype(np.float64))
    assert np.all(err <= sw[None, :].astype(np.float64) / 2 * (1 + 2.0 ** -21))
    assert np.array_equal(sw, np.abs(Ws).max(axis=0) / F32(127))
    assert np.all(np.abs(Wq).max(axis=0) == 127)


def test_smoothing_invariance_fp64():
    # X W = (X diag(s)^-1)(diag(s) W): the identity behind Eq. 1 / Algorithm 1 step 1
    X = _acts(7, 20, 128).astype(np.float64)
    W = hi.gaussian_weight(7, 0, 128, 48).astype(np.float64)
    s = offline.quantize_linear(X.astype(np.float16), W.astype(F32))[0].astype(np.float64)
    a, b = X @ W, (X / s[None, :]) @ (s[:, None] * W)
    assert np.max(np.abs(a - b)) <= 1e-12 * np.max(np.abs(a))


# ----------------------------------------------------------------- O3 GEMM
def test_gemm_brute_force_tiny():
    rng = np.random.default_rng(8)
    for T, K, N in [(1, 1, 1), (2, 3, 5), (5, 8, 3), (8, 7, 8)]:
        q = rng.integers(-127, 128, (T, K)).astype(np.int8)
        W = rng.integers(-127, 128, (K, N)).astype(np.int8)
        acc = oracle.gemm_i8(q, W)
        for t, n in itertools.product(range(T), range(N)):
            assert acc[t, n] == sum(int(q[t, k]) * int(W[k, n]) for k in range(K))


def test_gemm_not_symmetric_inputs_vs_numpy_int64():
    rng = np.random.default_rng(9)
    q = rng.integers(-127, 128, (13, 257)).astype(np.int8)
    W = rng.integers(-127, 128, (257, 31)).astype(np.int8)
    assert np.array_equal(oracle.gemm_i8(q, W), (q.astype(np.int64) @ W.astype(np.int64)).astype(np.int32))


def test_gemm_extreme_accumulators():
    K = 16384
    q = np.full((2, K), 127, np.int8)
    q[1] = -127
    W = np.full((K, 3), 127, np.int8)
    W[:, 1] = -127
    W[:, 2] = 1
    acc = oracle.gemm_i8(q, W)
    m = 127 * 127 * K
    assert acc.tolist() == [[m, -m, 127 * K], [-m, m, -127 * K]]


# ----------------------------------------------------------------- O4 epilogue, O1..O4 chain
def test_epilogue_scale_orientation_relu_and_rounding():
    acc = np.array([[1, -1, 3], [2, 5, -7]], np.int32)
    sx = np.array([1, 2], F32)         # per token (row)
    sw = np.array([1, 10, 100], F32)   # per output channel (column)
    Y = oracle.epilogue(acc, sx, sw, "none").astype(F32)
    assert Y.tolist() == [[1, -10, 300], [4, 100, -1400]]
    Yr = oracle.epilogue(acc, sx, sw, "relu").astype(F32)
    assert Yr.tolist() == [[1, 0, 300], [4, 100, 0]]
    # binary16 rounding (2049 -> 2048, 2051 -> 2052: ties to even) and overflow to inf
    Y = oracle.epilogue(np.array([[2049, 2051, 70000, -70000]], np.int32), np.ones(1, F32), np.ones(4, F32))
    assert Y.astype(F32).tolist() == [[2048, 2052, np.inf, -np.inf]]


def test_linear_integer_closed_form():
    # integer X and W' with absmax 127 and s = 1: both scales are 1, Y = fp16(exact product)
    rng = np.random.default_rng(10)
    X = rng.integers(-5, 6, (6, 32)).astype(np.float16)
    X[:, 0] = 127
    W = rng.integers(-4, 5, (32, 10)).astype(F32)
    W[0, :] = 127
    Wq, sw = oracle.quant_weight(W, None)
    assert np.all(sw == 1) and np.array_equal(Wq, W.astype(np.int8))
    Y, acc, q, sx = oracle.w8a8_linear(X, None, Wq, sw, "none", full=True)
    exact = X.astype(np.int64) @ W.astype(np.int64)
    assert np.array_equal(acc, exact)
    assert np.array_equal(Y, exact.astype(np.float16))


def _apriori_bound(X, s, W, sx, sw):
    """Per-output bound on |dequant(acc) - X W| from half-a-step errors of both operands."""
    y = np.abs(X.astype(np.float64) / s[None, :])
    w = np.abs(s[:, None].astype(np.float64) * W.astype(np.float64))
    sx = sx.astype(np.float64)[:, None]
    sw = sw.astype(np.float64)[None, :]
    K = y.shape[1]
    return y.sum(1, keepdims=True) * sw / 2 + sx / 2 * w.sum(0, keepdims=True) + K * sx * sw / 4


def test_linear_within_apriori_bound_of_exact_product():
    wl = hi.OPT125M_LINEAR
    X, _, _ = hi.hidden_states(wl.seed, wl.T, wl.K, wl.n_outlier, wl.mult)
    W = hi.gaussian_weight(wl.seed, 0, wl.K, 256)
    s, Wq, sw = offline.quantize_linear(X, W)
    Y, acc, q, sx = oracle.w8a8_linear(X, s, Wq, sw, "none", full=True)
    exact = X.astype(np.float64) @ W.astype(np.float64)
    bound = _apriori_bound(X, s, W, sx, sw)
    half_ulp = np.spacing(np.abs(Y).astype(np.float16)).astype(np.float64)
    err = np.abs(Y.astype(np.float64) - exact)
    assert np.all(err <= bound * (1 + 1e-5) + half_ulp)
    # and it is a good approximation, not merely a bounded one
    assert np.sqrt(np.mean(err ** 2)) < 0.02 * np.sqrt(np.mean(exact ** 2))


def test_smoothing_reduces_joint_quantisation_error():
    # Table I's ordering RTN > Smooth in proxy form: with outlier channels, alpha = 0.5 beats s = 1
    X, _, _ = hi.hidden_states(11, 64, 512, 4, 50.0)
    W = hi.gaussian_weight(11, 0, 512, 128)
    exact = X.astype(np.float64) @ W.astype(np.float64)
    s, Wq, sw = offline.quantize_linear(X, W)
    Wq1, sw1 = oracle.quant_weight(W, None)
    mse_s = np.mean((oracle.w8a8_linear(X, s, Wq, sw).astype(np.float64) - exact) ** 2)
    mse_1 = np.mean((oracle.w8a8_linear(X, None, Wq1, sw1).astype(np.float64) - exact) ** 2)
    assert mse_s < 0.5 * mse_1


# ----------------------------------------------------------------- O5 router
def test_router_properties_and_closed_form():
    rng = np.random.default_rng(12)
    logits = (rng.standard_normal((500, 8)) * 3).astype(np.float16)
    idx, gw = oracle.route_top2(logits)
    l = logits.astype(np.float64)
    order = np.argsort(-l, axis=1, kind="stable")
    assert np.array_equal(idx, order[:, :2].astype(np.int32))
    assert np.all(idx[:, 0] != idx[:, 1])
    assert np.all(gw[:, 0] >= gw[:, 1]) and np.all(gw > 0)
    assert np.max(np.abs(gw.sum(1) - 1)) <= 2 ** -22
    l0 = np.take_along_axis(l, idx[:, :1].astype(np.int64), 1)[:, 0]
    l1 = np.take_along_axis(l, idx[:, 1:].astype(np.int64), 1)[:, 0]
    g0 = 1 / (1 + np.exp(l1 - l0))  # softmax renormalised over two = logistic of the logit gap
    assert np.max(np.abs(gw[:, 0] - g0)) < 5e-7


def test_router_ties_pick_lowest_index():
    logits = np.array([[1, 1, 1, 1], [0, 2, 2, 1], [3, 0, 3, 3], [-1, -1, 5, -1], [0, 0, 0, 7]], np.float16)
    idx, gw = oracle.route_top2(logits)
    assert idx.tolist() == [[0, 1], [1, 2], [0, 2], [2, 0], [3, 0]]
    assert gw[0].tolist() == [0.5, 0.5] and gw[1].tolist() == [0.5, 0.5]


# ----------------------------------------------------------------- O6 permutation
def test_permutation_properties():
    rng = np.random.default_rng(13)
    T, E = 301, 8
    idx = np.stack([rng.permutation(E)[:2] for _ in range(T)]).astype(np.int32)
    idx[idx == 5] = 4  # expert 5 gets nothing; duplicates in a token are still legal input here
    counts, offsets, perm, inv = oracle.permute(idx, E)
    flat = idx.ravel()
    assert np.array_equal(counts, np.bincount(flat, minlength=E))
    assert counts[5] == 0 and counts.sum() == 2 * T
    assert np.array_equal(offsets, np.concatenate([[0], np.cumsum(counts)]))
    assert np.array_equal(np.sort(perm), np.arange(2 * T))
    assert np.array_equal(inv[perm], np.arange(2 * T)) and np.array_equal(perm[inv], np.arange(2 * T))
    for e in range(E):
        seg = perm[offsets[e]:offsets[e + 1]]
        assert np.all(flat[seg] == e) and np.all(np.diff(seg) > 0)  # grouped by expert, stable inside
    assert np.array_equal(perm, np.argsort(flat, kind="stable"))


# ----------------------------------------------------------------- O7 / O8 routed expert FFN
def _float_moe_reference(X, weights, idx, gw):
    """Unquantised binary64 top-2 SwiGLU MoE."""
    X = X.astype(np.float64)
    out = np.zeros((X.shape[0], weights[0][2].shape[1]))
    for t in range(X.shape[0]):
        for k in range(2):
            w1, w3, w2 = (w.astype(np.float64) for w in weights[idx[t, k]])
            g, u = X[t] @ w1, X[t] @ w3
            out[t] += gw[t, k] * ((g / (1 + np.exp(-g)) * u) @ w2)
    return out


def test_moe_close_to_float_reference():
    m = offline.small_moe(seed=14, T=24, H=128, I=320, E=8)
    out = oracle.moe_ffn(m["X"], m["idx"], m["gw"], m["s_in"], m["experts"]).astype(np.float64)
    ref = _float_moe_reference(m["X"], m["weights"], m["idx"], m["gw"].astype(np.float64))
    rel = np.sqrt(np.mean((out - ref) ** 2) / np.mean(ref ** 2))
    assert rel < 0.03, rel


def _chain_from_pinned_pieces(X, idx, gw, s_in, experts):
    """The same layer assembled in Python from the separately pinned pieces."""
    T, H = X.shape
    q, sx = oracle.smooth_quant_act(X, s_in)
    out = np.zeros((T, H), np.float16)
    for t in range(T):
        ys = []
        for k in range(2):
            ex = experts[idx[t, k]]
            a1, a3 = oracle.gemm_i8(q[t:t + 1], ex.w1)[0], oracle.gemm_i8(q[t:t + 1], ex.w3)[0]
            g = (a1.astype(F32) * sx[t]) * ex.sw1
            u = (a3.astype(F32) * sx[t]) * ex.sw3
            silu = g / (F32(1) + oracle.exp_spec(-g))
            h = oracle.float_to_half(silu * u)
            y = oracle.w8a8_linear(h[None, :], ex.s_mid, ex.w2, ex.sw2)[0]
            ys.append(y.astype(F32))
        out[t] = oracle.float_to_half(gw[t, 0] * ys[0] + gw[t, 1] * ys[1])
    return out


def test_moe_equals_chain_of_pinned_pieces_and_token_subset():
    m = offline.small_moe(seed=15, T=19, H=128, I=192, E=8)
    X, idx, gw, s_in, ex = m["X"], m["idx"], m["gw"], m["s_in"], m["experts"]
    out, mid, hq, sh, y = oracle.moe_ffn(X, idx, gw, s_in, ex, dumps=True)
    assert np.array_equal(out.view(np.uint16), _chain_from_pinned_pieces(X, idx, gw, s_in, ex).view(np.uint16))
    tok = np.array([17, 3, 3, 0], np.int32)
    sub, mid_s, hq_s, sh_s, y_s = oracle.moe_ffn(X, idx, gw, s_in, ex, tokens=tok, dumps=True)
    assert np.array_equal(sub.view(np.uint16), out[tok].view(np.uint16))
    rows = (2 * tok[:, None] + np.arange(2)[None, :]).ravel()
    assert np.array_equal(mid_s.view(np.uint16), mid[rows].view(np.uint16))
    assert np.array_equal(hq_s, hq[rows]) and np.array_equal(sh_s, sh[rows])
    assert np.array_equal(y_s.view(np.uint16), y[rows].view(np.uint16))
    # the requantised intermediate is O1 applied to the fp16 intermediate with the expert's s_mid
    r = 5
    e = idx.ravel()[r]
    q_r, s_r = oracle.smooth_quant_act(mid[r:r + 1], ex[e].s_mid)
    assert np.array_equal(q_r[0], hq[r]) and s_r[0] == sh[r]


def test_moe_identical_experts_reduce_to_dense_ffn():
    # with the same weights in every expert the gate weights (g0 + g1 = 1) drop out
    m = offline.small_moe(seed=16, T=11, H=128, I=192, E=4)
    ex0 = m["experts"][0]
    same = [ex0] * 4
    out, _, _, _, y = oracle.moe_ffn(m["X"], m["idx"], m["gw"], m["s_in"], same, dumps=True)
    assert np.array_equal(y[0::2].view(np.uint16), y[1::2].view(np.uint16))
    dense = y[0::2].astype(np.float64)
    assert np.max(np.abs(out.astype(np.float64) - dense)) <= np.max(np.spacing(np.abs(y[0::2]))) * 1.01


def test_moe_two_experts_every_token_visits_both():
    m = offline.small_moe(seed=17, T=9, H=128, I=192, E=2)
    assert np.all(np.sort(m["idx"], axis=1) == np.array([0, 1]))
    out = oracle.moe_ffn(m["X"], m["idx"], m["gw"], m["s_in"], m["experts"]).astype(np.float64)
    ref = _float_moe_reference(m["X"], m["weights"], m["idx"], m["gw"].astype(np.float64))
    assert np.sqrt(np.mean((out - ref) ** 2) / np.mean(ref ** 2)) < 0.03


def test_mid_absmax_matches_dumped_intermediate():
    m = offline.small_moe(seed=18, T=21, H=128, I=192, E=8)
    _, mid, _, _, _ = oracle.moe_ffn(m["X"], m["idx"], m["gw"], m["s_in"], m["experts"], dumps=True)
    ax = oracle.moe_mid_absmax(m["X"], m["idx"], m["s_in"], m["experts"])
    flat = m["idx"].ravel()
    for e in range(8):
        rows = np.abs(mid[flat == e].astype(F32))
        ref = rows.max(axis=0) if rows.size else np.zeros(192, F32)
        assert np.array_equal(ax[e], ref)


# ----------------------------------------------------------------- adaptive smoothing (Algorithm 1 step 1)
def test_matmul_f64_is_the_library_product():
    rng = np.random.default_rng(21)
    X = (rng.standard_normal((13, 70)) * 3).astype(np.float16)
    W = rng.standard_normal((70, 29)).astype(F32)
    ref = X.astype(np.float64) @ W.astype(np.float64)  # library routine; shapes are not square: a transpose fails
    got = oracle.matmul_f64(X, W)
    assert got.shape == (13, 29)
    assert np.allclose(got, ref, rtol=1e-13, atol=1e-13)
    # exactly representable case: small integers give an exact product
    Xi = rng.integers(-8, 9, (5, 16)).astype(np.float16)
    Wi = rng.integers(-8, 9, (16, 7)).astype(F32)
    assert np.array_equal(oracle.matmul_f64(Xi, Wi), (Xi.astype(np.int64) @ Wi.astype(np.int64)).astype(np.float64))


def test_mse_f64_closed_forms():
    T, N = 6, 10
    Y = np.ones((T, N), np.float16)
    assert oracle.mse_f64(Y, np.full((T, N), 0.5)) == 0.25            # every difference is 1/2
    ref = np.ones((T, N)) - np.arange(T)[:, None]                      # row t is off by t
    assert oracle.mse_f64(Y, ref) == sum(t * t for t in range(T)) / T
    ref2 = np.ones((T, N))
    ref2[2, 3] = -2.0                                                  # a single entry off by 3
    assert oracle.mse_f64(Y, ref2) == 9.0 / (T * N)
    assert oracle.mse_f64(Y, np.ones((T, N))) == 0.0


def _flat_magnitude_case(seed, T=24, K=128, N=40):
    """Activations whose every channel has absmax exactly 4 and weights whose every input
    channel has absmax exactly 1/4: the smoothing vector is then a power of two for
    e in {0, 1/2, 1}, and dividing / multiplying by a power of two is exact, so the quantised
    layer produces bit-identical outputs for those exponents."""
    rng = np.random.default_rng(seed)
    X = rng.uniform(-3.9, 3.9, (T, K)).astype(np.float16)
    X[rng.integers(0, T, K), np.arange(K)] = np.float16(4.0) * rng.choice([-1, 1], K).astype(np.float16)
    W = rng.uniform(-0.24, 0.24, (K, N)).astype(F32)
    W[np.arange(K), rng.integers(0, N, K)] = F32(0.25)
    return X, W


def test_smoothing_search_ties_keep_the_first_exponent():
    X, W = _flat_magnitude_case(22)
    grid = [0.0, 0.5, 1.0]
    losses, best, s = oracle.smoothing_search(X, W, grid, use_weight=False)
    assert losses[0] == losses[1] == losses[2] and losses[0] > 0   # s = 1, 2, 4: the same bits come out
    assert best == 0 and np.array_equal(s, np.ones(128, F32))
    # balanced form: ax^e / aw^(1-e) = 4^e * 4^(1-e) = 4 whatever e is
    losses_b, best_b, s_b = oracle.smoothing_search(X, W, [0.25, 0.5, 0.75], use_weight=True)
    assert losses_b[0] == losses_b[1] == losses_b[2] == losses[0]
    assert best_b == 0 and np.array_equal(s_b, np.full(128, 4.0, F32))
    # put a better candidate last and a worse one first: the order of the grid must not matter
    # for which loss is minimal, and the strict comparison keeps the first of the equal ones
    losses_r, best_r, _ = oracle.smoothing_search(X, W, [1.0, 0.0, 0.5], use_weight=False)
    assert best_r == 0 and np.array_equal(losses_r, losses)


def test_smoothing_search_finds_the_minimum_on_outlier_activations():
    X, _, _ = hi.hidden_states(23, 96, 512, 4, 50.0)
    W = hi.gaussian_weight(23, 0, 512, 160)
    grid = [i / 10 for i in range(11)]
    losses, best, s = oracle.smoothing_search(X, W, grid)
    assert best == int(np.argmin(losses))                     # numpy's argmin is also first-of-equals
    assert 0 < best < 10                                      # an interior exponent (outliers need some, not full, migration)
    assert losses[best] < 0.5 * losses[0]                     # and it beats no smoothing clearly
    assert np.array_equal(s, oracle.smoothing_vector(oracle.col_absmax_f16(X), None, grid[best]))
    # the loss of the e = 0 candidate is that of the unsmoothed layer, computed independently
    Wq1, sw1 = oracle.quant_weight(W, None)
    exact = X.astype(np.float64) @ W.astype(np.float64)
    mse_1 = np.mean((oracle.w8a8_linear(X, None, Wq1, sw1).astype(np.float64) - exact) ** 2)
    assert np.isclose(losses[0], mse_1, rtol=1e-12)
    # the balanced form at e = 1/2 is the fixed-alpha recipe used for the other workloads
    s_half, Wq, sw = offline.quantize_linear(X, W, 0.5)
    mse_h = np.mean((oracle.w8a8_linear(X, s_half, Wq, sw).astype(np.float64) - exact) ** 2)
    losses_b, _, _ = oracle.smoothing_search(X, W, [0.5], use_weight=True)
    assert np.isclose(losses_b[0], mse_h, rtol=1e-12)


# ----------------------------------------------------------------- Hessian-aware weight quantisation (Eq. 4-6)
def _correlated_activations(seed, T, K, rank):
    """Activations with strong correlation between channels (a few latent factors + noise)."""
    rng = np.random.default_rng(seed)
    Z = rng.standard_normal((T, rank))
    A = rng.standard_normal((rank, K))
    return (Z @ A + 0.1 * rng.standard_normal((T, K))).astype(np.float16)


def test_hessian_is_twice_the_gram_matrix_plus_damping():
    X = _correlated_activations(31, 90, 48, 6)
    X[:, 7] = 0                                            # a channel that never fires
    s = np.exp(np.random.default_rng(31).normal(0, 0.5, 48)).astype(F32)
    H = oracle.hessian(X, s, 0.01)
    Xs = (X.astype(F32) / s).astype(np.float64)            # the binary32 division of the activation path
    G = 2.0 * Xs.T @ Xs                                    # library product
    G[7, 7] = 1.0
    G += 0.01 * np.mean(np.diag(G)) * np.eye(48)
    assert np.allclose(H, G, rtol=1e-12, atol=1e-12) and np.array_equal(H, H.T)
    assert np.allclose(oracle.hessian(X, None, 0.0)[np.arange(48) != 7][:, np.arange(48) != 7],
                       (2.0 * X.astype(np.float64).T @ X.astype(np.float64))[np.arange(48) != 7][:, np.arange(48) != 7],
                       rtol=1e-12)


def test_inverse_cholesky_upper_against_library_routines():
    X = _correlated_activations(32, 150, 40, 5)
    H = oracle.hessian(X, None, 0.01)
    U = oracle.inverse_cholesky_upper(H)
    assert np.array_equal(U, np.triu(U)) and np.all(np.diag(U) > 0)
    assert np.allclose(U.T @ U @ H, np.eye(40), atol=1e-8)
    assert np.allclose(U, np.linalg.cholesky(np.linalg.inv(H)).T, rtol=1e-8, atol=1e-12)
    # row i of U is row i of the inverse Hessian of the remaining channels i.., up to the factor U_ii
    for i in (0, 3, 17, 39):
        HF_inv = np.linalg.inv(H[i:, i:])
        assert np.allclose(U[i, i:] * U[i, i], HF_inv[0], rtol=1e-7, atol=1e-12)
    with pytest.raises(ValueError):
        oracle.inverse_cholesky_upper(np.array([[1.0, 2.0], [2.0, 1.0]]))   # indefinite


def test_gptq_two_channel_closed_form():
    # K = 2, one output channel: Eq. 6 by hand with the explicit inverse
    H = np.array([[4.0, 1.0], [1.0, 3.0]])
    U = oracle.inverse_cholesky_upper(H)
    W = np.array([[0.30], [-1.27]], F32)                   # absmax 1.27 -> scale 0.01
    Wq, sw = oracle.gptq(W, None, U)
    scale = float(sw[0])
    assert np.isclose(scale, 1.27 / 127)
    q0 = np.rint(np.float64(W[0, 0]) / scale)
    Hinv = np.linalg.inv(H)
    w1 = np.float64(W[1, 0]) - (np.float64(W[0, 0]) - q0 * scale) / Hinv[0, 0] * Hinv[1, 0]
    assert Wq[0, 0] == q0 and Wq[1, 0] == np.clip(np.rint(w1 / scale), -127, 127)
    # a case where the compensation moves a code.  A third, uncorrelated channel pins the scale to 0.01;
    # channel 0 rounds 1.49 -> 1 and leaves +0.0049, of which -Hinv10/Hinv00 = 1/3 moves to channel 1:
    # 5.40 + 0.163 = 5.563 rounds to 6, where plain rounding gives 5
    H3 = np.array([[4.0, 1.0, 0.0], [1.0, 3.0, 0.0], [0.0, 0.0, 2.0]])
    W3 = np.array([[0.0149], [0.0540], [1.27]], F32)
    Wq3, sw3 = oracle.gptq(W3, None, oracle.inverse_cholesky_upper(H3))
    assert np.isclose(float(sw3[0]), 0.01)
    assert Wq3[:, 0].tolist() == [1, 6, 127]
    assert oracle.quant_weight(W3, None)[0][:, 0].tolist() == [1, 5, 127]


def test_gptq_equals_plain_rounding_for_uncorrelated_channels():
    # orthogonal activation columns: H is diagonal, U is diagonal, nothing is compensated
    rng = np.random.default_rng(33)
    Q, _ = np.linalg.qr(rng.standard_normal((64, 32)))
    X = np.zeros((64, 32), np.float16)
    X[np.arange(32), np.arange(32)] = (rng.uniform(1, 3, 32)).astype(np.float16)   # one token per channel
    W = rng.standard_normal((32, 24)).astype(F32)
    s = np.exp(rng.normal(0, 0.3, 32)).astype(F32)
    Wq, sw = oracle.hessian_quant_weight(X, W, s)
    Wr, swr = oracle.quant_weight(W, s)
    assert np.array_equal(Wq, Wr) and np.array_equal(sw, swr)


def test_gptq_matches_the_definition_with_explicit_remaining_inverse():
    # Eq. 5-6 verbatim on a tiny layer: at every step the inverse Hessian of the channels not yet
    # quantised is recomputed with a library inverse; the codes must agree
    X = _correlated_activations(34, 60, 12, 3)
    W = (np.random.default_rng(34).standard_normal((12, 5)) * 0.05).astype(F32)
    H = oracle.hessian(X, None, 0.01)
    Wq, sw = oracle.gptq(W, None, oracle.inverse_cholesky_upper(H))
    Wd = W.astype(np.float64).copy()
    ref = np.zeros((12, 5), np.int8)
    for i in range(12):
        HF_inv = np.linalg.inv(H[i:, i:])                  # F = {i, ..., 11}
        for n in range(5):
            q = np.clip(np.rint(Wd[i, n] / float(sw[n])), -127, 127)
            ref[i, n] = q
            delta = -(Wd[i, n] - q * float(sw[n])) / HF_inv[0, 0] * HF_inv[:, 0]
            Wd[i + 1:, n] += delta[1:]
    assert np.array_equal(Wq, ref)


def test_gptq_lowers_the_output_error_on_correlated_activations():
    # the objective of Eq. 4 against plain rounding (Table I's ordering of GPTQ-style vs RTN in proxy form)
    X = _correlated_activations(35, 256, 128, 8)
    W = hi.gaussian_weight(35, 0, 128, 96)
    Wq, sw = oracle.hessian_quant_weight(X, W, None)
    Wr, swr = oracle.quant_weight(W, None)
    Xd, Wd = X.astype(np.float64), W.astype(np.float64)
    err_g = np.sum((Xd @ Wd - Xd @ (Wq * sw.astype(np.float64))) ** 2)
    err_r = np.sum((Xd @ Wd - Xd @ (Wr * swr.astype(np.float64))) ** 2)
    assert err_g < 0.6 * err_r
    assert np.array_equal(sw, swr) and np.abs(Wq.astype(int)).max() <= 127


# ----------------------------------------------------------------- asymmetric activations
def test_asym_codes_reconstruct_within_one_step_and_use_the_whole_range():
    rng = np.random.default_rng(41)
    X = (rng.standard_normal((40, 96)) * 2 + 1.5).astype(np.float16)   # skewed rows
    X[3] = 0
    X[4] = np.abs(X[4])                                                 # a non-negative row
    s = np.exp(rng.normal(0, 0.4, 96)).astype(F32)
    q, sx, zp = oracle.asym_quant_act(X, s)
    y = X.astype(F32) / s
    rec = (q.astype(np.int32) - zp[:, None]).astype(np.float64) * sx[:, None].astype(np.float64)
    # rounding the zero point moves the grid by at most half a step, rounding the code by another half
    assert np.all(np.abs(rec - y) <= sx[:, None].astype(np.float64) * (1 + 1e-6))
    live = sx > 0
    neg = live & (y.min(axis=1) < 0)
    assert np.all(q[neg].min(axis=1) == 0) and np.all(q[live].max(axis=1) >= 254)
    assert sx[3] == 0 and zp[3] == 0 and not q[3].any()
    assert zp[4] == 0 and np.isclose(sx[4], y[4].max() / 255, rtol=1e-6)        # range starts at 0
    assert np.all((zp >= 0) & (zp <= 255))


def test_asym_integer_data_is_exact():
    # integers in [-100, 155]: range 255, scale 1, zero point 100, codes = x + 100, exact accumulators
    rng = np.random.default_rng(42)
    X = rng.integers(-100, 156, (9, 64)).astype(np.float16)
    X[:, 0], X[:, 1] = -100, 155
    Wq = rng.integers(-127, 128, (64, 24)).astype(np.int8)
    q, sx, zp = oracle.asym_quant_act(X, None)
    assert np.all(sx == 1) and np.all(zp == 100) and np.array_equal(q.astype(int), X.astype(int) + 100)
    acc = oracle.asym_gemm(q, zp, Wq)
    assert np.array_equal(acc, X.astype(np.int64) @ Wq.astype(np.int64))
    Y = oracle.w8a8_linear_asym(X, None, Wq, np.full(24, 2.0 ** -8, F32))
    assert np.array_equal(Y, ((X.astype(np.int64) @ Wq.astype(np.int64)) * 2.0 ** -8).astype(np.float16))


def test_asym_beats_symmetric_on_one_sided_activations():
    # post-ReLU-like inputs: the symmetric grid wastes its negative half
    X, _, _ = hi.hidden_states(43, 64, 256, 2, 10.0)
    X = np.maximum(X, 0).astype(np.float16)
    W = hi.gaussian_weight(43, 0, 256, 64)
    Wq, sw = oracle.quant_weight(W, None)
    exact = X.astype(np.float64) @ (Wq.astype(np.float64) * sw.astype(np.float64))   # isolate the activation error
    e_sym = np.mean((oracle.w8a8_linear(X, None, Wq, sw).astype(np.float64) - exact) ** 2)
    e_asym = np.mean((oracle.w8a8_linear_asym(X, None, Wq, sw).astype(np.float64) - exact) ** 2)
    assert e_asym < 0.4 * e_sym        # twice the resolution: about a quarter of the squared error


# ----------------------------------------------------------------- offload scheduler (Section III.C)
def test_lru_trace_textbook_reference_string():
    # the classic 20-reference string with 3 frames: 12 misses under LRU (15 under FIFO, 9 under OPT)
    refs = [7, 0, 1, 2, 0, 3, 0, 4, 2, 3, 0, 3, 2, 1, 2, 0, 1, 7, 0, 1]
    hits, cache = oracle.lru_trace(refs, 3)
    assert len(hits) - sum(hits) == 12
    assert hits[:8] == [False, False, False, False, True, False, True, False]
    assert cache == [7, 0, 1]                      # least recently used first
    # capacity >= distinct keys: only compulsory misses; capacity 1: a hit only on immediate repeats
    assert sum(oracle.lru_trace(refs, 6)[0]) == len(refs) - 6
    assert oracle.lru_trace([1, 1, 2, 2, 2, 1], 1)[0] == [False, True, False, True, True, False]
    # LRU differs from FIFO here: after 1 2 3 1 4, LRU evicted 2 (FIFO would have evicted 1)
    assert oracle.lru_trace([1, 2, 3, 1, 4], 3)[1] == [3, 1, 4]


def test_n_critical_is_the_break_even_batch():
    # T_CPU = n, T_sum = 10 + n/2: equal at n = 20, the GPU wins from 21 on
    assert oracle.n_critical(10.0, 1.0, 0.5) == 20
    assert oracle.n_critical(10.1, 1.0, 0.5) == 20 and oracle.n_critical(9.9, 1.0, 0.5) == 19
    assert oracle.n_critical(0.0, 1.0, 0.5) == 0      # free transfer: any batch goes to the GPU
    assert oracle.n_critical(5.0, 1.0, 1.0) is None   # the CPU is never slower
    for t_e, lc, lg in [(12.7, 0.9, 0.004), (3.0, 0.25, 0.125), (1e-3, 2.0, 1.0)]:
        n = oracle.n_critical(t_e, lc, lg)
        assert n * lc <= t_e + n * lg and (n + 1) * lc > t_e + (n + 1) * lg


def test_select_experts_worked_example():
    # one layer, 8 experts.  Paths (top-2 pairs at this layer) by frequency: (3,5) 40, (5,1) 30, (0,2) 5.
    paths = [[((0, 2), 5), ((3, 5), 40), ((5, 1), 30)]]
    freq = [[(0, 10), (1, 30), (2, 8), (3, 45), (4, 33), (5, 70), (6, 2), (7, 31)]]
    # stage I with top_k = 3: 3, 5 from the hottest path, then 5 (already in), 1 -> stop at three
    assert oracle.select_experts(1, 3, 0, paths, freq) == [[3, 5, 1]]
    # stage II adds by expert frequency, skipping what is in: 5 (in), 3 (in), 4, 7
    assert oracle.select_experts(1, 3, 2, paths, freq) == [[3, 5, 1, 4, 7]]
    # top_k = 2 stops inside the first path; equal frequencies keep input order
    assert oracle.select_experts(1, 2, 1, paths, [[(0, 9), (6, 9), (3, 9)]]) == [[3, 5, 0]]
    # layers are independent
    two = oracle.select_experts(2, 1, 1, [paths[0], [((7, 6), 1)]], [freq[0], [(6, 5), (2, 4)]])
    assert two == [[3, 5], [7, 6]]


# ----------------------------------------------------------------- input recipe sanity
def test_zipf_router_bias_reaches_target_popularity():
    wl = hi.MoeWorkload("zipf_small", 19, 2048, 256, 64, 8, "zipf")
    X, _, _ = hi.hidden_states(wl.seed, wl.T, wl.H)
    idx, _ = oracle.route_top2(hi.moe_logits(wl, X))
    share = np.bincount(idx.ravel(), minlength=8) / (2 * wl.T)
    assert np.max(np.abs(share - hi.zipf_shares(8))) < 0.02
    assert np.all(np.diff(share) < 0.01)


def test_outlier_channels_are_fixed_and_large():
    X, idx, mult = hi.hidden_states(1, 256, 4096)
    assert idx.size == 21 or idx.size == 20
    a = np.abs(X.astype(F32)).max(axis=0)
    rest = np.delete(a, idx)
    assert a[idx].min() > 3 * rest.max()
    X2, idx2, _ = hi.hidden_states(1, 64, 4096)
    assert np.array_equal(idx, idx2)


# ----------------------------------------------------------------- asymmetric codes inside the routed expert FFN
def _asym_chain_from_pinned_pieces(X, idx, gw, s_in, experts):
    """The asymmetric layer assembled in Python from the separately pinned pieces."""
    T, H = X.shape
    q, sx, zp = oracle.asym_quant_act(X, s_in)
    out = np.zeros((T, H), np.float16)
    mids, ys = [], []
    for t in range(T):
        y2 = []
        for k in range(2):
            ex = experts[idx[t, k]]
            a1 = oracle.asym_gemm(q[t:t + 1], zp[t:t + 1], ex.w1)[0]
            a3 = oracle.asym_gemm(q[t:t + 1], zp[t:t + 1], ex.w3)[0]
            g = (a1.astype(F32) * sx[t]) * ex.sw1
            u = (a3.astype(F32) * sx[t]) * ex.sw3
            h = oracle.float_to_half((g / (F32(1) + oracle.exp_spec(-g))) * u)
            y = oracle.w8a8_linear_asym(h[None, :], ex.s_mid, ex.w2, ex.sw2)[0]
            mids.append(h)
            ys.append(y)
            y2.append(y.astype(F32))
        out[t] = oracle.float_to_half(gw[t, 0] * y2[0] + gw[t, 1] * y2[1])
    return out, np.stack(mids), np.stack(ys)


def test_moe_asym_equals_chain_of_pinned_pieces_and_token_subset():
    m = offline.small_moe(seed=115, T=19, H=128, I=192, E=8)
    X, idx, gw, s_in, ex = m["X"], m["idx"], m["gw"], m["s_in"], m["experts"]
    out, mid, hq, sh, zh, y = oracle.moe_ffn_asym(X, idx, gw, s_in, ex, dumps=True)
    out_c, mid_c, y_c = _asym_chain_from_pinned_pieces(X, idx, gw, s_in, ex)
    assert np.array_equal(out.view(np.uint16), out_c.view(np.uint16))
    assert np.array_equal(mid.view(np.uint16), mid_c.view(np.uint16)) and np.array_equal(y.view(np.uint16), y_c.view(np.uint16))
    r = 7
    q_r, s_r, z_r = oracle.asym_quant_act(mid[r:r + 1], ex[idx.ravel()[r]].s_mid)
    assert np.array_equal(q_r[0], hq[r]) and s_r[0] == sh[r] and z_r[0] == zh[r]
    tok = np.array([17, 3, 3, 0], np.int32)
    sub, mid_s, hq_s, sh_s, zh_s, y_s = oracle.moe_ffn_asym(X, idx, gw, s_in, ex, tokens=tok, dumps=True)
    rows = (2 * tok[:, None] + np.arange(2)[None, :]).ravel()
    assert np.array_equal(sub.view(np.uint16), out[tok].view(np.uint16))
    assert np.array_equal(hq_s, hq[rows]) and np.array_equal(zh_s, zh[rows]) and np.array_equal(sh_s, sh[rows])
    assert np.array_equal(y_s.view(np.uint16), y[rows].view(np.uint16)) and np.array_equal(mid_s.view(np.uint16), mid[rows].view(np.uint16))


def test_moe_asym_exact_integer_case():
    """Integer tokens in [-100, 155] (scale 1, zero point 100, like the dense pin) and power-of-two weight scales:
    the gate/up values are exact integers / 2^k, so the intermediate must be silu(g) u to fp16 accuracy; the down
    accumulator is then pinned through the dumped codes: y = fp16((sum (hq - zh) w2) sh sw2) with exact integers."""
    rng = np.random.default_rng(116)
    T, H, I, E = 6, 64, 96, 4
    X = rng.integers(-100, 156, (T, H)).astype(np.float16)
    X[:, 0], X[:, 1] = -100, 155
    experts = []
    for e in range(E):
        experts.append(oracle.Expert(rng.integers(-127, 128, (H, I)).astype(np.int8), rng.integers(-127, 128, (H, I)).astype(np.int8),
                                     rng.integers(-127, 128, (I, H)).astype(np.int8), np.full(I, 2.0 ** -17, F32),
                                     np.full(I, 2.0 ** -16, F32), np.full(H, 2.0 ** -9, F32), np.ones(I, F32)))
    logits = rng.standard_normal((T, E)).astype(np.float16)
    idx, gw = oracle.route_top2(logits)
    out, mid, hq, sh, zh, y = oracle.moe_ffn_asym(X, idx, gw, np.ones(H, F32), experts, dumps=True)
    Xi = X.astype(np.int64)
    for r in range(2 * T):
        ex = experts[idx.ravel()[r]]
        g = (Xi[r // 2] @ ex.w1.astype(np.int64)) * 2.0 ** -17
        u = (Xi[r // 2] @ ex.w3.astype(np.int64)) * 2.0 ** -16
        ref = g / (1 + np.exp(-g)) * u
        assert np.all(np.abs(mid[r].astype(np.float64) - ref) <= np.spacing(np.abs(ref).astype(np.float16)).astype(np.float64))
        acc2 = (hq[r].astype(np.int64) - zh[r]) @ ex.w2.astype(np.int64)
        assert np.array_equal(y[r], ((acc2.astype(F32) * sh[r]) * ex.sw2).astype(np.float16))
        rec = (hq[r].astype(np.float64) - zh[r]) * sh[r]
        assert np.all(np.abs(rec - mid[r].astype(np.float64)) <= sh[r] * (1 + 1e-6))
    assert np.array_equal(out.view(np.uint16), oracle.combine(y, gw).view(np.uint16))


def test_moe_asym_identical_experts_reduce_to_dense_ffn_and_track_the_float_reference():
    m = offline.small_moe(seed=117, T=12, H=128, I=192, E=4)
    same = [m["experts"][0]] * 4
    out, _, _, _, _, y = oracle.moe_ffn_asym(m["X"], m["idx"], m["gw"], m["s_in"], same, dumps=True)
    assert np.array_equal(y[0::2].view(np.uint16), y[1::2].view(np.uint16))
    assert np.max(np.abs(out.astype(np.float64) - y[0::2].astype(np.float64))) <= np.max(np.spacing(np.abs(y[0::2]))) * 1.01
    out = oracle.moe_ffn_asym(m["X"], m["idx"], m["gw"], m["s_in"], m["experts"]).astype(np.float64)
    ref = _float_moe_reference(m["X"], m["weights"], m["idx"], m["gw"].astype(np.float64))
    assert np.sqrt(np.mean((out - ref) ** 2) / np.mean(ref ** 2)) < 0.03


# ----------------------------------------------------------------- the CPU side: floating point on dequantised weights
def test_dequantised_copy_and_fp_linear():
    rng = np.random.default_rng(120)
    Wq = rng.integers(-127, 128, (70, 33)).astype(np.int8)
    sw = np.exp(rng.normal(-5, 1, 33)).astype(F32)
    Wf = oracle.dequant_weight(Wq, sw)
    assert Wf.dtype == F32 and np.array_equal(Wf.astype(np.float64), (Wq.astype(np.float64) * sw.astype(np.float64)).astype(F32).astype(np.float64))
    # exact integer case: small integers, power-of-two smoothing entries -> the exact product
    Xi = rng.integers(-64, 65, (5, 70)).astype(F32)
    s2 = (2.0 ** rng.integers(-2, 3, 70)).astype(F32)
    Wi = rng.integers(-127, 128, (70, 33)).astype(F32)
    Y = oracle.fp_linear(Xi * s2, s2, Wi)
    assert np.array_equal(Y.astype(np.int64), Xi.astype(np.int64) @ Wi.astype(np.int64))
    # general case: within the forward error bound of a length-K binary32 sum, and s divides per input channel
    X = rng.standard_normal((5, 70)).astype(F32)
    s = np.exp(rng.normal(0, 1, 70)).astype(F32)
    Y = oracle.fp_linear(X, s, Wf).astype(np.float64)
    xs = (X / s).astype(np.float64)
    ref = xs @ Wf.astype(np.float64)
    bound = 70 * 2.0 ** -24 * (np.abs(xs) @ np.abs(Wf.astype(np.float64))) * 1.01
    assert np.all(np.abs(Y - ref) <= bound)
    assert not np.allclose(Y, X.astype(np.float64) @ Wf.astype(np.float64), rtol=1e-3)   # s really is applied


def test_cpu_expert_follows_its_definition_and_has_no_activation_quantisation_error():
    m = offline.small_moe(seed=121, T=16, H=128, I=320, E=4)
    ex = m["experts"][1]
    ce = oracle.cpu_expert(ex)
    X, s_in = m["X"], m["s_in"]
    Y, mid = oracle.cpu_expert_ffn(X, s_in, ce, dumps=True)
    xs = (X.astype(F32) / s_in).astype(np.float64)
    g, u = xs @ ce.w1f.astype(np.float64), xs @ ce.w3f.astype(np.float64)
    h = g / (1 + np.exp(-g)) * u
    assert np.allclose(mid.astype(np.float64), h, rtol=2e-3, atol=1e-4 * np.abs(h).max())
    ref = (mid.astype(F32) / ex.s_mid).astype(np.float64) @ ce.w2f.astype(np.float64)
    assert np.allclose(Y.astype(np.float64), ref, rtol=2e-3, atol=1e-4 * np.abs(ref).max())
    # the same expert through the W8A8 path deviates from that floating-point result by the activation
    # quantisation error; the CPU path by binary16 / binary32 roundings only
    idx = np.full((16, 2), 1, np.int32)
    _, _, _, _, y8 = oracle.moe_ffn(X, idx, np.full((16, 2), 0.5, F32), s_in, m["experts"], dumps=True)
    full = ((h.astype(np.float16).astype(F32) / ex.s_mid).astype(np.float64)) @ ce.w2f.astype(np.float64)
    e_cpu = np.mean((Y.astype(np.float64) - full) ** 2)
    e_w8a8 = np.mean((y8[0::2].astype(np.float64) - full) ** 2)
    assert e_cpu < 0.05 * e_w8a8


def test_hybrid_layer_swaps_exactly_the_cpu_experts_rows():
    m = offline.small_moe(seed=122, T=23, H=128, I=192, E=8)
    X, idx, gw, s_in, ex = m["X"], m["idx"], m["gw"], m["s_in"], m["experts"]
    out8, _, _, _, y8 = oracle.moe_ffn(X, idx, gw, s_in, ex, dumps=True)
    assert np.array_equal(oracle.combine(y8, gw).view(np.uint16), out8.view(np.uint16))      # the combination step alone
    out0, y0 = oracle.moe_ffn_hybrid(X, idx, gw, s_in, ex, on_cpu=())
    assert np.array_equal(out0.view(np.uint16), out8.view(np.uint16))
    on_cpu = (2, 5)
    out, y = oracle.moe_ffn_hybrid(X, idx, gw, s_in, ex, on_cpu)
    flat = idx.ravel()
    cpu_rows = np.isin(flat, on_cpu)
    assert cpu_rows.any() and np.array_equal(y[~cpu_rows].view(np.uint16), y8[~cpu_rows].view(np.uint16))
    for e in on_cpu:
        rows = np.nonzero(flat == e)[0]
        assert np.array_equal(y[rows].view(np.uint16), oracle.cpu_expert_ffn(X[rows // 2], s_in, oracle.cpu_expert(ex[e])).view(np.uint16))
    untouched = ~np.isin(idx, on_cpu).any(axis=1)
    assert np.array_equal(out[untouched].view(np.uint16), out8[untouched].view(np.uint16))
    assert np.max(np.abs(out.astype(np.float64) - out8.astype(np.float64))) < 0.05 * np.abs(out8.astype(np.float64)).max()
