"""Offline quantisation of the synthetic workloads, done with the CPU oracle only.

Produces the hot path's inputs (smoothing vectors, int8 weights, scales) from the
full-precision tensors of haq_inputs, the way Algorithm 1's smoothing step plus
plain round-to-nearest weight quantisation would, for a fixed exponent alpha.
Both the oracle and the HIP library are then fed these same bytes.
"""
from __future__ import annotations

import numpy as np

import haq_inputs as hi
import oracle

CALIB_TOKENS = 256


def quantize_linear(X, W, alpha=0.5):
    """s from (X, W), then Q(W s).  Returns s [K], Wq int8 [K,N], sw [N]."""
    s = oracle.smoothing_vector(oracle.col_absmax_f16(X), oracle.row_absmax_f32(W), alpha)
    Wq, sw = oracle.quant_weight(W, s)
    return s, Wq, sw


def quantize_ffn(X, W1, W2, alpha=0.5):
    """Two chained linears (ReLU between): the second one is calibrated on the
    fp16 output the quantised first one produces."""
    s1, W1q, sw1 = quantize_linear(X, W1, alpha)
    Hmid = oracle.w8a8_linear(X, s1, W1q, sw1, "relu")
    s2, W2q, sw2 = quantize_linear(Hmid, W2, alpha)
    return (s1, W1q, sw1), (s2, W2q, sw2)


def quantize_moe(X, idx, weights, alpha=0.5, calib_tokens=CALIB_TOKENS):
    """weights: list over experts of (w1 [H,I], w3 [H,I], w2 [I,H]) fp32.

    s_in is shared by w1/w3 of all experts (they all see the same X); s_mid[e] is
    per expert, calibrated on the intermediate of the first `calib_tokens` tokens.
    Returns s_in [H], list[oracle.Expert].
    """
    E = len(weights)
    H, I = weights[0][0].shape
    aw = np.zeros(H, np.float32)
    for w1, w3, _ in weights:
        oracle.row_absmax_f32(w1, aw)
        oracle.row_absmax_f32(w3, aw)
    s_in = oracle.smoothing_vector(oracle.col_absmax_f16(X), aw, alpha)
    ones = np.ones(I, np.float32)
    stage1 = []
    for w1, w3, w2 in weights:
        w1q, sw1 = oracle.quant_weight(w1, s_in)
        w3q, sw3 = oracle.quant_weight(w3, s_in)
        stage1.append(oracle.Expert(w1q, w3q, np.zeros((I, H), np.int8), sw1, sw3, np.zeros(H, np.float32), ones))
    n_cal = min(calib_tokens, X.shape[0])
    ax_mid = oracle.moe_mid_absmax(X[:n_cal], idx[:n_cal], s_in, stage1)
    experts = []
    for e, (w1, w3, w2) in enumerate(weights):
        s_mid = oracle.smoothing_vector(ax_mid[e], oracle.row_absmax_f32(w2), alpha)
        w2q, sw2 = oracle.quant_weight(w2, s_mid)
        st = stage1[e]
        experts.append(oracle.Expert(st.w1, st.w3, w2q, st.sw1, st.sw3, sw2, s_mid))
    return s_in, experts


def small_moe(seed=7, T=37, H=128, I=320, E=8, routing="gate"):
    """A Mixtral-shaped layer shrunk so the oracle finishes in milliseconds."""
    wl = hi.MoeWorkload(f"small_moe_{routing}", seed, T, H, I, E, routing)
    X, _, _ = hi.hidden_states(seed, T, H, n_outlier=max(1, H // 64))
    if routing == "popularity":
        logits = hi.gumbel_logits(seed, T, tuple(np.asarray(hi.OFFLOAD_POPULARITY[:E]) / sum(hi.OFFLOAD_POPULARITY[:E])))
    else:
        logits = hi.moe_logits(wl, X)
    weights = [tuple(hi.moe_weight(wl, e, w) for w in ("w1", "w3", "w2")) for e in range(E)]
    idx, gw = oracle.route_top2(logits)
    s_in, experts = quantize_moe(X, idx, weights)
    return dict(wl=wl, X=X, logits=logits, weights=weights, idx=idx, gw=gw, s_in=s_in, experts=experts)
