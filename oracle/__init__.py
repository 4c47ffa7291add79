"""ctypes front-end of the CPU oracle (test infrastructure, not the product).

Only tests/, the smoke check and the benchmark's cpu_baseline leg import this.
The HIP library never does, and this module imports nothing from it.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_DIR, "haq_oracle.cpp")
_LIB = os.path.join(_DIR, "libhaq_oracle.so")

CXXFLAGS = ["-O3", "-march=x86-64-v3", "-std=c++17", "-fno-fast-math", "-ffp-contract=off",
            "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (a couple of seconds)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.run(["g++", *CXXFLAGS, _SRC, "-o", tmp], check=True)
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
    return _lib


def _p(a: np.ndarray | None):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def half_to_float(h: np.ndarray) -> np.ndarray:
    h = _c(h.view(np.uint16), np.uint16)
    out = np.empty(h.shape, np.float32)
    lib().oracle_half_to_float(_p(h), C.c_int64(h.size), _p(out))
    return out


def float_to_half(f: np.ndarray) -> np.ndarray:
    f = _c(f, np.float32)
    out = np.empty(f.shape, np.uint16)
    lib().oracle_float_to_half(_p(f), C.c_int64(f.size), _p(out))
    return out.view(np.float16)


def exp_spec(t: np.ndarray) -> np.ndarray:
    t = _c(t, np.float32)
    out = np.empty(t.shape, np.float32)
    lib().oracle_exp_spec(_p(t), C.c_int64(t.size), _p(out))
    return out


def col_absmax_f16(X: np.ndarray) -> np.ndarray:
    X = _c(X, np.float16)
    T, K = X.shape
    ax = np.empty(K, np.float32)
    lib().oracle_col_absmax_f16(_p(X), C.c_int64(K), T, K, _p(ax))
    return ax


def row_absmax_f32(W: np.ndarray, aw: np.ndarray | None = None) -> np.ndarray:
    W = _c(W, np.float32)
    K, N = W.shape
    if aw is None:
        aw = np.zeros(K, np.float32)
    lib().oracle_row_absmax_f32(_p(W), K, N, _p(aw))
    return aw


def smoothing_vector(ax: np.ndarray, aw: np.ndarray | None, alpha: float = 0.5) -> np.ndarray:
    ax = _c(ax, np.float32)
    K = ax.size
    s = np.empty(K, np.float32)
    use_w = aw is not None
    aw_ = _c(aw, np.float32) if use_w else None
    lib().oracle_smoothing_vector(_p(ax), _p(aw_), K, C.c_double(alpha), int(use_w), _p(s))
    return s


def smooth_quant_act(X: np.ndarray, s: np.ndarray | None):
    X = _c(X, np.float16)
    T, K = X.shape
    q = np.empty((T, K), np.int8)
    sx = np.empty(T, np.float32)
    s_ = None if s is None else _c(s, np.float32)
    lib().oracle_smooth_quant_act(_p(X), C.c_int64(K), _p(s_), T, K, _p(q), C.c_int64(K), _p(sx))
    return q, sx


def quant_weight(W: np.ndarray, s: np.ndarray | None):
    W = _c(W, np.float32)
    K, N = W.shape
    Wq = np.empty((K, N), np.int8)
    sw = np.empty(N, np.float32)
    s_ = None if s is None else _c(s, np.float32)
    lib().oracle_quant_weight(_p(W), _p(s_), K, N, _p(Wq), _p(sw))
    return Wq, sw


def gemm_i8(q: np.ndarray, Wq: np.ndarray) -> np.ndarray:
    q = _c(q, np.int8)
    Wq = _c(Wq, np.int8)
    T, K = q.shape
    K2, N = Wq.shape
    assert K == K2
    acc = np.empty((T, N), np.int32)
    lib().oracle_gemm_i8(_p(q), C.c_int64(K), _p(Wq), T, K, N, _p(acc))
    return acc


ACT = {"none": 0, "relu": 1}


def epilogue(acc: np.ndarray, sx: np.ndarray, sw: np.ndarray, act: str = "none") -> np.ndarray:
    acc = _c(acc, np.int32)
    T, N = acc.shape
    Y = np.empty((T, N), np.float16)
    lib().oracle_epilogue(_p(acc), _p(_c(sx, np.float32)), _p(_c(sw, np.float32)), T, N, ACT[act],
                          _p(Y), C.c_int64(N))
    return Y


def w8a8_linear(X, s, Wq, sw, act="none", full=False):
    """The public linear: quantise activations, int8 GEMM, dequantise + activation."""
    q, sx = smooth_quant_act(X, s)
    acc = gemm_i8(q, Wq)
    Y = epilogue(acc, sx, sw, act)
    return (Y, acc, q, sx) if full else Y


def route_top2(logits: np.ndarray):
    logits = _c(logits, np.float16)
    T, E = logits.shape
    idx = np.empty((T, 2), np.int32)
    gw = np.empty((T, 2), np.float32)
    lib().oracle_route_top2(_p(logits), C.c_int64(E), T, E, _p(idx), _p(gw))
    return idx, gw


def permute(idx: np.ndarray, E: int):
    idx = _c(idx, np.int32)
    T = idx.shape[0]
    counts = np.empty(E, np.int32)
    offsets = np.empty(E + 1, np.int32)
    perm = np.empty(2 * T, np.int32)
    inv = np.empty(2 * T, np.int32)
    lib().oracle_permute(_p(idx), T, E, _p(counts), _p(offsets), _p(perm), _p(inv))
    return counts, offsets, perm, inv


class _ExpertStruct(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("w1", "w3", "w2", "sw1", "sw3", "sw2", "s_mid")]


@dataclass
class Expert:
    """One expert's offline-quantised weights: int8 [H,I], [H,I], [I,H] + scales + s_mid."""
    w1: np.ndarray
    w3: np.ndarray
    w2: np.ndarray
    sw1: np.ndarray
    sw3: np.ndarray
    sw2: np.ndarray
    s_mid: np.ndarray


def _expert_array(experts: list[Expert]):
    arr = (_ExpertStruct * len(experts))()
    for i, e in enumerate(experts):
        for n, dt in (("w1", np.int8), ("w3", np.int8), ("w2", np.int8), ("sw1", np.float32),
                      ("sw3", np.float32), ("sw2", np.float32), ("s_mid", np.float32)):
            a = getattr(e, n)
            assert a.dtype == dt and a.flags.c_contiguous, n
            setattr(arr[i], n, a.ctypes.data)
    return arr


def moe_ffn(X, idx, gw, s_in, experts: list[Expert], tokens=None, dumps=False):
    X = _c(X, np.float16)
    T, H = X.shape
    I = experts[0].w1.shape[1]
    idx = _c(idx, np.int32)
    gw = _c(gw, np.float32)
    tok = None if tokens is None else _c(tokens, np.int32)
    n_tok = T if tok is None else tok.size
    out = np.empty((n_tok, H), np.float16)
    mid = hq = sh = y = None
    if dumps:
        mid = np.empty((2 * n_tok, I), np.float16)
        hq = np.empty((2 * n_tok, I), np.int8)
        sh = np.empty(2 * n_tok, np.float32)
        y = np.empty((2 * n_tok, H), np.float16)
    arr = _expert_array(experts)
    lib().oracle_moe_ffn(_p(X), C.c_int64(H), _p(idx), _p(gw), _p(_c(s_in, np.float32)), arr, T, H, I,
                         _p(tok), n_tok, _p(out), _p(mid), _p(hq), _p(sh), _p(y))
    return (out, mid, hq, sh, y) if dumps else out


def moe_mid_absmax(X, idx, s_in, experts: list[Expert]) -> np.ndarray:
    X = _c(X, np.float16)
    T, H = X.shape
    I = experts[0].w1.shape[1]
    E = len(experts)
    ax = np.empty((E, I), np.float32)
    arr = _expert_array(experts)
    lib().oracle_moe_mid_absmax(_p(X), C.c_int64(H), _p(_c(idx, np.int32)), _p(_c(s_in, np.float32)), arr,
                                T, H, I, E, _p(ax))
    return ax


# ---- adaptive smoothing (Algorithm 1 step 1, Eq. 3) ----------------------------------------
def matmul_f64(X: np.ndarray, W: np.ndarray) -> np.ndarray:
    """Full-precision X W (binary16 activations, binary32 weights, binary64 arithmetic)."""
    X = _c(X, np.float16)
    W = _c(W, np.float32)
    T, K = X.shape
    K2, N = W.shape
    assert K == K2
    Y = np.empty((T, N), np.float64)
    lib().oracle_matmul_f64(_p(X), C.c_int64(K), _p(W), T, K, N, _p(Y))
    return Y


def mse_f64(Y: np.ndarray, Yref: np.ndarray) -> float:
    Y = _c(Y, np.float16)
    Yref = _c(Yref, np.float64)
    T, N = Y.shape
    assert Yref.shape == (T, N)
    f = lib().oracle_mse_f64
    f.restype = C.c_double
    return float(f(_p(Y), C.c_int64(N), _p(Yref), T, N))


def smoothing_search(X: np.ndarray, W: np.ndarray, exponents, use_weight: bool = False):
    """Grid search of the smoothing exponent e (Algorithm 1 step 1).

    For every e of the grid, in order: s = ax^e (Eq. 3; with use_weight the balanced form
    ax^e / aw^(1-e)), the weight is folded and quantised, Q(W s), the calibration
    activations go through the quantised layer, Q(W s) Q(X / s), and the loss is the mean
    squared error against the full-precision X W (the norm of Eq. 1 read as Frobenius^2 /
    size).  A candidate replaces the incumbent only if its loss is strictly smaller, so
    the first of equal minima wins.  Returns (losses [n_e] float64, best index, best s).
    """
    ax = col_absmax_f16(X)
    aw = row_absmax_f32(W) if use_weight else None
    Yref = matmul_f64(X, W)
    losses = np.empty(len(exponents), np.float64)
    best, best_loss, best_s = -1, np.inf, None
    for i, e in enumerate(exponents):
        s = smoothing_vector(ax, aw, float(e))
        Wq, sw = quant_weight(W, s)
        Y = w8a8_linear(X, s, Wq, sw, "none")
        losses[i] = mse_f64(Y, Yref)
        if losses[i] < best_loss:
            best, best_loss, best_s = i, losses[i], s
    return losses, best, best_s


# ---- offload scheduler (Section III.C: cost model, LRU expert cache, Algorithm 2) -----------
# Plain host logic, written out step by step.
def n_critical(t_e: float, latency_cpu: float, latency_gpu: float):
    """Critical batch size of Eq. 7-8.  Computing an expert on the CPU costs
    T_CPU = n * latency_cpu, moving it to the GPU and computing there costs
    T_sum = t_e + n * latency_gpu; the expert is transferred when n > n_critical, and
    n_critical is the largest n for which the CPU is not slower (T_CPU <= T_sum).
    None when the CPU is never slower."""
    if not latency_cpu > latency_gpu:
        return None
    n = 0
    while (n + 1) * latency_cpu <= t_e + (n + 1) * latency_gpu:
        n += 1
    return n


def lru_trace(accesses, capacity: int):
    """Least-recently-used cache of `capacity` entries over a sequence of keys.
    Returns (hit flags per access, cache content from least to most recently used)."""
    cache = []  # least recently used first
    hits = []
    for key in accesses:
        if key in cache:
            hits.append(True)
            cache.remove(key)
        else:
            hits.append(False)
            if len(cache) >= capacity:
                cache.pop(0)
        cache.append(key)
    return hits, cache


def select_experts(num_layers: int, top_k: int, supplement_k: int, path_stats, expert_freq):
    """Algorithm 2.  path_stats[layer] = [(experts of one activation path at this layer,
    frequency), ...]; expert_freq[layer] = [(expert, frequency), ...].  Stage I walks the
    layer's paths from the most frequent down and takes their experts until top_k are
    selected (top_k >= 1); stage II adds the layer's most frequently activated experts
    until top_k + supplement_k are selected.  Equal frequencies keep their input order.
    Returns a list of expert lists in order of selection."""
    selected = [[] for _ in range(num_layers)]
    for layer in range(num_layers):
        paths = sorted(path_stats[layer], key=lambda pf: -pf[1])  # stable
        for path, _ in paths:
            for e in path:
                if e not in selected[layer]:
                    selected[layer].append(e)
                if len(selected[layer]) >= top_k:
                    break
            if len(selected[layer]) >= top_k:
                break
    for layer in range(num_layers):
        experts = sorted(expert_freq[layer], key=lambda ef: -ef[1])
        for e, _ in experts:
            if len(selected[layer]) >= top_k + supplement_k:
                break
            if e not in selected[layer]:
                selected[layer].append(e)
    return selected


# ---- Hessian-aware weight quantisation (Section III.B.2; Algorithm 1 step 2) -------------------
def hessian(X: np.ndarray, s: np.ndarray | None, percdamp: float = 0.01) -> np.ndarray:
    X = _c(X, np.float16)
    T, K = X.shape
    H = np.empty((K, K), np.float64)
    s_ = None if s is None else _c(s, np.float32)
    lib().oracle_hessian(_p(X), C.c_int64(K), _p(s_), T, K, C.c_double(percdamp), _p(H))
    return H


def inverse_cholesky_upper(H: np.ndarray) -> np.ndarray:
    H = _c(H, np.float64)
    K = H.shape[0]
    U = np.empty((K, K), np.float64)
    rc = lib().oracle_inverse_cholesky_upper(_p(H), K, _p(U))
    if rc != 0:
        raise ValueError(f"the Hessian is not positive definite (pivot {rc - 1})")
    return U


def gptq(W: np.ndarray, s: np.ndarray | None, U: np.ndarray):
    W = _c(W, np.float32)
    K, N = W.shape
    Wq = np.empty((K, N), np.int8)
    sw = np.empty(N, np.float32)
    s_ = None if s is None else _c(s, np.float32)
    lib().oracle_gptq(_p(W), _p(s_), _p(_c(U, np.float64)), K, N, _p(Wq), _p(sw))
    return Wq, sw


def hessian_quant_weight(X: np.ndarray, W: np.ndarray, s: np.ndarray | None, percdamp: float = 0.01):
    """Q(W s) with error compensation along the input channels (Eq. 4-6): returns (Wq, sw)."""
    return gptq(W, s, inverse_cholesky_upper(hessian(X, s, percdamp)))


# ---- asymmetric activations ------------------------------------------------------------------
def asym_quant_act(X: np.ndarray, s: np.ndarray | None):
    """Per-token asymmetric uint8 codes: returns (q uint8 [T,K], scale [T], zero point int32 [T])."""
    X = _c(X, np.float16)
    T, K = X.shape
    q = np.empty((T, K), np.uint8)
    sx = np.empty(T, np.float32)
    zp = np.empty(T, np.int32)
    s_ = None if s is None else _c(s, np.float32)
    lib().oracle_asym_quant_act(_p(X), C.c_int64(K), _p(s_), T, K, _p(q), C.c_int64(K), _p(sx), _p(zp))
    return q, sx, zp


def asym_gemm(q: np.ndarray, zp: np.ndarray, Wq: np.ndarray) -> np.ndarray:
    q = _c(q, np.uint8)
    Wq = _c(Wq, np.int8)
    T, K = q.shape
    N = Wq.shape[1]
    acc = np.empty((T, N), np.int32)
    lib().oracle_asym_gemm(_p(q), C.c_int64(K), _p(_c(zp, np.int32)), _p(Wq), T, K, N, _p(acc))
    return acc


def w8a8_linear_asym(X, s, Wq, sw, act="none", full=False):
    """The linear layer with asymmetric activation codes and symmetric weights."""
    q, sx, zp = asym_quant_act(X, s)
    acc = asym_gemm(q, zp, Wq)
    Y = epilogue(acc, sx, sw, act)
    return (Y, acc, q, sx, zp) if full else Y


def moe_ffn_asym(X, idx, gw, s_in, experts: list[Expert], tokens=None, dumps=False):
    """The routed expert FFN with asymmetric activation codes for the tokens and for the requantised
    intermediate.  With dumps: (out, mid fp16, hq uint8, sh, zh int32, y fp16), pair rows ordered by
    (token position in `tokens`, slot)."""
    X = _c(X, np.float16)
    T, H = X.shape
    I = experts[0].w1.shape[1]
    idx = _c(idx, np.int32)
    gw = _c(gw, np.float32)
    tok = None if tokens is None else _c(tokens, np.int32)
    n_tok = T if tok is None else tok.size
    out = np.empty((n_tok, H), np.float16)
    mid = hq = sh = zh = y = None
    if dumps:
        mid = np.empty((2 * n_tok, I), np.float16)
        hq = np.empty((2 * n_tok, I), np.uint8)
        sh = np.empty(2 * n_tok, np.float32)
        zh = np.empty(2 * n_tok, np.int32)
        y = np.empty((2 * n_tok, H), np.float16)
    arr = _expert_array(experts)
    lib().oracle_moe_ffn_asym(_p(X), C.c_int64(H), _p(idx), _p(gw), _p(_c(s_in, np.float32)), arr, T, H, I,
                              _p(tok), n_tok, _p(out), _p(mid), _p(hq), _p(sh), _p(zh), _p(y))
    return (out, mid, hq, sh, zh, y) if dumps else out


# ---- the CPU side of the heterogeneous deployment (Section III.B.3, III.C.1a) ------------------
def dequant_weight(Wq: np.ndarray, sw: np.ndarray) -> np.ndarray:
    """The floating-point copy the CPU caches at load time: float(code) * scale, binary32."""
    Wq = _c(Wq, np.int8)
    K, N = Wq.shape
    Wf = np.empty((K, N), np.float32)
    lib().oracle_dequant_weight(_p(Wq), _p(_c(sw, np.float32)), K, N, _p(Wf))
    return Wf


def fp_linear(X: np.ndarray, s: np.ndarray | None, Wf: np.ndarray) -> np.ndarray:
    """(X / s) Wf in binary32: one accumulator per output, k ascending, fused multiply-adds."""
    X = _c(X, np.float32)
    Wf = _c(Wf, np.float32)
    T, K = X.shape
    N = Wf.shape[1]
    Y = np.empty((T, N), np.float32)
    s_ = None if s is None else _c(s, np.float32)
    lib().oracle_fp_linear(_p(X), C.c_int64(K), _p(s_), _p(Wf), T, K, N, _p(Y))
    return Y


@dataclass
class CpuExpert:
    """An expert's floating-point copy on the CPU: W1f, W3f [H,I], W2f [I,H] binary32, and s_mid."""
    w1f: np.ndarray
    w3f: np.ndarray
    w2f: np.ndarray
    s_mid: np.ndarray


def cpu_expert(ex: Expert) -> CpuExpert:
    return CpuExpert(dequant_weight(ex.w1, ex.sw1), dequant_weight(ex.w3, ex.sw3), dequant_weight(ex.w2, ex.sw2), ex.s_mid)


def cpu_expert_ffn(X: np.ndarray, s_in, ce: CpuExpert, dumps=False):
    """One SwiGLU expert in floating point on its CPU copy: rows of X (fp16) -> y fp16 [rows, H]."""
    X = _c(X, np.float16)
    n, H = X.shape
    I = ce.w1f.shape[1]
    Y = np.empty((n, H), np.float16)
    mid = np.empty((n, I), np.float16) if dumps else None
    lib().oracle_cpu_expert_ffn(_p(X), C.c_int64(H), _p(_c(s_in, np.float32)), _p(_c(ce.w1f, np.float32)),
                                _p(_c(ce.w3f, np.float32)), _p(_c(ce.w2f, np.float32)), _p(_c(ce.s_mid, np.float32)),
                                n, H, I, _p(Y), C.c_int64(H), _p(mid))
    return (Y, mid) if dumps else Y


def combine(y: np.ndarray, gw: np.ndarray) -> np.ndarray:
    """out[t] = fp16(g0 y[2t] + g1 y[2t+1]) (y in pair order)."""
    y = _c(y, np.float16)
    P, H = y.shape
    out = np.empty((P // 2, H), np.float16)
    lib().oracle_combine(_p(y), _p(_c(gw, np.float32)), P // 2, H, _p(out))
    return out


def moe_ffn_hybrid(X, idx, gw, s_in, experts: list[Expert], on_cpu):
    """The routed expert FFN when the experts in `on_cpu` are computed on the CPU (option A of the
    cost-benefit analysis: floating point on the dequantised copy) and the others by the W8A8 path;
    the per-pair outputs are combined as always.  Returns (out, y per pair)."""
    T = X.shape[0]
    idx = _c(idx, np.int32)
    _, _, _, _, y = moe_ffn(X, idx, gw, s_in, experts, dumps=True)
    y = y.copy()
    flat = idx.ravel()
    for e in sorted(set(int(v) for v in on_cpu)):
        rows = np.nonzero(flat == e)[0]
        if rows.size:
            y[rows] = cpu_expert_ffn(X[rows // 2], s_in, cpu_expert(experts[e]))
    return combine(y, gw), y
