"""ctypes binding of libhaq.so: argument marshalling only.

Function names are those of include/haq.h.  Tensors are torch tensors on the GPU
(they own the memory); work is enqueued on torch's current stream.  There is no
fallback: if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

__all__ = [
    "HaqError", "lib", "haq_version", "haq_smooth_quant_act", "haq_channel_absmax_f16", "haq_weight_row_absmax",
    "haq_smoothing_vector", "haq_quant_weight", "haq_packed_bytes", "haq_pack_weight", "haq_pack_gate_up",
    "haq_linear_workspace_bytes", "haq_w8a8_linear", "haq_packed_act_rows", "haq_packed_act_bytes",
    "haq_quant_act_packed", "haq_gemm_w8a8_packed", "haq_ffn_workspace_bytes", "haq_w8a8_ffn",
    "haq_moe_workspace_bytes", "haq_moe_w8a8_ffn",
    "haq_ctx_create", "haq_ctx_destroy", "ExpertWeights", "MoeDebug", "HAQ_ACT_NONE", "HAQ_ACT_RELU",
    "HAQ_LOC_DEVICE", "HAQ_LOC_HOST_PINNED", "EXPORTED_SYMBOLS", "HAQ_DECISION_GPU_CACHED", "HAQ_DECISION_TRANSFER", "HAQ_DECISION_CPU",
    "haq_smoothing_search_workspace_bytes", "haq_reference_matmul_f64", "haq_quant_loss_f64", "haq_smoothing_search",
    "haq_ctx_cache_stats", "haq_ctx_cache_invalidate", "haq_offload_n_critical", "haq_select_experts", "haq_lru_plan",
    "haq_cpu_expert_create", "haq_cpu_expert_destroy", "haq_cpu_expert_ffn", "haq_ctx_set_offload_policy", "haq_ctx_register_cpu_expert", "haq_ctx_last_decisions",
    "haq_linear_kn_workspace_bytes", "haq_w8a8_linear_kn",
    "haq_moe_w8a8_ffn_static", "haq_moe_asym_workspace_bytes", "haq_moe_w8a8_ffn_asym", "haq_ctx_last_call_timing", "haq_profile_enable", "haq_profile_read", "haq_probe_mfma_i8", "haq_probe_kloop_i8", "haq_probe_clock",
    "haq_hessian_quant_workspace_bytes", "haq_inverse_cholesky_workspace_bytes", "haq_hessian_f64",
    "haq_inverse_cholesky_upper_f64", "haq_hessian_quant_weight",
    "haq_weight_colsum", "haq_linear_asym_workspace_bytes", "haq_w8a8_linear_asym",
    "haq_quantize_layer_workspace_bytes", "haq_quantize_layer",
]

HAQ_ACT_NONE, HAQ_ACT_RELU = 0, 1
HAQ_LOC_DEVICE, HAQ_LOC_HOST_PINNED = 0, 1
HAQ_DECISION_GPU_CACHED, HAQ_DECISION_TRANSFER, HAQ_DECISION_CPU = 0, 1, 2

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libhaq.so")

EXPORTED_SYMBOLS = [
    "haq_version", "haq_last_error", "haq_smooth_quant_act", "haq_channel_absmax_f16", "haq_weight_row_absmax",
    "haq_smoothing_vector", "haq_quant_weight", "haq_packed_bytes", "haq_pack_weight", "haq_pack_gate_up",
    "haq_linear_workspace_bytes", "haq_w8a8_linear", "haq_packed_act_rows", "haq_packed_act_bytes",
    "haq_quant_act_packed", "haq_gemm_w8a8_packed", "haq_ffn_workspace_bytes", "haq_w8a8_ffn", "haq_ctx_create",
    "haq_ctx_destroy",
    "haq_moe_workspace_bytes", "haq_moe_w8a8_ffn",
    "haq_smoothing_search_workspace_bytes", "haq_reference_matmul_f64", "haq_quant_loss_f64", "haq_smoothing_search",
    "haq_ctx_cache_stats", "haq_ctx_cache_invalidate", "haq_offload_n_critical", "haq_select_experts", "haq_lru_plan",
    "haq_cpu_expert_create", "haq_cpu_expert_destroy", "haq_cpu_expert_ffn", "haq_ctx_set_offload_policy", "haq_ctx_register_cpu_expert", "haq_ctx_last_decisions",
    "haq_linear_kn_workspace_bytes", "haq_w8a8_linear_kn",
    "haq_moe_w8a8_ffn_static", "haq_moe_asym_workspace_bytes", "haq_moe_w8a8_ffn_asym", "haq_ctx_last_call_timing", "haq_profile_enable", "haq_profile_read", "haq_probe_mfma_i8", "haq_probe_kloop_i8", "haq_probe_clock",
    "haq_hessian_quant_workspace_bytes", "haq_inverse_cholesky_workspace_bytes", "haq_hessian_f64",
    "haq_inverse_cholesky_upper_f64", "haq_hessian_quant_weight",
    "haq_weight_colsum", "haq_linear_asym_workspace_bytes", "haq_w8a8_linear_asym",
    "haq_quantize_layer_workspace_bytes", "haq_quantize_layer",
]


class HaqError(RuntimeError):
    pass


class _ExpertDesc(C.Structure):
    _fields_ = [("w13", C.c_void_p), ("w2", C.c_void_p), ("sw1", C.c_void_p), ("sw3", C.c_void_p),
                ("sw2", C.c_void_p), ("s_mid", C.c_void_p), ("location", C.c_int32), ("reserved", C.c_int32)]


_DBG_FIELDS = ("topk_idx", "topk_w", "counts", "offsets", "perm", "inv", "q", "sx", "mid_fp16", "hq", "sh", "y_fp16")


class _MoeDebug(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _DBG_FIELDS]


_lib = None


def lib() -> C.CDLL:
    """Loads libhaq.so (building it first only if it has never been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            from .build import build
            build()
        L = C.CDLL(LIB_PATH)
        L.haq_last_error.restype = C.c_char_p
        for n in ("haq_packed_bytes", "haq_linear_workspace_bytes", "haq_moe_workspace_bytes", "haq_packed_act_bytes",
                  "haq_ffn_workspace_bytes", "haq_smoothing_search_workspace_bytes", "haq_hessian_quant_workspace_bytes",
                  "haq_inverse_cholesky_workspace_bytes", "haq_linear_asym_workspace_bytes",
                  "haq_quantize_layer_workspace_bytes", "haq_moe_asym_workspace_bytes", "haq_linear_kn_workspace_bytes"):
            getattr(L, n).restype = C.c_size_t
        L.haq_packed_act_rows.restype = C.c_int64
        _lib = L
    return _lib


def _check(rc: int):
    if rc != 0:
        raise HaqError(f"libhaq error {rc}: {lib().haq_last_error().decode()}")


def _ptr(t):
    if t is None:
        return None
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ws(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def haq_version() -> int:
    return int(lib().haq_version())


def haq_smooth_quant_act(x: torch.Tensor, s: torch.Tensor | None):
    """x fp16 [T,K], s fp32 [K] or None -> (q int8 [T,K], row_scale fp32 [T])."""
    T, K = x.shape
    q = torch.empty((T, K), dtype=torch.int8, device=x.device)
    sx = torch.empty((T,), dtype=torch.float32, device=x.device)
    _check(lib().haq_smooth_quant_act(_ptr(x), C.c_int64(x.stride(0)), _ptr(s), T, K, _ptr(q), C.c_int64(K),
                                      _ptr(sx), _stream()))
    return q, sx


def haq_channel_absmax_f16(x: torch.Tensor, ax: torch.Tensor | None = None) -> torch.Tensor:
    T, K = x.shape
    if ax is None:
        ax = torch.zeros((K,), dtype=torch.float32, device=x.device)
    _check(lib().haq_channel_absmax_f16(_ptr(x), C.c_int64(x.stride(0)), T, K, _ptr(ax), _stream()))
    return ax


def haq_weight_row_absmax(w: torch.Tensor, aw: torch.Tensor | None = None) -> torch.Tensor:
    K, N = w.shape
    if aw is None:
        aw = torch.zeros((K,), dtype=torch.float32, device=w.device)
    _check(lib().haq_weight_row_absmax(_ptr(w), K, N, _ptr(aw), _stream()))
    return aw


def haq_smoothing_vector(ax: torch.Tensor, aw: torch.Tensor | None, alpha: float = 0.5) -> torch.Tensor:
    """Host-side formula on host copies of the magnitudes; returns s on ax's device."""
    ax_h = ax.detach().to("cpu", torch.float32).contiguous()
    aw_h = None if aw is None else aw.detach().to("cpu", torch.float32).contiguous()
    s_h = torch.empty_like(ax_h)
    _check(lib().haq_smoothing_vector(_ptr(ax_h), _ptr(aw_h), ax_h.numel(), C.c_double(alpha), _ptr(s_h)))
    return s_h.to(ax.device)


def haq_quant_weight(w: torch.Tensor, s: torch.Tensor | None):
    """w fp32 [K,N] -> (wq int8 [K,N] canonical, w_scale fp32 [N])."""
    K, N = w.shape
    wq = torch.empty((K, N), dtype=torch.int8, device=w.device)
    sw = torch.empty((N,), dtype=torch.float32, device=w.device)
    _check(lib().haq_quant_weight(_ptr(w), _ptr(s), K, N, _ptr(wq), _ptr(sw), _stream()))
    return wq, sw


def haq_packed_bytes(K: int, N: int) -> int:
    return int(lib().haq_packed_bytes(K, N))


def haq_pack_weight(wq: torch.Tensor) -> torch.Tensor:
    K, N = wq.shape
    out = torch.empty((haq_packed_bytes(K, N),), dtype=torch.int8, device=wq.device)
    _check(lib().haq_pack_weight(_ptr(wq), K, N, _ptr(out), _stream()))
    return out


def haq_pack_gate_up(w1q: torch.Tensor, w3q: torch.Tensor) -> torch.Tensor:
    K, N = w1q.shape
    out = torch.empty((haq_packed_bytes(K, 2 * N),), dtype=torch.int8, device=w1q.device)
    _check(lib().haq_pack_gate_up(_ptr(w1q), _ptr(w3q), K, N, _ptr(out), _stream()))
    return out


def haq_linear_workspace_bytes(T: int, K: int, N: int) -> int:
    return int(lib().haq_linear_workspace_bytes(T, K, N))


def haq_w8a8_linear(x, s, w_packed, w_scale, N: int, act: int = HAQ_ACT_NONE, *, out=None, workspace=None,
                    debug: bool = False):
    """x fp16 [T,K] -> y fp16 [T,N]; with debug=True also (acc int32 [T,N], q int8 [T,K], sx [T])."""
    T, K = x.shape
    dev = x.device
    y = out if out is not None else torch.empty((T, N), dtype=torch.float16, device=dev)
    if workspace is None:
        workspace = _ws(haq_linear_workspace_bytes(T, K, N), dev)
    acc = q = sx = None
    if debug:
        acc = torch.empty((T, N), dtype=torch.int32, device=dev)
        q = torch.empty((T, K), dtype=torch.int8, device=dev)
        sx = torch.empty((T,), dtype=torch.float32, device=dev)
    _check(lib().haq_w8a8_linear(_ptr(x), C.c_int64(x.stride(0)), _ptr(s), _ptr(w_packed), _ptr(w_scale), T, K, N, act,
                                 _ptr(y), C.c_int64(y.stride(0)), _ptr(acc), _ptr(q), _ptr(sx), _ptr(workspace),
                                 C.c_size_t(workspace.numel()), _stream()))
    return (y, acc, q, sx) if debug else y


def haq_linear_kn_workspace_bytes(T: int, K: int, N: int) -> int:
    return int(lib().haq_linear_kn_workspace_bytes(T, K, N))


def haq_w8a8_linear_kn(x, s, wq_kn, w_scale, act: int = HAQ_ACT_NONE, *, out=None, workspace=None):
    """x fp16 [T,K], canonical int8 weights wq_kn [K,N] (packed per call into the workspace) -> y fp16 [T,N]."""
    T, K = x.shape
    N = wq_kn.shape[1]
    y = out if out is not None else torch.empty((T, N), dtype=torch.float16, device=x.device)
    if workspace is None:
        workspace = _ws(haq_linear_kn_workspace_bytes(T, K, N), x.device)
    _check(lib().haq_w8a8_linear_kn(_ptr(x), C.c_int64(x.stride(0)), _ptr(s), _ptr(wq_kn), _ptr(w_scale), T, K, N, act, _ptr(y),
                                    C.c_int64(y.stride(0)), _ptr(workspace), C.c_size_t(workspace.numel()), _stream()))
    return y


def haq_packed_act_rows(T: int) -> int:
    return int(lib().haq_packed_act_rows(T))


def haq_packed_act_bytes(T: int, K: int) -> int:
    return int(lib().haq_packed_act_bytes(T, K))


def haq_quant_act_packed(x, s, *, q_packed=None, row_scale=None):
    """x fp16 [T,K] -> (codes in the packed MFMA operand layout (flat int8), row_scale [T])."""
    T, K = x.shape
    if q_packed is None:
        q_packed = torch.empty((haq_packed_act_bytes(T, K),), dtype=torch.int8, device=x.device)
    if row_scale is None:
        row_scale = torch.empty((T,), dtype=torch.float32, device=x.device)
    _check(lib().haq_quant_act_packed(_ptr(x), C.c_int64(x.stride(0)), _ptr(s), T, K, _ptr(q_packed), _ptr(row_scale),
                                      _stream()))
    return q_packed, row_scale


def haq_gemm_w8a8_packed(q_packed, row_scale, w_packed, w_scale, T: int, K: int, N: int, act: int = HAQ_ACT_NONE, *,
                         out=None):
    y = out if out is not None else torch.empty((T, N), dtype=torch.float16, device=q_packed.device)
    _check(lib().haq_gemm_w8a8_packed(_ptr(q_packed), _ptr(row_scale), _ptr(w_packed), _ptr(w_scale), T, K, N, act,
                                      _ptr(y), C.c_int64(y.stride(0)), None, _stream()))
    return y


def haq_ffn_workspace_bytes(T: int, K: int, F: int, N: int) -> int:
    return int(lib().haq_ffn_workspace_bytes(T, K, F, N))


def haq_w8a8_ffn(x, s1, w1_packed, w1_scale, F: int, act: int, s2, w2_packed, w2_scale, N: int, *, out=None,
                 workspace=None, debug: bool = False):
    """x fp16 [T,K] -> y fp16 [T,N] through two chained W8A8 linears; debug=True also returns H fp16 [T,F]."""
    T, K = x.shape
    dev = x.device
    y = out if out is not None else torch.empty((T, N), dtype=torch.float16, device=dev)
    if workspace is None:
        workspace = _ws(haq_ffn_workspace_bytes(T, K, F, N), dev)
    h = torch.empty((T, F), dtype=torch.float16, device=dev) if debug else None
    _check(lib().haq_w8a8_ffn(_ptr(x), C.c_int64(x.stride(0)), _ptr(s1), _ptr(w1_packed), _ptr(w1_scale), act, _ptr(s2),
                              _ptr(w2_packed), _ptr(w2_scale), T, K, F, N, _ptr(y), C.c_int64(y.stride(0)), _ptr(h),
                              _ptr(workspace), C.c_size_t(workspace.numel()), _stream()))
    return (y, h) if debug else y


@dataclass
class ExpertWeights:
    """Device (or pinned host, for w13/w2) tensors of one expert, as haq_expert_desc wants them."""
    w13: torch.Tensor
    w2: torch.Tensor
    sw1: torch.Tensor
    sw3: torch.Tensor
    sw2: torch.Tensor
    s_mid: torch.Tensor
    location: int = HAQ_LOC_DEVICE


@dataclass
class MoeDebug:
    topk_idx: torch.Tensor
    topk_w: torch.Tensor
    counts: torch.Tensor
    offsets: torch.Tensor
    perm: torch.Tensor
    inv: torch.Tensor
    q: torch.Tensor
    sx: torch.Tensor
    mid_fp16: torch.Tensor
    hq: torch.Tensor
    sh: torch.Tensor
    y_fp16: torch.Tensor


def haq_moe_workspace_bytes(T: int, H: int, I: int, E: int) -> int:
    return int(lib().haq_moe_workspace_bytes(T, H, I, E))


def haq_ctx_create(H: int, I: int, n_slots: int):
    ctx = C.c_void_p()
    _check(lib().haq_ctx_create(H, I, n_slots, C.byref(ctx)))
    return ctx


def haq_ctx_destroy(ctx) -> None:
    _check(lib().haq_ctx_destroy(ctx))


def haq_moe_w8a8_ffn(x, logits, s_in, experts: list[ExpertWeights], I: int, *, ctx=None, out=None, workspace=None,
                     debug=False):
    """x fp16 [T,H], logits fp16 [T,E] -> out fp16 [T,H] (and a MoeDebug when debug is set: True asks for
    every intermediate, a tuple of field names for those only -- the others stay None)."""
    T, H = x.shape
    E = len(experts)
    dev = x.device
    y = out if out is not None else torch.empty((T, H), dtype=torch.float16, device=dev)
    if workspace is None:
        workspace = _ws(haq_moe_workspace_bytes(T, H, I, E), dev)
    descs = (_ExpertDesc * E)()
    for i, e in enumerate(experts):
        descs[i].w13, descs[i].w2 = e.w13.data_ptr(), e.w2.data_ptr()
        descs[i].sw1, descs[i].sw3, descs[i].sw2 = e.sw1.data_ptr(), e.sw3.data_ptr(), e.sw2.data_ptr()
        descs[i].s_mid, descs[i].location = e.s_mid.data_ptr(), e.location
    dbg = None
    dbg_c = None
    if debug:
        P = 2 * T
        i32, f32, f16, i8 = torch.int32, torch.float32, torch.float16, torch.int8
        mk = lambda shape, dt: torch.empty(shape, dtype=dt, device=dev)
        spec = (((T, 2), i32), ((T, 2), f32), ((E,), i32), ((E + 1,), i32), ((P,), i32), ((P,), i32),
                ((T, H), i8), ((T,), f32), ((P, I), f16), ((P, I), i8), ((P,), f32), ((P, H), f16))
        want = _DBG_FIELDS if debug is True else tuple(debug)
        if set(want) - set(_DBG_FIELDS):
            raise ValueError(f"unknown debug fields {sorted(set(want) - set(_DBG_FIELDS))}")
        dbg = MoeDebug(*[mk(*sp) if n in want else None for n, sp in zip(_DBG_FIELDS, spec)])
        dbg_c = _MoeDebug(*[getattr(dbg, n).data_ptr() if n in want else None for n in _DBG_FIELDS])
    _check(lib().haq_moe_w8a8_ffn(ctx, _ptr(x), C.c_int64(x.stride(0)), _ptr(logits), C.c_int64(logits.stride(0)),
                                  _ptr(s_in), descs, T, H, I, E, 2, _ptr(y), C.c_int64(y.stride(0)),
                                  C.byref(dbg_c) if dbg_c is not None else None, _ptr(workspace),
                                  C.c_size_t(workspace.numel()), _stream()))
    return (y, dbg) if debug else y


def haq_moe_w8a8_ffn_static(x, logits, s_in, experts, I: int, *, out):
    """haq_moe_w8a8_ffn on the library's built-in scratch array: nothing is allocated, so `out` is required."""
    T, H = x.shape
    E = len(experts)
    descs = (_ExpertDesc * E)()
    for i, e in enumerate(experts):
        descs[i].w13, descs[i].w2 = e.w13.data_ptr(), e.w2.data_ptr()
        descs[i].sw1, descs[i].sw3, descs[i].sw2 = e.sw1.data_ptr(), e.sw3.data_ptr(), e.sw2.data_ptr()
        descs[i].s_mid, descs[i].location = e.s_mid.data_ptr(), e.location
    _check(lib().haq_moe_w8a8_ffn_static(_ptr(x), C.c_int64(x.stride(0)), _ptr(logits), C.c_int64(logits.stride(0)), _ptr(s_in),
                                         descs, T, H, I, E, 2, _ptr(out), C.c_int64(out.stride(0)), _stream()))
    return out


class _ExpertColsum(C.Structure):
    _fields_ = [("cs1", C.c_void_p), ("cs3", C.c_void_p), ("cs2", C.c_void_p)]


class _MoeDebugAsym(C.Structure):
    _fields_ = [("base", _MoeDebug), ("zx", C.c_void_p), ("zh", C.c_void_p)]


def haq_moe_asym_workspace_bytes(T: int, H: int, I: int, E: int) -> int:
    return int(lib().haq_moe_asym_workspace_bytes(T, H, I, E))


def haq_moe_w8a8_ffn_asym(x, logits, s_in, experts, colsums, I: int, *, out=None, workspace=None, debug=False):
    """The routed expert FFN with asymmetric activation codes.  colsums: per expert (cs1 [I], cs3 [I], cs2 [H]) int32
    tensors from haq_weight_colsum.  With debug=True returns (y, MoeDebug with uint8 q / hq, zx [T], zh [2T])."""
    T, H = x.shape
    E = len(experts)
    dev = x.device
    y = out if out is not None else torch.empty((T, H), dtype=torch.float16, device=dev)
    if workspace is None:
        workspace = _ws(haq_moe_asym_workspace_bytes(T, H, I, E), dev)
    descs = (_ExpertDesc * E)()
    cs = (_ExpertColsum * E)()
    for i, (e, c) in enumerate(zip(experts, colsums)):
        descs[i].w13, descs[i].w2 = e.w13.data_ptr(), e.w2.data_ptr()
        descs[i].sw1, descs[i].sw3, descs[i].sw2 = e.sw1.data_ptr(), e.sw3.data_ptr(), e.sw2.data_ptr()
        descs[i].s_mid, descs[i].location = e.s_mid.data_ptr(), e.location
        cs[i].cs1, cs[i].cs3, cs[i].cs2 = c[0].data_ptr(), c[1].data_ptr(), c[2].data_ptr()
    dbg = zx = zh = None
    dbg_c = None
    if debug:
        P = 2 * T
        i32, f32, f16, u8 = torch.int32, torch.float32, torch.float16, torch.uint8
        mk = lambda shape, dt: torch.empty(shape, dtype=dt, device=dev)
        spec = (((T, 2), i32), ((T, 2), f32), ((E,), i32), ((E + 1,), i32), ((P,), i32), ((P,), i32),
                ((T, H), u8), ((T,), f32), ((P, I), f16), ((P, I), u8), ((P,), f32), ((P, H), f16))
        dbg = MoeDebug(*[mk(*sp) for sp in spec])
        zx, zh = mk((T,), i32), mk((P,), i32)
        dbg_c = _MoeDebugAsym(_MoeDebug(*[getattr(dbg, n).data_ptr() for n in _DBG_FIELDS]), zx.data_ptr(), zh.data_ptr())
    _check(lib().haq_moe_w8a8_ffn_asym(_ptr(x), C.c_int64(x.stride(0)), _ptr(logits), C.c_int64(logits.stride(0)), _ptr(s_in),
                                       descs, cs, T, H, I, E, 2, _ptr(y), C.c_int64(y.stride(0)),
                                       C.byref(dbg_c) if dbg_c is not None else None, _ptr(workspace),
                                       C.c_size_t(workspace.numel()), _stream()))
    return (y, dbg, zx, zh) if debug else y


# ---- the CPU side of the offload runtime (Section III.B.3, III.C.1a-b) ----------------------------
def haq_cpu_expert_create(w1q, w3q, w2q, sw1, sw3, sw2, s_mid, keep_codes: bool = False):
    """CPU tensors: canonical int8 matrices w1q, w3q [H,I], w2q [I,H], their scales and s_mid.  Returns an opaque handle
    to the expert's dequantised floating-point copy (free it with haq_cpu_expert_destroy)."""
    H, I = w1q.shape
    for t in (w1q, w3q, w2q, sw1, sw3, sw2, s_mid):
        assert t.device.type == "cpu" and t.is_contiguous()
    h = C.c_void_p()
    _check(lib().haq_cpu_expert_create(_ptr(w1q), _ptr(w3q), _ptr(w2q), _ptr(sw1), _ptr(sw3), _ptr(sw2), _ptr(s_mid), H, I, int(bool(keep_codes)), C.byref(h)))
    return h


def haq_cpu_expert_destroy(handle):
    _check(lib().haq_cpu_expert_destroy(handle))


def haq_cpu_expert_ffn(handle, x, s_in, H: int, n_threads: int = 0):
    """x fp16 [n, H] CPU tensor, s_in fp32 [H] CPU tensor or None -> y fp16 [n, H] (CPU)."""
    n = x.shape[0]
    y = torch.empty((n, H), dtype=torch.float16)
    _check(lib().haq_cpu_expert_ffn(handle, _ptr(x), C.c_int64(x.stride(0)), _ptr(s_in), n, _ptr(y), C.c_int64(H), n_threads))
    return y


def haq_ctx_set_offload_policy(ctx, t_e: float, latency_cpu: float, latency_gpu: float, s_in_host=None, cpu_threads: int = 0):
    _check(lib().haq_ctx_set_offload_policy(ctx, C.c_double(t_e), C.c_double(latency_cpu), C.c_double(latency_gpu),
                                            _ptr(s_in_host), cpu_threads))


def haq_ctx_register_cpu_expert(ctx, expert_weights, handle):
    """expert_weights: the ExpertWeights (host resident) whose w13 address keys the entry; handle None removes it."""
    _check(lib().haq_ctx_register_cpu_expert(ctx, C.c_void_p(expert_weights.w13.data_ptr()), handle))


def haq_ctx_last_decisions(ctx):
    """([(expert, n_inputs, decision), ...], n_critical) of the context's last call."""
    n = C.c_int32(0)
    ex, ni, de = (C.c_int32 * 32)(), (C.c_int32 * 32)(), (C.c_int32 * 32)()
    nc = C.c_int64(0)
    _check(lib().haq_ctx_last_decisions(ctx, 32, C.byref(n), ex, ni, de, C.byref(nc)))
    return [(int(ex[i]), int(ni[i]), int(de[i])) for i in range(n.value)], int(nc.value)


# ---- measurement aids ------------------------------------------------------------------------
def haq_profile_enable(on: bool):
    _check(lib().haq_profile_enable(int(bool(on))))


def haq_profile_read():
    """[(stage name, milliseconds), ...] of the last profiled block-level call (waits for it)."""
    n = C.c_int32(0)
    names = (C.c_char_p * 16)()
    ms = (C.c_float * 16)()
    _check(lib().haq_profile_read(16, C.byref(n), names, ms))
    return [(names[i].decode(), float(ms[i])) for i in range(n.value)]


def haq_probe_mfma_i8(data, iters: int, work_groups: int, *, out=None):
    """data int8 [>= 24576] device.  Returns the int32 [256, 8, 16] accumulators of work-group 0."""
    assert data.numel() >= 24576
    if out is None:
        out = torch.empty((256, 8, 16), dtype=torch.int32, device=data.device)
    _check(lib().haq_probe_mfma_i8(_ptr(data), iters, work_groups, _ptr(out), _stream()))
    return out


def haq_probe_kloop_i8(data, level: int, iters: int, work_groups: int, *, out=None):
    """The K loop of the GEMM kernel rebuilt on the probe's operands: level 1 adds the LDS fragment reads, 2 the barrier
    per K-step, 3 the direct-to-LDS loads (4: the same refill through registers).  Same accumulators as haq_probe_mfma_i8 for the same iters."""
    assert data.numel() >= 24576
    if out is None:
        out = torch.empty((256, 8, 16), dtype=torch.int32, device=data.device)
    _check(lib().haq_probe_kloop_i8(_ptr(data), level, iters, work_groups, _ptr(out), _stream()))
    return out


def haq_probe_clock(ticks_100mhz: int, *, out=None, stream=None):
    """Enqueues the clock probe (on `stream`, default: the current one); out[0] / out[1] * 100 = MHz once it has run."""
    if out is None:
        out = torch.zeros((2,), dtype=torch.int64, device="cuda")
    st = C.c_void_p(stream.cuda_stream) if stream is not None else _stream()
    _check(lib().haq_probe_clock(_ptr(out), C.c_int64(ticks_100mhz), st))
    return out


# ---- adaptive smoothing (Algorithm 1 step 1) --------------------------------------------
def haq_smoothing_search_workspace_bytes(T: int, K: int, N: int, n_e: int) -> int:
    return int(lib().haq_smoothing_search_workspace_bytes(T, K, N, n_e))


def haq_reference_matmul_f64(x, w, *, out=None):
    """x fp16 [T,K], w fp32 [K,N] -> X W in binary64 [T,N]."""
    T, K = x.shape
    N = w.shape[1]
    y = out if out is not None else torch.empty((T, N), dtype=torch.float64, device=x.device)
    _check(lib().haq_reference_matmul_f64(_ptr(x), C.c_int64(x.stride(0)), _ptr(w), T, K, N, _ptr(y), _stream()))
    return y


def haq_quant_loss_f64(y, yref):
    """mean (y - yref)^2 over all entries, binary64; returns a 1-element device tensor."""
    T, N = y.shape
    scratch = torch.empty((T,), dtype=torch.float64, device=y.device)
    loss = torch.empty((1,), dtype=torch.float64, device=y.device)
    _check(lib().haq_quant_loss_f64(_ptr(y), C.c_int64(y.stride(0)), _ptr(yref), T, N, _ptr(scratch), _ptr(loss), _stream()))
    return loss


def haq_smoothing_search(x, w, exponents, use_weight: bool = False, *, workspace=None):
    """Grid search of the smoothing exponent; returns (losses: list[float], best: int, s_best [K] device)."""
    T, K = x.shape
    N = w.shape[1]
    n_e = len(exponents)
    grid = (C.c_double * n_e)(*[float(e) for e in exponents])
    losses = (C.c_double * n_e)()
    best = C.c_int32(-1)
    s_best = torch.empty((K,), dtype=torch.float32, device=x.device)
    if workspace is None:
        workspace = _ws(haq_smoothing_search_workspace_bytes(T, K, N, n_e), x.device)
    _check(lib().haq_smoothing_search(_ptr(x), C.c_int64(x.stride(0)), _ptr(w), T, K, N, grid, n_e, int(bool(use_weight)),
                                      losses, C.byref(best), _ptr(s_best), _ptr(workspace), C.c_size_t(workspace.numel()),
                                      _stream()))
    return list(losses), int(best.value), s_best


# ---- expert cache and offload planning (Section III.C) -----------------------------------
def haq_ctx_cache_stats(ctx):
    """(hits, misses, bytes_copied, [address cached in each slot or None])."""
    h, m, b = C.c_int64(0), C.c_int64(0), C.c_int64(0)
    keys = (C.c_void_p * 32)()
    _check(lib().haq_ctx_cache_stats(ctx, C.byref(h), C.byref(m), C.byref(b), keys))
    return int(h.value), int(m.value), int(b.value), list(keys)


def haq_ctx_last_call_timing(ctx):
    """(total ms, ms from first copy issued to last copy landed, ms after the last copy) of the last offload call."""
    a, b, c = C.c_float(0), C.c_float(0), C.c_float(0)
    _check(lib().haq_ctx_last_call_timing(ctx, C.byref(a), C.byref(b), C.byref(c)))
    return float(a.value), float(b.value), float(c.value)


def haq_ctx_cache_invalidate(ctx):
    _check(lib().haq_ctx_cache_invalidate(ctx))


def haq_lru_plan(slot_keys: list, slot_ticks: list, tick: int, keys: list):
    """One batch of look-ups on a copy of an LRU cache's state.  Returns (slot_of, hit, prev_user, slot_keys,
    slot_ticks, tick) with the state after the batch."""
    n_slots, n = len(slot_keys), len(keys)
    sk = (C.c_uint64 * n_slots)(*slot_keys)
    stk = (C.c_uint64 * n_slots)(*slot_ticks)
    tk = C.c_uint64(tick)
    kk = (C.c_uint64 * max(1, n))(*keys)
    so, hi, pu = (C.c_int32 * max(1, n))(), (C.c_int32 * max(1, n))(), (C.c_int32 * max(1, n))()
    _check(lib().haq_lru_plan(n_slots, sk, stk, C.byref(tk), kk, n, so, hi, pu))
    return list(so)[:n], [bool(h) for h in list(hi)[:n]], list(pu)[:n], list(sk), list(stk), int(tk.value)


def haq_offload_n_critical(t_e: float, latency_cpu: float, latency_gpu: float):
    """Largest batch for which computing on the CPU is not slower; None if it never is."""
    n = C.c_int64(0)
    _check(lib().haq_offload_n_critical(C.c_double(t_e), C.c_double(latency_cpu), C.c_double(latency_gpu), C.byref(n)))
    return None if n.value < 0 else int(n.value)


def haq_select_experts(num_layers: int, experts_per_layer: int, top_k: int, supplement_k: int, path_stats, expert_freq):
    """path_stats[layer] = [(experts of the path at this layer, frequency), ...]; expert_freq[layer] =
    [frequency of expert 0, 1, ...].  Returns the selected experts of every layer in order of selection."""
    path_len = next((len(p[0]) for layer in path_stats for p in layer), 1)
    offs, flat, freq = [0], [], []
    for layer in range(num_layers):
        for path, f in path_stats[layer]:
            assert len(path) == path_len
            flat.extend(int(e) for e in path)
            freq.append(float(f))
        offs.append(len(freq))
    ef = [float(expert_freq[l][e]) for l in range(num_layers) for e in range(experts_per_layer)]
    cap = top_k + supplement_k
    sel = (C.c_int32 * max(1, num_layers * cap))()
    nsel = (C.c_int32 * max(1, num_layers))()
    _check(lib().haq_select_experts(num_layers, experts_per_layer, top_k, supplement_k, (C.c_int32 * len(offs))(*offs),
                                    (C.c_int32 * max(1, len(flat)))(*flat), path_len, (C.c_double * max(1, len(freq)))(*freq),
                                    (C.c_double * len(ef))(*ef), sel, nsel))
    return [[int(sel[l * cap + i]) for i in range(nsel[l])] for l in range(num_layers)]


# ---- Hessian-aware weight quantisation (Algorithm 1 step 2) ---------------------------------
def haq_hessian_quant_workspace_bytes(K: int, N: int) -> int:
    return int(lib().haq_hessian_quant_workspace_bytes(K, N))


def haq_inverse_cholesky_workspace_bytes(K: int) -> int:
    return int(lib().haq_inverse_cholesky_workspace_bytes(K))


def haq_hessian_f64(x, s, percdamp: float = 0.01):
    T, K = x.shape
    H = torch.empty((K, K), dtype=torch.float64, device=x.device)
    _check(lib().haq_hessian_f64(_ptr(x), C.c_int64(x.stride(0)), _ptr(s), T, K, C.c_double(percdamp), _ptr(H), _stream()))
    return H


def haq_inverse_cholesky_upper_f64(H):
    K = H.shape[0]
    U = torch.empty((K, K), dtype=torch.float64, device=H.device)
    ws = _ws(int(lib().haq_inverse_cholesky_workspace_bytes(K)), H.device)
    _check(lib().haq_inverse_cholesky_upper_f64(_ptr(H), K, _ptr(U), _ptr(ws), C.c_size_t(ws.numel()), _stream()))
    return U


def haq_hessian_quant_weight(x, w, s, percdamp: float = 0.01, *, workspace=None):
    """x fp16 [T,K] calibration activations, w fp32 [K,N], s [K] or None -> (wq int8 [K,N], w_scale [N])."""
    T, K = x.shape
    N = w.shape[1]
    wq = torch.empty((K, N), dtype=torch.int8, device=w.device)
    sw = torch.empty((N,), dtype=torch.float32, device=w.device)
    if workspace is None:
        workspace = _ws(int(lib().haq_hessian_quant_workspace_bytes(K, N)), w.device)
    _check(lib().haq_hessian_quant_weight(_ptr(x), C.c_int64(x.stride(0)), T, _ptr(w), _ptr(s), K, N, C.c_double(percdamp),
                                          _ptr(wq), _ptr(sw), _ptr(workspace), C.c_size_t(workspace.numel()), _stream()))
    return wq, sw


# ---- asymmetric activation codes ---------------------------------------------------------------
def haq_weight_colsum(wq):
    K, N = wq.shape
    out = torch.empty((N,), dtype=torch.int32, device=wq.device)
    _check(lib().haq_weight_colsum(_ptr(wq), K, N, _ptr(out), _stream()))
    return out


def haq_linear_asym_workspace_bytes(T: int, K: int, N: int) -> int:
    return int(lib().haq_linear_asym_workspace_bytes(T, K, N))


def haq_w8a8_linear_asym(x, s, w_packed, w_scale, w_colsum, N: int, act: int = HAQ_ACT_NONE, *, out=None, workspace=None,
                         debug: bool = False):
    """x fp16 [T,K] -> y fp16 [T,N]; with debug=True also (acc int32 [T,N], q uint8 [T,K], scale [T], zp int32 [T])."""
    T, K = x.shape
    dev = x.device
    y = out if out is not None else torch.empty((T, N), dtype=torch.float16, device=dev)
    if workspace is None:
        workspace = _ws(haq_linear_asym_workspace_bytes(T, K, N), dev)
    acc = q = sx = zp = None
    if debug:
        acc = torch.empty((T, N), dtype=torch.int32, device=dev)
        q = torch.empty((T, K), dtype=torch.uint8, device=dev)
        sx = torch.empty((T,), dtype=torch.float32, device=dev)
        zp = torch.empty((T,), dtype=torch.int32, device=dev)
    _check(lib().haq_w8a8_linear_asym(_ptr(x), C.c_int64(x.stride(0)), _ptr(s), _ptr(w_packed), _ptr(w_scale), _ptr(w_colsum),
                                      T, K, N, act, _ptr(y), C.c_int64(y.stride(0)), _ptr(acc), _ptr(q), _ptr(sx), _ptr(zp),
                                      _ptr(workspace), C.c_size_t(workspace.numel()), _stream()))
    return (y, acc, q, sx, zp) if debug else y


# ---- Algorithm 1 for one linear layer ------------------------------------------------------------
def haq_quantize_layer_workspace_bytes(T: int, K: int, N: int, n_e: int) -> int:
    return int(lib().haq_quantize_layer_workspace_bytes(T, K, N, n_e))


def haq_quantize_layer(x, w, exponents, use_weight: bool = False, percdamp: float = 0.01, *, workspace=None):
    """Smoothing search, then Hessian-aware quantisation with the chosen vector.
    Returns (s [K], wq int8 [K,N], w_scale [N], losses: list[float], best: int)."""
    T, K = x.shape
    N = w.shape[1]
    n_e = len(exponents)
    grid = (C.c_double * n_e)(*[float(e) for e in exponents])
    losses = (C.c_double * n_e)()
    best = C.c_int32(-1)
    s = torch.empty((K,), dtype=torch.float32, device=x.device)
    wq = torch.empty((K, N), dtype=torch.int8, device=x.device)
    sw = torch.empty((N,), dtype=torch.float32, device=x.device)
    if workspace is None:
        workspace = _ws(haq_quantize_layer_workspace_bytes(T, K, N, n_e), x.device)
    _check(lib().haq_quantize_layer(_ptr(x), C.c_int64(x.stride(0)), T, _ptr(w), K, N, grid, n_e, int(bool(use_weight)),
                                    C.c_double(percdamp), _ptr(s), _ptr(wq), _ptr(sw), losses, C.byref(best), _ptr(workspace),
                                    C.c_size_t(workspace.numel()), _stream()))
    return s, wq, sw, list(losses), int(best.value)
