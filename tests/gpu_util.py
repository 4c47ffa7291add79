"""Helpers shared by the GPU parity tests: upload oracle-quantised layers, compare."""
from __future__ import annotations

import concurrent.futures as cf

import numpy as np
import torch

import haq_inputs as hi
import oracle
import paper_2508_07329_amd as haq
from tests import offline

DEV = "cuda:0"


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().numpy()


def bits_equal(a: np.ndarray, b: np.ndarray) -> bool:
    a, b = np.ascontiguousarray(a), np.ascontiguousarray(b)
    assert a.shape == b.shape and a.dtype == b.dtype, (a.shape, b.shape, a.dtype, b.dtype)
    return np.array_equal(a.view(np.uint8), b.view(np.uint8))


def diff_report(gpu: np.ndarray, cpu: np.ndarray, n: int = 6) -> str:
    """Where and how two arrays differ bitwise (for assertion messages)."""
    g, c = np.ascontiguousarray(gpu), np.ascontiguousarray(cpu)
    if g.shape != c.shape or g.dtype != c.dtype:
        return f"shape/dtype {g.shape}{g.dtype} vs {c.shape}{c.dtype}"
    w = {1: np.uint8, 2: np.uint16, 4: np.uint32}[g.dtype.itemsize]
    bad = np.argwhere(g.view(w) != c.view(w))
    lines = [f"{len(bad)} of {g.size} differ"]
    for ix in bad[:n]:
        ix = tuple(int(i) for i in ix)
        lines.append(f"  {ix}: gpu {g[ix]!r} ({int(g.view(w)[ix]):#x}) cpu {c[ix]!r} ({int(c.view(w)[ix]):#x})")
    return "\n".join(lines)


def fp16_close(gpu: np.ndarray, cpu: np.ndarray) -> bool:
    """The stated floating-point bar: |gpu - cpu| <= 1e-3 |cpu| + 1e-3 rms(cpu row)."""
    g, c = gpu.astype(np.float64), cpu.astype(np.float64)
    rms = np.sqrt(np.mean(c ** 2, axis=-1, keepdims=True))
    return bool(np.all(np.abs(g - c) <= 1e-3 * np.abs(c) + 1e-3 * rms))


def upload_experts(experts: list[oracle.Expert]) -> list[haq.ExpertWeights]:
    out = []
    for ex in experts:
        w13 = haq.haq_pack_gate_up(dev(ex.w1), dev(ex.w3))
        w2 = haq.haq_pack_weight(dev(ex.w2))
        out.append(haq.ExpertWeights(w13, w2, dev(ex.sw1), dev(ex.sw3), dev(ex.sw2), dev(ex.s_mid)))
    torch.cuda.synchronize()
    return out


def mixtral_layer():
    """The Mixtral-shaped layer (seed 2), quantised offline by the oracle on 256
    calibration tokens.  Returns dict(s_in, experts (oracle), dev_experts)."""
    wl = hi.MIXTRAL_CALIB
    names = [(e, w) for e in range(wl.E) for w in ("w1", "w3", "w2")]
    with cf.ThreadPoolExecutor(8) as pool:
        mats = list(pool.map(lambda ew: hi.moe_weight(wl, *ew), names))
    weights = [tuple(mats[3 * e:3 * e + 3]) for e in range(wl.E)]
    X = hi.moe_hidden_states(wl)
    idx, _ = oracle.route_top2(hi.moe_logits(wl, X))
    s_in, experts = offline.quantize_moe(X, idx, weights)
    del weights, mats
    return dict(s_in=s_in, experts=experts, dev_experts=upload_experts(experts), dev_s_in=dev(s_in))
