"""CPU-only checks of the C ABI: the library loads, exports what include/haq.h
declares, and rejects bad arguments on the host before any HIP call."""
import ctypes as C
import os
import re

import numpy as np

import oracle
import paper_2508_07329_amd as haq
from paper_2508_07329_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    txt = open(os.path.join(ROOT, "include", "haq.h")).read()
    txt = re.sub(r"/\*.*?\*/", "", txt, flags=re.S)
    return sorted(set(re.findall(r"\b(haq_[a-z0-9_]+)\s*\(", txt)))


def test_every_declared_symbol_is_exported():
    L = haq.lib()
    names = _declared()
    assert set(names) == set(binding.EXPORTED_SYMBOLS)
    for n in names:
        assert getattr(L, n) is not None
    assert haq.haq_version() == 1


def test_sizes_and_layout_queries():
    assert haq.haq_packed_bytes(768, 3072) == 768 * 3072
    assert haq.haq_packed_bytes(64, 48) == 64 * 256          # output channels padded to 256
    assert haq.haq_packed_bytes(0, 5) == 0
    assert haq.haq_linear_workspace_bytes(2048, 4096, 16384) >= 2048 * 4096
    assert haq.haq_moe_workspace_bytes(64, 4096, 14336, 8) >= 128 * 14336 * 3


def test_argument_errors_are_reported_on_the_host():
    L = haq.lib()
    err = lambda: L.haq_last_error().decode()
    one = C.c_void_p(16)  # never dereferenced: validation fails first
    assert L.haq_smooth_quant_act(one, C.c_int64(64), None, -1, 64, one, C.c_int64(64), one, None) == -1
    assert "T=-1" in err()
    assert L.haq_smooth_quant_act(one, C.c_int64(100), None, 4, 100, one, C.c_int64(100), one, None) == -2
    assert L.haq_smooth_quant_act(None, C.c_int64(64), None, 4, 64, one, C.c_int64(64), one, None) == -1
    assert L.haq_smooth_quant_act(C.c_void_p(8), C.c_int64(64), None, 4, 64, one, C.c_int64(64), one, None) == -1
    assert "aligned" in err()
    assert L.haq_smooth_quant_act(one, C.c_int64(32), None, 4, 64, one, C.c_int64(64), one, None) == -1
    # T == 0 is a no-op that needs no buffers
    assert L.haq_smooth_quant_act(None, C.c_int64(64), None, 0, 64, None, C.c_int64(64), None, None) == 0
    z = C.c_size_t(0)
    assert L.haq_w8a8_linear(one, C.c_int64(64), None, one, one, 4, 64, 16, 7, one, C.c_int64(16), None, None, None,
                             None, z, None) == -2
    assert L.haq_w8a8_linear(one, C.c_int64(64), None, one, one, 4, 64, 16, 0, one, C.c_int64(16), None, None, None,
                             None, z, None) == -3
    assert "workspace" in err()
    assert L.haq_w8a8_linear(one, C.c_int64(64), None, one, one, 4, 64, 24, 0, one, C.c_int64(24), None, None, None,
                             None, z, None) == -2
    assert L.haq_moe_w8a8_ffn(None, one, C.c_int64(64), one, C.c_int64(8), None, one, 4, 64, 64, 8, 3, one,
                              C.c_int64(64), None, None, z, None) == -2
    assert "top_k" in err()
    assert L.haq_moe_w8a8_ffn(None, one, C.c_int64(64), one, C.c_int64(8), None, one, 4, 64, 64, 1, 2, one,
                              C.c_int64(64), None, None, z, None) == -2
    assert L.haq_pack_weight(one, 100, 16, one, None) == -2
    assert L.haq_quant_weight(None, None, 4, 4, one, one, None) == -1


def test_smoothing_vector_host_function_matches_oracle():
    rng = np.random.default_rng(0)
    ax = rng.uniform(0, 300, 257).astype(np.float32)
    aw = rng.uniform(0, 1, 257).astype(np.float32)
    ax[3] = 0
    aw[9] = 0
    L = haq.lib()
    for alpha, use_w in [(0.5, True), (0.3, True), (1.0, True), (0.0, True), (0.5, False)]:
        s = np.empty(257, np.float32)
        rc = L.haq_smoothing_vector(ax.ctypes.data_as(C.c_void_p), aw.ctypes.data_as(C.c_void_p) if use_w else None,
                                    257, C.c_double(alpha), s.ctypes.data_as(C.c_void_p))
        assert rc == 0
        assert np.array_equal(s, oracle.smoothing_vector(ax, aw if use_w else None, alpha))
    assert L.haq_smoothing_vector(ax.ctypes.data_as(C.c_void_p), None, 257, C.c_double(1.5), s.ctypes.data_as(C.c_void_p)) == -1


def test_n_critical_host_function_matches_oracle():
    rng = np.random.default_rng(5)
    cases = [(10.0, 1.0, 0.5), (10.1, 1.0, 0.5), (9.9, 1.0, 0.5), (0.0, 1.0, 0.5), (5.0, 1.0, 1.0), (5.0, 0.5, 1.0),
             (12.7e-3, 0.9e-3, 0.004e-3), (3.0, 0.25, 0.125)]
    cases += [tuple(rng.uniform(0.01, 20.0, 3)) for _ in range(200)]
    for t_e, lc, lg in cases:
        assert haq.haq_offload_n_critical(t_e, lc, lg) == oracle.n_critical(t_e, lc, lg), (t_e, lc, lg)
    import pytest
    with pytest.raises(haq.HaqError):
        haq.haq_offload_n_critical(-1.0, 1.0, 0.5)


def test_select_experts_host_function_matches_oracle():
    # the worked example of the oracle's pin, with dense frequency arrays
    paths = [[((0, 2), 5), ((3, 5), 40), ((5, 1), 30)]]
    freq = [[10, 30, 8, 45, 33, 70, 2, 31]]
    assert haq.haq_select_experts(1, 8, 3, 2, paths, freq) == [[3, 5, 1, 4, 7]]
    # random layers, ties included (integer frequencies from a small range)
    rng = np.random.default_rng(6)
    for trial in range(50):
        L, E = int(rng.integers(1, 5)), int(rng.integers(2, 17))
        top_k, supp = int(rng.integers(1, 5)), int(rng.integers(0, 4))
        path_stats, expert_freq = [], []
        for _ in range(L):
            n_paths = int(rng.integers(0, 7))
            path_stats.append([(tuple(int(e) for e in rng.choice(E, 2, replace=False)), int(rng.integers(0, 5)))
                               for _ in range(n_paths)])
            expert_freq.append([int(f) for f in rng.integers(0, 6, E)])
        ref = oracle.select_experts(L, top_k, supp, path_stats, [list(enumerate(f)) for f in expert_freq])
        got = haq.haq_select_experts(L, E, top_k, supp, path_stats, expert_freq)
        assert got == ref, (trial, path_stats, expert_freq, top_k, supp)


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr


def test_algorithm2_reproduces_the_resident_set_of_the_offload_workload():
    """The offload workload keeps experts 0-3 resident: that is Algorithm 2 on one layer applied to the
    popularity the workload draws its routing from (stage I: the most likely activation path, stage II: the
    next two experts by popularity; equal popularities keep index order)."""
    import itertools

    import haq_inputs as hi
    wl = hi.MIXTRAL_OFFLOAD
    pop = list(hi.OFFLOAD_POPULARITY[:wl.E])
    path_stats = [[((a, b), pop[a] * pop[b]) for a, b in itertools.combinations(range(wl.E), 2)]]
    sel = haq.haq_select_experts(1, wl.E, 2, 2, path_stats, [pop])
    assert sel == [[0, 1, 2, 3]] and sorted(sel[0]) == sorted(wl.resident)
    assert sel == oracle.select_experts(1, 2, 2, path_stats, [list(enumerate(pop))])


def test_lru_plan_follows_a_plain_lru_cache():
    """The cache planner of the offload path, batch after batch, against the oracle's LRU trace (which is
    pinned by the textbook reference string): same hits, same final content, and prev_user names exactly
    the earlier request of the same batch whose slot a request takes over."""
    rng = np.random.default_rng(11)
    for n_slots in (1, 2, 3, 5):
        keys, ticks, tick = [0] * n_slots, [0] * n_slots, 0
        trace, hits = [], []
        for _ in range(40):
            batch = [int(k) for k in rng.permutation(np.arange(1, 9))[:int(rng.integers(0, 7))]]
            so, hi, pu, keys, ticks, tick = haq.haq_lru_plan(keys, ticks, tick, batch)
            trace += batch
            hits += hi
            last = {}
            for k, (slot, h, prev) in enumerate(zip(so, hi, pu)):
                assert 0 <= slot < n_slots
                assert prev == (-1 if h else last.get(slot, -1))
                last[slot] = k
            for slot, k in last.items():
                assert keys[slot] == batch[k]
        hit_ref, cache_ref = oracle.lru_trace(trace, n_slots)
        assert hits == hit_ref
        assert sorted(k for k in keys if k) == sorted(cache_ref)
        # least recently used first = ascending last-use time
        assert [k for _, k in sorted((t, k) for t, k in zip(ticks, keys) if k)] == cache_ref
    L = haq.lib()
    two = (C.c_uint64 * 2)(5, 5)
    st = (C.c_uint64 * 2)()
    i2 = (C.c_int32 * 2)()
    assert L.haq_lru_plan(2, st, st, C.byref(C.c_uint64(0)), two, 2, i2, i2, i2) == -1
    assert "equal" in L.haq_last_error().decode()


def test_moe_rejects_misaligned_debug_buffers():
    L = haq.lib()
    one = C.c_void_p(16)
    descs = (binding._ExpertDesc * 2)()
    for d in descs:
        d.w13 = d.w2 = d.sw1 = d.sw3 = d.sw2 = d.s_mid = 16
    for field in ("q", "hq", "mid_fp16", "y_fp16"):
        dbg = binding._MoeDebug()
        setattr(dbg, field, 24)
        rc = L.haq_moe_w8a8_ffn(None, one, C.c_int64(64), one, C.c_int64(8), None, descs, 4, 64, 64, 2, 2, one,
                                C.c_int64(64), C.byref(dbg), one, C.c_size_t(0), None)
        assert rc == -1 and "debug buffers" in L.haq_last_error().decode(), field


def test_cpu_expert_matches_the_oracle_bit_for_bit_for_any_thread_count():
    """The host code of the offload runtime's option A (floating point on the dequantised copy) against the oracle's
    plain statement of it; it runs without a GPU."""
    import torch

    from tests import offline
    for seed, T, H, I in ((131, 7, 128, 320), (132, 1, 64, 192), (133, 21, 192, 448)):
        m = offline.small_moe(seed=seed, T=T, H=H, I=I, E=2)
        ex = m["experts"][1]
        ref, mid_ref = oracle.cpu_expert_ffn(m["X"], m["s_in"], oracle.cpu_expert(ex), dumps=True)
        t = lambda a: torch.from_numpy(np.ascontiguousarray(a))
        for keep_codes in (False, True):   # the binary32 copy made at load time; the codes dequantised in the inner loop
            h = haq.haq_cpu_expert_create(t(ex.w1), t(ex.w3), t(ex.w2), t(ex.sw1), t(ex.sw3), t(ex.sw2), t(ex.s_mid), keep_codes)
            try:
                for nt in (1, 3, 0):
                    y = haq.haq_cpu_expert_ffn(h, t(m["X"]), t(m["s_in"]), H, nt).numpy()
                    assert np.array_equal(y.view(np.uint16), ref.view(np.uint16)), (seed, nt, keep_codes)
                y0 = haq.haq_cpu_expert_ffn(h, t(m["X"]), None, H, 2).numpy()
                assert np.array_equal(y0.view(np.uint16), oracle.cpu_expert_ffn(m["X"], np.ones(H, np.float32), oracle.cpu_expert(ex)).view(np.uint16))
            finally:
                haq.haq_cpu_expert_destroy(h)
