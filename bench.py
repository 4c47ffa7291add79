#!/usr/bin/env python3
"""Benchmark of the smoothed W8A8 expert-FFN path on one MI355X.

Default workload: the OPT-6.7B-shaped FFN block (2048 tokens, 4096 -> 16384 ->
4096, ReLU, smoothing alpha 0.5), one "step" = the whole path over the batch:
quantise X, fc1 GEMM + ReLU epilogue, requantise, fc2 GEMM + epilogue.  Inputs
are seeded synthetic tensors already resident in HBM; weights are quantised and
packed once, outside the timed region, by the library's own offline kernels.

Prints ONE JSON line.  `roofline` is for the dominant kernel (the int8 MFMA
GEMM), timed with events around its launches; `cpu_baseline` is the CPU oracle
timed on a bounded sample of the same workload.  With no --workload the line
also carries `configs`: one record (time per step, metric, roofline, bounded
CPU-oracle baseline) for each of the other configurations of the metric -- the
OPT-125m linear, the Mixtral-shaped layer in prefill (4096 tokens, Zipf
routing), in decode (1, 8, 64 tokens: HBM GB/s and tokens/s) and with 4 of 8
experts streamed from host memory; the Mixtral layer is built once for all of them.

Single workloads (--workload): ffn, linear, moe_prefill, moe_decode_b1 / _b8 /
_b64, moe_offload, smooth_search and hessian_quant (the offline grid search of
the smoothing exponent and the Hessian-aware weight quantiser, on fc1 of the
default block), and gemm_sweep (the GEMM stage alone over shapes, K and rows).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_INT8_TOPS = 5033.0  # dense int8 MFMA, 256 CU x 8192 op/clk x 2.4 GHz
INT8_OPS_PER_CLOCK = 256 * 8192  # whole chip, per shader clock
PEAK_HBM_GBS = 8000.0
PEAK_FP64_TFLOPS = 78.6  # vector fp64 FMA
# Vector ALU issue rate for plain (unpacked, non-fused) fp32 instructions: 256 CU x 4 SIMD x 16 lanes
# x 2.4 GHz = 39.3 T lane-instructions/s (the published 157.3 TFLOP/s counts a packed FMA as 4 flop).
PEAK_VALU_TLANE_INSTR = 256 * 4 * 16 * 2.4e9 / 1e12
# fp32 vector instructions the activation-quantisation kernels spend per element (two divisions by reused
# divisors through reciprocals, absmax, rounding, packing; counted from rocprofv3 --pmc SQ_INSTS_VALU x 64
# lanes / elements, see profiles/): the kernel's ALU floor is this many lane-instructions per element
QUANT_VALU_PER_ELEMENT = 24.0
# Fabric-side bytes of one GEMM launch of the default workload (average of fc1 and fc2), from two
# rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE, each scaled by what the same counter reads for a plain
# 256 MiB device copy); the counters cannot be read from inside this process, so the figure is the one
# of the committed summary profiles/gemm_i8_kernel__opt6.7b_ffn.md and only applies to that workload.
GEMM_TRAFFIC_BYTES_OPT67B_FFN = 2.77e+08
# The same for the single GEMM launch of the small linear (16 x 768 x 3072: 3.29 MB read, 0.10 MB written) and for the
# grouped gate/up and down launches of the prefill layer (profiles/gemm_i8_kernel__mixtral_prefill.md).
GEMM_TRAFFIC_BYTES_OPT125M_LINEAR = 3.39e+06
PREFILL_TRAFFIC_BYTES = {"gate_up": 3.12e+09, "down": 1.93e+09}
# The same for one call of the decode layer (all its kernels; reads only, the writes are a few MB), from
# profiles/decode_kernels__mixtral_decode.md: within 0.3-2 % of the algorithmic weight bytes.
DECODE_TRAFFIC_BYTES = {"moe_decode_b1": 3.55e+08, "moe_decode_b8": 1.063e+09, "moe_decode_b64": 1.440e+09}


def _events(torch, n):
    return [torch.cuda.Event(enable_timing=True) for _ in range(n)]


SETTLE_SECONDS = 0.5


def _settle(torch, step, seconds=SETTLE_SECONDS):
    """Part of set-up, before the warm-up steps: the device comes out of idle with low clocks and needs a
    few tens of milliseconds of load before its clocks settle (the same step measures 350 us right after
    idle and 300 us from then on, for as long as the load lasts).  A serving process is never idle
    between steps, so the settled state is the one to measure."""
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        for _ in range(10):
            step()
        torch.cuda.synchronize()


def _time_steps(torch, step, steps, warmup, settle=SETTLE_SECONDS):
    _settle(torch, step, settle)
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def _stage_times(torch, haq, step, steps):
    """Average duration of every stage of a block-level call, from the events the library records at its
    stage boundaries on the launch stream (a second pass of `steps` steps, after the wall-clock one)."""
    haq.haq_profile_enable(True)
    try:
        acc = {}
        for _ in range(steps):
            step()
            for name, ms in haq.haq_profile_read():
                acc.setdefault(name, []).append(ms)
    finally:
        haq.haq_profile_enable(False)
    return {name: float(np.mean(v)) for name, v in acc.items()}


def _quant_record(name, rows, cols, ms):
    """An activation-quantisation kernel against its two bounds: HBM (3 bytes per element: fp16 in, int8 out)
    and the vector ALUs (QUANT_VALU_PER_ELEMENT lane-instructions per element)."""
    el = float(rows) * cols
    sec = ms * 1e-3
    return {"kernel": name, "rows": int(rows), "cols": int(cols), "ms": ms,
            "hbm": {"achieved": 3.0 * el / sec / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": 3.0 * el / sec / 1e9 / PEAK_HBM_GBS},
            "alu": {"achieved": QUANT_VALU_PER_ELEMENT * el / sec / 1e12, "peak": PEAK_VALU_TLANE_INSTR, "unit": "T lane-instr/s",
                    "frac": QUANT_VALU_PER_ELEMENT * el / sec / 1e12 / PEAK_VALU_TLANE_INSTR,
                    "lane_instr_per_element": QUANT_VALU_PER_ELEMENT}}


def _mfma_ceiling(torch, haq, data, work_groups, seconds, level=0):
    """Sustained rate of the pure-MFMA loop (operands in registers, no memory traffic) on `data`; level 1-3: the
    same loop with the GEMM kernel's K-loop ingredients added (LDS fragment reads; + barrier; + direct-to-LDS loads)."""
    iters = 20000
    out = torch.empty((256, 8, 16), dtype=torch.int32, device=data.device)
    if level == 0:
        launch = lambda: haq.haq_probe_mfma_i8(data, iters, work_groups, out=out)
    else:
        launch = lambda: haq.haq_probe_kloop_i8(data, level, iters, work_groups, out=out)
    ev = _events(torch, 2)
    launch()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    launch()
    torch.cuda.synchronize()
    n = max(3, int(seconds / max(time.perf_counter() - t0, 1e-4)))
    for _ in range(max(1, n // 3)):  # settle
        launch()
    side = torch.cuda.Stream()
    clk = torch.zeros((2,), dtype=torch.int64, device=data.device)
    torch.cuda.synchronize()  # the fill above is on this stream; the probe writes from another one
    for _ in range(max(1, n // 6)):
        launch()
    ev[0].record()
    for _ in range(n):
        launch()
    ev[1].record()
    haq.haq_probe_clock(1000000, out=clk, stream=side)  # 10 ms of the loop's steady state, from a second stream
    torch.cuda.synchronize()
    sec = ev[0].elapsed_time(ev[1]) * 1e-3
    c, w = (int(v) for v in clk.tolist())
    return n * work_groups * 4.0 * iters * 32 * 65536 / sec / 1e12, sec, c / max(w, 1) * 100.0


def _fragment_sets(torch, q_packed, R, w_packed, Npad):
    """24 KiB of operand fragments for the MFMA probe cut out of packed operands of the workload: four sets of
    2 token + 4 weight fragments, each 32 rows x 32 consecutive k (two neighbouring 16-byte chunks)."""
    qa = q_packed.view(-1, R, 16)
    wb = w_packed.view(-1, Npad, 16)
    g = torch.Generator(device="cpu").manual_seed(0)
    frags = []
    for _ in range(4):
        for src, rows, n in ((qa, R - 256 - 32, 2), (wb, Npad - 32, 4)):
            for _ in range(n):
                c = int(torch.randint(0, src.shape[0] // 2, (1,), generator=g)) * 2
                r = int(torch.randint(0, max(1, rows), (1,), generator=g))
                frags.append(torch.cat([src[c, r:r + 32].reshape(-1), src[c + 1, r:r + 32].reshape(-1)]))
    return torch.cat(frags).contiguous()


def _clock_mhz_under(torch, haq, launch, n_launches, ticks=300000):
    """Shader clock while `launch` x n_launches run on the current stream, read by a one-wave probe on a second
    stream (default priority) that spins for `ticks` periods of the 100 MHz counter."""
    side = torch.cuda.Stream()
    out = torch.zeros((2,), dtype=torch.int64, device="cuda:0")
    torch.cuda.synchronize()
    for _ in range(n_launches):
        launch()
    haq.haq_probe_clock(ticks, out=out, stream=side)
    torch.cuda.synchronize()
    c, w = (int(v) for v in out.tolist())
    return c / max(w, 1) * 100.0


def bench_ffn(args, torch, haq, hi, cpu_seconds=10.0):
    wl = hi.OPT67B_FFN if args.workload in ("ffn", "all") else None
    dev = "cuda:0"
    if wl is not None:
        T, K, F, name = wl.T, wl.H, wl.F, wl.name
        X_h, _, _ = hi.hidden_states(wl.seed, T, K, wl.n_outlier, wl.mult)
        W1_h = hi.gaussian_weight(wl.seed, 0, K, F)
        W2_h = hi.gaussian_weight(wl.seed, 1, F, K)
        n_out = K
    else:  # single OPT-125m linear
        l = hi.OPT125M_LINEAR
        T, K, F, name = l.T, l.K, l.N, l.name
        X_h, _, _ = hi.hidden_states(l.seed, T, K, l.n_outlier, l.mult)
        W1_h = hi.gaussian_weight(l.seed, 0, K, F)
        W2_h = None
        n_out = F
    X = torch.from_numpy(X_h).to(dev)

    def offline(x, w_h):
        w = torch.from_numpy(w_h).to(dev)
        s = haq.haq_smoothing_vector(haq.haq_channel_absmax_f16(x), haq.haq_weight_row_absmax(w), 0.5)
        wq, sw = haq.haq_quant_weight(w, s)
        return s, haq.haq_pack_weight(wq), sw

    torch.cuda.synchronize()
    t_off = time.perf_counter()
    s1, w1p, sw1 = offline(X, W1_h)
    torch.cuda.synchronize()
    t_off = time.perf_counter() - t_off  # upload + magnitudes + s + Q(W s) + packing of one matrix (not in the metric)
    ws1 = torch.empty(haq.haq_linear_workspace_bytes(T, K, F), dtype=torch.uint8, device=dev)
    h = torch.empty((T, F), dtype=torch.float16, device=dev)
    haq.haq_w8a8_linear(X, s1, w1p, sw1, F, haq.HAQ_ACT_RELU, out=h, workspace=ws1)
    two = W2_h is not None
    if two:
        s2, w2p, sw2 = offline(h, W2_h)
        y = torch.empty((T, K), dtype=torch.float16, device=dev)
        wsf = torch.empty(haq.haq_ffn_workspace_bytes(T, K, F, K), dtype=torch.uint8, device=dev)

    def step():
        if two:  # the whole block in one call: quantise, fc1 + ReLU, requantise, fc2
            haq.haq_w8a8_ffn(X, s1, w1p, sw1, F, haq.HAQ_ACT_RELU, s2, w2p, sw2, K, out=y, workspace=wsf)
        else:
            haq.haq_w8a8_linear(X, s1, w1p, sw1, F, haq.HAQ_ACT_RELU, out=h, workspace=ws1)

    sec = _time_steps(torch, step, args.steps, args.warmup)
    ops_per_gemm = 2.0 * T * K * F
    n_gemm = 2 if two else 1
    tops = n_gemm * ops_per_gemm / sec / 1e12

    # dominant kernel (int8 GEMM + epilogue) and the quantisation kernels, events around each launch
    q1, sx1 = haq.haq_quant_act_packed(X, s1)
    if two:
        q2, sx2 = haq.haq_quant_act_packed(h, s2)
    per = 2 * n_gemm + 1
    ev = _events(torch, per * args.steps)
    torch.cuda.synchronize()
    for i in range(args.steps):
        ev[per * i].record()
        haq.haq_quant_act_packed(X, s1, q_packed=q1, row_scale=sx1)
        ev[per * i + 1].record()
        haq.haq_gemm_w8a8_packed(q1, sx1, w1p, sw1, T, K, F, haq.HAQ_ACT_RELU, out=h)
        ev[per * i + 2].record()
        if two:
            haq.haq_quant_act_packed(h, s2, q_packed=q2, row_scale=sx2)
            ev[per * i + 3].record()
            haq.haq_gemm_w8a8_packed(q2, sx2, w2p, sw2, T, F, K, haq.HAQ_ACT_NONE, out=y)
            ev[per * i + 4].record()
    torch.cuda.synchronize()
    span = lambda j: float(np.mean([ev[per * i + j].elapsed_time(ev[per * i + j + 1]) for i in range(args.steps)]))
    gemm_ms = [span(1)] + ([span(3)] if two else [])
    gemm_avg = float(np.mean(gemm_ms)) * 1e-3
    achieved = ops_per_gemm / gemm_avg / 1e12
    quant = [_quant_record("activation quantisation of X (fp16 -> packed int8 + row scales)", T, K, span(0))]
    if two:
        quant.append(_quant_record("requantisation of the fp16 intermediate", T, F, span(2)))

    roof = {"bound": "mfma", "kernel": "gemm_i8_kernel (int8 MFMA GEMM + dequant epilogue)",
            "achieved": achieved, "peak": PEAK_INT8_TOPS, "unit": "TOP/s", "frac": achieved / PEAK_INT8_TOPS,
            "avg_launch_ms": gemm_avg * 1e3, "launch_ms": gemm_ms, "ops_per_launch": ops_per_gemm,
            "traffic": GEMM_TRAFFIC_BYTES_OPT67B_FFN if wl is not None else GEMM_TRAFFIC_BYTES_OPT125M_LINEAR,
            "traffic_unit": "bytes per launch"}
    if two and not args.no_ceilings:
      try:
        # the peak at the clock the chip really runs this kernel at, and what the matrix cores sustain on a
        # pure-MFMA loop (no memory traffic at all) fed with operands of this very workload and with uniform
        # random codes: the distance from the nominal peak that no kernel design can recover on this data
        gemm1 = lambda: haq.haq_gemm_w8a8_packed(q1, sx1, w1p, sw1, T, K, F, haq.HAQ_ACT_RELU, out=h)
        _settle(torch, gemm1, 0.2)
        mhz = float(np.median([_clock_mhz_under(torch, haq, gemm1, 80) for _ in range(3)]))
        roof["clock_mhz_under_kernel"] = mhz
        roof["peak_measured"] = INT8_OPS_PER_CLOCK * mhz * 1e6 / 1e12
        roof["frac_measured"] = achieved / roof["peak_measured"]
        R, Npad = int(haq.haq_packed_act_rows(T)), (F + 255) // 256 * 256
        data_wl = _fragment_sets(torch, q1, R, w1p, Npad)
        g = torch.Generator(device="cuda:0").manual_seed(1)
        data_rnd = torch.randint(-127, 128, (24576,), dtype=torch.int8, device=dev, generator=g)
        ceil = {}
        for label, data in (("workload_codes", data_wl), ("uniform_random_codes", data_rnd)):
            for wgs, tag in ((256, "1_wave_per_simd"), (512, "2_waves_per_simd")):
                v, dur, clk = _mfma_ceiling(torch, haq, data, wgs, 0.5)
                ceil[f"{label}/{tag}"] = {"TOPs": v, "seconds": dur, "clock_mhz": clk}
        best = max(v["TOPs"] for k, v in ceil.items() if k.startswith("workload_codes"))
        roof["sustained_mfma_ceiling"] = ceil
        roof["peak_sustained"] = best
        roof["frac_sustained"] = achieved / best
        # the same loop (two work-groups per CU, workload codes) with the K loop's ingredients added one at a time:
        # what each of them costs the matrix pipes; the GEMM's own K-loop rate follows from gemm_sweep's K sweep
        ladder = {"0_mfma_only_registers": ceil["workload_codes/2_waves_per_simd"]["TOPs"]}
        for level, label in ((1, "1_plus_lds_fragment_reads"), (2, "2_plus_barrier_per_k_step"), (3, "3_plus_direct_to_lds_loads_from_l2"),
                             (4, "4_as_3_but_refill_through_registers")):
            v, dur, clk = _mfma_ceiling(torch, haq, data_wl, 512, 0.3, level=level)
            ladder[label] = v
            ladder[label + "_clock_mhz"] = clk
        roof["k_loop_ladder_TOPs"] = ladder
      except Exception as exc:  # noqa: BLE001 - the probes are aids: their failure is reported, the measurement stands
        roof["ceilings_error"] = f"{type(exc).__name__}: {exc}"

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        n_rows = min(T, args.cpu_rows)
        rows = np.arange(n_rows)
        so1 = oracle.smoothing_vector(oracle.col_absmax_f16(X_h), oracle.row_absmax_f32(W1_h), 0.5)
        W1q, swo1 = oracle.quant_weight(W1_h, so1)
        if two:
            h_all = oracle.w8a8_linear(X_h[rows], so1, W1q, swo1, "relu")
            so2 = oracle.smoothing_vector(oracle.col_absmax_f16(h_all), oracle.row_absmax_f32(W2_h), 0.5)
            W2q, swo2 = oracle.quant_weight(W2_h, so2)
        reps, dt = 0, 0.0
        while dt < cpu_seconds and reps < 1000:
            t0 = time.perf_counter()
            hh = oracle.w8a8_linear(X_h[rows], so1, W1q, swo1, "relu")
            if two:
                oracle.w8a8_linear(hh, so2, W2q, swo2, "none")
            dt += time.perf_counter() - t0
            reps += 1
        cpu = {"value": reps * n_gemm * 2.0 * n_rows * K * F / dt / 1e12, "unit": "TOPS", "cores": oracle.num_threads(),
               "kind": "oracle",
               "sample": f"first {n_rows} of {T} token rows through the whole {'block' if two else 'linear'}, {reps} repetitions, {dt:.2f} s"}

    return {
        "metric": "W8A8 expert-FFN int8 TOPS (prefill)", "value": tops, "unit": "TOPS",
        "ms_per_step": sec * 1e3, "dtype": "int8",
        "config": {"workload": name, "tokens": T, "in_features": K, "hidden_features": F, "out_features": n_out,
                   "act": "relu", "smoothing_alpha": 0.5, "gemms_per_step": n_gemm},
        "offline_quantise_and_pack_ms_per_matrix": t_off * 1e3,
        "roofline": roof, "other_kernels": quant,
        "cpu_baseline": cpu,
    }


# ---- the Mixtral-shaped layer: built once, shared by the prefill, decode and offload records -------------
def build_mixtral(torch, haq, hi, keep_host=False):
    """Offline quantisation of the layer by the library's own kernels: s_in from 256 calibration tokens and all
    gate/up matrices, s_mid per expert from the library's own intermediate on the calibration tokens."""
    dev = "cuda:0"
    wl = cal = hi.MIXTRAL_CALIB
    H, I, E = wl.H, wl.I, wl.E
    Xc = torch.from_numpy(hi.moe_hidden_states(cal)).to(dev)
    ax = haq.haq_channel_absmax_f16(Xc)
    aw = torch.zeros(H, dtype=torch.float32, device=dev)
    from concurrent.futures import ThreadPoolExecutor
    names = [(e, w) for e in range(E) for w in ("w1", "w3", "w2")]
    with ThreadPoolExecutor(8) as pool:
        host_mats = list(pool.map(lambda ew: hi.moe_weight(wl, *ew), names))
    mats = {ew: torch.from_numpy(m).to(dev) for ew, m in zip(names, host_mats)}
    if not keep_host:
        host_mats = None
    for e in range(E):
        haq.haq_weight_row_absmax(mats[(e, "w1")], aw)
        haq.haq_weight_row_absmax(mats[(e, "w3")], aw)
    s_in = haq.haq_smoothing_vector(ax, aw, 0.5)
    ones = torch.ones(I, dtype=torch.float32, device=dev)
    stage1, cs13, colsums = [], [], []
    for e in range(E):
        w1q, sw1 = haq.haq_quant_weight(mats[(e, "w1")], s_in)
        w3q, sw3 = haq.haq_quant_weight(mats[(e, "w3")], s_in)
        w2q, sw2 = haq.haq_quant_weight(mats[(e, "w2")], None)
        stage1.append(haq.ExpertWeights(haq.haq_pack_gate_up(w1q, w3q), haq.haq_pack_weight(w2q), sw1, sw3, sw2, ones))
        cs13.append((haq.haq_weight_colsum(w1q), haq.haq_weight_colsum(w3q)))
    cal_logits = torch.from_numpy(hi.moe_logits(cal, hi.moe_hidden_states(cal))).to(dev)
    _, dbg = haq.haq_moe_w8a8_ffn(Xc, cal_logits, s_in, stage1, I, debug=True)
    offs = dbg.offsets.cpu().numpy()
    experts, canon = [], {}
    cold = [e for e in range(E) if e not in hi.MIXTRAL_OFFLOAD.resident]
    for e in range(E):
        rows = dbg.mid_fp16[offs[e]:offs[e + 1]]
        ax_mid = haq.haq_channel_absmax_f16(rows) if rows.shape[0] else torch.zeros(I, dtype=torch.float32, device=dev)
        s_mid = haq.haq_smoothing_vector(ax_mid, haq.haq_weight_row_absmax(mats[(e, "w2")]), 0.5)
        w2q, sw2 = haq.haq_quant_weight(mats[(e, "w2")], s_mid)
        st = stage1[e]
        experts.append(haq.ExpertWeights(st.w13, haq.haq_pack_weight(w2q), st.sw1, st.sw3, sw2, s_mid))
        colsums.append((cs13[e][0], cs13[e][1], haq.haq_weight_colsum(w2q)))  # for the asymmetric-code variant
        if e in cold:  # canonical codes of the experts the offload workload keeps in host memory (for their CPU copies)
            w1q, _ = haq.haq_quant_weight(mats[(e, "w1")], s_in)
            w3q, _ = haq.haq_quant_weight(mats[(e, "w3")], s_in)
            canon[e] = tuple(t.cpu().contiguous() for t in (w1q, w3q, w2q, st.sw1, st.sw3, sw2, s_mid))
    del mats, stage1, dbg
    torch.cuda.synchronize()
    return {"s_in": s_in, "experts": experts, "host_mats": host_mats, "sets": None, "oracle": None, "canon": canon,
            "colsums": colsums}


def oracle_mixtral(hi, host_mats=None):
    """The CPU oracle's own copy of the layer, quantised offline by the oracle itself (smoothing vectors from
    the 256 calibration tokens, alpha 0.5)."""
    import oracle
    from concurrent.futures import ThreadPoolExecutor
    cal = hi.MIXTRAL_CALIB
    H, I, E = cal.H, cal.I, cal.E
    if host_mats is None:
        names = [(e, w) for e in range(E) for w in ("w1", "w3", "w2")]
        with ThreadPoolExecutor(8) as pool:
            host_mats = list(pool.map(lambda ew: hi.moe_weight(cal, *ew), names))
    mats = host_mats
    Xc = hi.moe_hidden_states(cal)
    idx_c, _ = oracle.route_top2(hi.moe_logits(cal, Xc))
    aw = np.zeros(H, np.float32)
    for e in range(E):
        oracle.row_absmax_f32(mats[3 * e], aw)
        oracle.row_absmax_f32(mats[3 * e + 1], aw)
    s_in = oracle.smoothing_vector(oracle.col_absmax_f16(Xc), aw, 0.5)
    ones = np.ones(I, np.float32)
    stage1 = []
    for e in range(E):
        w1q, sw1 = oracle.quant_weight(mats[3 * e], s_in)
        w3q, sw3 = oracle.quant_weight(mats[3 * e + 1], s_in)
        stage1.append(oracle.Expert(w1q, w3q, np.zeros((I, H), np.int8), sw1, sw3, np.zeros(H, np.float32), ones))
    ax_mid = oracle.moe_mid_absmax(Xc, idx_c, s_in, stage1)
    experts = []
    for e in range(E):
        s_mid = oracle.smoothing_vector(ax_mid[e], oracle.row_absmax_f32(mats[3 * e + 2]), 0.5)
        w2q, sw2 = oracle.quant_weight(mats[3 * e + 2], s_mid)
        st = stage1[e]
        experts.append(oracle.Expert(st.w1, st.w3, w2q, st.sw1, st.sw3, sw2, s_mid))
    return {"s_in": s_in, "experts": experts}


def _moe_workload(hi, name):
    if name == "moe_prefill":
        return hi.MIXTRAL_PREFILL
    if name == "moe_offload":
        return hi.MIXTRAL_OFFLOAD
    return {w.T: w for w in hi.MIXTRAL_DECODE}[int(name.rsplit("b", 1)[1])]


def bench_moe(args, torch, haq, hi, workload, layer, cpu_seconds=10.0):
    dev = "cuda:0"
    wl = _moe_workload(hi, workload)
    T, H, I, E = wl.T, wl.H, wl.I, wl.E
    s_in, experts = layer["s_in"], layer["experts"]
    X_h = hi.moe_hidden_states(wl)
    logits_h = hi.moe_logits(wl, X_h)
    X, logits = torch.from_numpy(X_h).to(dev), torch.from_numpy(logits_h).to(dev)
    ws = torch.empty(haq.haq_moe_workspace_bytes(T, H, I, E), dtype=torch.uint8, device=dev)
    out = torch.empty((T, H), dtype=torch.float16, device=dev)
    _, dbg = haq.haq_moe_w8a8_ffn(X, logits, s_in, experts, I, debug=("counts",))
    counts = dbg.counts.cpu().numpy()
    prefill = workload == "moe_prefill"
    if workload == "moe_offload":
        res = bench_offload(args, torch, haq, wl, X, logits, s_in, experts, counts, ws, out, layer.get("canon"))
    else:
        res = _bench_moe_resident(args, torch, haq, hi, wl, workload, layer, X, logits, counts, ws)
    if not args.no_cpu_baseline:
        if layer["oracle"] is None:
            layer["oracle"] = oracle_mixtral(hi, layer["host_mats"])
            layer["host_mats"] = None
        res["cpu_baseline"] = _moe_cpu_baseline(layer["oracle"], wl, X_h, logits_h, prefill, workload == "moe_offload", cpu_seconds)
    return res


def _bench_moe_resident(args, torch, haq, hi, wl, workload, layer, X, logits, counts, ws):
    dev = "cuda:0"
    T, H, I, E = wl.T, wl.H, wl.I, wl.E
    s_in, experts = layer["s_in"], layer["experts"]
    prefill = workload == "moe_prefill"
    # Inputs of one step.  Decode is bound by reading each activated expert's weights once, and in a
    # model no weight is touched twice per token; here one layer is replayed, and the 256 MB last-level
    # cache would keep part of a working set that comes round again too soon.  So a replay walks over
    # four copies of the layer's weights at distinct addresses (5.6 GB between two reads of the same
    # bytes), and the single-token step in addition over four tokens (drawn from the 64-token batch of
    # the same workload family) whose expert pairs are disjoint.
    pool = [(X, logits)]
    if T == 1:
        wl64 = {w.T: w for w in hi.MIXTRAL_DECODE}[64]
        X64_h = hi.moe_hidden_states(wl64)
        L64_h = hi.moe_logits(wl64, X64_h)
        X64, L64 = torch.from_numpy(X64_h).to(dev), torch.from_numpy(L64_h).to(dev)
        _, d64 = haq.haq_moe_w8a8_ffn(X64, L64, s_in, experts, I, debug=("topk_idx",))
        pairs = d64.topk_idx.cpu().numpy()
        chosen, used = [], set()
        for t in range(64):
            if not (set(pairs[t].tolist()) & used):
                chosen.append(t)
                used |= set(pairs[t].tolist())
        pool = [(X64[t:t + 1].contiguous(), L64[t:t + 1].contiguous()) for t in chosen]
    n_sets = 1 if prefill else 4
    if n_sets > 1 and layer["sets"] is None:
        layer["sets"] = [[haq.ExpertWeights(ex.w13.clone(), ex.w2.clone(), ex.sw1, ex.sw3, ex.sw2, ex.s_mid) for ex in experts]
                         for _ in range(n_sets - 1)]
    sets = [experts] + (layer["sets"] if n_sets > 1 else [])
    calls = [(x_i, l_i, ws_i) for ws_i in sets for (x_i, l_i) in pool]
    outs = [torch.empty((T, H), dtype=torch.float16, device=dev) for _ in calls]
    torch.cuda.synchronize()
    # the launch sequence of one step is captured once and replayed: the decode layer is a handful
    # of short kernels and would otherwise be bound by host launch overhead
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for (x_i, l_i, ex_i), o_i in zip(calls, outs):
            haq.haq_moe_w8a8_ffn(x_i, l_i, s_in, ex_i, I, out=o_i, workspace=ws)

    def step():
        graph.replay()

    sec = _time_steps(torch, step, args.steps, args.warmup) / len(calls)
    eager = haq.haq_moe_w8a8_ffn(pool[0][0], pool[0][1], s_in, experts, I)
    torch.cuda.synchronize()
    if not torch.equal(eager, outs[0]):
        raise SystemExit("bench.py: graph replay and eager call disagree")
    # stage durations from the library's own events (eager launches over the same inputs)
    k = [0]

    def eager_step():
        x_i, l_i, ex_i = calls[k[0] % len(calls)]
        k[0] += 1
        haq.haq_moe_w8a8_ffn(x_i, l_i, s_in, ex_i, I, out=outs[0], workspace=ws)

    stages = _stage_times(torch, haq, eager_step, max(args.steps, len(calls)))
    # the same layer with asymmetric activation codes (uint8 with zero points; same weights, same launch recipe)
    ws_a = torch.empty(haq.haq_moe_asym_workspace_bytes(T, H, I, E), dtype=torch.uint8, device=dev)
    graph_a = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph_a):
        for (x_i, l_i, ex_i), o_i in zip(calls, outs):
            haq.haq_moe_w8a8_ffn_asym(x_i, l_i, s_in, ex_i, layer["colsums"], I, out=o_i, workspace=ws_a)
    sec_a = _time_steps(torch, graph_a.replay, max(5, args.steps // 4), max(2, args.warmup // 4), settle=0.2) / len(calls)
    del graph_a, ws_a
    pairs = int(counts.sum())
    ops = pairs * 2.0 * 3 * H * I
    n_active = int((counts > 0).sum())
    w_bytes = n_active * (3.0 * H * I + 4.0 * (2 * I + H + I))
    res = {
        "ms_per_step": sec * 1e3, "dtype": "int8",
        "config": {"workload": wl.name, "tokens": T, "hidden": H, "intermediate": I, "experts": E, "top_k": 2,
                   "pairs_per_expert": counts.tolist(), "activated_experts": n_active,
                   "launch": "hipGraph replay", "calls_per_replay": len(calls), "weight_copies": n_sets},
        "tokens_per_s": T / sec, "layer_tops": ops / sec / 1e12, "weight_stream_GBs": w_bytes / sec / 1e9,
        "stage_ms_eager": stages, "cpu_baseline": None,
        "asymmetric_codes": {"entry_point": "haq_moe_w8a8_ffn_asym", "ms_per_step": sec_a * 1e3, "vs_symmetric": sec_a / sec},
    }
    if prefill:
        res.update(metric="W8A8 expert-FFN int8 TOPS (prefill)", value=ops / sec / 1e12, unit="TOPS")
        gu_ms = stages.get("grouped gate/up GEMM + SwiGLU")
        dn_ms = stages.get("grouped down GEMM")
        gu_ops, dn_ops = pairs * 2.0 * H * 2 * I, pairs * 2.0 * I * H
        n_active_e = int((counts > 0).sum())
        res["roofline"] = {"bound": "mfma", "kernel": "gemm_i8_kernel, grouped gate/up launch (int8 MFMA GEMM + SwiGLU epilogue)",
                           "achieved": gu_ops / (gu_ms * 1e-3) / 1e12, "peak": PEAK_INT8_TOPS, "unit": "TOP/s",
                           "frac": gu_ops / (gu_ms * 1e-3) / 1e12 / PEAK_INT8_TOPS, "avg_launch_ms": gu_ms, "ops_per_launch": gu_ops,
                           "down_launch": {"achieved": dn_ops / (dn_ms * 1e-3) / 1e12, "frac": dn_ops / (dn_ms * 1e-3) / 1e12 / PEAK_INT8_TOPS,
                                           "avg_launch_ms": dn_ms, "ops_per_launch": dn_ops,
                                           "traffic": PREFILL_TRAFFIC_BYTES["down"],
                                           "algorithmic_bytes": pairs * I + n_active_e * I * H + pairs * H * 2.0},
                           "whole_layer": {"achieved": ops / sec / 1e12, "frac": ops / sec / 1e12 / PEAK_INT8_TOPS},
                           "traffic": PREFILL_TRAFFIC_BYTES["gate_up"], "traffic_unit": "bytes per launch",
                           "algorithmic_bytes": pairs * H + n_active_e * 2.0 * H * I + pairs * I * 2.0}
        res["other_kernels"] = [
            _quant_record("requantisation of the fp16 intermediate (per-expert smoothing vectors)", pairs, I,
                          stages.get("requantise intermediate"))]
    else:
        res.update(metric="MoE layer tokens/s (decode)", value=T / sec, unit="tokens/s")
        res["roofline"] = {"bound": "hbm", "kernel": "whole layer (expert weight streaming dominates)",
                           "achieved": w_bytes / sec / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                           "frac": w_bytes / sec / 1e9 / PEAK_HBM_GBS, "algorithmic_bytes": w_bytes,
                           "traffic": DECODE_TRAFFIC_BYTES.get(workload), "traffic_unit": "bytes per layer call"}
    return res


def _moe_cpu_baseline(ol, wl, X_h, logits_h, prefill, offload, seconds):
    """The CPU oracle on a bounded sample of the MoE workload: whole tokens through routing, both expert FFNs
    and the combination (`ol`: the oracle's own copy of the layer)."""
    import oracle
    H, I = wl.H, wl.I
    idx, gw = oracle.route_top2(logits_h)
    n_tok = min(wl.T, 32)
    tokens = np.arange(n_tok)
    reps, dt = 0, 0.0
    while dt < seconds and reps < 1000:
        t0 = time.perf_counter()
        oracle.moe_ffn(X_h, idx, gw, ol["s_in"], ol["experts"], tokens=tokens)
        dt += time.perf_counter() - t0
        reps += 1
    if prefill:
        value, unit = reps * n_tok * 2 * 2.0 * 3 * H * I / dt / 1e12, "TOPS"
    elif offload:
        value, unit = dt / reps * wl.T / n_tok * 1e3, "ms"   # the whole 256-token layer at the sampled rate
    else:
        value, unit = reps * n_tok / dt, "tokens/s"
    return {"value": value, "unit": unit, "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"first {n_tok} of {wl.T} tokens through the whole layer (weights in host memory), {reps} repetitions, {dt:.2f} s"
                      + (f"; scaled to {wl.T} tokens" if offload else "")}


def _offload_policy(torch, haq, wl, X, logits, s_in, experts, mixed, cold, counts, canon, t_copy_per_expert, t_gpu_per_pair):
    """Section III.C.1a-b on this machine: the cost model of Eq. 7-8 calibrated here (CPU latency per token of an expert on its
    dequantised copy, GPU latency per pair, transfer time of one expert), the break-even batch, and the layer with the
    rule in force: for this workload's batches, and for a single token (the decode case the paper argues from)."""
    T, H, I = wl.T, wl.H, wl.I
    # the CPU experts keep the int8 codes and form float(code) * scale in the inner loop (same values as the binary32
    # copy made at load time, a quarter of the host memory traffic); one binary32-copy handle is timed beside it
    handles = {e: haq.haq_cpu_expert_create(*canon[e], keep_codes=True) for e in cold}
    s_host = s_in.cpu()
    e0 = cold[0]
    x_host = X[:8].cpu()

    def cpu_ms(h, n):
        haq.haq_cpu_expert_ffn(h, x_host[:n], s_host, H)
        t0 = time.perf_counter()
        for _ in range(3):
            haq.haq_cpu_expert_ffn(h, x_host[:n], s_host, H)
        return (time.perf_counter() - t0) / 3

    lat = {n: cpu_ms(handles[e0], n) for n in (1, 8)}
    h32 = haq.haq_cpu_expert_create(*canon[e0])
    lat32 = cpu_ms(h32, 1)
    haq.haq_cpu_expert_destroy(h32)
    # Eq. 7 is linear in the batch while the CPU expert's cost is concave (one pass over the weights serves up to four
    # rows): the per-token latency measured near the break-even batch is the one that places n_critical correctly
    latency_cpu = lat[8] / 8
    ctx = haq.haq_ctx_create(H, I, 2)
    res = {"t_e_ms": t_copy_per_expert * 1e3, "latency_cpu_ms_per_token": latency_cpu * 1e3,
           "cpu_expert_ms": {"1_token": lat[1] * 1e3, "8_tokens": lat[8] * 1e3, "1_token_on_the_binary32_copy": lat32 * 1e3},
           "latency_gpu_ms_per_token": t_gpu_per_pair * 1e3,
           "cpu_copy": "int8 codes in blocks of eight output channels, dequantised in the inner loop (3 H I bytes per expert)"}
    try:
        haq.haq_ctx_set_offload_policy(ctx, t_copy_per_expert, latency_cpu, t_gpu_per_pair, s_host)
        for e in cold:
            haq.haq_ctx_register_cpu_expert(ctx, mixed[e], handles[e])
        out = torch.empty((T, H), dtype=torch.float16, device=X.device)
        ws = torch.empty(haq.haq_moe_workspace_bytes(T, H, I, wl.E), dtype=torch.uint8, device=X.device)

        def timed(x, l, o, reps):
            haq.haq_ctx_cache_invalidate(ctx)
            haq.haq_moe_w8a8_ffn(x, l, s_in, mixed, I, ctx=ctx, out=o, workspace=ws)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                haq.haq_ctx_cache_invalidate(ctx)   # cold cache every call, as in the streamed measurement
                haq.haq_moe_w8a8_ffn(x, l, s_in, mixed, I, ctx=ctx, out=o, workspace=ws)
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / reps

        names = {0: "gpu_cached", 1: "transfer", 2: "cpu"}
        ms = timed(X, logits, out, 5) * 1e3
        dec, nc = haq.haq_ctx_last_decisions(ctx)
        res.update(n_critical=nc, layer_ms=ms, decisions=[{"expert": e, "n_inputs": n, "decision": names[d]} for e, n, d in dec])
        # one token routed to two host-resident experts (logits forced), with the rule and with plain transfers
        l1 = torch.full((1, wl.E), -30.0, dtype=torch.float16, device=X.device)
        l1[0, cold[0]], l1[0, cold[1]] = 5.0, 4.0
        o1 = torch.empty((1, H), dtype=torch.float16, device=X.device)
        ms1 = timed(X[:1], l1, o1, 5) * 1e3
        dec1, _ = haq.haq_ctx_last_decisions(ctx)
        haq.haq_ctx_set_offload_policy(ctx, -1.0, 0.0, 0.0)
        ms1_t = timed(X[:1], l1, o1, 5) * 1e3
        res["single_token_two_host_experts"] = {"with_rule_ms": ms1, "decisions": [names[d] for _, _, d in dec1], "always_transfer_ms": ms1_t}
    finally:
        torch.cuda.synchronize()
        haq.haq_ctx_destroy(ctx)
        for h in handles.values():
            haq.haq_cpu_expert_destroy(h)
    return res


def bench_offload(args, torch, haq, wl, X, logits, s_in, experts, counts, ws, out, canon=None):
    """4 of 8 experts resident; the others are streamed from pinned host memory on every call."""
    T, H, I, E = wl.T, wl.H, wl.I, wl.E
    cold = [e for e in range(E) if e not in wl.resident]
    mixed = []
    for e, ex in enumerate(experts):
        if e in cold:
            w13 = torch.empty(ex.w13.shape, dtype=torch.int8, pin_memory=True).copy_(ex.w13)
            w2 = torch.empty(ex.w2.shape, dtype=torch.int8, pin_memory=True).copy_(ex.w2)
            mixed.append(haq.ExpertWeights(w13, w2, ex.sw1, ex.sw3, ex.sw2, ex.s_mid, haq.HAQ_LOC_HOST_PINNED))
        else:
            mixed.append(ex)
    torch.cuda.synchronize()
    steps = max(3, min(args.steps, 20))
    ctx = haq.haq_ctx_create(H, I, 2)
    ref = haq.haq_moe_w8a8_ffn(X, logits, s_in, experts, I)
    t_all_resident = _time_steps(torch, lambda: haq.haq_moe_w8a8_ffn(X, logits, s_in, experts, I, out=out, workspace=ws),
                                 steps, args.warmup, 0.2)
    # one timeline per timed call from the events the call records on its two streams
    lines = []

    def streamed_call():
        haq.haq_moe_w8a8_ffn(X, logits, s_in, mixed, I, ctx=ctx, out=out, workspace=ws)

    for _ in range(3):
        streamed_call()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        streamed_call()
        lines.append(haq.haq_ctx_last_call_timing(ctx))
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / steps
    same = bool(torch.equal(out, ref))
    total_ms, copies_ms, tail_ms = (float(np.mean([l[i] for l in lines])) for i in range(3))
    # pinned-copy peak of this machine: the same bytes, copies only
    stage = [torch.empty_like(experts[e].w13) for e in cold[:1]] + [torch.empty_like(experts[cold[0]].w2)]

    def copies():
        for e in cold:
            if counts[e] > 0:
                stage[0].copy_(mixed[e].w13, non_blocking=True)
                stage[1].copy_(mixed[e].w2, non_blocking=True)

    t_copy = _time_steps(torch, copies, max(3, steps // 4), 1, 0.1)
    torch.cuda.synchronize()
    _, misses2, _, _ = haq.haq_ctx_cache_stats(ctx)
    haq.haq_ctx_destroy(ctx)
    # the same layer with as many cache slots as cold experts: after the first call every lookup hits
    ctx4 = haq.haq_ctx_create(H, I, len(cold))
    t_cached = _time_steps(torch, lambda: haq.haq_moe_w8a8_ffn(X, logits, s_in, mixed, I, ctx=ctx4, out=out, workspace=ws),
                           steps, args.warmup, 0.2)
    same_cached = bool(torch.equal(out, ref))
    hits4, misses4, _, _ = haq.haq_ctx_cache_stats(ctx4)
    haq.haq_ctx_destroy(ctx4)
    streamed = sum(float(mixed[e].w13.numel() + mixed[e].w2.numel()) for e in cold if counts[e] > 0)
    resident_ms = t_all_resident * 1e3
    policy = None
    if canon:
        n_streamed = max(1, sum(1 for e in cold if counts[e] > 0))
        policy = _offload_policy(torch, haq, wl, X, logits, s_in, experts, mixed, cold, counts, canon, t_copy / n_streamed,
                                 t_all_resident / float(counts.sum()))
    return {
        "metric": "MoE layer latency with 4 of 8 experts streamed from host (ms)", "value": sec * 1e3, "unit": "ms",
        "ms_per_step": sec * 1e3, "dtype": "int8", "higher_is_better": False,
        "config": {"workload": wl.name, "tokens": T, "hidden": H, "intermediate": I, "experts": E, "top_k": 2,
                   "resident": list(wl.resident), "staging_slots": 2, "pairs_per_expert": counts.tolist()},
        "h2d_GBs": streamed / sec / 1e9, "h2d_copy_only_GBs": streamed / t_copy / 1e9, "streamed_MB": streamed / 1e6,
        "all_resident_ms": resident_ms,
        # timeline of a call, from events on the launch stream and on the copy stream: everything the layer computes
        # except what runs after the last copy has landed is hidden under the copies
        "timeline_ms": {"call": total_ms, "first_copy_issued_to_last_copy_landed": copies_ms, "after_last_copy": tail_ms},
        "overlap_efficiency": min(1.0, max(0.0, (resident_ms - tail_ms) / resident_ms)),
        "matches_all_resident_bitwise": same and same_cached,
        "offload_policy": policy,
        "lru_cache": {"slots_2": {"misses": misses2, "ms": sec * 1e3},
                      f"slots_{len(cold)}": {"hits": hits4, "misses": misses4, "ms": t_cached * 1e3}},
        "roofline": {"bound": "host link", "kernel": "hipMemcpyAsync pinned host to HBM", "achieved": streamed / sec / 1e9,
                     "peak": streamed / t_copy / 1e9, "unit": "GB/s", "frac": min(1.0, t_copy / sec), "traffic": streamed,
                     "traffic_unit": "bytes per layer call over the host link (algorithmic = counted: whole experts are copied)",
                     "note": "peak = the same bytes as back-to-back pinned copies on this box, measured in this run"},
        "cpu_baseline": None,
    }


def bench_gemm_sweep(args, torch, haq, hi):
    """haq_gemm_w8a8_packed over shapes of equal work, over K, and over the row count (events around 200 launches each):
    separates the K-loop rate from the fixed cost of a round of tiles and shows what operand footprints do."""
    dev = "cuda:0"
    g = torch.Generator(device=dev).manual_seed(0)

    def run(T, K, N, reps=200):
        x = torch.randn((T, K), device=dev, generator=g).half()
        x[:, :20] *= 50
        wq = torch.clamp((torch.randn((K, N), device=dev, generator=g) * 30).round(), -127, 127).to(torch.int8)
        wp, sw = haq.haq_pack_weight(wq), torch.full((N,), 1e-3, device=dev)
        q, sx = haq.haq_quant_act_packed(x, None)
        y = torch.empty((T, N), dtype=torch.float16, device=dev)
        f = lambda: haq.haq_gemm_w8a8_packed(q, sx, wp, sw, T, K, N, haq.HAQ_ACT_NONE, out=y)
        _settle(torch, f, 0.3)
        ev = _events(torch, 2)
        ev[0].record()
        for _ in range(reps):
            f()
        ev[1].record()
        torch.cuda.synchronize()
        us = ev[0].elapsed_time(ev[1]) / reps * 1e3
        return {"T": T, "K": K, "N": N, "us": us, "TOPs": 2.0 * T * K * N / us / 1e6}

    shapes = [(1024, 4096, 16384), (4096, 4096, 4096), (2048, 4096, 8192), (8192, 4096, 2048), (16384, 4096, 1024)]
    ksweep = [(4096, k, 4096) for k in (1024, 2048, 4096, 8192, 16384)]
    rows = [(t, 4096, 16384) for t in (256, 512, 1024, 2048, 4096, 8192)]
    t0 = time.perf_counter()
    res = {"equal_work": [run(*s) for s in shapes], "k_sweep": [run(*s) for s in ksweep], "row_sweep": [run(*s) for s in rows]}
    k = res["k_sweep"]
    slope = (k[-1]["us"] - k[-2]["us"]) / (k[-1]["K"] - k[-2]["K"])   # us per unit of K in one round of 512 tiles
    res["k_loop_TOPs"] = 2.0 * 4096 * 4096 / slope / 1e6
    res["fixed_us_per_round"] = k[0]["us"] - slope * k[0]["K"]
    best = max(r["TOPs"] for v in (res["equal_work"], res["k_sweep"], res["row_sweep"]) for r in v)
    return {"metric": "int8 GEMM + epilogue TOPS over a shape sweep (best)", "value": best, "unit": "TOPS",
            "ms_per_step": (time.perf_counter() - t0) * 1e3, "dtype": "int8", "config": {"workload": "gemm_sweep"},
            "sweep": res, "roofline": {"bound": "mfma", "achieved": best, "peak": PEAK_INT8_TOPS, "unit": "TOP/s",
                                       "frac": best / PEAK_INT8_TOPS, "traffic": None}, "cpu_baseline": None}


def bench_search(args, torch, haq, hi):
    """Adaptive smoothing (Algorithm 1 step 1): 11 exponents on fc1 of the OPT-6.7B-shaped block."""
    wl = hi.OPT67B_FFN
    T, K, N = wl.T, wl.H, wl.F
    X_h, _, _ = hi.hidden_states(wl.seed, T, K, wl.n_outlier, wl.mult)
    W_h = hi.gaussian_weight(wl.seed, 0, K, N)
    X, W = torch.from_numpy(X_h).to("cuda:0"), torch.from_numpy(W_h).to("cuda:0")
    grid = [i / 10 for i in range(11)]
    ws = torch.empty(haq.haq_smoothing_search_workspace_bytes(T, K, N, len(grid)), dtype=torch.uint8, device="cuda:0")
    result = {}

    def step():
        result["r"] = haq.haq_smoothing_search(X, W, grid, False, workspace=ws)

    sec = _time_steps(torch, step, args.steps, args.warmup)
    losses, best, _ = result["r"]
    yref = torch.empty((T, N), dtype=torch.float64, device="cuda:0")
    ev = _events(torch, 2 * args.steps)
    for i in range(args.steps):
        ev[2 * i].record()
        haq.haq_reference_matmul_f64(X, W, out=yref)
        ev[2 * i + 1].record()
    torch.cuda.synchronize()
    ref_s = float(np.mean([ev[2 * i].elapsed_time(ev[2 * i + 1]) for i in range(args.steps)])) * 1e-3
    flops = 2.0 * T * K * N
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        t0 = time.perf_counter()
        lo, bo, _ = oracle.smoothing_search(X_h, W_h, grid)
        dt = time.perf_counter() - t0
        cpu = {"value": len(grid) / dt, "unit": "candidates/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": f"the whole search once ({len(grid)} exponents, all {T} rows), {dt:.2f} s",
               "same_best_exponent": bool(bo == best), "same_losses_bitwise": bool(np.array_equal(lo, np.asarray(losses)))}
    return {
        "metric": "smoothing grid search candidates/s (offline)", "value": len(grid) / sec, "unit": "candidates/s",
        "ms_per_step": sec * 1e3, "dtype": "int8 candidates, fp64 reference and loss",
        "config": {"workload": "opt-6.7b fc1 smoothing search", "tokens": T, "in_features": K, "out_features": N,
                   "exponents": grid, "form": "s = ax^e"},
        "best_exponent": grid[best], "losses": losses,
        "roofline": {"bound": "alu", "kernel": "ref_gemm_f64_kernel (binary64 reference product, once per search)",
                     "achieved": flops / ref_s / 1e12, "peak": PEAK_FP64_TFLOPS, "unit": "TFLOP/s",
                     "frac": flops / ref_s / 1e12 / PEAK_FP64_TFLOPS, "avg_launch_ms": ref_s * 1e3, "traffic": None},
        "cpu_baseline": cpu,
    }


def bench_hessian(args, torch, haq, hi):
    """Hessian-aware weight quantisation (Algorithm 1 step 2) of fc1 of the OPT-6.7B-shaped block."""
    wl = hi.OPT67B_FFN
    T, K, N = wl.T, wl.H, wl.F
    X_h, _, _ = hi.hidden_states(wl.seed, T, K, wl.n_outlier, wl.mult)
    W_h = hi.gaussian_weight(wl.seed, 0, K, N)
    X, W = torch.from_numpy(X_h).to("cuda:0"), torch.from_numpy(W_h).to("cuda:0")
    s = haq.haq_smoothing_vector(haq.haq_channel_absmax_f16(X), haq.haq_weight_row_absmax(W), 0.5)
    ws = torch.empty(haq.haq_hessian_quant_workspace_bytes(K, N), dtype=torch.uint8, device="cuda:0")
    out = {}

    def step():
        out["r"] = haq.haq_hessian_quant_weight(X, W, s, 0.01, workspace=ws)

    sec = _time_steps(torch, step, args.steps, args.warmup)
    wq, sw = out["r"]
    # what it buys on the run-time path: loss of the W8A8 layer against the binary64 product, both quantisers
    yref = haq.haq_reference_matmul_f64(X, W)
    wr, swr = haq.haq_quant_weight(W, s)
    loss = {}
    for name, (q, sc) in (("hessian_aware", (wq, sw)), ("round_to_nearest", (wr, swr))):
        y = haq.haq_w8a8_linear(X, s, haq.haq_pack_weight(q), sc, N)
        loss[name] = float(haq.haq_quant_loss_f64(y, yref).cpu()[0])
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        Ks, Ns = 1024, 2048
        t0 = time.perf_counter()
        oracle.hessian_quant_weight(X_h[:, :Ks], W_h[:Ks, :Ns], s.cpu().numpy()[:Ks], 0.01)
        dt = time.perf_counter() - t0
        cpu = {"value": Ks * Ns / dt / 1e6, "unit": "Mweights/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": f"first {Ks} input channels x first {Ns} output channels, all {T} calibration rows, once, {dt:.2f} s "
                         "(the cost grows faster than the weight count: K^2 T + K^3 + K^2 N)"}
    flops = float(K) * K * N  # the compensation sweep: K^2 N / 2 fused multiply-adds
    return {
        "metric": "Hessian-aware weight quantisation throughput (offline)", "value": K * N / sec / 1e6, "unit": "Mweights/s",
        "ms_per_step": sec * 1e3, "dtype": "f64",
        "config": {"workload": "opt-6.7b fc1 hessian-aware quantisation", "calibration_rows": T, "in_features": K,
                   "out_features": N, "percdamp": 0.01, "smoothing_alpha": 0.5},
        "w8a8_layer_loss": loss, "codes_changed_vs_rtn": float((wq != wr).float().mean().cpu()),
        "roofline": {"bound": "alu", "kernel": "whole call (binary64 chains: Hessian, factorisation, inverse, sweep)",
                     "achieved": (2.0 * K * K * T + K ** 3 / 3.0 + K ** 3 / 3.0 + flops) / sec / 1e12, "peak": PEAK_FP64_TFLOPS,
                     "unit": "TFLOP/s", "frac": (2.0 * K * K * T + 2.0 * K ** 3 / 3.0 + flops) / sec / 1e12 / PEAK_FP64_TFLOPS,
                     "traffic": None},
        "cpu_baseline": cpu,
    }


def _record(res, args):
    line = {"metric": res.pop("metric"), "value": res.pop("value"), "unit": res.pop("unit"), "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "ms_per_step": res.pop("ms_per_step"),
            "higher_is_better": res.pop("higher_is_better", True), "scaling": "weak", "vs_baseline": None,
            "dtype": res.pop("dtype"),
            "data": "synthetic"}
    line.update(res)
    return line


MOE_WORKLOADS = ["moe_prefill", "moe_decode_b1", "moe_decode_b8", "moe_decode_b64", "moe_offload"]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="all",
                    choices=["all", "ffn", "linear", *MOE_WORKLOADS, "smooth_search", "hessian_quant", "gemm_sweep"],
                    help="all (default): the OPT-6.7B FFN block as the headline plus one record per other configuration")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the measured-clock peak and the pure-MFMA ceiling (2.5 s)")
    ap.add_argument("--calibration-copy-mb", type=int, default=0,
                    help="also run one plain device-to-device copy of this many MB (reference for rocprofv3 --pmc byte counters)")
    ap.add_argument("--cpu-rows", type=int, default=2048, help="token rows of the workload the CPU oracle is timed on")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (--gpus 1); nothing here shards across GPUs", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    import haq_inputs as hi
    import paper_2508_07329_amd as haq
    haq.lib()
    torch.cuda.set_device(0)
    if args.calibration_copy_mb > 0:
        src = torch.ones(args.calibration_copy_mb * (1 << 20), dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    everything = args.workload == "all"
    if args.workload in ("all", "ffn", "linear"):
        res = bench_ffn(args, torch, haq, hi)
    elif args.workload == "smooth_search":
        res = bench_search(args, torch, haq, hi)
    elif args.workload == "hessian_quant":
        res = bench_hessian(args, torch, haq, hi)
    elif args.workload == "gemm_sweep":
        res = bench_gemm_sweep(args, torch, haq, hi)
    else:
        res = bench_moe(args, torch, haq, hi, args.workload, build_mixtral(torch, haq, hi, keep_host=not args.no_cpu_baseline))
    line = _record(res, args)
    if everything:
        # the other configurations of the metric, each with a short CPU-oracle baseline of its own
        t0 = time.perf_counter()
        # (a configuration that fails is reported as such in its record; the headline line is printed regardless)
        configs = []

        def add(name, run):
            try:
                configs.append(_record(run(), args))
            except Exception as exc:  # noqa: BLE001 - reported, not hidden
                configs.append({"config": {"workload": name}, "error": f"{type(exc).__name__}: {exc}"})
            print(f"bench.py: {name} done at {time.perf_counter() - t0:.0f} s", file=sys.stderr, flush=True)

        args.workload = "linear"
        add("linear", lambda: bench_ffn(args, torch, haq, hi, cpu_seconds=2.0))
        torch.cuda.empty_cache()
        try:
            layer = build_mixtral(torch, haq, hi, keep_host=not args.no_cpu_baseline)
        except Exception as exc:  # noqa: BLE001
            layer = None
            configs.append({"config": {"workload": "mixtral layer set-up"}, "error": f"{type(exc).__name__}: {exc}"})
        if layer is not None:
            for w in MOE_WORKLOADS:
                add(w, lambda w=w: bench_moe(args, torch, haq, hi, w, layer, cpu_seconds=2.5))
        line["configs"] = configs
    print(json.dumps(line))


if __name__ == "__main__":
    main()
