#!/usr/bin/env python3
"""Benchmark of the dynamic-M dense hot path on one MI355X.

Headline workload: the BERT-large shaped FFN at a ragged total token count
(M = sum of 32 sequence lengths, each uniform in 1..512; 64 seeded draws).  One
step is one pass of the whole path over one draw: read the run-time shape,
shape function, allocate the outputs from it, dispatch on M, and the two dense
kernels (1024->4096 with bias+GELU, 4096->1024 with bias).  Inputs and weights
are resident in HBM before the timed region.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBPS = 8000.0      # MI355X HBM3E


def _to_dev(arr):
    import numpy as np
    import torch
    t = torch.from_numpy(np.ascontiguousarray(arr.bits).view(np.int16).copy())
    return t.view(torch.bfloat16).cuda()


def _traffic_note():
    """HBM-side bytes per dense launch from two rocprofv3 --pmc runs (FETCH_SIZE, then
    WRITE_SIZE, each scaled by a plain copy of known size); the summary of those runs is
    profiles/dense_config5_hbm_traffic.txt, which carries the figure on one line."""
    path = os.path.join(ROOT, "profiles", "dense_config5_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.strip().startswith("hbm_bytes_per_launch:"):
                return float(line.split(":", 1)[1])
    except OSError:
        pass
    return None


def _roof(bound, achieved, unit, **more):
    """A roofline record: achieved algorithmic rate against the nominal peak of what bounds the kernel."""
    peak = PEAK_BF16_TFLOPS if bound == "mfma" else PEAK_HBM_GBPS
    d = {"bound": bound, "achieved": round(achieved, 2), "peak": peak, "unit": unit, "frac": round(achieved / peak, 4)}
    d.update(more)
    return d


def _single_call_latency_us(fn, reps: int = 20) -> float:
    """Host-to-completion latency of one call on an idle stream: the host clock from just before the
    call until the device has finished it (median of `reps`)."""
    import statistics

    import torch
    fn()
    torch.cuda.synchronize()
    ts = []
    for _ in range(reps):
        t0 = time.perf_counter()
        fn()
        torch.cuda.synchronize()
        ts.append((time.perf_counter() - t0) * 1e6)
    return round(statistics.median(ts), 2)


PREHEAT_MS = 60.0   # the clocks take about 10 ms of work to come up after idle; the timed region starts past that
PREHEAT_MAX_MS = 600.0
REPEATS = 5         # the timed loop of exactly `steps` steps runs this often; the median repeat is reported


def bench_config5(steps: int, warmup: int):
    import statistics

    import numpy as np
    import torch

    import paper_2006_03031_amd as nb
    import workloads as wl
    from paper_2006_03031_amd import runtime as rt

    (n1, K1, N1, e1), (n2, K2, N2, e2) = wl.BERT_LARGE_FFN
    epi = {"bias": nb.EPI_BIAS, "bias_gelu": nb.EPI_BIAS_GELU_ERF}
    Ms = [int(m) for m in wl.config5_token_counts()]
    w1, b1 = wl.dense_weights(5, 0, N1, K1)
    w2, b2 = wl.dense_weights(5, 1, N2, K2)
    dw1, db1, dw2, db2 = _to_dev(w1), _to_dev(b1), _to_dev(w2), _to_dev(b2)
    x_all = _to_dev(wl.activations(5, 0, max(Ms), K1))  # a draw of M tokens reads the first M rows
    torch.cuda.synchronize()

    # a3: outputs are carved out of one storage sized for the largest draw (storage coalescing)
    arena = rt.StorageArena(max(Ms) * (N1 + N2) * 2 + 4096)

    def step(i):
        M = Ms[i % len(Ms)]
        x = x_all[:M]                      # a1: run-time shape of this draw
        arena.reset()
        # a2 shape function -> a3 allocation from it -> a4 dispatch on M -> a5 kernel, twice
        h = rt.dense(x, dw1, db1, epi[e1], arena=arena)
        y = rt.dense(h, dw2, db2, epi[e2], arena=arena)
        return y

    # untimed pre-heat of the same step for a fixed wall time: a short --warmup (the default command of
    # the harness warms up for 5 steps, under a millisecond) would otherwise leave the timed region
    # inside the clock ramp after idle, which runs 10-15 % slower
    # (some boxes of the pool are still speeding up after 60 ms: the pre-heat goes on, in chunks of 64 steps
    # over the whole cycle of draws, until three chunks in a row agree within 2 %, or PREHEAT_MAX_MS)
    t_pre = time.perf_counter()
    n_pre = 0
    chunks = []
    while True:
        t_c = time.perf_counter()
        for i in range(64):
            step(n_pre + i)
        n_pre += 64
        torch.cuda.synchronize()
        chunks.append(time.perf_counter() - t_c)
        heated = (time.perf_counter() - t_pre) * 1e3
        settled = len(chunks) >= 3 and max(chunks[-3:]) <= 1.02 * min(chunks[-3:])
        if (heated >= PREHEAT_MS and settled) or heated >= PREHEAT_MAX_MS:
            break
    preheat_ms = (time.perf_counter() - t_pre) * 1e3
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    walls, kernel_ms = [], []
    for rep in range(REPEATS):
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        ev0.record()
        for i in range(steps):
            step(i)
        ev1.record()
        torch.cuda.synchronize()
        walls.append(time.perf_counter() - t0)
        # HIP events on the launch stream bracket the timed loop, which holds nothing but the
        # dense launches (two nimble_dense_dyn calls per step)
        kernel_ms.append(ev0.elapsed_time(ev1))
    events = [(Ms[i % len(Ms)],) for i in range(steps)]

    total_flops = sum(2.0 * M * (N1 * K1 + N2 * K2) for M, *_ in events)
    elapsed = statistics.median(walls)
    k_ms = statistics.median(kernel_ms)
    launches = 2 * steps
    achieved = total_flops / (k_ms * 1e-3) / 1e12
    plans = sorted({nb.dense_plan(M, N1, K1).name for M in Ms} | {nb.dense_plan(M, N2, K2).name for M in Ms})
    roofline = _roof("mfma", achieved, "TFLOP/s", traffic=_traffic_note(),
                     traffic_source="profiles/dense_config5_hbm_traffic.txt (rocprofv3 --pmc runs of this "
                                    "command, bytes per dense launch; not measured by this run)",
                     kernel="gemm_ring_kernel (" + ",".join(plans) + ")", launches=launches,
                     avg_launch_us=round(k_ms * 1e3 / launches, 2), flops_per_launch=round(total_flops / launches))
    return {
        "value": total_flops / elapsed / 1e12, "ms_per_step": elapsed * 1e3 / steps, "roofline": roofline,
        "mean_M": sum(M for M, *_ in events) / len(events), "preheat_ms": round(preheat_ms, 1),
        "repeats": REPEATS, "ms_per_step_each_repeat": [round(w * 1e3 / steps, 4) for w in walls],
    }


def small_m_probe():
    """Secondary figures (not the headline): weight-streaming dense at M <= 16 with
    weights rotated through 512 MB so that they come from HBM, and one LSTM step."""
    import numpy as np
    import torch

    import paper_2006_03031_amd as nb
    import workloads as wl
    from paper_2006_03031_amd import runtime as rt

    out = {}
    N, K = 4096, 1024
    sets = 64  # 64 x 8 MB = 512 MB of distinct weights
    w = torch.empty((sets, N, K), dtype=torch.bfloat16, device="cuda").normal_(0, 0.02)
    b = torch.zeros((N,), dtype=torch.bfloat16, device="cuda")
    for M in (1, 16):
        x = torch.empty((M, K), dtype=torch.bfloat16, device="cuda").uniform_(-1, 1)
        y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        for i in range(sets):
            rt.dense(x, w[i], b, nb.EPI_BIAS, out=y)
        torch.cuda.synchronize()
        s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 4 * sets
        s.record()
        for i in range(reps):
            rt.dense(x, w[i % sets], b, nb.EPI_BIAS, out=y)
        e.record()
        torch.cuda.synchronize()
        us = s.elapsed_time(e) * 1e3 / reps
        nbytes = N * K * 2 + N * 2 + M * K * 2 + M * N * 2
        # the same 64 launches (one per weight set, as 64 layers in a row would be) as one HIP graph:
        # what the GPU needs once the host's per-call cost is out of the way
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for i in range(sets):
                rt.dense(x, w[i], b, nb.EPI_BIAS, out=y)
        graph.replay()
        torch.cuda.synchronize()
        s.record()
        for _ in range(4):
            graph.replay()
        e.record()
        torch.cuda.synchronize()
        us_g = s.elapsed_time(e) * 1e3 / (4 * sets)
        # warm: the same 8 MB of weights every call (they stay in the L2s / memory-side cache, so
        # this is an effective bandwidth, not an HBM one)
        warm = torch.cuda.CUDAGraph()
        with torch.cuda.graph(warm):
            for i in range(sets):
                rt.dense(x, w[0], b, nb.EPI_BIAS, out=y)
        warm.replay()
        torch.cuda.synchronize()
        s.record()
        for _ in range(4):
            warm.replay()
        e.record()
        torch.cuda.synchronize()
        us_w = s.elapsed_time(e) * 1e3 / (4 * sets)
        out[f"dense_{K}x{N}_M{M}_rotating"] = {"us_per_call": round(us, 2), "GBps": round(nbytes / us / 1e3, 1),
                                                 "hbm_frac": round(nbytes / us / 1e3 / PEAK_HBM_GBPS, 4),
                                                 "us_per_call_graph": round(us_g, 2),
                                                 "hbm_frac_graph": round(nbytes / us_g / 1e3 / PEAK_HBM_GBPS, 4),
                                                 "us_per_call_graph_warm": round(us_w, 2),
                                                 "effective_GBps_warm": round(nbytes / us_w / 1e3, 1),
                                                 "roofline": _roof("hbm", nbytes / us_g / 1e3, "GB/s", timing="64 launches, one per "
                                                                   "weight set (512 MB in rotation), replayed as one HIP graph",
                                                                   note="8 MB of weights are 1 us of HBM time: launch-bound")}
    del w
    # the same at a size where HBM, not launch latency, is the bound: one 8192 x 8192 layer (134 MB)
    N2 = K2 = 8192
    w = torch.empty((4, N2, K2), dtype=torch.bfloat16, device="cuda").normal_(0, 0.02)
    b2 = torch.zeros((N2,), dtype=torch.bfloat16, device="cuda")
    for M in (1, 16):
        x = torch.empty((M, K2), dtype=torch.bfloat16, device="cuda").uniform_(-1, 1)
        y = torch.empty((M, N2), dtype=torch.bfloat16, device="cuda")
        for i in range(4):
            rt.dense(x, w[i], b2, nb.EPI_BIAS, out=y)
        torch.cuda.synchronize()
        s.record()
        for i in range(16):
            rt.dense(x, w[i % 4], b2, nb.EPI_BIAS, out=y)
        e.record()
        torch.cuda.synchronize()
        us = s.elapsed_time(e) * 1e3 / 16
        nbytes = N2 * K2 * 2 + N2 * 2 + M * K2 * 2 + M * N2 * 2
        plan = nb.dense_plan(M, N2, K2, nb.EPI_BIAS)
        out[f"dense_{K2}x{N2}_M{M}_rotating"] = {"us_per_call": round(us, 2), "GBps": round(nbytes / us / 1e3, 1),
                                                   "hbm_frac": round(nbytes / us / 1e3 / PEAK_HBM_GBPS, 4),
                                                   "plan": plan.name + (f"/sk{plan.split_k}" if plan.split_k > 1 and plan.variant > 1 else ""),
                                                   "roofline": _roof("hbm", nbytes / us / 1e3, "GB/s", timing="16 back-to-back calls over "
                                                                     "4 weight sets (537 MB in rotation), HIP events")}
    del w
    lw = wl.config2_weights()
    dw, db = _to_dev(lw.w), _to_dev(lw.b)
    for B in (1, 4, 16, 64):
        x = torch.empty((B, 512), dtype=torch.bfloat16, device="cuda").uniform_(-1, 1)
        h0 = torch.zeros((B, 512), dtype=torch.bfloat16, device="cuda")
        h1 = torch.zeros_like(h0)
        c = torch.zeros((B, 512), dtype=torch.float32, device="cuda")
        for _ in range(16):
            rt.lstm_step(x, h0, dw, db, c, h_out=h1, c_out=c)
            h0, h1 = h1, h0
        torch.cuda.synchronize()
        s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s.record()
        for _ in range(128):
            rt.lstm_step(x, h0, dw, db, c, h_out=h1, c_out=c)
            h0, h1 = h1, h0
        e.record()
        torch.cuda.synchronize()
        us = s.elapsed_time(e) * 1e3 / 128
        nbytes = 2048 * 1024 * 2 + 4096 + 7168 * B
        # the same 128-step loop captured as a HIP graph (one graph per batch size)
        seq = rt.LstmSequenceGraph(dw, db, B, 128, 512, 512)
        seq.run()
        torch.cuda.synchronize()
        s.record()
        for _ in range(4):
            seq.graph.replay()
        e.record()
        torch.cuda.synchronize()
        us_g = s.elapsed_time(e) * 1e3 / (4 * 128)
        # the inputs' product for all 128 tokens hoisted into one dense call (M = 128 B) ahead of
        # the loop: each step then streams only the recurrent half of the weight
        seq_p = rt.LstmSequenceGraph(dw, db, B, 128, 512, 512, project_inputs=True)
        seq_p.run()
        torch.cuda.synchronize()
        s.record()
        for _ in range(4):
            seq_p.graph.replay()
        e.record()
        torch.cuda.synchronize()
        us_p = s.elapsed_time(e) * 1e3 / (4 * 128)
        lat = _single_call_latency_us(lambda: rt.lstm_step(x, h0, dw, db, c, h_out=h1, c_out=c))
        out[f"lstm_step_B{B}_warm"] = {"us_per_step": round(us, 2), "us_per_step_graph": round(us_g, 2),
                                       "eff_GBps_graph": round(nbytes / us_g / 1e3, 1),
                                       "us_per_step_graph_inputs_projected": round(us_p, 2),
                                       "single_call_host_to_completion_us": lat,
                                       "roofline": _roof("hbm", nbytes / us_g / 1e3, "GB/s", timing="128-step token loop replayed "
                                                         "as a HIP graph", note="effective: the same 4.2 MB of weights every step "
                                                         "stay in the L2s / memory-side cache")}
        # the loop over the 128 tokens as ONE launch (recurrent weights in registers, h_t handed over through
        # memory inside the kernel), timed on the loop alone like the projected-inputs graph minus its dense call
        if nb.lstm_seq_supported(B, 512):
            T = 512
            pre = torch.empty((T, B, 2048), dtype=torch.float32, device="cuda").uniform_(-2, 2)
            w_h = rt.split_lstm_weight(dw, 512)[1]
            hz = torch.zeros((B, 512), dtype=torch.bfloat16, device="cuda")
            cz = torch.zeros((B, 512), dtype=torch.float32, device="cuda")
            hseq = torch.empty((T, B, 512), dtype=torch.bfloat16, device="cuda")
            cT = torch.empty((B, 512), dtype=torch.float32, device="cuda")
            ws = torch.empty(nb.lstm_seq_workspace_bytes(B, 512), dtype=torch.uint8, device="cuda")
            st = torch.cuda.current_stream().cuda_stream

            def one_launch():
                nb.nimble_lstm_seq_pre_dyn(pre.data_ptr(), w_h.data_ptr(), hz.data_ptr(), cz.data_ptr(), hseq.data_ptr(),
                                           cT.data_ptr(), T, B, 512, ws.data_ptr(), ws.numel(), rt.LSTM_SEQ_MAX_POLLS, st)
            one_launch()
            gave_up = nb.nimble_lstm_seq_status(ws.data_ptr(), st)
            best = 1e9
            for _ in range(3):
                s.record()
                one_launch()
                e.record()
                torch.cuda.synchronize()
                best = min(best, s.elapsed_time(e) * 1e3 / T)
            out[f"lstm_step_B{B}_warm"]["us_per_step_one_launch"] = round(best, 2)
            out[f"lstm_step_B{B}_warm"]["one_launch_gave_up"] = bool(gave_up)
            nb_rec = 1024 * 1024 * 2 + 8192 * B + 1024 * B  # recurrent weights + this step's pre + h
            out[f"lstm_step_B{B}_warm"]["roofline_one_launch"] = _roof(
                "hbm", nb_rec / best / 1e3, "GB/s", timing="512-token loop in one launch, HIP events",
                note="effective: the 2.1 MB of recurrent weights stay in registers; a step is bound by the hand-over of h")
        del seq, seq_p
    # the same token loop as bytecode on the interpreter: shape_of, shape function, allocation from
    # the pool and invoke per token (about two dozen coarse instructions), host cost per token split
    # into kernel dispatch+launch and everything else
    from paper_2006_03031_amd import vm
    exe = vm.Executable.from_assembler(vm.lstm_sequence_program(), [dw, db])
    pool = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
    for B in (1, 64):
        xs = torch.empty((128, B, 512), dtype=torch.bfloat16, device="cuda").uniform_(-1, 1)
        h0 = torch.zeros((B, 512), dtype=torch.bfloat16, device="cuda")
        c0 = torch.zeros((B, 512), dtype=torch.float32, device="cuda")
        exe.run([xs, h0, c0], pool)
        torch.cuda.synchronize()
        s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s.record()
        for _ in range(4):
            exe.run([xs, h0, c0], pool)
        e.record()
        torch.cuda.synchronize()
        prof = exe.profile()
        launch_ns = prof["packed"]["lstm_gates"][1]
        out[f"vm_lstm_B{B}"] = {"us_per_step": round(s.elapsed_time(e) * 1e3 / (4 * 128), 2),
                                "instructions_per_step": round(prof["instructions"] / 128, 1),
                                "host_us_per_step_launch": round(launch_ns / 128e3, 2),
                                "host_us_per_step_others": round((prof["host_ns"] - launch_ns) / 128e3, 2),
                                "pool_high_water_bytes": prof["pool_high_water"]}
    del pool
    # attention, 12 heads x 64, one launch versus the three-call chain
    for L in (128, 512):
        q = torch.empty((12, L, 64), dtype=torch.bfloat16, device="cuda").uniform_(-1, 1)
        k, v, o = q.clone(), q.clone(), torch.empty_like(q)
        res = {}
        for name, fn, reps in (("fused", lambda: rt.fused_attention(q, k, v, out=o), 64),
                               ("chain", lambda: rt.attention(q, k, v), 16)):
            fn()
            torch.cuda.synchronize()
            s.record()
            for _ in range(reps):
                fn()
            e.record()
            torch.cuda.synchronize()
            res[name + "_us"] = round(s.elapsed_time(e) * 1e3 / reps, 2)
        # the fused call replayed as a HIP graph of 20 launches: its GPU time without the host's share
        gr = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gr):
            for _ in range(20):
                rt.fused_attention(q, k, v, out=o)
        gr.replay()
        torch.cuda.synchronize()
        s.record()
        for _ in range(4):
            gr.replay()
        e.record()
        torch.cuda.synchronize()
        res["fused_us_graph"] = round(s.elapsed_time(e) * 1e3 / 80, 2)
        del gr
        # algorithmic bytes: q, k, v in and o out for the fused kernel; the chain adds S (f32 out and in) and P
        # (bf16 out and in): 144 L^2
        res["roofline"] = _roof("hbm", 6144.0 * L / res["fused_us_graph"] / 1e3, "GB/s", kernel="attention64_kernel",
                                timing="20 launches replayed as a HIP graph",
                                note="latency-bound: a few hundred KB per call, 24-96 workgroups")
        res["roofline_chain"] = _roof("hbm", (6144.0 * L + 144.0 * L * L) / res["chain_us"] / 1e3, "GB/s",
                                      kernel="batch_matmul, softmax_rows, batch_matmul")
        res["single_call_host_to_completion_us"] = _single_call_latency_us(lambda: rt.fused_attention(q, k, v, out=o))
        out[f"attention_L{L}"] = res
    return out


def achievable_peaks():
    """What this GPU sustains on a register-only bf16 MFMA loop (one and two waves per SIMD, real
    operand data) and on a plain streaming read of 2 GiB: the ceilings any kernel here works
    under, printed next to the nominal peaks the roofline fractions are taken against."""
    import torch

    import paper_2006_03031_amd as nb

    out = {}
    seed = torch.empty(32768, dtype=torch.bfloat16, device="cuda").uniform_(-1, 1)
    sink = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    stream = torch.cuda.current_stream().cuda_stream
    for waves in (1, 2):
        nb.nimble_probe_mfma_bf16(seed.data_ptr(), sink.data_ptr(), waves, 4000, stream)
        torch.cuda.synchronize()
        s.record()
        flops = nb.nimble_probe_mfma_bf16(seed.data_ptr(), sink.data_ptr(), waves, 20000, stream)
        e.record()
        torch.cuda.synchronize()
        out[f"mfma_bf16_TFLOPs_{waves}_wave_per_simd"] = round(flops / (s.elapsed_time(e) * 1e-3) / 1e12, 1)
    buf = torch.ones(2 << 30, dtype=torch.uint8, device="cuda")
    nb.nimble_probe_hbm_read(buf.data_ptr(), buf.numel(), sink.data_ptr(), stream)
    torch.cuda.synchronize()
    s.record()
    for _ in range(8):
        nb.nimble_probe_hbm_read(buf.data_ptr(), buf.numel(), sink.data_ptr(), stream)
    e.record()
    torch.cuda.synchronize()
    out["hbm_read_GBps"] = round(8 * buf.numel() / (s.elapsed_time(e) * 1e-3) / 1e9, 1)
    return out


def config_1_and_3_probe():
    """Configs 1 and 3 at their own sizes: microseconds per call with the launches of one pass
    replayed as a HIP graph (what the GPU needs) and launched one by one (what a Python caller
    sees).  Config 1 (128 -> 128, M <= 64) is launch-bound: 33 KB of weights are 4 ns of HBM time."""
    import numpy as np
    import torch

    import paper_2006_03031_amd as nb
    import workloads as wl
    from paper_2006_03031_amd import runtime as rt
    from paper_2006_03031_amd.tune import _time_us

    out = {}
    calls = wl.config1_calls()
    w, b = _to_dev(calls[0].w), _to_dev(calls[0].b)
    xs = [_to_dev(c.x) for c in calls]
    ys = [torch.empty((x.shape[0], 128), dtype=torch.bfloat16, device="cuda") for x in xs]

    def pass1():
        for x, y in zip(xs, ys):
            rt.dense(x, w, b, nb.EPI_BIAS, out=y)
    pass1()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(8):
        pass1()
    torch.cuda.synchronize()
    us_eager = (time.perf_counter() - t0) * 1e6 / (8 * len(xs))
    us_graph = _time_us(pass1, reps=1) / len(xs)
    mean_bytes = sum(32768 + 256 + 512 * x.shape[0] for x in xs) / len(xs)
    mid = len(xs) // 2
    out["config1_dense_128x128"] = {"us_per_call_eager": round(us_eager, 2), "us_per_call_graph": round(us_graph, 2),
                                    "single_call_host_to_completion_us": _single_call_latency_us(
                                        lambda: rt.dense(xs[mid], w, b, nb.EPI_BIAS, out=ys[mid])),
                                    "roofline": _roof("hbm", mean_bytes / us_graph / 1e3, "GB/s", timing="the 64 calls replayed "
                                                      "as one HIP graph", note="launch-bound: 33 KB of weights are 4 ns of HBM time")}
    epi = {"bias": nb.EPI_BIAS, "bias_gelu": nb.EPI_BIAS_GELU_ERF}
    weights = [(_to_dev(wb[0]), _to_dev(wb[1]), K, N, epi[e]) for i, (n, K, N, e) in enumerate(wl.BERT_BASE_GEMMS)
               for wb in (wl.dense_weights(3, i, N, K),)]
    for L in (1, 16, 128, 384, 512):
        bufs = [(torch.empty((L, K), dtype=torch.bfloat16, device="cuda").uniform_(-1, 1),
                 torch.empty((L, N), dtype=torch.bfloat16, device="cuda")) for _, _, K, N, _ in weights]

        def layer():
            for (wt, bt, K, N, e), (x, y) in zip(weights, bufs):
                rt.dense(x, wt, bt, e, out=y)
        us = _time_us(layer, reps=8)
        flops = 2.0 * L * sum(K * N for _, _, K, N, _ in weights)
        plans = [nb.dense_plan(L, N, K, e) for _, _, K, N, e in weights]
        nbytes = 14155776.0 + 24576.0 * L + 2 * sum(N for _, _, _, N, _ in weights)
        out[f"config3_bert_base_L{L}"] = {"us_4_gemms_graph": round(us, 2), "TFLOPs": round(flops / us / 1e6, 1),
                                          "plans": [pl.name + (f"/sk{pl.split_k}" if pl.split_k > 1 and pl.variant > 1 else "") for pl in plans],
                                          "single_call_host_to_completion_us": _single_call_latency_us(
                                              lambda: rt.dense(bufs[2][0], weights[2][0], weights[2][1], weights[2][4], out=bufs[2][1])),
                                          "roofline": _roof("hbm", nbytes / us / 1e3, "GB/s", timing="the four launches replayed as a HIP "
                                                            "graph", note="effective: 14 MB of weights stay cache-resident between replays"),
                                          "roofline_mfma": _roof("mfma", flops / us / 1e6, "TFLOP/s")}
    return out


def allocation_probe():
    """Step a3 measured (the memory-planning section's allocation count and latency): outputs of
    the two FFN calls over the 64 ragged draws allocated per call from torch's caching allocator,
    against carved out of one storage block sized once for the largest draw."""
    import torch

    import paper_2006_03031_amd as nb
    import workloads as wl
    from paper_2006_03031_amd import runtime as rt

    (n1, K1, N1, e1), (n2, K2, N2, e2) = wl.BERT_LARGE_FFN
    Ms = [int(m) for m in wl.config5_token_counts()]
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    before = torch.cuda.memory_stats()
    t0 = time.perf_counter()
    for _ in range(8):
        for M in Ms:
            h = rt._alloc((M, N1), nb.BF16, "cuda")
            y = rt._alloc((M, N2), nb.BF16, "cuda")
    t_torch = (time.perf_counter() - t0) / (16 * len(Ms))
    after = torch.cuda.memory_stats()
    del h, y
    arena = rt.StorageArena(max(Ms) * (N1 + N2) * 2 + 4096)
    mid = torch.cuda.memory_stats()
    t0 = time.perf_counter()
    for _ in range(8):
        for M in Ms:
            arena.reset()
            h = arena.alloc((M, N1), nb.BF16)
            y = arena.alloc((M, N2), nb.BF16)
    t_arena = (time.perf_counter() - t0) / (16 * len(Ms))
    end = torch.cuda.memory_stats()
    key_a, key_s = "allocation.all.allocated", "segment.all.allocated"
    # the same two allocations made by the bytecode interpreter from its pool (C++, no Python):
    # alloc_storage + alloc_tensor per output, host nanoseconds from the interpreter's own profile
    from paper_2006_03031_amd import vm
    w1, b1 = wl.dense_weights(5, 0, N1, K1)
    w2, b2 = wl.dense_weights(5, 1, N2, K2)
    exe = vm.Executable.from_assembler(vm.ffn_block_program(), [_to_dev(w1), _to_dev(b1), _to_dev(w2), _to_dev(b2)])
    pool = torch.empty(max(Ms) * (N1 + N2) * 2 + (1 << 20), dtype=torch.uint8, device="cuda")
    x = torch.empty((Ms[0], K1), dtype=torch.bfloat16, device="cuda").uniform_(-1, 1)
    for _ in range(3):
        exe.run([x], pool)
    torch.cuda.synchronize()
    prof = exe.profile()
    alloc_ns = sum(prof["opcodes"].get(op, (0, 0))[1] for op in ("AllocStorage", "AllocTensor", "AllocTensorReg"))
    alloc_n = sum(prof["opcodes"].get(op, (0, 0))[0] for op in ("AllocStorage",))
    del pool
    return {"per_output_us_interpreter_pool": round(alloc_ns / max(alloc_n, 1) / 1e3, 3),"per_output_us_caching_allocator": round(t_torch * 1e6, 2), "per_output_us_arena": round(t_arena * 1e6, 2),
            "allocator_requests_per_step_caching": (after[key_a] - before[key_a]) / (8 * len(Ms)),
            "allocator_requests_per_step_arena": (end[key_a] - mid[key_a]) / (8 * len(Ms)),
            "device_segments_caching": after[key_s] - before[key_s],
            "device_segments_arena": 1 + end[key_s] - mid[key_s]}


def two_requests_in_flight(steps: int = 256, warmup: int = 64):
    """The headline workload with two requests in flight on two streams (alternate draws, each
    stream with its own arena and K-split workspace): kernels of one request fill the launch
    gaps, partial last rounds and output-write phases of the other.  Reported beside the
    headline, which stays one request at a time on one stream."""
    import torch

    import paper_2006_03031_amd as nb
    import workloads as wl
    from paper_2006_03031_amd import runtime as rt

    (n1, K1, N1, e1), (n2, K2, N2, e2) = wl.BERT_LARGE_FFN
    epi = {"bias": nb.EPI_BIAS, "bias_gelu": nb.EPI_BIAS_GELU_ERF}
    Ms = [int(m) for m in wl.config5_token_counts()]
    w1, b1 = wl.dense_weights(5, 0, N1, K1)
    w2, b2 = wl.dense_weights(5, 1, N2, K2)
    dw1, db1, dw2, db2 = _to_dev(w1), _to_dev(b1), _to_dev(w2), _to_dev(b2)
    x_all = _to_dev(wl.activations(5, 0, max(Ms), K1))
    streams = [torch.cuda.Stream() for _ in range(2)]   # default priority
    arenas = [rt.StorageArena(max(Ms) * (N1 + N2) * 2 + 4096) for _ in range(2)]
    spaces = [torch.empty(rt.WORKSPACE_BYTES, dtype=torch.uint8, device="cuda") for _ in range(2)]
    torch.cuda.synchronize()

    def step(i):
        s = i & 1
        with torch.cuda.stream(streams[s]):
            M = Ms[i % len(Ms)]
            arenas[s].reset()
            h = rt.dense(x_all[:M], dw1, db1, epi[e1], arena=arenas[s], workspace=spaces[s])
            rt.dense(h, dw2, db2, epi[e2], arena=arenas[s], workspace=spaces[s])

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    t = time.perf_counter() - t0
    flops = sum(2.0 * Ms[i % len(Ms)] * (N1 * K1 + N2 * K2) for i in range(steps))
    return {"TFLOPs": round(flops / t / 1e12, 1), "ms_per_step": round(t / steps * 1e3, 4), "steps": steps}


def vendor_reference():
    """Context, not part of the path: the vendor's tuned GEMM library (hipBLASLt behind torch.matmul) on the two
    FFN shapes at M = 8192, timed the same way as this library's kernels beside it.  It shows what fraction of the
    nominal MFMA peak a tuned kernel reaches on these shapes on this GPU."""
    import torch

    import paper_2006_03031_amd as nb
    from paper_2006_03031_amd import runtime as rt

    out = {}
    s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(fn, reps=20):
        for _ in range(5):
            fn()
        torch.cuda.synchronize()
        best = float("inf")
        for _ in range(3):
            s.record()
            for _ in range(reps):
                fn()
            e.record()
            torch.cuda.synchronize()
            best = min(best, s.elapsed_time(e) * 1e3 / reps)
        return best

    for name, (M, N, K), epi in (("ffn1_8192x4096x1024", (8192, 4096, 1024), nb.EPI_BIAS_GELU_ERF),
                                 ("ffn2_8192x1024x4096", (8192, 1024, 4096), nb.EPI_BIAS)):
        x = torch.empty((M, K), dtype=torch.bfloat16, device="cuda").uniform_(-1, 1)
        w = torch.empty((N, K), dtype=torch.bfloat16, device="cuda").normal_(0, 0.02)
        b = torch.zeros((N,), dtype=torch.bfloat16, device="cuda")
        y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        flops = 2.0 * M * N * K
        t_lib = timed(lambda: torch.matmul(x, w.t(), out=y))
        t_plain = timed(lambda: rt.dense(x, w, b, nb.EPI_BIAS, out=y))
        t_epi = timed(lambda: rt.dense(x, w, b, epi, out=y))
        out[name] = {"vendor_matmul_no_epilogue_us": round(t_lib, 1), "vendor_TFLOPs": round(flops / t_lib / 1e6, 1),
                     "vendor_frac_of_peak": round(flops / t_lib / 1e6 / PEAK_BF16_TFLOPS, 4),
                     "this_library_bias_us": round(t_plain, 1), "this_library_config_epilogue_us": round(t_epi, 1),
                     "this_library_TFLOPs": round(flops / t_epi / 1e6, 1)}

    # the BERT-base layers of config 3 at a few lengths, both sides as 20 launches replayed as one HIP graph
    # (microseconds per call: this library with the layer's epilogue / the vendor's matmul without one)
    def graph_us(fn, n=20):
        fn()
        torch.cuda.synchronize()
        gr = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gr):
            for _ in range(n):
                fn()
        gr.replay()
        torch.cuda.synchronize()
        best = float("inf")
        for _ in range(3):
            s.record()
            gr.replay()
            e.record()
            torch.cuda.synchronize()
            best = min(best, s.elapsed_time(e) * 1e3 / n)
        return best

    mid = {}
    for (N, K, epi) in ((2304, 768, nb.EPI_BIAS), (768, 768, nb.EPI_BIAS), (3072, 768, nb.EPI_BIAS_GELU_ERF),
                        (768, 3072, nb.EPI_BIAS)):
        w = torch.empty((N, K), dtype=torch.bfloat16, device="cuda").normal_(0, 0.02)
        b = torch.zeros((N,), dtype=torch.bfloat16, device="cuda")
        for M in (64, 128, 512, 2048):
            x = torch.empty((M, K), dtype=torch.bfloat16, device="cuda").uniform_(-1, 1)
            y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
            mid[f"{M}x{N}x{K}"] = [round(graph_us(lambda: rt.dense(x, w, b, epi, out=y)), 2),
                                   round(graph_us(lambda: torch.matmul(x, w.t(), out=y)), 2)]
    out["bert_base_layers_us_this_library_vs_vendor"] = mid
    return out


def _extras():
    out = small_m_probe()
    out.update(config_1_and_3_probe())
    out["allocation"] = allocation_probe()
    out["two_requests_in_flight"] = two_requests_in_flight()
    out["achievable"] = achievable_peaks()
    out["vendor_gemm_reference"] = vendor_reference()
    return out


def cpu_baseline():
    """The oracle as it stands, timed on the host cores on a bounded sample of the
    same workload: the draws with the smallest, quartile, median and largest M, both FFN GEMMs
    (about 10 s on 16 host threads)."""
    import numpy as np

    import oracle
    import workloads as wl

    (n1, K1, N1, e1), (n2, K2, N2, e2) = wl.BERT_LARGE_FFN
    Ms = wl.config5_token_counts()
    order = np.argsort(Ms)
    draws = [int(order[0]), int(order[len(Ms) // 4]), int(order[len(Ms) // 2]), int(order[3 * len(Ms) // 4]),
             int(order[-1])]
    w1, b1 = wl.dense_weights(5, 0, N1, K1)
    w2, b2 = wl.dense_weights(5, 1, N2, K2)
    flops = 0.0
    t = 0.0
    for d in draws:
        M = int(Ms[d])
        x = wl.activations(5, d, M, K1).f32
        t0 = time.perf_counter()
        h = oracle.dense(x, w1.f32, b1.f32, e1)
        y = oracle.dense(h, w2.f32, b2.f32, e2)
        t += time.perf_counter() - t0
        flops += 2.0 * M * (N1 * K1 + N2 * K2)
        del h, y
    # the same oracle on one host thread (its OpenMP team is set to one thread through the OpenMP
    # runtime the oracle library is linked against; the oracle itself is untouched): the first 768
    # rows of the smallest draw, both GEMMs
    single = None
    try:
        import ctypes
        omp = ctypes.CDLL("libgomp.so.1")
        threads = oracle.num_threads()
        rows = 768
        x = wl.activations(5, draws[0], int(Ms[draws[0]]), K1).f32[:rows]
        omp.omp_set_num_threads(1)
        try:
            t0 = time.perf_counter()
            h = oracle.dense(x, w1.f32, b1.f32, e1)
            y = oracle.dense(h, w2.f32, b2.f32, e2)
            t1 = time.perf_counter() - t0
        finally:
            omp.omp_set_num_threads(threads)
        f1 = 2.0 * rows * (N1 * K1 + N2 * K2)
        single = {"value": round(f1 / t1 / 1e12, 5), "unit": "TFLOP/s", "cores": 1,
                  "sample": f"first {rows} rows of the smallest draw, FFN1+FFN2, {f1 / 1e9:.0f} GFLOP in {t1:.1f} s"}
    except OSError:
        pass
    return {"value": round(flops / t / 1e12, 5), "unit": "TFLOP/s", "cores": oracle.num_threads(),
            "kind": "oracle", "sample": f"draws with M={[int(Ms[d]) for d in draws]} (smallest, quartiles, largest), "
                                        f"FFN1+FFN2, {flops / 1e9:.0f} GFLOP in {t:.1f} s",
            "single_thread": single}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # the timed loop runs `steps` steps REPEATS times (median reported) after an untimed pre-heat of
    # fixed wall time and `warmup` further steps
    ap.add_argument("--steps", type=int, default=256)
    ap.add_argument("--warmup", type=int, default=64)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true")
    ap.add_argument("--extra-only", action="store_true",
                    help="run only the secondary probes (small-M dense, LSTM step, attention) and print them")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a plain 512 MiB device copy (calibrates the FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (--gpus must be 1)", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2006_03031_amd as nb

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)
    nb.load()
    torch.cuda.set_device(0)

    if args.copy_probe:
        src = torch.empty(512 * 1024 * 1024, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if args.extra_only:
        print(json.dumps({"extra": _extras()}))
        return
    res = bench_config5(args.steps, args.warmup)
    line = {
        "metric": "dynamic-M dense TFLOP/s (bf16) over M sweep; % of MFMA/HBM roofline",
        "value": round(res["value"], 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(res["ms_per_step"], 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "BERT-large FFN (1024->4096 bias+GELU, 4096->1024 bias) at ragged token count "
                               "M = sum of 32 lengths U{1..512}, 64 seeded draws, one draw per step",
                   "mean_M": round(res["mean_M"], 1), "weights": "bf16 N(0,0.02)",
                   "activations": "bf16 U[-1,1)", "accumulate": "f32"},
        "preheat_ms": res["preheat_ms"], "repeats": res["repeats"],
        "ms_per_step_each_repeat": res["ms_per_step_each_repeat"],
        "roofline": res["roofline"],
    }
    if not args.no_extra:
        line["extra"] = _extras()
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline()
    print(json.dumps(line))


if __name__ == "__main__":
    main()
