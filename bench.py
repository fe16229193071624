#!/usr/bin/env python3
"""Benchmark of the quantized LSTM step (and the kernels it is made of) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--sections a,b,...] [--no-cpu]

A step is one pass of the whole hot path -- on-line quantization of x_t and h_{t-1}, the
binary products with both weight blocks, the coefficient epilogue and the cell -- over one
batch of synthetic input that already sits in HBM.  The primary line reports the batch-64
LSTM (hidden 1024, W3/A3) in steps/s; `also` carries the batch-1 LSTM (hidden 300, W2/A2),
the streamed batch-1 LSTM step and binary GEMV in GB/s (the HBM-bound kernels), the cache-resident
GEMV latency, the GRU + projection step and the offline weight quantizer.  `roofline` describes the
kernel of the primary workload that takes the most time, `roofline_lstm_b1` and `roofline_gemv` the
HBM-bound kernels (each fraction against the nominal 8 TB/s and against a read-only streaming probe
measured in the same run).  `cpu_baseline` is the CPU oracle timed on a bounded sample of the primary
workload.

The primary line never times fewer than 100 sequence calls after 10 warm-up calls, whatever --steps
and --warmup say; `steps` and `warmup` in the line are what was really run.

One GPU only: nothing here shards, and --gpus above 1 is refused.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0                       # MI355X HBM3E
VALU_PEAK_TOPS = 256 * 4 * 16 * 2.4e9 / 1e12  # 39.3 T integer lane-ops/s: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz
FP4_MFMA_PEAK_TFLOPS = 10100.0               # dense fp4 matrix cores
# HBM bytes per launch of the streamed W2/A2 GEMV from the rocprofv3 counter runs summarised in
# profiles/gemv_streamed_4096x1024.md: 2.0 x FETCH_SIZE + 1.0 x WRITE_SIZE (scale factors from a plain
# 512 MiB device copy and a 1 GiB read) = (2 x 270918.5 + 8192.2) KiB
GEMV_TRAFFIC_BYTES = (2 * 270918.5 + 8192.2) * 1024
# the same for the two kernels of the primary workload (profiles/lstm_step_1024_b64_w3a3.md) and for the
# streamed batch-1 LSTM step (profiles/lstm_step_b1_streamed_1024_w3a3.md)
LSTM_FUSED_TRAFFIC_BYTES = (2 * 2109.4 + 512.0) * 1024
LSTM_QUANT_TRAFFIC_BYTES = (2 * 358.0 + 53.0) * 1024
LSTM_B1_TRAFFIC_BYTES = (2 * 271843.8 + 1368.0) * 1024
LSTM_FRONT_TRAFFIC_BYTES = (2 * 1309.9 + 1077.0) * 1024   # step_front_kernel, steady-state form
LSTM_BACK_TRAFFIC_BYTES = (2 * 1721.4 + 512.0) * 1024     # step_back_kernel
FP32_VALU_PEAK_TFLOPS = 157.3                # vector fp32
MIN_TIMED_CALLS = 100
MIN_WARMUP_CALLS = 10


def dv(a, dev):
    import torch
    a = np.ascontiguousarray(a)
    return torch.from_numpy(a.view(np.int32) if a.dtype == np.uint32 else a).to(dev)


def event_time_ms(fn, iters, warmup):
    """Average duration of fn() in ms from HIP events on the current stream."""
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters


def wall_time_ms(fn, iters, warmup):
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(iters):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / iters


def timed_calls(fn, calls, warmup):
    """`calls` calls of fn() after `warmup` untimed ones.  Every call sits between two HIP events on the
    current stream, and the wall clock brackets the whole run between two device synchronisations.
    Returns the per-call wall mean and the median / min / mean of the per-call event times (ms)."""
    import torch
    for _ in range(warmup):
        fn()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(calls + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev[0].record()
    for i in range(calls):
        fn()
        ev[i + 1].record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3 / calls
    per = np.array([ev[i].elapsed_time(ev[i + 1]) for i in range(calls)])
    return {"calls": calls, "warmup_calls": warmup, "wall_mean_ms": wall, "event_median_ms": float(np.median(per)),
            "event_min_ms": float(per.min()), "event_mean_ms": float(per.mean())}


# ------------------------------------------------------------------------------ workloads

def setup_lstm(amq, cfg, dev):
    k_w, T = cfg["k_w"], cfg["T"]
    Wxp, ax = amq.quantize_weights(dv(cfg["Wx"], dev), k_w, T)
    Whp, ah = amq.quantize_weights(dv(cfg["Wh"], dev), k_w, T)
    return Wxp, ax, Whp, ah


def bench_lstm_steps(amq, cfg, dev, steps, warmup):
    """Per-step launches of lstm_step over resident inputs, state carried on the GPU."""
    import torch
    I, H, B, k_a, T = cfg["I"], cfg["H"], cfg["B"], cfg["k_a"], cfg["T"]
    q = setup_lstm(amq, cfg, dev)
    xs = dv(cfg["xs"], dev)
    S = xs.shape[0]
    h = torch.zeros((B, H), device=dev)
    c = torch.zeros((B, H), device=dev)
    ws = amq.lstm_workspace(I, H, B, k_a, dev)
    state = {"t": 0}

    def step():
        t = state["t"]
        if t % S == 0:
            h.zero_()
            c.zero_()
        amq.lstm_step(*q, I, H, None, xs[t % S], h, c, k_a, T, ws=ws, h_out=h, c_out=c)
        state["t"] = t + 1

    ms = wall_time_ms(step, steps, warmup)
    return ms, q


def bench_lstm_sequence(amq, cfg, dev, seqs, warmup):
    import torch
    I, H, B, k_a, T = cfg["I"], cfg["H"], cfg["B"], cfg["k_a"], cfg["T"]
    q = setup_lstm(amq, cfg, dev)
    xs = dv(cfg["xs"], dev)
    S = xs.shape[0]
    state = torch.zeros((2, B, H), device=dev)   # h and c side by side: one fill per sequence
    h, c = state[0], state[1]
    ws = amq.lstm_sequence_workspace(I, H, B, k_a, dev)

    def seq():
        state.zero_()
        amq.lstm_sequence(*q, I, H, None, xs, h, c, k_a, T, ws=ws)

    st = timed_calls(seq, seqs, warmup)
    st["steps_per_call"] = S
    return st


def bench_lstm_graph(amq, cfg, dev, replays=100, warmup=10):
    """One sequence as per-step calls of lstm_step recorded once into a HIP graph and replayed."""
    import torch
    I, H, B, k_a, T = cfg["I"], cfg["H"], cfg["B"], cfg["k_a"], cfg["T"]
    q = setup_lstm(amq, cfg, dev)
    xs = dv(cfg["xs"], dev)
    S = xs.shape[0]
    h = torch.zeros((B, H), device=dev)
    c = torch.zeros((B, H), device=dev)
    ws = amq.lstm_workspace(I, H, B, k_a, dev)

    def seq():
        h.zero_()
        c.zero_()
        for t in range(S):
            amq.lstm_step(*q, I, H, None, xs[t], h, c, k_a, T, ws=ws, h_out=h, c_out=c)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        seq()                       # per-device kernel configuration happens outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    eager = (h.clone(), c.clone())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        seq()
    for _ in range(3):              # every replay gives the eager result
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(h, eager[0]) and torch.equal(c, eager[1]), "graph replay differs from the eager sequence"
    st = timed_calls(g.replay, replays, warmup)
    st["steps_per_call"] = S
    return st


def bench_lstm_fused_kernel(amq, cfg, dev, q, iters=300):
    """Average launch duration of the fused products + epilogue + cell kernel of one LSTM step
    (operands quantized beforehand, so nothing else runs between the events)."""
    import torch
    I, H, B, k_a, T = cfg["I"], cfg["H"], cfg["B"], cfg["k_a"], cfg["T"]
    x = dv(cfg["xs"][0], dev)
    h = dv(np.tanh(cfg["xs"][1][:, :H]).astype(np.float32), dev)
    c = torch.zeros((B, H), device=dev)
    Xp, bx = amq.quantize_activations(x, k_a, T)
    Hp, bh = amq.quantize_activations(h, k_a, T)
    ho, co = torch.empty_like(c), torch.empty_like(c)
    L = amq.binding.lib()
    s = torch.cuda.current_stream().cuda_stream
    k_w = q[0].shape[0]
    ptr = [t.data_ptr() for t in q]
    ms_fused = event_time_ms(lambda: L.amq_lstm_step_packed(ptr[0], ptr[1], ptr[2], ptr[3], I, H, k_w, None,
                                                            Xp.data_ptr(), bx.data_ptr(), Hp.data_ptr(),
                                                            bh.data_ptr(), c.data_ptr(), B, k_a, ho.data_ptr(),
                                                            co.data_ptr(), s), iters, 20)
    # the other kernel of a step: on-line quantization of the 2B vectors x_t, h_{t-1}
    xh = torch.cat([x, h], 0).contiguous()
    planes = torch.empty((k_a, 2 * B, amq.wpr(I)), dtype=torch.int32, device=dev)
    beta = torch.empty((2 * B, k_a), device=dev)
    ms_quant = event_time_ms(lambda: L.amq_quantize_activations(xh.data_ptr(), 2 * B, I, k_a, T, planes.data_ptr(),
                                                                beta.data_ptr(), s), iters, 20)
    return ms_fused, ms_quant


def bench_lstm_split_launches(amq, cfg, dev, q, iters=300):
    """Average duration of the two launches of a steady-state step of the batched sequence path, each alone:
    the front launch (quantize h_{t-1} and x_{t+1}, x-side sums of step t) and the back launch (h-side sums +
    stored x-side sums + cell).  Returns None where the sequence call does not take that path."""
    import torch
    I, H, B, k_a, T = cfg["I"], cfg["H"], cfg["B"], cfg["k_a"], cfg["T"]
    k_w = q[0].shape[0]
    xs = dv(cfg["xs"][:3], dev)
    h = torch.zeros((B, H), device=dev)
    c = torch.zeros((B, H), device=dev)
    ws = amq.lstm_sequence_workspace(I, H, B, k_a, dev)
    amq.lstm_sequence(*q, I, H, None, xs, h, c, k_a, T, ws=ws)   # leaves valid codes and sums in the workspace
    L = amq.binding.lib()
    s = torch.cuda.current_stream().cuda_stream
    ptr = [t.data_ptr() for t in q]

    def half(which):
        return L.amq_debug_lstm_split_half(ptr[0], ptr[1], ptr[2], ptr[3], I, H, k_w, None, xs[2].data_ptr(),
                                           h.data_ptr(), c.data_ptr(), B, k_a, T, ws.data_ptr(), ws.numel(), which, s)

    if half(0) != 0:
        return None
    return (event_time_ms(lambda: half(0), iters, 20), event_time_ms(lambda: half(1), iters, 20))


def gemm_algorithmic(m, n, k_w, k_a, batch):
    """Bit-MACs, integer lane-ops (xor + popcount-accumulate per 32 bit-MACs) and bytes of one product."""
    macs = float(m) * n * k_w * k_a * batch
    lane_ops = 2.0 * macs / 32.0
    wpr = 4 * ((n + 127) // 128)
    nbytes = k_w * m * wpr * 4 + m * k_w * 4 + batch * (k_a * wpr * 4 + k_a * 4) + batch * m * 4
    return macs, lane_ops, nbytes


def bench_gemm_kernel(amq, dev, m, n, k_w, k_a, batch, iters=200):
    """Average launch duration of the binary GEMM kernel at the shape the LSTM step uses."""
    import torch
    g = torch.Generator(device="cpu").manual_seed(1)
    wpr = amq.wpr(n)
    Wp = torch.randint(-2 ** 31, 2 ** 31 - 1, (k_w, m, wpr), dtype=torch.int32, generator=g).to(dev)
    Xp = torch.randint(-2 ** 31, 2 ** 31 - 1, (k_a, batch, wpr), dtype=torch.int32, generator=g).to(dev)
    alpha = torch.rand((m, k_w), generator=g).to(dev)
    beta = torch.rand((batch, k_a), generator=g).to(dev)
    Y = torch.empty((batch, m), device=dev)
    L = amq.binding.lib()
    s = torch.cuda.current_stream().cuda_stream
    ms = event_time_ms(lambda: L.amq_binary_gemm(Wp.data_ptr(), alpha.data_ptr(), m, n, k_w, Xp.data_ptr(),
                                                 beta.data_ptr(), batch, k_a, None, 0, Y.data_ptr(), s), iters, 20)
    return ms


def bench_gemv_stream(amq, dev, m, n, k_w, k_a, total_bytes=512 << 20, iters=20):
    """Grouped batch-1 GEMV over enough independent matrices that every plane byte comes from HBM."""
    import torch
    wpr = amq.wpr(n)
    per = k_w * m * wpr * 4
    G = max(1, total_bytes // per)
    g = torch.Generator(device="cpu").manual_seed(2)
    Wp = torch.randint(-2 ** 31, 2 ** 31 - 1, (G, k_w, m, wpr), dtype=torch.int32, generator=g).to(dev)
    Xp = torch.randint(-2 ** 31, 2 ** 31 - 1, (G, k_a, wpr), dtype=torch.int32, generator=g).to(dev)
    alpha = torch.rand((G, m, k_w), generator=g).to(dev)
    beta = torch.rand((G, k_a), generator=g).to(dev)
    Y = torch.empty((G, m), device=dev)
    ms = event_time_ms(lambda: amq.binary_gemv_grouped(Wp, alpha, n, Xp, beta, Y=Y), iters, 3)
    _, _, nbytes = gemm_algorithmic(m, n, k_w, k_a, 1)
    return ms, G, G * nbytes


def bench_stream_probe(amq, dev, nbytes=1 << 30, iters=20):
    """Read-only streaming kernel over 1 GiB: the bandwidth a plain read reaches on this GPU."""
    import torch
    buf = torch.empty(nbytes // 4, dtype=torch.int32, device=dev).random_()
    sink = torch.empty(amq.binding.STREAM_PROBE_SINK_WORDS, dtype=torch.int64, device=dev)
    ms = event_time_ms(lambda: amq.stream_read_probe(buf, sink), iters, 3)
    return nbytes / (ms * 1e-3) / 1e9, ms


def bench_lstm_b1_stream(amq, dev, I, H, k_w, k_a, total_bytes=512 << 20, iters=20):
    """G independent batch-1 LSTM steps on packed operands in one launch, G x (bytes of one cell's weight
    planes) >= 512 MiB, so every plane byte comes from HBM.  Returns ms, G and the algorithmic bytes:
    planes + alpha of both blocks, codes + beta of x and h, c_prev in, h and c out."""
    import torch
    wx, wh = amq.wpr(I), amq.wpr(H)
    per_planes = k_w * 4 * H * (wx + wh) * 4
    G = (total_bytes + per_planes - 1) // per_planes
    g = torch.Generator(device="cpu").manual_seed(4)

    def words(*shape):
        return torch.randint(-2 ** 31, 2 ** 31 - 1, shape, dtype=torch.int32, generator=g).to(dev)

    Wxp, Whp = words(G, k_w, 4 * H, wx), words(G, k_w, 4 * H, wh)
    ax = (torch.rand((G, 4 * H, k_w), generator=g) * 0.02).to(dev)
    ah = (torch.rand((G, 4 * H, k_w), generator=g) * 0.02).to(dev)
    Xp, Hp = words(G, k_a, wx), words(G, k_a, wh)
    bx, bh = torch.rand((G, k_a), generator=g).to(dev), torch.rand((G, k_a), generator=g).to(dev)
    c = torch.randn((G, H), generator=g).to(dev)
    ho, co = torch.empty_like(c), torch.empty_like(c)
    ms = event_time_ms(lambda: amq.lstm_step_packed_grouped(Wxp, ax, Whp, ah, I, H, None, Xp, bx, Hp, bh, c,
                                                            h_out=ho, c_out=co), iters, 3)
    per = per_planes + 2 * 4 * H * k_w * 4 + k_a * (wx + wh) * 4 + 2 * k_a * 4 + 3 * H * 4
    return ms, G, G * per


def bench_gemv_warm(amq, dev, m, n, k, iters=2000):
    import torch
    g = torch.Generator(device="cpu").manual_seed(3)
    wpr = amq.wpr(n)
    Wp = torch.randint(-2 ** 31, 2 ** 31 - 1, (k, m, wpr), dtype=torch.int32, generator=g).to(dev)
    Xp = torch.randint(-2 ** 31, 2 ** 31 - 1, (k, 1, wpr), dtype=torch.int32, generator=g).to(dev)
    alpha = torch.rand((m, k), generator=g).to(dev)
    beta = torch.rand((1, k), generator=g).to(dev)
    Y = torch.empty((1, m), device=dev)
    L = amq.binding.lib()
    s = torch.cuda.current_stream().cuda_stream
    return event_time_ms(lambda: L.amq_binary_gemv(Wp.data_ptr(), alpha.data_ptr(), m, n, k, Xp.data_ptr(),
                                                   beta.data_ptr(), k, None, 0, Y.data_ptr(), s), iters, 50)


def bench_quantizer(amq, dev, k, iters=10):
    import torch
    from paper_1802_00150_amd import inputs
    W = dv(inputs.heavy_tailed(), dev)
    rows, cols = W.shape
    planes = torch.empty((k, rows, amq.wpr(cols)), dtype=torch.int32, device=dev)
    alpha = torch.empty((rows, k), device=dev)
    L = amq.binding.lib()
    s = torch.cuda.current_stream().cuda_stream
    st = timed_calls(lambda: L.amq_quantize_weights(W.data_ptr(), rows, cols, cols, k, 2, planes.data_ptr(),
                                                    alpha.data_ptr(), s), max(10, iters), 3)
    nbytes = rows * cols * 4 + planes.numel() * 4 + alpha.numel() * 4
    return st, nbytes, rows * cols


def bench_gru(amq, dev, steps, warmup):
    import torch
    from paper_1802_00150_amd import inputs
    cfg = inputs.gru_proj(steps=8)
    I, H, B, k_w, k_a, k_p, T = cfg["I"], cfg["H"], cfg["B"], cfg["k_w"], cfg["k_a"], cfg["k_proj"], cfg["T"]
    q = setup_lstm(amq, cfg, dev)
    Wsp, as_ = amq.quantize_weights(dv(cfg["Ws"], dev), k_w, T)
    xs = dv(cfg["xs"], dev)
    h = torch.zeros((B, H), device=dev)
    ws = amq.gru_workspace(I, H, B, k_a, dev)
    logits = torch.empty((B, cfg["V"]), device=dev)
    state = {"t": 0}

    def step():
        t = state["t"]
        amq.gru_step(*q, I, H, None, None, xs[t % 8], h, k_a, T, ws=ws, h_out=h)
        pH, bH = amq.quantize_activations(h, k_p, T)
        amq.binary_gemm(Wsp, as_, H, pH, bH, Y=None)
        state["t"] = t + 1

    ms = wall_time_ms(step, steps, warmup)

    # The same work when the inputs of a sequence are given: 16 recurrent steps keep their h_t, then
    # one quantize launch and one projection take all 16 x 256 rows.
    n = 16
    hs = torch.zeros((n, B, H), device=dev)
    xs16 = torch.cat([xs, xs], 0).contiguous()
    h16 = torch.zeros((B, H), device=dev)
    ws_seq = amq.gru_sequence_workspace(I, H, B, k_a, dev)
    pH = torch.empty((k_p, n * B, amq.wpr(H)), dtype=torch.int32, device=dev)
    bH = torch.empty((n * B, k_p), device=dev)
    Y = torch.empty((n * B, cfg["V"]), device=dev)
    L = amq.binding.lib()
    s = torch.cuda.current_stream().cuda_stream

    def seq():
        amq.gru_sequence(*q, I, H, None, None, xs16, h16, k_a, T, ws=ws_seq, hs=hs)
        st = L.amq_quantize_activations(hs.data_ptr(), n * B, H, k_p, T, pH.data_ptr(), bH.data_ptr(), s)
        assert st == 0, st
        st = L.amq_binary_gemm(Wsp.data_ptr(), as_.data_ptr(), cfg["V"], H, k_w, pH.data_ptr(), bH.data_ptr(), n * B,
                               k_p, None, 0, Y.data_ptr(), s)
        assert st == 0, st

    ms_seq = wall_time_ms(seq, max(2, steps // n), 2) / n
    return ms, ms_seq


def bench_gru_sequence(amq, dev, B=64, S=35, calls=30, warmup=5):
    """GRU 1024/1024 W2/A2 at a batch where the sequence call takes the input products off the recurrent chain:
    ms per step through amq_gru_sequence and through per-step amq_gru_step calls."""
    import torch
    from paper_1802_00150_amd import inputs
    cfg = inputs.gru_proj(steps=8)
    I, H, k_w, k_a, T = cfg["I"], cfg["H"], cfg["k_w"], cfg["k_a"], cfg["T"]
    q = setup_lstm(amq, cfg, dev)
    g = torch.Generator(device="cpu").manual_seed(11)
    xs = torch.randn((S, B, I), generator=g).to(dev)
    h = torch.zeros((B, H), device=dev)
    ws = amq.gru_sequence_workspace(I, H, B, k_a, dev)

    def seq():
        h.zero_()
        amq.gru_sequence(*q, I, H, None, None, xs, h, k_a, T, ws=ws)

    def steps():
        h.zero_()
        for t in range(S):
            amq.gru_step(*q, I, H, None, None, xs[t], h, k_a, T, ws=ws, h_out=h)

    return wall_time_ms(seq, calls, warmup) / S, wall_time_ms(steps, calls, warmup) / S


def bench_lm(amq, dev, B, steps, warmup):
    """Whole language-model steps (token ids -> log-probabilities), hidden 1024, vocabulary 42000, W2/A2."""
    import torch
    from paper_1802_00150_amd import inputs
    cfg = inputs.language_model(steps=8, B=B)
    E, H, V, k, T = cfg["E"], cfg["H"], cfg["V"], cfg["k_w"], cfg["T"]
    Ep, ae = amq.quantize_weights(dv(cfg["emb"], dev), k, T)
    Wxp, ax = amq.quantize_weights(dv(cfg["Wx"], dev), k, T)
    Whp, ah = amq.quantize_weights(dv(cfg["Wh"], dev), k, T)
    Wsp, as_ = amq.quantize_weights(dv(cfg["Ws"], dev), k, T)
    bs = dv(cfg["bs"], dev)
    ids = torch.from_numpy(cfg["ids"]).to(dev)
    h = torch.zeros((B, H), device=dev)
    c = torch.zeros((B, H), device=dev)
    ws = amq.lm_workspace(E, H, V, B, k, k, dev)
    logprob = torch.empty((B, V), device=dev)
    state = {"t": 0}

    def step():
        t = state["t"]
        amq.lm_step(Ep, ae, E, Wxp, ax, Whp, ah, H, None, Wsp, as_, bs, ids[t % 8], h, c, k, k, T, ws=ws,
                    logprob=logprob)
        state["t"] = t + 1

    ms = wall_time_ms(step, steps, warmup)
    # the same as whole 35-step sequences through one call
    ids35 = torch.from_numpy(inputs.language_model(steps=35, B=B)["ids"]).to(dev)
    wsq = torch.empty(int(amq.binding.lib().amq_lm_sequence_workspace_bytes(E, H, V, B, k, k)), dtype=torch.uint8,
                      device=dev)
    lp35 = torch.empty((35, B, V), device=dev)
    ms_seq = wall_time_ms(lambda: amq.lm_sequence(Ep, ae, E, Wxp, ax, Whp, ah, H, None, Wsp, as_, bs, ids35, h, c, k, k,
                                                  T, ws=wsq, logprob=lp35), 10, 2) / 35
    # scoring: only the log-probability of a given next word per step and batch entry
    tg35 = torch.randint(0, V, (35, B), dtype=torch.int64, generator=torch.Generator().manual_seed(7)).to(dev)
    wss = torch.empty(int(amq.binding.lib().amq_lm_sequence_score_workspace_bytes(E, H, V, B, k, k)), dtype=torch.uint8,
                      device=dev)
    sc35 = torch.empty((35, B), device=dev)
    ms_score = wall_time_ms(lambda: amq.lm_sequence_score(Ep, ae, E, Wxp, ax, Whp, ah, H, None, Wsp, as_, bs, ids35, tg35,
                                                          h, c, k, k, T, ws=wss, out=sc35), 10, 2) / 35
    ws2 = amq.softmax_layer_workspace(V, H, B, k, dev)
    ms_layer = event_time_ms(lambda: amq.softmax_layer(Wsp, as_, H, bs, h, k, T, ws=ws2, logprob=logprob), 200, 20)
    ms_lsm = event_time_ms(lambda: amq.log_softmax(logprob, out=logprob), 200, 20)
    return ms, ms_layer, ms_lsm, ms_seq, ms_score


def bench_relative_mse(amq, dev):
    """Relative MSE of greedy (T = 0), refined greedy and alternating (T = 2) quantization of the
    config-3 gate matrix (4096 x 2048, Gaussian) and of a heavy-tailed 4096 x 4096 matrix."""
    from paper_1802_00150_amd import inputs
    cfg = inputs.lstm_large(steps=1)
    mats = {"lstm_4096x2048_gaussian": np.concatenate([cfg["Wx"], cfg["Wh"]], axis=1),
            "heavy_tailed_4096x4096": inputs.heavy_tailed(rows=4096, cols=4096)}
    out = {}
    for name, W in mats.items():
        d = dv(W, dev)
        tab = {}
        for k in (2, 3, 4):
            row = {}
            for method, (pl, al) in (("greedy", amq.quantize_weights(d, k, 0)),
                                     ("refined", amq.quantize_refined_greedy(d, k)),
                                     ("alternating", amq.quantize_weights(d, k, 2))):
                row[method] = float(amq.relative_mse(d, pl, al)[0][2].item())
            tab["k%d" % k] = row
        pl, al = amq.quantize_ternary(d, 2)   # the 2-bit case with equal coefficients
        tab["ternary"] = float(amq.relative_mse(d, pl, al)[0][2].item())
        out[name] = tab
    return out


def cpu_baseline_lstm(cfg, budget_s=15.0):
    """The oracle, as it stands, on the same LSTM workload: whole steps on all host threads."""
    import oracle
    threads = oracle.set_threads(oracle.host_threads())
    I, H, B, k_w, k_a, T = cfg["I"], cfg["H"], cfg["B"], cfg["k_w"], cfg["k_a"], cfg["T"]
    Wxp, ax = oracle.quantize_rows(cfg["Wx"], k_w, T)
    Whp, ah = oracle.quantize_rows(cfg["Wh"], k_w, T)
    h = np.zeros((B, H), np.float32)
    c = np.zeros((B, H), np.float32)
    n = 0
    t0 = time.perf_counter()
    while True:
        h, c = oracle.lstm_step(Wxp, ax, Whp, ah, I, H, None, cfg["xs"][n % cfg["xs"].shape[0]], h, c, k_a, T)
        n += 1
        el = time.perf_counter() - t0
        if el > budget_s or n >= 140:
            break
    return {"value": n / el, "unit": "steps/s", "cores": threads, "kind": "oracle",
            "sample": "%d whole LSTM steps of the primary workload (B=%d, hidden %d, W%d/A%d), OpenMP over rows"
                      % (n, B, H, k_w, k_a)}


SECTIONS = ["primary", "lstm_b1", "gemv", "gemm", "gru", "lm", "quantizer", "mse", "cpu"]   # + probe, copy_probe


def copy_probe(dev, nbytes=512 << 20, iters=10):
    """A plain device copy of known size: the yardstick that scales the HBM byte counters."""
    import torch
    src = torch.empty(nbytes // 4, dtype=torch.int32, device=dev).random_()
    dst = torch.empty_like(src)
    ms = event_time_ms(lambda: dst.copy_(src), iters, 2)
    return {"bytes_read": nbytes, "bytes_written": nbytes, "ms": ms, "GBps": 2 * nbytes / (ms * 1e-3) / 1e9}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=700)
    ap.add_argument("--warmup", type=int, default=70)
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--counters", action="store_true",
                    help="run under a counter-collecting profiler: few launches of everything (timings are then meaningless)")
    ap.add_argument("--sections", default=",".join(SECTIONS),
                    help="comma list out of %s, plus copy_probe (for counter calibration)" % SECTIONS)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus %d is not supported "
              "(no sharding or collectives are part of it)" % args.gpus, file=sys.stderr)
        sys.exit(2)
    sections = set(args.sections.split(","))
    if args.no_cpu:
        sections.discard("cpu")

    import torch
    import paper_1802_00150_amd as amq
    from paper_1802_00150_amd import inputs
    amq.binding.lib()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)

    out = {"metric": "quantized LSTM steps/sec (batch 64)", "value": None, "unit": "steps/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": None,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "1-bit codes (fp4 MFMA / u32 popcount, exact) + f32",
           "data": "synthetic",
           "config": {"workload": "config 3: LSTM input 1024 hidden 1024, batch 64, 35-step sequences, "
                                  "weights row-wise 3-bit, activations 3-bit on line, T=2",
                      "global_batch": 64, "seq_len": 35}}
    also = {}
    cfg = inputs.lstm_large()

    probe_gbps = None
    if sections & {"lstm_b1", "gemv", "quantizer", "probe"}:
        probe_gbps, probe_ms = bench_stream_probe(amq, dev)
        also["stream_read_probe_1GiB_GBps"] = probe_gbps
        also["stream_read_probe_frac_of_nominal"] = probe_gbps / HBM_PEAK_GBPS

    def hbm_roofline(kernel, gbps, ms, nbytes, traffic, source):
        # `traffic` is the counter figure recorded in the named summary (a separate rocprofv3 run of this
        # file), not something measured in this run
        return {"kernel": kernel, "bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": gbps / HBM_PEAK_GBPS, "frac_of_stream_read_probe": gbps / probe_gbps if probe_gbps else None,
                "traffic": traffic, "traffic_source": source, "launch_ms": ms, "bytes_per_launch": nbytes}

    if "primary" in sections:
        # config 3, LSTM 1024/1024, batch 64, W3/A3, T=2: whole 35-step sequences through
        # amq_lstm_sequence (launches issued from C, state carried on the GPU); never fewer than
        # 100 timed calls after 10 warm-up calls
        H, B, k_w, k_a, T = cfg["H"], cfg["B"], cfg["k_w"], cfg["k_a"], cfg["T"]
        S = cfg["xs"].shape[0]
        seqs = max(MIN_TIMED_CALLS, (args.steps + S - 1) // S)
        warm = max(MIN_WARMUP_CALLS, (args.warmup + S - 1) // S)
        if args.counters:
            seqs, warm = 3, 2
        st = bench_lstm_sequence(amq, cfg, dev, seqs, warm)
        out["steps"] = seqs * S
        out["warmup"] = warm * S
        ms_step = st["wall_mean_ms"] / S          # whole-job figure: wall clock over every timed call
        out["value"] = 1e3 / ms_step
        out["ms_per_step"] = ms_step
        out["timing"] = {"sequence_calls": seqs, "warmup_calls": warm, "steps_per_call": S,
                         "wall_us_per_step": ms_step * 1e3,
                         "event_us_per_step_median": st["event_median_ms"] / S * 1e3,
                         "event_us_per_step_min": st["event_min_ms"] / S * 1e3,
                         "event_us_per_step_mean": st["event_mean_ms"] / S * 1e3}
        ms_call, q = bench_lstm_steps(amq, cfg, dev, 35 if args.counters else max(args.steps, 700),
                                      35 if args.counters else max(args.warmup, 70))
        also["lstm_b64_per_step_call_steps_per_s"] = 1e3 / ms_call
        # The two kernels of a step as amq_lstm_step runs it: on-line quantization of the 2B vectors x_t,
        # h_{t-1}, then the products with both weight blocks + coefficient epilogue + cell on the fp4 matrix
        # cores (codes as {-1,+1}).
        ms_fused, ms_quant = bench_lstm_fused_kernel(amq, cfg, dev, q, iters=20 if args.counters else 300)
        also["lstm_b64_fused_kernel_us"] = ms_fused * 1e3
        also["lstm_b64_quantize_kernel_us"] = ms_quant * 1e3
        macs_block = 4.0 * H * cfg["I"] * k_w * k_a * B       # one weight block: bit-level multiply-adds
        n = cfg["I"]
        # Sec. 3 cost of Alg. 2 per n-vector: 2 T k^2 n binary + 2 (T+1) k n non-binary operations
        qops = 2 * B * (2.0 * T * k_a * k_a * n + 2.0 * (T + 1) * k_a * n)
        split = bench_lstm_split_launches(amq, cfg, dev, q, iters=20 if args.counters else 300)
        if split is not None:
            # The sequence call runs a step as a front and a back launch; `roofline` is the longer one.
            ms_front, ms_back = split
            also["lstm_b64_front_launch_us"] = ms_front * 1e3
            also["lstm_b64_back_launch_us"] = ms_back * 1e3
            r_front = {"kernel": "step_front_kernel<3,3,lstm>: Alg. 2 on the 64 vectors of h_{t-1} (the chain; 64 "
                                 "workgroups of 4 waves, latency-bound) with, in its shadow, Alg. 2 on the 64 vectors of "
                                 "x_{t+1} and the W3/A3 product W_x x_t (4096x1024, B=64) on the matrix cores",
                       "bound": "alu", "achieved": qops / (ms_front * 1e-3) / 1e12, "peak": FP32_VALU_PEAK_TFLOPS,
                       "unit": "TFLOP/s", "frac": qops / (ms_front * 1e-3) / 1e12 / FP32_VALU_PEAK_TFLOPS,
                       "traffic": LSTM_FRONT_TRAFFIC_BYTES, "traffic_source": "profiles/lstm_step_1024_b64_w3a3.md",
                       "launch_ms": ms_front, "flops_per_launch": qops,
                       "shadow_matrix_flops_per_launch": 2.0 * macs_block,
                       "note": "operations = Sec. 3's count for the 128 vectors; the launch lasts as long as the chain "
                               "of five dependent workgroup-wide reductions of one vector"}
            ach = 2.0 * macs_block / (ms_back * 1e-3) / 1e12
            r_back = {"kernel": "step_back_kernel<3,3,lstm>: W3/A3 product W_h h_{t-1} (4096x1024, B=64) + stored "
                                "x-side sums + cell",
                      "bound": "mfma", "achieved": ach, "peak": FP4_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                      "frac": ach / FP4_MFMA_PEAK_TFLOPS, "traffic": LSTM_BACK_TRAFFIC_BYTES,
                      "traffic_source": "profiles/lstm_step_1024_b64_w3a3.md", "launch_ms": ms_back,
                      "flops_per_launch": 2.0 * macs_block}
            first, second = (r_front, r_back) if ms_front >= ms_back else (r_back, r_front)
        else:
            achieved = 4.0 * macs_block / (ms_fused * 1e-3) / 1e12
            r_prod = {"kernel": "mfma4p_kernel<3,3,1,lstm,8>: W3/A3 products with both 4096x1024 blocks (B=64) + cell",
                      "bound": "mfma", "achieved": achieved, "peak": FP4_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                      "frac": achieved / FP4_MFMA_PEAK_TFLOPS, "traffic": LSTM_FUSED_TRAFFIC_BYTES,
                      "traffic_source": "profiles/lstm_step_1024_b64_w3a3.md", "launch_ms": ms_fused,
                      "flops_per_launch": 4.0 * macs_block}
            qach = qops / (ms_quant * 1e-3) / 1e12
            r_quant = {"kernel": "quantize_kernel<3,4,4>: Alg. 2 on the 128 vectors x_t, h_{t-1} of length 1024 "
                                 "(128 workgroups of 4 waves: latency-bound, half the CUs idle)",
                       "bound": "alu", "achieved": qach, "peak": FP32_VALU_PEAK_TFLOPS, "unit": "TFLOP/s",
                       "frac": qach / FP32_VALU_PEAK_TFLOPS, "traffic": LSTM_QUANT_TRAFFIC_BYTES,
                       "traffic_source": "profiles/lstm_step_1024_b64_w3a3.md", "launch_ms": ms_quant,
                       "flops_per_launch": qops}
            first, second = (r_prod, r_quant) if ms_fused >= ms_quant else (r_quant, r_prod)
        out["roofline"] = first
        out["roofline_second_kernel"] = second

    if "lstm_b1" in sections:
        # batch-1 LSTM, config 1 (hidden 300): (i) one launch pair per step, (ii) the same launches replayed
        # from a HIP graph, (iii) one call per sequence (grid-persistent kernel, weights on chip)
        cb = inputs.lstm_large(B=1)
        if not args.counters:
            c1 = inputs.lstm_small()
            ms1, _ = bench_lstm_steps(amq, c1, dev, 700, 70)
            st1 = bench_lstm_sequence(amq, c1, dev, 100, 10)
            stg = bench_lstm_graph(amq, c1, dev)
            also["lstm_b1_hidden300_steps_per_s"] = 1e3 / ms1
            also["lstm_b1_hidden300_hip_graph_steps_per_s"] = 1e3 * stg["steps_per_call"] / stg["event_median_ms"]
            also["lstm_b1_hidden300_sequence_call_steps_per_s"] = 1e3 * st1["steps_per_call"] / st1["event_median_ms"]
            msb, _ = bench_lstm_steps(amq, cb, dev, 700, 70)
            stb = bench_lstm_sequence(amq, cb, dev, 100, 10)
            also["lstm_b1_hidden1024_w3a3_steps_per_s"] = 1e3 / msb
            also["lstm_b1_hidden1024_w3a3_sequence_call_steps_per_s"] = (1e3 * stb["steps_per_call"] /
                                                                         stb["event_median_ms"])
        # the HBM-bound form of the batch-1 step: config 3's shape at B = 1, G independent cells streamed
        ms, G, nbytes = bench_lstm_b1_stream(amq, dev, cb["I"], cb["H"], cb["k_w"], cb["k_a"])
        gbps = nbytes / (ms * 1e-3) / 1e9
        also["lstm_b1_hidden1024_w3a3_streamed_GBps"] = gbps
        out["roofline_lstm_b1"] = hbm_roofline("bmv_kernel<3,3,1,lstm>: batch-1 LSTM step 1024/1024 W3/A3 on packed "
                                               "operands, %d independent cells streamed" % G, gbps, ms, nbytes,
                                               LSTM_B1_TRAFFIC_BYTES, "profiles/lstm_step_b1_streamed_1024_w3a3.md")

    if "gemv" in sections:
        # batch-1 GEMV, config 2: streamed from HBM (grouped) and cache-resident latency
        for k in (2, 3):
            ms, G, nbytes = bench_gemv_stream(amq, dev, 4096, 1024, k, k)
            gbps = nbytes / (ms * 1e-3) / 1e9
            also["gemv_b1_w%da%d_streamed_GBps" % (k, k)] = gbps
            if k == 2:
                out["roofline_gemv"] = hbm_roofline("binary GEMV 4096x1024 W2/A2 batch 1, %d matrices streamed" % G,
                                                    gbps, ms, nbytes, GEMV_TRAFFIC_BYTES,
                                                    "profiles/gemv_streamed_4096x1024.md")
            also["gemv_b1_w%da%d_warm_call_us" % (k, k)] = bench_gemv_warm(amq, dev, 4096, 1024, k) * 1e3

    if "gemm" in sections:
        for b in (8, 64):
            for k in (2, 3):
                ms = bench_gemm_kernel(amq, dev, 4096, 1024, k, k, b)
                also["gemm_b%d_w%da%d_us" % (b, k, k)] = ms * 1e3
        # config 4's output projection: 10000 x 1024, W2 / A3, batch 256 -> fp32 logits
        ms = bench_gemm_kernel(amq, dev, 10000, 1024, 2, 3, 256)
        also["projection_10000x1024_w2a3_b256_us"] = ms * 1e3
        also["projection_10000x1024_w2a3_b256_TFLOPs"] = 2.0 * 10000 * 1024 * 6 * 256 / (ms * 1e-3) / 1e12
        # the same kernel where issue rate rather than the latency of one launch decides: batch 1024
        for (m, k) in ((42000, 2), (16384, 3)):
            ms = bench_gemm_kernel(amq, dev, m, 1024, k, k, 1024, iters=50)
            also["gemm_%dx1024_w%da%d_b1024_us" % (m, k, k)] = ms * 1e3
            also["gemm_%dx1024_w%da%d_b1024_TFLOPs" % (m, k, k)] = 2.0 * m * 1024 * k * k * 1024 / (ms * 1e-3) / 1e12

    if "gru" in sections:
        ms, ms_seq = bench_gru(amq, dev, 100, 10)
        also["gru_b256_with_projection_steps_per_s"] = 1e3 / ms
        also["gru_b256_projection_over_16_steps_at_once_steps_per_s"] = 1e3 / ms_seq
        ms_gs, ms_gp = bench_gru_sequence(amq, dev)
        also["gru_h1024_b64_w2a2_sequence_call_steps_per_s"] = 1e3 / ms_gs
        also["gru_h1024_b64_w2a2_per_step_call_steps_per_s"] = 1e3 / ms_gp

    if "lm" in sections:
        # full language-model step at the paper's large shape: embedding lookup, LSTM 1024, output layer
        # 42000 x 1024 with log-softmax, W2/A2
        for b in (1, 64):
            ms, ms_layer, ms_lsm, ms_seq, ms_score = bench_lm(amq, dev, b, 300, 30)
            also["lm_h1024_v42000_w2a2_b%d_steps_per_s" % b] = 1e3 / ms
            also["lm_h1024_v42000_w2a2_b%d_sequence_call_steps_per_s" % b] = 1e3 / ms_seq
            also["lm_h1024_v42000_w2a2_b%d_sequence_score_steps_per_s" % b] = 1e3 / ms_score
            also["lm_output_layer_42000x1024_b%d_us" % b] = ms_layer * 1e3
            also["lm_log_softmax_42000_b%d_us" % b] = ms_lsm * 1e3

    if "quantizer" in sections:
        # config 5.  Per k: time against max(bytes / HBM rate, operations / vector-ALU rate), with the bytes
        # 4 + k/8 per entry and the operations of Sec. 3's cost model, 2 T k^2 + 2 (T+1) k per entry at T = 2,
        # priced at one lane-operation each
        qz = {}
        for k in (1, 2, 3, 4):
            st, nbytes, entries = bench_quantizer(amq, dev, k)
            ms = st["event_median_ms"]
            t_hbm = nbytes / (HBM_PEAK_GBPS * 1e9) * 1e3
            t_alu = entries * (2.0 * 2 * k * k + 2.0 * 3 * k) / (VALU_PEAK_TOPS * 1e12) * 1e3
            qz["k%d" % k] = {"us_median": ms * 1e3, "us_min": st["event_min_ms"] * 1e3, "launches": st["calls"],
                             "GBps": nbytes / (ms * 1e-3) / 1e9, "hbm_floor_us": t_hbm * 1e3,
                             "alu_floor_us": t_alu * 1e3, "bound": "hbm" if t_hbm >= t_alu else "alu",
                             "frac_of_floor": max(t_hbm, t_alu) / ms,
                             "frac_of_stream_read_probe": nbytes / (ms * 1e-3) / 1e9 / probe_gbps}
            also["quantize_weights_16384x4096_k%d_GBps" % k] = nbytes / (ms * 1e-3) / 1e9
        also["quantize_weights_16384x4096"] = qz

    if "mse" in sections:
        also["relative_mse"] = bench_relative_mse(amq, dev)

    if "copy_probe" in sections:
        also["copy_probe"] = copy_probe(dev)

    out["also"] = also
    if "cpu" in sections:
        out["cpu_baseline"] = cpu_baseline_lstm(cfg)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
