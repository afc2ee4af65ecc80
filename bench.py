#!/usr/bin/env python3
"""Benchmark of the SWA+LTE hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline] [--no-decode] [--no-train]

One "step" = one pass of the whole hot path over the prefill_bf16 workload (B=4 sequences x 4096 tokens,
H=16, D=64, window 512, budget 256, CNN width 5 / 32 channels): ltea_prefill (scoring CNN -> capped
retention + cache fill -> window + retained attention) followed by one ltea_decode_step that continues
every sequence by one token on the cache just produced.  Inputs are synthetic, seeded, and resident in HBM
before the timed region; four rotating copies of the inputs keep the 256 MB Infinity Cache from standing
in for HBM.  `value` = tokens (prefill + decoded) per second over blocks of exactly K timed steps, each between two
synchronizations, repeated until 100 ms are timed (`timing` holds the block and per-step-event minima and medians).

Also reported on the same JSON line:
  roofline      the dominant kernel of the step (the prefill attention kernel) against the bf16 MFMA peak:
                algorithmic FLOPs (4*D per unmasked query-key pair, counted from the actual retained sets)
                / its average duration measured with HIP events on the launch stream in an instrumented
                repeat of the same steps (entry points called one by one).
  configs       the long_prefill_bf16, varlen_prefill_bf16 and paper_stack_bf16 configurations through the same
                step, each with its own attention and scoring roofline objects (fewer steps; --no-other-configs skips).
  decode        the decode_bf16 workload (B=64, H=16, D=128, window 1024 + 512 retained, n_seen 8192):
                256 consecutive steps timed as a whole; us/step, us/token, and the streaming attention
                kernel's achieved HBM bandwidth; `lazy`: the same steps without per-step scoring plus one
                batched scoring per ltea_lazy_period() steps.
  train         training-side forward + backward (no cap) on the paper's module shape, every head keeping
                budget/N of its tokens; ms per pass and the backward kernels against the bf16 MFMA peak; the scoring
                CNN's own backward is timed beside it (cnn_backward_ms).
  seqlen_sweep  (--seqlen-sweep) the attention kernel alone and the paper's whole LTE layer against the sequence
                length at batch 32 (the shapes of the paper's efficiency figures).
  cpu_baseline  the fp64 NumPy oracle timed on this machine's host cores on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E


WORKLOAD_TEXT = {
    "prefill": "prefill_bf16: B=4 x n=4096, H=16, D=64, window=512, budget=256, CNN k=5 C=32, "
               "Q,K,V~N(0,1)/sqrt(D), weights~N(0,0.05); + 1 decode step per sequence",
    "long": "long_prefill_bf16: B=1 x n=32768, H=32, D=128, window=2048, budget=1024, CNN k=7 C=32, Q,K,V~N(0,1); "
            "+ 1 decode step",
    "varlen": "varlen_prefill_bf16: 16 sequences of 1024..16384 tokens packed, H=16, D=128, window=1024, budget=512, "
              "CNN k=5 C=32, 1% planted near-duplicate keys; + 1 decode step per sequence",
    "paper": "paper_stack_bf16: B=4 x n=4096, Hq=32 on Hkv=8, D=64, window=768, budget=512, sink=4, CNN 3 x (k=3, "
             "dilation 2) with 64/32/16 channels, Q,K,V~N(0,1); + 1 decode step per sequence",
}


def measured_traffic(workload, kernel):
    """HBM bytes per launch (fetch + write) of a kernel from the committed rocprofv3 counter summary, or None."""
    try:
        with open(os.path.join(ROOT, "profiles", "traffic_per_launch.json")) as f:
            t = json.load(f)[workload][kernel]
        return t["fetch_bytes"] + t["write_bytes"]
    except (OSError, KeyError, ValueError):
        return None


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def up(x, dtype):
    import torch
    from paper_2510_20787_amd import binding as B
    return torch.from_numpy(np.ascontiguousarray(x)).to("cuda", B.torch_dtype(dtype))


def attention_pairs(w, ret_pos, ret_count):
    """Unmasked (query, key) pairs per the index set: window pairs + for every retained j the n-w-j queries
    that see it, summed over sequences and query heads."""
    G = w.Hq // w.Hkv
    pairs = 0
    for s in range(w.n_seqs):
        n = int(w.cu_seqlens[s + 1] - w.cu_seqlens[s])
        i = np.arange(n)
        win = int(np.minimum(i + 1, w.window).sum())
        for h in range(w.Hkv):
            c = int(ret_count[s, h])
            p = ret_pos[s, h, :c].astype(np.int64)
            pairs += G * (win + int(np.maximum(n - w.window - p, 0).sum()))
    return pairs


TRAFFIC_SOURCE = ("profiles/traffic_per_launch.json: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command, scaled by "
                  "a plain copy of known size, committed with the sources; not measured in this run")


def timed_blocks(step, steps, warmup, min_region_ms):
    """`warmup` untimed steps, then blocks of exactly `steps` steps, each bracketed by a synchronize on both sides,
    repeated until the blocks add up to `min_region_ms` (a single block of a 0.15 ms step is shorter than the noise of
    its own two synchronizations).  Returns (mean ms per step over all blocks, ms per step of every block, steps run)."""
    import torch
    for i in range(warmup):
        step(i)
    blocks, total, n = [], 0.0, 0
    while not blocks or total < min_region_ms:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            step(n + i)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) * 1e3
        blocks.append(dt / steps)
        total += dt
        n += steps
    return total / n, blocks, n


def per_step_events(step, steps):
    """Every step between two events of its own on the launch stream: (median, min) ms."""
    import torch
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for i, (a, b) in enumerate(evs):
        a.record()
        step(i)
        b.record()
    torch.cuda.synchronize()
    ts = sorted(a.elapsed_time(b) for a, b in evs)
    return ts[len(ts) // 2], ts[0]


def bench_prefill(workload, steps, warmup, min_region_ms=100.0):
    import torch
    from paper_2510_20787_amd import binding as B
    from paper_2510_20787_amd import workloads as wl

    w = {"prefill": wl.config_prefill_bf16, "long": wl.config_long_prefill_bf16,
         "varlen": wl.config_varlen_prefill_bf16, "paper": wl.config_paper_stack_bf16}[workload]()
    cfg = B.make_cfg(w.Hq, w.Hkv, w.D, w.window, w.budget, w.sink, w.tau, 0.0, w.dtype)
    c = w.cnn
    cnn = B.upload_cnn(c.kernel, c.dilation, c.w, c.bias, c.w_out, c.b_out, w.dtype)
    cu = torch.from_numpy(w.cu_seqlens).cuda()
    T, nB = w.total_tokens, w.n_seqs
    # rotating copies of the inputs keep the 256 MB Infinity Cache from standing in for HBM; the larger workloads
    # exceed it on their own
    in_bytes = (w.q.size + w.k.size + w.v.size) * 2
    n_copies = max(1, min(4, int(np.ceil(300e6 / in_bytes))))
    sets = []
    for _ in range(n_copies):
        sets.append(dict(q=up(w.q, w.dtype), k=up(w.k, w.dtype), v=up(w.v, w.dtype),
                         out=torch.empty((T, w.Hq, w.D), dtype=torch.bfloat16, device="cuda"),
                         cache=B.alloc_cache(cfg, nB)))
    dq, dk, dv = wl.decode_inputs(w.seed, 0, w.dtype, nB, w.Hq, w.Hkv, w.D)
    dq, dk, dv = up(dq, w.dtype), up(dk, w.dtype), up(dv, w.dtype)
    dout = torch.empty((nB, w.Hq, w.D), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(max(B.ltea_workspace_bytes(cfg, cnn, nB, T, w.max_seqlen), 16), dtype=torch.uint8, device="cuda")
    dws = B.decode_workspace(cfg, cnn, nB)
    logits = torch.empty((w.Hkv, T), dtype=torch.float32, device="cuda")

    def step(i):
        s = sets[i % n_copies]
        B.ltea_prefill(cfg, cnn, s["q"], s["k"], s["v"], cu, w.max_seqlen, s["cache"], out=s["out"], workspace=ws)
        B.ltea_decode_step(cfg, cnn, dq, dk, dv, s["cache"], out=dout, workspace=dws)

    ms_per_step, blocks, timed_steps = timed_blocks(step, steps, warmup, min_region_ms)
    step_median, step_min = per_step_events(step, steps)
    tokens_per_step = T + nB
    value = tokens_per_step / (ms_per_step * 1e-3)

    # the same steps with the conv weights re-laid once beforehand (ltea_cnn_prepare) instead of on every call:
    # what a server that loads its weights once sees.  Reported beside the headline, which keeps the per-call re-layout.
    cnn_once = B.prepare_cnn(cfg, B.upload_cnn(c.kernel, c.dilation, c.w, c.bias, c.w_out, c.b_out, w.dtype))

    def step_prepared(i):
        s = sets[i % n_copies]
        B.ltea_prefill(cfg, cnn_once, s["q"], s["k"], s["v"], cu, w.max_seqlen, s["cache"], out=s["out"], workspace=ws)
        B.ltea_decode_step(cfg, cnn_once, dq, dk, dv, s["cache"], out=dout, workspace=dws)

    prepared_ms, _, _ = timed_blocks(step_prepared, steps, warmup, min_region_ms)

    # instrumented repeat: same work, entry points one by one, HIP events on the launch stream
    names = ["score", "retain", "attention", "decode_step"]
    per = {n: [] for n in names}
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(steps)]
    for i in range(steps):
        s = sets[i % n_copies]
        e = evs[i]
        e[0].record()
        B.ltea_score(cfg, cnn, s["k"], s["v"], cu, w.max_seqlen, logits=logits, workspace=ws)
        e[1].record()
        B.ltea_retain(cfg, logits, s["k"], s["v"], cu, w.max_seqlen, cnn.rho, s["cache"])
        e[2].record()
        B.ltea_sparse_attention(cfg, s["q"], s["k"], s["v"], cu, w.max_seqlen, s["cache"], out=s["out"])
        e[3].record()
        B.ltea_decode_step(cfg, cnn, dq, dk, dv, s["cache"], out=dout, workspace=dws)
        e[4].record()
    torch.cuda.synchronize()
    for e in evs:
        for j, n in enumerate(names):
            per[n].append(e[j].elapsed_time(e[j + 1]))
    kern_ms = {n: float(np.mean(per[n])) for n in names}
    kern_min_ms = {n: float(np.min(per[n])) for n in names}

    # algorithmic work of the attention kernel from the actual retained sets (after a clean prefill)
    s = sets[0]
    B.ltea_prefill(cfg, cnn, s["q"], s["k"], s["v"], cu, w.max_seqlen, s["cache"], out=s["out"], workspace=ws)
    torch.cuda.synchronize()
    pairs = attention_pairs(w, s["cache"].ret_pos.cpu().numpy(), s["cache"].ret_count.cpu().numpy())
    flops = 4.0 * w.D * pairs
    achieved = flops / (kern_ms["attention"] * 1e-3) / 1e12
    score_bytes = 2 * T * w.Hkv * w.D * 2 + 4 * T * w.Hkv
    traffic = measured_traffic(w.name, "attention_mfma_kernel")
    res = dict(value=value, ms_per_step=ms_per_step, tokens_per_step=tokens_per_step, kern_ms=kern_ms,
               kern_min_ms=kern_min_ms, prepared_ms=prepared_ms, input_copies=n_copies,
               timing=dict(timed_steps=timed_steps, blocks=len(blocks), block_ms_per_step_min=min(blocks),
                           block_ms_per_step_median=float(np.median(blocks)), step_event_ms_median=step_median,
                           step_event_ms_min=step_min,
                           note=f"`steps` steps per block between two synchronizations, blocks repeated until {min_region_ms:.0f} ms "
                                "are timed; ms_per_step and value are the mean over all of them; the step_event figures "
                                "bracket every step of one more block with HIP events of its own"),
               roofline=dict(bound="mfma", kernel="prefill attention (window + retained)", achieved=achieved,
                             peak=PEAK_BF16_TFLOPS, unit="TFLOP/s", frac=achieved / PEAK_BF16_TFLOPS,
                             traffic=traffic, traffic_source=TRAFFIC_SOURCE if traffic is not None else None,
                             algorithmic_flops=flops, avg_ms=kern_ms["attention"], min_ms=kern_min_ms["attention"]),
               scoring=dict(bound="hbm", achieved=score_bytes / (kern_ms["score"] * 1e-3) / 1e9, peak=PEAK_HBM_GBS,
                            unit="GB/s", frac=score_bytes / (kern_ms["score"] * 1e-3) / 1e9 / PEAK_HBM_GBS,
                            avg_ms=kern_ms["score"], min_ms=kern_min_ms["score"], algorithmic_bytes=score_bytes,
                            note="ltea_score as the step calls it: weight re-layout + scoring kernel(s)"),
               workload=w)
    del sets
    torch.cuda.empty_cache()
    return res


def bench_decode(args):
    import torch
    from paper_2510_20787_amd import binding as B
    from paper_2510_20787_amd import workloads as wl

    t0 = time.time()
    st = wl.config_decode_bf16()
    log(f"[bench] decode state generated in {time.time() - t0:.1f}s")
    cfg = B.make_cfg(st.Hq, st.Hkv, st.D, st.window, st.budget, st.sink, st.tau, 0.0, st.dtype)
    c = st.cnn
    cnn = B.upload_cnn(c.kernel, c.dilation, c.w, c.bias, c.w_out, c.b_out, st.dtype)
    dt = st.dtype
    cache = B.wrap_cache(up(st.k_win, dt), up(st.v_win, dt),
                         torch.zeros((st.B, st.Hkv, st.window), dtype=torch.float32, device="cuda"),
                         up(st.k_ret, dt), up(st.v_ret, dt), torch.from_numpy(st.ret_score).cuda(),
                         torch.from_numpy(st.ret_pos).cuda(), torch.from_numpy(st.ret_count).cuda(),
                         torch.from_numpy(st.n_seen).cuda(),
                         torch.from_numpy(np.maximum(st.n_seen - c.rho, 0).astype(np.int32)).cuda())
    # ring logits = scoring kernel on the ring contents (n_seen is a multiple of the window: slot order = position order)
    cu = torch.tensor([0, st.window], dtype=torch.int32, device="cuda")
    for b in range(st.B):
        kb = cache.k_win[b].permute(1, 0, 2)   # [window, Hkv, D] view
        vb = cache.v_win[b].permute(1, 0, 2)
        cache.win_score[b].copy_(B.ltea_score(cfg, cnn, kb, vb, cu, st.window))
    n_steps = 256
    steps_in = []
    for i in range(n_steps):
        q, k, v = wl.decode_inputs(st.seed, i, dt, st.B, st.Hq, st.Hkv, st.D)
        steps_in.append((up(q, dt), up(k, dt), up(v, dt)))
    out = torch.empty((st.B, st.Hq, st.D), dtype=torch.bfloat16, device="cuda")
    ws = B.decode_workspace(cfg, cnn, st.B)
    for i in range(8):   # warm-up steps also advance the state; the ring just keeps rotating
        q, k, v = steps_in[i]
        B.ltea_decode_step(cfg, cnn, q, k, v, cache, out=out, workspace=ws)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    # the 256-step sequence timed as a whole, three times over (the state keeps advancing: same work every time)
    runs, walls = [], []
    for _ in range(3):
        t0 = time.perf_counter()
        e0.record()
        for i in range(n_steps):
            q, k, v = steps_in[i]
            B.ltea_decode_step(cfg, cnn, q, k, v, cache, out=out, workspace=ws)
        e1.record()
        torch.cuda.synchronize()
        walls.append((time.perf_counter() - t0) * 1e6 / n_steps)
        runs.append(e0.elapsed_time(e1) * 1e3 / n_steps)
    wall_us = float(np.median(walls))
    us_per_step = float(np.median(runs))
    us_per_step_min = float(np.min(runs))
    cnt = cache.ret_count.cpu().numpy().astype(np.int64)
    bytes_per_step = int(((st.window + cnt) * 2 * st.D * 2).sum())
    gbs = bytes_per_step / (us_per_step * 1e-6) / 1e9
    # the same eager steps recorded once into a HIP graph (16 steps per graph) and replayed: what a caller that
    # captures its decode loop sees (the entry points only enqueue kernels, so they can be captured as they are)
    def graph_us(enqueue_step):
        per_graph = 16
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            enqueue_step(0)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for i in range(per_graph):
                enqueue_step(i)
        g.replay()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(n_steps // per_graph):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / n_steps

    def eager_step(i):
        q, k, v = steps_in[i]
        B.ltea_decode_step(cfg, cnn, q, k, v, cache, out=out, workspace=ws)

    graph_eager_us = graph_us(eager_step)
    # lazy scoring: the same steps without per-step scoring + one batched scoring per ltea_lazy_period() steps
    period = B.ltea_lazy_period(cfg, cnn)
    rws = torch.empty(B.ltea_rescore_workspace_bytes(cfg, cnn, st.B), dtype=torch.uint8, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    lws = B.decode_workspace(cfg, None, st.B)
    for i in range(8):
        q, k, v = steps_in[i]
        B.ltea_decode_step_lazy(cfg, q, k, v, cache, out=out, status=status, workspace=lws)
    torch.cuda.synchronize()
    e0.record()
    for i in range(n_steps):
        q, k, v = steps_in[i]
        B.ltea_decode_step_lazy(cfg, q, k, v, cache, out=out, status=status, workspace=lws)
    e1.record()
    torch.cuda.synchronize()
    lazy_us = e0.elapsed_time(e1) * 1e3 / n_steps
    oldest = torch.clamp(cache.n_seen - st.window + c.rho, min=0)   # a batched scoring at the last allowed moment
    B.ltea_rescore(cfg, cnn, cache, status=status, workspace=rws)
    reps = 5
    rescore_ms = 0.0
    for _ in range(reps):
        cache.n_scored.copy_(oldest)
        torch.cuda.synchronize()
        e0.record()
        B.ltea_rescore(cfg, cnn, cache, status=status, workspace=rws)
        e1.record()
        torch.cuda.synchronize()
        rescore_ms += e0.elapsed_time(e1) / reps
    assert int(status.item()) == 0, "lazy decode reported late scoring"
    def lazy_step(i):
        q, k, v = steps_in[i]
        B.ltea_decode_step_lazy(cfg, q, k, v, cache, out=out, status=status, workspace=lws)

    graph_lazy_us = graph_us(lazy_step)
    B.ltea_rescore(cfg, cnn, cache, status=status, workspace=rws)
    torch.cuda.synchronize()
    assert int(status.item()) == 0, "lazy decode reported late scoring"
    lazy = dict(us_per_step=lazy_us, graph_us_per_step=graph_lazy_us, rescore_us=rescore_ms * 1e3, period=period,
                amortised_us_per_step=lazy_us + rescore_ms * 1e3 / period,
                frac_of_hbm_peak=bytes_per_step / ((lazy_us + rescore_ms * 1e3 / period) * 1e-6) / 1e9 / PEAK_HBM_GBS)
    return dict(workload="decode_bf16: B=64 H=16 D=128 window=1024 retained=512 n_seen=8192, 256 steps, cnn k5 c32",
                us_per_step=us_per_step, us_per_step_min=us_per_step_min, us_per_token=us_per_step / st.B,
                wall_us_per_step=wall_us,
                timing_note="256 consecutive steps timed as a whole with HIP events, three times: median (us_per_step) and min",
                graph_us_per_step=graph_eager_us,
                graph_frac_of_hbm_peak=bytes_per_step / (graph_eager_us * 1e-6) / 1e9 / PEAK_HBM_GBS,
                algorithmic_bytes_per_step=bytes_per_step, lazy=lazy,
                roofline=dict(bound="hbm", kernel="decode step (all launches)", achieved=gbs, peak=PEAK_HBM_GBS,
                              unit="GB/s", frac=gbs / PEAK_HBM_GBS,
                              traffic=measured_traffic("decode_bf16", "decode_main_kernel")))


def bench_train(args):
    """Training-side forward + backward on the paper's module shape (no cap): ltea_train_forward, then
    ltea_train_backward for a random d(out).  Pairs = (query, visible key) pairs counted from the logits."""
    import torch
    from paper_2510_20787_amd import binding as B
    from paper_2510_20787_amd import workloads as wl

    w = wl.config_paper_stack_bf16()
    cfg = B.make_cfg(w.Hq, w.Hkv, w.D, w.window, w.budget, w.sink, w.tau, 0.0, w.dtype)
    c = w.cnn
    cnn = B.upload_cnn(c.kernel, c.dilation, c.w, c.bias, c.w_out, c.b_out, w.dtype)
    cu = torch.from_numpy(w.cu_seqlens).cuda()
    q, k, v = up(w.q, w.dtype), up(w.k, w.dtype), up(w.v, w.dtype)
    # The training regulariser aims every head at <= budget candidates per N tokens (512 of 4096): shift each head's
    # output bias so that exactly that share of its logits is positive (the last layer is linear, so this moves the
    # logits by a constant per head).
    z0 = B.ltea_score(cfg, cnn, k, v, cu, w.max_seqlen).cpu().numpy()
    share = w.budget / w.max_seqlen
    shift = np.quantile(z0, 1.0 - share, axis=1).astype(np.float32)
    cnn = B.upload_cnn(c.kernel, c.dilation, c.w, c.bias, c.w_out, c.b_out - shift, w.dtype)
    rng = np.random.default_rng(w.seed + 99)
    dout = up(wl.to_storage(rng.standard_normal(w.q.shape, dtype=np.float32), w.dtype), w.dtype)
    lam = torch.full((w.Hkv,), 1e-3, dtype=torch.float32, device="cuda")
    ws = torch.empty(B.ltea_train_workspace_bytes(cfg, cnn, w.n_seqs, w.total_tokens, w.max_seqlen), dtype=torch.uint8,
                     device="cuda")
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    fwd_ms = bwd_ms = 0.0
    reps = 3
    for it in range(reps + 1):
        ev[0].record()
        out, lse, logits, _ = B.ltea_train_forward(cfg, cnn, q, k, v, cu, w.max_seqlen, workspace=ws)
        ev[1].record()
        grads = B.ltea_train_backward(cfg, q, k, v, cu, w.max_seqlen, out, dout, lse, logits, lam, ws)
        ev[2].record()
        torch.cuda.synchronize()
        if it > 0:
            fwd_ms += ev[0].elapsed_time(ev[1]) / reps
            bwd_ms += ev[1].elapsed_time(ev[2]) / reps
    # the scoring CNN's own backward on the d logits just produced (fp32-accurate products on the fp32 matrix
    # instruction or, with the fp32 operand split into three bf16 terms, on the bf16 one; not part of tokens_per_s)
    cws = torch.empty(int(B.lib().ltea_cnn_backward_workspace_bytes(B.C.byref(cfg), B.C.byref(cnn.struct), w.total_tokens)),
                      dtype=torch.uint8, device="cuda")
    B.ltea_cnn_backward(cfg, cnn, k, v, cu, w.max_seqlen, grads[3], workspace=cws)
    ev[0].record()
    B.ltea_cnn_backward(cfg, cnn, k, v, cu, w.max_seqlen, grads[3], workspace=cws)
    ev[1].record()
    torch.cuda.synchronize()
    cnn_bwd_ms = ev[0].elapsed_time(ev[1])
    z = logits.cpu().numpy()
    G = w.Hq // w.Hkv
    pairs = 0
    for s_ in range(w.n_seqs):
        lo, hi = int(w.cu_seqlens[s_]), int(w.cu_seqlens[s_ + 1])
        n = hi - lo
        i = np.arange(n)
        n_win = np.minimum(i + 1, w.window)
        for h in range(w.Hkv):
            keep = z[h, lo:hi] > w.tau
            keep[:w.sink] = True
            left = np.concatenate([[0], np.cumsum(keep)])          # kept positions below an index
            n_far = left[np.maximum(i - w.window + 1, 0)]
            pairs += int((n_win + n_far).sum()) * G
    kept_frac = float(grads[4].sum().item()) / (w.total_tokens * w.Hkv)
    flops_bwd = 10.0 * w.D * pairs                                # S, dP, dV, dK, dQ: 2 D flop each per pair
    tf = flops_bwd / (bwd_ms * 1e-3) / 1e12
    return dict(workload="paper_stack_bf16 without the cap (training): B=4 x n=4096, Hq=32 on Hkv=8, D=64, window=768, "
                         f"output biases shifted so that every head keeps {share:.3f} of its tokens (measured {kept_frac:.3f})", forward_ms=fwd_ms, backward_ms=bwd_ms,
                cnn_backward_ms=cnn_bwd_ms, tokens_per_s=w.total_tokens / ((fwd_ms + bwd_ms) * 1e-3), pairs=pairs,
                roofline=dict(bound="mfma", kernel="train_dq_mfma_kernel + train_dkv_mfma_kernel (both passes)",
                              achieved=tf, peak=PEAK_BF16_TFLOPS, unit="TFLOP/s", frac=tf / PEAK_BF16_TFLOPS, traffic=None,
                              note="algorithmic flops = 10 D per (query, key) pair (S, dP, dV, dK, dQ); the two kernels "
                                   "each recompute S and dP, so they issue 14 D"))


def bench_chunked(args):
    """The prefill workload fed in `--chunks` equal pieces per sequence: ltea_prefill for the first piece,
    ltea_prefill_append for the others (same final state and last-piece rows as the one-shot call)."""
    import torch
    from paper_2510_20787_amd import binding as B
    from paper_2510_20787_amd import workloads as wl

    w = wl.config_prefill_bf16()
    K = args.chunks
    n = int(w.cu_seqlens[1] - w.cu_seqlens[0])
    assert n % K == 0, "--chunks must divide the sequence length"
    m = n // K
    cfg = B.make_cfg(w.Hq, w.Hkv, w.D, w.window, w.budget, w.sink, w.tau, 0.0, w.dtype)
    c = w.cnn
    cnn = B.upload_cnn(c.kernel, c.dilation, c.w, c.bias, c.w_out, c.b_out, w.dtype)
    q, k, v = up(w.q, w.dtype), up(w.k, w.dtype), up(w.v, w.dtype)
    pieces = []
    for j in range(K):
        idx = torch.cat([torch.arange(int(w.cu_seqlens[s]) + j * m, int(w.cu_seqlens[s]) + (j + 1) * m) for s in range(w.n_seqs)]).cuda()
        pieces.append((q[idx].contiguous(), k[idx].contiguous(), v[idx].contiguous()))
    cu = (torch.arange(0, w.n_seqs + 1, dtype=torch.int32) * m).cuda()
    cache = B.alloc_cache(cfg, w.n_seqs)
    out = torch.empty((w.n_seqs * m, w.Hq, w.D), dtype=torch.bfloat16, device="cuda")
    ws1 = torch.empty(max(B.ltea_workspace_bytes(cfg, cnn, w.n_seqs, w.n_seqs * m, m), 16), dtype=torch.uint8, device="cuda")
    ws2 = torch.empty(max(B.ltea_append_workspace_bytes(cfg, cnn, w.n_seqs, w.n_seqs * m, m), 16), dtype=torch.uint8, device="cuda")

    def step():
        B.ltea_prefill(cfg, cnn, *pieces[0], cu, m, cache, out=out, workspace=ws1)
        for j in range(1, K):
            B.ltea_prefill_append(cfg, cnn, *pieces[j], cu, m, cache, out=out, workspace=ws2)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    return {"workload": f"prefill_bf16 in {K} pieces of {m} tokens per sequence (1 ltea_prefill + {K - 1} ltea_prefill_append)",
            "ms_per_pass": ms, "tokens_per_s": w.total_tokens / (ms * 1e-3)}


def bench_seqlen_sweep(args):
    """Attention kernel alone against the sequence length, on the shape of the paper's kernel comparison (Section 4.3,
    Figure 4a): the 1.4B model's heads (Hq=32 on Hkv=8, D=64), batch 32, window 1024 and an artificial half-full
    out-of-window cache (256 of budget 512 entries per head, positions drawn uniformly, the same for every length so
    that only the sequence length changes).  Three index sets through the same kernel: window + kept entries, window
    only (budget 0), full causal attention (window = n).  Inputs are drawn on the device (timing only)."""
    import torch
    from paper_2510_20787_amd import binding as B
    Hq, Hkv, D, window, budget, kept, batch = 32, 8, 64, 1024, 512, 256, 32
    gen = torch.Generator(device="cuda").manual_seed(4)
    rows = []
    for n in (2048, 4096, 8192, 16384, 32768):
        T = batch * n
        q = torch.randn((T, Hq, D), generator=gen, device="cuda", dtype=torch.bfloat16)
        k = torch.randn((T, Hkv, D), generator=gen, device="cuda", dtype=torch.bfloat16)
        v = torch.randn((T, Hkv, D), generator=gen, device="cuda", dtype=torch.bfloat16)
        out = torch.empty_like(q)
        cu = torch.arange(batch + 1, dtype=torch.int32, device="cuda") * n
        row = {"n": n, "tokens": T}
        for name, w_, b_, c_ in (("lte", window, budget, kept), ("swa", window, 0, 0), ("full", n, 0, 0)):
            cfg = B.make_cfg(Hq, Hkv, D, w_, b_, 0, 0.0, 0.0, "bf16")
            cache = B.alloc_cache(cfg, batch)
            pairs = Hq * batch * (w_ * (w_ + 1) // 2 + (n - w_) * w_)
            if c_:
                pos = torch.rand((batch, Hkv, n - w_), generator=gen, device="cuda").argsort(dim=-1)[..., :c_]
                pos = pos.sort(dim=-1).values
                cache.ret_pos[..., :c_] = pos.to(torch.int32)
                cache.ret_count.fill_(c_)
                tok = (pos + (torch.arange(batch, device="cuda") * n)[:, None, None]).reshape(-1)
                hd = torch.arange(Hkv, device="cuda")[None, :, None].expand(batch, Hkv, c_).reshape(-1)
                cache.k_ret[:, :, :c_] = k[tok, hd].reshape(batch, Hkv, c_, D)
                cache.v_ret[:, :, :c_] = v[tok, hd].reshape(batch, Hkv, c_, D)
                pairs += (Hq // Hkv) * int((n - w_ - pos.to(torch.int64)).clamp_(min=0).sum().item())
            reps = 1 if name == "full" and n >= 16384 else 3
            B.ltea_sparse_attention(cfg, q, k, v, cu, n, cache, out=out)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                B.ltea_sparse_attention(cfg, q, k, v, cu, n, cache, out=out)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / reps
            row[name] = {"ms": ms, "tflops": 4.0 * D * pairs / (ms * 1e-3) / 1e12}
            log(f"[bench] seqlen sweep n={n} {name}: {ms:.3f} ms, {row[name]['tflops']:.0f} TFLOP/s")
            del cache
        rows.append(row)
        del q, k, v, out
    res = {"workload": f"attention kernel alone, B={batch}, Hq={Hq} on Hkv={Hkv}, D={D}, window={window}, {kept} kept "
                       f"entries per head (artificial, budget {budget}); lte = window + kept, swa = window only, "
                       "full = causal", "rows": rows}
    res["layer"] = bench_paper_layer(args)
    return res


def bench_paper_layer(args):
    """The whole token mixer of the paper's LTE layers (Section 4.3, Figure 4b/4c): 3 x (k=3, dilation 2) CNN, Hq=32 on
    Hkv=8, D=64, window 768, budget 512, sink 4, batch 32.  Prefill (scoring + retention + cache fill + attention)
    against the sequence length, then decode steps after a 4096-token prompt: eager (one logit finalised per step)
    and lazy (one batched scoring per ltea_lazy_period() steps, amortised).  With the seeded random weights a head keeps
    about 260 entries on N(0,1) inputs (reported), close to the mean the paper observed on its trained models.
    Q, K, V are drawn on the device (timing only)."""
    import torch
    from paper_2510_20787_amd import binding as B
    from paper_2510_20787_amd import workloads as wl
    batch = 32
    w = wl.config_paper_stack_bf16(n=64, B=1)          # the CNN weights and the shape
    cfg = B.make_cfg(w.Hq, w.Hkv, w.D, w.window, w.budget, w.sink, w.tau, 0.0, "bf16")
    c = w.cnn
    cnn = B.prepare_cnn(cfg, B.upload_cnn(c.kernel, c.dilation, c.w, c.bias, c.w_out, c.b_out, "bf16"))
    gen = torch.Generator(device="cuda").manual_seed(6)
    draw = lambda *shape: torch.randn(shape, generator=gen, device="cuda", dtype=torch.bfloat16)
    prefill = []
    cache = B.alloc_cache(cfg, batch)
    for n in (2048, 4096, 8192, 16384):
        T = batch * n
        q, k, v = draw(T, w.Hq, w.D), draw(T, w.Hkv, w.D), draw(T, w.Hkv, w.D)
        out = torch.empty_like(q)
        cu = torch.arange(batch + 1, dtype=torch.int32, device="cuda") * n
        ws = torch.empty(B.ltea_workspace_bytes(cfg, cnn, batch, T, n), dtype=torch.uint8, device="cuda")
        B.ltea_prefill(cfg, cnn, q, k, v, cu, n, cache, out=out, workspace=ws)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(3):
            B.ltea_prefill(cfg, cnn, q, k, v, cu, n, cache, out=out, workspace=ws)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 3
        prefill.append({"n": n, "ms": ms, "tokens_per_s": T / (ms * 1e-3)})
        log(f"[bench] paper layer prefill B={batch} n={n}: {ms:.3f} ms, {T / (ms * 1e-3) / 1e6:.1f} M tokens/s")
        if n != 4096:
            continue
        # decode after this 4096-token prompt
        kept = float(cache.ret_count.float().mean().item())
        snap = {name: getattr(cache, name).clone() for name in ("k_win", "v_win", "win_score", "k_ret", "v_ret",
                                                                 "ret_score", "ret_pos", "ret_count", "n_seen", "n_scored")}
        dq, dk, dv = draw(batch, w.Hq, w.D), draw(batch, w.Hkv, w.D), draw(batch, w.Hkv, w.D)
        dout = torch.empty_like(dq)
        dws = B.decode_workspace(cfg, cnn, batch)
        steps = 200
        def timed(fn):
            for _ in range(10):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / steps * 1e6
        eager_us = timed(lambda: B.ltea_decode_step(cfg, cnn, dq, dk, dv, cache, out=dout, workspace=dws))
        period = B.ltea_lazy_period(cfg, cnn)
        status = torch.zeros(1, dtype=torch.int32, device="cuda")
        rws = torch.empty(B.ltea_rescore_workspace_bytes(cfg, cnn, batch), dtype=torch.uint8, device="cuda")
        lws = B.decode_workspace(cfg, None, batch)
        assert 210 < period
        lazy_us = timed(lambda: B.ltea_decode_step_lazy(cfg, dq, dk, dv, cache, out=dout, status=status, workspace=lws))
        # one batched scoring of a full period's worth of positions
        B.ltea_rescore(cfg, cnn, cache, status=status, workspace=rws)
        oldest = torch.clamp(cache.n_seen - w.window + c.rho, min=0)
        rescore_us = 0.0
        for _ in range(5):
            cache.n_scored.copy_(oldest)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            B.ltea_rescore(cfg, cnn, cache, status=status, workspace=rws)
            torch.cuda.synchronize()
            rescore_us += (time.perf_counter() - t0) / 5 * 1e6
        streamed = int(batch * w.Hkv * (w.window + kept) * w.D * 2 * 2)
        lazy_total = lazy_us + rescore_us / period
        decode = {"prompt": n, "kept_per_head": kept, "eager_us_per_step": eager_us, "lazy_us_per_step": lazy_us,
                  "rescore_us": rescore_us, "period": period, "lazy_amortised_us_per_step": lazy_total,
                  "bytes_streamed_per_step": streamed, "lazy_gbs": streamed / (lazy_total * 1e-6) / 1e9,
                  "status": int(status.item())}
        log(f"[bench] paper layer decode B={batch} after {n}: eager {eager_us:.1f} us/step, lazy {lazy_us:.1f} + "
            f"{rescore_us:.0f}/{period} = {lazy_total:.1f} us/step")
        for name, t in snap.items():
            getattr(cache, name).copy_(t)
        del q, k, v, out, ws
    return {"workload": f"paper LTE layer: B={batch}, Hq={w.Hq} on Hkv={w.Hkv}, D={w.D}, window={w.window}, "
                        f"budget={w.budget}, sink={w.sink}, CNN 3 x (k=3, dilation 2), weights re-laid once",
            "prefill": prefill, "decode": decode}


def cpu_baseline(w):
    """The oracle as it stands on a bounded sample of the same workload: whole sequences (all heads: scoring +
    retention + attention), as many as fit in about 12 s of wall time."""
    import psutil
    from oracle import ltea_oracle as orc
    cfg = orc.OracleCfg(w.Hq, w.Hkv, w.D, w.window, w.budget, w.sink, w.tau)
    c = w.cnn
    cnn = orc.cnn_from_arrays(c.kernel, c.dilation, c.w, c.bias, c.w_out, c.b_out)
    proc = psutil.Process()
    c0, t0 = proc.cpu_times(), time.perf_counter()
    tokens, n_done = 0, 0
    for s in range(w.n_seqs):
        lo, hi = int(w.cu_seqlens[s]), int(w.cu_seqlens[s + 1])
        orc.prefill(w.q[lo:hi], w.k[lo:hi], w.v[lo:hi], cfg, cnn, [0, hi - lo])
        tokens += hi - lo
        n_done += 1
        if time.perf_counter() - t0 > 12.0:
            break
    dt = time.perf_counter() - t0
    c1 = proc.cpu_times()
    cpu = (c1.user - c0.user) + (c1.system - c0.system)
    return dict(value=tokens / dt, unit="tokens/s", cores=max(1, int(round(cpu / dt))), kind="oracle",
                sample=f"{n_done} of {w.n_seqs} sequences ({tokens} tokens, all {w.Hq} heads): scoring + retention + "
                       f"attention, {dt:.1f}s wall; host has {os.cpu_count()} logical cores")


def measure_ceilings():
    """What the chip sustains on the two roofline resources: a register-resident bf16 MFMA loop and a streaming
    read of 2 GiB with non-temporal loads (both library entry points, timed here with events on the current stream)."""
    import torch
    from paper_2510_20787_amd import binding as B
    sink = B.ltea_diag_sink()
    src = torch.empty(2 << 30, dtype=torch.uint8, device="cuda").fill_(3)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    out = {}
    for name, fn in (("mfma", lambda: B.ltea_diag_mfma_loop(1000, sink)), ("read", lambda: B.ltea_diag_stream_read(src, sink))):
        fn()
        torch.cuda.synchronize()
        best = None
        for _ in range(3):
            e0, e1 = ev(), ev()
            e0.record()
            work = fn()
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            best = ms if best is None or ms < best else best
        out[name] = work / (best * 1e-3)
    del src
    return {"mfma_bf16_tflops": out["mfma"] / 1e12, "hbm_read_gbs": out["read"] / 1e9,
            "how": "ltea_diag_mfma_loop (4096 workgroups x 4 waves x 8000 MFMAs 32x32x16 bf16) and "
                   "ltea_diag_stream_read (2 GiB, non-temporal 16-byte loads, one contiguous share per workgroup), best of 3"}


def add_measured_fraction(roof, ceilings):
    if roof is None:
        return
    top = ceilings["mfma_bf16_tflops"] if roof["bound"] == "mfma" else ceilings["hbm_read_gbs"]
    roof["measured_ceiling"] = top
    roof["frac_of_measured"] = roof["achieved"] / top


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--train", action="store_true", help="(default) also time the training-side forward + backward")
    ap.add_argument("--no-train", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the long / varlen / paper prefill configurations that the default run reports under `configs`")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three plain 256 MiB device-to-device copies (a kernel of known traffic, used to "
                         "scale rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--chunks", type=int, default=1,
                    help="also time the prefill workload fed in this many pieces per sequence (continued prefill)")
    ap.add_argument("--seqlen-sweep", action="store_true",
                    help="also time the attention kernel alone against the sequence length (batch 32, 1.4B head "
                         "shape, half-full artificial cache) for three index sets: window + kept, window, full causal; "
                         "and the paper's whole LTE layer (CNN scoring, retention, attention; decode after a 4096-token "
                         "prompt) at batch 32")
    ap.add_argument("--workload", choices=["prefill", "long", "varlen", "paper"], default="prefill",
                    help="prefill = the benchmark configuration (default); long / varlen / paper = the other prefill "
                         "configurations, for kernel measurements (no CPU baseline, no decode section)")
    args = ap.parse_args()
    if args.workload != "prefill":
        args.no_decode = args.no_cpu_baseline = args.no_train = True
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (every (sequence, KV head) is independent, so the path "
                 "shards over batch x heads without any exchange; no multi-GPU run is implemented). Run with --gpus 1.")
    import torch
    from paper_2510_20787_amd import binding as B
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    B.lib()
    torch.cuda.set_device(0)
    log(f"[bench] device: {torch.cuda.get_device_name(0)}")
    if args.calibrate_copy:
        src = torch.full((256 << 20,), 1, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    pre = bench_prefill(args.workload, args.steps, args.warmup)
    log(f"[bench] {args.workload} step {pre['ms_per_step']:.3f} ms over {pre['timing']['timed_steps']} steps; kernels (ms): {pre['kern_ms']}")
    w = pre.pop("workload")
    line = {
        "metric": "SWA+LTE prefill tokens/s (scoring + retention + attention + one decode step per sequence)",
        "value": pre["value"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": pre["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": WORKLOAD_TEXT[args.workload],
                   "tokens_per_step": pre["tokens_per_step"], "input_copies_rotated": pre["input_copies"]},
        "timing": pre["timing"],
        "roofline": pre["roofline"],
        "kernel_ms": pre["kern_ms"],
        "kernel_min_ms": pre["kern_min_ms"],
        "kernel_ms_note": "the four entry points called one by one with an event between them; their sum exceeds "
                          "ms_per_step because ltea_prefill enqueues the same kernels without the host gaps between "
                          "separate calls",
        "prepared_cnn": {"ms_per_step": pre["prepared_ms"], "tokens_per_s": pre["tokens_per_step"] / (pre["prepared_ms"] * 1e-3),
                         "note": "same steps with the conv weights re-laid once by ltea_cnn_prepare instead of on every call"},
        "scoring_roofline": pre["scoring"],
    }
    ceilings = measure_ceilings()
    log(f"[bench] measured ceilings: {ceilings['mfma_bf16_tflops']:.0f} TFLOP/s bf16 MFMA, {ceilings['hbm_read_gbs']:.0f} GB/s read")
    line["ceilings"] = ceilings
    add_measured_fraction(line["roofline"], ceilings)
    add_measured_fraction(line["scoring_roofline"], ceilings)
    if args.workload == "prefill" and not args.no_other_configs:
        # the other prefill configurations, fewer steps each: the same step, the same two roofline objects
        line["configs"] = {}
        for name in ("long", "varlen", "paper"):
            o = bench_prefill(name, max(5, args.steps // 5), 3, min_region_ms=50.0)
            ow = o.pop("workload")
            add_measured_fraction(o["roofline"], ceilings)
            add_measured_fraction(o["scoring"], ceilings)
            line["configs"][ow.name] = {
                "workload": WORKLOAD_TEXT[name], "tokens_per_step": o["tokens_per_step"], "value": o["value"],
                "unit": "tokens/s", "ms_per_step": o["ms_per_step"], "timing": o["timing"], "kernel_ms": o["kern_ms"],
                "kernel_min_ms": o["kern_min_ms"], "prepared_cnn_ms_per_step": o["prepared_ms"],
                "roofline": o["roofline"], "scoring_roofline": o["scoring"]}
            log(f"[bench] {ow.name}: step {o['ms_per_step']:.3f} ms; kernels (ms): {o['kern_ms']}; attention "
                f"{o['roofline']['frac']:.3f} of MFMA peak, scoring {o['scoring']['frac']:.3f} of HBM peak")
            del ow, o
    if not args.no_decode:
        dec = bench_decode(args)
        log(f"[bench] decode {dec['us_per_step']:.1f} us/step ({dec['graph_us_per_step']:.1f} replayed from a graph); lazy {dec['lazy']['us_per_step']:.1f} us/step + "
            f"{dec['lazy']['rescore_us']:.0f} us per {dec['lazy']['period']} steps")
        add_measured_fraction(dec.get("roofline"), ceilings)
        line["decode"] = dec
    if not args.no_train:
        line["train"] = bench_train(args)
        log(f"[bench] train forward {line['train']['forward_ms']:.3f} ms, backward {line['train']['backward_ms']:.3f} ms")
    if args.chunks > 1:
        line["chunked_prefill"] = bench_chunked(args)
        log(f"[bench] chunked prefill: {line['chunked_prefill']['ms_per_pass']:.3f} ms per pass")
    if args.seqlen_sweep:
        line["seqlen_sweep"] = bench_seqlen_sweep(args)
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
