"""GPU parity at the full sizes of the named configurations, in the launch configuration bench.py times.

The oracle scores every token of every head (library matmuls make that seconds), so logits and retained
sets are checked on ALL heads; attention outputs are checked on sampled query rows the oracle computes one
by one (first/last rows, window edges, tile edges, random rows); cache contents on sampled slots.
For the decode configuration the eviction rule is replayed by the oracle for ALL 1024 (sequence, head)
pairs (it needs only logits), while outputs are compared on sampled sequences."""
import numpy as np
import pytest
import torch

from oracle import ltea_oracle as orc
from paper_2510_20787_amd import binding as B
from paper_2510_20787_amd import workloads as wl
from tests.gpu_util import (LOGIT_TOL, OUT_TOL, DeviceWorkload, check_sets, check_sets_strict, dev, gpu_retained_sets,
                            to_np)
from tests.helpers import oracle_cfg, oracle_cnn

pytestmark = pytest.mark.gpu


def sample_rows(n, window, rng, k=6):
    fixed = [0, 1, window - 2, window - 1, window, window + 1, 63, 64, 127, 128, 129, n // 2, n - 129, n - 2, n - 1]
    rows = {r for r in fixed if 0 <= r < n}
    rows |= {int(x) for x in rng.integers(0, n, size=k)}
    return sorted(rows)


def run_full_prefill(w, logit_tol=None):
    ocfg, ocnn = oracle_cfg(w), oracle_cnn(w.cnn)
    d = DeviceWorkload(w)
    cache = d.new_cache()
    logits = torch.empty((w.Hkv, w.total_tokens), dtype=torch.float32, device="cuda")
    out = B.ltea_prefill(d.cfg, d.cnn, d.q, d.k, d.v, d.cu, d.max_seqlen, cache, logits=logits)
    torch.cuda.synchronize()
    print(f"[{w.name}] gpu prefill done; scoring oracle on {w.total_tokens} tokens x {w.Hkv} heads", flush=True)
    z64 = orc.score(w.k, w.v, ocnn, w.cu_seqlens)
    zg = to_np(logits)
    diff = np.abs(zg.astype(np.float64) - z64)
    tol = LOGIT_TOL[w.dtype] if logit_tol is None else logit_tol
    assert np.all(diff <= tol * np.maximum(1.0, np.abs(z64))), f"logit error {diff.max()}"
    eps = float(diff.max())
    print(f"[{w.name}] logits ok (max diff {eps:.3e}); checking retained sets on all heads", flush=True)
    n_strict = check_sets_strict(cache, zg, w)          # level 1: every head, no margin
    near = check_sets(cache, z64, w, eps)               # level 2: end to end against the oracle's own logits
    print(f"[{w.name}] strict set check on {n_strict} heads ok; {len(near)} head(s) inside the decision margin of the "
          f"end-to-end check: {near}", flush=True)
    assert len(near) <= max(1, (w.n_seqs * w.Hkv) // 32), f"too many heads inside the decision margin: {near}"
    skip = set(near)
    # outputs on sampled rows
    rng = np.random.default_rng(12345)
    G = w.Hq // w.Hkv
    rho = w.cnn.rho
    worst, scale, n_rows = 0.0, 0.0, 0
    pairs = []
    for s in range(w.n_seqs):
        lo, hi = int(w.cu_seqlens[s]), int(w.cu_seqlens[s + 1])
        n = hi - lo
        rows = sample_rows(n, w.window, rng)
        heads = range(w.Hq) if w.n_seqs * w.Hq <= 64 else sorted({int(x) for x in rng.integers(0, w.Hq, size=4)})
        kept = {}
        for hq in heads:
            h = hq // G
            if (s, h) in skip:
                continue
            if h not in kept:
                kept[h] = orc.retain(z64[h, lo:hi], n, w.window, w.budget, w.sink, w.tau)
            got = out[lo + torch.tensor(rows, device="cuda"), hq].float().cpu().numpy()
            for r, i in enumerate(rows):
                ref = orc.attention_row(w.q[lo:hi], w.k[lo:hi], w.v[lo:hi], ocfg, kept[h], i, hq)
                worst = max(worst, float(np.abs(got[r] - ref).max()))
                scale = max(scale, float(np.abs(ref).max()))
                n_rows += 1
        # cache contents: counters, a few ring slots and retained rows of a few heads
        assert int(cache.n_seen[s]) == n and int(cache.n_scored[s]) == max(0, n - rho)
        for h in sorted({int(x) for x in rng.integers(0, w.Hkv, size=2)}):
            for p in sorted({max(0, n - w.window), n - 1, n - 1 - rho} | {int(x) for x in rng.integers(max(0, n - w.window), n, size=3)}):
                slot = p % w.window
                np.testing.assert_array_equal(to_np(cache.k_win[s, h, slot]), w.k[lo + p, h])
                np.testing.assert_array_equal(to_np(cache.v_win[s, h, slot]), w.v[lo + p, h])
                assert float(cache.win_score[s, h, slot]) == float(zg[h, lo + p])
            cnt, pos = gpu_retained_sets(cache, s, h)
            if cnt:
                for r in {0, cnt // 2, cnt - 1}:
                    np.testing.assert_array_equal(to_np(cache.k_ret[s, h, r]), w.k[lo + pos[r], h])
                    np.testing.assert_array_equal(to_np(cache.v_ret[s, h, r]), w.v[lo + pos[r], h])
                    assert float(cache.ret_score[s, h, r]) == float(zg[h, lo + pos[r]]) or pos[r] < w.sink
    tol = OUT_TOL[w.dtype]
    print(f"[{w.name}] {n_rows} sampled rows: max-abs err {worst:.3e}, largest reference magnitude {scale:.3e}", flush=True)
    assert worst <= tol and worst <= tol * scale
    return cache, z64


def test_full_prefill_bf16():
    run_full_prefill(wl.config_prefill_bf16())


def test_full_long_prefill_bf16():
    run_full_prefill(wl.config_long_prefill_bf16())


def test_full_paper_stack_bf16():
    """The paper's own module shape: 3-layer dilated CNN, sink 4, 32 query heads on 8 KV heads, window 768."""
    run_full_prefill(wl.config_paper_stack_bf16())


def test_full_append_prefill_bf16():
    """prefill_bf16 at full size, fed in two calls (3072 tokens by ltea_prefill, the last 1024 by
    ltea_prefill_append): kept sets on all heads and sampled appended rows against the one-shot oracle."""
    w = wl.config_prefill_bf16()
    ocfg, ocnn = oracle_cfg(w), oracle_cnn(w.cnn)
    d = DeviceWorkload(w)
    cache = d.new_cache()
    n, cut = 4096, 3072
    cu = w.cu_seqlens
    first = np.concatenate([np.arange(int(cu[s]), int(cu[s]) + cut) for s in range(w.n_seqs)])
    rest = np.concatenate([np.arange(int(cu[s]) + cut, int(cu[s + 1])) for s in range(w.n_seqs)])
    f_idx, r_idx = torch.from_numpy(first).cuda(), torch.from_numpy(rest).cuda()
    cu1 = torch.arange(0, w.n_seqs + 1, dtype=torch.int32, device="cuda") * cut
    cu2 = torch.arange(0, w.n_seqs + 1, dtype=torch.int32, device="cuda") * (n - cut)
    B.ltea_prefill(d.cfg, d.cnn, d.q[f_idx].contiguous(), d.k[f_idx].contiguous(), d.v[f_idx].contiguous(), cu1, cut, cache)
    out = B.ltea_prefill_append(d.cfg, d.cnn, d.q[r_idx].contiguous(), d.k[r_idx].contiguous(), d.v[r_idx].contiguous(),
                                cu2, n - cut, cache)
    torch.cuda.synchronize()
    print("[append] gpu done; scoring oracle", flush=True)
    z64 = orc.score(w.k, w.v, ocnn, w.cu_seqlens)
    # level 1 on every head: the device's own logits of the whole history (one scoring call over all 4096 tokens;
    # a token's logit does not depend on how the history was cut into calls)
    n_strict = check_sets_strict(cache, to_np(B.ltea_score(d.cfg, d.cnn, d.k, d.v, d.cu, d.max_seqlen)), w)
    near = check_sets(cache, z64, w, 1e-5)
    print(f"[append] strict set check on {n_strict} heads ok; {len(near)} head(s) inside the decision margin: {near}", flush=True)
    assert len(near) <= 2, near
    skip = set(near)
    rng = np.random.default_rng(99)
    worst, scale = 0.0, 0.0
    for s in range(w.n_seqs):
        lo = int(cu[s])
        assert int(cache.n_seen[s]) == n and int(cache.n_scored[s]) == n - w.cnn.rho
        kept = {}
        for hq in sorted({int(x) for x in rng.integers(0, w.Hq, size=3)}):
            if (s, hq) in skip:
                continue
            kept[hq] = orc.retain(z64[hq, lo:lo + n], n, w.window, w.budget, w.sink, w.tau)
            for i in sorted({cut, cut + 1, cut + 63, cut + 64, cut + 511, cut + 512, n - 1} | {int(x) for x in rng.integers(cut, n, size=4)}):
                ref = orc.attention_row(w.q[lo:lo + n], w.k[lo:lo + n], w.v[lo:lo + n], ocfg, kept[hq], i, hq)
                got = out[s * (n - cut) + (i - cut), hq].float().cpu().numpy()
                worst = max(worst, float(np.abs(got - ref).max()))
                scale = max(scale, float(np.abs(ref).max()))
    print(f"[append] sampled appended rows: max-abs err {worst:.3e}, largest reference magnitude {scale:.3e}", flush=True)
    assert worst <= OUT_TOL["bf16"] and worst <= OUT_TOL["bf16"] * scale


def test_full_varlen_prefill_bf16():
    w = wl.config_varlen_prefill_bf16()
    cache, z64 = run_full_prefill(w)
    # planted near-duplicate keys: the oracle row for the query each was planted for is covered by the sampled
    # check only by chance, so check a handful of (planted key, its query) pairs explicitly on KV head 0
    ocfg = oracle_cfg(w)
    d = DeviceWorkload(w)
    cache2 = d.new_cache()
    out = B.ltea_prefill(d.cfg, d.cnn, d.q, d.k, d.v, d.cu, d.max_seqlen, cache2)
    worst = 0.0
    for s, (js, iq) in enumerate(w.notes["planted"][:4]):
        lo, hi = int(w.cu_seqlens[s]), int(w.cu_seqlens[s + 1])
        kept = orc.retain(z64[0, lo:hi], hi - lo, w.window, w.budget, w.sink, w.tau)
        for i in iq[:5]:
            ref = orc.attention_row(w.q[lo:hi], w.k[lo:hi], w.v[lo:hi], ocfg, kept, int(i - lo), 0)
            worst = max(worst, float(np.abs(out[int(i), 0].float().cpu().numpy() - ref).max()))
    assert worst <= OUT_TOL["bf16"]


def oracle_state_of_sequence(st, b, win_z64, cfg):
    """Oracle state of sequence b of a directly filled cache. win_z64[h][i] = oracle logit of ring position
    n_seen - window + i (ring slot order equals position order when n_seen is a multiple of the window)."""
    n = int(st.n_seen[b])
    assert n % st.window == 0
    rho = st.cnn.rho
    s = orc.empty_state(cfg)
    s.n_seen, s.n_scored = n, n - rho
    for h in range(st.Hkv):
        hs = s.heads[h]
        for i in range(st.window):
            p = n - st.window + i
            hs.win_pos.append(p)
            hs.win_k.append(st.k_win[b, h, i].astype(np.float64))
            hs.win_v.append(st.v_win[b, h, i].astype(np.float64))
            if p < s.n_scored:
                hs.win_z[p] = float(win_z64[h][i])
        for r in range(int(st.ret_count[b, h])):
            hs.ret_pos.append(int(st.ret_pos[b, h, r]))
            hs.ret_key.append(np.float32(st.ret_score[b, h, r]))
            hs.ret_k.append(st.k_ret[b, h, r].astype(np.float64))
            hs.ret_v.append(st.v_ret[b, h, r].astype(np.float64))
    return s


_decode_state_cache = {}


def decode_bf16_with_oracle_logits():
    if "st" not in _decode_state_cache:
        st = wl.config_decode_bf16()
        ocnn = oracle_cnn(st.cnn)
        print("[decode_bf16] scoring 1024 rings with the oracle", flush=True)
        win_z = np.zeros((st.B, st.Hkv, st.window), dtype=np.float64)
        for b in range(st.B):
            kb = np.transpose(st.k_win[b], (1, 0, 2))   # [window, Hkv, D]
            vb = np.transpose(st.v_win[b], (1, 0, 2))
            win_z[b] = orc.score_sequence(kb, vb, ocnn)
        _decode_state_cache["st"] = (st, ocnn, win_z)
    return _decode_state_cache["st"]


@pytest.mark.parametrize("lazy", [False, True])
def test_full_decode_bf16(lazy):
    """decode_bf16 at full size (B=64, H=16, D=128, window 1024, 512 retained): ring logits from the oracle on all
    1024 rings, 48 steps on the GPU; outputs against the oracle on two sampled sequences at every step; the
    eviction rule replayed by the oracle on ALL (sequence, head) pairs.
    lazy: the cache starts with only the oldest rho logits of each ring final (the latest moment a batched scoring
    may come); ltea_rescore must reproduce the oracle's logits of ALL rings, then the steps are lazy ones."""
    st, ocnn, win_z = decode_bf16_with_oracle_logits()
    ocfg = orc.OracleCfg(st.Hq, st.Hkv, st.D, st.window, st.budget, st.sink, st.tau)
    rho = st.cnn.rho
    dt = st.dtype
    cfg = B.make_cfg(st.Hq, st.Hkv, st.D, st.window, st.budget, st.sink, st.tau, 0.0, dt)
    c = st.cnn
    cnn = B.upload_cnn(c.kernel, c.dilation, c.w, c.bias, c.w_out, c.b_out, dt)
    z0 = win_z.astype(np.float32)
    scored0 = (st.n_seen - rho).astype(np.int32)
    if lazy:
        z0 = z0.copy()
        z0[:, :, rho:] = np.nan                       # ring slot i holds position n - window + i (n % window == 0)
        scored0 = (st.n_seen - st.window + rho).astype(np.int32)
    cache = B.wrap_cache(dev(st.k_win, dt), dev(st.v_win, dt), torch.from_numpy(z0).cuda(),
                         dev(st.k_ret, dt), dev(st.v_ret, dt), torch.from_numpy(st.ret_score).cuda(),
                         torch.from_numpy(st.ret_pos).cuda(), torch.from_numpy(st.ret_count).cuda(),
                         torch.from_numpy(st.n_seen).cuda(), torch.from_numpy(scored0).cuda())
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    if lazy:
        assert B.ltea_lazy_period(cfg, cnn) == st.window - 2 * rho
        B.ltea_rescore(cfg, cnn, cache, status=status)
        zg = cache.win_score.cpu().numpy().astype(np.float64)
        ref = win_z[:, :, :st.window - rho]
        assert np.all(np.abs(zg[:, :, :st.window - rho] - ref) <= LOGIT_TOL["bf16"] * np.maximum(1.0, np.abs(ref)))
        assert np.all(np.isnan(zg[:, :, st.window - rho:]))        # provisional positions are not written
        assert np.all(cache.n_scored.cpu().numpy() == st.n_seen - rho) and int(status.item()) == 0
    sampled = [0, 37]
    states = {b: oracle_state_of_sequence(st, b, win_z[b], ocfg) for b in sampled}
    # position-only oracle records for every (sequence, head): the eviction rule needs logits and keys only
    light = [[orc.HeadState(ret_pos=[int(x) for x in st.ret_pos[b, h, :st.ret_count[b, h]]],
                            ret_key=[np.float32(x) for x in st.ret_score[b, h, :st.ret_count[b, h]]],
                            ret_k=[None] * int(st.ret_count[b, h]), ret_v=[None] * int(st.ret_count[b, h]))
              for h in range(st.Hkv)] for b in range(st.B)]
    n_steps = 48
    n0 = int(st.n_seen[0])
    worst, scale = 0.0, 0.0
    for step in range(n_steps):
        q, k, v = wl.decode_inputs(st.seed, step, dt, st.B, st.Hq, st.Hkv, st.D)
        if lazy:
            out = B.ltea_decode_step_lazy(cfg, dev(q, dt), dev(k, dt), dev(v, dt), cache, status=status)
        else:
            out = B.ltea_decode_step(cfg, cnn, dev(q, dt), dev(k, dt), dev(v, dt), cache)
        og = out[sampled].float().cpu().numpy()
        for i, b in enumerate(sampled):
            ref = orc.decode_step(states[b], q[b], k[b], v[b], ocfg, ocnn)
            worst = max(worst, float(np.abs(og[i] - ref).max()))
            scale = max(scale, float(np.abs(ref).max()))
        # the token leaving every ring at this step is initial ring position i = step (its logit is final: i < window - rho)
        e = n0 - st.window + step
        for b in range(st.B):
            for h in range(st.Hkv):
                orc.evict_into_retained(light[b][h], e, win_z[b, h, step], None, None, ocfg)
        if step % 16 == 15:
            print(f"[decode_bf16] step {step + 1}/{n_steps}: max-abs err so far {worst:.3e}", flush=True)
    assert worst <= OUT_TOL["bf16"] and worst <= OUT_TOL["bf16"] * scale
    torch.cuda.synchronize()
    assert np.all(cache.n_seen.cpu().numpy() == n0 + n_steps)
    if lazy:
        assert np.all(cache.n_scored.cpu().numpy() == n0 - rho)
        B.ltea_rescore(cfg, cnn, cache, status=status)
        assert np.all(cache.n_scored.cpu().numpy() == n0 + n_steps - rho) and int(status.item()) == 0
    pos = cache.ret_pos.cpu().numpy()
    cnt = cache.ret_count.cpu().numpy()
    for b in range(st.B):
        for h in range(st.Hkv):
            np.testing.assert_array_equal(np.sort(pos[b, h, :cnt[b, h]]), np.sort(light[b][h].ret_pos),
                                          err_msg=f"retained set of sequence {b} head {h}")
    for b in sampled:
        for h in range(st.Hkv):
            np.testing.assert_array_equal(np.sort(pos[b, h, :cnt[b, h]]), orc.retained_positions(states[b])[h])
            for p, zp in states[b].heads[h].win_z.items():
                if p >= n0 - rho:      # logits finalised by the decode steps themselves
                    zg = float(cache.win_score[b, h, p % st.window])
                    assert abs(zg - zp) <= LOGIT_TOL["bf16"] * max(1.0, abs(zp))


def test_full_train_paper_stack_bf16():
    """Training forward + backward at the paper's module shape (B=4 x n=4096, 32 query heads on 8 KV heads, D=64,
    window 768, no cap): one (sequence, KV head) group per run through the fp64 oracle (dense n x n), all rows;
    retention counts of every (sequence, head) against the oracle's logits."""
    w = wl.config_paper_stack_bf16()
    d = DeviceWorkload(w)
    rng = np.random.default_rng(w.seed + 99)
    dout = wl.to_storage(rng.standard_normal(w.q.shape, dtype=np.float32), "bf16")
    lam = np.full(w.Hkv, 1e-3, dtype=np.float32)
    out, lse, logits, ws = B.ltea_train_forward(d.cfg, d.cnn, d.q, d.k, d.v, d.cu, d.max_seqlen)
    dq, dk, dv, dz, counts = B.ltea_train_backward(d.cfg, d.q, d.k, d.v, d.cu, d.max_seqlen, out, dev(dout, "bf16"), lse,
                                                   logits, torch.from_numpy(lam).cuda(), ws)
    torch.cuda.synchronize()
    cnn = oracle_cnn(w.cnn)
    z64 = orc.score(w.k, w.v, cnn, w.cu_seqlens)
    zg = to_np(logits)
    eps = float(np.max(np.abs(zg - z64)))
    assert eps <= LOGIT_TOL["bf16"] * max(1.0, float(np.max(np.abs(z64))))
    cnt_g = counts.cpu().numpy()
    G = w.Hq // w.Hkv
    n_checked = 0
    for s, h in ((0, 2), (3, 4)):                       # heads with a mixed kept / dropped population
        lo, hi = int(w.cu_seqlens[s]), int(w.cu_seqlens[s + 1])
        zh = z64[h:h + 1, lo:hi]
        if np.min(np.abs(zh)) <= 2 * eps:
            continue                                    # a logit inside the scoring error of the threshold
        n_checked += 1
        print(f"[train paper_stack] oracle backward for sequence {s}, KV head {h} (kept {float((zh > 0).mean()):.2f})", flush=True)
        sub = orc.OracleCfg(G, 1, w.D, w.window, 1, w.sink, w.tau)
        qs = w.q[lo:hi, h * G:(h + 1) * G]; ks = w.k[lo:hi, h:h + 1]; vs = w.v[lo:hi, h:h + 1]
        o_ref, lse_ref, _ = orc.train_forward_sequence(qs, ks, vs, zh, sub)
        dq_ref, dk_ref, dv_ref, dz_ref, c_ref = orc.train_backward_sequence(qs, ks, vs, zh, dout[lo:hi, h * G:(h + 1) * G], sub,
                                                                             lam[h:h + 1].astype(np.float64))
        pairs = ((to_np(out[lo:hi, h * G:(h + 1) * G]), o_ref, "out"), (to_np(dq[lo:hi, h * G:(h + 1) * G]), dq_ref, "dq"),
                 (to_np(dk[lo:hi, h:h + 1]), dk_ref, "dk"), (to_np(dv[lo:hi, h:h + 1]), dv_ref, "dv"),
                 (to_np(dz[h:h + 1, lo:hi]), dz_ref, "dz"))
        for got, ref, what in pairs:
            scale = float(np.max(np.abs(ref)))
            err = float(np.max(np.abs(got.astype(np.float64) - ref)))
            assert err <= OUT_TOL["bf16"] * scale, (s, h, what, err, scale)
        assert float(np.max(np.abs(to_np(lse[h * G:(h + 1) * G, lo:hi]) - lse_ref))) <= 2e-3
        assert int(cnt_g[s, h]) == int(c_ref[0])
    assert n_checked >= 1
    # counts of every (sequence, head): exact wherever no logit sits inside the scoring error of the threshold
    for s in range(w.n_seqs):
        lo, hi = int(w.cu_seqlens[s]), int(w.cu_seqlens[s + 1])
        for h in range(w.Hkv):
            zh = z64[h, lo:hi]
            unsure = int((np.abs(zh) <= 2 * eps).sum())
            assert abs(int(cnt_g[s, h]) - int((zh.astype(np.float32) > 0).sum())) <= unsure
    # the scoring CNN's backward at this size (16 token chunks of the two-stage sums), on a random d logits so that the
    # comparison does not inherit the attention backward's error: every parameter and input gradient, all heads
    dz_in = rng.standard_normal((w.Hkv, w.total_tokens)).astype(np.float32)
    got = B.ltea_cnn_backward(d.cfg, d.cnn, d.k, d.v, d.cu, d.max_seqlen, torch.from_numpy(dz_in).cuda())
    ref = orc.score_backward(w.k, w.v, cnn, w.cu_seqlens, dz_in)
    flat_g = list(got[0]) + list(got[1]) + [got[2], got[3]]
    flat_r = list(ref[0]) + list(ref[1]) + [ref[2], ref[3]]
    for i, (a, b) in enumerate(zip(flat_g, flat_r)):
        a = a.float().cpu().numpy().astype(np.float64)
        assert float(np.abs(a - b).max()) <= 1e-4 * float(np.abs(b).max()), (i, float(np.abs(a - b).max()), float(np.abs(b).max()))
    for a, b, what in ((got[4], ref[4], "dk"), (got[5], ref[5], "dv")):
        a = a.float().cpu().numpy().astype(np.float64)
        assert float(np.abs(a - b).max()) <= 2 ** -7 * float(np.abs(b).max()), what


@pytest.mark.parametrize("lazy", [False, True])
def test_full_paper_stack_decode(lazy):
    """Decode at the paper's module shape (B=4, 32 query heads on 8 KV heads, window 768, 512 retained, 3-layer dilated
    CNN) after the full-size prefill: 40 steps, eager (packed-window scoring) or lazy with one batched scoring in the
    middle; one whole sequence through the oracle at every step (outputs of all 32 heads, retained sets of all 8)."""
    w = wl.config_paper_stack_bf16()
    ocfg, ocnn = oracle_cfg(w), oracle_cnn(w.cnn)
    d = DeviceWorkload(w)
    cache = d.new_cache()
    logits = torch.empty((w.Hkv, w.total_tokens), dtype=torch.float32, device="cuda")
    B.ltea_prefill(d.cfg, d.cnn, d.q, d.k, d.v, d.cu, d.max_seqlen, cache, logits=logits)
    z64 = orc.score(w.k, w.v, ocnn, w.cu_seqlens)
    eps = float(np.max(np.abs(to_np(logits) - z64)))
    n_strict = check_sets_strict(cache, to_np(logits), w)
    near = check_sets(cache, z64, w, eps)
    print(f"[paper_stack decode] strict set check on {n_strict} heads ok; {len(near)} head(s) inside the margin: {near}", flush=True)
    s = next(x for x in range(w.n_seqs) if all(ss != x for ss, _ in near))
    lo, hi = int(w.cu_seqlens[s]), int(w.cu_seqlens[s + 1])
    rho = w.cnn.rho
    kept = [orc.retain(z64[h, lo:hi], hi - lo, w.window, w.budget, w.sink, w.tau) for h in range(w.Hkv)]
    st = orc.state_after_prefill(w.k[lo:hi], w.v[lo:hi], z64[:, lo:hi], ocfg, rho, kept)
    ws = B.decode_workspace(d.cfg, d.cnn, w.n_seqs)
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    worst, scale = 0.0, 0.0
    for step in range(40):
        q, k, v = wl.decode_inputs(w.seed, step, w.dtype, w.n_seqs, w.Hq, w.Hkv, w.D)
        if lazy:
            if step == 20:
                B.ltea_rescore(d.cfg, d.cnn, cache, status=status)
            out = B.ltea_decode_step_lazy(d.cfg, dev(q, "bf16"), dev(k, "bf16"), dev(v, "bf16"), cache, status=status)
        else:
            out = B.ltea_decode_step(d.cfg, d.cnn, dev(q, "bf16"), dev(k, "bf16"), dev(v, "bf16"), cache, workspace=ws)
        ref = orc.decode_step(st, q[s], k[s], v[s], ocfg, ocnn)
        got = out[s].float().cpu().numpy()
        worst = max(worst, float(np.abs(got - ref).max()))
        scale = max(scale, float(np.abs(ref).max()))
        if step % 10 == 9:
            for h in range(w.Hkv):
                cnt, pos = gpu_retained_sets(cache, s, h)
                np.testing.assert_array_equal(np.sort(pos), orc.retained_positions(st)[h], err_msg=f"step {step} head {h}")
    assert worst <= OUT_TOL["bf16"] and worst <= OUT_TOL["bf16"] * scale, (worst, scale)
    if lazy:
        B.ltea_rescore(d.cfg, d.cnn, cache, status=status)
        assert int(status.item()) == 0
    assert int(cache.n_seen[s]) == st.n_seen and int(cache.n_scored[s]) == st.n_scored
    for h in range(w.Hkv):
        for p, zp in st.heads[h].win_z.items():
            if p >= hi - lo - rho:        # logits finalised during decoding
                zg = float(cache.win_score[s, h, p % w.window])
                assert abs(zg - zp) <= LOGIT_TOL["bf16"] * max(1.0, abs(zp)), (h, p, zg, zp)


def test_full_very_long_sequence():
    """One sequence of 400 000 tokens next to a short one (the streaming path of the selection, thousands of query
    tiles, 32-bit byte offsets inside a sequence far from their limit but far from small)."""
    w = wl.make_prefill("very_long", 321, "bf16", [400000, 5000], 4, 2, 64, 1024, 512, 4, 0.0, cnn_kernel=(5,),
                        cnn_channels=(32,), qkv_scale=1.0, w_std=0.05)
    run_full_prefill(w)


def test_full_decode_large_batch():
    """640 sequences of the decode_bf16 shape: every cache tensor is larger than 2^31 bytes, so any 32-bit offset in
    the decode, batched-scoring or lazy kernels would show.  The state is drawn on the device; ring logits come from
    ltea_rescore over the whole batch; three sequences (first, middle, last) are stepped through the oracle."""
    Bn, Hq, Hkv, D, window, budget, n0 = 640, 16, 16, 128, 1024, 512, 4096
    rng = np.random.default_rng(77)
    cnnw = wl.make_cnn(rng, "bf16", Hkv, D, (5,), (32,), [1], 0.05)
    cfg = B.make_cfg(Hq, Hkv, D, window, budget, 0, 0.0, 0.0, "bf16")
    cnn = B.upload_cnn(cnnw.kernel, cnnw.dilation, cnnw.w, cnnw.bias, cnnw.w_out, cnnw.b_out, "bf16")
    ocfg, ocnn = orc.OracleCfg(Hq, Hkv, D, window, budget, 0, 0.0), oracle_cnn(cnnw)
    rho = cnnw.rho
    gen = torch.Generator("cuda").manual_seed(99)
    rnd = lambda *shape: torch.randn(shape, device="cuda", generator=gen, dtype=torch.float32).to(torch.bfloat16)
    k_win, v_win = rnd(Bn, Hkv, window, D), rnd(Bn, Hkv, window, D)
    k_ret, v_ret = rnd(Bn, Hkv, budget, D), rnd(Bn, Hkv, budget, D)
    assert k_win.numel() * 2 > 2 ** 31
    ret_score = torch.rand((Bn, Hkv, budget), device="cuda", generator=gen) * 0.05 + 0.001
    # distinct positions below n0 - window, ascending
    ret_pos = torch.sort(torch.argsort(torch.rand((Bn, Hkv, n0 - window), device="cuda", generator=gen), dim=2)[:, :, :budget],
                         dim=2).values.to(torch.int32).contiguous()
    cache = B.wrap_cache(k_win, v_win, torch.full((Bn, Hkv, window), float("nan"), device="cuda"), k_ret, v_ret, ret_score,
                         ret_pos, torch.full((Bn, Hkv), budget, dtype=torch.int32, device="cuda"),
                         torch.full((Bn,), n0, dtype=torch.int32, device="cuda"),
                         torch.full((Bn,), n0 - window + rho, dtype=torch.int32, device="cuda"))
    # the oldest rho ring logits must be final already: score them per sampled sequence below, zero elsewhere (those
    # tokens are evicted in the first rho steps; a zero logit is "not a candidate", the same on both sides)
    cache.win_score[:, :, :rho] = 0.0
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    B.ltea_rescore(cfg, cnn, cache, status=status)
    torch.cuda.synchronize()
    assert int(status.item()) == 0 and bool((cache.n_scored == n0 - rho).all())
    sampled = [0, Bn // 2, Bn - 1]
    states = {}
    for b in sampled:
        st = orc.empty_state(ocfg)
        st.n_seen, st.n_scored = n0, n0 - rho
        kb, vb = to_np(k_win[b]), to_np(v_win[b])
        z = orc.score_sequence(np.transpose(kb, (1, 0, 2)), np.transpose(vb, (1, 0, 2)), ocnn)
        zg = cache.win_score[b].cpu().numpy()
        # slot i holds position n0 - window + i (n0 is a multiple of the window); positions rho .. window-rho-1 were
        # scored by the batched scoring with their whole receptive field inside the ring
        ref = z[:, rho:window - rho]
        assert np.all(np.abs(zg[:, rho:window - rho] - ref) <= LOGIT_TOL["bf16"] * np.maximum(1.0, np.abs(ref)))
        for h in range(Hkv):
            hs = st.heads[h]
            for i in range(window):
                hs.win_pos.append(n0 - window + i)
                hs.win_k.append(kb[h, i].astype(np.float64)); hs.win_v.append(vb[h, i].astype(np.float64))
                if i < rho:
                    hs.win_z[n0 - window + i] = 0.0
                elif i < window - rho:
                    hs.win_z[n0 - window + i] = float(z[h, i])
            kr, vr = to_np(k_ret[b, h]), to_np(v_ret[b, h])
            sc, ps = ret_score[b, h].cpu().numpy(), ret_pos[b, h].cpu().numpy()
            for r in range(budget):
                hs.ret_pos.append(int(ps[r])); hs.ret_key.append(np.float32(sc[r]))
                hs.ret_k.append(kr[r].astype(np.float64)); hs.ret_v.append(vr[r].astype(np.float64))
        states[b] = st
    worst, scale = 0.0, 0.0
    for step in range(12):
        q, k, v = rnd(Bn, Hq, D), rnd(Bn, Hkv, D), rnd(Bn, Hkv, D)
        if step < 6:
            out = B.ltea_decode_step(cfg, cnn, q, k, v, cache)
        else:
            out = B.ltea_decode_step_lazy(cfg, q, k, v, cache, status=status)
        for b in sampled:
            ref = orc.decode_step(states[b], to_np(q[b]), to_np(k[b]), to_np(v[b]), ocfg, ocnn)
            worst = max(worst, float(np.abs(to_np(out[b]) - ref).max()))
            scale = max(scale, float(np.abs(ref).max()))
    assert worst <= OUT_TOL["bf16"] and worst <= OUT_TOL["bf16"] * scale, (worst, scale)
    assert int(status.item()) == 0 and bool((cache.n_seen == n0 + 12).all())
    for b in sampled:
        for h in range(Hkv):
            cnt, pos = gpu_retained_sets(cache, b, h)
            np.testing.assert_array_equal(np.sort(pos), orc.retained_positions(states[b])[h])


def test_full_prefill_batch_above_2gib_matches_single_sequences():
    """300 sequences x 4000 tokens, 8 KV heads, D=128: K and V are 2.4 GB each, so any 32-bit element or byte offset
    across sequences would show.  Property checked (the small-case parity against the oracle is established
    elsewhere): packing is invisible, i.e. three sequences taken out of the batch and run alone give the same bits
    (outputs, logits, retained sets) as inside it."""
    n_seqs, n, Hq, Hkv, D, window, budget = 300, 4000, 8, 8, 128, 512, 256
    rng = np.random.default_rng(5)
    cnnw = wl.make_cnn(rng, "bf16", Hkv, D, (5,), (32,), [1], 0.05)
    cfg = B.make_cfg(Hq, Hkv, D, window, budget, 2, 0.0, 0.0, "bf16")
    cnn = B.upload_cnn(cnnw.kernel, cnnw.dilation, cnnw.w, cnnw.bias, cnnw.w_out, cnnw.b_out, "bf16")
    gen = torch.Generator("cuda").manual_seed(7)
    T = n_seqs * n
    rnd = lambda h: torch.randn((T, h, D), device="cuda", generator=gen, dtype=torch.float32).to(torch.bfloat16)
    q, k, v = rnd(Hq), rnd(Hkv), rnd(Hkv)
    assert k.numel() * 2 > 2 ** 31
    cu = torch.arange(0, T + 1, n, dtype=torch.int32, device="cuda")
    cache = B.alloc_cache(cfg, n_seqs)
    logits = torch.empty((Hkv, T), dtype=torch.float32, device="cuda")
    out = B.ltea_prefill(cfg, cnn, q, k, v, cu, n, cache, logits=logits)
    torch.cuda.synchronize()
    cu1 = torch.tensor([0, n], dtype=torch.int32, device="cuda")
    for s in (0, 171, n_seqs - 1):
        sl = slice(s * n, (s + 1) * n)
        c1 = B.alloc_cache(cfg, 1)
        l1 = torch.empty((Hkv, n), dtype=torch.float32, device="cuda")
        o1 = B.ltea_prefill(cfg, cnn, q[sl], k[sl], v[sl], cu1, n, c1, logits=l1)
        assert torch.equal(o1, out[sl]) and torch.equal(l1, logits[:, sl])
        assert torch.equal(c1.ret_count[0], cache.ret_count[s]) and torch.equal(c1.ret_pos[0], cache.ret_pos[s])
        assert torch.equal(c1.k_ret[0], cache.k_ret[s]) and torch.equal(c1.k_win[0], cache.k_win[s])
        assert torch.equal(c1.win_score[0], cache.win_score[s])
