"""Seeded sweep over odd configurations: every entry point on shapes nobody would pick by hand (odd windows and
budgets, group sizes 1..4, sinks, thresholds, stacks of 1..3 conv layers, empty and one-token sequences), each
against the oracle on the same inputs.  Sizes are small; the point is the corners of the index arithmetic.

Bars as in the other GPU tests.  Retained sets must match on every head whose decision margin exceeds twice the
measured logit error; heads inside the margin are skipped (and counted), and so is everything downstream of them."""
import numpy as np
import pytest
import torch

from oracle import ltea_oracle as orc
from paper_2510_20787_amd import binding as B
from paper_2510_20787_amd import workloads as wl
from tests.gpu_util import LOGIT_TOL_SWEEP, OUT_TOL, DeviceWorkload, boundary_margin, dev, gpu_retained_sets, to_np
from tests.helpers import oracle_cfg, oracle_cnn

pytestmark = pytest.mark.gpu


def draw_config(seed, scale=1):
    """scale multiplies the window range, the budgets and the sequence lengths (1 in the committed tests)."""
    rng = np.random.default_rng(90000 + seed)
    dtype = "bf16" if rng.random() < 0.75 else "f32"
    D = int(rng.choice([64, 128]))
    Hkv = int(rng.integers(1, 4))
    G = int(rng.choice([1, 2, 3, 4]))
    n_layers = int(rng.integers(1, 4))
    kernel = tuple(int(rng.choice([1, 3, 5, 7] if n_layers == 1 else [1, 3, 5])) for _ in range(n_layers))
    dilation = tuple(int(rng.integers(1, 3)) for _ in range(n_layers))
    widths = [int(rng.choice([8, 16, 32, 48, 64] if n_layers > 1 else [4, 8, 16, 24, 32])) for _ in range(n_layers)]
    rho = sum(d * (k - 1) // 2 for k, d in zip(kernel, dilation))
    # the per-step scoring of the eager decode keeps (2 rho + 1) rows of the widest layer twice in 48 KB of LDS
    while 2 * (2 * rho + 1) * max(2 * D, max(widths)) * 4 > 48 * 1024:
        dilation = tuple(1 for _ in dilation)
        kernel = tuple(min(k, 3) for k in kernel)
        rho = sum(d * (k - 1) // 2 for k, d in zip(kernel, dilation))
    window = int(rng.integers(2 * rho + 1, 2 * rho + 90 * scale))
    budget = int(rng.choice([0, 1, 2, 7, 16, 31, 40])) * scale
    sink = int(rng.integers(0, 5))
    tau = float(rng.choice([0.0, 0.0, -np.inf, 0.02]))
    n_seqs = int(rng.integers(1, 6))
    lens = [int(x) for x in rng.integers(0, 330 * scale, size=n_seqs)]
    if rng.random() < 0.5:
        lens[int(rng.integers(0, n_seqs))] = int(rng.choice([0, 1, 2]))
    if sum(lens) == 0:
        lens[0] = 77
    return dict(dtype=dtype, D=D, Hkv=Hkv, Hq=Hkv * G, kernel=kernel, dilation=dilation, widths=tuple(widths),
                window=window, budget=budget, sink=sink, tau=tau, lens=lens)


def head_margins(z64, w):
    """Decision margin of every (sequence, head) at the final length."""
    m = {}
    for s in range(w.n_seqs):
        lo, hi = int(w.cu_seqlens[s]), int(w.cu_seqlens[s + 1])
        for h in range(w.Hkv):
            m[(s, h)] = boundary_margin(orc.selection_key(z64[h, lo:hi], w.sink), hi - lo, w.window, w.budget, w.sink, w.tau)
    return m


@pytest.mark.parametrize("seed", range(24))
def test_random_configuration(seed, scale=1):
    c = draw_config(seed, scale)
    w = wl.make_prefill(f"random{seed}", 90000 + seed, c["dtype"], c["lens"], c["Hq"], c["Hkv"], c["D"], c["window"],
                        c["budget"], c["sink"], c["tau"], cnn_kernel=c["kernel"], cnn_channels=c["widths"],
                        cnn_dilation=c["dilation"], qkv_scale=1.0, w_std=0.08)
    print(f"[random {seed}] {c}", flush=True)
    cfg, cnn = oracle_cfg(w), oracle_cnn(w.cnn)
    dt = w.dtype
    tol = OUT_TOL[dt]
    d = DeviceWorkload(w)
    G = w.Hq // w.Hkv

    # ---- prefill -------------------------------------------------------------------------------------------
    ref_out, states, z64, kept = orc.prefill(w.q, w.k, w.v, cfg, cnn, w.cu_seqlens)
    cache = d.new_cache()
    logits = torch.empty((w.Hkv, w.total_tokens), dtype=torch.float32, device="cuda")
    out = to_np(B.ltea_prefill(d.cfg, d.cnn, d.q, d.k, d.v, d.cu, d.max_seqlen, cache, logits=logits))
    zg = to_np(logits)
    assert np.all(np.abs(zg - z64) <= LOGIT_TOL_SWEEP[dt] * np.maximum(1.0, np.abs(z64)))
    eps = float(np.max(np.abs(zg - z64))) if z64.size else 0.0
    margins = head_margins(z64, w)
    unsure = {key for key, m in margins.items() if m <= 2 * eps}
    scale = max(float(np.max(np.abs(ref_out))), 1e-30)
    for s in range(w.n_seqs):
        lo, hi = int(w.cu_seqlens[s]), int(w.cu_seqlens[s + 1])
        assert int(cache.n_seen[s]) == hi - lo and int(cache.n_scored[s]) == max(0, hi - lo - w.cnn.rho)
        for h in range(w.Hkv):
            if (s, h) in unsure:
                continue
            cnt, pos = gpu_retained_sets(cache, s, h)
            np.testing.assert_array_equal(pos, kept[s][h], err_msg=f"prefill seq {s} head {h}")
            if hi > lo:
                err = float(np.max(np.abs(out[lo:hi, h * G:(h + 1) * G] - ref_out[lo:hi, h * G:(h + 1) * G])))
                assert err <= tol * max(1.0, scale) and err <= tol * scale, (s, h, err, scale)
    assert len(unsure) <= 1, f"too many heads inside the decision margin: {unsure}"

    # ---- decode: three eager steps, then lazy steps with a batched scoring in between -----------------------
    period = B.ltea_lazy_period(d.cfg, d.cnn)
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    n_lazy = min(period, 6)
    for step in range(3 + n_lazy):
        q, k, v = wl.decode_inputs(w.seed, step, dt, w.n_seqs, w.Hq, w.Hkv, w.D)
        if step < 3:
            got = to_np(B.ltea_decode_step(d.cfg, d.cnn, dev(q, dt), dev(k, dt), dev(v, dt), cache))
        else:
            if step == 3 + n_lazy // 2:
                B.ltea_rescore(d.cfg, d.cnn, cache, status=status)
            got = to_np(B.ltea_decode_step_lazy(d.cfg, dev(q, dt), dev(k, dt), dev(v, dt), cache, status=status))
        ref = np.stack([orc.decode_step(states[s], q[s], k[s], v[s], cfg, cnn) for s in range(w.n_seqs)])
        # a logit finalised during decoding may land inside the error of the threshold: such heads drop out
        for s in range(w.n_seqs):
            for h in range(w.Hkv):
                for p, zp in states[s].heads[h].win_z.items():
                    if abs(zp - w.tau) <= 2 * max(eps, LOGIT_TOL_SWEEP[dt]):
                        unsure.add((s, h))
        for s in range(w.n_seqs):
            for h in range(w.Hkv):
                if (s, h) in unsure:
                    continue
                cnt, pos = gpu_retained_sets(cache, s, h)
                np.testing.assert_array_equal(np.sort(pos), orc.retained_positions(states[s])[h],
                                              err_msg=f"decode step {step} seq {s} head {h}")
                err = float(np.max(np.abs(got[s, h * G:(h + 1) * G] - ref[s, h * G:(h + 1) * G])))
                sc = float(np.max(np.abs(ref[s, h * G:(h + 1) * G])))
                assert err <= tol and err <= tol * max(sc, 1e-30), (step, s, h, err, sc)
    B.ltea_rescore(d.cfg, d.cnn, cache, status=status)
    assert int(status.item()) == 0
    for s in range(w.n_seqs):
        assert int(cache.n_seen[s]) == states[s].n_seen and int(cache.n_scored[s]) == states[s].n_scored
    assert len(unsure) <= 2, f"too many heads inside the decision margin: {unsure}"

    # ---- training forward / backward on the same sequences (no cap) -----------------------------------------
    if np.isfinite(w.tau) and z64.size and np.min(np.abs(z64 - w.tau)) > 2 * eps:
        rng = np.random.default_rng(w.seed + 5)
        dout = wl.to_storage(rng.standard_normal((w.total_tokens, w.Hq, w.D), dtype=np.float32), dt)
        lam = np.abs(rng.standard_normal(w.Hkv)).astype(np.float32) * np.float32(0.1)
        o_g, lse, lg, ws = B.ltea_train_forward(d.cfg, d.cnn, d.q, d.k, d.v, d.cu, d.max_seqlen)
        grads = B.ltea_train_backward(d.cfg, d.q, d.k, d.v, d.cu, d.max_seqlen, o_g, dev(dout, dt), lse, lg,
                                      torch.from_numpy(lam).cuda(), ws)
        names = ("dq", "dk", "dv", "dz")
        got = {n: to_np(x) for n, x in zip(names, grads[:4])}
        refs = {"dq": np.zeros(got["dq"].shape), "dk": np.zeros(got["dk"].shape), "dv": np.zeros(got["dv"].shape),
                "dz": np.zeros(got["dz"].shape)}
        for s in range(w.n_seqs):
            lo, hi = int(w.cu_seqlens[s]), int(w.cu_seqlens[s + 1])
            if hi == lo:
                continue
            r = orc.train_backward_sequence(w.q[lo:hi], w.k[lo:hi], w.v[lo:hi], z64[:, lo:hi], dout[lo:hi], cfg,
                                            lam.astype(np.float64))
            refs["dq"][lo:hi], refs["dk"][lo:hi], refs["dv"][lo:hi], refs["dz"][:, lo:hi] = r[0], r[1], r[2], r[3]
            np.testing.assert_array_equal(grads[4][s].cpu().numpy(), r[4])
        gtol = 2e-5 if dt == "f32" else 2e-2
        for n in names:
            sc = float(np.max(np.abs(refs[n])))
            err = float(np.max(np.abs(got[n].astype(np.float64) - refs[n])))
            # a reference that is exactly zero (one-token sequences: p = 1, dP = delta) is met up to rounding only
            assert err <= gtol * (sc if sc > 1e-3 else 1.0), (n, err, sc)


@pytest.mark.parametrize("seed", range(12))
def test_random_append(seed, scale=1):
    """The same kind of configurations through ltea_prefill + ltea_prefill_append with random cut points (bf16; the
    continuation's scoring tolerance is the prefill's): final state and last-chunk rows equal the one-shot oracle."""
    from tests.test_gpu_append import check_final_state, cu_of, pack
    c = draw_config(1000 + seed, scale)
    lens = [x + 40 for x in c["lens"]]
    w = wl.make_prefill(f"random_append{seed}", 91000 + seed, "bf16", lens, c["Hq"], c["Hkv"], c["D"], c["window"],
                        c["budget"], c["sink"], c["tau"], cnn_kernel=c["kernel"], cnn_channels=c["widths"],
                        cnn_dilation=c["dilation"], qkv_scale=1.0, w_std=0.05)
    print(f"[random append {seed}] {c}", flush=True)
    cfg, cnn = oracle_cfg(w), oracle_cnn(w.cnn)
    ref_out, ref_states, z64, kept = orc.prefill(w.q, w.k, w.v, cfg, cnn, w.cu_seqlens)
    d = DeviceWorkload(w)
    rng = np.random.default_rng(92000 + seed)
    cu = w.cu_seqlens
    n_cuts = int(rng.integers(1, 4))
    cuts = [[0] * w.n_seqs]
    for _ in range(n_cuts):
        cuts.append([int(rng.integers(cuts[-1][s], lens[s] + 1)) for s in range(w.n_seqs)])
    cuts.append(lens)
    cache = d.new_cache()
    last = np.zeros_like(ref_out, dtype=np.float32)
    for ci in range(len(cuts) - 1):
        a, b = cuts[ci], cuts[ci + 1]
        m = [b[s] - a[s] for s in range(w.n_seqs)]
        q, k, v = (dev(pack(x, cu, a, b), "bf16") for x in (w.q, w.k, w.v))
        cu_c = torch.from_numpy(cu_of(m)).cuda()
        if ci == 0:
            out = B.ltea_prefill(d.cfg, d.cnn, q, k, v, cu_c, max(max(m), 1), cache)
        else:
            out = B.ltea_prefill_append(d.cfg, d.cnn, q, k, v, cu_c, max(max(m), 1), cache)
        o = to_np(out)
        off = 0
        for s in range(w.n_seqs):
            last[int(cu[s]) + a[s]: int(cu[s]) + b[s]] = o[off: off + m[s]]
            off += m[s]
    torch.cuda.synchronize()
    zmax = float(np.max(np.abs(z64))) if z64.size else 1.0
    skip = check_final_state(w, cache, ref_states, z64, LOGIT_TOL_SWEEP["bf16"] * max(1.0, zmax))
    G = w.Hq // w.Hkv
    a = cuts[-2]
    for s in range(w.n_seqs):
        if a[s] == lens[s] or len(cuts) == 2:
            continue
        rows = slice(int(cu[s]) + a[s], int(cu[s]) + lens[s])
        for hq in range(w.Hq):
            if (s, hq // G) in skip:
                continue
            sc = float(np.max(np.abs(ref_out[rows, hq])))
            err = float(np.max(np.abs(last[rows, hq] - ref_out[rows, hq])))
            assert err <= OUT_TOL["bf16"] and err <= OUT_TOL["bf16"] * sc, (s, hq, err, sc)


@pytest.mark.parametrize("seed", range(10))
def test_random_decode_mix(seed):
    """Token-by-token decoding from an empty cache with small windows (rings wrap, compact segments overflow),
    switching at random between eager steps and lazy steps (a batched scoring whenever one is due or at random),
    then a continuation chunk (bf16) on top of the decoded state.  Reference: the oracle's per-step decode, and
    the oracle's one-shot prefill for the state after the continuation."""
    from tests.test_gpu_append import check_final_state, cu_of
    c = draw_config(2000 + seed)
    rng = np.random.default_rng(93000 + seed)
    rho = sum(dd * (kk - 1) // 2 for kk, dd in zip(c["kernel"], c["dilation"]))
    window = int(rng.integers(2 * rho + 1, 2 * rho + 30))
    n_dec, n_app, B_ = 110, int(rng.integers(1, 60)), int(rng.integers(1, 4))
    n = n_dec + n_app
    w = wl.make_prefill(f"random_mix{seed}", 93000 + seed, c["dtype"], [n] * B_, c["Hq"], c["Hkv"], c["D"], window,
                        c["budget"], c["sink"], c["tau"], cnn_kernel=c["kernel"], cnn_channels=c["widths"],
                        cnn_dilation=c["dilation"], qkv_scale=1.0, w_std=0.08)
    print(f"[random mix {seed}] window {window} {c}", flush=True)
    cfg, cnn = oracle_cfg(w), oracle_cnn(w.cnn)
    dt = w.dtype
    d = DeviceWorkload(w)
    cache = d.new_cache()
    states = [orc.empty_state(cfg) for _ in range(B_)]
    q3 = w.q.reshape(B_, n, w.Hq, w.D); k3 = w.k.reshape(B_, n, w.Hkv, w.D); v3 = w.v.reshape(B_, n, w.Hkv, w.D)
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    period = B.ltea_lazy_period(d.cfg, d.cnn)
    since, lazy_mode = 0, False
    G = w.Hq // w.Hkv
    unsure = set()
    tol = OUT_TOL[dt]
    # decision margins of every prefix from the oracle's final logits: a head drops out of the comparison once two
    # keys competing for the last slot (or a logit and the threshold) are closer than the scoring error
    z_all = orc.score(w.k, w.v, cnn, w.cu_seqlens)
    z_eps = 1e-6                          # running maximum of the measured logit error (ring logits against the oracle's)
    for t in range(n_dec):
        want_lazy = rng.random() < 0.6
        if lazy_mode and (not want_lazy or since >= period or rng.random() < 0.1):
            B.ltea_rescore(d.cfg, d.cnn, cache, status=status)      # also restores the eager step's invariant
            since = 0
        lazy_mode = want_lazy
        args = (dev(q3[:, t], dt), dev(k3[:, t], dt), dev(v3[:, t], dt), cache)
        if lazy_mode:
            got = to_np(B.ltea_decode_step_lazy(d.cfg, *args, status=status))
            since += 1
        else:
            got = to_np(B.ltea_decode_step(d.cfg, d.cnn, *args))
            since = 0
        ref = np.stack([orc.decode_step(states[s], q3[s, t], k3[s, t], v3[s, t], cfg, cnn) for s in range(B_)])
        if not lazy_mode:
            zw = cache.win_score.cpu().numpy()
            for s in range(B_):
                for h in range(w.Hkv):
                    for p, zp in states[s].heads[h].win_z.items():
                        z_eps = max(z_eps, abs(float(zw[s, h, p % window]) - zp))
            assert z_eps <= LOGIT_TOL_SWEEP[dt] * max(1.0, float(np.max(np.abs(z_all))))
        for s in range(B_):
            for h in range(w.Hkv):
                if (s, h) not in unsure:
                    key = orc.selection_key(z_all[h, s * n:s * n + t + 1], w.sink)
                    if boundary_margin(key, t + 1, window, w.budget, w.sink, w.tau) <= 2 * z_eps:
                        unsure.add((s, h))
                if (s, h) in unsure:
                    continue
                cnt, pos = gpu_retained_sets(cache, s, h)
                np.testing.assert_array_equal(np.sort(pos), orc.retained_positions(states[s])[h], err_msg=f"t {t} seq {s} head {h}")
                err = float(np.max(np.abs(got[s, h * G:(h + 1) * G] - ref[s, h * G:(h + 1) * G])))
                sc = float(np.max(np.abs(ref[s, h * G:(h + 1) * G])))
                assert err <= tol and err <= tol * max(sc, 1e-30), (t, s, h, err, sc)
    if lazy_mode:
        B.ltea_rescore(d.cfg, d.cnn, cache, status=status)
    assert int(status.item()) == 0
    assert len(unsure) <= max(2, B_ * w.Hkv // 2), unsure
    if dt != "bf16" or unsure:
        return
    # ---- continuation on top of the decoded state --------------------------------------------------------
    ref_out, ref_states, z64, kept = orc.prefill(w.q, w.k, w.v, cfg, cnn, w.cu_seqlens)
    idx = np.concatenate([np.arange(s * n + n_dec, (s + 1) * n) for s in range(B_)])
    out = to_np(B.ltea_prefill_append(d.cfg, d.cnn, dev(w.q[idx], dt), dev(w.k[idx], dt), dev(w.v[idx], dt),
                                      torch.from_numpy(cu_of([n_app] * B_)).cuda(), n_app, cache))
    zmax = float(np.max(np.abs(z64)))
    skip = check_final_state(w, cache, ref_states, z64, LOGIT_TOL_SWEEP["bf16"] * max(1.0, zmax))
    for s in range(B_):
        for hq in range(w.Hq):
            if (s, hq // G) in skip:
                continue
            ref = ref_out[s * n + n_dec:(s + 1) * n, hq]
            err = float(np.max(np.abs(out[s * n_app:(s + 1) * n_app, hq] - ref)))
            assert err <= tol * float(np.max(np.abs(ref))), (s, hq, err)


@pytest.mark.parametrize("seed", range(8))
def test_random_rotated_cache(seed):
    """Lazy decoding of a cache that holds rotated keys, from empty, on random configurations: random rotary width
    (a multiple of 16 up to D), either pairing, random cadence of the batched scoring (never later than allowed).
    Reference: the oracle's lazy procedure with its own inverse rotation, rounded to the storage type."""
    rotated_cache_run(seed, eager=False)


@pytest.mark.parametrize("seed", range(6))
def test_random_rotated_cache_eager(seed):
    """The same caches driven by ltea_decode_step_feat (one logit finalised per step from the ring rotated back).
    Reference: the oracle's lazy step followed by its batched scoring after every step."""
    rotated_cache_run(100 + seed, eager=True)


def rotated_cache_run(seed, eager):
    c = draw_config(3000 + seed)
    rng = np.random.default_rng(94000 + seed)
    rho = sum(dd * (kk - 1) // 2 for kk, dd in zip(c["kernel"], c["dilation"]))
    window = int(rng.integers(2 * rho + 1, 2 * rho + 40))
    n, B_ = 100, int(rng.integers(1, 4))
    rot = int(rng.choice([r for r in (16, 32, 48, 64, 96, 128) if r <= c["D"]]))
    inter = bool(rng.integers(0, 2))
    dt = c["dtype"]
    w = wl.make_prefill(f"random_rope{seed}", 94000 + seed, dt, [n] * B_, c["Hq"], c["Hkv"], c["D"], window, c["budget"],
                        c["sink"], c["tau"], cnn_kernel=c["kernel"], cnn_channels=c["widths"], cnn_dilation=c["dilation"],
                        qkv_scale=1.0, w_std=0.1)
    print(f"[random rope {seed}] window {window} rot {rot} interleaved {inter} {c}", flush=True)
    cfg, cnn = oracle_cfg(w), oracle_cnn(w.cnn)
    cos, sin = wl.rope_tables(n + 4, rot, 50.0)
    rope_o = orc.OracleRope(cos.astype(np.float64), sin.astype(np.float64), inter)
    rope_g = B.upload_rope(cos, sin, inter)
    rounder = (lambda x: wl.to_storage(x.astype(np.float32), dt).astype(np.float64))
    d = DeviceWorkload(w)
    cache = d.new_cache()
    states = [orc.empty_state(cfg) for _ in range(B_)]
    q3 = w.q.reshape(B_, n, w.Hq, w.D); k3 = w.k.reshape(B_, n, w.Hkv, w.D); v3 = w.v.reshape(B_, n, w.Hkv, w.D)
    period = B.ltea_lazy_period(d.cfg, d.cnn)
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    G = w.Hq // w.Hkv
    since, z_eps, unsure = 0, 1e-6, set()
    tol = OUT_TOL[dt]
    def scored_both_sides():
        nonlocal z_eps
        zw = cache.win_score.cpu().numpy()
        for s in range(B_):
            orc.rescore(states[s], cfg, cnn, rope_o, rounder)
            assert int(cache.n_scored[s]) == states[s].n_scored
            for h in range(w.Hkv):
                for p, zp in states[s].heads[h].win_z.items():
                    z_eps = max(z_eps, abs(float(zw[s, h, p % window]) - zp))

    for t in range(n):
        if not eager and (since >= period or (since > 0 and rng.random() < 0.15)):
            B.ltea_rescore(d.cfg, d.cnn, cache, rope=rope_g, status=status)
            scored_both_sides()
            since = 0
        if eager:
            got = to_np(B.ltea_decode_step_feat(d.cfg, d.cnn, dev(q3[:, t], dt), dev(k3[:, t], dt), dev(v3[:, t], dt), cache,
                                                rope=rope_g, status=status))
        else:
            got = to_np(B.ltea_decode_step_lazy(d.cfg, dev(q3[:, t], dt), dev(k3[:, t], dt), dev(v3[:, t], dt), cache,
                                                status=status))
        since += 1
        # the oracle's keep decisions of this step, with their margins, before it takes the step
        for s in range(B_):
            for h in range(w.Hkv):
                hs = states[s].heads[h]
                if len(hs.win_pos) == window and (s, h) not in unsure:
                    e = hs.win_pos[0]
                    ze = hs.win_z[e]
                    close = [abs(ze - w.tau)] if e >= w.sink else []
                    if len(hs.ret_pos) >= w.budget > 0 and e >= w.sink:
                        close.append(abs(float(min(hs.ret_key)) - ze))
                    if close and min(close) <= 2 * z_eps + 1e-6:
                        unsure.add((s, h))
        ref = np.stack([orc.decode_step_lazy(states[s], q3[s, t], k3[s, t], v3[s, t], cfg) for s in range(B_)])
        for s in range(B_):
            for h in range(w.Hkv):
                if (s, h) in unsure:
                    continue
                cnt, pos = gpu_retained_sets(cache, s, h)
                np.testing.assert_array_equal(np.sort(pos), orc.retained_positions(states[s])[h], err_msg=f"t {t} seq {s} head {h}")
                err = float(np.max(np.abs(got[s, h * G:(h + 1) * G] - ref[s, h * G:(h + 1) * G])))
                sc = float(np.max(np.abs(ref[s, h * G:(h + 1) * G])))
                assert err <= tol and err <= tol * max(sc, 1e-30), (t, s, h, err, sc)
        if eager:   # the oracle's batched scoring after its lazy step finalises the logit the device just finalised
            scored_both_sides()
    assert int(status.item()) == 0
    assert z_eps <= (2e-3 if dt == "bf16" else 1e-4) * 4, z_eps
    assert len(unsure) <= max(2, B_ * w.Hkv // 2), unsure


@pytest.mark.parametrize("seed", range(10))
def test_random_rotary_append(seed):
    """Continued prefill of a rotary model on random configurations: random cut per sequence (empty first or second
    parts included), random rotary width and pairing, new keys given unrotated or rotated back by the library."""
    from tests.test_gpu_append import rotary_append_run
    c = draw_config(5000 + seed)
    rng = np.random.default_rng(95000 + seed)
    w = wl.make_prefill(f"random_rotary_append{seed}", 95000 + seed, c["dtype"], c["lens"], c["Hq"], c["Hkv"], c["D"],
                        c["window"], c["budget"], c["sink"], c["tau"], cnn_kernel=c["kernel"], cnn_channels=c["widths"],
                        cnn_dilation=c["dilation"], qkv_scale=1.0, w_std=0.08)
    cut = [int(rng.integers(0, n + 1)) for n in c["lens"]]
    rot = int(rng.choice([r for r in (16, 32, 48, 64, 96, 128) if r <= c["D"]]))
    inter, give = bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
    print(f"[random rotary append {seed}] cut {cut} rot {rot} interleaved {inter} k_feat {give} {c}", flush=True)
    near = rotary_append_run(w, cut, rot, inter, give)
    assert len(near) <= max(1, w.n_seqs * w.Hkv // 3), near
