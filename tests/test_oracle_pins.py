"""Pins for the CPU oracle: each test checks it against something fixed by the paper or by
mathematics (brute force from eq. 5, special cases, invariants, closed forms, a library conv).
CPU only.  The paper prints no numeric worked example of the mechanism, so there is no golden
value file for it; tests/golden/ holds only the hyper-parameters the paper states."""
import json
import os

import numpy as np
import pytest

from oracle import ltea_oracle as orc
from tests.helpers import (brute_force_keep, dense_masked_attention, oracle_cfg, oracle_cnn, small_prefill)

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def run_prefill(w):
    cfg, cnn = oracle_cfg(w), oracle_cnn(w.cnn)
    return cfg, cnn, orc.prefill(w.q, w.k, w.v, cfg, cnn, w.cu_seqlens)


# ---- P1: dense masked softmax from eq. 5 == sparse path --------------------------------------
@pytest.mark.parametrize("seed,n,window,budget,sink,G", [(0, 40, 12, 5, 0, 1), (1, 57, 9, 7, 2, 2),
                                                         (2, 33, 16, 3, 4, 1), (3, 64, 8, 40, 0, 2)])
def test_p1_dense_mask_equals_sparse(seed, n, window, budget, sink, G):
    w = small_prefill(seed=seed, seqlens=(n,), Hq=2 * G, Hkv=2, window=window, budget=budget, sink=sink)
    cfg, cnn, (out, states, z, kept) = run_prefill(w)
    keep = [brute_force_keep(orc.selection_key(z[h], sink), n, window, budget, sink, 0.0) for h in range(2)]
    for h in range(2):
        assert list(kept[0][h]) == keep[h]
    ref = dense_masked_attention(w.q, w.k, w.v, keep, window, cfg.sigma, G)
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-12)


# ---- P2 / P3: special cases ------------------------------------------------------------------
def test_p2_budget_zero_is_sliding_window():
    w = small_prefill(seed=4, seqlens=(50,), window=10, budget=0, sink=3)
    cfg, cnn, (out, states, z, kept) = run_prefill(w)
    assert all(len(r) == 0 for r in kept[0])
    ref = dense_masked_attention(w.q, w.k, w.v, [[], []], 10, cfg.sigma, 1)
    np.testing.assert_allclose(out, ref, atol=1e-12)
    # textbook SWA row: query 30 sees exactly positions 21..30
    q = w.q.astype(np.float64); k = w.k.astype(np.float64); v = w.v.astype(np.float64)
    s = cfg.sigma * (k[21:31, 0] @ q[30, 0]); p = np.exp(s - s.max()); p /= p.sum()
    np.testing.assert_allclose(out[30, 0], p @ v[21:31, 0], atol=1e-12)


def test_p3_window_covers_sequence_is_full_causal():
    w = small_prefill(seed=5, seqlens=(30,), window=30, budget=8)
    cfg, cnn, (out, states, z, kept) = run_prefill(w)
    assert all(len(r) == 0 for r in kept[0])
    n = 30
    q = w.q.astype(np.float64); k = w.k.astype(np.float64); v = w.v.astype(np.float64)
    for h in range(2):
        s = cfg.sigma * (q[:, h] @ k[:, h].T)
        s = np.where(np.tril(np.ones((n, n), bool)), s, -np.inf)
        p = np.exp(s - s.max(1, keepdims=True)); p /= p.sum(1, keepdims=True)
        np.testing.assert_allclose(out[:, h], p @ v[:, h], atol=1e-12)


# ---- P4: budget invariants -------------------------------------------------------------------
def test_p4_budget_invariants():
    w = small_prefill(seed=6, seqlens=(80,), window=10, budget=6, sink=2)
    cnn = oracle_cnn(w.cnn)
    z = orc.score(w.k, w.v, cnn, w.cu_seqlens)
    for h in range(2):
        prev = set()
        for b in range(0, 75):
            R = orc.retain(z[h], 80, 10, b, 2, 0.0)
            assert len(R) <= b
            assert all(0 <= j < 70 for j in R)
            assert all((j < 2) or np.float32(z[h, j]) > 0 for j in R)
            assert prev <= set(R)                       # nested in the budget
            if b >= 2:
                assert {0, 1} <= set(R)                 # sinks are never displaced
            prev = set(R)
            assert list(R) == brute_force_keep(orc.selection_key(z[h], 2), 80, 10, b, 2, 0.0)


def test_p4_kept_set_is_nested_in_the_prefix_length():
    """What a continued prefill relies on: a token outside the kept set of a prefix is outside the kept set of every
    longer prefix, so re-selecting among (kept set of the prefix) + (tokens that leave the window afterwards) gives
    the kept set of the longer prefix.  Heavy ties included (quantised logits)."""
    rng = np.random.default_rng(21)
    n, window, sink, tau = 140, 11, 2, 0.0
    for budget in (0, 1, 5, 17):
        for quant in (None, 0.5):
            z = rng.standard_normal(n)
            if quant:
                z = np.round(z / quant) * quant
            key = orc.selection_key(z, sink)
            for n1 in (0, 5, window, window + 1, 60, 139):
                R1 = orc.retain(z[:n1], n1, window, budget, sink, tau)
                for n2 in (n1, n1 + 1, n1 + window, n):
                    if n2 > n:
                        continue
                    R2 = orc.retain(z[:n2], n2, window, budget, sink, tau)
                    leaving = [j for j in range(max(0, n1 - window), max(0, n2 - window))]
                    pool = sorted(set(int(j) for j in R1) | {j for j in leaving if j < sink or np.float32(z[j]) > np.float32(tau)})
                    pool.sort(key=lambda j: (-float(key[j]) if np.isfinite(key[j]) else -np.inf, j))
                    assert sorted(pool[:budget]) == [int(j) for j in R2], (budget, quant, n1, n2)


def test_p4_ties_and_nan():
    z = np.array([0.5, 0.5, np.nan, 0.5, 0.7, 0.5, -1.0, 0.5] + [0.0] * 4, dtype=np.float64)
    # n=12, window=4 -> evictable 0..7; candidates: 0,1,3,4,5,7 (NaN and -1 never)
    assert list(orc.retain(z, 12, 4, 10, 0, 0.0)) == [0, 1, 3, 4, 5, 7]
    # cap 3: best key 0.7 (pos 4), then equal keys by ascending position: 0, 1
    assert list(orc.retain(z, 12, 4, 3, 0, 0.0)) == [0, 1, 4]
    # tau = -inf: pure top-b, NaN still never a candidate
    assert list(orc.retain(z, 12, 4, 7, 0, -np.inf)) == [0, 1, 3, 4, 5, 6, 7]
    # +inf logits are legal and tie with sinks by position
    z2 = np.array([0.1, np.inf, 0.2, np.inf, 0.3, 0.0, 0.0, 0.0], dtype=np.float64)
    assert list(orc.retain(z2, 8, 3, 2, 1, 0.0)) == [0, 1]


# ---- P5: streaming retention == batch retention; prefill + decode == longer prefill ---------
@pytest.mark.parametrize("seed,n,window,budget,sink,kernel,dil", [(7, 45, 9, 4, 0, (3,), None), (8, 60, 13, 6, 2, (5,), None),
                                                                  (9, 50, 15, 5, 1, (3, 3), (2, 1))])
def test_p5_decode_from_empty_matches_prefill_state(seed, n, window, budget, sink, kernel, dil):
    ch = (4,) * len(kernel)
    w = small_prefill(seed=seed, seqlens=(n,), window=window, budget=budget, sink=sink, kernel=kernel, channels=ch, dilation=dil)
    cfg, cnn, (out, states, z, kept) = run_prefill(w)
    st = orc.empty_state(cfg)
    for t in range(n):
        orc.decode_step(st, w.q[t], w.k[t], w.v[t], cfg, cnn)
        # streaming set after token t == batch rule on the prefix of length t+1
        for h in range(cfg.Hkv):
            ref = orc.retain(z[h, :t + 1], t + 1, window, budget, sink, 0.0)
            assert list(orc.retained_positions(st)[h]) == list(ref), (t, h)
    ref_state = states[0]
    assert st.n_seen == ref_state.n_seen and st.n_scored == ref_state.n_scored
    for h in range(cfg.Hkv):
        a, b = st.heads[h], ref_state.heads[h]
        assert a.win_pos == b.win_pos
        assert sorted(a.ret_pos) == sorted(b.ret_pos)
        for j in b.win_z:
            assert abs(a.win_z[j] - b.win_z[j]) < 1e-12
        ia, ib = np.argsort(a.ret_pos), np.argsort(b.ret_pos)
        np.testing.assert_array_equal(np.array(a.ret_key)[ia], np.array(b.ret_key)[ib])
        np.testing.assert_allclose(np.stack(a.win_k), np.stack(b.win_k))
        if b.ret_pos:
            np.testing.assert_allclose(np.stack(a.ret_k)[ia], np.stack(b.ret_k)[ib])
            np.testing.assert_allclose(np.stack(a.ret_v)[ia], np.stack(b.ret_v)[ib])


def test_p5_prefill_then_decode_equals_longer_prefill():
    n, extra = 40, 17
    w = small_prefill(seed=10, seqlens=(n + extra,), window=11, budget=5, sink=1, kernel=(5,))
    cfg, cnn = oracle_cfg(w), oracle_cnn(w.cnn)
    _, st_long, z_long, kept_long = orc.prefill(w.q, w.k, w.v, cfg, cnn, [0, n + extra])
    _, st_short, _, _ = orc.prefill(w.q[:n], w.k[:n], w.v[:n], cfg, cnn, [0, n])
    st = st_short[0]
    for t in range(n, n + extra):
        orc.decode_step(st, w.q[t], w.k[t], w.v[t], cfg, cnn)
    for h in range(cfg.Hkv):
        assert list(orc.retained_positions(st)[h]) == list(kept_long[0][h])
        assert st.heads[h].win_pos == st_long[0].heads[h].win_pos
        for j, zj in st_long[0].heads[h].win_z.items():
            assert abs(st.heads[h].win_z[j] - zj) < 1e-12


# ---- P6: when the cap never binds, prefill == step-by-step decode == uncapped eq. 5 ---------
def test_p6_cap_not_binding_prefill_equals_decode():
    n = 48
    w = small_prefill(seed=11, seqlens=(n,), window=10, budget=n, sink=2)
    cfg, cnn, (out, states, z, kept) = run_prefill(w)
    st = orc.empty_state(cfg)
    dec = np.stack([orc.decode_step(st, w.q[t], w.k[t], w.v[t], cfg, cnn) for t in range(n)])
    np.testing.assert_allclose(dec, out, atol=1e-12)
    keep = [[j for j in range(n) if j < 2 or np.float32(z[h, j]) > 0] for h in range(2)]   # eq. 5, no cap
    ref = dense_masked_attention(w.q, w.k, w.v, keep, 10, cfg.sigma, 1)
    np.testing.assert_allclose(out, ref, atol=1e-12)


# ---- P7: library grouped convolution ---------------------------------------------------------
@pytest.mark.parametrize("kernel,dil,ch", [((5,), (1,), (6,)), ((3, 3, 3), (2, 2, 2), (8, 4, 2)), ((7,), (1,), (3,))])
def test_p7_library_grouped_conv(kernel, dil, ch):
    import torch
    import torch.nn.functional as F
    n, Hkv, D = 37, 3, 4
    w = small_prefill(seed=12, seqlens=(n,), Hq=Hkv, Hkv=Hkv, D=D, kernel=kernel, channels=ch, dilation=dil, window=20)
    cnn = oracle_cnn(w.cnn)
    z = orc.score(w.k, w.v, cnn, w.cu_seqlens)
    x = torch.from_numpy(np.concatenate([w.k, w.v], axis=2).astype(np.float64))      # [n, Hkv, 2D]
    x = x.permute(1, 2, 0).reshape(1, Hkv * 2 * D, n)
    for l, (ks, d) in enumerate(zip(kernel, dil)):
        W = torch.from_numpy(w.cnn.w[l].astype(np.float64))                          # [Hkv, Co, Ci, ks]
        Wg = W.reshape(Hkv * W.shape[1], W.shape[2], ks)
        b = torch.from_numpy(w.cnn.bias[l].astype(np.float64)).reshape(-1)
        x = F.silu(F.conv1d(x, Wg, b, padding=d * (ks - 1) // 2, dilation=d, groups=Hkv))
    Wo = torch.from_numpy(w.cnn.w_out.astype(np.float64)).reshape(Hkv, -1, 1)
    zz = F.conv1d(x, Wo, torch.from_numpy(w.cnn.b_out.astype(np.float64)), groups=Hkv)[0].numpy()
    np.testing.assert_allclose(z, zz, atol=1e-12)


# ---- P8: closed forms of the CNN --------------------------------------------------------------
def test_p8_cnn_closed_forms():
    n, Hkv, D, C, ks = 20, 2, 3, 2, 5
    rng = np.random.default_rng(13)
    k = rng.standard_normal((n, Hkv, D)); v = rng.standard_normal((n, Hkv, D))
    W = np.zeros((Hkv, C, 2 * D, ks)); bias = np.zeros((Hkv, C))
    w_out = np.array([[1.5, 0.0], [0.0, -2.0]]); b_out = np.array([0.25, -0.5])
    # all-zero conv weights: z == b_out everywhere
    z = orc.score(k, v, orc.cnn_from_arrays([ks], [1], [W], [bias], w_out, b_out), [0, n])
    np.testing.assert_allclose(z, np.repeat(b_out[:, None], n, 1), atol=0)
    # ... so with b_out > tau the kept set is the budget's lowest positions; with b_out <= tau only sinks
    assert list(orc.retain(z[0], n, 4, 3, 0, 0.0)) == [0, 1, 2]
    assert list(orc.retain(z[1], n, 4, 3, 2, 0.0)) == [0, 1]
    sil = lambda x: x / (1 + np.exp(-x))
    # one-hot centre tap on key channel 1 (head 0, out channel 0) / value channel 2 (head 1, channel 1)
    W1 = W.copy(); W1[0, 0, 1, 2] = 1.0; W1[1, 1, D + 2, 2] = 1.0
    z = orc.score(k, v, orc.cnn_from_arrays([ks], [1], [W1], [bias], w_out, b_out), [0, n])
    np.testing.assert_allclose(z[0], 0.25 + 1.5 * sil(k[:, 0, 1]), atol=1e-14)
    np.testing.assert_allclose(z[1], -0.5 - 2.0 * sil(v[:, 1, 2]), atol=1e-14)
    # one-hot tap 0 reads position j-2 (past), tap 4 reads j+2 (future); outside -> zero
    W2 = W.copy(); W2[0, 0, 1, 0] = 1.0; W2[1, 1, D + 2, 4] = 1.0
    z = orc.score(k, v, orc.cnn_from_arrays([ks], [1], [W2], [bias], w_out, b_out), [0, n])
    past = np.concatenate([np.zeros(2), k[:-2, 0, 1]])
    fut = np.concatenate([v[2:, 1, 2], np.zeros(2)])
    np.testing.assert_allclose(z[0], 0.25 + 1.5 * sil(past), atol=1e-14)
    np.testing.assert_allclose(z[1], -0.5 - 2.0 * sil(fut), atol=1e-14)
    # dilation 3 on tap 0 reads j-6
    z = orc.score(k, v, orc.cnn_from_arrays([ks], [3], [W2], [bias], w_out, b_out), [0, n])
    np.testing.assert_allclose(z[0], 0.25 + 1.5 * sil(np.concatenate([np.zeros(6), k[:-6, 0, 1]])), atol=1e-14)
    # bias path and sigmoid
    bias2 = np.array([[0.3, 0.0], [0.0, -0.7]])
    z = orc.score(k, v, orc.cnn_from_arrays([ks], [1], [W], [bias2], w_out, b_out), [0, n])
    np.testing.assert_allclose(z[0], 0.25 + 1.5 * sil(0.3), atol=1e-14)
    np.testing.assert_allclose(orc.retention_score(np.array([0.0, np.log(3.0)])), [0.5, 0.75], atol=1e-15)


def test_p8_paper_stack_receptive_field():
    with open(os.path.join(GOLDEN, "paper_hyperparameters.json")) as f:
        hp = json.load(f)
    ks, dil = hp["lte_cnn"]["kernel"], hp["lte_cnn"]["dilation"]
    n, D = 40, 4
    ch = [2 * D // 2, 2 * D // 4, 2 * D // 8]
    w = small_prefill(seed=14, seqlens=(n,), Hq=1, Hkv=1, D=D, kernel=ks, channels=ch, dilation=dil, window=20)
    cnn = oracle_cnn(w.cnn)
    assert 2 * cnn.rho + 1 == hp["lte_cnn"]["receptive_field"]
    z0 = orc.score(w.k, w.v, cnn, [0, n])[0]
    # perturbing one token changes exactly the logits within rho of it (and no others)
    k2 = w.k.copy(); k2[20, 0, 1] += 1.0
    z1 = orc.score(k2, w.v, cnn, [0, n])[0]
    changed = np.nonzero(np.abs(z1 - z0) > 0)[0]
    assert changed.min() >= 20 - cnn.rho and changed.max() <= 20 + cnn.rho
    assert set(changed) >= {20 - cnn.rho, 20, 20 + cnn.rho}


def test_lazy_period_of_the_paper_shape_against_the_printed_cadence():
    """Section 3.1.3 (lazy scoring) prints one batched scoring per w - R steps; for the paper's w = 768, R = 13 that is
    755.  The reading taken here (scoring is due when the next token would overwrite the left context of the oldest
    unscored position) allows one step more, w - 2*rho = w - R + 1 = 756; the difference is the paper counting the
    step that triggers the scoring."""
    with open(os.path.join(GOLDEN, "paper_hyperparameters.json")) as f:
        hp = json.load(f)
    ks, dil = hp["lte_cnn"]["kernel"], hp["lte_cnn"]["dilation"]
    cnn = orc.cnn_from_arrays(ks, dil, [np.zeros((1, 2, 2, k)) for k in ks], [np.zeros((1, 2))] * 3, np.zeros((1, 2)), np.zeros(1))
    cfg = orc.OracleCfg(1, 1, 1, hp["window"]["w"], hp["budget"]["b"], hp["sink"]["s"], hp["threshold"]["logit"])
    assert hp["window"]["w"] - hp["lte_cnn"]["receptive_field"] == hp["lazy_scoring_period"]["steps"]
    assert orc.lazy_period(cfg, cnn) == hp["lazy_scoring_period"]["steps"] + 1


# ---- P9: closed forms of the softmax ----------------------------------------------------------
def test_p9_softmax_closed_forms():
    n, window, D = 30, 6, 4
    w = small_prefill(seed=15, seqlens=(n,), Hq=1, Hkv=1, D=D, window=window, budget=4)
    cfg = oracle_cfg(w)
    k = np.tile(np.array([[0.3, -0.2, 0.1, 0.5]]), (n, 1))[:, None, :]
    kept = [np.array([1, 5, 20])]
    out = orc.sparse_attention_sequence(w.q, k, w.v, cfg, kept)
    v = w.v.astype(np.float64)
    for i in (0, 3, 9, 29):
        S = [j for j in kept[0] if j <= i - window] + list(range(max(0, i - window + 1), i + 1))
        np.testing.assert_allclose(out[i, 0], v[S, 0].mean(axis=0), atol=1e-13)
    # one dominant key: output is (almost exactly) that key's value
    k2 = np.zeros((n, 1, D)); k2[5, 0, 0] = 1000.0
    q2 = np.zeros((n, 1, D)); q2[:, 0, 0] = 1.0
    out = orc.sparse_attention_sequence(q2, k2, w.v, cfg, kept)
    np.testing.assert_allclose(out[25, 0], v[5, 0], atol=1e-12)          # 5 is kept and out of window
    np.testing.assert_allclose(out[7, 0], v[5, 0], atol=1e-12)           # 5 is inside the window
    out_nokeep = orc.sparse_attention_sequence(q2, k2, w.v, cfg, [np.array([1, 20])])
    assert np.abs(out_nokeep[25, 0] - v[5, 0]).max() > 1e-3              # evicted -> invisible


# ---- P10: physical order of the cache is irrelevant ------------------------------------------
def test_p10_cache_order_irrelevant():
    n = 50
    w = small_prefill(seed=16, seqlens=(n + 1,), window=9, budget=6)
    cfg, cnn = oracle_cfg(w), oracle_cnn(w.cnn)
    _, sts, _, _ = orc.prefill(w.q[:n], w.k[:n], w.v[:n], cfg, cnn, [0, n])
    _, sts2, _, _ = orc.prefill(w.q[:n], w.k[:n], w.v[:n], cfg, cnn, [0, n])
    rng = np.random.default_rng(0)
    for hs in sts2[0].heads:
        perm = rng.permutation(len(hs.ret_pos))
        hs.ret_pos = [hs.ret_pos[i] for i in perm]; hs.ret_key = [hs.ret_key[i] for i in perm]
        hs.ret_k = [hs.ret_k[i] for i in perm]; hs.ret_v = [hs.ret_v[i] for i in perm]
    o1 = orc.decode_step(sts[0], w.q[n], w.k[n], w.v[n], cfg, cnn)
    o2 = orc.decode_step(sts2[0], w.q[n], w.k[n], w.v[n], cfg, cnn)
    np.testing.assert_allclose(o1, o2, atol=1e-12)
    assert [sorted(h.ret_pos) for h in sts[0].heads] == [sorted(h.ret_pos) for h in sts2[0].heads]


# ---- P11: packed sequences == each sequence alone --------------------------------------------
def test_p11_varlen_packing():
    lens = (23, 1, 40, 7, 0, 31)
    w = small_prefill(seed=17, seqlens=lens, window=8, budget=4, sink=1)
    cfg, cnn, (out, states, z, kept) = run_prefill(w)
    cu = w.cu_seqlens
    for s, n in enumerate(lens):
        lo, hi = cu[s], cu[s + 1]
        o, st, zz, kk = orc.prefill(w.q[lo:hi], w.k[lo:hi], w.v[lo:hi], cfg, cnn, [0, n])
        np.testing.assert_allclose(out[lo:hi], o, atol=0)
        np.testing.assert_allclose(z[:, lo:hi], zz, atol=0)
        for h in range(cfg.Hkv):
            assert list(kept[s][h]) == list(kk[0][h])
        assert states[s].n_seen == n


# ---- P12: uniform-stride keep pattern fed straight to the attention --------------------------
def test_p12_uniform_stride_keep_mask():
    n, window, stride = 70, 10, 7
    w = small_prefill(seed=18, seqlens=(n,), window=window, budget=0)
    cfg = oracle_cfg(w)
    keep = [np.arange(0, n, stride), np.arange(3, n, stride)]
    out = orc.sparse_attention_sequence(w.q, w.k, w.v, cfg, keep)
    ref = dense_masked_attention(w.q, w.k, w.v, keep, window, cfg.sigma, 1)
    np.testing.assert_allclose(out, ref, atol=1e-12)


# ---- P13: grouped queries share their KV head's kept set -------------------------------------
def test_p13_gqa_shares_kept_set():
    n = 44
    w = small_prefill(seed=19, seqlens=(n,), Hq=6, Hkv=2, window=9, budget=5)
    cfg, cnn, (out, states, z, kept) = run_prefill(w)
    assert z.shape == (2, n) and len(kept[0]) == 2
    # a query head moved to another slot of the same group gives the same output row
    q2 = w.q.copy(); q2[:, 1] = w.q[:, 0]
    out2, *_ = orc.prefill(q2, w.k, w.v, cfg, cnn, w.cu_seqlens)
    np.testing.assert_allclose(out2[:, 1], out[:, 0], atol=0)
    keepb = [brute_force_keep(orc.selection_key(z[h], 0), n, 9, 5, 0, 0.0) for h in range(2)]
    np.testing.assert_allclose(out, dense_masked_attention(w.q, w.k, w.v, keepb, 9, cfg.sigma, 3), atol=1e-12)


# ---- P14: the rotation used to undo RoPE on cached keys ---------------------------------------
def _rope(n_pos=64, rot=8, interleaved=False, base=100.0):
    ang = np.arange(n_pos, dtype=np.float64)[:, None] * base ** (-np.arange(0, rot, 2, dtype=np.float64) / rot)[None, :]
    return orc.OracleRope(np.cos(ang), np.sin(ang), interleaved)


def test_p14_rotation_is_complex_multiplication_and_has_an_inverse():
    rng = np.random.default_rng(0)
    D, rot = 12, 8
    x = rng.normal(size=(5, D))
    for inter in (False, True):
        rope = _rope(rot=rot, interleaved=inter)
        for pos in (0, 1, 17, 63):
            y = orc.rope_rotate(x, pos, rope)
            a = x[:, 0:rot:2] if inter else x[:, :rot // 2]
            b = x[:, 1:rot:2] if inter else x[:, rot // 2:rot]
            zc = (a + 1j * b) * (rope.cos[pos] + 1j * rope.sin[pos])       # library complex product
            ya = y[:, 0:rot:2] if inter else y[:, :rot // 2]
            yb = y[:, 1:rot:2] if inter else y[:, rot // 2:rot]
            np.testing.assert_allclose(ya, zc.real, atol=1e-14)
            np.testing.assert_allclose(yb, zc.imag, atol=1e-14)
            np.testing.assert_array_equal(y[:, rot:], x[:, rot:])           # features past rot_dim untouched
            np.testing.assert_allclose(np.linalg.norm(y, axis=1), np.linalg.norm(x, axis=1), rtol=1e-14)
            np.testing.assert_allclose(orc.rope_rotate(y, pos, rope, inverse=True), x, atol=1e-14)
    # quarter turn: (a, b) -> (-b, a)
    quarter = orc.OracleRope(np.zeros((1, 2)), np.ones((1, 2)), False)
    np.testing.assert_allclose(orc.rope_rotate(np.array([1.0, 2.0, 3.0, 4.0]), 0, quarter), [-3.0, -4.0, 1.0, 2.0])
    quarter_i = orc.OracleRope(np.zeros((1, 2)), np.ones((1, 2)), True)
    np.testing.assert_allclose(orc.rope_rotate(np.array([1.0, 2.0, 3.0, 4.0]), 0, quarter_i), [-2.0, 1.0, -4.0, 3.0])


def test_p14_rotated_dot_products_depend_on_the_offset_only():
    rng = np.random.default_rng(1)
    rope = _rope(n_pos=80, rot=8)
    q, k = rng.normal(size=8), rng.normal(size=8)
    ref = float(orc.rope_rotate(q, 30, rope) @ orc.rope_rotate(k, 19, rope))
    for shift in (1, 7, 40):
        assert abs(float(orc.rope_rotate(q, 30 + shift, rope) @ orc.rope_rotate(k, 19 + shift, rope)) - ref) < 1e-12
    assert abs(float(orc.rope_rotate(q, 11, rope) @ k) - ref) < 1e-12


# ---- P15: deferred batched scoring gives what per-step scoring gives ----------------------------
def _lazy_run(w, cfg, cnn, st, q, k, v, rope=None, rounder=None):
    """Drive lazy decode with the paper's trigger; returns the number of batched scorings."""
    calls = 0
    outs = []
    for t in range(len(q)):
        if orc.rescore_due(st, cfg, cnn):
            orc.rescore(st, cfg, cnn, rope, rounder)
            calls += 1
        outs.append(orc.decode_step_lazy(st, q[t], k[t], v[t], cfg))
    return calls, outs


@pytest.mark.parametrize("seed,n0,steps,window,budget,sink,kernel,dil", [(30, 0, 70, 13, 5, 1, (3,), None),
                                                                         (31, 25, 60, 11, 4, 0, (5,), None),
                                                                         (32, 40, 90, 21, 6, 2, (3, 3), (2, 1)),
                                                                         (33, 3, 50, 9, 3, 0, (3, 3), (1, 1))])
def test_p15_lazy_scoring_equals_per_step_scoring(seed, n0, steps, window, budget, sink, kernel, dil):
    ch = (4,) * len(kernel)
    w = small_prefill(seed=seed, seqlens=(n0 + steps,), window=window, budget=budget, sink=sink, kernel=kernel,
                      channels=ch, dilation=dil)
    cfg, cnn = oracle_cfg(w), oracle_cnn(w.cnn)
    def start():
        if n0 == 0:
            return orc.empty_state(cfg)
        return orc.prefill(w.q[:n0], w.k[:n0], w.v[:n0], cfg, cnn, [0, n0])[1][0]
    eager, lazy = start(), start()
    calls = 0
    for t in range(n0, n0 + steps):
        o_e = orc.decode_step(eager, w.q[t], w.k[t], w.v[t], cfg, cnn)
        if orc.rescore_due(lazy, cfg, cnn):
            orc.rescore(lazy, cfg, cnn)
            calls += 1
        o_l = orc.decode_step_lazy(lazy, w.q[t], w.k[t], w.v[t], cfg)
        np.testing.assert_allclose(o_l, o_e, atol=1e-13)
        for h in range(cfg.Hkv):
            assert sorted(lazy.heads[h].ret_pos) == sorted(eager.heads[h].ret_pos), (t, h)
    # the trigger fires once per (window - 2 rho) steps once the window is full
    period = orc.lazy_period(cfg, cnn)
    assert period == window - 2 * cnn.rho
    full_from = max(n0, window)
    expect = (n0 + steps - full_from) / period
    assert abs(calls - expect) <= 1.5, (calls, expect)
    orc.rescore(lazy, cfg, cnn)
    assert lazy.n_scored == eager.n_scored
    for h in range(cfg.Hkv):
        for j, zj in eager.heads[h].win_z.items():
            assert abs(lazy.heads[h].win_z[j] - zj) < 1e-12
    # skipping the batched scoring is noticed
    late = start()
    with pytest.raises(AssertionError):
        for t in range(n0, n0 + steps):
            orc.decode_step_lazy(late, w.q[t], w.k[t], w.v[t], cfg)


# ---- P16: un-rotated cached keys give the scores of the keys before rotation ---------------------
@pytest.mark.parametrize("interleaved", [False, True])
def test_p16_inverse_rope_on_cached_keys_restores_the_scoring_features(interleaved):
    n = 75
    w = small_prefill(seed=40, seqlens=(n,), window=15, budget=5, sink=1, kernel=(3, 3), channels=(4, 4), dilation=(2, 1))
    cfg, cnn = oracle_cfg(w), oracle_cnn(w.cnn)
    rope = _rope(n_pos=n, rot=8, interleaved=interleaved)
    k_pre = np.asarray(w.k, np.float64)
    k_post = np.stack([orc.rope_rotate(k_pre[p], p, rope) for p in range(n)])
    eager = orc.empty_state(cfg)      # scores the keys before rotation, step by step
    lazy = orc.empty_state(cfg)       # holds rotated keys, scores them in batches after rotating back
    for t in range(n):
        orc.decode_step(eager, w.q[t], k_pre[t], w.v[t], cfg, cnn)
        if orc.rescore_due(lazy, cfg, cnn):
            orc.rescore(lazy, cfg, cnn, rope)
        orc.decode_step_lazy(lazy, w.q[t], k_post[t], w.v[t], cfg)
        for h in range(cfg.Hkv):
            assert sorted(lazy.heads[h].ret_pos) == sorted(eager.heads[h].ret_pos), (t, h)
    orc.rescore(lazy, cfg, cnn, rope)
    for h in range(cfg.Hkv):
        assert len(eager.heads[h].win_z) > 0
        for j, zj in eager.heads[h].win_z.items():
            assert abs(lazy.heads[h].win_z[j] - zj) < 1e-10
    # without the inverse rotation, or with it taken at a shifted position, the logits come out different
    for broken in ("none", "shifted"):
        st = orc.empty_state(cfg)
        bad_rope = None if broken == "none" else orc.OracleRope(np.roll(rope.cos, 1, axis=0), np.roll(rope.sin, 1, axis=0), interleaved)
        for t in range(20):
            if orc.rescore_due(st, cfg, cnn):
                orc.rescore(st, cfg, cnn, bad_rope)
            orc.decode_step_lazy(st, w.q[t], k_post[t], w.v[t], cfg)
        orc.rescore(st, cfg, cnn, bad_rope)
        ref = orc.score_sequence(k_pre[:20], np.asarray(w.v[:20], np.float64), cnn)
        got = np.array([[st.heads[h].win_z[j] for j in sorted(st.heads[h].win_z)] for h in range(cfg.Hkv)])
        js = sorted(st.heads[0].win_z)
        assert np.abs(got - ref[:, js]).max() > 1e-4, broken


# ---- planted mistakes: the pins above must notice them ---------------------------------------
def test_pins_catch_planted_mistakes(monkeypatch):
    w = small_prefill(seed=20, seqlens=(40,), window=8, budget=4)
    cfg, cnn = oracle_cfg(w), oracle_cnn(w.cnn)
    good, _, z, kept = orc.prefill(w.q, w.k, w.v, cfg, cnn, w.cu_seqlens)
    keep = [brute_force_keep(orc.selection_key(z[h], 0), 40, 8, 4, 0, 0.0) for h in range(2)]
    ref = dense_masked_attention(w.q, w.k, w.v, keep, 8, cfg.sigma, 1)
    # (a) off-by-one window in the oracle
    cfg_bad = orc.OracleCfg(cfg.Hq, cfg.Hkv, cfg.D, cfg.window + 1, cfg.budget)
    bad = orc.sparse_attention_sequence(w.q, w.k, w.v, cfg_bad, kept[0])
    assert np.abs(bad - ref).max() > 1e-6
    # (b) missing softmax scale
    monkeypatch.setattr(orc, "attend", lambda qv, K, V, s: _unscaled(qv, K, V))
    bad = orc.sparse_attention_sequence(w.q, w.k, w.v, cfg, kept[0])
    assert np.abs(bad - ref).max() > 1e-6
    monkeypatch.undo()
    # (c) mirrored conv taps
    flipped = orc.cnn_from_arrays(cnn.kernel, cnn.dilation, [x[..., ::-1] for x in cnn.w], cnn.bias, cnn.w_out, cnn.b_out)
    assert np.abs(orc.score(w.k, w.v, flipped, w.cu_seqlens) - z).max() > 1e-6
    assert np.abs(good - ref).max() < 1e-12


def _unscaled(qv, K, V):
    s = K @ qv
    p = np.exp(s - s.max())
    return (p / p.sum()) @ V


# ---- P17: training-side forward / backward ---------------------------------------------------
def _train_case(seed=50, n=40, window=9, sink=1, G=2, Hkv=2, D=8):
    w = small_prefill(seed=seed, seqlens=(n,), Hq=Hkv * G, Hkv=Hkv, D=D, window=window, budget=5, sink=sink, kernel=(3,))
    cfg, cnn = oracle_cfg(w), oracle_cnn(w.cnn)
    z = orc.score(w.k, w.v, cnn, w.cu_seqlens) * 20.0          # spread the logits so that both signs occur
    rng = np.random.default_rng(seed + 1)
    dout = rng.normal(size=(n, cfg.Hq, D))
    return w, cfg, z, dout


def test_p17_training_forward_is_the_uncapped_mask_of_eq5():
    w, cfg, z, _ = _train_case()
    out, lse, P = orc.train_forward_sequence(w.q, w.k, w.v, z, cfg)
    n = w.q.shape[0]
    keep = [[j for j in range(n) if j < cfg.sink or np.float32(z[h, j]) > 0] for h in range(cfg.Hkv)]
    assert 0 < len(keep[0]) < n
    ref = dense_masked_attention(w.q, w.k, w.v, keep, cfg.window, cfg.sigma, cfg.G)
    np.testing.assert_allclose(out, ref, atol=1e-12)
    np.testing.assert_allclose(P.sum(axis=2), 1.0, atol=1e-12)
    # equals the inference prefill whenever the cap does not bind (budget >= n)
    big = orc.OracleCfg(cfg.Hq, cfg.Hkv, cfg.D, cfg.window, n, cfg.sink, cfg.tau)
    kept = [orc.retain(z[h], n, cfg.window, n, cfg.sink, cfg.tau) for h in range(cfg.Hkv)]
    np.testing.assert_allclose(out, orc.sparse_attention_sequence(w.q, w.k, w.v, big, kept), atol=1e-12)
    # the normaliser: exp(s - lse) are the probabilities
    s00 = cfg.sigma * (np.asarray(w.q[5, 0], np.float64) @ np.asarray(w.k[5, 0], np.float64))
    assert abs(np.exp(s00 - lse[0, 5]) - P[0, 5, 5]) < 1e-12


def test_p17_backward_matches_library_autograd_and_finite_differences():
    torch = pytest.importorskip("torch")
    w, cfg, z, dout = _train_case()
    lam = np.array([0.3, 0.0])
    dq, dk, dv, dz, c = orc.train_backward_sequence(w.q, w.k, w.v, z, dout, cfg, lam)
    n = w.q.shape[0]
    # library autograd through a dense masked softmax
    tq = torch.tensor(np.asarray(w.q, np.float64), requires_grad=True)
    tk = torch.tensor(np.asarray(w.k, np.float64), requires_grad=True)
    tv = torch.tensor(np.asarray(w.v, np.float64), requires_grad=True)
    i = torch.arange(n)[:, None]; j = torch.arange(n)[None, :]
    loss = 0.0
    for hq in range(cfg.Hq):
        h = hq // cfg.G
        keep = torch.tensor(orc.train_keep_mask(z[h], cfg.sink, cfg.tau))
        allowed = (j <= i) & ((j > i - cfg.window) | keep[None, :])
        s = (tq[:, hq] @ tk[:, h].T) * cfg.sigma
        p = torch.softmax(s.masked_fill(~allowed, float("-inf")), dim=1)
        loss = loss + ((p @ tv[:, h]) * torch.tensor(dout[:, hq])).sum()
    loss.backward()
    np.testing.assert_allclose(dq, tq.grad.numpy(), atol=1e-11)
    np.testing.assert_allclose(dk, tk.grad.numpy(), atol=1e-11)
    np.testing.assert_allclose(dv, tv.grad.numpy(), atol=1e-11)
    # finite differences on the oracle's own forward for a few entries
    def L(q, k, v):
        return float((orc.train_forward_sequence(q, k, v, z, cfg)[0] * dout).sum())
    rng = np.random.default_rng(3)
    base = [np.asarray(x, np.float64) for x in (w.q, w.k, w.v)]
    for which, grad in ((0, dq), (1, dk), (2, dv)):
        for _ in range(4):
            idx = tuple(int(rng.integers(0, s)) for s in base[which].shape)
            hi = [x.copy() for x in base]; lo = [x.copy() for x in base]
            hi[which][idx] += 1e-6; lo[which][idx] -= 1e-6
            assert abs((L(*hi) - L(*lo)) / 2e-6 - grad[idx]) < 1e-6


def test_p17_surrogate_gradient_of_the_retention_score():
    """d(loss)/d r_j is the derivative with respect to a multiplier on v_j (mask held fixed); the penalty adds
    lam_h where the token is active; both pass through the sigmoid's slope."""
    w, cfg, z, dout = _train_case(seed=51)
    lam = np.array([0.25, 0.5])
    dq, dk, dv, dz, c = orc.train_backward_sequence(w.q, w.k, w.v, z, dout, cfg, lam)
    v = np.asarray(w.v, np.float64)
    r = 1.0 / (1.0 + np.exp(-z))
    for (h, j) in ((0, 3), (1, 17), (0, 30), (1, 0)):
        def L(mult):
            v2 = v.copy(); v2[j, h] *= mult
            return float((orc.train_forward_sequence(w.q, w.k, v2, z, cfg)[0] * dout).sum())
        ste = (L(1 + 1e-6) - L(1 - 1e-6)) / 2e-6
        active = 1.0 if np.float32(z[h, j]) > 0 else 0.0
        assert abs(dz[h, j] - (ste + lam[h] * active) * r[h, j] * (1 - r[h, j])) < 1e-7
    np.testing.assert_array_equal(c, (z.astype(np.float32) > 0).sum(axis=1))
    # penalty alone: zero upstream gradient leaves lam * 1[r > 0.5] * r (1 - r)
    *_, dz0, _ = orc.train_backward_sequence(w.q, w.k, w.v, z, np.zeros_like(dout), cfg, lam)
    np.testing.assert_allclose(dz0, lam[:, None] * (z.astype(np.float32) > 0) * r * (1 - r), atol=1e-15)
    # and it is the derivative of sum_h lam_h sum_j ReLU(r_j - 0.5) with respect to z
    pen = lambda zz: float((lam[:, None] * np.maximum(1.0 / (1.0 + np.exp(-zz)) - 0.5, 0.0)).sum())
    zz = z.copy(); h, j = 0, int(np.argmax(z[0])); zz[h, j] += 1e-6
    zl = z.copy(); zl[h, j] -= 1e-6
    assert abs((pen(zz) - pen(zl)) / 2e-6 - dz0[h, j]) < 1e-8
    assert orc.sparsity_threshold(0.0) == 0.5 and orc.sparsity_threshold(-np.inf) == 0.0


def test_p17_penalty_weight_feedback_follows_algorithm_1():
    lam = np.array([1e-9, 0.5, 0.9, 2e-9, 0.0, 0.0, 1e-3])
    cbar = np.array([600.0, 600.0, 600.0, 100.0, 600.0, 100.0, 500.0])       # cap 512: 0.95 cap = 486.4
    got = orc.lambda_update(lam, cbar, 512.0, 2.0)
    # grow x2 (clamped at 1) above the cap, shrink /2 below 0.95 cap (flushed to 0 under 1e-9), restart from 1e-9
    # where it is zero but the count is too high, untouched inside the dead band
    np.testing.assert_allclose(got, [2e-9, 1.0, 1.0, 1e-9, 1e-9, 0.0, 1e-3], rtol=1e-12)
    np.testing.assert_allclose(orc.lambda_update(np.array([1.5e-9]), np.array([10.0]), 512.0, 2.0), [0.0])
    # moving average: coefficient 2 / (1 + u/2)
    np.testing.assert_allclose(orc.ema_count(np.array([100.0]), np.array([200.0]), 32), [2 / 17 * 100 + 15 / 17 * 200])


# --------------------------------------------------------------------------
# P18: backward of the scoring CNN
# --------------------------------------------------------------------------
def _tiny_cnn(rng, Hkv, D, kernel, channels, dilation):
    w, bias, cin = [], [], 2 * D
    for ks, c in zip(kernel, channels):
        w.append(rng.normal(0, 0.3, (Hkv, c, cin, ks)))
        bias.append(rng.normal(0, 0.3, (Hkv, c)))
        cin = c
    return orc.cnn_from_arrays(kernel, dilation, w, bias, rng.normal(0, 0.5, (Hkv, cin)), rng.normal(0, 0.5, (Hkv,)))


def test_p18_cnn_backward_matches_finite_differences():
    """L = sum dz * z with z from the forward oracle; every gradient family is checked by central differences on
    random entries (two sequences, so that the sequence boundary is exercised: no gradient crosses it)."""
    rng = np.random.default_rng(18)
    Hkv, D = 2, 4
    cnn = _tiny_cnn(rng, Hkv, D, (3, 5), (6, 3), (2, 1))
    cu = [0, 9, 14]
    k, v = rng.normal(0, 1, (14, Hkv, D)), rng.normal(0, 1, (14, Hkv, D))
    dz = rng.normal(0, 1, (Hkv, 14))
    loss = lambda: float(np.sum(dz * orc.score(k, v, cnn, cu)))
    dw, dbias, dw_out, db_out, dk, dv = orc.score_backward(k, v, cnn, cu, dz)

    def check(arr, grad, n=12, eps=1e-6):
        for _ in range(n):
            idx = tuple(int(rng.integers(0, s)) for s in arr.shape)
            old = arr[idx]
            arr[idx] = old + eps; up = loss()
            arr[idx] = old - eps; dn = loss()
            arr[idx] = old
            assert abs((up - dn) / (2 * eps) - grad[idx]) <= 1e-6 * max(1.0, abs(grad[idx])), idx

    for l in range(2):
        check(cnn.w[l], dw[l])
        check(cnn.bias[l], dbias[l])
    check(cnn.w_out, dw_out)
    check(cnn.b_out, db_out, n=2)
    check(k, dk)
    check(v, dv)
    # a token of the second sequence does not feel the first sequence's logits
    dz2 = dz.copy(); dz2[:, 9:] = 0.0
    g = orc.score_backward(k, v, cnn, cu, dz2)
    assert np.all(g[4][9:] == 0.0) and np.all(g[5][9:] == 0.0)


def test_p18_cnn_backward_of_a_pointwise_layer_is_the_textbook_rule():
    """kernel 1: the CNN is a per-token MLP.  d w_out = sum_j dz_j * silu(y_j); d bias = sum_j dz_j w_out silu'(y_j);
    d input = W^T (dz_j w_out silu'(y_j)), written out independently of the oracle's loops."""
    rng = np.random.default_rng(181)
    D, n = 3, 7
    cnn = _tiny_cnn(rng, 1, D, (1,), (4,), (1,))
    k, v = rng.normal(0, 1, (n, 1, D)), rng.normal(0, 1, (n, 1, D))
    dz = rng.normal(0, 1, (1, n))
    dw, dbias, dw_out, db_out, dk, dv = orc.score_backward(k, v, cnn, [0, n], dz)
    x = np.concatenate([k[:, 0], v[:, 0]], axis=1)                 # [n, 2D]
    W, b, wo = cnn.w[0][0][:, :, 0], cnn.bias[0][0], cnn.w_out[0]
    y = x @ W.T + b
    sig = 1 / (1 + np.exp(-y))
    dy = dz[0][:, None] * wo[None, :] * (sig * (1 + y * (1 - sig)))
    np.testing.assert_allclose(dw_out[0], dz[0] @ (y * sig), rtol=1e-12)
    np.testing.assert_allclose(dbias[0][0], dy.sum(0), rtol=1e-12)
    np.testing.assert_allclose(dw[0][0][:, :, 0], dy.T @ x, rtol=1e-12)
    np.testing.assert_allclose(np.concatenate([dk[:, 0], dv[:, 0]], axis=1), dy @ W, rtol=1e-12)
    assert abs(db_out[0] - dz.sum()) < 1e-12
