"""Shared test helpers: turn a generated workload into oracle objects.
Test code may import both the generator and the oracle; the product may not."""
import numpy as np

from oracle import ltea_oracle as orc
from paper_2510_20787_amd import workloads as wl


def oracle_cfg(w) -> orc.OracleCfg:
    return orc.OracleCfg(Hq=w.Hq, Hkv=w.Hkv, D=w.D, window=w.window, budget=w.budget, sink=w.sink, tau=w.tau)


def oracle_cnn(c: wl.CnnWeights) -> orc.OracleCnn:
    return orc.cnn_from_arrays(c.kernel, c.dilation, c.w, c.bias, c.w_out, c.b_out)


def small_prefill(seed=0, seqlens=(40,), Hq=2, Hkv=2, D=8, window=12, budget=5, sink=0, tau=0.0,
                  kernel=(3,), channels=(4,), dilation=None, dtype="f32", w_std=0.3, qkv_scale=1.0):
    return wl.make_prefill("small", seed, dtype, list(seqlens), Hq, Hkv, D, window, budget, sink, tau,
                           cnn_kernel=kernel, cnn_channels=channels, cnn_dilation=dilation,
                           qkv_scale=qkv_scale, w_std=w_std)


def brute_force_keep(key32: np.ndarray, n: int, window: int, budget: int, sink: int, tau: float):
    """Independent statement of the capped keep set (eq. 5 + Section 3.1.3): start from every
    out-of-window candidate and throw out the worst (lowest key; among equal keys the latest
    position) until the budget holds."""
    n_out = max(0, n - window)
    cand = [j for j in range(n_out) if j < sink or key32[j] > np.float32(tau)]
    key = [np.float32(np.inf) if j < sink else np.float32(key32[j]) for j in range(n)]
    while len(cand) > budget:
        worst = cand[0]
        for j in cand[1:]:
            if key[j] < key[worst] or (key[j] == key[worst] and j > worst):
                worst = j
        cand.remove(worst)
    return sorted(cand)


def dense_masked_attention(q, k, v, keep, window, sigma, G):
    """Brute force from the index set of eq. 5: an n x n mask, allowed(i, j) iff j <= i and
    (j in the window of i, or j kept). Dense softmax in fp64."""
    q = np.asarray(q, np.float64); k = np.asarray(k, np.float64); v = np.asarray(v, np.float64)
    n, Hq, D = q.shape
    out = np.zeros_like(q)
    i = np.arange(n)[:, None]
    j = np.arange(n)[None, :]
    for hq in range(Hq):
        h = hq // G
        flag = np.zeros(n, dtype=bool)
        flag[np.asarray(keep[h], dtype=np.int64)] = True
        allowed = (j <= i) & ((j > i - window) | flag[None, :])
        s = sigma * (q[:, hq, :] @ k[:, h, :].T)
        s = np.where(allowed, s, -np.inf)
        s = s - s.max(axis=1, keepdims=True)
        p = np.exp(s)
        p /= p.sum(axis=1, keepdims=True)
        out[:, hq, :] = p @ v[:, h, :]
    return out
