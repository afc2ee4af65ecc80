"""CPU oracle for the SWA+LTE token mixer: TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 NumPy statement of what the hot path computes, written
from the paper. It shares no code with the HIP path, is never imported by the
product package, and is only used by tests, the smoke check and the bench's
CPU-baseline leg.

Conventions (0-based positions inside one sequence of length n):
  * window w counts the current token: query i sees positions i-w+1 .. i
    (Section 2.1's sliding-window pattern; the cache holds the last w KVs,
    Section 3.1.3 "Cached prefilling and decoding").
  * token j is a retention candidate once it is out of the window, if it is a
    sink (j < s) or its retention score exceeds 0.5, i.e. its logit z_j > tau
    with tau = 0 (Section 3.1.1, eq. 5).  At most b candidates per head are
    kept; on overflow the b highest-scoring ones (Section 3.1.3 "Capped
    capacity").  Ties are ordered by (key descending, position ascending);
    sinks carry key +inf.
  * selection compares logits in fp32 (the precision the kernels produce them
    in); everything else is fp64.

Every function cites the passage of the paper it follows.

Pins (tests/test_oracle_pins.py): dense masked softmax built from eq. 5,
special cases b=0 / w>=n, budget invariants, streaming-vs-batch retention,
prefill-vs-decode agreement when the cap does not bind, a library grouped
convolution, closed forms for the CNN and the softmax, packing and GQA
invariants; for the lazy path: complex multiplication and the relative-position
identity for the rotation, deferred == per-step scoring, and un-rotated cached
keys reproducing the scores of the unrotated ones.  No value printed by the
paper exists for this mechanism.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np

NEG_INF = -np.inf


# --------------------------------------------------------------------------
# parameters
# --------------------------------------------------------------------------
@dataclass
class OracleCnn:
    """Per-KV-head 1-D CNN of the LTE module (Section 3.1.1; Appendix A).
    w[l]: [Hkv, C_out, C_in, kernel]; bias[l]: [Hkv, C_out]; w_out: [Hkv, C_last]; b_out: [Hkv]."""
    kernel: List[int]
    dilation: List[int]
    w: List[np.ndarray]
    bias: List[np.ndarray]
    w_out: np.ndarray
    b_out: np.ndarray

    @property
    def rho(self) -> int:
        return sum(d * (k - 1) // 2 for k, d in zip(self.kernel, self.dilation))


@dataclass
class OracleCfg:
    Hq: int
    Hkv: int
    D: int
    window: int
    budget: int
    sink: int = 0
    tau: float = 0.0
    scale: Optional[float] = None   # None -> D**-0.5 (Section 2.1)

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def sigma(self) -> float:
        return float(self.D) ** -0.5 if self.scale is None else float(self.scale)


def cnn_from_arrays(kernel, dilation, w, bias, w_out, b_out) -> OracleCnn:
    return OracleCnn(list(kernel), list(dilation),
                     [np.asarray(x, dtype=np.float64) for x in w],
                     [np.asarray(x, dtype=np.float64) for x in bias],
                     np.asarray(w_out, dtype=np.float64), np.asarray(b_out, dtype=np.float64))


# --------------------------------------------------------------------------
# O1: scoring CNN (Section 3.1.1 "LTE module"; Appendix A)
# --------------------------------------------------------------------------
def silu(x: np.ndarray) -> np.ndarray:
    """Swish with beta = 1."""
    return x / (1.0 + np.exp(-x))


def score_sequence(k_seq: np.ndarray, v_seq: np.ndarray, cnn: OracleCnn) -> np.ndarray:
    """Logits z[h, j] for one sequence. k_seq, v_seq: [n, Hkv, D].

    Input features are concat(key, value) per head (keys first).  Each conv is
    a cross-correlation: tap t reads position j + (t - (kernel-1)/2)*dilation;
    positions outside [0, n) contribute zero at every layer.  Swish follows
    each conv; a per-head linear map gives the scalar logit, whose sigmoid is
    the retention score r."""
    k_seq = np.asarray(k_seq, dtype=np.float64)
    v_seq = np.asarray(v_seq, dtype=np.float64)
    n, Hkv, _ = k_seq.shape
    z = np.zeros((Hkv, n), dtype=np.float64)
    for h in range(Hkv):
        a = np.concatenate([k_seq[:, h, :], v_seq[:, h, :]], axis=1)      # [n, 2D]
        for l, (ks, dil) in enumerate(zip(cnn.kernel, cnn.dilation)):
            W = cnn.w[l][h]                                               # [C_out, C_in, ks]
            y = np.tile(cnn.bias[l][h][None, :], (n, 1))                  # [n, C_out]
            for t in range(ks):
                off = (t - (ks - 1) // 2) * dil
                lo, hi = max(0, -off), min(n, n - off)                    # rows j with 0 <= j+off < n
                if hi > lo:
                    y[lo:hi] += a[lo + off:hi + off] @ W[:, :, t].T
            a = silu(y)
        z[h] = a @ cnn.w_out[h] + cnn.b_out[h]
    return z


def score(k: np.ndarray, v: np.ndarray, cnn: OracleCnn, cu_seqlens: Sequence[int]) -> np.ndarray:
    """Logits [Hkv, T] for packed sequences; the conv never crosses a sequence boundary."""
    T, Hkv, _ = k.shape
    z = np.zeros((Hkv, T), dtype=np.float64)
    for s in range(len(cu_seqlens) - 1):
        lo, hi = int(cu_seqlens[s]), int(cu_seqlens[s + 1])
        if hi > lo:
            z[:, lo:hi] = score_sequence(k[lo:hi], v[lo:hi], cnn)
    return z


def retention_score(z: np.ndarray) -> np.ndarray:
    """r = sigmoid(z) (Section 3.1.1)."""
    return 1.0 / (1.0 + np.exp(-np.asarray(z, dtype=np.float64)))


# --------------------------------------------------------------------------
# O2: retention under a cap (eq. 5; Section 3.1.3 "Capped capacity")
# --------------------------------------------------------------------------
def selection_key(z_head: np.ndarray, sink: int) -> np.ndarray:
    """fp32 logits with sinks lifted to +inf."""
    key = np.asarray(z_head, dtype=np.float32).copy()
    key[:sink] = np.inf
    return key


def retain(z_head: np.ndarray, n: int, window: int, budget: int, sink: int = 0, tau: float = 0.0) -> np.ndarray:
    """Positions kept outside the window after n tokens, ascending.

    Evictable positions are 0 .. n-window-1.  Candidates: sinks, or logit >
    tau (NaN never passes).  Keep the first `budget` in the order
    (key descending, position ascending)."""
    n_out = max(0, n - window)
    key = selection_key(z_head[:n], sink)
    tau32 = np.float32(tau)
    cand = [j for j in range(n_out) if (j < sink) or (key[j] > tau32)]
    cand.sort(key=lambda j: (-float(key[j]), j))
    kept = cand[:max(0, budget)]
    return np.array(sorted(kept), dtype=np.int64)


# --------------------------------------------------------------------------
# attention of one query over an explicit index set (Section 2.1)
# --------------------------------------------------------------------------
def attend(qv: np.ndarray, K: np.ndarray, V: np.ndarray, sigma: float) -> np.ndarray:
    """softmax(sigma * K qv) V over the rows of K, V (fp64, max-subtracted)."""
    s = sigma * (K @ qv)
    p = np.exp(s - np.max(s))
    return (p / np.sum(p)) @ V


# --------------------------------------------------------------------------
# O3: prefill outputs for given retained sets (Section 3.1.3)
# --------------------------------------------------------------------------
def attention_row(q_seq, k_seq, v_seq, cfg: OracleCfg, retained_h: np.ndarray, i: int, hq: int) -> np.ndarray:
    """Output of query i, query head hq: attention over its window i-w+1..i plus the kept positions
    j <= i-w of its KV head (kept entries still inside the window are not counted twice)."""
    h = hq // cfg.G
    R = np.asarray(retained_h, dtype=np.int64)
    lo = max(0, i - cfg.window + 1)
    far = R[R <= i - cfg.window]
    idx = np.concatenate([far, np.arange(lo, i + 1)])
    return attend(np.asarray(q_seq[i, hq], dtype=np.float64), np.asarray(k_seq[idx, h], dtype=np.float64),
                  np.asarray(v_seq[idx, h], dtype=np.float64), cfg.sigma)


def sparse_attention_sequence(q_seq, k_seq, v_seq, cfg: OracleCfg, retained: List[np.ndarray]) -> np.ndarray:
    """q_seq [n,Hq,D], k_seq/v_seq [n,Hkv,D], retained[h] = ascending kept positions of KV head h."""
    q_seq = np.asarray(q_seq, dtype=np.float64)
    k_seq = np.asarray(k_seq, dtype=np.float64)
    v_seq = np.asarray(v_seq, dtype=np.float64)
    n = q_seq.shape[0]
    out = np.zeros((n, cfg.Hq, cfg.D), dtype=np.float64)
    for hq in range(cfg.Hq):
        for i in range(n):
            out[i, hq] = attention_row(q_seq, k_seq, v_seq, cfg, retained[hq // cfg.G], i, hq)
    return out


# --------------------------------------------------------------------------
# O4: cache state (Section 3.1.3, cache-layout figure)
# --------------------------------------------------------------------------
@dataclass
class HeadState:
    """State of one (sequence, KV head). Physical order is not part of the
    contract; entries are kept as position-tagged records."""
    win_pos: List[int] = field(default_factory=list)        # positions in the window, ascending
    win_k: List[np.ndarray] = field(default_factory=list)
    win_v: List[np.ndarray] = field(default_factory=list)
    win_z: dict = field(default_factory=dict)               # position -> final fp64 logit (only final ones)
    ret_pos: List[int] = field(default_factory=list)
    ret_key: List[np.float32] = field(default_factory=list)  # fp32 selection key (+inf for sinks)
    ret_k: List[np.ndarray] = field(default_factory=list)
    ret_v: List[np.ndarray] = field(default_factory=list)


@dataclass
class SeqState:
    heads: List[HeadState]
    n_seen: int = 0
    n_scored: int = 0


def empty_state(cfg: OracleCfg) -> SeqState:
    return SeqState([HeadState() for _ in range(cfg.Hkv)], 0, 0)


def state_after_prefill(k_seq, v_seq, z_seq, cfg: OracleCfg, rho: int, retained: List[np.ndarray]) -> SeqState:
    """Window = last min(n, w) tokens with the logits that are already final
    (j + rho <= n-1); retained segment = the kept out-of-window positions."""
    k_seq = np.asarray(k_seq, dtype=np.float64)
    v_seq = np.asarray(v_seq, dtype=np.float64)
    n = k_seq.shape[0]
    st = empty_state(cfg)
    st.n_seen = n
    st.n_scored = max(0, n - rho)
    for h in range(cfg.Hkv):
        hs = st.heads[h]
        key = selection_key(z_seq[h], cfg.sink)
        for j in range(max(0, n - cfg.window), n):
            hs.win_pos.append(j)
            hs.win_k.append(k_seq[j, h].copy())
            hs.win_v.append(v_seq[j, h].copy())
            if j < st.n_scored:
                hs.win_z[j] = float(z_seq[h, j])
        for j in retained[h]:
            j = int(j)
            hs.ret_pos.append(j)
            hs.ret_key.append(key[j])
            hs.ret_k.append(k_seq[j, h].copy())
            hs.ret_v.append(v_seq[j, h].copy())
    return st


def prefill(q, k, v, cfg: OracleCfg, cnn: OracleCnn, cu_seqlens: Sequence[int]):
    """O1 + O2 + O3 + O4 for packed sequences.
    Returns (out [T,Hq,D] fp64, states [n_seqs], logits [Hkv,T] fp64, retained[s][h])."""
    assert cfg.window >= 2 * cnn.rho + 1, "window must cover the CNN receptive field (w >> R)"
    T = q.shape[0]
    z = score(k, v, cnn, cu_seqlens)
    out = np.zeros((T, cfg.Hq, cfg.D), dtype=np.float64)
    states, kept_all = [], []
    for s in range(len(cu_seqlens) - 1):
        lo, hi = int(cu_seqlens[s]), int(cu_seqlens[s + 1])
        n = hi - lo
        kept = [retain(z[h, lo:hi], n, cfg.window, cfg.budget, cfg.sink, cfg.tau) for h in range(cfg.Hkv)]
        if n > 0:
            out[lo:hi] = sparse_attention_sequence(q[lo:hi], k[lo:hi], v[lo:hi], cfg, kept)
        states.append(state_after_prefill(k[lo:hi], v[lo:hi], z[:, lo:hi], cfg, cnn.rho, kept))
        kept_all.append(kept)
    return out, states, z, kept_all


# --------------------------------------------------------------------------
# O5: one decode step (Section 3.1.3: cache replacement; lazy scoring)
# --------------------------------------------------------------------------
def _score_from_window(hs: HeadState, h: int, j: int, cnn: OracleCnn) -> float:
    """Final logit of position j from the window's records: the CNN applied to
    positions j-rho .. j+rho (all inside the window or before position 0)."""
    rho = cnn.rho
    first = hs.win_pos[0]
    lo, hi = j - rho, j + rho
    assert hi <= hs.win_pos[-1] and (lo >= first or first == 0), "receptive field must be in the window"
    rows_k, rows_v = [], []
    for p in range(max(lo, 0), hi + 1):
        rows_k.append(hs.win_k[p - first])
        rows_v.append(hs.win_v[p - first])
    kk = np.stack(rows_k)[:, None, :]
    vv = np.stack(rows_v)[:, None, :]
    sub = OracleCnn(cnn.kernel, cnn.dilation, [w[h:h + 1] for w in cnn.w], [b[h:h + 1] for b in cnn.bias],
                    cnn.w_out[h:h + 1], cnn.b_out[h:h + 1])
    zz = score_sequence(kk, vv, sub)[0]
    # The slice starts at max(lo,0): when lo >= 0 the slice's own left padding is
    # never reached by position j (it sits rho rows in); when lo < 0 the zero
    # padding is the sequence's real left edge.
    return float(zz[j - max(lo, 0)])


def evict_into_retained(hs: HeadState, e: int, z_e: float, ek, ev, cfg: OracleCfg) -> None:
    """Position e has just left the window with final logit z_e (Section 3.1.3, cache replacement): if it is a
    candidate, append it to the retained segment, or, when that is full, let it displace the lowest-key entry
    (among equal lowest keys the latest position) iff its own key is strictly higher. Decisions in fp32."""
    ze = np.float32(z_e)
    ekey = np.float32(np.inf) if e < cfg.sink else ze
    if cfg.budget <= 0 or not (e < cfg.sink or ze > np.float32(cfg.tau)):
        return
    if len(hs.ret_pos) < cfg.budget:
        hs.ret_pos.append(e); hs.ret_key.append(ekey); hs.ret_k.append(ek); hs.ret_v.append(ev)
        return
    m = 0
    for i in range(1, len(hs.ret_pos)):
        if (hs.ret_key[i] < hs.ret_key[m]) or (hs.ret_key[i] == hs.ret_key[m] and hs.ret_pos[i] > hs.ret_pos[m]):
            m = i
    if ekey > hs.ret_key[m]:
        hs.ret_pos[m] = e; hs.ret_key[m] = ekey; hs.ret_k[m] = ek; hs.ret_v[m] = ev


def decode_step(st: SeqState, q_t, k_t, v_t, cfg: OracleCfg, cnn: OracleCnn) -> np.ndarray:
    """Consume token t = st.n_seen of one sequence. q_t [Hq,D], k_t/v_t [Hkv,D]. Returns o_t [Hq,D].

    Order: push the new KV; give final logits to every position whose right
    context is now complete; pop the token that left the window and, if it is
    a candidate, append it to the retained segment or let it displace the
    lowest-key entry when it scores strictly higher (among equal lowest keys
    the latest position goes); then attend over window + retained."""
    assert cfg.window >= 2 * cnn.rho + 1
    q_t = np.asarray(q_t, dtype=np.float64)
    k_t = np.asarray(k_t, dtype=np.float64)
    v_t = np.asarray(v_t, dtype=np.float64)
    t = st.n_seen
    rho = cnn.rho
    out = np.zeros((cfg.Hq, cfg.D), dtype=np.float64)
    for h in range(cfg.Hkv):
        hs = st.heads[h]
        hs.win_pos.append(t)
        hs.win_k.append(k_t[h].copy())
        hs.win_v.append(v_t[h].copy())
        for j in range(st.n_scored, t - rho + 1):
            hs.win_z[j] = _score_from_window(hs, h, j, cnn)
        if len(hs.win_pos) > cfg.window:
            e = hs.win_pos.pop(0)
            ek, ev = hs.win_k.pop(0), hs.win_v.pop(0)
            evict_into_retained(hs, e, hs.win_z.pop(e), ek, ev, cfg)
        K = np.stack(hs.ret_k + hs.win_k)
        V = np.stack(hs.ret_v + hs.win_v)
        for g in range(cfg.G):
            hq = h * cfg.G + g
            out[hq] = attend(q_t[hq], K, V, cfg.sigma)
    st.n_seen = t + 1
    st.n_scored = max(st.n_scored, t - rho + 1, 0)
    return out


def retained_positions(st: SeqState) -> List[np.ndarray]:
    return [np.array(sorted(hs.ret_pos), dtype=np.int64) for hs in st.heads]


def window_positions(st: SeqState) -> List[np.ndarray]:
    return [np.array(sorted(hs.win_pos), dtype=np.int64) for hs in st.heads]


# --------------------------------------------------------------------------
# O6: rotary encoding from cached sinusoids and its inverse (Section 3.1.3 "Lazy scoring")
# --------------------------------------------------------------------------
@dataclass
class OracleRope:
    """cos, sin: [n_pos, rot_dim/2] tables the model rotates its keys with (row = position).  Pair i of a
    vector x is (x[i], x[i + rot_dim/2]), or (x[2i], x[2i+1]) when interleaved; features from rot_dim on are
    not rotated."""
    cos: np.ndarray
    sin: np.ndarray
    interleaved: bool = False

    @property
    def rot_dim(self) -> int:
        return 2 * self.cos.shape[1]


def rope_rotate(x: np.ndarray, pos: int, rope: OracleRope, inverse: bool = False) -> np.ndarray:
    """Rotate every pair (a, b) of x [..., D] by the angle of table row `pos`:
    (a, b) -> (a cos - b sin, a sin + b cos).  The inverse is the same rotation with the sines negated,
    which is how the cached post-rotation keys are turned back into scoring features."""
    x = np.asarray(x, dtype=np.float64)
    c = np.asarray(rope.cos[pos], dtype=np.float64)
    s = np.asarray(rope.sin[pos], dtype=np.float64)
    if inverse:
        s = -s
    r = rope.rot_dim
    out = x.copy()
    if rope.interleaved:
        a, b = x[..., 0:r:2], x[..., 1:r:2]
        out[..., 0:r:2] = a * c - b * s
        out[..., 1:r:2] = a * s + b * c
    else:
        a, b = x[..., :r // 2], x[..., r // 2:r]
        out[..., :r // 2] = a * c - b * s
        out[..., r // 2:r] = a * s + b * c
    return out


# --------------------------------------------------------------------------
# O7: deferred, batched scoring during decode (Section 3.1.3 "Lazy scoring")
# --------------------------------------------------------------------------
def lazy_period(cfg: OracleCfg, cnn: OracleCnn) -> int:
    """Decode steps that may pass between two batched scorings: window minus the receptive field's reach on
    both sides."""
    return cfg.window - 2 * cnn.rho


def rescore_due(st: SeqState, cfg: OracleCfg, cnn: OracleCnn) -> bool:
    """True when the next token would push out of the window a position that the oldest unscored token's
    receptive field still needs (N - w = j - rho in the paper's notation, or already past it)."""
    leaving = st.n_seen - cfg.window
    return leaving >= 0 and st.n_scored - cnn.rho <= leaving


def rescore(st: SeqState, cfg: OracleCfg, cnn: OracleCnn, rope: Optional[OracleRope] = None, round_features=None) -> None:
    """Give final logits to all positions n_scored .. n_seen-rho-1 at once from the window's records.  With
    `rope` the cached keys are post-rotation and are rotated back (negated sines, each at its own position)
    before the CNN sees them; `round_features` (a function on arrays) models the storage precision the
    un-rotated keys are held in."""
    rho, n = cnn.rho, st.n_seen
    first_new, end_new = st.n_scored, n - rho
    if end_new <= first_new:
        return
    lo = max(0, first_new - rho)
    for h, hs in enumerate(st.heads):
        first = hs.win_pos[0]
        assert lo >= first, "the receptive field of the oldest unscored token has left the window"
        feats = []
        for p in range(lo, n):
            kp = hs.win_k[p - first]
            if rope is not None:
                kp = rope_rotate(kp, p, rope, inverse=True)
                if round_features is not None:
                    kp = round_features(kp)
            feats.append(kp)
        kk = np.stack(feats)[:, None, :]
        vv = np.stack([hs.win_v[p - first] for p in range(lo, n)])[:, None, :]
        sub = OracleCnn(cnn.kernel, cnn.dilation, [w[h:h + 1] for w in cnn.w], [b[h:h + 1] for b in cnn.bias],
                        cnn.w_out[h:h + 1], cnn.b_out[h:h + 1])
        zz = score_sequence(kk, vv, sub)[0]
        # the slice's left edge is either the sequence start (lo == 0: real zero padding) or rho rows before
        # the first position that is read out; its right edge is the newest token, rho rows past the last one
        for j in range(first_new, end_new):
            hs.win_z[j] = float(zz[j - lo])
    st.n_scored = end_new


def decode_step_lazy(st: SeqState, q_t, k_t, v_t, cfg: OracleCfg) -> np.ndarray:
    """decode_step without the scoring: the token that leaves the window must already hold a final logit
    (rescore() was called in time)."""
    q_t = np.asarray(q_t, dtype=np.float64)
    k_t = np.asarray(k_t, dtype=np.float64)
    v_t = np.asarray(v_t, dtype=np.float64)
    t = st.n_seen
    out = np.zeros((cfg.Hq, cfg.D), dtype=np.float64)
    for h in range(cfg.Hkv):
        hs = st.heads[h]
        hs.win_pos.append(t)
        hs.win_k.append(k_t[h].copy())
        hs.win_v.append(v_t[h].copy())
        if len(hs.win_pos) > cfg.window:
            e = hs.win_pos.pop(0)
            ek, ev = hs.win_k.pop(0), hs.win_v.pop(0)
            assert e < st.n_scored, "token leaves the window before it was scored"
            evict_into_retained(hs, e, hs.win_z.pop(e), ek, ev, cfg)
        K = np.stack(hs.ret_k + hs.win_k)
        V = np.stack(hs.ret_v + hs.win_v)
        for g in range(cfg.G):
            hq = h * cfg.G + g
            out[hq] = attend(q_t[hq], K, V, cfg.sigma)
    st.n_seen = t + 1
    return out


# --------------------------------------------------------------------------
# O8: training-side forward and backward (Section 3.1.2 "Adaptive training"; Algorithm 1)
# --------------------------------------------------------------------------
def train_keep_mask(z_head: np.ndarray, sink: int, tau: float) -> np.ndarray:
    """Uncapped eq. 5: token j stays visible after it has left a query's window iff it is a sink or its fp32
    logit exceeds tau (no budget during training)."""
    z32 = np.asarray(z_head, dtype=np.float32)
    keep = z32 > np.float32(tau)
    keep[:sink] = True
    return keep


def train_forward_sequence(q_seq, k_seq, v_seq, z_seq, cfg: OracleCfg):
    """Masked attention of one sequence as used in training: query i sees j <= i with j > i-w, or kept j.
    Returns (out [n,Hq,D], lse [Hq,n] natural-log normaliser of the scaled scores, P [Hq,n,n])."""
    q = np.asarray(q_seq, np.float64); k = np.asarray(k_seq, np.float64); v = np.asarray(v_seq, np.float64)
    n = q.shape[0]
    i = np.arange(n)[:, None]
    j = np.arange(n)[None, :]
    out = np.zeros((n, cfg.Hq, cfg.D)); lse = np.zeros((cfg.Hq, n)); P = np.zeros((cfg.Hq, n, n))
    for hq in range(cfg.Hq):
        h = hq // cfg.G
        keep = train_keep_mask(z_seq[h], cfg.sink, cfg.tau)
        allowed = (j <= i) & ((j > i - cfg.window) | keep[None, :])
        s = np.where(allowed, cfg.sigma * (q[:, hq] @ k[:, h].T), NEG_INF)
        m = s.max(axis=1, keepdims=True)
        e = np.exp(s - m)
        l = e.sum(axis=1, keepdims=True)
        P[hq] = e / l
        lse[hq] = (m + np.log(l))[:, 0]
        out[:, hq] = P[hq] @ v[:, h]
    return out, lse, P


def sparsity_threshold(tau: float) -> float:
    """Retention score at the logit threshold (0.5 for tau = 0)."""
    return 0.0 if tau == NEG_INF else 1.0 / (1.0 + np.exp(-float(tau)))


def train_backward_sequence(q_seq, k_seq, v_seq, z_seq, dout, cfg: OracleCfg, lam: np.ndarray):
    """Gradients of a loss with d(loss)/d(out) = dout through train_forward_sequence, plus the surrogate gradient
    of the retention scores: d(loss)/d r_j := <v_j, d(loss)/d v_j> (straight-through estimator on a conceptual
    mask multiplying v_j), and the gradient of the sparsity penalty sum_h lam_h sum_j ReLU(r_j - r_tau).  Both
    reach the logits through r = sigmoid(z).  Returns dq [n,Hq,D], dk, dv [n,Hkv,D], dz [Hkv,n] and the
    retention counts c [Hkv] = #{j : r_j > r_tau}."""
    q = np.asarray(q_seq, np.float64); k = np.asarray(k_seq, np.float64); v = np.asarray(v_seq, np.float64)
    do = np.asarray(dout, np.float64)
    n = q.shape[0]
    out, lse, P = train_forward_sequence(q, k, v, z_seq, cfg)
    dq = np.zeros_like(q); dk = np.zeros_like(k); dv = np.zeros_like(v)
    for hq in range(cfg.Hq):
        h = hq // cfg.G
        dv[:, h] += P[hq].T @ do[:, hq]
        dP = do[:, hq] @ v[:, h].T
        delta = np.sum(do[:, hq] * out[:, hq], axis=1, keepdims=True)
        dS = P[hq] * (dP - delta)
        dq[:, hq] = cfg.sigma * (dS @ k[:, h])
        dk[:, h] += cfg.sigma * (dS.T @ q[:, hq])
    z = np.asarray(z_seq, np.float64)
    r = retention_score(z)
    active = np.asarray(z_seq, np.float32) > np.float32(cfg.tau)       # r > r_tau, decided on the fp32 logit
    g_r = np.einsum("nhd,nhd->hn", v, dv) + np.asarray(lam, np.float64)[:, None] * active
    dz = g_r * r * (1.0 - r)
    return dq, dk, dv, dz, active.sum(axis=1).astype(np.int64)


def ema_count(c_bar: np.ndarray, c: np.ndarray, u: int) -> np.ndarray:
    """Moving average of the retention counts with coefficient 2 / (1 + u/2) (Appendix, training details)."""
    a = 2.0 / (1.0 + u / 2.0)
    return a * np.asarray(c_bar, np.float64) + (1.0 - a) * np.asarray(c, np.float64)


def lambda_update(lam: np.ndarray, c_bar: np.ndarray, cap: float, alpha: float) -> np.ndarray:
    """Feedback step on the penalty weights (Algorithm 1): grow by alpha where the averaged count exceeds the cap,
    shrink where it is below 0.95 cap, clamp to <= 1, flush values below 1e-9 to zero, and restart from 1e-9
    where the count is too high while the weight is zero."""
    lam = np.asarray(lam, np.float64).copy()
    c_bar = np.asarray(c_bar, np.float64)
    s = (c_bar > cap).astype(np.float64) - (c_bar < 0.95 * cap).astype(np.float64)
    lam = lam * alpha ** s
    lam = np.minimum(lam, 1.0)
    lam[lam < 1e-9] = 0.0
    lam[(c_bar > cap) & (lam == 0.0)] = 1e-9
    return lam


# --------------------------------------------------------------------------
# O9: backward of the scoring CNN (Section 3.1.1 module, trained through the gradient of Section 3.1.2)
# --------------------------------------------------------------------------
def silu_grad(y: np.ndarray) -> np.ndarray:
    """d/dy of y * sigmoid(y)."""
    s = 1.0 / (1.0 + np.exp(-y))
    return s * (1.0 + y * (1.0 - s))


def score_backward_sequence(k_seq: np.ndarray, v_seq: np.ndarray, cnn: OracleCnn, dz_seq: np.ndarray):
    """Gradients of L = sum_{h,j} dz[h, j] * z[h, j] for one sequence, z = score_sequence(k_seq, v_seq, cnn).
    Returns (dw list [Hkv, C_out, C_in, kernel], dbias list [Hkv, C_out], dw_out [Hkv, C_last], db_out [Hkv],
    dk [n, Hkv, D], dv [n, Hkv, D]).  The chain rule through the layers of score_sequence, in reverse order."""
    k_seq = np.asarray(k_seq, dtype=np.float64)
    v_seq = np.asarray(v_seq, dtype=np.float64)
    n, Hkv, D = k_seq.shape
    L = len(cnn.kernel)
    dw = [np.zeros_like(w) for w in cnn.w]
    dbias = [np.zeros_like(b) for b in cnn.bias]
    dw_out, db_out = np.zeros_like(cnn.w_out), np.zeros_like(cnn.b_out)
    dk, dv = np.zeros_like(k_seq), np.zeros_like(v_seq)
    for h in range(Hkv):
        acts = [np.concatenate([k_seq[:, h, :], v_seq[:, h, :]], axis=1)]       # inputs of each layer
        pre = []                                                                # pre-activations of each layer
        for l, (ks, dil) in enumerate(zip(cnn.kernel, cnn.dilation)):
            W = cnn.w[l][h]
            y = np.tile(cnn.bias[l][h][None, :], (n, 1))
            for t in range(ks):
                off = (t - (ks - 1) // 2) * dil
                lo, hi = max(0, -off), min(n, n - off)
                if hi > lo:
                    y[lo:hi] += acts[l][lo + off:hi + off] @ W[:, :, t].T
            pre.append(y)
            acts.append(silu(y))
        g = np.asarray(dz_seq[h], dtype=np.float64)                             # [n]
        dw_out[h] = g @ acts[L]
        db_out[h] = g.sum()
        da = g[:, None] * cnn.w_out[h][None, :]                                 # d L / d output of the last layer
        for l in reversed(range(L)):
            ks, dil = cnn.kernel[l], cnn.dilation[l]
            W = cnn.w[l][h]
            dy = da * silu_grad(pre[l])                                         # [n, C_out]
            dbias[l][h] = dy.sum(axis=0)
            da_prev = np.zeros_like(acts[l])
            for t in range(ks):
                off = (t - (ks - 1) // 2) * dil
                lo, hi = max(0, -off), min(n, n - off)
                if hi > lo:
                    dw[l][h][:, :, t] = dy[lo:hi].T @ acts[l][lo + off:hi + off]
                    da_prev[lo + off:hi + off] += dy[lo:hi] @ W[:, :, t]
            da = da_prev
        dk[:, h, :] = da[:, :D]
        dv[:, h, :] = da[:, D:]
    return dw, dbias, dw_out, db_out, dk, dv


def score_backward(k: np.ndarray, v: np.ndarray, cnn: OracleCnn, cu_seqlens: Sequence[int], dz: np.ndarray):
    """score_backward_sequence over packed sequences: weight gradients summed over the sequences."""
    T, Hkv, D = k.shape
    dw = [np.zeros_like(w) for w in cnn.w]
    dbias = [np.zeros_like(b) for b in cnn.bias]
    dw_out, db_out = np.zeros_like(cnn.w_out), np.zeros_like(cnn.b_out)
    dk, dv = np.zeros((T, Hkv, D)), np.zeros((T, Hkv, D))
    for s in range(len(cu_seqlens) - 1):
        lo, hi = int(cu_seqlens[s]), int(cu_seqlens[s + 1])
        if hi > lo:
            g = score_backward_sequence(k[lo:hi], v[lo:hi], cnn, np.asarray(dz)[:, lo:hi])
            for l in range(len(dw)):
                dw[l] += g[0][l]
                dbias[l] += g[1][l]
            dw_out += g[2]
            db_out += g[3]
            dk[lo:hi], dv[lo:hi] = g[4], g[5]
    return dw, dbias, dw_out, db_out, dk, dv
