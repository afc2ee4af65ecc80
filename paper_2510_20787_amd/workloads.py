"""Seeded synthetic inputs for the SWA+LTE token mixer (host side, NumPy only).

This module draws random numbers and rounds them to the storage type; it holds
none of the method's arithmetic (no convolution, no selection, no attention).
Both the CPU oracle's tests and the GPU path's tests/bench read their inputs
from here, so the two sides see identical bits.

All floating arrays are returned as float32 whose values are exactly
representable in the workload's storage dtype ("f32" or "bf16"): widening them
to fp64 (oracle) or narrowing them to bf16 (GPU) is lossless.

Shapes follow the packed-token convention: Q is [T, Hq, D], K and V are
[T, Hkv, D] with T = cu_seqlens[-1]; conv weights are
[Hkv, C_out, C_in, kernel] with C_in(layer 0) = 2*D (K channels first, then V).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence

import numpy as np


# --------------------------------------------------------------------------
# storage rounding
# --------------------------------------------------------------------------
def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); result is
    float32 holding bf16-representable values. NaN/Inf pass through."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    special = (u & np.uint32(0x7F800000)) == np.uint32(0x7F800000)
    r = np.where(special, u & np.uint32(0xFFFF0000) | ((u & np.uint32(0x007FFFFF)) != 0) * np.uint32(0x00400000), r)
    return r.astype(np.uint32).view(np.float32).reshape(x.shape)


def to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "bf16":
        return round_to_bf16(x)
    raise ValueError(f"unknown dtype {dtype!r}")


# --------------------------------------------------------------------------
# containers
# --------------------------------------------------------------------------
@dataclass
class CnnWeights:
    """Scoring CNN parameters for every KV head (plain arrays, no arithmetic)."""
    kernel: List[int]
    dilation: List[int]
    c_out: List[int]
    w: List[np.ndarray]          # per layer [Hkv, C_out, C_in, kernel] float32 (storage-rounded)
    bias: List[np.ndarray]       # per layer [Hkv, C_out] float32
    w_out: np.ndarray            # [Hkv, C_last] float32 (storage-rounded)
    b_out: np.ndarray            # [Hkv] float32

    @property
    def n_layers(self) -> int:
        return len(self.kernel)

    @property
    def rho(self) -> int:
        """Half receptive field: sum over layers of dilation*(kernel-1)/2."""
        return sum(d * (k - 1) // 2 for k, d in zip(self.kernel, self.dilation))


@dataclass
class PrefillWorkload:
    name: str
    dtype: str                   # "f32" | "bf16"
    Hq: int
    Hkv: int
    D: int
    window: int
    budget: int
    sink: int
    tau: float                   # logit threshold (0 == retention score > 0.5)
    cu_seqlens: np.ndarray       # int32 [n_seqs+1]
    q: np.ndarray                # [T, Hq, D]
    k: np.ndarray                # [T, Hkv, D]
    v: np.ndarray                # [T, Hkv, D]
    cnn: CnnWeights
    seed: int = 0
    notes: Dict[str, object] = field(default_factory=dict)

    @property
    def n_seqs(self) -> int:
        return len(self.cu_seqlens) - 1

    @property
    def total_tokens(self) -> int:
        return int(self.cu_seqlens[-1])

    @property
    def max_seqlen(self) -> int:
        return int(np.max(np.diff(self.cu_seqlens))) if self.n_seqs else 0


@dataclass
class DecodeState:
    """A directly filled cache state (ring window + compact retained segment).

    The ring slot of position p is p % window. `win_score` is left to the
    caller (it is the scoring CNN's output on the ring contents, which is the
    method's arithmetic and so is not computed here)."""
    name: str
    dtype: str
    B: int
    Hq: int
    Hkv: int
    D: int
    window: int
    budget: int
    sink: int
    tau: float
    k_win: np.ndarray            # [B, Hkv, window, D]
    v_win: np.ndarray
    k_ret: np.ndarray            # [B, Hkv, budget, D]
    v_ret: np.ndarray
    ret_score: np.ndarray        # [B, Hkv, budget] float32
    ret_pos: np.ndarray          # [B, Hkv, budget] int32
    ret_count: np.ndarray        # [B, Hkv] int32
    n_seen: np.ndarray           # [B] int32
    cnn: CnnWeights
    seed: int = 0


# --------------------------------------------------------------------------
# generators
# --------------------------------------------------------------------------
def make_cnn(rng: np.random.Generator, dtype: str, Hkv: int, D: int,
             kernel: Sequence[int], c_out: Sequence[int], dilation: Sequence[int],
             w_std: float) -> CnnWeights:
    """Draw order: per layer W then bias; then w_out, b_out."""
    ws, bs = [], []
    c_in = 2 * D
    for k, c, _ in zip(kernel, c_out, dilation):
        ws.append(to_storage(rng.standard_normal((Hkv, c, c_in, k), dtype=np.float32) * np.float32(w_std), dtype))
        bs.append((rng.standard_normal((Hkv, c), dtype=np.float32) * np.float32(w_std)).astype(np.float32))
        c_in = c
    w_out = to_storage(rng.standard_normal((Hkv, c_in), dtype=np.float32) * np.float32(w_std), dtype)
    b_out = (rng.standard_normal((Hkv,), dtype=np.float32) * np.float32(w_std)).astype(np.float32)
    return CnnWeights(list(kernel), list(dilation), list(c_out), ws, bs, w_out, b_out)


def make_prefill(name: str, seed: int, dtype: str, seqlens: Sequence[int], Hq: int, Hkv: int, D: int,
                 window: int, budget: int, sink: int = 0, tau: float = 0.0,
                 cnn_kernel: Sequence[int] = (5,), cnn_channels: Sequence[int] = (32,),
                 cnn_dilation: Optional[Sequence[int]] = None,
                 qkv_scale: float = 1.0, w_std: float = 0.05,
                 plant_fraction: float = 0.0) -> PrefillWorkload:
    """Draw order: Q, K, V, then the CNN (make_cnn), then optional planted keys."""
    rng = np.random.default_rng(seed)
    seqlens = [int(n) for n in seqlens]
    cu = np.zeros(len(seqlens) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(seqlens)
    T = int(cu[-1])
    sc = np.float32(qkv_scale)
    q = rng.standard_normal((T, Hq, D), dtype=np.float32) * sc
    k = rng.standard_normal((T, Hkv, D), dtype=np.float32) * sc
    v = rng.standard_normal((T, Hkv, D), dtype=np.float32) * sc
    if cnn_dilation is None:
        cnn_dilation = [1] * len(cnn_kernel)
    cnn = make_cnn(rng, dtype, Hkv, D, cnn_kernel, cnn_channels, cnn_dilation, w_std)
    notes: Dict[str, object] = {}
    if plant_fraction > 0.0:
        notes["planted"] = _plant_near_duplicates(rng, q, k, cu, Hq // Hkv, plant_fraction)
    return PrefillWorkload(name, dtype, Hq, Hkv, D, window, budget, sink, float(tau), cu,
                           to_storage(q, dtype), to_storage(k, dtype), to_storage(v, dtype), cnn, seed, notes)


def _plant_near_duplicates(rng, q, k, cu, G, fraction, cosine=0.95):
    """Overwrite a fraction of keys so each is a near-duplicate (cosine ~0.95)
    of a later query of the same sequence and (first) query head of its group,
    keeping the key's norm. Returns the list of (token index, query index)."""
    planted = []
    Hkv, D = k.shape[1], k.shape[2]
    for s in range(len(cu) - 1):
        lo, hi = int(cu[s]), int(cu[s + 1])
        n = hi - lo
        m = max(0, int(round(fraction * n)))
        if n < 2 or m == 0:
            continue
        for h in range(Hkv):
            js = rng.choice(n - 1, size=m, replace=False)
            iq = js + 1 + (rng.random(m) * (n - 1 - js)).astype(np.int64)
            iq = np.minimum(iq, n - 1)
            qh = q[lo + iq, h * G, :].astype(np.float64)
            qh /= np.linalg.norm(qh, axis=1, keepdims=True)
            u = rng.standard_normal((m, D))
            u -= np.sum(u * qh, axis=1, keepdims=True) * qh
            u /= np.linalg.norm(u, axis=1, keepdims=True)
            norm = np.linalg.norm(k[lo + js, h, :].astype(np.float64), axis=1, keepdims=True)
            k[lo + js, h, :] = (norm * (cosine * qh + np.sqrt(1.0 - cosine * cosine) * u)).astype(np.float32)
            if h == 0:
                planted.append((lo + js, lo + iq))
    return planted


def make_decode_state(name: str, seed: int, dtype: str, B: int, Hq: int, Hkv: int, D: int,
                      window: int, budget: int, n_seen: int, ret_fill: Optional[int] = None,
                      sink: int = 0, tau: float = 0.0,
                      cnn_kernel: Sequence[int] = (5,), cnn_channels: Sequence[int] = (32,),
                      w_std: float = 0.05, score_mu: float = 0.0, score_sigma: float = 0.05) -> DecodeState:
    """Fill a cache state directly: ring K,V ~ N(0,1) (slot of position p is
    p % window), retained K,V ~ N(0,1), retained scores ~ N(mu, sigma) folded
    above tau, retained positions distinct and < n_seen - window, ascending.
    Draw order: CNN, k_win, v_win, k_ret, v_ret, ret_score, ret_pos."""
    assert n_seen >= window, "a directly filled state has a full ring"
    rng = np.random.default_rng(seed)
    cnn = make_cnn(rng, dtype, Hkv, D, cnn_kernel, cnn_channels, [1] * len(cnn_kernel), w_std)
    if ret_fill is None:
        ret_fill = budget
    ret_fill = min(ret_fill, budget, n_seen - window)

    def normal(shape):
        out = np.empty(shape, dtype=np.float32)
        flat = out.reshape(-1)
        step = 1 << 24
        for i in range(0, flat.size, step):
            flat[i:i + step] = to_storage(rng.standard_normal(min(step, flat.size - i), dtype=np.float32), dtype)
        return out

    k_win = normal((B, Hkv, window, D))
    v_win = normal((B, Hkv, window, D))
    k_ret = normal((B, Hkv, budget, D))
    v_ret = normal((B, Hkv, budget, D))
    sc = rng.standard_normal((B, Hkv, budget), dtype=np.float32) * np.float32(score_sigma) + np.float32(score_mu)
    t = np.float32(tau)
    sc = (t + np.abs(sc - t) + np.float32(1e-6)).astype(np.float32)
    pos = np.zeros((B, Hkv, budget), dtype=np.int32)
    n_out = n_seen - window
    for b in range(B):
        for h in range(Hkv):
            if ret_fill:
                pos[b, h, :ret_fill] = np.sort(rng.choice(n_out, size=ret_fill, replace=False)).astype(np.int32)
    if sink:
        for b in range(B):
            for h in range(Hkv):
                m = pos[b, h, :ret_fill] < sink
                sc[b, h, :ret_fill][m] = np.inf
    sc[:, :, ret_fill:] = 0.0
    cnt = np.full((B, Hkv), ret_fill, dtype=np.int32)
    return DecodeState(name, dtype, B, Hq, Hkv, D, window, budget, sink, float(tau),
                       k_win, v_win, k_ret, v_ret, sc, pos, cnt,
                       np.full((B,), n_seen, dtype=np.int32), cnn, seed)


def decode_inputs(seed: int, step: int, dtype: str, B: int, Hq: int, Hkv: int, D: int, scale: float = 1.0):
    """Fresh q [B,Hq,D], k,v [B,Hkv,D] for decode step `step` (counter-seeded)."""
    rng = np.random.default_rng([seed, 7919, step])
    s = np.float32(scale)
    q = to_storage(rng.standard_normal((B, Hq, D), dtype=np.float32) * s, dtype)
    k = to_storage(rng.standard_normal((B, Hkv, D), dtype=np.float32) * s, dtype)
    v = to_storage(rng.standard_normal((B, Hkv, D), dtype=np.float32) * s, dtype)
    return q, k, v


# --------------------------------------------------------------------------
# the five named configurations
# --------------------------------------------------------------------------
CONFIG_NAMES = ["tiny_f32", "prefill_bf16", "decode_bf16", "long_prefill_bf16", "varlen_prefill_bf16"]


def rope_tables(n_pos: int, rot_dim: int, base: float = 10000.0):
    """Cached sinusoids of a rotary position encoding, as a model would hold them: cos, sin [n_pos, rot_dim/2]
    fp32 with angle(p, i) = p * base**(-2i/rot_dim).  Input data for the lazy-scoring path; applying them is the
    library's (and, separately, the oracle's) business."""
    inv_freq = base ** (-np.arange(0, rot_dim, 2, dtype=np.float64) / rot_dim)
    ang = np.arange(n_pos, dtype=np.float64)[:, None] * inv_freq[None, :]
    return np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)


def config_tiny_f32() -> PrefillWorkload:
    return make_prefill("tiny_f32", 0, "f32", [512], 2, 2, 64, window=64, budget=32,
                        cnn_kernel=(5,), cnn_channels=(16,), qkv_scale=1.0, w_std=0.1)


def config_prefill_bf16(n: int = 4096, B: int = 4, H: int = 16) -> PrefillWorkload:
    return make_prefill("prefill_bf16", 1, "bf16", [n] * B, H, H, 64, window=512, budget=256,
                        cnn_kernel=(5,), cnn_channels=(32,), qkv_scale=64 ** -0.5, w_std=0.05)


def config_decode_bf16(B: int = 64, H: int = 16, window: int = 1024, budget: int = 512,
                       n_seen: int = 8192) -> DecodeState:
    return make_decode_state("decode_bf16", 2, "bf16", B, H, H, 128, window, budget, n_seen,
                             cnn_kernel=(5,), cnn_channels=(32,), w_std=0.05)


def config_long_prefill_bf16(n: int = 32768, H: int = 32) -> PrefillWorkload:
    return make_prefill("long_prefill_bf16", 3, "bf16", [n], H, H, 128, window=2048, budget=1024,
                        cnn_kernel=(7,), cnn_channels=(32,), qkv_scale=1.0, w_std=0.05)


def varlen_lengths(seed: int = 4, n_seqs: int = 16, lo: int = 1024, hi: int = 16384) -> List[int]:
    return [int(x) for x in np.random.default_rng([seed, 1]).integers(lo, hi + 1, size=n_seqs)]


def config_varlen_prefill_bf16(seqlens: Optional[Sequence[int]] = None, H: int = 16) -> PrefillWorkload:
    if seqlens is None:
        seqlens = varlen_lengths()
    return make_prefill("varlen_prefill_bf16", 4, "bf16", seqlens, H, H, 128, window=1024, budget=512,
                        cnn_kernel=(5,), cnn_channels=(32,), qkv_scale=1.0, w_std=0.05, plant_fraction=0.01)


def config_paper_stack_bf16(n: int = 4096, B: int = 4) -> PrefillWorkload:
    """The LTE module and mixer shape of the paper's own models (Section 3.1.1, Appendix A): three k=3,
    dilation-2 convolutions (receptive field 13) halving the channels 2D -> D -> D/2 -> D/4, attention sink of 4,
    32 query heads sharing 8 KV heads of dimension 64, window 768, budget 512."""
    return make_prefill("paper_stack_bf16", 5, "bf16", [n] * B, 32, 8, 64, window=768, budget=512, sink=4,
                        cnn_kernel=(3, 3, 3), cnn_channels=(64, 32, 16), cnn_dilation=(2, 2, 2),
                        qkv_scale=1.0, w_std=0.05)
