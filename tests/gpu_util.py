"""Helpers for the GPU parity tests: upload a generated workload, read the cache state back, and
compare retained sets / outputs against the oracle at the bars the tests state."""
import numpy as np
import torch

from oracle import ltea_oracle as orc
from paper_2510_20787_amd import binding as B

# Output tolerances (max-abs vs the fp64 oracle, absolute and relative to the largest reference magnitude).
OUT_TOL = {"f32": 1e-5, "bf16": 2e-2}
# Logit tolerance: |z_gpu - z_oracle| <= LOGIT_TOL * max(1, |z|). Inputs and weights are exactly representable,
# products are exact in fp32, so the difference is fp32 accumulation order plus the fp32 Swish (and, in the
# multi-layer bf16 kernels, the 16-bit hi + lo activations).  Measured maxima of that ratio per scoring kernel on one
# MI355X (prefill_bf16, long_prefill_bf16 / varlen_prefill_bf16, paper_stack_bf16, a 2-layer D=128 stack, fp32 stacks):
LOGIT_EPS_MEASURED = {"score_reg_kernel": 3.4e-8, "score_mfma_kernel": 1.1e-6, "score_deep_reg_kernel": 2.5e-7,
                      "score_deep_kernel": 7.9e-7, "score_generic": 8.6e-8}
# The bar is about ten times the largest of them.
LOGIT_TOL = {"f32": 1e-5, "bf16": 1e-5}
assert all(e * 9 <= LOGIT_TOL["bf16"] for e in LOGIT_EPS_MEASURED.values())
# The random-configuration sweeps (and the training forward, which shifts the output biases) draw wider stacks, larger
# weights and logits of several units; their bar is five times wider.
LOGIT_TOL_SWEEP = {dt: 5 * t for dt, t in LOGIT_TOL.items()}


def dev(x: np.ndarray, dtype: str) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(x)).to(device="cuda", dtype=B.torch_dtype(dtype))


class DeviceWorkload:
    def __init__(self, w):
        self.w = w
        self.cfg = B.make_cfg(w.Hq, w.Hkv, w.D, w.window, w.budget, w.sink, w.tau, 0.0, w.dtype)
        c = w.cnn
        self.cnn = B.upload_cnn(c.kernel, c.dilation, c.w, c.bias, c.w_out, c.b_out, w.dtype)
        self.q, self.k, self.v = dev(w.q, w.dtype), dev(w.k, w.dtype), dev(w.v, w.dtype)
        self.cu = torch.from_numpy(w.cu_seqlens.astype(np.int32)).cuda()
        self.max_seqlen = w.max_seqlen
        self.n_seqs = w.n_seqs

    def new_cache(self):
        return B.alloc_cache(self.cfg, self.n_seqs)


def to_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy() if t.dtype in (torch.bfloat16, torch.float32) else t.detach().cpu().numpy()


def gpu_retained_sets(cache, s: int, h: int):
    cnt = int(cache.ret_count[s, h].item())
    pos = cache.ret_pos[s, h, :cnt].cpu().numpy().astype(np.int64)
    return cnt, pos


def boundary_margin(key32: np.ndarray, n: int, window: int, budget: int, sink: int, tau: float):
    """Smallest distance that could flip a membership decision of the capped keep rule for this head:
    the gap between the budget-th and (budget+1)-th candidate keys when the cap binds; candidates at
    the threshold matter only when the cap does not bind."""
    n_out = max(0, n - window)
    kk = key32[:n_out].astype(np.float64)
    isc = np.array([(j < sink) or (key32[j] > np.float32(tau)) for j in range(n_out)], dtype=bool)
    cand = np.sort(kk[isc])[::-1]
    if len(cand) > budget:
        if budget == 0:
            return np.inf
        if cand[budget - 1] == cand[budget] == np.inf:      # more sinks than budget: the order among them is by position
            return np.inf
        return float(cand[budget - 1] - cand[budget])
    nonsink = kk[sink:] if n_out > sink else np.array([])
    nonsink = nonsink[np.isfinite(nonsink)]
    return float(np.min(np.abs(nonsink - tau))) if len(nonsink) else np.inf


def check_sets(cache, z64: np.ndarray, w, eps: float):
    """Retained sets of every (sequence, KV head) against the oracle's rule applied to the oracle's
    logits (decision taken in fp32 on both sides).  Sets must be identical wherever the head's decision
    margin exceeds 2*eps (eps = measured logit difference); heads inside the margin are returned."""
    near = []
    for s in range(w.n_seqs):
        lo, hi = int(w.cu_seqlens[s]), int(w.cu_seqlens[s + 1])
        n = hi - lo
        for h in range(w.Hkv):
            ref = orc.retain(z64[h, lo:hi], n, w.window, w.budget, w.sink, w.tau)
            cnt, pos = gpu_retained_sets(cache, s, h)
            assert cnt <= w.budget
            assert len(set(pos.tolist())) == cnt, "duplicate retained positions"
            got = np.sort(pos)
            if len(got) == len(ref) and np.array_equal(got, ref):
                continue
            margin = boundary_margin(orc.selection_key(z64[h, lo:hi], w.sink), n, w.window, w.budget, w.sink, w.tau)
            assert margin <= 2 * eps, f"retained set differs at seq {s} head {h} with margin {margin} > 2*{eps}"
            near.append((s, h))
    return near


def check_sets_strict(cache, z_gpu: np.ndarray, w):
    """Level-1 check, no margin: the keep rule of eq. 5 + the cap (Section 3.1.3) applied by the oracle to the
    device's OWN fp32 logits must give the device's retained set on EVERY (sequence, KV head).  This isolates
    selection, tie-break and compaction from the scoring arithmetic."""
    n_heads = 0
    for s in range(w.n_seqs):
        lo, hi = int(w.cu_seqlens[s]), int(w.cu_seqlens[s + 1])
        for h in range(w.Hkv):
            ref = orc.retain(z_gpu[h, lo:hi], hi - lo, w.window, w.budget, w.sink, w.tau)
            cnt, pos = gpu_retained_sets(cache, s, h)
            assert cnt == len(ref) and np.array_equal(np.sort(pos), ref), \
                f"retained set of seq {s} head {h} differs from the keep rule on the device's own logits"
            n_heads += 1
    return n_heads


def check_output(got: np.ndarray, ref: np.ndarray, dtype: str, what: str = "output"):
    tol = OUT_TOL[dtype]
    err = float(np.max(np.abs(got.astype(np.float64) - ref)))
    scale = float(np.max(np.abs(ref)))
    assert err <= tol, f"{what}: max-abs error {err} > {tol}"
    assert err <= tol * max(scale, 1e-30), f"{what}: max-abs error {err} exceeds {tol} x largest reference magnitude {scale}"
    return err, scale
