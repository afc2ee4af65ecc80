"""Thin ctypes binding over libltea.so (C ABI in include/ltea.h).

Argument marshalling only: tensors are PyTorch device tensors (PyTorch is used for device memory and
streams, nothing else); every computation happens inside the library's HIP kernels.  There is no CPU
or PyTorch fallback: if the shared library is missing, or a call returns an error status, an exception
is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libltea.so")

LTEA_F32, LTEA_BF16 = 0, 1
LTEA_OK, LTEA_EINVAL, LTEA_EUNSUPPORTED, LTEA_EWORKSPACE, LTEA_EHIP = 0, -1, -2, -3, -4
LTEA_LATE_SCORING, LTEA_ROPE_RANGE = 1, 2
MAX_LAYERS = 4


class LteaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} (status {status})")


class ltea_cnn(C.Structure):
    _fields_ = [("n_layers", C.c_int32),
                ("kernel", C.c_int32 * MAX_LAYERS), ("dilation", C.c_int32 * MAX_LAYERS),
                ("c_out", C.c_int32 * MAX_LAYERS),
                ("w", C.c_void_p * MAX_LAYERS), ("bias", C.c_void_p * MAX_LAYERS),
                ("w_out", C.c_void_p), ("b_out", C.c_void_p), ("panels", C.c_void_p)]


class ltea_cfg(C.Structure):
    _fields_ = [("Hq", C.c_int32), ("Hkv", C.c_int32), ("D", C.c_int32),
                ("window", C.c_int32), ("budget", C.c_int32), ("sink", C.c_int32),
                ("tau_logit", C.c_float), ("softmax_scale", C.c_float), ("dtype", C.c_int32)]


class ltea_cache(C.Structure):
    _fields_ = [("k_win", C.c_void_p), ("v_win", C.c_void_p), ("win_score", C.c_void_p),
                ("k_ret", C.c_void_p), ("v_ret", C.c_void_p), ("ret_score", C.c_void_p),
                ("ret_pos", C.c_void_p), ("ret_count", C.c_void_p), ("n_seen", C.c_void_p),
                ("n_scored", C.c_void_p)]


class ltea_cnn_grad(C.Structure):
    _fields_ = [("w", C.c_void_p * 4), ("bias", C.c_void_p * 4), ("w_out", C.c_void_p), ("b_out", C.c_void_p)]


class ltea_rope(C.Structure):
    _fields_ = [("cos", C.c_void_p), ("sin", C.c_void_p), ("n_pos", C.c_int32), ("rot_dim", C.c_int32),
                ("interleaved", C.c_int32)]


EXPORTS = ["ltea_strerror", "ltea_cnn_panels_bytes", "ltea_cnn_prepare", "ltea_workspace_bytes", "ltea_decode_workspace_bytes", "ltea_score", "ltea_retain",
           "ltea_sparse_attention", "ltea_prefill", "ltea_prefill_feat", "ltea_decode_step", "ltea_decode_step_static",
           "ltea_append_workspace_bytes",
           "ltea_prefill_append", "ltea_prefill_append_feat", "ltea_decode_feat_workspace_bytes",
           "ltea_decode_step_feat", "ltea_cnn_backward_workspace_bytes", "ltea_cnn_backward", "ltea_lazy_period", "ltea_rescore_workspace_bytes", "ltea_rescore",
           "ltea_decode_step_lazy", "ltea_train_workspace_bytes", "ltea_train_forward", "ltea_train_backward",
           "ltea_lambda_update", "ltea_diag_sink_bytes",
           "ltea_diag_mfma_loop", "ltea_diag_stream_read"]

_lib = None


def lib() -> C.CDLL:
    """Load libltea.so once; fail loudly if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} not found: build it with `python -m paper_2510_20787_amd.build` "
                           "(there is no fallback path)")
    L = C.CDLL(LIB_PATH)
    i32, i64, vp, sz = C.c_int32, C.c_int64, C.c_void_p, C.c_size_t
    P = C.POINTER
    L.ltea_strerror.restype = C.c_char_p
    L.ltea_strerror.argtypes = [C.c_int]
    L.ltea_cnn_panels_bytes.restype = sz
    L.ltea_cnn_panels_bytes.argtypes = [P(ltea_cfg), P(ltea_cnn)]
    L.ltea_cnn_prepare.restype = C.c_int
    L.ltea_cnn_prepare.argtypes = [P(ltea_cfg), P(ltea_cnn), vp, sz, vp]
    L.ltea_workspace_bytes.restype = sz
    L.ltea_workspace_bytes.argtypes = [P(ltea_cfg), P(ltea_cnn), i32, i64, i32]
    L.ltea_decode_workspace_bytes.restype = sz
    L.ltea_decode_workspace_bytes.argtypes = [P(ltea_cfg), P(ltea_cnn), i32]
    L.ltea_score.restype = C.c_int
    L.ltea_score.argtypes = [P(ltea_cfg), P(ltea_cnn), vp, vp, i64, i64, vp, i32, i64, i32, vp, vp, sz, vp]
    L.ltea_retain.restype = C.c_int
    L.ltea_retain.argtypes = [P(ltea_cfg), vp, vp, vp, i64, i64, vp, i32, i64, i32, i32, P(ltea_cache), vp, sz, vp]
    L.ltea_sparse_attention.restype = C.c_int
    L.ltea_sparse_attention.argtypes = [P(ltea_cfg), vp, i64, i64, vp, vp, i64, i64, vp, i32, i64, i32,
                                        P(ltea_cache), vp, vp, sz, vp]
    L.ltea_prefill.restype = C.c_int
    L.ltea_prefill.argtypes = [P(ltea_cfg), P(ltea_cnn), vp, i64, i64, vp, vp, i64, i64, vp, i32, i64, i32, vp,
                               P(ltea_cache), vp, vp, sz, vp]
    L.ltea_prefill_feat.restype = C.c_int
    L.ltea_prefill_feat.argtypes = [P(ltea_cfg), P(ltea_cnn), vp, i64, i64, vp, vp, vp, i64, i64, vp, i32, i64, i32, vp,
                                    P(ltea_cache), vp, vp, sz, vp]
    L.ltea_decode_step.restype = C.c_int
    L.ltea_decode_step.argtypes = [P(ltea_cfg), P(ltea_cnn), vp, vp, vp, vp, P(ltea_cache), i32, vp, sz, vp]
    L.ltea_decode_step_static.restype = C.c_int
    L.ltea_decode_step_static.argtypes = [P(ltea_cfg), P(ltea_cnn), vp, vp, vp, vp, P(ltea_cache), i32, vp]
    L.ltea_append_workspace_bytes.restype = sz
    L.ltea_append_workspace_bytes.argtypes = [P(ltea_cfg), P(ltea_cnn), i32, i64, i32]
    L.ltea_prefill_append.restype = C.c_int
    L.ltea_prefill_append.argtypes = [P(ltea_cfg), P(ltea_cnn), vp, i64, i64, vp, vp, i64, i64, vp, i32, i64, i32, vp,
                                      P(ltea_cache), vp, sz, vp]
    L.ltea_prefill_append_feat.restype = C.c_int
    L.ltea_prefill_append_feat.argtypes = [P(ltea_cfg), P(ltea_cnn), P(ltea_rope), vp, i64, i64, vp, vp, vp, i64, i64,
                                           vp, i32, i64, i32, vp, P(ltea_cache), vp, vp, sz, vp]
    L.ltea_decode_feat_workspace_bytes.restype = sz
    L.ltea_decode_feat_workspace_bytes.argtypes = [P(ltea_cfg), P(ltea_cnn), i32]
    L.ltea_decode_step_feat.restype = C.c_int
    L.ltea_decode_step_feat.argtypes = [P(ltea_cfg), P(ltea_cnn), P(ltea_rope), vp, vp, vp, vp, vp, P(ltea_cache), i32,
                                        vp, vp, sz, vp]
    L.ltea_cnn_backward_workspace_bytes.restype = sz
    L.ltea_cnn_backward_workspace_bytes.argtypes = [P(ltea_cfg), P(ltea_cnn), i64]
    L.ltea_cnn_backward.restype = C.c_int
    L.ltea_cnn_backward.argtypes = [P(ltea_cfg), P(ltea_cnn), vp, vp, i64, i64, vp, i32, i64, i32, vp, P(ltea_cnn_grad),
                                    vp, vp, vp, sz, vp]
    L.ltea_lazy_period.restype = i32
    L.ltea_lazy_period.argtypes = [P(ltea_cfg), P(ltea_cnn)]
    L.ltea_rescore_workspace_bytes.restype = sz
    L.ltea_rescore_workspace_bytes.argtypes = [P(ltea_cfg), P(ltea_cnn), i32]
    L.ltea_rescore.restype = C.c_int
    L.ltea_rescore.argtypes = [P(ltea_cfg), P(ltea_cnn), P(ltea_rope), P(ltea_cache), i32, vp, vp, sz, vp]
    L.ltea_decode_step_lazy.restype = C.c_int
    L.ltea_decode_step_lazy.argtypes = [P(ltea_cfg), vp, vp, vp, vp, P(ltea_cache), i32, vp, vp, sz, vp]
    L.ltea_train_workspace_bytes.restype = sz
    L.ltea_train_workspace_bytes.argtypes = [P(ltea_cfg), P(ltea_cnn), i32, i64, i32]
    L.ltea_train_forward.restype = C.c_int
    L.ltea_train_forward.argtypes = [P(ltea_cfg), P(ltea_cnn), vp, i64, i64, vp, vp, i64, i64, vp, i32, i64, i32, i32, vp,
                                     vp, vp, vp, sz, vp]
    L.ltea_train_backward.restype = C.c_int
    L.ltea_train_backward.argtypes = [P(ltea_cfg), vp, i64, i64, vp, vp, i64, i64, vp, i32, i64, i32, vp, vp, vp, vp, vp,
                                      vp, vp, vp, vp, vp, vp, sz, vp]
    L.ltea_lambda_update.restype = C.c_int
    L.ltea_lambda_update.argtypes = [P(C.c_float), P(C.c_float), i32, C.c_float, C.c_float]
    L.ltea_diag_sink_bytes.restype = sz
    L.ltea_diag_sink_bytes.argtypes = []
    L.ltea_diag_mfma_loop.restype = C.c_int
    L.ltea_diag_mfma_loop.argtypes = [i32, vp, P(C.c_double), vp]
    L.ltea_diag_stream_read.restype = C.c_int
    L.ltea_diag_stream_read.argtypes = [vp, sz, vp, vp]
    _lib = L
    return L


def strerror(status: int) -> str:
    return lib().ltea_strerror(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != LTEA_OK:
        raise LteaError(status, where)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def torch_dtype(dtype: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16}[dtype]


def make_cfg(Hq: int, Hkv: int, D: int, window: int, budget: int, sink: int = 0, tau: float = 0.0,
             softmax_scale: float = 0.0, dtype: str = "bf16") -> ltea_cfg:
    return ltea_cfg(Hq, Hkv, D, window, budget, sink, float(tau), float(softmax_scale),
                    LTEA_F32 if dtype == "f32" else LTEA_BF16)


@dataclass
class Cnn:
    """Device copies of the scoring CNN plus the C struct pointing at them."""
    struct: ltea_cnn
    tensors: List[torch.Tensor]
    rho: int


def upload_cnn(kernel: Sequence[int], dilation: Sequence[int], w: Sequence, bias: Sequence, w_out, b_out,
               dtype: str, device="cuda") -> Cnn:
    """w[l]: [Hkv, C_out, C_in, kernel]; bias[l]: [Hkv, C_out]; w_out: [Hkv, C]; b_out: [Hkv] (host arrays)."""
    td = torch_dtype(dtype)
    s = ltea_cnn()
    s.n_layers = len(kernel)
    keep: List[torch.Tensor] = []
    for l in range(len(kernel)):
        s.kernel[l], s.dilation[l], s.c_out[l] = int(kernel[l]), int(dilation[l]), int(w[l].shape[1])
        wt = torch.as_tensor(w[l]).to(device=device, dtype=td).contiguous()
        bt = torch.as_tensor(bias[l]).to(device=device, dtype=torch.float32).contiguous()
        keep += [wt, bt]
        s.w[l], s.bias[l] = wt.data_ptr(), bt.data_ptr()
    wo = torch.as_tensor(w_out).to(device=device, dtype=td).contiguous()
    bo = torch.as_tensor(b_out).to(device=device, dtype=torch.float32).contiguous()
    keep += [wo, bo]
    s.w_out, s.b_out = wo.data_ptr(), bo.data_ptr()
    rho = sum(int(d) * (int(k) - 1) // 2 for k, d in zip(kernel, dilation))
    return Cnn(s, keep, rho)


def prepare_cnn(cfg: ltea_cfg, cnn: Cnn) -> Cnn:
    """Re-lay the conv weights once for the matrix-core scoring kernels (ltea_cnn_prepare) and point cnn.struct.panels
    at the result; every later call with this Cnn then skips the per-call re-layout.  No-op for configurations whose
    kernels read the weights as they are."""
    nbytes = int(lib().ltea_cnn_panels_bytes(C.byref(cfg), C.byref(cnn.struct)))
    if nbytes == 0:
        return cnn
    panels = torch.empty(nbytes, dtype=torch.uint8, device=cnn.tensors[0].device)
    _check(lib().ltea_cnn_prepare(C.byref(cfg), C.byref(cnn.struct), _ptr(panels), nbytes, _stream()), "ltea_cnn_prepare")
    cnn.tensors.append(panels)
    cnn.struct.panels = panels.data_ptr()
    return cnn


@dataclass
class Cache:
    """Device arrays of the cache state for B sequences plus the C struct pointing at them."""
    struct: ltea_cache
    k_win: torch.Tensor
    v_win: torch.Tensor
    win_score: torch.Tensor
    k_ret: torch.Tensor
    v_ret: torch.Tensor
    ret_score: torch.Tensor
    ret_pos: torch.Tensor
    ret_count: torch.Tensor
    n_seen: torch.Tensor
    n_scored: torch.Tensor


def alloc_cache(cfg: ltea_cfg, B: int, device="cuda") -> Cache:
    """A zeroed cache (n_seen = 0: also the valid start state for decoding from scratch)."""
    td = torch.float32 if cfg.dtype == LTEA_F32 else torch.bfloat16
    z = lambda shape, dt: torch.zeros(shape, dtype=dt, device=device)
    bmin = max(cfg.budget, 1)
    t = dict(k_win=z((B, cfg.Hkv, cfg.window, cfg.D), td), v_win=z((B, cfg.Hkv, cfg.window, cfg.D), td),
             win_score=z((B, cfg.Hkv, cfg.window), torch.float32),
             k_ret=z((B, cfg.Hkv, bmin, cfg.D), td), v_ret=z((B, cfg.Hkv, bmin, cfg.D), td),
             ret_score=z((B, cfg.Hkv, bmin), torch.float32), ret_pos=z((B, cfg.Hkv, bmin), torch.int32),
             ret_count=z((B, cfg.Hkv), torch.int32), n_seen=z((B,), torch.int32), n_scored=z((B,), torch.int32))
    return wrap_cache(**t)


def wrap_cache(k_win, v_win, win_score, k_ret, v_ret, ret_score, ret_pos, ret_count, n_seen, n_scored) -> Cache:
    s = ltea_cache(k_win.data_ptr(), v_win.data_ptr(), win_score.data_ptr(), k_ret.data_ptr(), v_ret.data_ptr(),
                   ret_score.data_ptr(), ret_pos.data_ptr(), ret_count.data_ptr(), n_seen.data_ptr(),
                   n_scored.data_ptr())
    return Cache(s, k_win, v_win, win_score, k_ret, v_ret, ret_score, ret_pos, ret_count, n_seen, n_scored)


def _workspace(nbytes: int, device) -> Optional[torch.Tensor]:
    return torch.empty(max(int(nbytes), 16), dtype=torch.uint8, device=device)


def decode_workspace(cfg: ltea_cfg, cnn: Optional["Cnn"], n_seqs: int, device="cuda") -> torch.Tensor:
    """A workspace for ltea_decode_step, reusable across steps."""
    return _workspace(ltea_decode_workspace_bytes(cfg, cnn, n_seqs), device)


def _tok_head_strides(x: torch.Tensor):
    assert x.dim() == 3, "expected a [T, H, D] view"
    if x.numel() == 0:                      # an empty view has no meaningful strides: report the packed ones
        return x.shape[1] * x.shape[2], x.shape[2]
    assert x.stride(2) == 1, "expected a [T, H, D] view with contiguous last dimension"
    return x.stride(0), x.stride(1)


def ltea_workspace_bytes(cfg: ltea_cfg, cnn: Optional[Cnn], n_seqs: int, total_tokens: int, max_seqlen: int) -> int:
    return int(lib().ltea_workspace_bytes(C.byref(cfg), C.byref(cnn.struct) if cnn else None, n_seqs, total_tokens,
                                          max_seqlen))


def ltea_decode_workspace_bytes(cfg: ltea_cfg, cnn: Optional[Cnn], n_seqs: int) -> int:
    return int(lib().ltea_decode_workspace_bytes(C.byref(cfg), C.byref(cnn.struct) if cnn else None, n_seqs))


def ltea_score(cfg: ltea_cfg, cnn: Cnn, k: torch.Tensor, v: torch.Tensor, cu_seqlens: torch.Tensor,
               max_seqlen: int, logits: Optional[torch.Tensor] = None,
               workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    T = k.shape[0]
    n_seqs = cu_seqlens.numel() - 1
    st, sh = _tok_head_strides(k)
    assert _tok_head_strides(v) == (st, sh)
    if logits is None:
        logits = torch.empty((cfg.Hkv, T), dtype=torch.float32, device=k.device)
    if workspace is None:
        workspace = _workspace(ltea_workspace_bytes(cfg, cnn, n_seqs, T, max_seqlen), k.device)
    _check(lib().ltea_score(C.byref(cfg), C.byref(cnn.struct), _ptr(k), _ptr(v), st, sh, _ptr(cu_seqlens), n_seqs, T,
                            max_seqlen, _ptr(logits), _ptr(workspace), workspace.numel(), _stream()), "ltea_score")
    return logits


def ltea_retain(cfg: ltea_cfg, logits: torch.Tensor, k: torch.Tensor, v: torch.Tensor, cu_seqlens: torch.Tensor,
                max_seqlen: int, rho: int, cache: Cache) -> Cache:
    T = k.shape[0]
    n_seqs = cu_seqlens.numel() - 1
    st, sh = _tok_head_strides(k)
    assert _tok_head_strides(v) == (st, sh)
    _check(lib().ltea_retain(C.byref(cfg), _ptr(logits), _ptr(k), _ptr(v), st, sh, _ptr(cu_seqlens), n_seqs, T,
                             max_seqlen, rho, C.byref(cache.struct), None, 0, _stream()), "ltea_retain")
    return cache


def ltea_sparse_attention(cfg: ltea_cfg, q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, cu_seqlens: torch.Tensor,
                          max_seqlen: int, cache: Cache, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    T = q.shape[0]
    n_seqs = cu_seqlens.numel() - 1
    qst, qsh = _tok_head_strides(q)
    st, sh = _tok_head_strides(k)
    assert _tok_head_strides(v) == (st, sh)
    if out is None:
        out = torch.empty((T, cfg.Hq, cfg.D), dtype=q.dtype, device=q.device)
    _check(lib().ltea_sparse_attention(C.byref(cfg), _ptr(q), qst, qsh, _ptr(k), _ptr(v), st, sh, _ptr(cu_seqlens),
                                       n_seqs, T, max_seqlen, C.byref(cache.struct), _ptr(out), None, 0, _stream()),
           "ltea_sparse_attention")
    return out


def ltea_prefill(cfg: ltea_cfg, cnn: Cnn, q: torch.Tensor, k: torch.Tensor, v: torch.Tensor,
                 cu_seqlens: torch.Tensor, max_seqlen: int, cache: Cache, out: Optional[torch.Tensor] = None,
                 logits: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                 k_feat: Optional[torch.Tensor] = None) -> torch.Tensor:
    """k_feat (optional, same strides as k): the keys the CNN scores when they differ from the cached ones."""
    T = q.shape[0]
    n_seqs = cu_seqlens.numel() - 1
    qst, qsh = _tok_head_strides(q)
    st, sh = _tok_head_strides(k)
    assert _tok_head_strides(v) == (st, sh)
    if out is None:
        out = torch.empty((T, cfg.Hq, cfg.D), dtype=q.dtype, device=q.device)
    if workspace is None:
        workspace = _workspace(ltea_workspace_bytes(cfg, cnn, n_seqs, T, max_seqlen), q.device)
    if k_feat is not None:
        assert _tok_head_strides(k_feat) == (st, sh)
        _check(lib().ltea_prefill_feat(C.byref(cfg), C.byref(cnn.struct), _ptr(q), qst, qsh, _ptr(k), _ptr(v), _ptr(k_feat),
                                       st, sh, _ptr(cu_seqlens), n_seqs, T, max_seqlen, _ptr(out), C.byref(cache.struct),
                                       _ptr(logits), _ptr(workspace), workspace.numel(), _stream()), "ltea_prefill_feat")
        return out
    _check(lib().ltea_prefill(C.byref(cfg), C.byref(cnn.struct), _ptr(q), qst, qsh, _ptr(k), _ptr(v), st, sh,
                              _ptr(cu_seqlens), n_seqs, T, max_seqlen, _ptr(out), C.byref(cache.struct), _ptr(logits),
                              _ptr(workspace), workspace.numel(), _stream()), "ltea_prefill")
    return out


def ltea_append_workspace_bytes(cfg: ltea_cfg, cnn: Cnn, n_seqs: int, total_new: int, max_new: int) -> int:
    return int(lib().ltea_append_workspace_bytes(C.byref(cfg), C.byref(cnn.struct), n_seqs, total_new, max_new))


def ltea_prefill_append(cfg: ltea_cfg, cnn: Cnn, q: torch.Tensor, k: torch.Tensor, v: torch.Tensor,
                        cu_new: torch.Tensor, max_new: int, cache: Cache, out: Optional[torch.Tensor] = None,
                        workspace: Optional[torch.Tensor] = None, rope: Optional[Rope] = None,
                        k_feat: Optional[torch.Tensor] = None, status: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Continue a prefill: q, k, v hold the new tokens of every sequence, packed by cu_new.  rope (rotary models): the
    cached keys are rotated, the ring is rotated back for the scoring; k_feat: the new keys before the rotation
    (optional with rope: without it the new keys are rotated back too)."""
    T = q.shape[0]
    n_seqs = cu_new.numel() - 1
    qst, qsh = _tok_head_strides(q)
    st, sh = _tok_head_strides(k)
    assert _tok_head_strides(v) == (st, sh)
    assert k_feat is None or _tok_head_strides(k_feat) == (st, sh)
    if out is None:
        out = torch.empty((T, cfg.Hq, cfg.D), dtype=q.dtype, device=q.device)
    if workspace is None:
        workspace = _workspace(max(ltea_append_workspace_bytes(cfg, cnn, n_seqs, T, max_new), 16), q.device)
    if rope is None and k_feat is None and status is None:
        _check(lib().ltea_prefill_append(C.byref(cfg), C.byref(cnn.struct), _ptr(q), qst, qsh, _ptr(k), _ptr(v), st, sh,
                                         _ptr(cu_new), n_seqs, T, max_new, _ptr(out), C.byref(cache.struct),
                                         _ptr(workspace), workspace.numel(), _stream()), "ltea_prefill_append")
    else:
        _check(lib().ltea_prefill_append_feat(C.byref(cfg), C.byref(cnn.struct), C.byref(rope.struct) if rope else None,
                                              _ptr(q), qst, qsh, _ptr(k), _ptr(v), _ptr(k_feat), st, sh, _ptr(cu_new),
                                              n_seqs, T, max_new, _ptr(out), C.byref(cache.struct), _ptr(status),
                                              _ptr(workspace), workspace.numel(), _stream()),
               "ltea_prefill_append_feat")
    return out


def ltea_decode_step(cfg: ltea_cfg, cnn: Cnn, q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, cache: Cache,
                     out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    B = q.shape[0]
    assert q.is_contiguous() and k.is_contiguous() and v.is_contiguous()
    if out is None:
        out = torch.empty((B, cfg.Hq, cfg.D), dtype=q.dtype, device=q.device)
    if workspace is None:
        workspace = _workspace(ltea_decode_workspace_bytes(cfg, cnn, B), q.device)
    _check(lib().ltea_decode_step(C.byref(cfg), C.byref(cnn.struct), _ptr(q), _ptr(k), _ptr(v), _ptr(out),
                                  C.byref(cache.struct), B, _ptr(workspace), workspace.numel(), _stream()),
           "ltea_decode_step")
    return out


def ltea_decode_step_static(cfg: ltea_cfg, cnn: Cnn, q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, cache: Cache,
                            out: torch.Tensor) -> torch.Tensor:
    """The decode step on the library's own fixed scratch.  `out` is the caller's: nothing is allocated here."""
    assert q.is_contiguous() and k.is_contiguous() and v.is_contiguous() and out.is_contiguous()
    _check(lib().ltea_decode_step_static(C.byref(cfg), C.byref(cnn.struct), _ptr(q), _ptr(k), _ptr(v), _ptr(out),
                                         C.byref(cache.struct), q.shape[0], _stream()), "ltea_decode_step_static")
    return out


@dataclass
class Rope:
    """Device copies of the rotary tables plus the C struct pointing at them."""
    struct: ltea_rope
    tensors: List[torch.Tensor]


def upload_rope(cos, sin, interleaved: bool = False, device="cuda") -> Rope:
    """cos, sin: [n_pos, rot_dim/2] host arrays (fp32)."""
    ct = torch.as_tensor(cos).to(device=device, dtype=torch.float32).contiguous()
    st = torch.as_tensor(sin).to(device=device, dtype=torch.float32).contiguous()
    assert ct.shape == st.shape and ct.dim() == 2
    return Rope(ltea_rope(ct.data_ptr(), st.data_ptr(), ct.shape[0], 2 * ct.shape[1], 1 if interleaved else 0), [ct, st])


def ltea_decode_step_feat(cfg: ltea_cfg, cnn: Cnn, q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, cache: Cache,
                          rope: Optional[Rope] = None, k_feat: Optional[torch.Tensor] = None,
                          out: Optional[torch.Tensor] = None, status: Optional[torch.Tensor] = None,
                          workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Eager decode step of a rotary model: k is the rotated key (cached, attended); the scoring sees the ring rotated
    back and k_feat (the key before the rotation) or, without it, k rotated back."""
    B = q.shape[0]
    assert q.is_contiguous() and k.is_contiguous() and v.is_contiguous() and (k_feat is None or k_feat.is_contiguous())
    if out is None:
        out = torch.empty((B, cfg.Hq, cfg.D), dtype=q.dtype, device=q.device)
    if workspace is None:
        workspace = _workspace(int(lib().ltea_decode_feat_workspace_bytes(C.byref(cfg), C.byref(cnn.struct), B)), q.device)
    _check(lib().ltea_decode_step_feat(C.byref(cfg), C.byref(cnn.struct), C.byref(rope.struct) if rope else None,
                                       _ptr(q), _ptr(k), _ptr(v), _ptr(k_feat), _ptr(out), C.byref(cache.struct), B,
                                       _ptr(status), _ptr(workspace), workspace.numel(), _stream()),
           "ltea_decode_step_feat")
    return out


def ltea_lazy_period(cfg: ltea_cfg, cnn: Cnn) -> int:
    return int(lib().ltea_lazy_period(C.byref(cfg), C.byref(cnn.struct)))


def ltea_rescore_workspace_bytes(cfg: ltea_cfg, cnn: Cnn, n_seqs: int) -> int:
    return int(lib().ltea_rescore_workspace_bytes(C.byref(cfg), C.byref(cnn.struct), n_seqs))


def ltea_rescore(cfg: ltea_cfg, cnn: Cnn, cache: Cache, rope: Optional[Rope] = None,
                 status: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> None:
    """Batched scoring of the unscored in-window positions of every sequence of `cache`."""
    B = cache.n_seen.numel()
    if workspace is None:
        workspace = _workspace(ltea_rescore_workspace_bytes(cfg, cnn, B), cache.n_seen.device)
    _check(lib().ltea_rescore(C.byref(cfg), C.byref(cnn.struct), C.byref(rope.struct) if rope else None,
                              C.byref(cache.struct), B, _ptr(status), _ptr(workspace), workspace.numel(), _stream()),
           "ltea_rescore")


def ltea_decode_step_lazy(cfg: ltea_cfg, q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, cache: Cache,
                          out: Optional[torch.Tensor] = None, status: Optional[torch.Tensor] = None,
                          workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    B = q.shape[0]
    assert q.is_contiguous() and k.is_contiguous() and v.is_contiguous()
    if out is None:
        out = torch.empty((B, cfg.Hq, cfg.D), dtype=q.dtype, device=q.device)
    if workspace is None:
        workspace = _workspace(ltea_decode_workspace_bytes(cfg, None, B), q.device)
    _check(lib().ltea_decode_step_lazy(C.byref(cfg), _ptr(q), _ptr(k), _ptr(v), _ptr(out), C.byref(cache.struct), B,
                                       _ptr(status), _ptr(workspace), workspace.numel(), _stream()),
           "ltea_decode_step_lazy")
    return out


def ltea_train_workspace_bytes(cfg: ltea_cfg, cnn: Optional[Cnn], n_seqs: int, total_tokens: int, max_seqlen: int) -> int:
    return int(lib().ltea_train_workspace_bytes(C.byref(cfg), C.byref(cnn.struct) if cnn else None, n_seqs, total_tokens,
                                                max_seqlen))


def ltea_train_forward(cfg: ltea_cfg, cnn: Optional[Cnn], q: torch.Tensor, k: torch.Tensor, v: torch.Tensor,
                       cu_seqlens: torch.Tensor, max_seqlen: int, workspace: Optional[torch.Tensor] = None,
                       logits: Optional[torch.Tensor] = None, rho: int = 0):
    """Training forward (no cap).  Returns (out, lse, logits, workspace); the workspace holds the state the
    backward needs and must be passed to ltea_train_backward unchanged.  With cnn=None the caller supplies the
    logits ([Hkv, T] fp32) and the CNN's look-ahead rho."""
    T = q.shape[0]
    n_seqs = cu_seqlens.numel() - 1
    qst, qsh = _tok_head_strides(q)
    st, sh = _tok_head_strides(k)
    assert _tok_head_strides(v) == (st, sh)
    out = torch.empty((T, cfg.Hq, cfg.D), dtype=q.dtype, device=q.device)
    lse = torch.empty((cfg.Hq, T), dtype=torch.float32, device=q.device)
    if cnn is not None:
        logits = torch.empty((cfg.Hkv, T), dtype=torch.float32, device=q.device)
        rho = cnn.rho
    else:
        assert logits is not None and logits.dtype == torch.float32 and logits.is_contiguous()
    if workspace is None:
        workspace = _workspace(ltea_train_workspace_bytes(cfg, cnn, n_seqs, T, max_seqlen), q.device)
    _check(lib().ltea_train_forward(C.byref(cfg), C.byref(cnn.struct) if cnn else None, _ptr(q), qst, qsh, _ptr(k), _ptr(v),
                                    st, sh, _ptr(cu_seqlens), n_seqs, T, max_seqlen, int(rho), _ptr(out), _ptr(lse),
                                    _ptr(logits),
                                    _ptr(workspace), workspace.numel(), _stream()), "ltea_train_forward")
    return out, lse, logits, workspace


def ltea_train_backward(cfg: ltea_cfg, q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, cu_seqlens: torch.Tensor,
                        max_seqlen: int, out: torch.Tensor, dout: torch.Tensor, lse: torch.Tensor,
                        logits: torch.Tensor, lam: torch.Tensor, workspace: torch.Tensor):
    """Returns (dq, dk, dv, dz, counts)."""
    T = q.shape[0]
    n_seqs = cu_seqlens.numel() - 1
    qst, qsh = _tok_head_strides(q)
    st, sh = _tok_head_strides(k)
    assert _tok_head_strides(v) == (st, sh) and out.is_contiguous() and dout.is_contiguous()
    dq = torch.empty((T, cfg.Hq, cfg.D), dtype=q.dtype, device=q.device)
    dk = torch.empty((T, cfg.Hkv, cfg.D), dtype=q.dtype, device=q.device)
    dv = torch.empty((T, cfg.Hkv, cfg.D), dtype=q.dtype, device=q.device)
    dz = torch.empty((cfg.Hkv, T), dtype=torch.float32, device=q.device)
    counts = torch.empty((n_seqs, cfg.Hkv), dtype=torch.int32, device=q.device)
    _check(lib().ltea_train_backward(C.byref(cfg), _ptr(q), qst, qsh, _ptr(k), _ptr(v), st, sh, _ptr(cu_seqlens), n_seqs,
                                     T, max_seqlen, _ptr(out), _ptr(dout), _ptr(lse), _ptr(logits), _ptr(lam), _ptr(dq),
                                     _ptr(dk), _ptr(dv), _ptr(dz), _ptr(counts), _ptr(workspace), workspace.numel(),
                                     _stream()), "ltea_train_backward")
    return dq, dk, dv, dz, counts


def ltea_cnn_backward(cfg: ltea_cfg, cnn: Cnn, k_feat: torch.Tensor, v: torch.Tensor, cu_seqlens: torch.Tensor,
                      max_seqlen: int, dz: torch.Tensor, want_inputs: bool = True, workspace: Optional[torch.Tensor] = None):
    """Gradients of sum(dz * logits) through the scoring CNN.  Returns (dw list, dbias list, dw_out, db_out, dk_feat,
    dv); the last two are None without want_inputs."""
    T = k_feat.shape[0]
    n_seqs = cu_seqlens.numel() - 1
    st, sh = _tok_head_strides(k_feat)
    assert _tok_head_strides(v) == (st, sh)
    s = cnn.struct
    dev = k_feat.device
    f32 = lambda *shape: torch.empty(shape, dtype=torch.float32, device=dev)
    dw, dbias, cin = [], [], 2 * cfg.D
    for l in range(s.n_layers):
        dw.append(f32(cfg.Hkv, s.c_out[l], cin, s.kernel[l]))
        dbias.append(f32(cfg.Hkv, s.c_out[l]))
        cin = s.c_out[l]
    dw_out, db_out = f32(cfg.Hkv, cin), f32(cfg.Hkv)
    g = ltea_cnn_grad()
    for l in range(s.n_layers):
        g.w[l] = dw[l].data_ptr()
        g.bias[l] = dbias[l].data_ptr()
    g.w_out, g.b_out = dw_out.data_ptr(), db_out.data_ptr()
    dk = torch.empty((T, cfg.Hkv, cfg.D), dtype=k_feat.dtype, device=dev) if want_inputs else None
    dv = torch.empty((T, cfg.Hkv, cfg.D), dtype=k_feat.dtype, device=dev) if want_inputs else None
    if workspace is None:
        workspace = _workspace(int(lib().ltea_cnn_backward_workspace_bytes(C.byref(cfg), C.byref(s), T)), dev)
    _check(lib().ltea_cnn_backward(C.byref(cfg), C.byref(s), _ptr(k_feat), _ptr(v), st, sh, _ptr(cu_seqlens), n_seqs, T,
                                   max_seqlen, _ptr(dz), C.byref(g), _ptr(dk), _ptr(dv), _ptr(workspace),
                                   workspace.numel(), _stream()), "ltea_cnn_backward")
    return dw, dbias, dw_out, db_out, dk, dv


def ltea_lambda_update(lam, c_bar, cap: float, alpha: float):
    """Host-side feedback step on the penalty weights; lam and c_bar are float32 numpy arrays (lam is updated)."""
    import numpy as np
    assert lam.dtype == np.float32 and c_bar.dtype == np.float32 and lam.size == c_bar.size
    assert lam.flags["C_CONTIGUOUS"] and c_bar.flags["C_CONTIGUOUS"]
    _check(lib().ltea_lambda_update(lam.ctypes.data_as(C.POINTER(C.c_float)), c_bar.ctypes.data_as(C.POINTER(C.c_float)),
                                    lam.size, float(cap), float(alpha)), "ltea_lambda_update")
    return lam


def ltea_diag_sink(device="cuda") -> torch.Tensor:
    """Device buffer the two measurement aids write their checksums to."""
    return torch.empty(int(lib().ltea_diag_sink_bytes()), dtype=torch.uint8, device=device)


def ltea_diag_mfma_loop(iters: int, sink: torch.Tensor) -> float:
    """Enqueue the register-resident MFMA loop; returns the flops of the launch."""
    flops = C.c_double(0.0)
    _check(lib().ltea_diag_mfma_loop(int(iters), _ptr(sink), C.byref(flops), _stream()), "ltea_diag_mfma_loop")
    return float(flops.value)


def ltea_diag_stream_read(src: torch.Tensor, sink: torch.Tensor) -> int:
    """Enqueue one streaming read of `src`; returns the bytes read."""
    nbytes = src.numel() * src.element_size()
    _check(lib().ltea_diag_stream_read(_ptr(src), nbytes, _ptr(sink), _stream()), "ltea_diag_stream_read")
    return nbytes
