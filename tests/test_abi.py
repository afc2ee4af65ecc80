"""CPU-only checks of the boundary: the library loads, exports exactly what include/ltea.h declares, and
rejects bad arguments on the host before anything could be launched (no compute call is made here)."""
import ctypes as C
import os
import re

import numpy as np

import pytest

from paper_2510_20787_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "ltea.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ltea_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = B.lib()
    names = declared_functions()
    assert names == sorted(B.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def test_strerror():
    assert B.strerror(0) == "ok"
    for s in (-1, -2, -3, -4, -99):
        assert len(B.strerror(s)) > 3


def good_cfg(**kw):
    d = dict(Hq=4, Hkv=2, D=64, window=16, budget=8, sink=0, tau=0.0, softmax_scale=0.0, dtype="bf16")
    d.update(kw)
    return B.make_cfg(**d)


def fake_cnn(kernel=(5,), dilation=(1,), c_out=(16,), n_layers=None):
    s = B.ltea_cnn()
    s.n_layers = len(kernel) if n_layers is None else n_layers
    for l in range(len(kernel)):
        s.kernel[l], s.dilation[l], s.c_out[l] = kernel[l], dilation[l], c_out[l]
        s.w[l] = 0x1000
        s.bias[l] = 0x1000
    s.w_out = 0x1000
    s.b_out = 0x1000
    return s


def score_status(cfg, cnn, k=0x1000, v=0x1000, st=128, sh=64, cu=0x1000, n_seqs=1, total=32, max_len=32, logits=0x1000,
                 ws=0x1000, ws_bytes=1 << 30):
    return B.lib().ltea_score(C.byref(cfg) if cfg else None, C.byref(cnn) if cnn else None, k, v, st, sh, cu, n_seqs,
                              total, max_len, logits, ws, ws_bytes, None)


@pytest.mark.parametrize("case,expect", [
    ("null_cfg", B.LTEA_EINVAL), ("null_cnn", B.LTEA_EINVAL), ("bad_D", B.LTEA_EUNSUPPORTED),
    ("gqa_mismatch", B.LTEA_EINVAL), ("window0", B.LTEA_EINVAL), ("neg_budget", B.LTEA_EINVAL),
    ("even_kernel", B.LTEA_EINVAL), ("layers0", B.LTEA_EINVAL), ("layers5", B.LTEA_EINVAL),
    ("window_lt_field", B.LTEA_EINVAL), ("null_k", B.LTEA_EINVAL), ("null_cu", B.LTEA_EINVAL),
    ("small_stride", B.LTEA_EINVAL), ("odd_stride", B.LTEA_EINVAL), ("misaligned", B.LTEA_EINVAL),
    ("null_logits", B.LTEA_EINVAL), ("no_workspace", B.LTEA_EWORKSPACE), ("neg_total", B.LTEA_EINVAL),
    ("total_gt_cap", B.LTEA_EINVAL), ("bad_dtype", B.LTEA_EINVAL), ("null_weight", B.LTEA_EINVAL),
    ("misaligned_workspace", B.LTEA_EINVAL), ("huge_token_stride", B.LTEA_EUNSUPPORTED),
])
def test_score_argument_errors(case, expect):
    cfg, cnn, kw = good_cfg(), fake_cnn(), {}
    if case == "null_cfg": cfg = None
    elif case == "null_cnn": cnn = None
    elif case == "bad_D": cfg = good_cfg(D=96)
    elif case == "gqa_mismatch": cfg = good_cfg(Hq=5)
    elif case == "window0": cfg = good_cfg(window=0)
    elif case == "neg_budget": cfg = good_cfg(budget=-1)
    elif case == "even_kernel": cnn = fake_cnn(kernel=(4,))
    elif case == "layers0": cnn = fake_cnn(n_layers=0)
    elif case == "layers5": cnn = fake_cnn(n_layers=5)
    elif case == "window_lt_field": cfg = good_cfg(window=4)          # needs >= 2*2+1
    elif case == "null_k": kw = dict(k=None)
    elif case == "null_cu": kw = dict(cu=None)
    elif case == "small_stride": kw = dict(sh=32)
    elif case == "odd_stride": kw = dict(st=132)                      # not a multiple of 8 bf16 elements
    elif case == "misaligned": kw = dict(v=0x1004)
    elif case == "null_logits": kw = dict(logits=None)
    elif case == "no_workspace": cfg = good_cfg(dtype="f32"); kw = dict(ws=None, ws_bytes=0)   # fp32 uses the layered path
    elif case == "neg_total": kw = dict(total=-1)
    elif case == "total_gt_cap": kw = dict(total=64, max_len=32)
    elif case == "bad_dtype": cfg = good_cfg(); cfg.dtype = 7
    elif case == "null_weight": cnn = fake_cnn(); cnn.w[0] = None
    elif case == "misaligned_workspace": kw = dict(ws=0x1040)         # workspaces are 256-byte aligned
    elif case == "huge_token_stride": kw = dict(st=1 << 21)           # the matrix-core kernels' 32-bit row offsets
    assert score_status(cfg, cnn, **kw) == expect


def test_empty_inputs_are_ok_without_touching_the_device():
    cfg, cnn = good_cfg(), fake_cnn()
    assert score_status(cfg, cnn, total=0, n_seqs=0, max_len=0) == B.LTEA_OK
    cache = B.ltea_cache()
    for f, _ in B.ltea_cache._fields_:
        setattr(cache, f, 0x1000)
    L = B.lib()
    assert L.ltea_decode_step(C.byref(cfg), C.byref(cnn), 0x1000, 0x1000, 0x1000, 0x1000, C.byref(cache), 0, None, 0, None) == 0
    assert L.ltea_prefill(C.byref(cfg), C.byref(cnn), None, 0, 0, None, None, 0, 0, 0x1000, 0, 0, 0, None,
                          C.byref(cache), None, None, 0, None) == 0


def test_decode_and_prefill_argument_errors():
    L = B.lib()
    cfg, cnn = good_cfg(), fake_cnn()
    cache = B.ltea_cache()
    for f, _ in B.ltea_cache._fields_:
        setattr(cache, f, 0x1000)
    # workspace too small
    assert L.ltea_decode_step(C.byref(cfg), C.byref(cnn), 0x1000, 0x1000, 0x1000, 0x1000, C.byref(cache), 2, 0x1000, 16, None) == B.LTEA_EWORKSPACE
    # null cache member
    bad = B.ltea_cache()
    assert L.ltea_decode_step(C.byref(cfg), C.byref(cnn), 0x1000, 0x1000, 0x1000, 0x1000, C.byref(bad), 2, 0x1000, 1 << 30, None) == B.LTEA_EINVAL
    assert L.ltea_decode_step(C.byref(cfg), C.byref(cnn), None, 0x1000, 0x1000, 0x1000, C.byref(cache), 2, 0x1000, 1 << 30, None) == B.LTEA_EINVAL
    assert L.ltea_decode_step(C.byref(cfg), C.byref(cnn), 0x1000, 0x1000, 0x1000, 0x1000, C.byref(cache), -1, 0x1000, 1 << 30, None) == B.LTEA_EINVAL
    # per-step scoring pyramid too large for LDS: scored through the packed-window path, which needs the larger workspace
    big = fake_cnn(kernel=(63,), c_out=(16,))
    cfgw = good_cfg(window=256, D=128)
    basic = L.ltea_decode_workspace_bytes(C.byref(cfgw), None, 2)
    full = L.ltea_decode_workspace_bytes(C.byref(cfgw), C.byref(big), 2)
    assert full > basic and full >= L.ltea_decode_feat_workspace_bytes(C.byref(cfgw), C.byref(big), 2)
    assert L.ltea_decode_step(C.byref(cfgw), C.byref(big), 0x1000, 0x1000, 0x1000, 0x1000, C.byref(cache), 2, 0x1000, basic, None) == B.LTEA_EWORKSPACE
    # prefill: null out
    assert L.ltea_prefill(C.byref(cfg), C.byref(cnn), 0x1000, 256, 64, 0x1000, 0x1000, 128, 64, 0x1000, 1, 32, 32, None,
                          C.byref(cache), None, 0x1000, 1 << 30, None) == B.LTEA_EINVAL
    # retain: rho inconsistent with window
    assert L.ltea_retain(C.byref(cfg), 0x1000, 0x1000, 0x1000, 128, 64, 0x1000, 1, 32, 32, 9, C.byref(cache), None, 0, None) == B.LTEA_EINVAL
    # workspace sizes: monotone in tokens, zero on bad config
    a = L.ltea_workspace_bytes(C.byref(cfg), C.byref(cnn), 1, 1000, 1000)
    b = L.ltea_workspace_bytes(C.byref(cfg), C.byref(cnn), 1, 2000, 2000)
    assert 0 < a < b
    assert L.ltea_workspace_bytes(C.byref(good_cfg(D=96)), C.byref(cnn), 1, 1000, 1000) == 0
    assert L.ltea_decode_workspace_bytes(C.byref(cfg), C.byref(cnn), 4) > 0


def test_diag_argument_errors():
    L = B.lib()
    assert L.ltea_diag_sink_bytes() >= 4 * 256
    assert L.ltea_diag_mfma_loop(0, 0x1000, None, None) == B.LTEA_EINVAL
    assert L.ltea_diag_mfma_loop(4, None, None, None) == B.LTEA_EINVAL
    assert L.ltea_diag_stream_read(None, 1024, 0x1000, None) == B.LTEA_EINVAL
    assert L.ltea_diag_stream_read(0x1000, 1000, 0x1000, None) == B.LTEA_EINVAL   # not a multiple of 16
    assert L.ltea_diag_stream_read(0x1008, 1024, 0x1000, None) == B.LTEA_EINVAL   # misaligned


def test_append_argument_errors():
    L = B.lib()
    cfg, cnn = good_cfg(), fake_cnn()
    cache = B.ltea_cache()
    for name, _ in cache._fields_:
        setattr(cache, name, 0x1000)
    args = lambda **kw: dict(dict(cfg=C.byref(cfg), cnn=C.byref(cnn), q=0x1000, qst=256, qsh=64, k=0x1000, v=0x1000,
                                  st=128, sh=64, cu=0x1000, n_seqs=1, total=32, max_new=32, out=0x1000,
                                  cache=C.byref(cache), ws=0x1000, ws_bytes=1 << 40, stream=None), **kw)
    call = lambda a: L.ltea_prefill_append(a["cfg"], a["cnn"], a["q"], a["qst"], a["qsh"], a["k"], a["v"], a["st"],
                                           a["sh"], a["cu"], a["n_seqs"], a["total"], a["max_new"], a["out"],
                                           a["cache"], a["ws"], a["ws_bytes"], a["stream"])
    assert call(args(cfg=None)) == B.LTEA_EINVAL
    assert call(args(cnn=None)) == B.LTEA_EINVAL
    assert call(args(cu=None)) == B.LTEA_EINVAL
    assert call(args(q=None)) == B.LTEA_EINVAL
    assert call(args(out=None)) == B.LTEA_EINVAL
    assert call(args(cache=None)) == B.LTEA_EINVAL
    assert call(args(ws=None)) == B.LTEA_EWORKSPACE
    assert call(args(ws_bytes=16)) == B.LTEA_EWORKSPACE
    assert call(args(n_seqs=0, total=0, max_new=0)) == B.LTEA_OK          # nothing to do
    # the packed extended sequences (budget + 2 window + new tokens per sequence) are indexed by int32 prefix sums
    big = good_cfg(window=1 << 20, budget=1 << 20)
    assert call(args(cfg=C.byref(big), n_seqs=1000, total=1000, max_new=1)) == B.LTEA_EUNSUPPORTED
    assert L.ltea_append_workspace_bytes(C.byref(cfg), C.byref(cnn), 1, 32, 32) > 0
    assert L.ltea_append_workspace_bytes(None, C.byref(cnn), 1, 32, 32) == 0
    # the rotary form: tables are validated, unrotated keys without tables are refused
    feat = lambda a, rope, kf: L.ltea_prefill_append_feat(a["cfg"], a["cnn"], rope, a["q"], a["qst"], a["qsh"], a["k"],
                                                          a["v"], kf, a["st"], a["sh"], a["cu"], a["n_seqs"], a["total"],
                                                          a["max_new"], a["out"], a["cache"], None, a["ws"],
                                                          a["ws_bytes"], a["stream"])
    rope = B.ltea_rope(0x1000, 0x1000, 64, 64, 0)
    assert feat(args(), None, 0x1000) == B.LTEA_EINVAL
    assert feat(args(ws=None), C.byref(rope), 0x1000) == B.LTEA_EWORKSPACE     # everything before the workspace passed
    assert feat(args(), C.byref(B.ltea_rope(0x1000, 0x1000, 64, 24, 0)), None) == B.LTEA_EINVAL   # rot_dim % 16
    assert feat(args(), C.byref(B.ltea_rope(None, 0x1000, 64, 64, 0)), None) == B.LTEA_EINVAL
    assert feat(args(), C.byref(rope), 0x1008) == B.LTEA_EINVAL                # misaligned k_feat
    assert feat(args(n_seqs=0, total=0, max_new=0), C.byref(rope), None) == B.LTEA_OK


def test_decode_feat_argument_errors():
    L = B.lib()
    cfg, cnn = good_cfg(), fake_cnn()
    cache = B.ltea_cache()
    for name, _ in cache._fields_:
        setattr(cache, name, 0x1000)
    need = L.ltea_decode_feat_workspace_bytes(C.byref(cfg), C.byref(cnn), 4)
    assert need > L.ltea_decode_workspace_bytes(C.byref(cfg), None, 4)
    assert L.ltea_decode_feat_workspace_bytes(None, C.byref(cnn), 4) == 0
    rope = B.ltea_rope(0x1000, 0x1000, 64, 64, 0)
    call = lambda **kw: (lambda a: L.ltea_decode_step_feat(a["cfg"], a["cnn"], a["rope"], a["q"], a["k"], a["v"], a["kf"],
                                                            a["out"], a["cache"], a["n"], None, a["ws"], a["wsb"], None))(
        dict(dict(cfg=C.byref(cfg), cnn=C.byref(cnn), rope=C.byref(rope), q=0x1000, k=0x1000, v=0x1000, kf=None,
                  out=0x1000, cache=C.byref(cache), n=4, ws=0x1000, wsb=need), **kw))
    assert call(cfg=None) == B.LTEA_EINVAL
    assert call(cnn=None) == B.LTEA_EINVAL
    assert call(cache=None) == B.LTEA_EINVAL
    assert call(q=None) == B.LTEA_EINVAL
    assert call(k=0x1004) == B.LTEA_EINVAL
    assert call(kf=0x1008) == B.LTEA_EINVAL
    assert call(rope=None, kf=0x1000) == B.LTEA_EINVAL                     # unrotated keys without tables
    assert call(rope=C.byref(B.ltea_rope(0x1000, None, 64, 64, 0))) == B.LTEA_EINVAL
    assert call(rope=C.byref(B.ltea_rope(0x1000, 0x1000, 64, 128, 0))) == B.LTEA_EINVAL   # rot_dim > D
    assert call(n=-1) == B.LTEA_EINVAL
    assert call(n=0) == B.LTEA_OK
    assert call(ws=None) == B.LTEA_EWORKSPACE
    assert call(wsb=need - 1) == B.LTEA_EWORKSPACE


def test_cnn_backward_argument_errors():
    L = B.lib()
    cfg, cnn = good_cfg(), fake_cnn()
    g = B.ltea_cnn_grad()
    for l in range(4):
        g.w[l] = 0x1000
        g.bias[l] = 0x1000
    g.w_out, g.b_out = 0x1000, 0x1000
    need = L.ltea_cnn_backward_workspace_bytes(C.byref(cfg), C.byref(cnn), 1000)
    assert need > 1000 * cfg.Hkv * 2 * cfg.D * 4 and L.ltea_cnn_backward_workspace_bytes(None, C.byref(cnn), 1000) == 0
    call = lambda **kw: (lambda a: L.ltea_cnn_backward(a["cfg"], a["cnn"], a["k"], a["v"], 128, 64, a["cu"], 1, a["T"], a["T"],
                                                        a["dz"], a["g"], a["dk"], None, a["ws"], a["wsb"], None))(
        dict(dict(cfg=C.byref(cfg), cnn=C.byref(cnn), k=0x1000, v=0x1000, cu=0x1000, T=1000, dz=0x1000, g=C.byref(g),
                  dk=0x1000, ws=0x1000, wsb=need), **kw))
    assert call(cfg=None) == B.LTEA_EINVAL
    assert call(cnn=None) == B.LTEA_EINVAL
    assert call(k=None) == B.LTEA_EINVAL
    assert call(cu=None) == B.LTEA_EINVAL
    assert call(dz=None) == B.LTEA_EINVAL
    assert call(g=None) == B.LTEA_EINVAL
    assert call(dk=0x1004) == B.LTEA_EINVAL
    assert call(ws=None) == B.LTEA_EWORKSPACE
    assert call(wsb=need - 1) == B.LTEA_EWORKSPACE
    assert call(ws=0x1010) == B.LTEA_EINVAL          # workspaces are 256-byte aligned
    bad = B.ltea_cnn_grad()
    assert call(g=C.byref(bad)) == B.LTEA_EINVAL


def test_lazy_argument_errors():
    L = B.lib()
    cfg, cnn = good_cfg(), fake_cnn()
    cache = B.ltea_cache()
    for name, _ in cache._fields_:
        setattr(cache, name, 0x1000)
    rho = 2
    assert L.ltea_lazy_period(C.byref(cfg), C.byref(cnn)) == cfg.window - 2 * rho
    assert L.ltea_lazy_period(None, C.byref(cnn)) == 0
    assert L.ltea_lazy_period(C.byref(cfg), None) == 0
    need = L.ltea_rescore_workspace_bytes(C.byref(cfg), C.byref(cnn), 3)
    assert need >= 2 * 3 * cfg.window * cfg.Hkv * cfg.D * 2
    assert L.ltea_rescore_workspace_bytes(C.byref(cfg), None, 3) == 0
    rs = lambda **kw: L.ltea_rescore(*[dict(dict(cfg=C.byref(cfg), cnn=C.byref(cnn), rope=None, cache=C.byref(cache), n=3,
                                                 status=None, ws=0x1000, ws_bytes=1 << 40, stream=None), **kw)[k]
                                       for k in ("cfg", "cnn", "rope", "cache", "n", "status", "ws", "ws_bytes", "stream")])
    assert rs(cfg=None) == B.LTEA_EINVAL
    assert rs(cnn=None) == B.LTEA_EINVAL
    assert rs(cache=None) == B.LTEA_EINVAL
    assert rs(n=-1) == B.LTEA_EINVAL
    assert rs(n=0) == B.LTEA_OK
    assert rs(ws=None) == B.LTEA_EWORKSPACE
    assert rs(ws_bytes=need - 1) == B.LTEA_EWORKSPACE
    rope = lambda **kw: C.byref(B.ltea_rope(**dict(dict(cos=0x1000, sin=0x1000, n_pos=100, rot_dim=32, interleaved=0), **kw)))
    assert rs(rope=rope(cos=None)) == B.LTEA_EINVAL
    assert rs(rope=rope(n_pos=0)) == B.LTEA_EINVAL
    assert rs(rope=rope(rot_dim=24)) == B.LTEA_EINVAL              # not a multiple of 16
    assert rs(rope=rope(rot_dim=128)) == B.LTEA_EINVAL             # wider than the head (D = 64)
    assert rs(rope=rope(interleaved=2)) == B.LTEA_EINVAL
    st = lambda **kw: L.ltea_decode_step_lazy(*[dict(dict(cfg=C.byref(cfg), q=0x1000, k=0x1000, v=0x1000, out=0x1000,
                                                          cache=C.byref(cache), n=2, status=None, ws=0x1000,
                                                          ws_bytes=1 << 30, stream=None), **kw)[k]
                                                for k in ("cfg", "q", "k", "v", "out", "cache", "n", "status", "ws", "ws_bytes", "stream")])
    assert st(cfg=None) == B.LTEA_EINVAL
    assert st(q=None) == B.LTEA_EINVAL
    assert st(out=0x1004) == B.LTEA_EINVAL
    assert st(cache=None) == B.LTEA_EINVAL
    assert st(n=-1) == B.LTEA_EINVAL
    assert st(n=0) == B.LTEA_OK
    assert st(ws_bytes=16) == B.LTEA_EWORKSPACE


def test_lambda_update_matches_the_oracle():
    """Host-side entry point: runs without a GPU."""
    from oracle import ltea_oracle as orc
    rng = np.random.default_rng(5)
    # the hand-set entries reach the oracle as the decimal values (2e-9 halves to exactly the floor 1e-9 and stays);
    # the library sees their fp32 images
    lam64 = np.concatenate([np.array([1e-9, 0.5, 0.9, 2e-9, 0.0, 0.0, 1e-3, 1.5e-9]),
                            (10.0 ** rng.uniform(-10, 0.3, size=200)).astype(np.float32).astype(np.float64)])
    lam = lam64.astype(np.float32)
    cbar = np.concatenate([np.array([600, 600, 600, 100, 600, 100, 500, 10], np.float32),
                           rng.uniform(300, 700, size=200).astype(np.float32)])
    ref = orc.lambda_update(lam64, cbar.astype(np.float64), 512.0, 2.0)
    got = B.ltea_lambda_update(lam.copy(), cbar, 512.0, 2.0)
    np.testing.assert_allclose(got, ref, rtol=1e-6, atol=0)
    assert np.array_equal(got == 0, ref == 0)
    assert (ref == 0).sum() > 3 and (ref == 1.0).sum() > 3 and (ref == 1e-9).sum() >= 1


def test_lambda_update_keeps_the_floor_inside_the_dead_band():
    """Algorithm 1 starts and restarts the multiplier at 1e-9 and zeroes it only below that.  Stored in fp32 the
    floor is 9.9999997e-10; a head at the floor whose count lies between 95 % of the cap and the cap must stay
    there (the oracle, given the decimal 1e-9, leaves it), also over repeated updates, and still restart from zero."""
    from oracle import ltea_oracle as orc
    lam = np.array([1e-9, 1e-9, 0.0, 1e-9], np.float32)
    cbar = np.array([500.0, 490.0, 600.0, 100.0], np.float32)          # dead band, dead band, overshoot, undershoot
    ref = orc.lambda_update(np.array([1e-9, 1e-9, 0.0, 1e-9]), cbar.astype(np.float64), 512.0, 2.0)
    got = lam.copy()
    for _ in range(3):
        got = B.ltea_lambda_update(got, np.array([500.0, 490.0, 500.0, 500.0], np.float32) if _ else cbar, 512.0, 2.0)
        if _ == 0:
            np.testing.assert_array_equal(got, ref.astype(np.float32))
    assert got[0] == np.float32(1e-9) and got[1] == np.float32(1e-9)    # never flushed
    assert got[2] == np.float32(1e-9)                                   # restarted once, then held in the dead band
    assert got[3] == 0.0                                                # shrunk below the floor: flushed


def test_train_argument_errors():
    L = B.lib()
    cfg, cnn = good_cfg(), fake_cnn()
    need = L.ltea_train_workspace_bytes(C.byref(cfg), C.byref(cnn), 2, 64, 32)
    assert need > 2 * 2 * cfg.Hkv * 32 * cfg.D * 2
    assert L.ltea_train_workspace_bytes(None, C.byref(cnn), 2, 64, 32) == 0
    fw = lambda **kw: L.ltea_train_forward(*[dict(dict(cfg=C.byref(cfg), cnn=C.byref(cnn), q=0x1000, qst=256, qsh=64, k=0x1000,
                                                       v=0x1000, st=128, sh=64, cu=0x1000, n=2, total=64, max_len=32, rho=0,
                                                       out=0x1000, lse=0x1000, logits=0x1000, ws=0x1000, ws_bytes=1 << 40,
                                                       stream=None), **kw)[k]
                                             for k in ("cfg", "cnn", "q", "qst", "qsh", "k", "v", "st", "sh", "cu", "n", "total",
                                                       "max_len", "rho", "out", "lse", "logits", "ws", "ws_bytes", "stream")])
    assert fw(cfg=None) == B.LTEA_EINVAL
    assert fw(cnn=None, rho=9) == B.LTEA_EINVAL         # caller's logits: the look-ahead must fit the window
    assert fw(cnn=None, rho=-1) == B.LTEA_EINVAL
    assert L.ltea_train_workspace_bytes(C.byref(cfg), None, 2, 64, 32) > 0
    assert fw(cu=None) == B.LTEA_EINVAL
    assert fw(lse=None) == B.LTEA_EINVAL
    assert fw(logits=None) == B.LTEA_EINVAL
    assert fw(ws=None) == B.LTEA_EWORKSPACE
    assert fw(ws_bytes=need - 1) == B.LTEA_EWORKSPACE
    assert fw(n=0, total=0, max_len=0) == B.LTEA_OK
    bw = lambda **kw: L.ltea_train_backward(*[dict(dict(cfg=C.byref(cfg), q=0x1000, qst=256, qsh=64, k=0x1000, v=0x1000,
                                                        st=128, sh=64, cu=0x1000, n=2, total=64, max_len=32, out=0x1000,
                                                        dout=0x1000, lse=0x1000, logits=0x1000, lam=0x1000, dq=0x1000,
                                                        dk=0x1000, dv=0x1000, dz=0x1000, counts=0x1000, ws=0x1000,
                                                        ws_bytes=1 << 40, stream=None), **kw)[k]
                                              for k in ("cfg", "q", "qst", "qsh", "k", "v", "st", "sh", "cu", "n", "total",
                                                        "max_len", "out", "dout", "lse", "logits", "lam", "dq", "dk", "dv",
                                                        "dz", "counts", "ws", "ws_bytes", "stream")])
    assert bw(cfg=None) == B.LTEA_EINVAL
    assert bw(dout=None) == B.LTEA_EINVAL
    assert bw(lam=None) == B.LTEA_EINVAL
    assert bw(counts=None) == B.LTEA_EINVAL
    assert bw(dz=None) == B.LTEA_EINVAL
    assert bw(ws_bytes=16) == B.LTEA_EWORKSPACE
    assert bw(n=0, total=0, max_len=0) == B.LTEA_OK
    lam = (C.c_float * 2)(0.5, 0.0)
    cb = (C.c_float * 2)(600.0, 600.0)
    assert L.ltea_lambda_update(lam, cb, 2, 512.0, 2.0) == B.LTEA_OK and lam[0] == 1.0 and abs(lam[1] - 1e-9) < 1e-15
    assert L.ltea_lambda_update(None, cb, 2, 512.0, 2.0) == B.LTEA_EINVAL
    assert L.ltea_lambda_update(lam, cb, 2, 512.0, 0.0) == B.LTEA_EINVAL


def test_cnn_prepare_argument_errors():
    L = B.lib()
    cfg, cnn = good_cfg(), fake_cnn()
    need = L.ltea_cnn_panels_bytes(C.byref(cfg), C.byref(cnn))
    assert need >= cfg.Hkv * 5 * 32 * 2 * cfg.D * 2                     # single layer, kernel 5, 32-channel panels
    assert L.ltea_cnn_panels_bytes(None, C.byref(cnn)) == 0
    assert L.ltea_cnn_panels_bytes(C.byref(good_cfg(dtype="f32")), C.byref(cnn)) == 0
    assert L.ltea_cnn_prepare(None, C.byref(cnn), 0x1000, need, None) == B.LTEA_EINVAL
    assert L.ltea_cnn_prepare(C.byref(cfg), None, 0x1000, need, None) == B.LTEA_EINVAL
    assert L.ltea_cnn_prepare(C.byref(cfg), C.byref(cnn), None, need, None) == B.LTEA_EWORKSPACE
    assert L.ltea_cnn_prepare(C.byref(cfg), C.byref(cnn), 0x1000, need - 1, None) == B.LTEA_EWORKSPACE
    assert L.ltea_cnn_prepare(C.byref(good_cfg(dtype="f32")), C.byref(cnn), None, 0, None) == B.LTEA_OK   # nothing to prepare
