"""The allocation-free decode entry point (ltea_decode_step_static: scratch in a fixed device array inside the
library) against ltea_decode_step (scratch in a caller workspace), through the C ABI, on two calls in a row, the
second with a smaller batch.  Both run the same kernels on the same split layout, so outputs and the whole cache
state must agree bit for bit, which is within every bar the parity tests state.  Collected last on purpose."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2510_20787_amd import binding as B
from paper_2510_20787_amd import workloads as wl
from tests.gpu_util import dev

pytestmark = pytest.mark.gpu

STATE_FIELDS = ("k_win", "v_win", "win_score", "k_ret", "v_ret", "ret_score", "ret_pos", "ret_count", "n_seen", "n_scored")


def clone_cache(c: B.Cache) -> B.Cache:
    return B.wrap_cache(*[getattr(c, f).clone() for f in STATE_FIELDS])


def state_equal(a: B.Cache, b: B.Cache, n_seqs: int):
    for f in STATE_FIELDS:
        x, y = getattr(a, f)[:n_seqs], getattr(b, f)[:n_seqs]
        # NaN logits (positions not scored yet) compare equal as bit patterns
        same = torch.equal(x.view(torch.int32), y.view(torch.int32)) if x.dtype == torch.float32 else torch.equal(x, y)
        assert same, f"cache field {f} differs"


def prefilled(seqlens, Hq, Hkv, D, window, budget, sink, seed, kernel=(5,), channels=(32,), dilation=None):
    w = wl.make_prefill("no_alloc", seed, "bf16", list(seqlens), Hq, Hkv, D, window, budget, sink, 0.0, cnn_kernel=kernel,
                        cnn_channels=channels, cnn_dilation=dilation, w_std=0.05)
    cfg = B.make_cfg(w.Hq, w.Hkv, w.D, w.window, w.budget, w.sink, w.tau, 0.0, "bf16")
    c = w.cnn
    cnn = B.upload_cnn(c.kernel, c.dilation, c.w, c.bias, c.w_out, c.b_out, "bf16")
    cache = B.alloc_cache(cfg, w.n_seqs)
    cu = torch.from_numpy(w.cu_seqlens.astype(np.int32)).cuda()
    B.ltea_prefill(cfg, cnn, dev(w.q, "bf16"), dev(w.k, "bf16"), dev(w.v, "bf16"), cu, w.max_seqlen, cache)
    return w, cfg, cnn, cache


@pytest.mark.parametrize("shape", ["mha_d128", "gqa_d64_deep"])
def test_static_scratch_step_equals_workspace_step(shape):
    if shape == "mha_d128":
        w, cfg, cnn, cache = prefilled([700, 333, 512, 90, 640, 1000], 8, 8, 128, 256, 96, 2, 41)
    else:   # the paper's module shape in small: 3-layer dilated CNN, grouped queries
        w, cfg, cnn, cache = prefilled([900, 40, 777, 300], 8, 2, 64, 192, 64, 4, 42, kernel=(3, 3, 3), channels=(64, 32, 16),
                                       dilation=(2, 2, 2))
    ref_cache, got_cache = clone_cache(cache), clone_cache(cache)
    for call, n_seqs in enumerate((w.n_seqs, 2)):          # second call: a smaller batch on the same scratch
        q, k, v = wl.decode_inputs(7, call, "bf16", n_seqs, w.Hq, w.Hkv, w.D)
        dq, dk, dv = dev(q, "bf16"), dev(k, "bf16"), dev(v, "bf16")
        sub = lambda c: B.wrap_cache(*[getattr(c, f)[:n_seqs] for f in STATE_FIELDS])   # leading sequences, same memory
        ref = B.ltea_decode_step(cfg, cnn, dq, dk, dv, sub(ref_cache))
        out = torch.full((n_seqs, w.Hq, w.D), float("nan"), dtype=torch.bfloat16, device="cuda")
        B.ltea_decode_step_static(cfg, cnn, dq, dk, dv, sub(got_cache), out)
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), ref.view(torch.int16)), f"call {call}: outputs differ"
        state_equal(ref_cache, got_cache, w.n_seqs)
        assert bool((got_cache.n_seen[:n_seqs] == torch.from_numpy(np.diff(w.cu_seqlens)).cuda()[:n_seqs] + call + 1).all())


def test_static_scratch_rejects_what_does_not_fit():
    """Sizes beyond the fixed scratch are refused on the host with LTEA_EWORKSPACE; nothing is launched."""
    cfg = B.make_cfg(16, 16, 128, 1024, 512, 0, 0.0, 0.0, "bf16")
    rng = np.random.default_rng(3)
    c = wl.make_cnn(rng, "bf16", 16, 128, (5,), (32,), [1], 0.05)
    cnn = B.upload_cnn(c.kernel, c.dilation, c.w, c.bias, c.w_out, c.b_out, "bf16")
    n_big = 4096
    assert B.ltea_decode_workspace_bytes(cfg, cnn, n_big) > (8 << 20)
    fake = B.ltea_cache()
    for name, _ in fake._fields_:
        setattr(fake, name, 0x1000)
    st = B.lib().ltea_decode_step_static(C.byref(cfg), C.byref(cnn.struct), 0x1000, 0x1000, 0x1000, 0x1000, C.byref(fake),
                                         n_big, None)
    assert st == B.LTEA_EWORKSPACE
    assert "scratch" in B.strerror(st)
