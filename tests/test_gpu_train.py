"""GPU parity of the training-side forward / backward (Section 3.1.2; Algorithm 1) against the oracle: outputs and
softmax normalisers of the uncapped masked attention, dQ / dK / dV, the straight-through gradient of the retention
scores plus the sparsity penalty (as d logits), and the retention counts.

Bars: counts bit-exact; fp32 gradients within 2e-5 and bf16 gradients within 2e-2 of the fp64 oracle, both relative
to the largest reference magnitude of the tensor (bf16: O, dQ, dK, dV are rounded to bf16 and the backward reads the
rounded O).  A logit within the scoring tolerance of the threshold may flip a token's visibility: seeds are chosen
so that no logit sits there (checked)."""
import numpy as np
import pytest
import torch

from oracle import ltea_oracle as orc
from paper_2510_20787_amd import binding as B
from paper_2510_20787_amd import workloads as wl
from tests.gpu_util import LOGIT_TOL_SWEEP, DeviceWorkload, dev, to_np
from tests.helpers import oracle_cfg, oracle_cnn

pytestmark = pytest.mark.gpu

GRAD_TOL = {"f32": 2e-5, "bf16": 2e-2}

CASES = {
    # name: (dtype, seqlens, Hq, Hkv, D, window, sink, kernel, channels, dilation, w_std)
    "f32_d64": ("f32", [150, 0, 67, 1], 4, 2, 64, 24, 1, (5,), (16,), None, 0.3),
    "f32_d128_deep": ("f32", [130, 90], 2, 2, 128, 32, 2, (3, 3, 3), (32, 16, 8), (2, 2, 2), 0.12),
    "bf16_d64_gqa": ("bf16", [300, 129, 40], 8, 2, 64, 48, 2, (5,), (32,), None, 0.2),
    "bf16_d128": ("bf16", [260, 77], 2, 2, 128, 64, 0, (7,), (32,), None, 0.2),
    "bf16_d128_gqa": ("bf16", [333, 140, 9], 4, 2, 128, 40, 1, (5,), (32,), None, 0.2),
    "bf16_d64_edges": ("bf16", [0, 1, 50, 200, 0, 129], 4, 4, 64, 64, 3, (5,), (32,), None, 0.2),
    "bf16_d64_deep": ("bf16", [280, 150], 4, 2, 64, 64, 4, (3, 3, 3), (64, 32, 16), (2, 2, 2), 0.12),
}


def max_err(got, ref):
    return float(np.max(np.abs(got.astype(np.float64) - ref)))


@pytest.mark.parametrize("name", list(CASES))
def test_train_forward_backward(name):
    dt, lens, Hq, Hkv, D, window, sink, ker, ch, dil, w_std = CASES[name]
    w = wl.make_prefill(name, sum(map(ord, name)), dt, lens, Hq, Hkv, D, window, 1, sink, 0.0, cnn_kernel=ker,
                        cnn_channels=ch, cnn_dilation=dil, qkv_scale=1.0, w_std=w_std)
    cfg, cnn = oracle_cfg(w), oracle_cnn(w.cnn)
    rng = np.random.default_rng(w.seed + 99)
    dout = wl.to_storage(rng.standard_normal((w.total_tokens, Hq, D), dtype=np.float32), dt)
    lam = np.abs(rng.standard_normal(Hkv)).astype(np.float32) * np.float32(0.1)
    z64 = orc.score(w.k, w.v, cnn, w.cu_seqlens)
    frac = float((z64 > 0).mean())
    assert 0.05 < frac < 0.95, f"both kept and dropped tokens are needed, kept fraction {frac}"
    d = DeviceWorkload(w)
    out, lse, logits, ws = B.ltea_train_forward(d.cfg, d.cnn, d.q, d.k, d.v, d.cu, d.max_seqlen)
    d_dout = dev(dout, dt)
    dq, dk, dv, dz, counts = B.ltea_train_backward(d.cfg, d.q, d.k, d.v, d.cu, d.max_seqlen, out, d_dout, lse, logits,
                                                   torch.from_numpy(lam).cuda(), ws)
    torch.cuda.synchronize()
    zg = to_np(logits)
    # the multi-layer bf16 kernel carries activations as bf16 hi + lo pairs: allow it a few 1e-5 at these weights
    eps = float(np.max(np.abs(zg - z64)))
    assert np.all(np.abs(zg - z64) <= LOGIT_TOL_SWEEP[dt] * np.maximum(1.0, np.abs(z64)))
    assert np.min(np.abs(z64)) > 2 * eps, "a logit sits inside the scoring error of the threshold: pick another seed"
    tol = GRAD_TOL[dt]
    out_g, lse_g, dq_g, dk_g, dv_g, dz_g = (to_np(x) for x in (out, lse, dq, dk, dv, dz))
    cnt_g = counts.cpu().numpy()
    refs = {key: np.zeros(shape) for key, shape in (("out", out_g.shape), ("lse", lse_g.shape), ("dq", dq_g.shape),
                                                     ("dk", dk_g.shape), ("dv", dv_g.shape), ("dz", dz_g.shape))}
    for s in range(w.n_seqs):
        lo, hi = int(w.cu_seqlens[s]), int(w.cu_seqlens[s + 1])
        if hi == lo:
            assert np.all(cnt_g[s] == 0)
            continue
        refs["out"][lo:hi], refs["lse"][:, lo:hi], _ = orc.train_forward_sequence(w.q[lo:hi], w.k[lo:hi], w.v[lo:hi],
                                                                                 z64[:, lo:hi], cfg)
        refs["dq"][lo:hi], refs["dk"][lo:hi], refs["dv"][lo:hi], refs["dz"][:, lo:hi], c_ref = orc.train_backward_sequence(
            w.q[lo:hi], w.k[lo:hi], w.v[lo:hi], z64[:, lo:hi], dout[lo:hi], cfg, lam.astype(np.float64))
        np.testing.assert_array_equal(cnt_g[s], c_ref)
    assert max_err(lse_g, refs["lse"]) <= (1e-4 if dt == "f32" else 2e-3)
    for key, got in (("out", out_g), ("dq", dq_g), ("dk", dk_g), ("dv", dv_g), ("dz", dz_g)):
        scale = float(np.max(np.abs(refs[key])))
        err = max_err(got, refs[key])
        assert scale > 0 and err <= tol * scale, (name, key, err, scale)
    # same inputs, same bits
    dq2, dk2, dv2, dz2, counts2 = B.ltea_train_backward(d.cfg, d.q, d.k, d.v, d.cu, d.max_seqlen, out, d_dout, lse, logits,
                                                        torch.from_numpy(lam).cuda(), ws)
    for a, b in ((dq, dq2), (dk, dk2), (dv, dv2), (dz, dz2), (counts, counts2)):
        assert torch.equal(a, b)


def test_train_forward_equals_prefill_when_the_cap_does_not_bind():
    """With budget >= n the inference prefill and the training forward are the same computation."""
    dt, lens, Hq, Hkv, D, window, sink, ker, ch, dil, w_std = CASES["bf16_d64_gqa"]
    w = wl.make_prefill("cap_free", 7, dt, lens, Hq, Hkv, D, window, max(lens), sink, 0.0, cnn_kernel=ker,
                        cnn_channels=ch, cnn_dilation=dil, qkv_scale=1.0, w_std=w_std)
    d = DeviceWorkload(w)
    out_t, lse, logits, ws = B.ltea_train_forward(d.cfg, d.cnn, d.q, d.k, d.v, d.cu, d.max_seqlen)
    cache = d.new_cache()
    out_p = B.ltea_prefill(d.cfg, d.cnn, d.q, d.k, d.v, d.cu, d.max_seqlen, cache)
    assert torch.equal(out_t, out_p)


def test_train_with_logits_supplied_by_the_caller():
    """cnn = NULL: the logits come from outside (here: random ones, unrelated to any CNN), so both sides take the
    visibility decisions on identical numbers."""
    dt, lens, Hq, Hkv, D, window, sink, ker, ch, dil, w_std = CASES["bf16_d64_gqa"]
    w = wl.make_prefill("supplied", 11, dt, lens, Hq, Hkv, D, window, 1, sink, 0.0, cnn_kernel=ker, cnn_channels=ch,
                        cnn_dilation=dil, qkv_scale=1.0, w_std=w_std)
    cfg = oracle_cfg(w)
    rng = np.random.default_rng(12)
    z32 = rng.standard_normal((Hkv, w.total_tokens)).astype(np.float32) - np.float32(0.8)     # about a fifth kept
    dout = wl.to_storage(rng.standard_normal((w.total_tokens, Hq, D), dtype=np.float32), dt)
    lam = np.array([0.05, 0.0], dtype=np.float32)
    d = DeviceWorkload(w)
    zt = torch.from_numpy(z32).cuda()
    out, lse, logits, ws = B.ltea_train_forward(d.cfg, None, d.q, d.k, d.v, d.cu, d.max_seqlen, logits=zt, rho=2)
    assert logits.data_ptr() == zt.data_ptr()
    dq, dk, dv, dz, counts = B.ltea_train_backward(d.cfg, d.q, d.k, d.v, d.cu, d.max_seqlen, out, dev(dout, dt), lse, zt,
                                                   torch.from_numpy(lam).cuda(), ws)
    z64 = z32.astype(np.float64)
    for s in range(w.n_seqs):
        lo, hi = int(w.cu_seqlens[s]), int(w.cu_seqlens[s + 1])
        o_ref, _, _ = orc.train_forward_sequence(w.q[lo:hi], w.k[lo:hi], w.v[lo:hi], z64[:, lo:hi], cfg)
        dq_ref, dk_ref, dv_ref, dz_ref, c_ref = orc.train_backward_sequence(w.q[lo:hi], w.k[lo:hi], w.v[lo:hi], z64[:, lo:hi],
                                                                             dout[lo:hi], cfg, lam.astype(np.float64))
        for got, ref, what in ((out[lo:hi], o_ref, "out"), (dq[lo:hi], dq_ref, "dq"), (dk[lo:hi], dk_ref, "dk"),
                               (dv[lo:hi], dv_ref, "dv"), (dz[:, lo:hi], dz_ref, "dz")):
            scale = float(np.max(np.abs(ref)))
            assert max_err(to_np(got), ref) <= GRAD_TOL[dt] * scale, (s, what)
        np.testing.assert_array_equal(counts[s].cpu().numpy(), c_ref)


@pytest.mark.parametrize("dtype,kernel,channels,dilation,lens",
                         [("f32", (5,), (16,), None, [70, 0, 33]), ("bf16", (3, 3, 3), (64, 32, 16), (2, 2, 2), [300, 41]),
                          ("bf16", (7,), (32,), None, [1500, 900, 1]), ("f32", (3, 1), (8, 24), (2, 1), [5, 2]),
                          ("f32", (3, 5), (10, 6), (40, 9), [200, 0, 90, 130]),
                          ("bf16", (3, 3), (16, 48), (1, 3), [257, 64]), ("bf16", (3, 3), (10, 6), (2, 1), [150, 77])])
def test_cnn_backward(dtype, kernel, channels, dilation, lens):
    """Gradients of sum(dz * logits) through the scoring CNN against the oracle's chain rule: every conv weight and
    bias, the output projection, and the scored keys / values.  Shapes cover one to three layers, both storage types,
    more than one token chunk of the two-stage sums, empty and one-token sequences, channel counts that are not
    multiples of four, dilations beyond and within the rows a tile stages for a group of taps, and every combination
    of narrow (<= 32) and wide channel counts on the two sides of a layer.  On bf16 storage the first layer's forward,
    its weight gradient and the products towards the input run on the bf16 matrix instruction (exact products, the
    fp32 operand split into three bf16 terms) when the channel counts allow; the last case takes the fp32 routes."""
    Hq, Hkv, D = 4, 2, 64
    rho = sum(d * (k - 1) // 2 for k, d in zip(kernel, dilation or [1] * len(kernel)))
    w = wl.make_prefill("cnn_bwd", 1800 + len(kernel) + len(lens), dtype, lens, Hq, Hkv, D, max(27, 2 * rho + 3), 4, 0, 0.0,
                        cnn_kernel=kernel, cnn_channels=channels, cnn_dilation=dilation, w_std=0.1)
    ocnn = oracle_cnn(w.cnn)
    rng = np.random.default_rng(77)
    dz = rng.standard_normal((Hkv, w.total_tokens)).astype(np.float32)
    ref = orc.score_backward(w.k, w.v, ocnn, w.cu_seqlens, dz)
    d = DeviceWorkload(w)
    got = B.ltea_cnn_backward(d.cfg, d.cnn, d.k, d.v, d.cu, d.max_seqlen, torch.from_numpy(dz).cuda())
    torch.cuda.synchronize()

    def close(a, b, what, rel):
        a, b = a.float().cpu().numpy().astype(np.float64), np.asarray(b, np.float64)
        scale = max(float(np.abs(b).max()), 1e-30)
        err = float(np.abs(a - b).max())
        assert err <= rel * scale, (what, err, scale)

    # fp32 sums of up to a few thousand terms; the storage type only enters through the rounded inputs (identical on
    # both sides) and, for dk / dv, through the rounding of the result
    for l in range(len(kernel)):
        close(got[0][l], ref[0][l], f"dw[{l}]", 2e-5)
        close(got[1][l], ref[1][l], f"dbias[{l}]", 2e-5)
    close(got[2], ref[2], "dw_out", 2e-5)
    close(got[3], ref[3], "db_out", 2e-5)
    out_rel = 2e-5 if dtype == "f32" else 2 ** -8
    close(got[4], ref[4], "dk", out_rel)
    close(got[5], ref[5], "dv", out_rel)
    # the same bits on a second run (fixed summation order), and parameter gradients alone on request
    again = B.ltea_cnn_backward(d.cfg, d.cnn, d.k, d.v, d.cu, d.max_seqlen, torch.from_numpy(dz).cuda(), want_inputs=False)
    assert again[4] is None and torch.equal(again[0][0], got[0][0]) and torch.equal(again[2], got[2])


@pytest.mark.parametrize("name", ["f32_d64", "f32_d128_deep", "bf16_d64_deep"])
def test_training_chain_from_dout_to_the_cnn_weights(name):
    """The three training entry points chained the way a training step uses them: forward, attention backward (which
    hands over d logits), CNN backward on those d logits.  Reference: the oracle's three functions chained the same
    way.  The weight gradients then carry the d-logit error of the attention backward, so the bar is GRAD_TOL relative
    to the largest entry of each gradient array."""
    dt, lens, Hq, Hkv, D, window, sink, ker, ch, dil, w_std = CASES[name]
    w = wl.make_prefill(name, sum(map(ord, name)), dt, lens, Hq, Hkv, D, window, 1, sink, 0.0, cnn_kernel=ker,
                        cnn_channels=ch, cnn_dilation=dil, qkv_scale=1.0, w_std=w_std)
    cfg, cnn = oracle_cfg(w), oracle_cnn(w.cnn)
    rng = np.random.default_rng(w.seed + 99)
    dout = wl.to_storage(rng.standard_normal((w.total_tokens, Hq, D), dtype=np.float32), dt)
    lam = np.abs(rng.standard_normal(Hkv)).astype(np.float32) * np.float32(0.1)
    z64 = orc.score(w.k, w.v, cnn, w.cu_seqlens)
    dz_ref = np.zeros((Hkv, w.total_tokens))
    for s in range(w.n_seqs):
        lo, hi = int(w.cu_seqlens[s]), int(w.cu_seqlens[s + 1])
        if hi > lo:
            dz_ref[:, lo:hi] = orc.train_backward_sequence(w.q[lo:hi], w.k[lo:hi], w.v[lo:hi], z64[:, lo:hi], dout[lo:hi],
                                                           cfg, lam.astype(np.float64))[3]
    ref = orc.score_backward(w.k, w.v, cnn, w.cu_seqlens, dz_ref)
    d = DeviceWorkload(w)
    out, lse, logits, ws = B.ltea_train_forward(d.cfg, d.cnn, d.q, d.k, d.v, d.cu, d.max_seqlen)
    grads = B.ltea_train_backward(d.cfg, d.q, d.k, d.v, d.cu, d.max_seqlen, out, dev(dout, dt), lse, logits,
                                  torch.from_numpy(lam).cuda(), ws)
    got = B.ltea_cnn_backward(d.cfg, d.cnn, d.k, d.v, d.cu, d.max_seqlen, grads[3])
    torch.cuda.synchronize()
    tol = GRAD_TOL[dt]
    names = [f"dw[{l}]" for l in range(len(ker))] + [f"dbias[{l}]" for l in range(len(ker))] + ["dw_out", "db_out", "dk", "dv"]
    arrays_g = list(got[0]) + list(got[1]) + [got[2], got[3], got[4], got[5]]
    arrays_r = list(ref[0]) + list(ref[1]) + [ref[2], ref[3], ref[4], ref[5]]
    for nm, a, b in zip(names, arrays_g, arrays_r):
        a = a.float().cpu().numpy().astype(np.float64)
        scale = max(float(np.abs(b).max()), 1e-30)
        assert float(np.abs(a - b).max()) <= tol * scale, (nm, float(np.abs(a - b).max()), scale)
