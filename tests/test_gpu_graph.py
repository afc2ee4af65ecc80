"""HIP graph capture of the entry points: every call only enqueues kernels on the caller's stream (no allocation,
no synchronisation, no memset nodes), so a caller can record a decode loop once and replay it.  Each replay is
compared bit for bit with a twin cache that takes the same steps eagerly; between replays the test does ordinary
eager work and synchronises, and the inputs of the recorded calls are refreshed in place."""
import numpy as np
import pytest
import torch

from paper_2510_20787_amd import binding as B
from paper_2510_20787_amd import workloads as wl
from tests.gpu_util import DeviceWorkload, dev
from tests.test_gpu_parity import make

pytestmark = pytest.mark.gpu


def clone_cache(cfg, cache):
    return B.wrap_cache(*(getattr(cache, f).clone() for f in ("k_win", "v_win", "win_score", "k_ret", "v_ret", "ret_score",
                                                              "ret_pos", "ret_count", "n_seen", "n_scored")))


def same_state(a, b):
    return all(torch.equal(getattr(a, f), getattr(b, f)) for f in ("k_win", "v_win", "k_ret", "v_ret", "ret_score", "ret_pos",
                                                                    "ret_count", "n_seen", "n_scored"))


def same_valid_state(a, b):
    """Equality of what the contract defines: compact slots past ret_count keep whatever an earlier call left there."""
    if not all(torch.equal(getattr(a, f), getattr(b, f)) for f in ("k_win", "v_win", "win_score", "ret_count", "n_seen", "n_scored")):
        return False
    valid = torch.arange(a.ret_pos.shape[2], device="cuda")[None, None, :] < a.ret_count[:, :, None]
    return all(torch.equal(getattr(a, f)[valid], getattr(b, f)[valid]) for f in ("k_ret", "v_ret", "ret_score", "ret_pos"))


@pytest.mark.parametrize("name,lazy", [("bf16_d64", False), ("bf16_d128_gqa", False), ("bf16_d64_deep", False),
                                       ("bf16_d64", True), ("f32_ragged_gqa", True)])
def test_decode_steps_replayed_from_a_graph(name, lazy):
    w = make(name)
    d = DeviceWorkload(w)
    dt = w.dtype
    cache = d.new_cache()
    B.ltea_prefill(d.cfg, d.cnn, d.q, d.k, d.v, d.cu, d.max_seqlen, cache)
    twin = clone_cache(d.cfg, cache)
    steps_per_graph = 3
    td = B.torch_dtype(dt)
    qs = torch.zeros((steps_per_graph, w.n_seqs, w.Hq, w.D), dtype=td, device="cuda")
    ks = torch.zeros((steps_per_graph, w.n_seqs, w.Hkv, w.D), dtype=td, device="cuda")
    vs = torch.zeros_like(ks)
    outs = torch.zeros_like(qs)
    ws = B.decode_workspace(d.cfg, None if lazy else d.cnn, w.n_seqs)
    status = torch.zeros(1, dtype=torch.int32, device="cuda")

    def enqueue(c, o, wsp):
        for i in range(steps_per_graph):
            if lazy:
                B.ltea_decode_step_lazy(d.cfg, qs[i], ks[i], vs[i], c, out=o[i], status=status, workspace=wsp)
            else:
                B.ltea_decode_step(d.cfg, d.cnn, qs[i], ks[i], vs[i], c, out=o[i], workspace=wsp)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # warm the capture stream up as torch asks
        enqueue(clone_cache(d.cfg, cache), torch.zeros_like(outs), B.decode_workspace(d.cfg, None if lazy else d.cnn, w.n_seqs))
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    snapshot = clone_cache(d.cfg, cache)
    with torch.cuda.graph(graph):
        enqueue(cache, outs, ws)
    torch.cuda.synchronize()
    # capturing does not execute: the state is untouched
    assert same_state(cache, snapshot)
    ws2 = B.decode_workspace(d.cfg, None if lazy else d.cnn, w.n_seqs)
    outs_twin = torch.zeros_like(outs)
    period = B.ltea_lazy_period(d.cfg, d.cnn)
    done = 0
    for replay in range(5):
        for i in range(steps_per_graph):
            q, k, v = wl.decode_inputs(w.seed, replay * steps_per_graph + i, dt, w.n_seqs, w.Hq, w.Hkv, w.D)
            qs[i].copy_(dev(q, dt)); ks[i].copy_(dev(k, dt)); vs[i].copy_(dev(v, dt))
        if lazy and done + steps_per_graph > period:
            B.ltea_rescore(d.cfg, d.cnn, cache)
            B.ltea_rescore(d.cfg, d.cnn, twin)
            done = 0
        graph.replay()
        # eager work of the program's own between the replays, then a synchronisation
        scratch = (outs.float() * 2).sum()
        enqueue(twin, outs_twin, ws2)
        torch.cuda.synchronize()
        done += steps_per_graph
        assert torch.equal(outs, outs_twin), f"replay {replay}"
        assert same_state(cache, twin), f"replay {replay}"
        assert bool(torch.isfinite(scratch))
    assert int(status.item()) == 0


def test_prefill_replayed_from_a_graph():
    w = make("bf16_d64_deep")
    d = DeviceWorkload(w)
    cache = d.new_cache()
    out = torch.zeros((w.total_tokens, w.Hq, w.D), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(max(B.ltea_workspace_bytes(d.cfg, d.cnn, w.n_seqs, w.total_tokens, d.max_seqlen), 16), dtype=torch.uint8,
                     device="cuda")
    q, k, v = d.q.clone(), d.k.clone(), d.v.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        B.ltea_prefill(d.cfg, d.cnn, q, k, v, d.cu, d.max_seqlen, d.new_cache(), out=torch.zeros_like(out), workspace=ws.clone())
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        B.ltea_prefill(d.cfg, d.cnn, q, k, v, d.cu, d.max_seqlen, cache, out=out, workspace=ws)
    rng = np.random.default_rng(3)
    for replay in range(3):
        # new inputs in place: a permutation of the heads gives different but equally well-formed tensors
        perm = torch.from_numpy(rng.permutation(w.Hkv)).cuda()
        k.copy_(d.k[:, perm]); v.copy_(d.v[:, perm])
        graph.replay()
        ref_cache = d.new_cache()
        ref = B.ltea_prefill(d.cfg, d.cnn, q, k, v, d.cu, d.max_seqlen, ref_cache)
        torch.cuda.synchronize()
        assert torch.equal(out, ref), f"replay {replay}"
        assert same_valid_state(cache, ref_cache), f"replay {replay}"
