"""The step under HIP graph capture: every entry point only enqueues kernels on the caller's stream (no host
synchronisation, no allocation, no memset nodes), so a caller may capture verify -> accept -> commit once and
replay it.  Replays are checked against eager runs of the same inputs, several times, with eager work and
synchronisations in between."""
import time

import numpy as np
import pytest
import torch

from paper_2605_08862_amd import workloads as W
from paper_2605_08862_amd.runtime import Engine, fuse_weights
from tests import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _setup(desc, Bn, k_max, ctx_lens, seed):
    w = W.make_weights(desc, seed=seed)
    eng = Engine(desc, fuse_weights(w, desc["dtype"], DEV), Bn, int(max(ctx_lens)) + 4 * (k_max + 1), B_max=Bn,
                 k_max=k_max, page_perm_seed=5)
    for b in range(Bn):
        if ctx_lens[b] > 0:
            for l, (k, v) in enumerate(W.context_kv(desc, int(ctx_lens[b]), seed * 100 + b)):
                eng.kv_write(l, b, 0, k.to(DEV), v.to(DEV))
    return eng


@pytest.mark.parametrize("shape,q_mode", [("mini_bf16", "onehot"), ("mini_bf16", "dense"), ("tiny", "dense")])
def test_step_replays_from_a_hip_graph(shape, q_mode):
    desc = W.shape(shape)
    Bn, k_max, V = 6, 4, desc["vocab"]
    ctx_lens = [70, 0, 130, 64, 5, 257]
    eng = _setup(desc, Bn, k_max, ctx_lens, seed=41)
    rng = np.random.default_rng(41)
    ctx0 = H.dev_i32(ctx_lens)
    slots = H.dev_i32(np.arange(Bn))
    last, drafts = H.dev_i32(rng.integers(0, V, Bn)), H.dev_i32(rng.integers(0, V, (Bn, k_max)))
    dl = H.dev_i32([4, 0, 3, 4, 1, 2])
    ua, us = (torch.tensor(a).to(DEV) for a in W.uniforms(5, Bn, k_max))
    q = None
    if q_mode == "dense":
        q = torch.randn(int(dl.sum().item()), V, device=DEV).to(torch.bfloat16 if desc["dtype"] == W.BS_BF16 else torch.float32)

    def step():
        eng.ctx_len.copy_(ctx0)
        eng.verify_step(slots, last, drafts, dl, k_max)
        out = eng.accept_resample(drafts, dl, k_max, ua, us, q_logits=q)
        eng.kv_commit(slots, out["n_accepted"] + 1)
        return out

    for _ in range(2):                                   # eager warm-up (also sets the kernels' LDS attributes)
        step()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            out_g = step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for trial in range(4):
        last.copy_(H.dev_i32(rng.integers(0, V, Bn)))
        drafts.copy_(H.dev_i32(rng.integers(0, V, (Bn, k_max))))
        a, s = W.uniforms(50 + trial, Bn, k_max)
        ua.copy_(torch.tensor(a).to(DEV)); us.copy_(torch.tensor(s).to(DEV))
        ref = {k: v.clone() for k, v in step().items()}
        ref_ctx = eng.ctx_len.clone()
        scratch = torch.randn(1 << 20, device=DEV).sum()              # unrelated eager work between replays
        torch.cuda.synchronize()
        eng.ctx_len.fill_(-7)                                         # the replay must restore and advance it itself
        graph.replay()
        torch.cuda.synchronize()
        for k in ref:
            assert torch.equal(out_g[k], ref[k]), (trial, k)
        assert torch.equal(eng.ctx_len, ref_ctx), trial
        assert torch.isfinite(scratch)
    assert eng.poll_status() == 0
    # launch-bound regime: wall time of a replay against the eager step (printed, not asserted)
    def wall(f, n=20):
        torch.cuda.synchronize(); t0 = time.perf_counter()
        for _ in range(n):
            f()
        torch.cuda.synchronize(); return (time.perf_counter() - t0) / n * 1e3
    print("eager %.3f ms, graph replay %.3f ms per step (%s, B=%d, k=%d)" % (wall(step), wall(graph.replay), shape, Bn, k_max))
    eng.close()


def test_replay_with_changing_row_counts_on_the_large_batch_paths():
    """The captured step has fixed grids; the row count lives on the device.  On a model wide enough for the
    large-batch launch paths (row limit 48 x 17 = 816 > 640: 128-row gate/up kernel, residual projections whose tile
    and K split follow the row count, RMSNorm summing that many slabs) the draft lengths are rewritten between
    replays - every block full (816 rows), mixed (about 430), no drafts at all (48) - and each replay must equal the
    eager step on the same inputs bit for bit."""
    desc = W.shape("mini_bf16", n_layers=1, d_model=3840, n_q_heads=16, n_kv_heads=4, d_ffn=512, vocab=640)
    Bn, k_max, V = 48, 16, desc["vocab"]
    rng = np.random.default_rng(43)
    ctx_lens = [int(x) for x in rng.integers(0, 150, Bn)]
    eng = _setup(desc, Bn, k_max, ctx_lens, seed=43)
    ctx0 = H.dev_i32(ctx_lens)
    slots = H.dev_i32(np.arange(Bn))
    last, drafts = H.dev_i32(rng.integers(0, V, Bn)), H.dev_i32(rng.integers(0, V, (Bn, k_max)))
    dl = H.dev_i32([16] * Bn)
    ua, us = (torch.tensor(a).to(DEV) for a in W.uniforms(6, Bn, k_max))

    def step():
        eng.ctx_len.copy_(ctx0)
        eng.verify_step(slots, last, drafts, dl, k_max)
        out = eng.accept_resample(drafts, dl, k_max, ua, us)
        eng.kv_commit(slots, out["n_accepted"] + 1)
        return out

    for _ in range(2):
        step()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            out_g = step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    lengths = [[16] * Bn, [int(x) for x in rng.integers(0, 17, Bn)], [0] * Bn, [16] * Bn, [int(x) for x in rng.integers(0, 17, Bn)]]
    for trial, k_b in enumerate(lengths):
        dl.copy_(H.dev_i32(k_b))
        drafts.copy_(H.dev_i32(rng.integers(0, V, (Bn, k_max))))
        ref = {k: v.clone() for k, v in step().items()}
        ref_ctx = eng.ctx_len.clone()
        torch.cuda.synchronize()
        eng.ctx_len.fill_(-7)
        graph.replay()
        torch.cuda.synchronize()
        for k in ref:
            assert torch.equal(out_g[k], ref[k]), (trial, k)
        assert torch.equal(eng.ctx_len, ref_ctx), trial
        assert int(out_g["n_emitted"].sum().item()) >= Bn
    assert eng.poll_status() == 0
    eng.close()
