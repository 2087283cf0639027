"""GPU parity, tiny float32 decoder (configuration 1): prefill through the library, speculative
decode steps with every proposal mode, checked element by element against the oracle."""
import numpy as np
import pytest
import torch

from oracle import accept as OA
from oracle import decoder as OD
from paper_2605_08862_amd import workloads as W
from paper_2605_08862_amd.runtime import Engine, fuse_weights
from tests import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _setup(k_max=15, n_slots=4, max_ctx=320, perm=7):
    desc = W.shape("tiny")
    w = W.make_weights(desc, seed=1001)
    eng = Engine(desc, fuse_weights(w, desc["dtype"], DEV), n_slots, max_ctx, B_max=n_slots, k_max=k_max,
                 page_perm_seed=perm)
    return desc, W.weights_to_numpy(w), eng


def _prefill(desc, wn, eng, prompts, chunk=16):
    """Prefill via verify_step + forced commit; returns oracle caches, last logits of both sides."""
    od = H.oracle_desc(desc)
    Bn = len(prompts)
    caches = [OD.SeqCache(od) for _ in range(Bn)]
    slots = H.dev_i32(np.arange(Bn))
    worst = 0.0
    for lo in range(0, prompts.shape[1], chunk):
        blk = prompts[:, lo:lo + chunk]
        k = blk.shape[1] - 1
        dl = np.full(Bn, k, dtype=np.int32)
        logits = eng.verify_step(slots, H.dev_i32(blk[:, 0]), H.dev_i32(blk[:, 1:]), H.dev_i32(dl), k, want_logits=True)
        eng.kv_commit(slots, H.dev_i32(dl + 1))
        got = logits.cpu().numpy().reshape(Bn, k + 1, -1)
        for b in range(Bn):
            ref = OD.verify_block(od, wn, caches[b], blk[b])
            caches[b].commit(k + 1)
            worst = max(worst, np.abs(got[b] - ref).max())
    return caches, worst


def test_prefill_logits_and_cache_match_oracle():
    desc, wn, eng = _setup()
    rng = np.random.default_rng(1001)
    prompts = rng.integers(0, desc["vocab"], size=(4, 128))
    caches, worst = _prefill(desc, wn, eng, prompts)
    assert worst <= H.TOL_LOGITS[W.BS_F32], worst
    assert eng.ctx_len.cpu().tolist() == [128] * 4
    for b in range(4):
        for l in range(desc["n_layers"]):
            k, v = eng.kv_read(l, b, 0, 128)
            np.testing.assert_allclose(k.cpu().numpy(), caches[b].k[l], atol=2e-5)
            np.testing.assert_allclose(v.cpu().numpy(), caches[b].v[l], atol=2e-5)
    assert eng.poll_status() == 0


@pytest.mark.parametrize("mode", ["dense_q", "one_hot", "greedy", "k0", "ragged"])
def test_decode_trace_replay(mode):
    """64 new tokens per sequence (fewer steps when drafts are accepted).  The oracle runs each step first
    and records drafts, q, uniforms and outputs; the device replays the step; after a near-tie divergence the
    device is re-synchronised to the oracle's tokens."""
    desc, wn, eng = _setup()
    od = H.oracle_desc(desc)
    V, Bn, k_max = desc["vocab"], 4, 4
    rng = np.random.default_rng({"dense_q": 11, "one_hot": 12, "greedy": 13, "k0": 14, "ragged": 15}[mode])
    prompts = rng.integers(0, V, size=(Bn, 128))
    caches, _ = _prefill(desc, wn, eng, prompts[:, :127], chunk=127 // 8 + 1)
    last = prompts[:, 127].copy()
    slots = H.dev_i32(np.arange(Bn))
    T = 0.0 if mode == "greedy" else 1.0
    produced = np.zeros(Bn, dtype=int)
    stats = dict(exact=0, near=0, steps=0, emitted=0, accepted=0, worst=0.0)
    step = 0
    while produced.min() < 64 and step < 80:
        # ---- oracle side: build drafts by sequential decode on a scratch copy of the cache
        k_b = {"k0": np.zeros(Bn, int), "ragged": rng.integers(0, k_max + 1, Bn)}.get(mode, np.full(Bn, k_max))
        drafts = np.full((Bn, k_max), -1, dtype=np.int64)
        qlog = []
        for b in range(Bn):
            scratch = OD.SeqCache(od)
            scratch.fill(caches[b].k, caches[b].v)
            tok = last[b]
            for j in range(k_b[b]):
                z = OD.decode_token(od, wn, scratch, tok)
                p = OD.softmax(z)
                if mode == "greedy":
                    tok = int(np.argmax(z)) if rng.random() < 0.8 else int(rng.integers(V))
                else:
                    qd = 0.6 * p + 0.4 / V                      # true proposal: target sample w.p. 0.6 else uniform
                    tok = int(rng.choice(V, p=qd / qd.sum()))
                    qlog.append(np.log(qd).astype(np.float32))
                drafts[b, j] = tok
        q_rows = np.stack(qlog) if (mode in ("dense_q", "ragged") and qlog) else None
        ua, us = W.uniforms(5000 + step, Bn, k_max)
        blocks = H.pack_rows(last, drafts, k_b)
        ref_logits = [OD.verify_block(od, wn, caches[b], blocks[b]) for b in range(Bn)]
        ref = OA.verify_batch(np.concatenate(ref_logits), drafts, k_b, ua, us, q_rows, T)
        # ---- device side
        dt, dl = H.dev_i32(drafts), H.dev_i32(k_b)
        logits = eng.verify_step(slots, H.dev_i32(last), dt, dl, k_max, want_logits=True)
        out = eng.accept_resample(dt, dl, k_max, H.dev_f32(ua), H.dev_f32(us),
                                  q_logits=None if q_rows is None else H.dev_f32(q_rows), temperature=T)
        M = int(k_b.sum() + Bn)
        got_logits = logits.cpu().numpy()[:M]
        stats["worst"] = max(stats["worst"], np.abs(got_logits - np.concatenate(ref_logits)).max())
        # Tier A: oracle rule on the device's own logits
        ex, nr, _ = H.compare_sampler(out, got_logits, drafts, k_b, ua, us, q_rows, T)
        stats["exact"] += ex
        stats["near"] += nr
        # Tier C: end to end against the oracle on its own logits; re-sync on (flagged) divergence
        n_acc = np.array([r.n_accepted for r in ref])
        eng.kv_commit(slots, H.dev_i32(n_acc + 1))
        for b in range(Bn):
            caches[b].commit(int(n_acc[b]) + 1)
            last[b] = ref[b].tokens[-1]
            produced[b] += len(ref[b].tokens)
            stats["emitted"] += len(ref[b].tokens)
            stats["accepted"] += ref[b].n_accepted
        assert eng.ctx_len.cpu().tolist() == [c.committed for c in caches]
        step += 1
    stats["steps"] = step
    print(mode, stats)
    assert stats["worst"] <= H.TOL_LOGITS[W.BS_F32], stats
    assert stats["near"] <= max(2, 0.02 * (stats["exact"] + stats["near"])), stats
    if mode == "k0":
        assert stats["accepted"] == 0 and stats["emitted"] == step * Bn
    assert eng.poll_status() == 0


def test_device_faults_are_flagged_not_fatal():
    desc, wn, eng = _setup()
    from paper_2605_08862_amd import binding as B
    slots = H.dev_i32([0, 1, 2, 3])
    last = H.dev_i32([1, 2, 3, desc["vocab"] + 5])               # bad token id
    drafts = H.dev_i32(np.zeros((4, 4)))
    dl = H.dev_i32([4, 9, 0, 1])                                 # 9 > k_max
    eng.ctx_len.copy_(H.dev_i32([10, 11, 12, 13]))
    eng.verify_step(slots, last, drafts, dl, 4)
    ua, us = W.uniforms(5, 4, 4)
    out = eng.accept_resample(drafts, dl, 4, H.dev_f32(ua), H.dev_f32(us))
    eng.kv_commit(slots, out["n_accepted"] + 1)
    st = eng.poll_status()
    assert st & B.BS_FAULT_DRAFT_LEN and st & B.BS_FAULT_TOKEN_ID
    assert eng.poll_status() == 0                                # cleared
    # the two offending sequences (1: draft length, 3: token id) were skipped altogether, the others stepped
    n_emit, n_acc = out["n_emitted"].cpu().numpy(), out["n_accepted"].cpu().numpy()
    toks = out["out_tokens"].cpu().numpy()
    assert n_emit[1] == 0 and n_emit[3] == 0 and n_acc[1] == 0 and n_acc[3] == 0
    assert (toks[1] == -1).all() and (toks[3] == -1).all()
    assert n_emit[0] >= 1 and n_emit[2] == 1
    got_len = eng.kv_lengths(slots).cpu().tolist()
    assert got_len == eng.ctx_len.cpu().tolist() == [10 + int(n_acc[0]) + 1, 11, 12 + 1, 13]
    # a bad draft token (not only a bad last token) also skips its sequence; a bad token beyond k_b is never read
    drafts_bad = H.dev_i32([[0, -7, 0, 0], [0, 0, 0, 0], [0, 0, desc["vocab"], 0], [5, 5, 5, 5]])
    eng.verify_step(slots, H.dev_i32([1, 2, 3, 4]), drafts_bad, H.dev_i32([4, 4, 2, 4]), 4)
    out = eng.accept_resample(drafts_bad, H.dev_i32([4, 4, 2, 4]), 4, H.dev_f32(ua), H.dev_f32(us))
    assert eng.poll_status() == B.BS_FAULT_TOKEN_ID
    n_emit = out["n_emitted"].cpu().numpy()
    assert n_emit[0] == 0 and n_emit[1] >= 1 and n_emit[2] >= 1 and n_emit[3] >= 1
    # bs_kv_lengths: batch order, bad slot -> -1 + fault
    assert eng.kv_lengths(H.dev_i32([3, 0, 77])).cpu().tolist() == [13, 10 + int(n_acc[0]) + 1, -1]
    assert eng.poll_status() == B.BS_FAULT_SLOT
    eng.ctx_len.fill_(320 - 2)                                   # not enough room for k+1 rows
    eng.verify_step(slots, H.dev_i32([1, 2, 3, 4]), drafts, H.dev_i32([4, 4, 4, 4]), 4)
    assert eng.poll_status() & B.BS_FAULT_KV_PAGES
    eng.ctx_len.fill_(0)
    eng.verify_step(H.dev_i32([0, 0, 1, 99]), H.dev_i32([1, 2, 3, 4]), drafts, H.dev_i32([1, 1, 1, 1]), 4)
    assert eng.poll_status() & B.BS_FAULT_SLOT
