"""GPU parity of the top-k / top-p filtered target distribution (Sec. 3.2: p_t "after temperature scaling and any
top-p/top-k filtering") against oracle/accept.py on the same float32 logits: the kept set of every row (exact; a
top-p boundary within 1e-8 of the cumulative mass is counted as a tie), the renormalisation, the integers of the
accept / resample step, the law of the emitted token, and the fused bf16 path of a small model."""
import numpy as np
import pytest
import torch
from scipy import stats

from oracle import accept as OA
from paper_2605_08862_amd import binding as B
from paper_2605_08862_amd import workloads as W
from paper_2605_08862_amd.runtime import Engine, fuse_weights
from tests import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def eng():
    desc = W.shape("tiny")
    w = W.make_weights(desc, seed=3)
    e = Engine(desc, fuse_weights(w, desc["dtype"], DEV), 1, 64, B_max=4096, k_max=8)
    yield e
    e.set_filter(0, 1.0)
    e.close()


def _call(eng, logits, drafts, k_b, ua, us, q=None, **kw):
    k_max = drafts.shape[1]
    qd = None if q is None else torch.as_tensor(q).to(DEV)
    return eng.accept_resample(H.dev_i32(drafts), H.dev_i32(k_b), k_max, H.dev_f32(ua), H.dev_f32(us), q_logits=qd,
                               logits=H.dev_f32(logits), **kw)


def _check_thresholds(eng, logits, T, top_k, top_p):
    """Device threshold of every row against the oracle's kept set; returns the number of boundary ties."""
    M, V = logits.shape
    key, idx, lse = (t.cpu().numpy() for t in B.bs_debug_filter_rows(eng.ctx, M))
    ties = 0
    for r in range(M):
        keep, margin = OA.kept_tokens(logits[r], T, top_k, top_p)
        got = H.device_kept(logits[r], key[r], idx[r])
        if not np.array_equal(got, np.sort(keep)):
            assert margin <= H.FILTER_TIE, (r, T, top_k, top_p, len(got), len(keep), margin)
            ties += 1
            continue
        x = logits[r].astype(np.float64) / T
        ref = x.max() + np.log(np.exp(x[keep] - x.max()).sum())
        assert abs(lse[r] - ref) <= 2e-6 * max(1.0, abs(ref)), (r, lse[r], ref)
    return ties


@pytest.mark.parametrize("V,T,top_k,top_p", [
    (37, 1.0, 5, 1.0), (37, 1.0, 0, 0.9), (37, 0.7, 5, 0.5), (1000, 1.3, 1, 1.0), (1000, 1.0, 999, 0.999),
    (4096, 1.0, 50, 0.95), (4096, 0.7, 0, 0.05), (4093, 1.0, 2048, 0.3), (513, 1.0, 0, 1e-6), (4096, 1.0, 4096, 0.9)])
def test_kept_set_of_every_row_matches_the_oracle(eng, V, T, top_k, top_p):
    rng = np.random.default_rng(V + top_k)
    Bn, k_max = 24, 3
    k_b = rng.integers(0, k_max + 1, Bn)
    M = int(k_b.sum() + Bn)
    logits = rng.normal(0, 2.0, (M, V)).astype(np.float32)
    logits[1] = np.round(logits[1])                      # many exact ties, also at the threshold
    logits[2] = 0.25                                     # a constant row: only the index cut decides
    logits[3, ::3] = -np.inf                             # masked tokens have no mass
    logits[4, :5] = [0.0, -0.0, 0.0, -0.0, 0.0]          # the two zeros rank equal
    drafts = rng.integers(0, V, (Bn, k_max)).astype(np.int32)
    ua, us = W.uniforms(V, Bn, k_max)
    eng.set_filter(top_k, top_p)
    out = _call(eng, logits, drafts, k_b.astype(np.int32), ua, us, temperature=T)
    assert _check_thresholds(eng, logits, T, top_k, top_p) <= 1
    exact, near, _ = H.compare_sampler(out, logits, drafts, k_b, ua, us, None, T, top_k=top_k, top_p=top_p)
    assert near <= 2, (exact, near)
    assert eng.poll_status() == 0


def test_filtered_accept_and_resample_integers_match_the_oracle(eng):
    """Ragged blocks, dense and one-hot proposals, greedy drafts so that many are accepted, EOS and no-bonus."""
    rng = np.random.default_rng(77)
    for V, T, q_mode, eos, bonus, top_k, top_p in [(1000, 1.0, "bf16", -1, True, 40, 0.9), (2049, 0.8, "f32", -1, True, 0, 0.7),
                                                   (333, 1.2, None, 5, True, 8, 1.0), (512, 1.0, "f32", -1, False, 100, 0.5),
                                                   (700, 0.0, None, -1, True, 3, 0.5)]:
        Bn, k_max = 150, 8
        k_b = rng.integers(0, k_max + 1, Bn)
        M, Td = int(k_b.sum() + Bn), int(k_b.sum())
        logits = rng.normal(0, 2.5, (M, V)).astype(np.float32)
        drafts = rng.integers(0, V, (Bn, k_max)).astype(np.int32)
        r0 = np.concatenate([[0], np.cumsum(k_b + 1)])
        for b in range(Bn):
            for j in range(k_b[b]):
                if rng.random() < 0.7:                     # a likely draft: one of the row's top tokens
                    drafts[b, j] = int(np.argsort(-logits[r0[b] + j])[rng.integers(0, 3)])
        q = qn = None
        if q_mode and Td > 0:
            qt = torch.tensor(rng.normal(0, 2.0, (Td, V)), dtype=torch.bfloat16 if q_mode == "bf16" else torch.float32)
            q, qn = qt, qt.float().numpy()
        ua, us = W.uniforms(V + 1, Bn, k_max)
        eng.set_filter(top_k, top_p)
        out = _call(eng, logits, drafts, k_b.astype(np.int32), ua, us, q=q, temperature=T, eos_id=eos, emit_bonus=bonus)
        exact, near, res = H.compare_sampler(out, logits, drafts, k_b, ua, us, qn, T, eos, bonus, top_k=top_k, top_p=top_p)
        assert near <= 3, (V, exact, near)
        if T > 0:                                          # every emitted token lies in its row's kept set
            toks, n_emit, n_acc = (out[k].cpu().numpy() for k in ("out_tokens", "n_emitted", "n_accepted"))
            for b in range(Bn):
                for i in range(n_emit[b]):
                    keep, _ = OA.kept_tokens(logits[r0[b] + i], T, top_k, top_p)
                    assert toks[b, i] in keep, (b, i)
    assert eng.poll_status() == 0


def test_filter_off_is_the_unfiltered_step_bit_for_bit(eng):
    rng = np.random.default_rng(9)
    V, Bn, k_max = 777, 64, 4
    k_b = rng.integers(0, k_max + 1, Bn).astype(np.int32)
    logits = rng.normal(0, 2.0, (int(k_b.sum() + Bn), V)).astype(np.float32)
    drafts = rng.integers(0, V, (Bn, k_max)).astype(np.int32)
    ua, us = W.uniforms(5, Bn, k_max)
    eng.set_filter(0, 1.0)
    ref = _call(eng, logits, drafts, k_b, ua, us)
    for top_k, top_p in ((V, 1.0), (V + 10, 2.0), (-3, 1.0)):
        eng.set_filter(top_k, top_p)
        out = _call(eng, logits, drafts, k_b, ua, us)
        for k in ref:
            assert torch.equal(out[k], ref[k]), (top_k, top_p, k)
    eng.set_filter(1, 1.0)                                 # top_k = 1: every emitted token is its row's arg-max
    out = _call(eng, logits, drafts, k_b, ua, us)
    eng.set_filter(0, 1.0)
    greedy = _call(eng, logits, drafts, k_b, ua, us, temperature=0.0)
    for k in ("n_accepted", "out_tokens", "n_emitted"):
        assert torch.equal(out[k], greedy[k]), k
    with pytest.raises(B.BsError):
        B.bs_set_filter(eng.ctx, 5, 0.0, None)


@pytest.mark.parametrize("mode", ["dense_q", "one_hot"])
def test_device_output_law_is_the_filtered_target(eng, mode):
    rng = np.random.default_rng(303)
    V, Bn, rounds, top_k, top_p = 16, 4096, 20, 9, 0.9
    z = rng.normal(0, 1.5, (2, V)).astype(np.float32)
    ql = rng.normal(0, 1.5, (1, V)).astype(np.float32)
    ref = OA.filtered_probs(z[0], 1.0, top_k, top_p)
    from scipy.special import softmax
    q = softmax(ql[0].astype(np.float64))
    eng.set_filter(top_k, top_p)
    counts = np.zeros(V)
    for r in range(rounds):
        drafts = (rng.choice(V, size=(Bn, 1), p=q) if mode == "dense_q" else np.full((Bn, 1), int(np.argmax(ref)))).astype(np.int32)
        ua, us = W.uniforms(9000 + r, Bn, 1)
        out = _call(eng, np.tile(z, (Bn, 1)), drafts, np.ones(Bn, np.int32), ua, us,
                    q=np.tile(ql, (Bn, 1)) if mode == "dense_q" else None)
        counts += np.bincount(out["out_tokens"].cpu().numpy()[:, 0], minlength=V)
    assert counts[ref == 0].sum() == 0
    nz = ref > 0
    n = counts.sum()
    chi2 = ((counts[nz] - n * ref[nz]) ** 2 / (n * ref[nz])).sum()
    assert stats.chi2.sf(chi2, df=nz.sum() - 1) > 1e-4, chi2


def test_full_vocabulary_rows(eng):
    """Rows of the bench's vocabulary size (151936) through a context of that vocabulary: near-flat rows (the
    synthetic models' regime, where the nucleus holds most of the vocabulary) and peaked ones."""
    desc = W.shape("s1p5b", n_layers=1)
    w = W.make_weights(desc, seed=1, device=DEV)
    big = Engine(desc, fuse_weights(w, desc["dtype"], DEV), 1, 64, B_max=8, k_max=1)
    try:
        rng = np.random.default_rng(4)
        V, Bn = desc["vocab"], 8
        k_b = np.array([1, 0, 1, 1, 0, 1, 1, 1], np.int32)
        M = int(k_b.sum() + Bn)
        logits = rng.normal(0, 0.3, (M, V)).astype(np.float32)
        logits[::2] *= 12.0                               # peaked rows
        logits[3] = np.round(logits[3] * 4) / 4           # a few distinct values, tens of thousands of tokens each:
        logits[5] = -1.5                                  # more equal keys than the kernel's LDS list holds
        logits[6] = np.round(logits[6])
        drafts = np.array([[int(np.argmax(logits[i]))] for i in np.concatenate([[0], np.cumsum(k_b + 1)])[:-1]], np.int32)
        ua, us = W.uniforms(11, Bn, 1)
        for top_k, top_p in ((50, 0.9), (0, 0.95), (20000, 1.0)):
            big.set_filter(top_k, top_p, )
            out = big.accept_resample(H.dev_i32(drafts), H.dev_i32(k_b), 1, H.dev_f32(ua), H.dev_f32(us),
                                      logits=H.dev_f32(logits))
            assert _check_thresholds(big, logits, 1.0, top_k, top_p) <= 1
            exact, near, _ = H.compare_sampler(out, logits, drafts, k_b, ua, us, None, 1.0, top_k=top_k, top_p=top_p)
            assert near <= 1
        assert big.poll_status() == 0
    finally:
        big.close()


def test_bf16_model_fused_path_with_filter():
    """bs_verify_step + bs_accept_resample of a small bf16 model: the filtered step on the fused LM-head path
    (logits written to the caller's scratch) equals the oracle's rule on the logits the same step reports."""
    desc = W.shape("mini_bf16")
    Bn, k_max, V = 12, 4, desc["vocab"]
    w = W.make_weights(desc, seed=8)
    eng = Engine(desc, fuse_weights(w, desc["dtype"], DEV), Bn, 128, B_max=Bn, k_max=k_max)
    try:
        rng = np.random.default_rng(8)
        slots = H.dev_i32(np.arange(Bn))
        last = rng.integers(0, V, Bn).astype(np.int32)
        drafts = rng.integers(0, V, (Bn, k_max)).astype(np.int32)
        k_b = rng.integers(0, k_max + 1, Bn).astype(np.int32)
        ua, us = W.uniforms(3, Bn, k_max)
        with pytest.raises(B.BsError):                     # bf16 model, filter on, no scratch
            B.bs_set_filter(eng.ctx, 5, 1.0, None)
            eng.verify_step(slots, H.dev_i32(last), H.dev_i32(drafts), H.dev_i32(k_b), k_max)
            eng.accept_resample(H.dev_i32(drafts), H.dev_i32(k_b), k_max, H.dev_f32(ua), H.dev_f32(us))
        for top_k, top_p, T in ((20, 0.9, 1.0), (0, 0.6, 0.8), (3, 1.0, 1.0)):
            eng.set_filter(top_k, top_p)
            logits = eng.verify_step(slots, H.dev_i32(last), H.dev_i32(drafts), H.dev_i32(k_b), k_max, want_logits=True)
            out = eng.accept_resample(H.dev_i32(drafts), H.dev_i32(k_b), k_max, H.dev_f32(ua), H.dev_f32(us), temperature=T)
            M = int(k_b.sum() + Bn)
            z = logits[:M].cpu().numpy()
            assert _check_thresholds(eng, z, T, top_k, top_p) <= 1
            exact, near, _ = H.compare_sampler(out, z, drafts, k_b, ua, us, None, T, top_k=top_k, top_p=top_p)
            assert near <= 2, (exact, near)
        assert eng.poll_status() == 0
    finally:
        eng.close()
