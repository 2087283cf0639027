"""GPU parity of the draft lookup against the brute-force oracle: bit-exact token ids and lengths."""
import numpy as np
import pytest
import torch

from oracle.lookup import lookup as oracle_lookup
from paper_2605_08862_amd import binding as Bn
from paper_2605_08862_amd import workloads as W
from paper_2605_08862_amd.runtime import Engine, fuse_weights
from tests import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _engine(B_max, k_max):
    desc = W.shape("tiny")
    w = W.make_weights(desc, seed=3)
    return Engine(desc, fuse_weights(w, desc["dtype"], DEV), 1, 64, B_max=B_max, k_max=k_max)


def _check(eng, pool, seq_prompt, tails, max_match, min_match, k_max):
    """Both retrieval paths against the oracle: the pool scan, then the prebuilt index (bs_index_build on the
    host, bound with bs_index_bind)."""
    toks, off, prb = pool
    eng.pool_bind(torch.tensor(toks), torch.tensor(off), torch.tensor(prb))
    refs = []
    for b in range(len(seq_prompt)):
        p = seq_prompt[b]
        rollouts = [toks[off[r]:off[r + 1]] for r in range(prb[p], prb[p + 1])]
        refs.append(oracle_lookup(rollouts, tails[b], max_match, min_match, k_max))
    for path in ("scan", "index"):
        eng.index_bind(Bn.bs_index_build(toks, off, prb) if path == "index" else None)
        dt, dl = eng.draft_lookup(H.dev_i32(seq_prompt), H.dev_i32(tails), max_match, min_match, k_max)
        dt, dl = dt.cpu().numpy(), dl.cpu().numpy()
        for b, ref in enumerate(refs):
            assert dl[b] == len(ref), (path, b, dl[b], ref, dt[b])
            assert list(dt[b][:dl[b]]) == ref, (path, b, dt[b], ref)
            assert all(t == -1 for t in dt[b][dl[b]:])
    eng.index_bind(None)
    return sum(len(r) > 0 for r in refs)


def test_small_vocab_dense_matches():
    """Tiny vocabularies: thousands of occurrences per context (pool rescans, hash-table class splitting),
    ties, rollout boundaries, padding."""
    eng = _engine(64, 16)
    for seed, V, n_roll, length in [(1, 2, 3, 50), (2, 3, 4, 400), (3, 5, 8, 3000), (4, 50, 8, 3000)]:
        rng = np.random.default_rng(seed)
        lens = rng.integers(1, length, size=2 * n_roll)
        off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
        toks = rng.integers(0, V, size=int(off[-1]), dtype=np.int32)
        prb = np.array([0, n_roll, 2 * n_roll], dtype=np.int32)
        B = 48
        seq_prompt = rng.integers(0, 2, B).astype(np.int32)
        tails = rng.integers(0, V, (B, 4)).astype(np.int32)
        tails[rng.random(B) < 0.2, 0] = -1
        tails[rng.random(B) < 0.1, :3] = -1
        for mm in (1, 2):
            assert _check(eng, (toks, off, prb), seq_prompt, tails, 4, mm, 16) > 0
    eng.close()


def test_many_distinct_successors():
    """One context followed by > 4096 distinct tokens: exercises the residue-class counting."""
    eng = _engine(4, 8)
    n = 6000
    toks = np.empty(2 * n + 40, dtype=np.int32)
    toks[0:2 * n:2] = 7
    toks[1:2 * n:2] = 100 + np.arange(n)
    toks[2 * n:] = np.tile([7, 105], 20)          # token 105 follows 7 most often
    off = np.array([0, len(toks)], dtype=np.int64)
    prb = np.array([0, 1], dtype=np.int32)
    tails = np.array([[-1, -1, -1, 7]] * 2, dtype=np.int32)
    assert _check(eng, (toks, off, prb), np.zeros(2, np.int32), tails, 4, 1, 8) == 2
    eng.close()


def test_pool_stress_shape():
    """Configuration-5 shape at reduced count: 8 prompts x 8 rollouts (lognormal lengths, median 8k), 152k
    vocabulary, tails planted in the pool, k_max 16."""
    eng = _engine(64, 16)
    pool = W.make_pool(5005, 8, 8, 8192, 151936)
    seq_prompt, tails = W.plant_tails(5006, pool, 64, 8, 4, vocab=151936)
    hits = _check(eng, pool, seq_prompt, tails, 4, 1, 16)
    assert hits >= 32
    eng.close()
