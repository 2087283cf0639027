"""CPU-only checks of the host-side index builder (bs_index_build): the blob is walked here in plain Python and
must return exactly what the brute-force oracle lookup returns (Sec. 3.2: longest occurring suffix of the last
tokens, then the most frequent continuation, ties to the smaller id, never across rollouts)."""
import numpy as np
import pytest

from oracle.lookup import lookup
from paper_2605_08862_amd import binding as B

MAGIC = 0x42535849


@pytest.fixture(scope="module", autouse=True)
def _lib():
    import os
    if not os.path.exists(B.LIB_PATH):
        from paper_2605_08862_amd import build
        build.build()
    return B.lib()


def _flatten(prompts):
    """prompts: list of prompts, each a list of rollouts (lists of ints) -> (pool_tokens, rollout_offsets, prompt_rollout_begin)."""
    toks, ro, pb = [], [0], [0]
    for rollouts in prompts:
        for r in rollouts:
            toks.extend(r)
            ro.append(len(toks))
        pb.append(len(ro) - 1)
    return np.array(toks, dtype=np.int32), np.array(ro, dtype=np.int64), np.array(pb, dtype=np.int32)


class _Blob:
    def __init__(self, a):
        assert a[0] == MAGIC
        self.np_, self.ns, self.ne = int(a[1]), int(a[2]), int(a[3])
        o = 8
        self.root = a[o:o + self.np_]; o += self.np_
        self.eb = a[o:o + self.ns + 1]; o += self.ns + 1
        self.bt = a[o:o + self.ns]; o += self.ns
        self.bn = a[o:o + self.ns]; o += self.ns
        self.et = a[o:o + self.ne]; o += self.ne
        self.en = a[o:o + self.ne]; o += self.ne
        assert o == len(a)

    def walk(self, prompt, tail, max_match, min_match, k_max):
        tail = [int(t) for t in tail][-max_match:]
        mm = 0
        while mm < len(tail) and tail[len(tail) - 1 - mm] >= 0:
            mm += 1
        st = -1
        if self.root[prompt] >= 0:
            for m in range(mm, min_match - 1, -1):
                v = int(self.root[prompt])
                for t in tail[len(tail) - m:]:
                    lo, hi = int(self.eb[v]), int(self.eb[v + 1])
                    seg = self.et[lo:hi]
                    assert np.all(seg[1:] > seg[:-1])                      # sorted, distinct
                    i = int(np.searchsorted(seg, t))
                    v = int(self.en[lo + i]) if i < len(seg) and seg[i] == t else -1
                    if v < 0:
                        break
                if v >= 0:
                    st = v
                    break
        out = []
        while st >= 0 and len(out) < k_max and self.bt[st] >= 0:
            out.append(int(self.bt[st]))
            st = int(self.bn[st])
        return out


def test_hand_worked_cases_through_the_index():
    pool = [[1, 2, 3, 4, 5, 6], [9, 2, 3, 4, 7, 8], [2, 3, 4, 7, 1]]
    blob = _Blob(B.bs_index_build(*_flatten([pool])))
    cases = [([0, 2, 3, 4], 4, 1, 3), ([1, 2, 3, 4], 4, 1, 8), ([5, 5, 5, 7], 4, 1, 2), ([4, 5, 6], 4, 1, 4),
             ([42, 43], 4, 1, 4), ([6, 9], 2, 2, 4), ([-1, -1, -1, 3], 4, 1, 2), ([-1, -1, -1, 3], 4, 2, 2),
             ([2, 3, 4], 4, 1, 0)]
    for tail, mx, mn, k in cases:
        pad = [-1] * (mx - len(tail)) + tail
        assert blob.walk(0, pad, mx, mn, k) == lookup(pool, tail, mx, mn, k), (tail, mx, mn, k)


@pytest.mark.parametrize("vocab,seed", [(3, 1), (5, 2), (40, 3), (1000, 4)])
def test_random_pools_match_the_oracle(vocab, seed):
    """Small vocabularies give dense, competing matches (ties, repeats, clones in the automaton); several prompts,
    an empty rollout, a prompt without tokens."""
    rng = np.random.default_rng(seed)
    prompts = []
    for p in range(5):
        n_r = int(rng.integers(1, 6))
        prompts.append([[int(x) for x in rng.integers(0, vocab, int(rng.integers(0, 60)))] for _ in range(n_r)])
    prompts[3] = [[], []]                                                   # no tokens at all
    prompts[1][0] = []                                                      # an empty rollout among others
    blob = _Blob(B.bs_index_build(*_flatten(prompts)))
    assert blob.root[3] == -1
    for trial in range(400):
        p = int(rng.integers(0, 5))
        mx = int(rng.integers(1, 9)); mn = int(rng.integers(1, mx + 1)); k = int(rng.integers(0, 12))
        flat = [t for r in prompts[p] for t in r]
        if flat and rng.random() < 0.7:                                     # a tail that occurs in the pool
            s = int(rng.integers(0, len(flat)))
            tail = flat[max(0, s - mx + 1):s + 1]
        else:
            tail = [int(x) for x in rng.integers(0, vocab, mx)]
        tail = [-1] * (mx - len(tail)) + tail
        assert blob.walk(p, tail, mx, mn, k) == lookup(prompts[p], tail, mx, mn, k), (p, tail, mx, mn, k)


def test_builder_rejects_bad_input():
    toks, ro, pb = _flatten([[[1, 2, 3]]])
    bad = toks.copy(); bad[1] = -5
    with pytest.raises(B.BsError):
        B.bs_index_build(bad, ro, pb)
    with pytest.raises(B.BsError):
        B.bs_index_build(toks, np.array([0, 5, 3], dtype=np.int64), np.array([0, 2], dtype=np.int32))
