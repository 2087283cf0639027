"""Pins for the top-k / top-p filtering of oracle/accept.py (CPU only).

Sec. 3.2 defines p_t as the decoding distribution after temperature scaling and any top-p / top-k
filtering.  The kept set is pinned by what defines it (checked by an independent brute force), by closed
forms, by its special cases, and the verify loop with a filtered target by the exactness claim of Sec. 3.2."""
import itertools

import numpy as np
import pytest
from scipy import stats
from scipy.special import softmax

from oracle import accept as A


def _brute_kept(z, T, top_k, top_p):
    """Independent of the oracle's code: rank with Python's tuple sort, grow the set one token at a time and
    stop by the definition (size k reached, or the mass ranked before the next token already >= top_p of
    the top-k mass), in exact rational-free float64 arithmetic on scipy's softmax."""
    V = len(z)
    p = softmax(np.asarray(z, dtype=np.float64) / T)
    ranked = [j for _, j in sorted((-float(z[j]), j) for j in range(V))]
    if 0 < top_k < V:
        ranked = ranked[:top_k]
    if top_p >= 1.0:
        return ranked
    total = sum(p[j] for j in ranked)
    kept, before = [], 0.0
    for j in ranked:
        if kept and before >= top_p * total:
            break
        kept.append(j)
        before += p[j]
    return kept


@pytest.mark.parametrize("seed", range(6))
def test_kept_set_matches_brute_force_and_its_defining_properties(seed):
    rng = np.random.default_rng(seed)
    for V, T in ((7, 1.0), (33, 0.7), (128, 1.3)):
        z = rng.normal(0, 2.0, V)
        if seed % 2:                                       # exact ties: quantised logits
            z = np.round(z * 2) / 2
        for top_k, top_p in itertools.product((0, 1, 3, V - 1, V, V + 5), (1.0, 0.95, 0.5, 0.05, 1e-9)):
            keep, margin = A.kept_tokens(z, T, top_k, top_p)
            keep = [int(j) for j in keep]
            if margin < 1e-12:
                continue                                   # a tie in the cumulative mass: either set is valid
            assert keep == _brute_kept(z, T, top_k, top_p), (V, T, top_k, top_p)
            p = softmax(z / T)
            dropped = sorted(set(range(V)) - set(keep))
            # (1) a top set under the ranking (logit descending, index ascending)
            if dropped:
                worst_kept = max((-z[j], j) for j in keep)
                best_dropped = min((-z[j], j) for j in dropped)
                assert worst_kept < best_dropped
            # (2) size limit, (3) mass reaches top_p of the top-k mass and is minimal
            k_eff = top_k if 0 < top_k < V else V
            assert 1 <= len(keep) <= k_eff
            if top_p < 1.0:
                ranked = [j for _, j in sorted((-float(z[j]), j) for j in range(V))][:k_eff]
                total = p[ranked].sum()
                assert p[keep].sum() >= top_p * total * (1 - 1e-12)
                assert p[keep[:-1]].sum() < top_p * total * (1 + 1e-12)
            else:
                assert len(keep) == k_eff


def test_filtered_probs_special_cases():
    rng = np.random.default_rng(3)
    V = 50
    z = rng.normal(0, 1.5, V)
    # filters off: the plain softmax, bit for bit
    assert np.array_equal(A.filtered_probs(z, 0.8, 0, 1.0), A.target_probs(z, 0.8))
    assert np.array_equal(A.filtered_probs(z, 0.8, V, 1.0), A.target_probs(z, 0.8))
    # top_k = 1 is the temperature-0 distribution (one-hot at the first arg-max), also with ties
    zt = z.copy(); zt[7] = zt[31] = z.max() + 1.0
    assert np.array_equal(A.filtered_probs(zt, 1.0, 1, 1.0), A.target_probs(zt, 0.0))
    assert A.filtered_probs(zt, 1.0, 1, 1.0)[7] == 1.0
    # a vanishing top_p keeps exactly the most probable token
    assert np.array_equal(A.filtered_probs(zt, 1.0, 0, 1e-12), A.target_probs(zt, 0.0))
    # renormalised: sums to one, proportional to the softmax on the kept set, zero elsewhere
    pf = A.filtered_probs(z, 1.0, 10, 0.9)
    keep = np.flatnonzero(pf)
    assert abs(pf.sum() - 1.0) < 1e-14 and len(keep) <= 10
    ref = softmax(z)[keep]
    assert np.allclose(pf[keep], ref / ref.sum(), rtol=1e-13)


def test_nucleus_of_a_geometric_distribution_closed_form():
    """p_j = 2^-(j+1) / (1 - 2^-V) on a shuffled vocabulary: the first n ranks hold 1 - 2^-n of the
    mass, so top_p keeps n = the smallest n with 1 - 2^-n >= top_p (1 - 2^-V)."""
    V = 40
    perm = np.random.default_rng(0).permutation(V)
    z = np.empty(V)
    z[perm] = -np.log(2.0) * np.arange(V)                  # token perm[r] has rank r
    for top_p, n in ((0.5, 1), (0.75, 2), (0.76, 3), (0.9, 4), (0.97, 6), (0.999, 10)):
        keep, _ = A.kept_tokens(z, 1.0, 0, top_p)
        assert [int(j) for j in keep] == [int(j) for j in perm[:n]], top_p
    # top-k first: with k = 3 the mass left is 7/8 and top_p refers to it: 0.9 * 7/8 = 0.7875 > 3/4 keeps 3
    keep, _ = A.kept_tokens(z, 1.0, 3, 0.9)
    assert len(keep) == 3
    keep, _ = A.kept_tokens(z, 1.0, 3, 0.85)               # 0.85 * 7/8 = 0.74375 <= 3/4 keeps 2
    assert len(keep) == 2
    # temperature acts before the filter: T = 0.5 squares the ratio (p_j ~ 4^-j): one token holds >= 0.75
    keep, _ = A.kept_tokens(z, 0.5, 0, 0.75)
    assert len(keep) == 1


def test_equal_logits_keep_lower_indices_first():
    z = np.zeros(10)
    keep, _ = A.kept_tokens(z, 1.0, 4, 1.0)
    assert [int(j) for j in keep] == [0, 1, 2, 3]
    keep, _ = A.kept_tokens(z, 1.0, 0, 0.35)               # 4 tokens of mass 0.1 reach 0.35
    assert [int(j) for j in keep] == [0, 1, 2, 3]


def test_draft_outside_the_kept_set_is_never_accepted_and_inside_uses_renormalised_p():
    rng = np.random.default_rng(5)
    V = 12
    z = rng.normal(0, 1.0, (2, V))
    pf = A.filtered_probs(z[0], 1.0, 3, 1.0)
    outside = int(np.flatnonzero(pf == 0)[0])
    inside = int(np.argmax(pf))
    r = A.verify_sequence(z, [outside], [0.0], 0.3, top_k=3)
    assert r.n_accepted == 0 and pf[r.tokens[0]] > 0       # recovered token comes from the kept set
    u = float(pf[inside])
    assert A.verify_sequence(z, [inside], [np.nextafter(u, 0)], 0.3, top_k=3).n_accepted == 1
    assert A.verify_sequence(z, [inside], [u], 0.3, top_k=3).n_accepted == 0


@pytest.mark.parametrize("mode", ["dense_q", "one_hot"])
def test_first_token_distribution_is_the_filtered_target(mode):
    """Sec. 3.2's exactness claim with p_t the filtered distribution: the emitted token follows it."""
    rng = np.random.default_rng(21)
    V, N = 16, 60_000
    z = rng.normal(0, 1.5, (2, V))
    ql = rng.normal(0, 1.5, (1, V))
    top_k, top_p = 9, 0.9
    keep = _brute_kept(z[0], 1.0, top_k, top_p)
    ref = np.zeros(V); ref[keep] = softmax(z[0])[keep]; ref /= ref.sum()
    q = softmax(ql[0])
    counts = np.zeros(V)
    for _ in range(N):
        if mode == "dense_q":
            d = int(rng.choice(V, p=q))
            r = A.verify_sequence(z, [d], rng.random(1), rng.random(), ql, top_k=top_k, top_p=top_p)
        else:
            d = int(rng.integers(V))
            r = A.verify_sequence(z, [d], rng.random(1), rng.random(), None, top_k=top_k, top_p=top_p)
        counts[r.tokens[0]] += 1
    assert counts[ref == 0].sum() == 0
    nz = ref > 0
    chi2 = ((counts[nz] - N * ref[nz]) ** 2 / (N * ref[nz])).sum()
    assert stats.chi2.sf(chi2, df=nz.sum() - 1) > 1e-4, chi2
    # the unfiltered target is rejected by the same data: the filter really acts
    p0 = softmax(z[0])
    chi2_0 = ((counts - N * p0) ** 2 / (N * p0)).sum()
    assert stats.chi2.sf(chi2_0, df=V - 1) < 1e-6
