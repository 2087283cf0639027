"""Pins for oracle/lookup.py (CPU only): hand-worked cases and an independently
built counted suffix trie (the structure Sec. 3.2 describes)."""
import numpy as np

from oracle.lookup import lookup


def test_hand_worked_cases():
    pool = [[1, 2, 3, 4, 5, 6], [9, 2, 3, 4, 7, 8], [2, 3, 4, 7, 1]]
    # context (2,3,4) occurs three times; continuation 7 twice, 5 once -> 7; then 8 / 1 tie -> 1
    assert lookup(pool, [0, 2, 3, 4], 4, 1, 3) == [7, 1]
    # 4-token context (1,2,3,4) occurs once -> follow that rollout
    assert lookup(pool, [1, 2, 3, 4], 4, 1, 8) == [5, 6]
    # falls back to shorter contexts: (.., 7) only
    assert lookup(pool, [5, 5, 5, 7], 4, 1, 2) == [1]          # successors of 7: 8 and 1 -> tie -> 1
    # match only at a rollout end: no successor -> empty
    assert lookup(pool, [4, 5, 6], 4, 1, 4) == []
    # no match at all
    assert lookup(pool, [42, 43], 4, 1, 4) == []
    # a context may not straddle two rollouts: (6, 9) is not an occurrence
    assert lookup(pool, [6, 9], 2, 2, 4) == []
    # padding never matches; min_match respected
    assert lookup(pool, [-1, -1, -1, 3], 4, 1, 2) == [4, 7]
    assert lookup(pool, [-1, -1, -1, 3], 4, 2, 2) == []
    assert lookup(pool, [2, 3, 4], 4, 1, 0) == []


class _Trie:
    def __init__(self):
        self.count, self.kids = 0, {}


def _build_trie(pool, depth):
    root = _Trie()
    for toks in pool:
        for s in range(len(toks)):
            node = root
            for t in toks[s:s + depth]:
                node = node.kids.setdefault(int(t), _Trie())
                node.count += 1
    return root


def _trie_lookup(root, tail, max_match, min_match, k_max):
    tail = [int(t) for t in tail]
    for m in range(min(max_match, len(tail)), min_match - 1, -1):
        node = root
        for t in tail[len(tail) - m:]:
            node = node.kids.get(t) if (node is not None and t >= 0) else None
        if node is not None:
            break
    else:
        return []
    out = []
    while len(out) < k_max and node.kids:
        t = min(node.kids, key=lambda t: (-node.kids[t].count, t))
        out.append(t)
        node = node.kids[t]
    return out


def test_brute_force_equals_counted_suffix_trie():
    rng = np.random.default_rng(0)
    for trial in range(60):
        V = int(rng.integers(2, 6))
        pool = [list(rng.integers(0, V, size=int(rng.integers(1, 40)))) for _ in range(int(rng.integers(1, 5)))]
        k_max = int(rng.integers(0, 7))
        root = _build_trie(pool, 4 + k_max)
        for _ in range(20):
            tail = list(rng.integers(0, V, size=4))
            if rng.random() < 0.2:
                tail[0] = -1
            mm = int(rng.integers(1, 4))
            assert lookup(pool, tail, 4, mm, k_max) == _trie_lookup(root, tail, 4, mm, k_max)
