"""Oracle: draft retrieval from a prompt's pool of pre-generated rollouts.

TEST INFRASTRUCTURE ONLY -- never imported by the product package.

Sec. 3.2 of the paper: pre-generated partial rollouts are gathered into one
token pool per prompt; at each decode step the current rollout suffix is matched
against the pool and a likely continuation of up to K tokens is returned
(Alg. 1, "retrieve a draft block"); candidates are chosen by how often they
occur after the matched context (Sec. 4.4, comparison with n-gram lookup).
The paper's index is a suffix tree; what it returns is a walk down the suffix
trie that always takes the most frequent child.  This oracle computes that walk
by brute force over the raw pool (the paper's "n-gram-style" cost model).

Reading taken where the paper is silent:
  * the match context is the last m tokens of the rollout, m from max_match
    down to min_match; the first m with at least one occurrence is used;
  * occurrences never straddle two rollouts of the pool;
  * ties between equally frequent continuations go to the smaller token id;
  * the draft ends when no occurrence has a successor inside its rollout.

Pin status: pinned (hand-worked cases, independent suffix-trie construction).
"""


def lookup(pool_rollouts, tail, max_match, min_match, k_max):
    """pool_rollouts: list of token lists (the rollouts of this prompt).
    tail: the most recent tokens of the sequence, newest last (entries < 0 are
    padding and never match).  Returns the draft token list (possibly empty)."""
    tail = [int(t) for t in tail]
    occ = []                                   # (rollout index, position of last matched token)
    for m in range(min(max_match, len(tail)), min_match - 1, -1):
        ctx = tail[len(tail) - m:]
        if any(t < 0 for t in ctx):
            continue
        occ = [(r, e) for r, toks in enumerate(pool_rollouts)
               for e in range(m - 1, len(toks))
               if all(int(toks[e - m + 1 + i]) == ctx[i] for i in range(m))]
        if occ:
            break
    draft = []
    while occ and len(draft) < k_max:
        counts = {}
        for r, e in occ:
            if e + 1 < len(pool_rollouts[r]):
                t = int(pool_rollouts[r][e + 1])
                counts[t] = counts.get(t, 0) + 1
        if not counts:
            break
        best = min(counts, key=lambda t: (-counts[t], t))
        draft.append(best)
        occ = [(r, e + 1) for r, e in occ
               if e + 1 < len(pool_rollouts[r]) and int(pool_rollouts[r][e + 1]) == best]
    return draft
