"""Oracle: draft acceptance and residual resampling (fp64 NumPy).

TEST INFRASTRUCTURE ONLY -- never imported by the product package.

Follows Sec. 3.2 (Eq. 2, Eq. 3) and Alg. 1 of the paper, in the order and
notation used there.  The paper states the rule for a deterministic draft
(proposal q_t with q_t(x~_t) = 1): accept x~_t with probability p_t(x~_t), on
rejection draw from r_t(x) = p_t(x) 1[x != x~_t] / (1 - p_t(x~_t)).  It notes
that this is rejection sampling with a degenerate proposal; the general rule it
specialises is: accept with probability min(1, p_t(x~_t)/q_t(x~_t)), on
rejection draw from max(0, p_t - q_t) normalised.  `q_logits=None` selects the
paper's one-hot proposal.

Readings taken where the paper is silent (each is an explicit argument or a
documented convention, not a hidden constant):
  * p_t = softmax(z_t / T); T == 0 means one-hot at the first arg-max.
  * q_t = softmax(q_logits_t) at temperature 1.
  * accept iff u < min(1, rho) with u in [0,1): rho >= 1 always accepts,
    rho == 0 never does; q_t(x~_t) == 0 gives rho = +inf (accept).
  * sampling is inverse-CDF in vocabulary-index order with an inclusive fp64
    running sum C: token = smallest j with C_j > u * C_last; if rounding leaves
    none, the last j with non-zero weight.
  * a residual whose total weight is 0 falls back to sampling p_t.
  * after a fully accepted block one more ("bonus") token is drawn from the
    last row when emit_bonus is set (Sec. 4.2 counts the recovered and the bonus
    token in the acceptance length); emit_bonus=False is Alg. 1 literally.
  * an accepted EOS ends the block (Alg. 1); nothing is emitted after it.
  * an empty draft block is plain sampling from row 0 (Alg. 1, first branch).
  * top-k / top-p (Sec. 3.2 defines p_t as the distribution "after temperature
    scaling and any top-p/top-k filtering" and says no more): tokens are ranked
    by logit, equal logits by lower index first; top-k keeps the first k of the
    ranking; top-p then keeps the shortest prefix of what is left whose mass
    reaches top_p times the mass of what is left (a token stays while the mass
    ranked before it is below that); the kept probabilities are renormalised.
    top_k <= 0 or >= V and top_p >= 1 switch the respective filter off.

Pin status: pinned (chi-square against the target distribution, closed-form
acceptance probabilities, greedy-path full acceptance, k = 0 == plain decode,
one-hot q == q_logits=None; filtering: top_k = 1 == temperature 0, filters off
== unfiltered, closed-form nucleus of a geometric distribution, the three
defining properties of the kept set checked by an independent brute force,
chi-square of the emitted token against the filtered target).
"""
import numpy as np


def target_probs(z, temperature):
    z = np.asarray(z, dtype=np.float64)
    if temperature == 0.0:
        p = np.zeros_like(z)
        p[int(np.argmax(z))] = 1.0          # np.argmax returns the first maximum
        return p
    x = z / temperature
    e = np.exp(x - np.max(x))
    return e / np.sum(e)


def kept_tokens(z, temperature, top_k=0, top_p=1.0):
    """Tokens that survive top-k then top-p, in ranking order, and the boundary margin.

    margin = distance of top_p * S from the nearer of the two cumulative masses
    that decide the last kept token, divided by S (inf when top-p is off): a
    tiny margin marks a decision that rounding could turn."""
    z = np.asarray(z, dtype=np.float64)
    V = z.shape[0]
    p = target_probs(z, temperature)
    order = np.lexsort((np.arange(V), -z))               # by logit descending, then index ascending
    if 0 < top_k < V:
        order = order[:top_k]
    margin = np.inf
    if top_p < 1.0:
        C = np.cumsum(p[order])
        t = float(top_p) * C[-1]
        n = int(np.searchsorted(C, t, side="left"))      # first n with C_n >= t
        n = min(n, len(order) - 1)
        below = C[n - 1] if n > 0 else 0.0
        margin = min(abs(C[n] - t), abs(t - below)) / C[-1]
        order = order[:n + 1]
    return order, margin


def filtered_probs(z, temperature, top_k=0, top_p=1.0):
    """p_t of Sec. 3.2: softmax(z / T), filtered and renormalised."""
    p = target_probs(z, temperature)
    if temperature == 0.0 or (not 0 < top_k < p.shape[0] and top_p >= 1.0):
        return p
    keep, _ = kept_tokens(z, temperature, top_k, top_p)
    out = np.zeros_like(p)
    out[keep] = p[keep] / np.sum(p[keep])
    return out


def proposal_probs(ql):
    ql = np.asarray(ql, dtype=np.float64)
    e = np.exp(ql - np.max(ql))
    return e / np.sum(e)


def inverse_cdf(weights, u):
    """Token drawn from unnormalised non-negative `weights` with uniform u.

    Returns (token, margin): margin = distance from u*S to the nearer edge of
    the chosen token's CDF interval, divided by that token's weight."""
    w = np.asarray(weights, dtype=np.float64)
    C = np.cumsum(w)
    S = C[-1]
    t = float(u) * S
    j = int(np.searchsorted(C, t, side="right"))       # first j with C_j > t
    if j >= w.shape[0]:
        j = int(np.flatnonzero(w > 0)[-1])
    lo = C[j - 1] if j > 0 else 0.0
    margin = min(abs(t - lo), abs(C[j] - t)) / w[j] if w[j] > 0 else 0.0
    return j, margin


class VerifyResult:
    __slots__ = ("n_accepted", "tokens", "accept_gap", "sample_margin", "sampled_row")

    def __init__(self):
        self.n_accepted = 0        # drafts accepted
        self.tokens = []           # emitted tokens: accepted drafts (+ recovered / bonus)
        self.accept_gap = []       # |rho - u| of every accept test that was evaluated
        self.sample_margin = None  # inverse-CDF margin of the sampled token (None if none)
        self.sampled_row = -1      # logits row the sampled token came from


def verify_sequence(logits, drafts, u_accept, u_sample, q_logits=None,
                    temperature=1.0, eos_id=-1, emit_bonus=True, top_k=0, top_p=1.0):
    """Alg. 1's verify loop for ONE sequence and ONE draft block.

    logits   [k+1, V]  row i = target logits after [last, x~_1..x~_i]
    drafts   [k]       x~_1..x~_k
    u_accept [>=k]     uniforms for the accept tests, one per draft position
    u_sample scalar    uniform for the single recovered / bonus / plain token
    q_logits None (one-hot proposal) or [k, V]
    """
    logits = np.asarray(logits, dtype=np.float64)
    k = len(drafts)
    assert logits.shape[0] == k + 1
    res = VerifyResult()
    for t in range(k):
        p = filtered_probs(logits[t], temperature, top_k, top_p)
        a = int(drafts[t])
        if q_logits is None:
            q = np.zeros_like(p)
            q[a] = 1.0
        else:
            q = proposal_probs(q_logits[t])
        rho = np.inf if q[a] == 0.0 else p[a] / q[a]
        u = float(u_accept[t])
        res.accept_gap.append(abs(rho - u))
        if u < min(1.0, rho):
            res.tokens.append(a)
            res.n_accepted += 1
            if a == eos_id:
                return res
            continue
        resid = np.maximum(0.0, p - q)
        if np.sum(resid) == 0.0:
            resid = p
        x, res.sample_margin = inverse_cdf(resid, u_sample)
        res.sampled_row = t
        res.tokens.append(x)
        return res
    if emit_bonus or k == 0:
        p = filtered_probs(logits[k], temperature, top_k, top_p)
        x, res.sample_margin = inverse_cdf(p, u_sample)
        res.sampled_row = k
        res.tokens.append(x)
    return res


def verify_batch(logits_rows, draft_tokens, draft_len, u_accept, u_sample,
                 q_logits_rows=None, temperature=1.0, eos_id=-1, emit_bonus=True, top_k=0, top_p=1.0):
    """Batch wrapper over packed rows.

    logits_rows   [M, V]   sequence b owns rows row0_b .. row0_b + k_b,
                           row0_b = sum_{b'<b} (k_b' + 1)
    draft_tokens  [B, k_max], draft_len [B]
    u_accept      [B, k_max], u_sample [B]
    q_logits_rows None or [T_d, V], sequence b owns rows sum_{b'<b} k_b' ...
    Returns a list of VerifyResult."""
    out = []
    r0 = 0
    d0 = 0
    for b in range(len(draft_len)):
        k = int(draft_len[b])
        ql = None if q_logits_rows is None else q_logits_rows[d0:d0 + k]
        out.append(verify_sequence(logits_rows[r0:r0 + k + 1], draft_tokens[b][:k],
                                   u_accept[b], u_sample[b], ql,
                                   temperature, eos_id, emit_bonus, top_k, top_p))
        r0 += k + 1
        d0 += k
    return out


def plain_sample(logits_row, u_sample, temperature=1.0, top_k=0, top_p=1.0):
    """Ordinary auto-regressive sampling of one token (no speculation)."""
    return inverse_cdf(filtered_probs(logits_row, temperature, top_k, top_p), u_sample)[0]


def rollout(next_logits, retrieve, prefix, max_len, uniforms, temperature=1.0,
            eos_id=-1, emit_bonus=True):
    """Alg. 1 for one sequence, written against callbacks.

    next_logits(prefix_tokens, block) -> [len(block)+1, V] logits of the target
        policy after prefix, prefix+block[:1], ...
    retrieve(prefix_tokens) -> list of draft tokens (may be empty)
    uniforms() -> next uniform in [0,1)
    Returns (tokens, n_steps)."""
    y = list(prefix)
    steps = 0
    while len(y) < max_len:
        d = list(retrieve(y))[:max(0, max_len - len(y) - 1)]
        z = next_logits(y, d)
        ua = [uniforms() for _ in d]
        us = uniforms()
        r = verify_sequence(z, d, ua, us, None, temperature, eos_id, emit_bonus)
        y.extend(r.tokens)
        steps += 1
        if r.tokens and r.tokens[-1] == eos_id:
            break
    return y, steps
