"""Speculative sampling, the non-greedy acceptance rule -- CPU oracle, TEST INFRASTRUCTURE ONLY.

Sec. 2 of the paper builds on speculative decoding and cites speculative sampling as its non-greedy
form; the paper itself (Alg. 1) is greedy only.  This file states that published rule in plain numpy,
fp64, one decision after the other, for the tests to compare the GPU path with.  Only tests may import it;
it imports nothing from the GPU package.

The rule, for one sequence and one round with proposals t_1..t_s drawn by the draft model:
  q_j = softmax(draft logits of step j / T),  p_j = softmax(target logits of row j / T)   (row j conditions on t_1..t_{j-1})
  for j = 1..s:  keep t_j  if  u_j * q_j[t_j] < p_j[t_j]      (probability min(1, p/q))
                 else emit one token drawn from  max(0, p_j - q_j) / sum(max(0, p_j - q_j))  and stop
  if all s were kept: emit one more token drawn from p_{s+1}.
The emitted tokens are then distributed exactly as if the target model had been sampled token by token.
With proposals that were not drawn from a distribution (a fixed table), q_j is the point mass at t_j.

Every random number is an argument: u in [0, 1).  A draw from weights w (not necessarily normalised) with u is
the smallest index i with w_0 + ... + w_i > u * sum(w).

Each function also returns a margin: how far (in probability) the nearest decision boundary was from the random
number that decided.  A comparison in another precision may legitimately differ where the margin is tiny.
"""
import numpy as np


def softmax_t(z, temperature):
    """softmax(z / T) in fp64, shifted by the maximum."""
    z = np.asarray(z, dtype=np.float64) / float(temperature)
    e = np.exp(z - z.max())
    return e / e.sum()


def draw(w, u):
    """(index, margin): smallest i with cumsum(w)[i] > u * sum(w); margin = distance of u from the two
    boundaries of that index's interval, as a fraction of the total."""
    w = np.asarray(w, dtype=np.float64)
    c = np.cumsum(w)
    total = c[-1]
    if not total > 0.0:
        raise ValueError("draw: weights sum to zero")
    x = u * total
    i = int(np.searchsorted(c, x, side="right"))   # first i with c[i] > x
    if i >= len(w):                                 # u * total rounded up to the total
        i = int(np.nonzero(w > 0)[0][-1])
    lo = c[i - 1] if i > 0 else 0.0
    margin = np.inf
    if np.any(w[:i] > 0):        # a token below could have been drawn instead
        margin = min(margin, x - lo)
    if np.any(w[i + 1:] > 0):    # or one above
        margin = min(margin, c[i] - x)
    return i, (float(margin / total) if np.isfinite(margin) else 1.0)


def sample_token(logits, temperature, u):
    """A draft step's proposal (or a plain sampling step): a draw from softmax(logits / T)."""
    return draw(softmax_t(logits, temperature), u)


def spec_sample_round(target_logits, draft_logits, proposals, u_accept, u_sample, temperature):
    """One sequence, one round.
    target_logits [s+1][V]; draft_logits [s][V], or None for proposals that come from no distribution;
    proposals [s]; u_accept [s]; u_sample [s+1] (entry j decides the token emitted at row j, if one is).
    Returns (l, emitted, margin): l kept proposals, emitted = the l kept tokens and one more, margin = the
    smallest margin of the decisions taken."""
    s = len(proposals)
    T = float(temperature)
    emitted, margin = [], 1.0
    for j in range(s):
        p = softmax_t(target_logits[j], T)
        t = int(proposals[j])
        if draft_logits is None:
            q = np.zeros_like(p)
            q[t] = 1.0
        else:
            q = softmax_t(draft_logits[j], T)
        ratio = p[t] / q[t]
        margin = min(margin, abs(ratio - u_accept[j]))
        if u_accept[j] * q[t] < p[t]:
            emitted.append(t)
            continue
        r = np.maximum(p - q, 0.0)
        if not r.sum() > 0.0:  # p == q everywhere: cannot be reached with u < 1, kept total
            r = p
        tok, m = draw(r, u_sample[j])
        emitted.append(tok)
        return j, emitted, min(margin, m)
    tok, m = draw(softmax_t(target_logits[s], T), u_sample[s])
    emitted.append(tok)
    return s, emitted, min(margin, m)
