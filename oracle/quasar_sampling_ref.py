"""CPU oracle for stochastic verification at temperature T > 0 (TEST INFRASTRUCTURE ONLY).

Plain numpy, fp64, no blocking.  Nothing in the product path imports this file and this file
imports nothing from the product path.

The passage followed is the verification rule of speculative decoding (Sec. 3.1, the
acceptance test r < min(1, p/q) and the resampling from norm(max(0, p - q)); Sec. 3.3
"Lossless Rejection Sampling": the logits recovered by the dequantisation are turned into the
distribution p by the final softmax and compared with the draft distribution).

Reading.  The drafter of the paper's experiments is a prompt-lookup n-gram drafter: it proposes
its tokens deterministically, so q is a point mass on the proposed token.  With q(x~_i) = 1:
  * the i-th candidate is accepted iff r_i < p_i(x~_i);
  * on the first rejection, at position n, the corrective token is drawn from p_n with the
    rejected token's mass removed and the rest renormalised (max(0, p - q) is p off the
    proposed token and 0 on it);
  * if all candidates are accepted, the bonus token is drawn from p at the next position.
Random numbers are inputs: r_i = u_accept[i]; the draw uses u_sample[n] through the inverse
CDF in vocabulary order: token = min{ v : C(v) > u * C(V-1) }, C the inclusive prefix sum of
the unnormalised masses (so zero-mass entries are never drawn and u = 0 gives the first entry
with positive mass).
"""
from __future__ import annotations

import numpy as np


def softmax(logits, temperature: float) -> np.ndarray:
    """p[m, v] = exp(z - max z) / sum exp(z - max z), z = logits / T, row by row, fp64."""
    if not temperature > 0:
        raise ValueError("temperature must be positive")
    z = np.asarray(logits, dtype=np.float64) / float(temperature)
    z = z - z.max(axis=-1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=-1, keepdims=True)


def inverse_cdf(mass, u: float):
    """Token drawn from the (unnormalised, non-negative) masses with the uniform number u in [0, 1).

    Returns (token, margin): margin is the distance of u * total from the nearer edge of the
    token's own interval of the cumulative sum, divided by the total (how far the draw is from
    flipping to a neighbouring token)."""
    mass = np.asarray(mass, dtype=np.float64)
    if mass.ndim != 1 or mass.size == 0 or np.any(mass < 0):
        raise ValueError("mass must be a non-empty vector of non-negative numbers")
    if not 0.0 <= u < 1.0:
        raise ValueError("u must be in [0, 1)")
    c = np.cumsum(mass)
    total = c[-1]
    if not total > 0:
        raise ValueError("no mass to draw from")
    target = u * total
    token = int(np.searchsorted(c, target, side="right"))     # first v with c[v] > target
    lo = c[token - 1] if token > 0 else 0.0
    margin = min(target - lo, c[token] - target) / total
    return token, float(margin)


def speculative_verify(logits, draft, temperature: float, u_accept, u_sample):
    """One verification step on the logits [M, V] of the M positions.

    draft: n_draft proposed tokens (n_draft <= M); position i scores candidate i.  If all are
    accepted the bonus token needs position n_draft, i.e. M >= n_draft + 1.
    Returns dict(n_acc, token, p_draft [n_draft], accept_margin [n_draft], sample_margin):
    n_acc leading candidates accepted; token = corrective or bonus token; accept_margin[i] =
    |u_accept[i] - p_i(x~_i)|.
    """
    logits = np.asarray(logits, dtype=np.float64)
    draft = np.asarray(draft, dtype=np.int64).reshape(-1)
    M, V = logits.shape
    n_draft = draft.size
    if n_draft > M:
        raise ValueError("more candidates than positions")
    u_accept = np.asarray(u_accept, dtype=np.float64).reshape(-1)
    u_sample = np.asarray(u_sample, dtype=np.float64).reshape(-1)
    p = softmax(logits, temperature)
    p_draft = np.array([p[i, draft[i]] if 0 <= draft[i] < V else 0.0 for i in range(n_draft)])
    n_acc = 0
    for i in range(n_draft):
        if u_accept[i] < min(1.0, p_draft[i] / 1.0):          # q(x~_i) = 1
            n_acc += 1
        else:
            break
    if n_acc < n_draft:
        mass = p[n_acc].copy()                                 # max(0, p - q): the proposed token loses all its mass
        if 0 <= draft[n_acc] < V:
            mass[draft[n_acc]] = 0.0
    else:
        if n_draft >= M:
            raise ValueError("the bonus token needs one position more than there are candidates")
        mass = p[n_draft]
    token, sample_margin = inverse_cdf(mass, float(u_sample[n_acc]))
    return {"n_acc": n_acc, "token": token, "p_draft": p_draft,
            "accept_margin": np.abs(u_accept[:n_draft] - p_draft), "sample_margin": sample_margin}
