"""Oracle for the logit-distance step of the audit -- TEST INFRASTRUCTURE ONLY.

Plain numpy in float64, written from the definitions:

* Logit distance (paper section 4.3, definition of the logit distance distribution): the
  distance Dis(l, l*) between the deployed logits l and the reference logits l* of one decision
  step, for Dis = total-variation distance and Dis = KL divergence of the two softmax
  distributions.  The paper names the two metrics and leaves their exact form to convention;
  the reading taken here is TV(p, q) = 1/2 sum_i |p_i - q_i| and KL(p || q) = sum_i p_i
  (log p_i - log q_i) with p = softmax(l) (deployed), q = softmax(l*) (reference).
* Per-request statistic (section 5.3): p(t1) = |{i : Dis_i > t1}| / T.
* Top-K distance (appendix "Optimization: Verification of Top-K"): the smallest L1 perturbation
  of the logits after which the claimed index set I is a valid top-K set.  ``topk_distance``
  follows the appendix: sort the logits, try every logit value as the threshold t, raise the
  members of I below t up to t, lower the non-members above t down to t, keep the cheapest.
  ``topk_distance_bruteforce`` evaluates the same cost for every candidate threshold by direct
  summation (quadratic; for small inputs).

Nothing here is imported by the product path.
"""
from __future__ import annotations

import numpy as np


def softmax64(logits: np.ndarray) -> np.ndarray:
    x = np.asarray(logits, dtype=np.float64)
    e = np.exp(x - x.max())
    return e / e.sum()


def tv_distance(l: np.ndarray, l_ref: np.ndarray) -> float:
    return 0.5 * float(np.abs(softmax64(l) - softmax64(l_ref)).sum())


def kl_divergence(l: np.ndarray, l_ref: np.ndarray) -> float:
    x = np.asarray(l, dtype=np.float64)
    y = np.asarray(l_ref, dtype=np.float64)
    logp = x - x.max() - np.log(np.exp(x - x.max()).sum())
    logq = y - y.max() - np.log(np.exp(y - y.max()).sum())
    return float((np.exp(logp) * (logp - logq)).sum())


def tail_density(dist: np.ndarray, t1: float) -> float:
    d = np.asarray(dist, dtype=np.float64)
    return float((d > t1).sum()) / d.size


def topk_cost(logits: np.ndarray, member: np.ndarray, t: float) -> float:
    """L1 cost of moving the logits so that t separates I from its complement."""
    x = np.asarray(logits, dtype=np.float64)
    down = np.clip(x[~member] - t, 0.0, None).sum()   # non-members above t come down to t
    up = np.clip(t - x[member], 0.0, None).sum()      # members below t go up to t
    return float(down + up)


def topk_distance_bruteforce(logits: np.ndarray, idx) -> float:
    x = np.asarray(logits, dtype=np.float64)
    member = np.zeros(x.size, dtype=bool)
    member[np.asarray(idx, dtype=np.int64)] = True
    return min(topk_cost(x, member, float(t)) for t in x)


def topk_distance(logits: np.ndarray, idx) -> float:
    """Sort once, then every logit value as threshold with running sums (linear after the sort)."""
    x = np.asarray(logits, dtype=np.float64)
    n = x.size
    member = np.zeros(n, dtype=bool)
    member[np.asarray(idx, dtype=np.int64)] = True
    order = np.argsort(-x, kind="stable")
    xs, ms = x[order], member[order]
    # With t = xs[u]: non-members at sorted positions < u lie above t, members at positions > u
    # below it.  Moving the threshold from xs[v] down to xs[v+1] lowers every non-member seen so far
    # by the gap, and moving it up from xs[v+1] to xs[v] raises every member still to come by the
    # gap, so both parts are running sums of non-negative terms (no cancellation).
    gaps = xs[:-1] - xs[1:]                              # >= 0, length n-1
    out_upto = np.cumsum(~ms)[:-1]                       # non-members among positions <= v
    in_after = (ms.sum() - np.cumsum(ms))[:-1]           # members among positions > v
    down = np.concatenate(([0.0], np.cumsum(out_upto * gaps)))
    up = np.concatenate((np.cumsum((in_after * gaps)[::-1])[::-1], [0.0]))
    return float((down + up).min())
