"""Plain CPU oracle for the evaluation side of MORLAX.  TEST INFRASTRUCTURE ONLY.

What the evaluation of a trained policy hypernetwork computes once the roll-outs are in
(Fig. 2a; Sec. II-A for returns and Pareto dominance, Sec. II-B for the hypervolume): the
return vector of every trade-off, which of them are Pareto optimal among the evaluated set,
and the hypervolume they dominate.  Imported only by `tests/`, `__graft_entry__.smoke()` and the
`cpu_baseline` leg of `bench.py`; it shares no code with the HIP path.  numpy float64 throughout.

Readings where the paper is silent:
  * the return vector of trade-off p is the mean, over the environments that ran pi_p, of the
    discounted sum of the vector reward from the first state up to and including the first
    `done` of that environment (Sec. II-A: J = E over initial states of V(s_0));
  * hypervolume is the Lebesgue measure of the part of objective space that is dominated by at
    least one point and dominates a reference point r (the paper gives the words "volume of
    objective space dominated by the discovered solutions" and no reference point: it is an
    input); a point that is not above r in every objective contributes nothing.

`hypervolume` is that definition written out on the grid spanned by the points' coordinates:
exact, and exponential in the number of objectives, so only for small cases.
Pinned by tests/test_oracle_eval.py: closed forms (one box, two boxes, a two-objective
staircase), inclusion-exclusion over all subsets, invariances, a Monte-Carlo estimate.
"""
from __future__ import annotations

import numpy as np


def discounted_returns(r, done, gamma, P):
    """J[p, k] = mean over the n_g environments of group p of sum_t gamma^t r[t, n, k] alive[t, n],
    alive[t, n] = 1 until (and at) the first done of environment n, 0 afterwards (Sec. II-A)."""
    r = np.asarray(r, dtype=np.float64)
    done = np.asarray(done).astype(bool)
    T, N, K = r.shape
    assert N % P == 0
    G = np.zeros((N, K))
    alive = np.ones(N, dtype=bool)
    disc = 1.0
    for t in range(T):
        G += np.where(alive[:, None], disc * r[t], 0.0)   # a selection: cells after the end never enter
        alive &= ~done[t]
        disc *= gamma
    return G.reshape(P, N // P, K).mean(axis=1)


def pareto_mask(J):
    """mask[i] = True when no other point dominates point i; j dominates i when J[j] >= J[i] in
    every objective and J[j] != J[i] (Sec. II-A).  Equal points do not dominate each other."""
    J = np.asarray(J, dtype=np.float64)
    n = J.shape[0]
    mask = np.ones(n, dtype=bool)
    for i in range(n):
        for j in range(n):
            if j != i and np.all(J[j] >= J[i]) and np.any(J[j] != J[i]):
                mask[i] = False
                break
    return mask


def hypervolume(J, ref):
    """Measure of the union over i of the boxes [ref, J[i]] (empty when J[i] is not above ref in
    every objective), Sec. II-B.  The coordinates of the points cut objective space into a grid of
    cells; a cell lies in the union exactly when its upper corner is below some point in every
    objective; the measure is the sum of the volumes of those cells."""
    J = np.asarray(J, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    n, K = J.shape
    V = np.maximum(J - ref[None, :], 0.0)          # box of point i is [0, V[i]]
    cuts = [np.unique(np.concatenate([[0.0], V[:, k]])) for k in range(K)]
    if any(len(c) < 2 for c in cuts):
        return 0.0
    widths = [np.diff(c) for c in cuts]
    uppers = [c[1:] for c in cuts]
    shape = tuple(len(u) for u in uppers)
    assert np.prod(shape, dtype=np.float64) <= 6e7, "grid too large for the plain definition"
    inside = np.zeros(shape, dtype=bool)
    for i in range(n):
        below = None
        for k in range(K):
            idx = [None] * K
            idx[k] = slice(None)
            b = (uppers[k] <= V[i, k])[tuple(idx)]
            below = b if below is None else (below & b)
        inside |= below
    vol = np.ones(shape)
    for k in range(K):
        idx = [None] * K
        idx[k] = slice(None)
        vol = vol * widths[k][tuple(idx)]
    return float(np.sum(vol[inside]))
