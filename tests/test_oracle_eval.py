"""Pins for oracle/eval_oracle.py against closed forms, brute force and invariances (no GPU)."""
import itertools

import numpy as np
import pytest

from oracle import eval_oracle as ev


# ---------------------------------------------------------------------------------- returns
def test_returns_constant_reward_geometric_sum():
    T, N, K, P, g = 20, 8, 3, 2, 0.9
    c = np.array([1.0, -2.0, 0.5])
    r = np.broadcast_to(c, (T, N, K)).copy()
    done = np.zeros((T, N), dtype=np.uint8)
    J = ev.discounted_returns(r, done, g, P)
    np.testing.assert_allclose(J, np.broadcast_to(c * (1 - g ** T) / (1 - g), (P, K)), rtol=1e-13)


def test_returns_stop_at_first_done_inclusive():
    T, N, K, P, g = 12, 4, 2, 2, 0.8
    r = np.ones((T, N, K))
    done = np.zeros((T, N), dtype=np.uint8)
    d = [0, 3, 11, 5]
    for n, t in enumerate(d):
        done[t, n] = 1
    done[7, 1] = 1            # a later done of the same environment changes nothing
    per_env = np.array([(1 - g ** (t + 1)) / (1 - g) for t in d])
    J = ev.discounted_returns(r, done, g, P)
    np.testing.assert_allclose(J[:, 0], per_env.reshape(P, 2).mean(axis=1), rtol=1e-13)
    np.testing.assert_allclose(J[:, 1], J[:, 0], rtol=0)


def test_returns_ignore_whatever_follows_the_end():
    r = np.ones((6, 2, 1))
    r[3:, 0, 0] = [np.inf, np.nan, -np.inf]
    done = np.zeros((6, 2), dtype=np.uint8)
    done[2, 0] = 1
    J = ev.discounted_returns(r, done, 0.5, 2)
    np.testing.assert_allclose(J[:, 0], [1.75, 2 - 0.5 ** 5], rtol=1e-15)


def test_returns_brute_force_loops():
    rng = np.random.default_rng(5)
    T, N, K, P, g = 9, 6, 3, 3, 0.97
    r = rng.standard_normal((T, N, K))
    done = (rng.random((T, N)) < 0.2).astype(np.uint8)
    ref = np.zeros((P, K))
    n_g = N // P
    for n in range(N):
        for k in range(K):
            s = 0.0
            for t in range(T):
                s += g ** t * r[t, n, k]
                if done[t, n]:
                    break
            ref[n // n_g, k] += s / n_g
    np.testing.assert_allclose(ev.discounted_returns(r, done, g, P), ref, rtol=1e-12, atol=1e-14)


def test_returns_undiscounted_is_plain_sum():
    rng = np.random.default_rng(6)
    r = rng.standard_normal((7, 4, 2))
    done = np.zeros((7, 4), dtype=np.uint8)
    np.testing.assert_allclose(ev.discounted_returns(r, done, 1.0, 4), r.sum(axis=0), rtol=1e-13)


# ---------------------------------------------------------------------------------- dominance
def test_pareto_mask_hand_example():
    J = np.array([[1, 5], [2, 4], [3, 3], [2, 2], [3, 3], [0, 6], [2, 3], [3, 1]], dtype=float)
    #             nd      nd      nd      dom     nd(dup)  nd     dom(by 2,4)  dom(by 3,3)
    assert ev.pareto_mask(J).tolist() == [True, True, True, False, True, True, False, False]


def test_pareto_mask_single_objective_keeps_the_maxima():
    J = np.array([[1.0], [3.0], [2.0], [3.0]])
    assert ev.pareto_mask(J).tolist() == [False, True, False, True]


def test_pareto_mask_brute_force_definition():
    rng = np.random.default_rng(7)
    J = rng.integers(0, 4, size=(30, 3)).astype(float)   # many ties
    m = ev.pareto_mask(J)
    for i in range(30):
        dom = any(all(J[j, k] >= J[i, k] for k in range(3)) and any(J[j, k] > J[i, k] for k in range(3))
                  for j in range(30))
        assert m[i] == (not dom)


# ---------------------------------------------------------------------------------- hypervolume
def test_hv_one_box():
    assert ev.hypervolume([[3.0, 4.0, 5.0]], [1.0, 1.0, 1.0]) == pytest.approx(2 * 3 * 4, rel=1e-15)
    assert ev.hypervolume([[3.0, 0.5, 5.0]], [1.0, 1.0, 1.0]) == 0.0      # not above the reference in objective 1
    assert ev.hypervolume([[2.5]], [1.0]) == pytest.approx(1.5)


def test_hv_two_boxes_union_formula():
    a, b, r = np.array([4.0, 1.0, 3.0]), np.array([2.0, 5.0, 2.0]), np.array([0.5, 0.25, 1.0])
    va, vb = np.prod(a - r), np.prod(b - r)
    vab = np.prod(np.minimum(a, b) - r)
    assert ev.hypervolume([a, b], r) == pytest.approx(va + vb - vab, rel=1e-14)


def test_hv_two_objective_staircase():
    rng = np.random.default_rng(8)
    J = rng.random((40, 2)) * 10
    order = np.argsort(-J[:, 0])
    area, top = 0.0, 0.0
    for i in order:                      # widest first: each point adds the strip above the current top
        if J[i, 1] > top:
            area += J[i, 0] * (J[i, 1] - top)
            top = J[i, 1]
    assert ev.hypervolume(J, [0.0, 0.0]) == pytest.approx(area, rel=1e-13)


def _inclusion_exclusion(J, ref):
    V = np.maximum(np.asarray(J, float) - np.asarray(ref, float), 0.0)
    n = len(V)
    tot = 0.0
    for m in range(1, n + 1):
        for S in itertools.combinations(range(n), m):
            tot += (-1) ** (m + 1) * np.prod(np.min(V[list(S)], axis=0))
    return tot


@pytest.mark.parametrize("K", [1, 2, 3, 4, 5, 6])
def test_hv_inclusion_exclusion(K):
    rng = np.random.default_rng(10 + K)
    n = 8 if K < 6 else 6
    J = rng.standard_normal((n, K)) + 1.0
    ref = np.full(K, -0.5)
    J[0, 0] = -1.0   # one point outside the reference box
    assert ev.hypervolume(J, ref) == pytest.approx(_inclusion_exclusion(J, ref), rel=1e-12, abs=1e-14)


def test_hv_invariances():
    rng = np.random.default_rng(20)
    J = rng.random((12, 3)) * 3
    ref = np.array([0.2, 0.1, 0.3])
    h = ev.hypervolume(J, ref)
    assert ev.hypervolume(J[rng.permutation(12)], ref) == pytest.approx(h, rel=1e-13)          # order of the points
    assert ev.hypervolume(J[:, [2, 0, 1]], ref[[2, 0, 1]]) == pytest.approx(h, rel=1e-13)      # order of the objectives
    assert ev.hypervolume(J + 5.0, ref + 5.0) == pytest.approx(h, rel=1e-12)                   # translation
    s = np.array([2.0, 1.0, 0.5])
    assert ev.hypervolume(J * s, ref * s) == pytest.approx(h * np.prod(s), rel=1e-13)          # scaling
    dominated = np.min(J, axis=0, keepdims=True)
    assert ev.hypervolume(np.vstack([J, dominated]), ref) == pytest.approx(h, rel=1e-13)       # a dominated point adds nothing
    front = J[ev.pareto_mask(J)]
    assert ev.hypervolume(front, ref) == pytest.approx(h, rel=1e-13)                           # only the front counts
    better = np.max(J, axis=0, keepdims=True) + 0.1
    assert ev.hypervolume(np.vstack([J, better]), ref) == pytest.approx(np.prod(better - ref), rel=1e-13)


def test_hv_monte_carlo():
    rng = np.random.default_rng(30)
    K, n = 4, 10
    J = rng.random((n, K))
    ref = np.zeros(K)
    S = 400000
    u = rng.random((S, K))
    hit = np.zeros(S, dtype=bool)
    for i in range(n):
        hit |= np.all(u <= J[i], axis=1)
    p = hit.mean()
    assert abs(ev.hypervolume(J, ref) - p) < 5 * np.sqrt(p * (1 - p) / S)
