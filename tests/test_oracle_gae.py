"""Pins for the oracle's vector GAE, index map and normalisation (CPU only).

Each test compares the oracle with something fixed by the mathematics rather than
by the oracle's own code: brute-force discounted sums, closed forms, a per-episode
direct-sum formulation written with plain Python loops, and invariants.
"""
import math

import numpy as np
import pytest

from oracle import morlax_oracle as orc

GAMMA, LAM = 0.99, 0.95


def _rand(T=9, N=6, K=3, P=2, seed=0, p_done=0.2):
    rng = np.random.default_rng(seed)
    r = rng.standard_normal((T, N, K))
    v = rng.standard_normal((T + 1, N, K))
    done = (rng.random((T, N)) < p_done).astype(np.uint8)
    w = rng.dirichlet(np.ones(K), size=P)
    return r, v, done, w


def test_env_pref_index_is_block_repeat():
    # Sec. III-C sampling phase: {w'_1 x N/P, ..., w'_P x N/P}
    for N, P in ((64, 4), (12, 3), (4096, 16), (6, 2)):
        table = []
        for p in range(P):
            table += [p] * (N // P)
        g = orc.env_pref_index(N, P)
        assert g.dtype == np.int32
        assert g.tolist() == table
    with pytest.raises(ValueError):
        orc.env_pref_index(10, 3)
    with pytest.raises(ValueError):
        orc.env_pref_index(8, 1)


def test_lambda1_no_dones_is_discounted_return():
    r, v, done, w = _rand(p_done=0.0)
    T, N, K = r.shape
    adv, vtarg, _ = orc.vec_gae(r, v, done, w, GAMMA, 1.0)
    for n in range(N):
        for k in range(K):
            for t in range(T):
                ret = sum(GAMMA ** (j - t) * r[j, n, k] for j in range(t, T)) + GAMMA ** (T - t) * v[T, n, k]
                assert abs(vtarg[t, n, k] - ret) < 1e-12
                assert abs(adv[t, n, k] - (ret - v[t, n, k])) < 1e-12


def test_lambda0_is_td_residual():
    r, v, done, w = _rand()
    adv, _, _ = orc.vec_gae(r, v, done, w, GAMMA, 0.0)
    nd = (done == 0)[..., None]
    delta = r + GAMMA * nd * v[1:] - v[:-1]
    assert np.allclose(adv, delta, atol=1e-13)


def test_all_done_is_reward_minus_value():
    r, v, done, w = _rand()
    done[:] = 1
    adv, vtarg, _ = orc.vec_gae(r, v, done, w, GAMMA, LAM)
    assert np.allclose(adv, r - v[:-1], atol=1e-13)
    assert np.allclose(vtarg, r, atol=1e-13)


def test_constant_reward_closed_form():
    T, N, K, c = 12, 4, 2, 0.7
    r = np.full((T, N, K), c)
    v = np.zeros((T + 1, N, K))
    done = np.zeros((T, N), dtype=np.uint8)
    w = np.full((2, K), 1.0 / K)
    adv, _, _ = orc.vec_gae(r, v, done, w, GAMMA, 1.0)
    for t in range(T):
        assert np.allclose(adv[t], c * (1 - GAMMA ** (T - t)) / (1 - GAMMA), rtol=1e-12)


def test_episode_direct_sum_with_dones():
    """Independent formulation: cut each series into episodes at the done flags; inside an
    episode A_t = sum_l (gamma lam)^l delta_{t+l}, the step that ends an episode has no
    bootstrap, the unfinished last episode bootstraps from v[T]."""
    r, v, done, w = _rand(T=11, N=6, K=2, seed=3, p_done=0.25)
    T, N, K = r.shape
    adv, vtarg, _ = orc.vec_gae(r, v, done, w, GAMMA, LAM)
    for n in range(N):
        # episode boundaries
        ends = [t for t in range(T) if done[t, n]]
        for k in range(K):
            for t in range(T):
                end = next((e for e in ends if e >= t), None)
                last = end if end is not None else T - 1
                a = 0.0
                for j in range(t, last + 1):
                    boot = 0.0 if (end is not None and j == end) else GAMMA * v[j + 1, n, k]
                    delta = r[j, n, k] + boot - v[j, n, k]
                    a += (GAMMA * LAM) ** (j - t) * delta
                assert abs(adv[t, n, k] - a) < 1e-12
                assert abs(vtarg[t, n, k] - (a + v[t, n, k])) < 1e-12


def test_linearity_scalarise_then_gae():
    """GAE is linear in (r, V): scalarising first with a fixed w gives the scalarised advantage."""
    r, v, done, w = _rand(T=10, N=8, K=3, P=4, seed=5)
    _, _, adv_s = orc.vec_gae(r, v, done, w, GAMMA, LAM)
    g = orc.env_pref_index(8, 4)
    wn = w[g]
    rs = (r * wn[None]).sum(-1, keepdims=True)
    vs = (v * wn[None]).sum(-1, keepdims=True)
    a1, _, _ = orc.vec_gae(rs, vs, done, np.ones((4, 1)), GAMMA, LAM)
    assert np.allclose(a1[..., 0], adv_s, atol=1e-12)


def test_scalarisation_uses_group_preference():
    r, v, done, w = _rand(T=4, N=6, K=3, P=3, seed=7)
    adv, _, adv_s = orc.vec_gae(r, v, done, w, GAMMA, LAM)
    for n in range(6):
        p = n // 2
        for t in range(4):
            assert abs(adv_s[t, n] - sum(w[p, k] * adv[t, n, k] for k in range(3))) < 1e-13


def test_nothing_leaks_backwards_through_a_done():
    r, v, done, w = _rand(T=10, N=4, K=2, seed=11, p_done=0.0)
    done[5, :] = 1
    a0, vt0, s0 = orc.vec_gae(r, v, done, w, GAMMA, LAM)
    r2, v2 = r.copy(), v.copy()
    r2[6:] = np.nan
    v2[6:] = np.inf
    a1, vt1, s1 = orc.vec_gae(r2, v2, done, w, GAMMA, LAM)
    assert np.array_equal(a0[:6], a1[:6])
    assert np.array_equal(vt0[:6], vt1[:6])
    assert np.array_equal(s0[:6], s1[:6])


def test_normalisation_stats_and_invariance():
    rng = np.random.default_rng(2)
    a = rng.standard_normal((7, 12)) * 3.0 + 5.0
    mask = np.ones_like(a, dtype=bool)
    mask[:, ::3] = False
    m, s = orc.adv_norm_stats(a, mask)
    ahat = (a - m) / (s + 1e-8)
    assert abs(ahat[mask].mean()) < 1e-12
    assert abs(ahat[mask].std() - 1.0) < 1e-6      # numpy std is the population std
    m2, s2 = orc.adv_norm_stats(2.5 * a - 4.0, mask)
    ahat2 = (2.5 * a - 4.0 - m2) / (s2 + 1e-8)
    assert np.allclose(ahat[mask], ahat2[mask], atol=1e-7)


def test_preferences_on_simplex():
    from paper_2603_09237_amd import configs, inputs
    for cid, cfg in configs.CONFIGS.items():
        w = inputs.make_preferences(cfg)
        assert w.shape == (cfg.P, cfg.K) and w.dtype == np.float32
        assert orc.check_preferences(w)
    assert not orc.check_preferences(np.array([[0.6, 0.6]]))
    assert not orc.check_preferences(np.array([[1.2, -0.2]]))
