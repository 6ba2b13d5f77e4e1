"""Pins for the oracle's optimiser step and truncation-aware GAE (CPU only).

Adam: closed forms that follow from the update rule (first step, constant gradient, zero betas) and
torch.optim.Adam on an independent float64 run.  Truncation: with no time limits the recursion is the
plain one; a time limit at step t makes the steps up to t an independent trajectory of horizon t + 1
that bootstraps from V_{t+1}, which is the plain (separately pinned) recursion on the cut data.
"""
import numpy as np
import pytest
import torch

from oracle import morlax_oracle as orc

GAMMA, LAM = 0.99, 0.95


def test_adam_first_step_is_lr_times_sign():
    rng = np.random.default_rng(0)
    th, g = rng.standard_normal(50), rng.standard_normal(50)
    lr, eps = 3e-4, 1e-8
    th1, m1, v1 = orc.adam_step(th, g, np.zeros(50), np.zeros(50), lr, 0.9, 0.999, eps, 1)
    # m_hat = g and v_hat = g^2 exactly, whatever the betas
    assert np.allclose(th1, th - lr * g / (np.abs(g) + eps), rtol=1e-12, atol=0)
    assert np.allclose(m1, 0.1 * g) and np.allclose(v1, 0.001 * g * g)


def test_adam_constant_gradient_moves_linearly():
    rng = np.random.default_rng(1)
    th0, g = rng.standard_normal(20), rng.standard_normal(20)
    lr, eps, steps = 1e-3, 1e-8, 25
    th, m, v = th0.copy(), np.zeros(20), np.zeros(20)
    for t in range(1, steps + 1):
        th, m, v = orc.adam_step(th, g, m, v, lr, 0.9, 0.999, eps, t)
    # the bias corrections cancel the geometric sums: m_hat = g, v_hat = g^2 at every step
    assert np.allclose(th, th0 - steps * lr * g / (np.abs(g) + eps), rtol=1e-10, atol=1e-14)


def test_adam_zero_betas_is_normalised_gradient_step():
    rng = np.random.default_rng(2)
    th, g = rng.standard_normal(30), rng.standard_normal(30)
    m, v = rng.standard_normal(30), rng.random(30)      # history must not matter
    th1, m1, v1 = orc.adam_step(th, g, m, v, 0.01, 0.0, 0.0, 1e-6, 7)
    assert np.allclose(th1, th - 0.01 * g / (np.abs(g) + 1e-6), rtol=1e-12)
    assert np.array_equal(m1, g) and np.array_equal(v1, g * g)


@pytest.mark.parametrize("betas,eps", [((0.9, 0.999), 1e-8), ((0.8, 0.95), 1e-5)])
def test_adam_matches_torch_optim(betas, eps):
    rng = np.random.default_rng(3)
    n, steps, lr = 40, 12, 2e-3
    th0 = rng.standard_normal(n)
    grads = rng.standard_normal((steps, n)) * np.exp(rng.standard_normal((steps, 1)))
    p = torch.tensor(th0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([p], lr=lr, betas=betas, eps=eps)
    th, m, v = th0.copy(), np.zeros(n), np.zeros(n)
    for t in range(steps):
        p.grad = torch.tensor(grads[t], dtype=torch.float64)
        opt.step()
        th, m, v = orc.adam_step(th, grads[t], m, v, lr, betas[0], betas[1], eps, t + 1)
        assert np.allclose(th, p.detach().numpy(), rtol=1e-11, atol=1e-13), t


@pytest.mark.parametrize("K", [2, 3, 6])
def test_sampled_preferences_are_uniform_on_the_simplex(K):
    """Every coordinate of a uniform point of the (K-1)-simplex is Beta(1, K-1) distributed, and for K = 3
    the pair (w_0, w_1) is uniform on the triangle, so P(w_0 < a, w_1 < b) = 2ab for a + b <= 1."""
    from scipy import stats
    rng = np.random.default_rng(100 + K)
    P = 20000
    w = orc.sample_preferences(rng.random((P, K)))
    assert (w >= 0).all() and np.allclose(w.sum(1), 1.0, rtol=0, atol=1e-12)
    for k in range(K):
        assert stats.kstest(w[:, k], stats.beta(1, K - 1).cdf).pvalue > 1e-3, k
    # normalised uniforms (a plausible mistake) are not uniform on the simplex
    bad = rng.random((P, K)); bad /= bad.sum(1, keepdims=True)
    if K > 2:
        assert stats.kstest(bad[:, 0], stats.beta(1, K - 1).cdf).pvalue < 1e-6
    if K == 3:
        for a, b in ((0.3, 0.4), (0.5, 0.5), (0.2, 0.7)):
            frac = np.mean((w[:, 0] < a) & (w[:, 1] < b))
            assert abs(frac - 2 * a * b) < 4 * np.sqrt(2 * a * b / P) + 1e-3


def test_extreme_trade_offs_are_the_last_rows():
    rng = np.random.default_rng(7)
    u = rng.random((8, 3))
    w0 = orc.sample_preferences(u, 0)
    w2 = orc.sample_preferences(u, 2)
    assert np.array_equal(w2[:6], w0[:6])
    assert np.array_equal(w2[6], [1.0, 0.0, 0.0]) and np.array_equal(w2[7], [0.0, 1.0, 0.0])
    assert orc.check_preferences(w2)
    with pytest.raises(ValueError):
        orc.sample_preferences(u, 4)


def _rand(T=11, N=6, K=3, P=2, seed=0):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((T, N, K)), rng.standard_normal((T + 1, N, K)),
            (rng.random((T, N)) < 0.15).astype(np.uint8), rng.dirichlet(np.ones(K), size=P))


def test_trunc_all_zero_is_plain_gae():
    r, v, done, w = _rand()
    a0 = orc.vec_gae(r, v, done, w, GAMMA, LAM)
    a1 = orc.vec_gae(r, v, done, w, GAMMA, LAM, trunc=np.zeros_like(done))
    for x, y in zip(a0, a1):
        assert np.array_equal(x, y)


def test_every_step_truncated_gives_one_step_td_errors():
    r, v, done, w = _rand(seed=1)
    done[:] = 0
    adv, vtarg, _ = orc.vec_gae(r, v, done, w, GAMMA, LAM, trunc=np.ones_like(done))
    assert np.allclose(adv, r + GAMMA * v[1:] - v[:-1], rtol=1e-13)
    assert np.allclose(vtarg, r + GAMMA * v[1:], rtol=1e-13)


def test_truncation_cuts_the_trajectory_but_keeps_the_bootstrap():
    r, v, done, w = _rand(T=13, seed=2)
    T, N, K = r.shape
    rng = np.random.default_rng(9)
    cut = rng.integers(1, T - 1, size=N)
    trunc = np.zeros((T, N), dtype=np.uint8)
    trunc[cut, np.arange(N)] = 1
    done[cut, np.arange(N)] = 0        # a time limit alone ends the episode
    adv, vtarg, adv_s = orc.vec_gae(r, v, done, w, GAMMA, LAM, trunc=trunc)
    g = orc.env_pref_index(N, w.shape[0])
    for n in range(N):
        c = int(cut[n])
        # steps 0..c: the plain recursion on a trajectory of horizon c + 1 whose last value is V_{c+1}
        a_head, vt_head, as_head = _plain_single(r[:c + 1, n], v[:c + 2, n], done[:c + 1, n], w[g[n]])
        assert np.allclose(adv[:c + 1, n], a_head, rtol=1e-12, atol=1e-13)
        assert np.allclose(vtarg[:c + 1, n], vt_head, rtol=1e-12, atol=1e-13)
        assert np.allclose(adv_s[:c + 1, n], as_head, rtol=1e-12, atol=1e-13)
        # steps after the cut never see it
        a_tail, vt_tail, as_tail = _plain_single(r[c + 1:, n], v[c + 1:, n], done[c + 1:, n], w[g[n]])
        assert np.allclose(adv[c + 1:, n], a_tail, rtol=1e-12, atol=1e-13)
        assert np.allclose(adv_s[c + 1:, n], as_tail, rtol=1e-12, atol=1e-13)


def _plain_single(r, v, done, wrow):
    """The untruncated recursion for one environment through the oracle's own (pinned) plain path: the
    environment is placed in a batch of two identical groups so that the preference map is valid."""
    T, K = r.shape
    rr = np.repeat(r[:, None, :], 2, axis=1)
    vv = np.repeat(v[:, None, :], 2, axis=1)
    dd = np.repeat(done[:, None], 2, axis=1)
    adv, vt, a_s = orc.vec_gae(rr, vv, dd, np.stack([wrow, wrow]), GAMMA, LAM)
    return adv[:, 0], vt[:, 0], a_s[:, 0]


def test_terminated_step_ignores_next_value_even_when_flagged_not_truncated():
    r, v, done, w = _rand(seed=4)
    done[:] = 0
    done[5] = 1
    trunc = np.zeros_like(done)
    v_bad = v.copy()
    v_bad[6] = np.nan                  # value behind a failure must not be read into step 5 or earlier
    a0 = orc.vec_gae(r, v, done, w, GAMMA, LAM, trunc=trunc)[0]
    a1 = orc.vec_gae(r, v_bad, done, w, GAMMA, LAM, trunc=trunc)[0]
    assert np.array_equal(a0[:6], a1[:6]) and np.isfinite(a1[:6]).all()


def test_update_step_with_optimizer_equals_manual_adam_on_its_gradients():
    """With the optimiser on, minibatch b + 1 sees the parameters Adam produced after minibatch b."""
    from paper_2603_09237_amd import inputs
    from paper_2603_09237_amd.configs import CONFIGS, scaled
    cfg = scaled(CONFIGS[1], name="opt", minibatches=2, epochs=1)
    d = inputs.make_all(cfg)
    opt = dict(lr_actor=3e-3, lr_critic=1e-2, beta1=0.9, beta2=0.999, eps=1e-8)
    args = (cfg, d["w"], d["hparams_actor_old"], d["hparams_critic_old"])
    tail = (d["obs"], d["rewards"], d["dones"], d["eps"], cfg.gamma, cfg.lam, cfg.clip_eps)
    res = orc.update_step(*args, d["hparams_actor"], d["hparams_critic"], *tail, minibatches=2, epochs=1,
                          optimizer=opt)
    # first minibatch's gradients are those of the optimiser-free step
    ref = orc.update_step(*args, d["hparams_actor"], d["hparams_critic"], *tail, minibatches=2, epochs=1)
    assert np.array_equal(res["grads"][0]["dhp_actor"], ref["grads"][0]["dhp_actor"])
    z = np.zeros_like(ref["grads"][0]["dhp_actor"])
    hp1, m1, v1 = orc.adam_step(d["hparams_actor"], ref["grads"][0]["dhp_actor"], z, z, 3e-3, 0.9, 0.999, 1e-8, 1)
    zc = np.zeros_like(ref["grads"][0]["dhp_critic"])
    hc1, _, _ = orc.adam_step(d["hparams_critic"], ref["grads"][0]["dhp_critic"], zc, zc, 1e-2, 0.9, 0.999, 1e-8, 1)
    # second minibatch evaluated at the stepped parameters
    ref2 = orc.update_step(*args, hp1, hc1, *tail, minibatches=2, epochs=1)
    assert np.allclose(res["grads"][1]["dhp_actor"], ref2["grads"][1]["dhp_actor"], rtol=1e-12, atol=1e-15)
    hp2, _, _ = orc.adam_step(hp1, ref2["grads"][1]["dhp_actor"], m1, v1, 3e-3, 0.9, 0.999, 1e-8, 2)
    assert np.allclose(res["hp_actor"], hp2, rtol=1e-12, atol=1e-15)
    assert not np.allclose(res["hp_actor"], d["hparams_actor"])


# ---- per-objective advantage normalisation before scalarisation ------------------------------------
def _tiny_cfg(K=3, P=2, N=6, T=5):
    from paper_2603_09237_amd.configs import CONFIGS, scaled
    return scaled(CONFIGS[1], name="advk", K=K, P=P, N=N, T=T)


def test_per_objective_normalisation_brute_force():
    """The definition written out with loops over cells and objectives, on a partial selection."""
    cfg = _tiny_cfg()
    rng = np.random.default_rng(3)
    adv = rng.standard_normal((cfg.T, cfg.N, cfg.K)) * np.array([1.0, 0.1, 10.0]) + np.array([0.5, -2.0, 7.0])
    w = rng.dirichlet(np.ones(cfg.K), size=cfg.P)
    rows = (1, 3, 1, 2)                       # t in 1..3, local environments 1..2 of every preference
    n_g = cfg.N // cfg.P
    cells = [(t, p * n_g + j) for t in range(1, 4) for p in range(cfg.P) for j in range(1, 3)]
    want = np.zeros((cfg.T, cfg.N))
    for k in range(cfg.K):
        vals = [adv[t, n, k] for t, n in cells]
        mean = sum(vals) / len(vals)
        std = (sum((x - mean) ** 2 for x in vals) / len(vals)) ** 0.5
        for t, n in cells:
            want[t, n] += w[n // n_g, k] * (adv[t, n, k] - mean) / (std + 1e-8)
    got = orc.scalarize_normalized(cfg, rows, adv, w)
    assert np.allclose(got, want, rtol=1e-12, atol=1e-14)
    outside = np.ones((cfg.T, cfg.N), bool)
    for t, n in cells:
        outside[t, n] = False
    assert np.all(got[outside] == 0.0)


def test_per_objective_normalisation_ignores_scale_and_offset_of_an_objective():
    """What the variant is for: an objective measured in other units (x c_k + b_k, c_k > 0) counts the same."""
    cfg = _tiny_cfg(K=3, P=3, N=12, T=7)
    rng = np.random.default_rng(4)
    adv = rng.standard_normal((cfg.T, cfg.N, cfg.K))
    w = rng.dirichlet(np.ones(cfg.K), size=cfg.P)
    rows = orc.full_rows(cfg, cfg.T)
    a = orc.scalarize_normalized(cfg, rows, adv, w)
    b = orc.scalarize_normalized(cfg, rows, adv * np.array([1.0, 0.1, 10.0]) + np.array([0.0, 3.0, -50.0]), w)
    assert np.allclose(a, b, rtol=0, atol=1e-6)
    # the scalarise-then-normalise reading does depend on the units
    s1 = orc.vec_gae(adv, np.zeros((cfg.T + 1, cfg.N, cfg.K)), np.ones((cfg.T, cfg.N)), w, 0.0, 0.0)[2]
    s2 = orc.vec_gae(adv * np.array([1.0, 0.1, 10.0]), np.zeros((cfg.T + 1, cfg.N, cfg.K)), np.ones((cfg.T, cfg.N)),
                     w, 0.0, 0.0)[2]
    m = np.ones((cfg.T, cfg.N), bool)
    n1 = (s1 - orc.adv_norm_stats(s1, m)[0]) / orc.adv_norm_stats(s1, m)[1]
    n2 = (s2 - orc.adv_norm_stats(s2, m)[0]) / orc.adv_norm_stats(s2, m)[1]
    assert not np.allclose(n1, n2, atol=1e-2)


def test_per_objective_normalisation_single_objective_is_the_scalar_normalisation():
    cfg = _tiny_cfg(K=1, P=2, N=8, T=6)
    rng = np.random.default_rng(5)
    adv = rng.standard_normal((cfg.T, cfg.N, 1)) * 3.0 + 1.0
    w = np.ones((cfg.P, 1))
    rows = (0, cfg.T, 0, 2)
    mask = orc.row_mask(cfg, rows, cfg.T)
    mean, std = orc.adv_norm_stats(adv[:, :, 0], mask)
    got = orc.scalarize_normalized(cfg, rows, adv, w)
    assert np.allclose(got[mask], (adv[:, :, 0][mask] - mean) / (std + 1e-8), rtol=1e-12, atol=0)


def test_per_objective_normalisation_vertex_gives_unit_variance_and_is_linear_in_w():
    cfg = _tiny_cfg(K=3, P=2, N=10, T=9)
    rng = np.random.default_rng(6)
    adv = rng.standard_normal((cfg.T, cfg.N, cfg.K)) * np.array([2.0, 30.0, 0.01])
    rows = orc.full_rows(cfg, cfg.T)
    parts = []
    for k in range(cfg.K):
        e = np.zeros((2, cfg.K)); e[:, k] = 1.0     # both preferences at vertex k
        z = orc.scalarize_normalized(cfg, rows, adv, e)
        std_k = adv[:, :, k].std()
        assert abs(z.mean()) < 1e-12 and abs(z.var() - (std_k / (std_k + 1e-8)) ** 2) < 1e-12
        parts.append(z)
    w = np.repeat(rng.dirichlet(np.ones(cfg.K), size=1), 2, axis=0)
    mix = orc.scalarize_normalized(cfg, rows, adv, w)
    assert np.allclose(mix, sum(w[0, k] * parts[k] for k in range(cfg.K)), rtol=1e-12, atol=1e-14)


def test_update_step_per_objective_uses_the_prenormalised_advantage():
    """The update step's variant = the plain loss (no further normalisation) on scalarize_normalized()."""
    from paper_2603_09237_amd import inputs
    from paper_2603_09237_amd.configs import CONFIGS, scaled
    cfg = scaled(CONFIGS[1], name="advk-step", minibatches=2, epochs=1)
    d = inputs.make_all(cfg)
    args = (cfg, d["w"], d["hparams_actor_old"], d["hparams_critic_old"], d["hparams_actor"], d["hparams_critic"],
            d["obs"], d["rewards"], d["dones"], d["eps"], cfg.gamma, cfg.lam, cfg.clip_eps)
    a = orc.update_step(*args, minibatches=2, epochs=1, adv_norm="per_objective", keep=True)
    b = orc.update_step(*args, minibatches=2, epochs=1, keep=True)
    # the critic's loss does not see the advantage; the actor's does
    assert np.array_equal(a["grads"][0]["dhp_critic"], b["grads"][0]["dhp_critic"])
    assert not np.allclose(a["grads"][0]["dhp_actor"], b["grads"][0]["dhp_actor"], rtol=1e-3)
    rows = orc.minibatch_rows(cfg, cfg.T, 0, 2)
    adv_b = orc.scalarize_normalized(cfg, rows, a["adv_vec"], d["w"])
    logsig = a["theta_vec_actor"][:, -cfg.act_dim:]
    dmu, dls, dv, st = orc.ppo_loss_grad(cfg, rows, a["mu"], logsig, a["act"], a["logp_old"], adv_b, a["v"],
                                         a["vtarg"], cfg.clip_eps, False)
    assert np.array_equal(dmu, a["dmu"]) and np.array_equal(dls, a["dlogsig"])
