"""GPU parity: every C-ABI entry point against the CPU oracle on the same seeded inputs.

fp32 results: |gpu - ref| <= 1e-5 + 1e-4 |ref|.  bf16 GEMM-derived results: |gpu - ref| <=
2e-2 * max(|ref|, RMS(ref)).  Index maps and done masking: bit-exact.  Where the oracle would take
minutes (the 4x512 networks at full size) it is evaluated on a sample of preferences; preferences
do not interact inside the grouped networks, so those rows are complete outputs.
"""
import sys

import numpy as np
import pytest

from oracle import morlax_oracle as orc
from paper_2603_09237_amd import configs, inputs
from paper_2603_09237_amd.configs import CONFIGS, scaled

from gpu_util import assert_close32, assert_close_bf16, assert_close_bf16_chain, bf16_chain_report, dev, rel_rms_err, to_np

pytestmark = pytest.mark.gpu

ACTOR, CRITIC = 0, 1


def say(msg):
    print(f"[gpu-parity] {msg}", flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def torch():
    import torch as t
    assert t.cuda.is_available(), "GPU tests need a GPU"
    return t


@pytest.fixture(autouse=True, scope="module")
def _float32_default(torch):
    # device buffers below are allocated with the default dtype and handed to fp32 kernels
    prev = torch.get_default_dtype()
    torch.set_default_dtype(torch.float32)
    yield
    torch.set_default_dtype(prev)


@pytest.fixture(scope="module")
def binding():
    from paper_2603_09237_amd import binding as b
    b.load()
    return b


RAGGED = scaled(CONFIGS[1], name="ragged-K3-P3-N69-T7", K=3, P=3, N=69, T=7, obs_dim=11, act_dim=3, n_hidden=2,
                width=48, act=1, rank=3, hyper_width=20)
RAGGED_BF16 = scaled(RAGGED, name="ragged-bf16", wdtype=1, N=3 * 150, T=5, width=144)
# enough tiles for the persistent GEMM kernel, with a cut last row tile (2016 rows per preference) and a cut
# last column tile (width 160), and an observation width that takes the gathered first-layer path
RAGGED_PERS = scaled(RAGGED, name="ragged-persistent-bf16", wdtype=1, P=32, N=32 * 126, T=16, width=160, obs_dim=32,
                     rank=4)
# the fused forward of all hidden layers (bf16, width 512, observation width a multiple of 64): three row
# tiles per preference with a cut last one (333 = 2 * 128 + 77 rows), tanh in one variant
RAGGED_FUSED = scaled(RAGGED, name="ragged-fused-bf16", wdtype=1, P=5, N=5 * 37, T=9, width=512, obs_dim=64, n_hidden=3,
                      rank=4)
RAGGED_FUSED_TANH = scaled(RAGGED_FUSED, name="ragged-fused-bf16-tanh", act=0, n_hidden=1, obs_dim=128)
# the widest observation the fused forward takes (eight super-steps in the first layer), deepest network
RAGGED_FUSED_WIDE = scaled(RAGGED_FUSED, name="ragged-fused-bf16-obs512", obs_dim=512, n_hidden=8, T=4, N=5 * 9)
# observation widths that are no multiple of 64: the fused forward zero-fills the first layer's contraction up to the
# next multiple (27 and 45: element-wise gather, narrow and general first-layer dW; 100: a multiple of 4 only;
# 72: whole 8-value pieces without the gathered copy; 96: with the gathered copy that the first layer's dW reads)
FUSED_ODD_OBS = [scaled(RAGGED_FUSED, name=f"ragged-fused-bf16-obs{o}", obs_dim=o) for o in (27, 45, 72, 96, 100)]
# the fused forward at width 256 (four waves, two output-layer passes per tile): the widest observation it takes,
# a multiple of 64, a narrow odd one, tanh, and the state-dependent sigma
FUSED_W256 = [scaled(RAGGED_FUSED, name="ragged-fused-w256-obs256", width=256, obs_dim=256),
              scaled(RAGGED_FUSED, name="ragged-fused-w256-obs64", width=256, obs_dim=64, n_hidden=4),
              scaled(RAGGED_FUSED, name="ragged-fused-w256-obs11", width=256, obs_dim=11),
              scaled(RAGGED_FUSED_TANH, name="ragged-fused-w256-tanh", width=256, obs_dim=128, n_hidden=2),
              scaled(RAGGED_FUSED, name="ragged-fused-w256-sigma", width=256, obs_dim=40, sigma_state=1)]
# state-dependent standard deviation (the actor's output layer is 2A wide): fp32, the widest allowed (2A = 16),
# a ragged fp32 case, and the fused bf16 forward
SIGMA_CASES = [scaled(CONFIGS[1], name="cfg1-sigma", sigma_state=1), scaled(CONFIGS[2], name="cfg2-sigma", sigma_state=1),
               scaled(RAGGED, name="ragged-sigma", sigma_state=1), scaled(RAGGED_FUSED, name="ragged-fused-sigma", sigma_state=1)]


def _random_fused_cases(n, seed):
    """Seeded random shapes and row selections for the fused forward (bf16, width 512): group sizes, horizons,
    observation widths 64 .. 512, depths, output widths, both activations, tanh on or off, both sigma forms."""
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        P, n_g, T = int(rng.integers(2, 5)), int(rng.integers(1, 60)), int(rng.integers(1, 7))
        O, L = int(rng.choice([64, 128, 192, 256, 320, 384, 448, 512])), int(rng.integers(1, 4))
        K, A = int(rng.integers(1, 7)), int(rng.integers(1, 9))
        act, sig, tanh = int(rng.integers(0, 2)), int(rng.integers(0, 2)), int(rng.integers(0, 2))
        cfg = scaled(RAGGED, name=f"fused-rand{i}-P{P}-g{n_g}-T{T}-O{O}-L{L}-K{K}-A{A}-a{act}s{sig}t{tanh}", wdtype=1, P=P,
                     N=P * n_g, T=T, obs_dim=O, n_hidden=L, width=512, K=K, act_dim=A, act=act, sigma_state=sig,
                     mean_tanh=tanh, rank=2)
        t0 = int(rng.integers(0, T)); tc = int(rng.integers(1, T - t0 + 1))
        j0 = int(rng.integers(0, n_g)); jc = int(rng.integers(1, n_g - j0 + 1))
        cases.append((cfg, (t0, tc, j0, jc)))
    return cases


RANDOM_FUSED = _random_fused_cases(8, 2024)


def all_cfgs():
    return [CONFIGS[i] for i in (1, 2, 3, 4, 5)]


# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("cfg", all_cfgs() + [RAGGED], ids=lambda c: c.name)
def test_env_pref_index_bit_exact(cfg, torch, binding):
    say(f"env_pref_index {cfg.name}")
    ctx = binding.Context.from_config(cfg)
    out = torch.full((cfg.N,), -1, dtype=torch.int32, device="cuda")
    ctx.env_pref_index(out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), orc.env_pref_index(cfg.N, cfg.P))


@pytest.mark.parametrize("cfg,kappa", [(CONFIGS[1], 0), (CONFIGS[1], 2), (RAGGED, 3), (CONFIGS[5], 6),
                                       (scaled(CONFIGS[2], name="P1024", P=1024, N=4096), 1)],
                         ids=lambda x: getattr(x, "name", str(x)))
def test_sample_preferences_matches_oracle(cfg, kappa, torch, binding):
    say(f"sample_preferences {cfg.name} kappa={kappa}")
    rng = np.random.default_rng(77)
    u = rng.random((cfg.P, cfg.K), dtype=np.float32)
    u = np.clip(u, 1e-7, 1.0 - 1e-7).astype(np.float32)
    ctx = binding.Context.from_config(cfg)
    w = torch.full((cfg.P, cfg.K), 7.0, device="cuda")
    ctx.sample_preferences(dev(u), kappa, w)
    torch.cuda.synchronize()
    got = to_np(w)
    assert_close32(got, orc.sample_preferences(u, kappa), "w")
    assert orc.check_preferences(got, tol=1e-5)
    if kappa:                                         # the extreme points are exact
        assert np.array_equal(got[cfg.P - kappa:], np.eye(cfg.K, dtype=np.float32)[:kappa])
    with pytest.raises(binding.MorlaxError):
        ctx.sample_preferences(dev(u), min(cfg.P, cfg.K) + 1, w)


# ------------------------------------------------------------------------------------------------
def run_gae(cfg, torch, binding, r, v, done, w, want_vec=True):
    ctx = binding.Context.from_config(cfg)
    T, N, K = cfg.T, cfg.N, cfg.K
    adv_vec = torch.full((T, N, K), 7.0, device="cuda") if want_vec else None
    vtarg = torch.full((T, N, K), 7.0, device="cuda")
    adv_s = torch.full((T, N), 7.0, device="cuda")
    ctx.vec_gae(dev(r), dev(v), dev(done), dev(w), cfg.gamma, cfg.lam, adv_vec, vtarg, adv_s)
    torch.cuda.synchronize()
    return (to_np(adv_vec) if want_vec else None), to_np(vtarg), to_np(adv_s)


@pytest.mark.parametrize("cfg", all_cfgs() + [RAGGED, scaled(RAGGED, name="ragged-K16", K=16, T=19),
                                              scaled(RAGGED, name="ragged-K1", K=1, T=1),
                                              # a horizon of several groups of chunks, the last chunk cut short
                                              scaled(RAGGED, name="ragged-T150", K=5, T=150)],
                         ids=lambda c: c.name)
def test_vec_gae_matches_oracle(cfg, torch, binding):
    say(f"vec_gae {cfg.name}")
    r = inputs.make_rewards(cfg) if cfg.K in (2, 3, 6) else \
        np.random.default_rng(1).standard_normal((cfg.T, cfg.N, cfg.K), dtype=np.float32)
    v = inputs.make_values(cfg)
    done = inputs.make_trajectory(cfg)["dones"] if cfg.N * cfg.T < 3e5 else \
        (np.random.default_rng(3).random((cfg.T, cfg.N)) < cfg.p_done).astype(np.uint8)
    w = inputs.make_preferences(cfg)
    adv, vtarg, adv_s = run_gae(cfg, torch, binding, r, v, done, w)
    o_adv, o_vtarg, o_adv_s = orc.vec_gae(r, v, done, w, cfg.gamma, cfg.lam)
    # absolute floor 1e-5 per unit of the output's own scale: an fp32 recurrence over T terms of
    # magnitude s carries ~ s * T * 2^-24 of rounding, which cancellation can leave on a small result
    for k in range(cfg.K):
        sk = max(1.0, float(np.sqrt(np.mean(o_adv[..., k] ** 2))))
        assert_close32(adv[..., k], o_adv[..., k], f"adv_vec[{k}]", abs_=1e-5 * sk)
        assert_close32(vtarg[..., k], o_vtarg[..., k], f"vtarg[{k}]", abs_=1e-5 * sk)
    ss = max(1.0, float(np.sqrt(np.mean(o_adv_s ** 2))))
    assert_close32(adv_s, o_adv_s, "adv_s", abs_=1e-5 * ss)
    # without the optional output the others are unchanged bit for bit
    _, vt2, as2 = run_gae(cfg, torch, binding, r, v, done, w, want_vec=False)
    assert np.array_equal(vt2, vtarg) and np.array_equal(as2, adv_s)


@pytest.mark.parametrize("cfg", [CONFIGS[1], RAGGED, CONFIGS[5], scaled(RAGGED, name="ragged-T150", K=5, T=150)],
                         ids=lambda c: c.name)
def test_vec_gae_trunc_matches_oracle(cfg, torch, binding):
    """Time limits keep the bootstrap and restart the sum; without any the plain scan is reproduced bit for bit."""
    say(f"vec_gae_trunc {cfg.name}")
    rng = np.random.default_rng(11)
    r = inputs.make_rewards(cfg)
    v = inputs.make_values(cfg)
    done = (rng.random((cfg.T, cfg.N)) < 0.02).astype(np.uint8)
    trunc = (rng.random((cfg.T, cfg.N)) < 0.03).astype(np.uint8)
    w = inputs.make_preferences(cfg)
    ctx = binding.Context.from_config(cfg)
    T, N, K = cfg.T, cfg.N, cfg.K

    def run(tr):
        adv = torch.full((T, N, K), 7.0, device="cuda")
        vt = torch.full((T, N, K), 7.0, device="cuda")
        a_s = torch.full((T, N), 7.0, device="cuda")
        args = (dev(r), dev(v), dev(done))
        if tr is None:
            ctx.vec_gae(*args, dev(w), cfg.gamma, cfg.lam, adv, vt, a_s)
        else:
            ctx.vec_gae_trunc(*args, dev(tr), dev(w), cfg.gamma, cfg.lam, adv, vt, a_s)
        torch.cuda.synchronize()
        return to_np(adv), to_np(vt), to_np(a_s)

    adv, vt, a_s = run(trunc)
    o_adv, o_vt, o_as = orc.vec_gae(r, v, done, w, cfg.gamma, cfg.lam, trunc=trunc)
    for k in range(K):
        sk = max(1.0, float(np.sqrt(np.mean(o_adv[..., k] ** 2))))
        assert_close32(adv[..., k], o_adv[..., k], f"adv_vec[{k}]", abs_=1e-5 * sk)
        assert_close32(vt[..., k], o_vt[..., k], f"vtarg[{k}]", abs_=1e-5 * sk)
    assert_close32(a_s, o_as, "adv_s", abs_=1e-5 * max(1.0, float(np.sqrt(np.mean(o_as ** 2)))))
    assert not np.allclose(o_adv, orc.vec_gae(r, v, done, w, cfg.gamma, cfg.lam)[0])   # the mask matters
    plain, zero = run(None), run(np.zeros_like(trunc))
    for x, y in zip(plain, zero):
        assert np.array_equal(x, y)


def test_vec_gae_done_is_a_select_bit_exact(torch, binding):
    """Data behind an episode end (even NaN / Inf) never reaches the steps before it."""
    cfg = scaled(CONFIGS[2], name="gae-mask", N=512, P=16, T=24)
    say("vec_gae done-mask " + cfg.name)
    rng = np.random.default_rng(5)
    r = rng.standard_normal((cfg.T, cfg.N, cfg.K), dtype=np.float32)
    v = rng.standard_normal((cfg.T + 1, cfg.N, cfg.K), dtype=np.float32)
    w = inputs.make_preferences(cfg)
    done = np.zeros((cfg.T, cfg.N), dtype=np.uint8)
    cut = rng.integers(0, cfg.T, size=cfg.N)
    done[cut, np.arange(cfg.N)] = 1
    a0, vt0, s0 = run_gae(cfg, torch, binding, r, v, done, w)
    r2, v2 = r.copy(), v.copy()
    for n in range(cfg.N):
        r2[cut[n] + 1:, n] = np.nan
        v2[cut[n] + 1:, n] = np.inf if n % 2 else np.nan
    a1, vt1, s1 = run_gae(cfg, torch, binding, r2, v2, done, w)
    keep = np.arange(cfg.T)[:, None] <= cut[None, :]
    assert np.array_equal(a0[keep], a1[keep])
    assert np.array_equal(vt0[keep], vt1[keep])
    assert np.array_equal(s0[keep], s1[keep])
    assert np.isfinite(a1[keep]).all()
    # all-done: A = r - V exactly in fp32
    done[:] = 1
    a2, vt2, _ = run_gae(cfg, torch, binding, r, v, done, w)
    assert np.array_equal(a2, r - v[:-1])


# ------------------------------------------------------------------------------------------------
def loss_inputs(cfg, seed=40):
    rng = np.random.default_rng(seed)
    T, N, A, K, P = cfg.T, cfg.N, cfg.act_dim, cfg.K, cfg.P
    f32 = np.float32
    mu = np.tanh(rng.standard_normal((T, N, A), dtype=f32))
    logsig = (-0.5 + 0.1 * rng.standard_normal((P, A))).astype(f32)
    g = orc.env_pref_index(N, P)
    eps = rng.standard_normal((T, N, A), dtype=f32)
    mu_old = np.clip(mu + 0.05 * rng.standard_normal((T, N, A), dtype=f32), -1, 1).astype(f32)
    act = (mu_old + np.exp(logsig[g])[None] * eps).astype(f32)
    logp_old = orc.gaussian_logp(act.astype(np.float64), mu_old.astype(np.float64), logsig[g][None].astype(np.float64)).astype(f32)
    adv_s = (rng.standard_normal((T, N), dtype=f32) * 2 + 0.5).astype(f32)
    v = rng.standard_normal((T, N, K), dtype=f32)
    vtarg = rng.standard_normal((T, N, K), dtype=f32)
    return mu, logsig, act, logp_old, adv_s, v, vtarg


@pytest.mark.parametrize("cfg,mb,norm", [(CONFIGS[1], 0, 1), (RAGGED, 0, 1), (RAGGED, 1, 0), (CONFIGS[2], 0, 1),
                                         (CONFIGS[3], 0, 1), (CONFIGS[4], 0, 1), (CONFIGS[5], 2, 1)],
                         ids=lambda x: getattr(x, "name", str(x)))
def test_ppo_loss_grad_matches_oracle(cfg, mb, norm, torch, binding):
    say(f"ppo_loss_grad {cfg.name} mb={mb} norm={norm}")
    if cfg is RAGGED and mb == 1:
        rows = (2, 4, 5, 11)
    else:
        MB = cfg.minibatches
        rows = (0, cfg.T, mb * (cfg.n_g // MB), cfg.n_g // MB) if MB > 1 else (0, cfg.T, 0, cfg.n_g)
    mu, logsig, act, logp_old, adv_s, v, vtarg = loss_inputs(cfg)
    ctx = binding.Context.from_config(cfg)
    SENT = 3.25
    dmu = torch.full(mu.shape, SENT, device="cuda")
    dv = torch.full(v.shape, SENT, device="cuda")
    dls = torch.full(logsig.shape, SENT, device="cuda")
    stats = torch.zeros(8, device="cuda")
    ws = torch.empty(ctx.workspace_bytes(None), dtype=torch.uint8, device="cuda")
    # logsig passed as a strided view, as the actor's theta_vec tail is
    stride = cfg.act_dim + 5
    ls_pad = np.zeros((cfg.P, stride), dtype=np.float32)
    ls_pad[:, :cfg.act_dim] = logsig
    ctx.ppo_loss_grad(rows, dev(mu), dev(ls_pad), stride, dev(act), dev(logp_old), dev(adv_s), dev(v), dev(vtarg),
                      cfg.clip_eps, norm, dmu, dls, dv, stats, ws)
    torch.cuda.synchronize()
    o_dmu, o_dls, o_dv, o_st = orc.ppo_loss_grad(cfg, rows, mu, logsig, act, logp_old, adv_s, v, vtarg,
                                                 cfg.clip_eps, bool(norm))
    mask = orc.row_mask(cfg, rows, cfg.T)
    g_dmu, g_dv = to_np(dmu), to_np(dv)
    assert np.all(g_dmu[~mask] == SENT) and np.all(g_dv[~mask] == SENT)   # untouched outside the rows
    # samples whose ratio sits on the clip boundary may legitimately fall on either side in fp32
    gidx = orc.env_pref_index(cfg.N, cfg.P)
    logp = orc.gaussian_logp(act.astype(np.float64), mu.astype(np.float64), logsig[gidx][None].astype(np.float64))
    rho = np.exp(logp - logp_old)
    kink = (np.abs(rho - (1 + cfg.clip_eps)) < 1e-5) | (np.abs(rho - (1 - cfg.clip_eps)) < 1e-5)
    B = mask.sum()
    sc = float(B)   # gradients carry 1/B: compare B * gradient so the absolute tolerance is meaningful
    assert_close32(g_dmu * sc, o_dmu * sc, "dmu*B", mask=(mask & ~kink)[..., None] & np.ones_like(o_dmu, bool))
    assert_close32(g_dv * sc, o_dv * sc, "dv*B", mask=mask[..., None] & np.ones_like(o_dv, bool))
    if not kink[mask].any():
        assert_close32(to_np(dls), o_dls, "dlogsig", rel=1e-4, abs_=1e-5)
    st = to_np(stats)
    assert_close32(st[[0, 1, 3, 4, 5, 6]], o_st[[0, 1, 3, 4, 5, 6]], "stats", rel=1e-4, abs_=1e-5)
    assert abs(st[2] - o_st[2]) <= 2.0 / B and st[7] == B
    assert 0.02 < o_st[2] < 0.6


# ------------------------------------------------------------------------------------------------
def hyper_case(cfg, net):
    return inputs.make_hparams(cfg, net), inputs.make_preferences(cfg)


# the strictly affine hypernetwork (rank = -1): a ragged fp32 case, a bf16 case, and workload 3's shapes
AFFINE_CASES = [scaled(RAGGED, name="ragged-affine", rank=-1), scaled(RAGGED_BF16, name="ragged-bf16-affine", rank=-1),
                scaled(CONFIGS[3], name="cfg3-affine", rank=-1)]


@pytest.mark.parametrize("cfg", all_cfgs() + [RAGGED, RAGGED_BF16, scaled(RAGGED, name="rank0", rank=0)] + AFFINE_CASES,
                         ids=lambda c: c.name)
def test_hypernet_fwd_matches_oracle(cfg, torch, binding):
    ctx = binding.Context.from_config(cfg)
    ws = torch.empty(ctx.workspace_bytes(None), dtype=torch.uint8, device="cuda")
    for net in (ACTOR, CRITIC):
        say(f"hypernet_fwd {cfg.name} net={net}")
        hp, w = hyper_case(cfg, net)
        wdt = torch.bfloat16 if cfg.wdtype == 1 else torch.float32
        tm = torch.zeros(cfg.P, ctx.theta_mat_len(net), dtype=wdt, device="cuda")
        tv = torch.zeros(cfg.P, ctx.theta_vec_len(net), device="cuda")
        ctx.hypernet_fwd(net, dev(hp), dev(w), tm, tv, ws)
        torch.cuda.synchronize()
        o_tm, o_tv = orc.hypernet_fwd(cfg, net, hp, w)
        assert_close32(to_np(tv), o_tv, "theta_vec")
        g_tm = to_np(tm)
        if cfg.wdtype == 0:
            assert_close32(g_tm, o_tm, "theta_mat")
        else:
            # every stored value is a bf16 within half an ulp (+ fp32 noise) of the exact weight, and
            # nearly all equal the oracle's own rounding
            nbad = int(np.sum(~(np.abs(g_tm - o_tm) <= 2.0 ** -8 * np.abs(o_tm) * (1 + 1e-3) + 1e-6)))
            assert nbad == 0, nbad
            same = np.mean(g_tm == orc.round_bf16(o_tm))
            assert same > 0.999, same


# (more than 128 preferences: the backward's two-pass dM / df kernels instead of the fused one)
@pytest.mark.parametrize("cfg", all_cfgs() + [RAGGED, scaled(RAGGED, name="rank0", rank=0),
                                             scaled(RAGGED, name="ragged-P130", P=130, N=260),
                                             scaled(RAGGED, name="ragged-P130-affine", P=130, N=260, rank=-1)] + AFFINE_CASES,
                         ids=lambda c: c.name)
def test_hypernet_bwd_matches_oracle(cfg, torch, binding):
    ctx = binding.Context.from_config(cfg)
    ws = torch.empty(ctx.workspace_bytes(None), dtype=torch.uint8, device="cuda")
    for net in (ACTOR, CRITIC):
        say(f"hypernet_bwd {cfg.name} net={net}")
        hp, w = hyper_case(cfg, net)
        rng = np.random.default_rng(70 + net)
        ml, vl = ctx.theta_mat_len(net), ctx.theta_vec_len(net)
        # gradient scale chosen so that the reduced outputs are O(1)
        dtm = (rng.standard_normal((cfg.P, ml), dtype=np.float32) / np.float32(np.sqrt(cfg.P * cfg.width))).astype(np.float32)
        dtv = (rng.standard_normal((cfg.P, vl), dtype=np.float32) / np.float32(np.sqrt(cfg.P))).astype(np.float32)
        dhp = torch.full((ctx.hparam_count(net),), 9.0, device="cuda")
        ctx.hypernet_bwd(net, dev(hp), dev(w), dev(dtm), dev(dtv), dhp, ws)
        torch.cuda.synchronize()
        ref = orc.hypernet_bwd(cfg, net, hp, w, dtm, dtv)
        got = to_np(dhp)
        lay = orc.hparam_layout(cfg, net)
        for name, (o, s) in lay.items():
            if name == "_total":
                continue
            n = int(np.prod(s))
            assert_close32(got[o:o + n], ref[o:o + n], f"dhparams[{name}]")


@pytest.mark.parametrize("cfg", [CONFIGS[1], RAGGED, CONFIGS[3], AFFINE_CASES[0]], ids=lambda c: c.name)
def test_hypernet_bwd_kept_equals_hypernet_bwd(cfg, torch, binding):
    """The backward pass that reads the forward pass's workspace gives the gradient of the one that recomputes,
    bit for bit."""
    ctx = binding.Context.from_config(cfg)
    for net in (ACTOR, CRITIC):
        say(f"hypernet_bwd_kept {cfg.name} net={net}")
        hp, w = hyper_case(cfg, net)
        rng = np.random.default_rng(90 + net)
        ml, vl = ctx.theta_mat_len(net), ctx.theta_vec_len(net)
        dtm = dev((rng.standard_normal((cfg.P, ml), dtype=np.float32) * 0.01).astype(np.float32))
        dtv = dev((rng.standard_normal((cfg.P, vl), dtype=np.float32) * 0.01).astype(np.float32))
        wdt = torch.bfloat16 if cfg.wdtype == 1 else torch.float32
        tm = torch.zeros(cfg.P, ml, dtype=wdt, device="cuda")
        tv = torch.zeros(cfg.P, vl, device="cuda")
        ws_f = torch.empty(ctx.workspace_bytes((0, 1, 0, 1)), dtype=torch.uint8, device="cuda")
        ws_b = torch.empty(ctx.workspace_bytes(None), dtype=torch.uint8, device="cuda")
        d_hp, d_w = dev(hp), dev(w)
        ctx.hypernet_fwd(net, d_hp, d_w, tm, tv, ws_f)
        g_kept = torch.full((ctx.hparam_count(net),), 9.0, device="cuda")
        ctx.hypernet_bwd_kept(net, d_hp, d_w, dtm, dtv, g_kept, ws_f)
        g_ref = torch.full((ctx.hparam_count(net),), 7.0, device="cuda")
        ctx.hypernet_bwd(net, d_hp, d_w, dtm, dtv, g_ref, ws_b)
        torch.cuda.synchronize()
        assert torch.equal(g_kept, g_ref)


# ------------------------------------------------------------------------------------------------
def theta_for(cfg, net, emulate):
    hp, w = hyper_case(cfg, net)
    tm, tv = orc.hypernet_fwd(cfg, net, hp, w)
    if cfg.wdtype == 1:
        tm = orc.round_bf16(tm)      # the bf16 weights are the network's weights on both sides
    else:
        tm = tm.astype(np.float32).astype(np.float64)
    return tm, tv


def sample_prefs(cfg):
    if cfg.P * cfg.N * cfg.T * cfg.width * cfg.width < 3e12:
        return None
    return sorted({0, cfg.P // 3 + 1, cfg.P - 1})


def pref_env_mask(cfg, prefs):
    if prefs is None:
        return np.ones(cfg.N, dtype=bool)
    g = orc.env_pref_index(cfg.N, cfg.P)
    return np.isin(g, prefs)


# every documented maximum at once: 16 objectives, 16 actions, observation width 1024, layer width 2048,
# factor rank 32, 64 hypernet features; two preferences.  fp32: the whole update step.  bf16: the target networks'
# forward and backward (1600 rows per preference), not the step -- with 26 M hypernet parameters the trunk's
# gradient is a heavily cancelling sum whose bf16 rounding noise alone passes 2 % of its RMS
LIMITS = scaled(RAGGED, name="limits-fp32", K=16, act_dim=16, obs_dim=1024, width=2048, n_hidden=2, rank=32,
                hyper_width=64, P=2, N=2 * 9, T=4, minibatches=1, epochs=1)
LIMITS_BF16 = scaled(LIMITS, name="limits-bf16", wdtype=1, N=2 * 400)


FWD_CASES = [(CONFIGS[1], None), (CONFIGS[1], (3, 9, 5, 7)), (RAGGED, None), (RAGGED, (1, 5, 2, 19)),
             (RAGGED_BF16, None), (RAGGED_BF16, (0, 3, 7, 140)), (CONFIGS[2], None), (CONFIGS[3], None),
             (CONFIGS[4], None), (CONFIGS[5], None), (CONFIGS[5], "mb"), (RAGGED_FUSED, None),
             (RAGGED_FUSED, (2, 5, 3, 30)), (RAGGED_FUSED_TANH, None)] + [(c, None) for c in SIGMA_CASES] + \
            [(SIGMA_CASES[2], (1, 5, 2, 19)), (RAGGED_FUSED, (3, 1, 5, 1)), (RAGGED_FUSED_WIDE, None), (LIMITS_BF16, None)] + \
            RANDOM_FUSED + [(c, None) for c in FUSED_ODD_OBS] + [(FUSED_ODD_OBS[0], (2, 5, 3, 30))] + \
            [(c, None) for c in FUSED_W256] + [(FUSED_W256[2], (2, 5, 3, 30)), (FUSED_W256[0], (3, 1, 5, 1))]


@pytest.mark.parametrize("cfg,rows", FWD_CASES, ids=lambda x: getattr(x, "name", str(x)))
def test_policy_fwd_matches_oracle(cfg, rows, torch, binding):
    ctx = binding.Context.from_config(cfg)
    traj = inputs.make_trajectory(cfg)
    x, eps = traj["obs"], traj["eps"]
    if rows == "mb":
        rows = (0, cfg.T, cfg.n_g // cfg.minibatches, cfg.n_g // cfg.minibatches)
    prefs = sample_prefs(cfg)
    emask = pref_env_mask(cfg, prefs)
    close = assert_close32 if cfg.wdtype == 0 else assert_close_bf16
    for net in (ACTOR, CRITIC):
        r = rows if rows is not None else ((0, cfg.T, 0, cfg.n_g) if net == ACTOR else (0, cfg.T + 1, 0, cfg.n_g))
        say(f"policy_fwd {cfg.name} net={net} rows={r} prefs={prefs}")
        tm, tv = theta_for(cfg, net, True)
        wdt = torch.bfloat16 if cfg.wdtype == 1 else torch.float32
        odim = orc.head_dim(cfg, net)
        SENT = -7.5
        out = torch.full((cfg.T + 1, cfg.N, odim), SENT, device="cuda")
        ws = torch.empty(ctx.workspace_bytes(r), dtype=torch.uint8, device="cuda")
        d_tm, d_tv, d_x = dev(tm, wdt), dev(tv.astype(np.float32)), dev(x)
        kw = {}
        if net == ACTOR:
            eps_pad = np.zeros((cfg.T + 1, cfg.N, cfg.act_dim), dtype=np.float32)
            eps_pad[:cfg.T] = eps
            act = torch.full((cfg.T + 1, cfg.N, cfg.act_dim), SENT, device="cuda")
            logp = torch.full((cfg.T + 1, cfg.N), SENT, device="cuda")
            kw = dict(eps=dev(eps_pad), act=act, logp=logp)
        ctx.policy_fwd(net, d_tm, d_tv, d_x, r, out, ws=ws, **kw)
        torch.cuda.synchronize()
        emu = cfg.wdtype == 1
        o_out, o_act, o_logp = orc.policy_fwd(cfg, net, tm, tv.astype(np.float32), x, r,
                                              eps=(eps_pad if net == ACTOR else None), emulate_bf16=emu,
                                              prefs=prefs)
        mask = orc.row_mask(cfg, r, cfg.T + 1)
        g_out = to_np(out)
        assert np.all(g_out[~mask] == SENT)
        cmp = mask & emask[None, :]
        m3 = cmp[..., None] & np.ones_like(o_out, bool)
        close(g_out, o_out, f"out net={net}", mask=m3)
        if net == ACTOR:
            g_act, g_logp = to_np(act), to_np(logp)
            assert np.all(g_act[~mask] == SENT) and np.all(g_logp[~mask] == SENT)
            close(g_act, o_act, "act", mask=cmp[..., None] & np.ones_like(o_act, bool))
            if cfg.sigma_state:
                close(g_logp, o_logp, "logp", mask=cmp)        # log sigma is an output of the network here
            else:
                assert_close32(g_logp, o_logp, "logp", mask=cmp)   # depends on eps and log sigma only
        if emu and prefs is None:
            # against exact activations (same bf16 weights) the difference is the bf16 rounding noise of
            # the method itself: small in RMS, a few-sigma tail on single elements
            o2, _, _ = orc.policy_fwd(cfg, net, tm, tv.astype(np.float32), x, r, emulate_bf16=False)
            e2 = rel_rms_err(g_out[m3], o2[m3])
            assert e2 < 1e-2, e2
        # saving activations for the backward pass must not change the outputs
        saved = torch.empty(ctx.saved_bytes(net, r), dtype=torch.uint8, device="cuda")
        out2 = torch.full_like(out, SENT)
        ctx.policy_fwd(net, d_tm, d_tv, d_x, r, out2, saved=saved, ws=ws)
        torch.cuda.synchronize()
        assert torch.equal(out, out2)


BWD_CASES = [(CONFIGS[1], None), (RAGGED, None), (RAGGED, (1, 5, 2, 19)), (RAGGED_BF16, None),
             (RAGGED_BF16, (0, 3, 7, 140)), (CONFIGS[2], None), (CONFIGS[3], None), (CONFIGS[4], None),
             (CONFIGS[5], "mb"), (RAGGED_FUSED, None), (RAGGED_FUSED_TANH, (1, 6, 0, 37))] + \
            [(c, None) for c in SIGMA_CASES] + \
            [(RAGGED_FUSED, (3, 1, 5, 1)), (scaled(RAGGED_FUSED_WIDE, name="ragged-fused-bf16-obs512-3layers", n_hidden=3), None)] + \
            RANDOM_FUSED + [(LIMITS_BF16, None)] + [(c, None) for c in FUSED_ODD_OBS] + [(FUSED_ODD_OBS[1], (2, 5, 3, 30))] + \
            [(c, None) for c in FUSED_W256] + [(FUSED_W256[1], (2, 5, 3, 30))]
# (the eight-layer network has a test of its own below, test_policy_bwd_eight_hidden_layers_bf16)


@pytest.mark.parametrize("cfg,rows", BWD_CASES, ids=lambda x: getattr(x, "name", str(x)))
def test_policy_bwd_matches_oracle(cfg, rows, torch, binding):
    ctx = binding.Context.from_config(cfg)
    x = inputs.make_trajectory(cfg)["obs"][:cfg.T]
    if rows == "mb":
        rows = (0, cfg.T, cfg.n_g // cfg.minibatches, cfg.n_g // cfg.minibatches)
    if rows is None:
        rows = (0, cfg.T, 0, cfg.n_g)
    prefs = sample_prefs(cfg)
    close = assert_close32 if cfg.wdtype == 0 else assert_close_bf16
    B = rows[1] * rows[3] * cfg.P
    for net in (ACTOR, CRITIC):
        say(f"policy_bwd {cfg.name} net={net} rows={rows} prefs={prefs}")
        tm, tv = theta_for(cfg, net, True)
        wdt = torch.bfloat16 if cfg.wdtype == 1 else torch.float32
        odim = orc.head_dim(cfg, net)
        rng = np.random.default_rng(80 + net)
        dout = (rng.standard_normal((cfg.T, cfg.N, odim), dtype=np.float32) / np.float32(np.sqrt(rows[1] * rows[3])))
        dls = rng.standard_normal((cfg.P, cfg.act_dim), dtype=np.float32) if (net == ACTOR and not cfg.sigma_state) else None
        d_tm, d_tv, d_x = dev(tm, wdt), dev(tv.astype(np.float32)), dev(x)
        ws = torch.empty(ctx.workspace_bytes(rows), dtype=torch.uint8, device="cuda")
        saved = torch.empty(ctx.saved_bytes(net, rows), dtype=torch.uint8, device="cuda")
        out = torch.zeros(cfg.T, cfg.N, odim, device="cuda")
        ctx.policy_fwd(net, d_tm, d_tv, d_x, rows, out, saved=saved, ws=ws)
        dtm = torch.full((cfg.P, ctx.theta_mat_len(net)), 5.0, device="cuda")
        dtv = torch.full((cfg.P, ctx.theta_vec_len(net)), 5.0, device="cuda")
        d_dout, d_dls = dev(dout), (dev(dls) if dls is not None else None)
        ctx.policy_bwd(net, d_tm, d_tv, d_x, rows, saved, d_dout, d_dls, dtm, dtv, ws)
        # every sum of the backward pass has a fixed order (split contractions and partial sums included): a second
        # call on the same saved activations returns the same bits
        dtm2, dtv2 = torch.full_like(dtm, -3.0), torch.full_like(dtv, -3.0)
        ctx.policy_bwd(net, d_tm, d_tv, d_x, rows, saved, d_dout, d_dls, dtm2, dtv2, ws)
        torch.cuda.synchronize()
        assert torch.equal(dtm, dtm2) and torch.equal(dtv, dtv2)
        del dtm2, dtv2
        emu = cfg.wdtype == 1
        o_dtm, o_dtv = orc.policy_bwd(cfg, net, tm, tv.astype(np.float32), x, rows, dout, dls, emulate_bf16=emu,
                                      prefs=prefs)
        g_dtm, g_dtv = to_np(dtm), to_np(dtv)
        sel = list(range(cfg.P)) if prefs is None else prefs
        moff = voff = 0
        for l, (do, di) in enumerate(orc.layer_shapes(cfg, net)):
            close(g_dtm[sel, moff:moff + do * di], o_dtm[sel, moff:moff + do * di], f"dW_{l} net={net}")
            close(g_dtv[sel, voff:voff + do], o_dtv[sel, voff:voff + do], f"db_{l} net={net}")
            moff += do * di
            voff += do
        if net == ACTOR and not cfg.sigma_state:
            assert np.array_equal(g_dtv[:, voff:], dls)
        else:
            assert voff == g_dtv.shape[1]
        if emu and prefs is None:
            o2, _ = orc.policy_bwd(cfg, net, tm, tv.astype(np.float32), x, rows, dout, dls, emulate_bf16=False)
            e = rel_rms_err(g_dtm, o2)
            assert e < 2e-2, e


def test_policy_bwd_eight_hidden_layers_bf16(torch, binding):
    """The deepest network the library takes (eight hidden layers), bf16.  Both sides re-round every activation and
    every dZ at every layer, so single elements of the first layers' gradients differ by accumulated rounding flips
    by more than the 2 % band of one rounding; what is bounded instead is each layer's error in the RMS sense,
    against the emulating oracle and against the exact one, with the element-wise band widened by sqrt(depth)."""
    cfg = RAGGED_FUSED_WIDE
    assert cfg.n_hidden == 8
    ctx = binding.Context.from_config(cfg)
    x = inputs.make_trajectory(cfg)["obs"][:cfg.T]
    rows = (0, cfg.T, 0, cfg.n_g)
    for net in (ACTOR, CRITIC):
        say(f"policy_bwd eight hidden layers {cfg.name} net={net}")
        tm, tv = theta_for(cfg, net, True)
        odim = orc.head_dim(cfg, net)
        rng = np.random.default_rng(80 + net)
        dout = (rng.standard_normal((cfg.T, cfg.N, odim), dtype=np.float32) / np.float32(np.sqrt(rows[1] * rows[3])))
        dls = rng.standard_normal((cfg.P, cfg.act_dim), dtype=np.float32) if net == ACTOR else None
        d_tm, d_tv, d_x = dev(tm, torch.bfloat16), dev(tv.astype(np.float32)), dev(x)
        ws = torch.empty(ctx.workspace_bytes(rows), dtype=torch.uint8, device="cuda")
        saved = torch.empty(ctx.saved_bytes(net, rows), dtype=torch.uint8, device="cuda")
        out = torch.zeros(cfg.T, cfg.N, odim, device="cuda")
        ctx.policy_fwd(net, d_tm, d_tv, d_x, rows, out, saved=saved, ws=ws)
        dtm = torch.full((cfg.P, ctx.theta_mat_len(net)), 5.0, device="cuda")
        dtv = torch.full((cfg.P, ctx.theta_vec_len(net)), 5.0, device="cuda")
        ctx.policy_bwd(net, d_tm, d_tv, d_x, rows, saved, dev(dout), dev(dls) if dls is not None else None, dtm, dtv, ws)
        torch.cuda.synchronize()
        o_dtm, o_dtv = orc.policy_bwd(cfg, net, tm, tv.astype(np.float32), x, rows, dout, dls, emulate_bf16=True)
        e_dtm, e_dtv = orc.policy_bwd(cfg, net, tm, tv.astype(np.float32), x, rows, dout, dls, emulate_bf16=False)
        g_dtm, g_dtv = to_np(dtm), to_np(dtv)
        moff = voff = 0
        depth = cfg.n_hidden + 1
        for l, (do, di) in enumerate(orc.layer_shapes(cfg, net)):
            sl, sv = slice(moff, moff + do * di), slice(voff, voff + do)
            r_emu, r_exact = rel_rms_err(g_dtm[:, sl], o_dtm[:, sl]), rel_rms_err(g_dtm[:, sl], e_dtm[:, sl])
            say(f"  layer {l}: rel. RMS error {r_emu:.4f} (emulating oracle) {r_exact:.4f} (exact oracle)")
            assert r_emu < 2e-2 and r_exact < 2e-2, (l, r_emu, r_exact)
            assert rel_rms_err(g_dtv[:, sv], o_dtv[:, sv]) < 2e-2
            wide = 2e-2 * float(np.sqrt(depth - l))       # roundings between this layer's dZ and the output
            assert_close_bf16(g_dtm[:, sl], o_dtm[:, sl], f"dW_{l} net={net}", rel=wide)
            assert_close_bf16(g_dtv[:, sv], o_dtv[:, sv], f"db_{l} net={net}", rel=wide)
            moff += do * di
            voff += do


# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("cfg,n_steps", [(CONFIGS[1], 4), (RAGGED, 3), (CONFIGS[5], 2)], ids=lambda x: getattr(x, "name", str(x)))
def test_adam_step_matches_oracle(cfg, n_steps, torch, binding):
    say(f"adam_step {cfg.name}")
    ctx = binding.Context.from_config(cfg)
    rng = np.random.default_rng(21)
    for net, lr in ((ACTOR, 3e-4), (CRITIC, 1e-3)):
        n = ctx.hparam_count(net)
        th = rng.standard_normal(n).astype(np.float32)
        m = np.zeros(n); v = np.zeros(n); ref = th.astype(np.float64)
        d_th, d_m, d_v = dev(th), torch.zeros(n, device="cuda"), torch.zeros(n, device="cuda")
        for t in range(1, n_steps + 1):
            g = (rng.standard_normal(n) * np.exp(rng.standard_normal(n))).astype(np.float32)
            before = to_np(d_th).astype(np.float64)
            ctx.adam_step(net, d_th, dev(g), d_m, d_v, lr, 0.9, 0.999, 1e-8, t)
            torch.cuda.synchronize()
            # one step from the device's own state (so fp32 drift of earlier steps is not compared twice)
            o_th, o_m, o_v = orc.adam_step(before, g, m, v, lr, 0.9, 0.999, 1e-8, t)
            got_th, got_m, got_v = to_np(d_th), to_np(d_m), to_np(d_v)
            # m mixes terms of either sign: fp32 rounding is relative to the operands, not to their sum
            err_m = np.abs(got_m - o_m)
            assert (err_m <= 1e-4 * np.abs(o_m) + 3e-7 * (np.abs(m) + np.abs(g))).all(), (net, t, float(err_m.max()))
            assert_close32(got_v, o_v, f"v net {net} t {t}", abs_=1e-12)
            # the step itself: relative 1e-4 of lr-sized moves, plus the fp32 rounding of theta - step
            assert_close32(got_th - before, o_th - before, f"step net {net} t {t}", rel=1e-4,
                           abs_=1e-4 * lr + 1.2e-7 * float(np.abs(before).max()))
            m, v = got_m.astype(np.float64), got_v.astype(np.float64)
        assert np.abs(to_np(d_th) - th).max() > 0.5 * lr


@pytest.mark.parametrize("schedule", ["serial", "side_hypernet", "two_streams"])
def test_update_step_with_optimizer_matches_oracle(schedule, torch, binding):
    """A true PPO update: each minibatch is followed by an Adam step with a learning rate per hypernet.  The
    stream schedules only reorder independent launches, so each must reach the same parameters."""
    from paper_2603_09237_amd.step import UpdateStep
    cfg = scaled(CONFIGS[1], name="cfg1-adam", minibatches=2, epochs=2)
    say(f"update_step + adam {cfg.name} {schedule}")
    opt = dict(lr_actor=3e-3, lr_critic=1e-2, beta1=0.9, beta2=0.999, eps=1e-8)
    st = UpdateStep(cfg, optimizer=opt, side_hypernet=(schedule == "side_hypernet"),
                    two_streams=(schedule == "two_streams"))
    d = inputs.make_all(cfg)
    st.load_inputs(d)
    st.run()
    torch.cuda.synchronize()
    res = orc.update_step(cfg, d["w"], d["hparams_actor_old"], d["hparams_critic_old"], d["hparams_actor"],
                          d["hparams_critic"], d["obs"], d["rewards"], d["dones"], d["eps"], cfg.gamma, cfg.lam,
                          cfg.clip_eps, cfg.minibatches, cfg.epochs, optimizer=opt)
    n_steps = cfg.minibatches * cfg.epochs
    for net, key, lr, start in ((ACTOR, "hp_actor", opt["lr_actor"], d["hparams_actor"]),
                                (CRITIC, "hp_critic", opt["lr_critic"], d["hparams_critic"])):
        got, ref = to_np(st.hp[net]).astype(np.float64), res[key]
        moved = np.abs(ref - start)
        assert moved.max() > 0.5 * lr          # the parameters did move
        # Adam's step is g / (|g| + eps)-like: where a gradient is within rounding of zero its sign, and so a
        # whole lr-sized move, is not determined; those coordinates get a budget of one move per step
        gkey = "dhp_actor" if net == ACTOR else "dhp_critic"
        small = np.zeros(ref.shape, dtype=bool)
        for name, (o, shp) in orc.hparam_layout(cfg, net).items():   # gradient rounding scales with its block
            if name == "_total":
                continue
            sl = slice(o, o + int(np.prod(shp)))
            for g in res["grads"]:
                small[sl] |= np.abs(g[gkey][sl]) < 2e-3 * max(float(np.abs(g[gkey][sl]).max()), 1e-30)
        err = np.abs(got - ref)
        assert (err[~small] <= 2e-2 * lr * n_steps + 1e-6).all(), (net, float(err[~small].max()))
        assert (err[small] <= 2.0 * lr * n_steps + 1e-6).all(), (net, float(err[small].max()))
        assert (~small).mean() > 0.5, float((~small).mean())


@pytest.mark.parametrize("cfg,rows", [(CONFIGS[1], None), (RAGGED, (1, 5, 2, 19)), (CONFIGS[3], None), (CONFIGS[5], "mb"),
                                      (scaled(RAGGED, name="ragged-K16", K=16, T=19), None)],
                         ids=lambda x: getattr(x, "name", str(x)))
def test_scalarize_normalized_matches_oracle(cfg, rows, torch, binding):
    """Per-objective standardisation + scalarisation of a vector advantage whose objectives differ in scale."""
    ctx = binding.Context.from_config(cfg)
    if rows == "mb":
        rows = (0, cfg.T, cfg.n_g // cfg.minibatches, cfg.n_g // cfg.minibatches)
    if rows is None:
        rows = (0, cfg.T, 0, cfg.n_g)
    say(f"scalarize_normalized {cfg.name} rows={rows}")
    rng = np.random.default_rng([11, cfg.K, cfg.N])
    scale = 10.0 ** rng.uniform(-1, 1, size=cfg.K)
    adv = (rng.standard_normal((cfg.T, cfg.N, cfg.K)) * scale + rng.standard_normal(cfg.K) * scale).astype(np.float32)
    w = inputs.make_all(cfg)["w"]
    SENT = -7.5
    out = torch.full((cfg.T, cfg.N), SENT, device="cuda")
    ws = torch.empty(ctx.workspace_bytes(rows), dtype=torch.uint8, device="cuda")
    ctx.scalarize_normalized(rows, dev(adv), dev(w), out, ws)
    torch.cuda.synchronize()
    ref = orc.scalarize_normalized(cfg, rows, adv, w)
    mask = orc.row_mask(cfg, rows, cfg.T)
    got = to_np(out)
    assert np.all(got[~mask] == SENT)                      # cells outside the selection are not written
    assert_close32(got, ref, "adv_out", mask=mask)
    assert np.abs(ref[mask]).max() > 0.5


def test_update_step_per_objective_normalisation_matches_oracle(torch, binding):
    from paper_2603_09237_amd.step import UpdateStep
    cfg = scaled(CONFIGS[1], name="cfg1-advk", minibatches=2, epochs=1)
    say(f"update_step per-objective normalisation {cfg.name}")
    st = UpdateStep(cfg, adv_norm="per_objective")
    d = inputs.make_all(cfg)
    st.load_inputs(d)
    grads = []

    def grab(e, b):
        torch.cuda.synchronize()
        grads.append((to_np(st.dhp[ACTOR]).copy(), to_np(st.dhp[CRITIC]).copy()))

    st.run(on_minibatch=grab)
    torch.cuda.synchronize()
    res = orc.update_step(cfg, d["w"], d["hparams_actor_old"], d["hparams_critic_old"], d["hparams_actor"],
                          d["hparams_critic"], d["obs"], d["rewards"], d["dones"], d["eps"], cfg.gamma, cfg.lam,
                          cfg.clip_eps, cfg.minibatches, cfg.epochs, adv_norm="per_objective")
    plain = orc.update_step(cfg, d["w"], d["hparams_actor_old"], d["hparams_critic_old"], d["hparams_actor"],
                            d["hparams_critic"], d["obs"], d["rewards"], d["dones"], d["eps"], cfg.gamma, cfg.lam,
                            cfg.clip_eps, cfg.minibatches, cfg.epochs)
    for i, (ga, gc) in enumerate(grads):
        for net, got, key in ((ACTOR, ga, "dhp_actor"), (CRITIC, gc, "dhp_critic")):
            ref = res["grads"][i][key]
            for name, (o, shp) in orc.hparam_layout(cfg, net).items():
                if name == "_total":
                    continue
                sl = slice(o, o + int(np.prod(shp)))
                sc = max(float(np.abs(ref[sl]).max()), 1e-30)
                assert np.abs(got[sl] - ref[sl]).max() <= 1e-3 * sc + 1e-7, (i, key, name)
        # and it is not the other reading
        assert np.abs(ga - plain["grads"][i]["dhp_actor"]).max() > 1e-2 * np.abs(ga).max()


@pytest.mark.parametrize("cfg", [SIGMA_CASES[0], SIGMA_CASES[1], SIGMA_CASES[2]], ids=lambda c: c.name)
def test_ppo_loss_grad_state_sigma_matches_oracle(cfg, torch, binding):
    """The loss with log sigma per cell (columns A .. 2A of the actor's output); its gradient stays per cell."""
    say(f"ppo_loss_grad state-dependent sigma {cfg.name}")
    A = cfg.act_dim
    mu, logsig, act, logp_old, adv_s, v, vtarg = loss_inputs(cfg)
    rng = np.random.default_rng(41)
    gidx = orc.env_pref_index(cfg.N, cfg.P)
    ls = (logsig[gidx][None] + 0.05 * rng.standard_normal(mu.shape)).astype(np.float32)     # per-cell log sigma
    out = np.concatenate([mu, ls], axis=-1).astype(np.float32)
    rows = (0, cfg.T, 0, cfg.n_g)
    ctx = binding.Context.from_config(cfg)
    SENT = 3.25
    dout = torch.full(out.shape, SENT, device="cuda")
    dv = torch.full(v.shape, SENT, device="cuda")
    stats = torch.zeros(8, device="cuda")
    ws = torch.empty(ctx.workspace_bytes(None), dtype=torch.uint8, device="cuda")
    ctx.ppo_loss_grad(rows, dev(out), None, 0, dev(act), dev(logp_old), dev(adv_s), dev(v), dev(vtarg), cfg.clip_eps, 1,
                      dout, None, dv, stats, ws)
    torch.cuda.synchronize()
    o_d, o_none, o_dv, o_st = orc.ppo_loss_grad(cfg, rows, out, None, act, logp_old, adv_s, v, vtarg, cfg.clip_eps, True)
    assert o_none is None and o_d.shape[-1] == 2 * A
    logp = orc.gaussian_logp(act.astype(np.float64), mu.astype(np.float64), ls.astype(np.float64))
    rho = np.exp(logp - logp_old)
    kink = (np.abs(rho - (1 + cfg.clip_eps)) < 1e-5) | (np.abs(rho - (1 - cfg.clip_eps)) < 1e-5)
    B = float(cfg.T * cfg.N)
    ok = (~kink)[..., None] & np.ones_like(o_d, bool)
    assert_close32(to_np(dout) * B, o_d * B, "d(out)*B", mask=ok)
    assert_close32(to_np(dv) * B, o_dv * B, "dv*B")
    st = to_np(stats)
    assert_close32(st[[0, 1, 3, 4, 5, 6]], o_st[[0, 1, 3, 4, 5, 6]], "stats", rel=1e-4, abs_=1e-5)
    assert np.abs(o_d[..., A:]).max() * B > 0.1          # the log-sigma gradient is there


def run_step(cfg, torch, keep_adv_vec=True):
    from paper_2603_09237_amd.step import UpdateStep
    st = UpdateStep(cfg, keep_adv_vec=keep_adv_vec)
    d = inputs.make_all(cfg)
    st.load_inputs(d)
    grads = []

    def grab(e, b):
        torch.cuda.synchronize()
        grads.append((to_np(st.dhp[ACTOR]).copy(), to_np(st.dhp[CRITIC]).copy(), to_np(st.stats).copy()))

    st.run(on_minibatch=grab)
    torch.cuda.synchronize()
    return st, d, grads


@pytest.mark.parametrize("cfg", [CONFIGS[1], scaled(CONFIGS[1], name="cfg1-mb2x2", minibatches=2, epochs=2),
                                 scaled(RAGGED, name="ragged-step", minibatches=1), CONFIGS[2], LIMITS,
                                 scaled(CONFIGS[1], name="cfg1-affine-step", rank=-1, minibatches=2, epochs=1),
                                 scaled(CONFIGS[1], name="cfg1-sigma-step", sigma_state=1, minibatches=2, epochs=1),
                                 scaled(RAGGED, name="ragged-sigma-step", sigma_state=1, minibatches=1)],
                         ids=lambda c: c.name)
def test_update_step_fp32_matches_oracle(cfg, torch, binding):
    say(f"update_step fp32 {cfg.name}")
    st, d, grads = run_step(cfg, torch)
    res = orc.update_step(cfg, d["w"], d["hparams_actor_old"], d["hparams_critic_old"], d["hparams_actor"],
                          d["hparams_critic"], d["obs"], d["rewards"], d["dones"], d["eps"], cfg.gamma, cfg.lam,
                          cfg.clip_eps, cfg.minibatches, cfg.epochs, keep=True)
    assert_close32(to_np(st.mu_old), res["mu_old"], "mu_old")
    assert_close32(to_np(st.act), res["act"], "act")
    assert_close32(to_np(st.logp_old), res["logp_old"], "logp_old")
    assert_close32(to_np(st.v_roll), res["v_roll"], "v_roll")
    assert_close32(to_np(st.adv_vec), res["adv_vec"], "adv_vec")
    assert_close32(to_np(st.vtarg), res["vtarg"], "vtarg")
    assert_close32(to_np(st.adv_s), res["adv_s"], "adv_s")
    assert len(grads) == cfg.minibatches * cfg.epochs
    for i, (ga, gc, stt) in enumerate(grads):
        ref = res["grads"][i]
        assert_close32(stt[[0, 1, 3, 4, 5, 6]], ref["stats"][[0, 1, 3, 4, 5, 6]], "stats")
        assert abs(stt[2] - ref["stats"][2]) <= 2.0 / stt[7]
        assert 0.02 < ref["stats"][2] < 0.6          # the clipped branch is exercised end to end
        # hypernet gradients, element by element at the fp32 tolerance; the absolute part is in units of the
        # block's largest entry (the gradients carry 1/B and differ in scale from block to block)
        for key, g, net in (("dhp_actor", ga, ACTOR), ("dhp_critic", gc, CRITIC)):
            lay = orc.hparam_layout(cfg, net)
            for name, (o, s) in lay.items():
                if name == "_total":
                    continue
                n = int(np.prod(s))
                r = ref[key][o:o + n]
                scale = max(float(np.abs(r).max()), 1e-12)
                assert_close32(g[o:o + n] / scale, r / scale, f"{key}[{name}] mb {i}")


@pytest.mark.parametrize("cfg", [scaled(RAGGED_BF16, name="ragged-bf16-step", minibatches=2), RAGGED_PERS, CONFIGS[3],
                                 scaled(RAGGED_FUSED, name="ragged-fused-step", minibatches=1, epochs=1),
                                 scaled(FUSED_ODD_OBS[0], name="ragged-fused-obs27-step", minibatches=1, epochs=1),
                                 scaled(FUSED_W256[2], name="ragged-fused-w256-obs11-step", minibatches=1, epochs=1),
                                 scaled(RAGGED_FUSED, name="ragged-fused-sigma-step", minibatches=1, epochs=1,
                                        sigma_state=1)],
                         ids=lambda c: c.name)
def test_update_step_bf16_matches_oracle(cfg, torch, binding):
    say(f"update_step bf16 {cfg.name}")
    st, d, grads = run_step(cfg, torch)
    res = orc.update_step(cfg, d["w"], d["hparams_actor_old"], d["hparams_critic_old"], d["hparams_actor"],
                          d["hparams_critic"], d["obs"], d["rewards"], d["dones"], d["eps"], cfg.gamma, cfg.lam,
                          cfg.clip_eps, cfg.minibatches, cfg.epochs, emulate_bf16=True, keep=True)
    assert_close_bf16(to_np(st.mu_old), res["mu_old"], "mu_old")
    assert_close_bf16(to_np(st.act), res["act"], "act")
    # (with a state-dependent sigma the log-density depends on a bf16 network output)
    (assert_close_bf16 if cfg.sigma_state else assert_close32)(to_np(st.logp_old), res["logp_old"], "logp_old")
    assert_close_bf16(to_np(st.v_roll), res["v_roll"], "v_roll")
    assert_close_bf16(to_np(st.vtarg), res["vtarg"], "vtarg")
    assert_close_bf16(to_np(st.adv_s), res["adv_s"], "adv_s")
    for i, (ga, gc, stt) in enumerate(grads):
        ref = res["grads"][i]
        assert_close_bf16(stt[:2], ref["stats"][:2], "losses")
        for key, g, net in (("dhp_actor", ga, ACTOR), ("dhp_critic", gc, CRITIC)):
            lay = orc.hparam_layout(cfg, net)
            for name, (o, s) in lay.items():
                if name == "_total":
                    continue
                n = int(np.prod(s))
                # (end of a chain of re-rounded layers: RMS bound, single-GEMM band with a small outlier budget)
                assert_close_bf16_chain(g[o:o + n], ref[key][o:o + n], f"{key}[{name}] mb {i}")


def _blocks_close(close, got, ref, cfg, net, what, **kw):
    for name, (o, shp) in orc.hparam_layout(cfg, net).items():
        if name == "_total":
            continue
        n = int(np.prod(shp))
        close(got[o:o + n], ref[o:o + n], f"{what}[{name}]", **kw)


@pytest.mark.parametrize("cfg", [CONFIGS[4], CONFIGS[5]], ids=lambda c: c.name)
def test_update_step_full_size_chain(cfg, torch, binding):
    """The bench configuration end to end, in the launch shapes the bench times.  The oracle cannot follow all
    P preferences of the 4 x 512 networks in seconds, so the chain is checked link by link, every link against the
    oracle on the GPU's own inputs to that link: rollout and GAE on a sample of preferences (preferences do not
    interact there, so their rows are complete outputs); then, in the first minibatch, the update forward on the
    same sample, the loss on every cell, the grouped backward on the sample (fed the GPU's dmu / dv), and the
    hypernet backward on the GPU's whole dtheta.  Size-independent properties are checked on all minibatches."""
    from paper_2603_09237_amd.step import UpdateStep
    say(f"update_step full size {cfg.name}")
    st = UpdateStep(cfg)
    d = inputs.make_all(cfg)
    st.load_inputs(d)
    grads, first = [], {}

    def grab(e, b):
        torch.cuda.synchronize()
        grads.append((to_np(st.dhp[ACTOR]).copy(), to_np(st.dhp[CRITIC]).copy(), to_np(st.stats).copy()))
        if e == 0 and b == 0:
            first.update(mu=to_np(st.mu).copy(), v=to_np(st.v).copy(), dmu=to_np(st.dmu).copy(), dv=to_np(st.dv).copy(),
                         dls=to_np(st.dlogsig).copy(), tv_a=to_np(st.theta_vec[ACTOR]).copy(),
                         dtm={n: st.dtheta_mat[n].clone() for n in (ACTOR, CRITIC)},
                         dtv={n: to_np(st.dtheta_vec[n]).copy() for n in (ACTOR, CRITIC)})

    st.run(on_minibatch=grab)
    torch.cuda.synchronize()
    prefs = sorted({0, cfg.P // 2 + 1, cfg.P - 1})
    emask = pref_env_mask(cfg, prefs)
    w = d["w"]
    T = cfg.T
    # ---- rollout and GAE on the sample
    tm_a, tv_a = orc.hypernet_fwd(cfg, ACTOR, d["hparams_actor_old"], w)
    tm_c, tv_c = orc.hypernet_fwd(cfg, CRITIC, d["hparams_critic_old"], w)
    tm_a, tm_c = orc.round_bf16(tm_a), orc.round_bf16(tm_c)
    mu, act, logp = orc.policy_fwd(cfg, ACTOR, tm_a, tv_a, d["obs"][:T], (0, T, 0, cfg.n_g), eps=d["eps"],
                                   emulate_bf16=True, prefs=prefs)
    v, _, _ = orc.policy_fwd(cfg, CRITIC, tm_c, tv_c, d["obs"], (0, T + 1, 0, cfg.n_g), emulate_bf16=True, prefs=prefs)
    _, vtarg, adv_s = orc.vec_gae(d["rewards"], v, d["dones"], w, cfg.gamma, cfg.lam)
    m2 = np.broadcast_to(emask[None, :], (T, cfg.N))
    m3a = np.broadcast_to(emask[None, :, None], mu.shape)
    m3k = np.broadcast_to(emask[None, :, None], vtarg.shape)
    g_act, g_logp, g_vtarg, g_adv = to_np(st.act), to_np(st.logp_old), to_np(st.vtarg), to_np(st.adv_s)
    assert_close_bf16(to_np(st.mu_old), mu, "mu_old", mask=m3a)
    assert_close_bf16(g_act, act, "act", mask=m3a)
    assert_close32(g_logp, logp, "logp_old", mask=m2)
    assert_close_bf16(to_np(st.v_roll)[:T], v[:T], "v_roll", mask=m3k)
    assert_close_bf16(g_vtarg, vtarg, "vtarg", mask=m3k)
    assert_close_bf16(g_adv, adv_s, "adv_s", mask=m2)
    # the scan itself on every environment, from the GPU's own critic values
    _, vt_all, as_all = orc.vec_gae(d["rewards"], to_np(st.v_roll), d["dones"], w, cfg.gamma, cfg.lam)
    for k in range(cfg.K):
        sk = max(1.0, float(np.sqrt(np.mean((vt_all[..., k] - to_np(st.v_roll)[:T, :, k]) ** 2))))
        assert_close32(g_vtarg[..., k], vt_all[..., k], f"vtarg[{k}] from the device's values", abs_=1e-5 * sk)
    assert_close32(g_adv, as_all, "adv_s from the device's values", abs_=1e-5 * max(1.0, float(np.sqrt(np.mean(as_all ** 2)))))
    # ---- first minibatch, link by link
    rows = st.mb_rows[0]
    rmask = orc.row_mask(cfg, rows, T)
    tm_a, tv_a = orc.hypernet_fwd(cfg, ACTOR, d["hparams_actor"], w)
    tm_c, tv_c = orc.hypernet_fwd(cfg, CRITIC, d["hparams_critic"], w)
    tm_a, tm_c = orc.round_bf16(tm_a), orc.round_bf16(tm_c)
    assert_close32(first["tv_a"], tv_a, "theta_vec actor (update-time parameters)")
    o_mu, _, _ = orc.policy_fwd(cfg, ACTOR, tm_a, tv_a, d["obs"][:T], rows, emulate_bf16=True, prefs=prefs)
    o_v, _, _ = orc.policy_fwd(cfg, CRITIC, tm_c, tv_c, d["obs"][:T], rows, emulate_bf16=True, prefs=prefs)
    sm = rmask & m2
    assert_close_bf16(first["mu"], o_mu, "mu (update forward)", mask=sm[..., None] & np.ones_like(o_mu, bool))
    assert_close_bf16(first["v"], o_v, "v (update forward)", mask=sm[..., None] & np.ones_like(o_v, bool))
    # the loss on every cell of the minibatch, from the device's own inputs
    logsig = first["tv_a"][:, -cfg.act_dim:]
    o_dmu, o_dls, o_dv, o_st = orc.ppo_loss_grad(cfg, rows, first["mu"], logsig, g_act, g_logp, g_adv, first["v"], g_vtarg,
                                                 cfg.clip_eps, True)
    B = float(rmask.sum())
    gi = orc.env_pref_index(cfg.N, cfg.P)
    lp = orc.gaussian_logp(g_act.astype(np.float64), first["mu"].astype(np.float64), logsig[gi][None].astype(np.float64))
    rho = np.exp(lp - g_logp)
    kink = (np.abs(rho - (1 + cfg.clip_eps)) < 1e-5) | (np.abs(rho - (1 - cfg.clip_eps)) < 1e-5)
    assert_close32(first["dmu"] * B, o_dmu * B, "dmu*B", mask=(rmask & ~kink)[..., None] & np.ones_like(o_dmu, bool))
    assert_close32(first["dv"] * B, o_dv * B, "dv*B", mask=rmask[..., None] & np.ones_like(o_dv, bool))
    stt = grads[0][2]
    assert_close32(stt[[0, 1, 3, 4, 5, 6]], o_st[[0, 1, 3, 4, 5, 6]], "stats", rel=1e-4, abs_=1e-5)
    assert abs(stt[2] - o_st[2]) <= (2.0 + kink[rmask].sum()) / B and stt[7] == B
    assert 0.02 < o_st[2] < 0.6                      # the clipped branch is exercised end to end
    if not kink[rmask].any():
        assert_close32(first["dls"], o_dls, "dlogsig", rel=1e-4, abs_=1e-5)
    # the grouped backward on the sample, fed the device's loss gradients
    for net, tm, tv, dout, dls in ((ACTOR, tm_a, tv_a, first["dmu"], first["dls"]), (CRITIC, tm_c, tv_c, first["dv"], None)):
        o_dtm, o_dtv = orc.policy_bwd(cfg, net, tm, tv, d["obs"][:T], rows, dout, dls, emulate_bf16=True, prefs=prefs)
        g_dtm = to_np(first["dtm"][net][prefs])
        g_dtv = first["dtv"][net]
        moff = voff = 0
        for l, (do, di) in enumerate(orc.layer_shapes(cfg, net)):
            assert_close_bf16(g_dtm[:, moff:moff + do * di], o_dtm[prefs, moff:moff + do * di], f"dW_{l} net={net}")
            assert_close_bf16(g_dtv[prefs, voff:voff + do], o_dtv[prefs, voff:voff + do], f"db_{l} net={net}")
            moff += do * di
            voff += do
        if net == ACTOR:
            assert np.array_equal(g_dtv[:, voff:], first["dls"])
    # the hypernet backward on the device's whole dtheta (fp32 arithmetic on both sides)
    for net, key in ((ACTOR, "hparams_actor"), (CRITIC, "hparams_critic")):
        ref = orc.hypernet_bwd(cfg, net, d[key], w, to_np(first["dtm"][net]), first["dtv"][net])
        _blocks_close(assert_close32, grads[0][net], ref, cfg, net, f"dhparams net={net}")
    first.clear()
    # ---- every minibatch
    assert len(grads) == cfg.minibatches * cfg.epochs
    for ga, gc, stt in grads:
        assert np.isfinite(ga).all() and np.isfinite(gc).all() and np.isfinite(stt).all()
        assert stt[7] == T * cfg.N // cfg.minibatches
        assert 0.02 < stt[2] < 0.6 and abs(stt[4]) < 10 * stt[5]
    # no optimiser step is taken, so epoch 2 repeats epoch 1 bit for bit (fixed-order reductions)
    MB = cfg.minibatches
    for b in range(MB):
        for e in range(1, cfg.epochs):
            assert np.array_equal(grads[b][0], grads[e * MB + b][0])
            assert np.array_equal(grads[b][1], grads[e * MB + b][1])


@pytest.mark.parametrize("cfg", [scaled(CONFIGS[4], name="cfg4-per-preference-shapes-P3", P=3, N=3 * CONFIGS[4].n_g),
                                 scaled(CONFIGS[5], name="cfg5-per-preference-shapes-P3", P=3, N=3 * CONFIGS[5].n_g)],
                         ids=lambda c: c.name)
def test_update_step_wide_networks_reduced_preferences(cfg, torch, binding):
    """The two widest workloads with their full per-preference shapes (all T steps, all n_g environments of a
    preference, every minibatch and epoch, the 4 x 512 bf16 networks) and three preferences instead of 64 / 128:
    the whole chain -- rollout, GAE, and per minibatch forward, loss, grouped backward, hypernet backward -- against
    the oracle as one chain, every rollout tensor and every block of both hypernet gradients."""
    say(f"update_step wide networks, reduced P {cfg.name}")
    st, d, grads = run_step(cfg, torch)
    res = orc.update_step(cfg, d["w"], d["hparams_actor_old"], d["hparams_critic_old"], d["hparams_actor"],
                          d["hparams_critic"], d["obs"], d["rewards"], d["dones"], d["eps"], cfg.gamma, cfg.lam,
                          cfg.clip_eps, cfg.minibatches, cfg.epochs, emulate_bf16=True, keep=True)
    assert_close_bf16(to_np(st.mu_old), res["mu_old"], "mu_old")
    assert_close_bf16(to_np(st.act), res["act"], "act")
    assert_close32(to_np(st.logp_old), res["logp_old"], "logp_old")
    assert_close_bf16(to_np(st.v_roll), res["v_roll"], "v_roll")
    assert_close_bf16(to_np(st.vtarg), res["vtarg"], "vtarg")
    assert_close_bf16(to_np(st.adv_s), res["adv_s"], "adv_s")
    assert len(grads) == cfg.minibatches * cfg.epochs
    for i, (ga, gc, stt) in enumerate(grads):
        ref = res["grads"][i]
        assert_close_bf16(stt[:2], ref["stats"][:2], "losses")
        assert 0.02 < ref["stats"][2] < 0.6 and abs(stt[2] - ref["stats"][2]) < 5e-3
        for net, g, key in ((ACTOR, ga, "dhp_actor"), (CRITIC, gc, "dhp_critic")):
            _blocks_close(assert_close_bf16_chain, g, ref[key], cfg, net, f"{key} mb {i}")
            rep = [bf16_chain_report(g[o:o + int(np.prod(shp))], ref[key][o:o + int(np.prod(shp))]) + (name,)
                   for name, (o, shp) in orc.hparam_layout(cfg, net).items() if name != "_total"]
            say(f"  mb {i} {key}: worst block by outliers {max(rep, key=lambda r: r[0])}, by RMS {max(rep, key=lambda r: r[2])}")


@pytest.mark.parametrize("cfg", [CONFIGS[1], scaled(RAGGED_FUSED, name="ragged-fused-graph", minibatches=1, epochs=2)],
                         ids=lambda c: c.name)
def test_update_step_graph_replays_equal_eager(cfg, torch, binding):
    """The step recorded into a HIP graph: every replay -- with eager work of the same library and synchronisations
    in between, and with new inputs in the same buffers -- gives the eager step's results bit for bit."""
    from paper_2603_09237_amd.step import UpdateStep
    say(f"update_step graph {cfg.name}")
    st = UpdateStep(cfg, keep_adv_vec=True)
    d = inputs.make_all(cfg)
    st.load_inputs(d)

    def snapshot():
        torch.cuda.synchronize()
        return [to_np(t).copy() for t in (st.dhp[ACTOR], st.dhp[CRITIC], st.stats, st.adv_s, st.vtarg, st.act, st.logp_old)]

    st.run()
    eager = snapshot()
    st.capture()
    other = scaled(cfg, name="other-seed", seed=7)
    d2 = inputs.make_all(other)
    ctx2 = binding.Context.from_config(cfg)
    for it in range(4):
        for t in (st.dhp[ACTOR], st.dhp[CRITIC], st.stats, st.adv_s, st.vtarg):
            t.fill_(float("nan"))                       # a replay has to write everything again
        if it == 2:                                     # new inputs in the same buffers: the graph follows the data
            st.load_inputs(d2)
            st.run()
            eager = snapshot()
            for t in (st.dhp[ACTOR], st.dhp[CRITIC], st.stats):
                t.fill_(float("nan"))
        st.replay()
        got = snapshot()
        for g, e in zip(got, eager):
            assert np.array_equal(g, e), it
        # eager work of the library between the replays
        out = torch.empty(cfg.N, dtype=torch.int32, device="cuda")
        ctx2.env_pref_index(out)
        torch.cuda.synchronize()
    assert np.isfinite(eager[0]).all() and np.abs(eager[0]).max() > 0


STRESS = scaled(CONFIGS[5], name="cfg5-stress-T256-N65536", T=256, N=65536, obs_dim=16)


def test_vec_gae_stress_shape_sampled(torch, binding):
    """The shape bench.py --stress times (T = 256, N = 65536: eight groups of chunks per workgroup).  Environments do
    not interact in the scan, so the oracle follows a sample of them (whole blocks of 32 and scattered single ones)
    column by column; all-done and no-done rows are planted to hit both branches at every chunk boundary."""
    cfg = STRESS
    say(f"vec_gae {cfg.name}")
    rng = np.random.default_rng(123)
    T, N, K = cfg.T, cfg.N, cfg.K
    r = rng.standard_normal((T, N, K), dtype=np.float32)
    v = rng.standard_normal((T + 1, N, K), dtype=np.float32)
    done = (rng.random((T, N)) < cfg.p_done).astype(np.uint8)
    done[:, 5] = 1
    done[:, 6] = 0
    done[7::8, 9] = 1                                   # an episode end at the last step of every chunk
    done[0::8, 10] = 1                                  # ... and at the first
    w = inputs.make_preferences(cfg)
    _, vtarg, adv_s = run_gae(cfg, torch, binding, r, v, done, w, want_vec=False)
    idx = np.unique(np.concatenate([np.arange(0, 64), np.arange(N - 32, N), rng.integers(0, N, size=400),
                                    np.arange(31 * cfg.n_g - 16, 31 * cfg.n_g + 48)]))
    g = orc.env_pref_index(N, cfg.P)[idx]
    # the oracle on the sampled columns: every sampled environment becomes a group of its own with its trade-off
    ws = np.repeat(w[g], 2, axis=0)                      # (the oracle wants P > 1 and P | N: two copies of each)
    rs, vs, ds = (np.repeat(a[:, idx], 2, axis=1) for a in (r, v, done))
    o_adv, o_vt, o_as = orc.vec_gae(rs, vs, ds, ws, cfg.gamma, cfg.lam)
    o_vt, o_as, o_adv = o_vt[:, ::2], o_as[:, ::2], o_adv[:, ::2]
    for k in range(K):
        sk = max(1.0, float(np.sqrt(np.mean(o_adv[..., k] ** 2))))
        assert_close32(vtarg[:, idx, k], o_vt[..., k], f"vtarg[{k}]", abs_=1e-5 * sk)
    assert_close32(adv_s[:, idx], o_as, "adv_s", abs_=1e-5 * max(1.0, float(np.sqrt(np.mean(o_as ** 2)))))
    assert np.array_equal(vtarg[:, 5], (r[:, 5] - v[:T, 5]) + v[:T, 5])    # all done: A = r - V, Vhat = A + V, in fp32
    assert np.isfinite(vtarg).all() and np.isfinite(adv_s).all()


def test_ppo_loss_grad_stress_shape_sampled(torch, binding):
    """The loss call at the stress shape on one of four minibatches (blocks take several groups of cells in sequence
    there): the statistics against float64 sums over every selected cell, the gradients against the oracle on a
    sample of preferences (cells interact only through the advantage statistics, which are handed to the oracle's
    formula through the normalised advantage)."""
    cfg = STRESS
    say(f"ppo_loss_grad {cfg.name}")
    T, N, A, K, P = cfg.T, cfg.N, cfg.act_dim, cfg.K, cfg.P
    mu, logsig, act, logp_old, adv_s, v, vtarg = loss_inputs(cfg, seed=41)
    rows = (0, T, cfg.n_g // 4, cfg.n_g // 4)
    ctx = binding.Context.from_config(cfg)
    SENT = 3.25
    dmu = torch.full(mu.shape, SENT, device="cuda")
    dv = torch.full(v.shape, SENT, device="cuda")
    dls = torch.full(logsig.shape, SENT, device="cuda")
    stats = torch.zeros(8, device="cuda")
    ws = torch.empty(ctx.workspace_bytes(rows), dtype=torch.uint8, device="cuda")
    ctx.ppo_loss_grad(rows, dev(mu), dev(logsig), A, dev(act), dev(logp_old), dev(adv_s), dev(v), dev(vtarg),
                      cfg.clip_eps, 1, dmu, dls, dv, stats, ws)
    torch.cuda.synchronize()
    mask = orc.row_mask(cfg, rows, T)
    B = float(mask.sum())
    sel = adv_s.astype(np.float64)[mask]
    mean, std = sel.mean(), np.sqrt(((sel - sel.mean()) ** 2).mean())
    st = to_np(stats)
    assert st[7] == B
    assert_close32(st[4:6], np.array([mean, std]), "advantage statistics")
    # the oracle on three preferences: a reduced problem with the same per-cell arithmetic, fed the normalised advantage
    prefs = [0, P // 2 + 3, P - 1]
    n_g = cfg.n_g
    cols = np.concatenate([np.arange(p * n_g, (p + 1) * n_g) for p in prefs])
    small = scaled(cfg, name="stress-sample", P=len(prefs), N=len(cols))
    ahat = ((adv_s.astype(np.float64) - mean) / (std + 1e-8))
    o_dmu, o_dls, o_dv, o_st = orc.ppo_loss_grad(small, rows, mu[:, cols], logsig[prefs], act[:, cols], logp_old[:, cols],
                                                 ahat[:, cols], v[:, cols], vtarg[:, cols], cfg.clip_eps, False)
    Bs = float(orc.row_mask(small, rows, T).sum())
    g_dmu, g_dv = to_np(dmu), to_np(dv)
    assert np.all(g_dmu[~mask] == SENT) and np.all(g_dv[~mask] == SENT)
    m_s = mask[:, cols]
    lp = orc.gaussian_logp(act[:, cols].astype(np.float64), mu[:, cols].astype(np.float64),
                           np.repeat(logsig[prefs], n_g, axis=0)[None].astype(np.float64))
    rho = np.exp(lp - logp_old[:, cols])
    kink = (np.abs(rho - (1 + cfg.clip_eps)) < 1e-5) | (np.abs(rho - (1 - cfg.clip_eps)) < 1e-5) | (np.abs(ahat[:, cols]) < 1e-6)
    # the oracle's gradients carry 1 / B of the reduced problem, the device's 1 / B of the whole selection
    assert_close32(g_dmu[:, cols] * B, o_dmu * Bs, "dmu*B", mask=(m_s & ~kink)[..., None] & np.ones_like(o_dmu, bool))
    assert_close32(g_dv[:, cols] * B, o_dv * Bs, "dv*B", mask=m_s[..., None] & np.ones_like(o_dv, bool))
    if not kink[m_s].any():
        assert_close32(to_np(dls)[prefs] * B, o_dls * Bs, "dlogsig*B", rel=1e-4, abs_=1e-5 * np.sqrt(Bs))
    # losses and clip fraction over every selected cell, in float64 from the same formulas
    gi = orc.env_pref_index(N, P)
    lp_all = orc.gaussian_logp(act.astype(np.float64), mu.astype(np.float64), logsig[gi][None].astype(np.float64))
    rho_all = np.exp(lp_all - logp_old)
    surr = np.minimum(rho_all * ahat, np.clip(rho_all, 1 - cfg.clip_eps, 1 + cfg.clip_eps) * ahat)
    L_pi = -surr[mask].mean()
    L_V = ((v.astype(np.float64) - vtarg) ** 2).sum(-1)[mask].mean()
    assert_close32(st[:2], np.array([L_pi, L_V]), "losses")
    assert abs(st[2] - (np.abs(rho_all - 1) > cfg.clip_eps)[mask].mean()) < 1e-4
    assert_close32(st[6:7], np.array([rho_all[mask].mean()]), "mean rho")
