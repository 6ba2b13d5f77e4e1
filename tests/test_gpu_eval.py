"""GPU parity of the evaluation entry points (returns, Pareto front, hypervolume) against oracle/eval_oracle.py.

Dominance flags: bit-exact.  Returns: fp32 results of fp64 sums, |gpu - ref| <= 1e-5 + 1e-4 |ref|.  Hypervolume:
both sides work in fp64 on the same fp32 inputs and differ only in the order of their sums of non-negative
terms: relative 1e-10.  Where the oracle's grid (n^K cells) is out of reach, properties that hold at any size.
"""
import sys

import numpy as np
import pytest

from oracle import eval_oracle as ev
from paper_2603_09237_amd import inputs
from paper_2603_09237_amd.configs import CONFIGS, scaled

from gpu_util import assert_close32, dev

pytestmark = pytest.mark.gpu
HV_REL = 1e-10


def say(msg):
    print(f"[gpu-eval] {msg}", flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def torch():
    import torch as t
    assert t.cuda.is_available(), "GPU tests need a GPU"
    return t


@pytest.fixture(scope="module")
def binding():
    from paper_2603_09237_amd import binding as b
    b.load()
    return b


RAGGED = scaled(CONFIGS[1], name="ragged-K3-P3-N69-T7", K=3, P=3, N=69, T=7, obs_dim=11, act_dim=3, n_hidden=2,
                width=48, act=1, rank=3, hyper_width=20)
WIDE_GROUP = scaled(CONFIGS[1], name="wide-group-K5-P2-N1400-T9", K=5, P=2, N=1400, T=9)   # 700 envs per group: several per thread


@pytest.mark.parametrize("cfg", [CONFIGS[1], CONFIGS[2], CONFIGS[3], CONFIGS[4], CONFIGS[5], RAGGED, WIDE_GROUP],
                         ids=lambda c: c.name)
def test_eval_returns_matches_oracle(cfg, torch, binding):
    say(f"eval_returns {cfg.name}")
    ctx = binding.Context.from_config(cfg)
    traj = inputs.make_trajectory(cfg)
    r, done = traj["rewards"], traj["dones"].copy()
    done[0, 0] = 1                       # an episode that ends at the first step
    done[:, cfg.N - 1] = 0               # and one that never ends
    for gamma in (cfg.gamma, 1.0):
        ref = ev.discounted_returns(r, done, float(np.float32(gamma)), cfg.P)
        J = torch.full((cfg.P, cfg.K), -7.0, device="cuda")
        ctx.eval_returns(dev(r), dev(done), gamma, J)
        torch.cuda.synchronize()
        assert_close32(J.cpu().numpy(), ref, f"J gamma={gamma}")


def run_hv(torch, binding, J, ref):
    J = np.ascontiguousarray(J, dtype=np.float32)
    ref = np.ascontiguousarray(ref, dtype=np.float32)
    n, K = J.shape
    nb = binding.hypervolume_workspace_bytes(n, K)
    assert nb > 0
    ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
    front = torch.full((n + 16,), 9, dtype=torch.uint8, device="cuda")
    hv = torch.full((2,), -1.0, dtype=torch.float64, device="cuda")
    d_ref = torch.zeros(16, device="cuda")
    d_ref[:K] = torch.from_numpy(ref).cuda()
    binding.pareto_hypervolume(dev(J), d_ref, n, K, front, hv, ws)
    torch.cuda.synchronize()
    f = front.cpu().numpy()
    assert np.all(f[n:] == 9), "front written past its end"
    h = hv.cpu().numpy()
    assert h[1] == -1.0
    return f[:n].astype(bool), float(h[0])


def point_set(seed, n, K, kind):
    rng = np.random.default_rng([seed, n, K])
    if kind == "front":          # a concave trade-off surface with noise: most points non-dominated
        w = rng.dirichlet(np.ones(K), size=n)
        J = np.sqrt(w) * (8.0 + rng.random((n, 1))) + 1.0
    elif kind == "ties":         # few distinct values: equal coordinates, duplicates, dominated points
        J = rng.integers(0, 4, size=(n, K)).astype(np.float64)
    else:                        # Gaussian cloud, partly below the reference point
        J = rng.standard_normal((n, K)) + 0.5
    return J.astype(np.float32)


ORACLE_CASES = [(1, 1, "cloud"), (37, 1, "cloud"), (1, 2, "front"), (2, 2, "cloud"), (130, 2, "front"), (1024, 2, "cloud"),
                (257, 2, "ties"), (64, 3, "front"), (130, 3, "cloud"), (100, 3, "ties"), (200, 3, "front"), (40, 4, "front"),
                (45, 4, "ties"), (20, 5, "cloud"), (9, 6, "front"), (7, 7, "front"), (6, 8, "front")]


@pytest.mark.parametrize("n,K,kind", ORACLE_CASES)
def test_pareto_hypervolume_matches_oracle(n, K, kind, torch, binding):
    say(f"pareto_hypervolume n={n} K={K} {kind}")
    J = point_set(3, n, K, kind)
    ref = np.full(K, 0.25 if kind != "ties" else -0.5, dtype=np.float32)
    front, hv = run_hv(torch, binding, J, ref)
    assert np.array_equal(front, ev.pareto_mask(J))
    want = ev.hypervolume(J, ref)
    assert hv == pytest.approx(want, rel=HV_REL, abs=1e-300), (hv, want)


def test_hypervolume_degenerate_sets(torch, binding):
    say("pareto_hypervolume degenerate sets")
    K = 3
    below = np.full((5, K), -1.0, dtype=np.float32)
    assert run_hv(torch, binding, below, np.zeros(K))[1] == 0.0            # nothing above the reference point
    one_dim_short = np.array([[2.0, 3.0, 0.0], [1.0, 1.0, -4.0]], dtype=np.float32)
    assert run_hv(torch, binding, one_dim_short, np.zeros(K))[1] == 0.0    # every box is flat in objective 2
    same = np.tile(np.array([[2.0, 3.0, 4.0]], dtype=np.float32), (6, 1))
    front, hv = run_hv(torch, binding, same, np.zeros(K))
    assert front.all() and hv == pytest.approx(24.0, rel=1e-15)           # duplicates: all on the front, one box


@pytest.mark.parametrize("n,K", [(128, 6), (256, 6), (1024, 4), (200, 5)])
def test_hypervolume_properties_at_sizes_beyond_the_oracle(n, K, torch, binding):
    """Workload-sized sets (P = 128 trade-offs, K = 6 objectives and larger): the oracle's grid has n^K cells, so
    the result is checked through properties of the measure, with the oracle on a subset it can handle."""
    say(f"pareto_hypervolume properties n={n} K={K}")
    J = point_set(11, n, K, "front")
    ref = np.full(K, 0.5, dtype=np.float32)
    front, hv = run_hv(torch, binding, J, ref)
    V = np.maximum(J.astype(np.float64) - ref, 0.0)
    boxes = np.prod(V, axis=1)
    assert boxes.max() <= hv * (1 + 1e-12) and hv <= boxes.sum() * (1 + 1e-12)      # between the largest box and the sum of boxes
    assert hv <= np.prod(V.max(axis=0)) * (1 + 1e-12)                              # inside the bounding box
    rng = np.random.default_rng(5)
    perm = rng.permutation(n)
    front_p, hv_p = run_hv(torch, binding, J[perm], ref)
    assert np.array_equal(front_p, front[perm]) and hv_p == pytest.approx(hv, rel=HV_REL)      # order of the points
    cols = rng.permutation(K)
    assert run_hv(torch, binding, J[:, cols], ref[cols])[1] == pytest.approx(hv, rel=HV_REL)    # order of the objectives
    _, hv_front = run_hv(torch, binding, J[front], ref)
    assert hv_front == pytest.approx(hv, rel=HV_REL)                                           # only the front counts
    s = np.array([2.0, 0.5, 4.0, 1.0, 0.25, 8.0, 2.0, 0.5], dtype=np.float32)[:K]             # powers of two: exact in fp32
    assert run_hv(torch, binding, J * s, ref * s)[1] == pytest.approx(hv * float(np.prod(s.astype(np.float64))), rel=HV_REL)
    m = 10 if K >= 5 else 24
    sub = J[:m]
    assert run_hv(torch, binding, sub, ref)[1] == pytest.approx(ev.hypervolume(sub, ref), rel=HV_REL)
    assert run_hv(torch, binding, sub, ref)[1] <= hv * (1 + 1e-12)                              # a subset dominates less
    # inclusion-exclusion of one point against the rest: HV(S) = HV(S without a) + vol(a) - HV({min(a, s) : s in S without a})
    a, rest = J[0], J[1:]
    clipped = np.minimum(rest, a[None, :])
    lhs = hv
    rhs = (run_hv(torch, binding, rest, ref)[1] + float(np.prod(np.maximum(a.astype(np.float64) - ref, 0.0)))
           - run_hv(torch, binding, clipped, ref)[1])
    assert lhs == pytest.approx(rhs, rel=1e-9)


@pytest.mark.parametrize("cfg", [CONFIGS[2], CONFIGS[3]], ids=lambda c: c.name)
def test_eval_sweep_matches_oracle(cfg, torch, binding):
    """The whole evaluation of a trade-off grid: actor family on the observations, returns, front, hypervolume."""
    from oracle import morlax_oracle as orc
    from paper_2603_09237_amd.evaluate import EvalSweep
    from gpu_util import assert_close_bf16
    say(f"eval sweep {cfg.name}")
    d = inputs.make_all(cfg)
    sweep = EvalSweep(cfg)
    out = torch.full((cfg.T + 1, cfg.N, cfg.act_dim), -7.0, device="cuda")
    sweep.actions(dev(d["hparams_actor"]), dev(d["w"]), dev(d["obs"]), out)
    tm, tv = orc.hypernet_fwd(cfg, 0, d["hparams_actor"], d["w"])
    bf16 = cfg.wdtype == 1
    tm = orc.round_bf16(tm) if bf16 else tm.astype(np.float32).astype(np.float64)
    prefs = [0, cfg.P // 2, cfg.P - 1]
    want = orc.policy_fwd(cfg, 0, tm, tv, d["obs"], (0, cfg.T + 1, 0, cfg.n_g), emulate_bf16=bf16, prefs=prefs)[0]
    emask = np.zeros(cfg.N, dtype=bool)
    for p in prefs:
        emask[p * cfg.n_g:(p + 1) * cfg.n_g] = True
    mask = np.broadcast_to(emask[None, :, None], want.shape)
    (assert_close_bf16 if bf16 else assert_close32)(out.cpu().numpy(), want, "mean actions", mask=mask)
    J_ref = ev.discounted_returns(d["rewards"], d["dones"], float(np.float32(cfg.gamma)), cfg.P)
    ref = (J_ref.min(axis=0) - 1.0).astype(np.float32)
    J, front, hv = sweep.score(dev(d["rewards"]), dev(d["dones"]), cfg.gamma, torch.from_numpy(ref).cuda())
    torch.cuda.synchronize()
    Jg = J.cpu().numpy()
    assert_close32(Jg, J_ref, "J")
    # front and hypervolume of the device's own fp32 return vectors (the decision is taken on the same numbers)
    assert np.array_equal(front.cpu().numpy().astype(bool), ev.pareto_mask(Jg))
    assert float(hv[0].item()) == pytest.approx(ev.hypervolume(Jg, ref), rel=HV_REL)
