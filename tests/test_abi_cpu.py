"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the header
declares, computes the layouts the oracle and the generator agree on, and rejects bad arguments
before any HIP call."""
import ctypes as C
import os
import re

import pytest

from oracle import morlax_oracle as orc
from paper_2603_09237_amd import binding, configs, inputs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2603_09237_amd import build
        build.build(verbose=False)
    return binding.load()


def test_every_declared_symbol_is_exported(lib):
    inc = os.path.join(ROOT, "include")
    hdr = "".join(open(os.path.join(inc, f)).read() for f in sorted(os.listdir(inc)) if f.endswith(".h"))
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = sorted(set(re.findall(r"\b(morlax_[a-z0-9_]+)\s*\(", hdr)))
    assert len(names) >= 15
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n


def test_layout_queries_match_oracle_and_generator(lib):
    affine = [configs.scaled(configs.CONFIGS[i], name=f"cfg{i}-affine", rank=-1) for i in (1, 5)]
    sigma = [configs.scaled(configs.CONFIGS[i], name=f"cfg{i}-sigma", sigma_state=1) for i in (1, 2)]
    for cfg in list(configs.CONFIGS.values()) + affine + sigma:
        ctx = binding.Context.from_config(cfg)
        for net in (0, 1):
            assert ctx.hparam_count(net) == orc.hparam_count(cfg, net) == inputs.hparam_count(cfg, net)
            assert ctx.theta_mat_len(net) == orc.theta_mat_len(cfg, net)
            assert ctx.theta_vec_len(net) == orc.theta_vec_len(cfg, net)
            assert ctx.saved_bytes(net, (0, cfg.T, 0, cfg.n_g // cfg.minibatches)) > 0
        assert ctx.workspace_bytes() >= ctx.workspace_bytes((0, 1, 0, 1)) > 0
        ctx.close()


def test_workspace_of_a_selection_covers_every_smaller_one(lib):
    """A caller sizes one buffer for the whole tensor and reuses it for time ranges and minibatches, so the
    size must not shrink when rows are added (the split and padded scratch regions depend on the row count)."""
    for i in (1, 2, 3, 4):
        cfg = configs.CONFIGS[i]
        ctx = binding.Context.from_config(cfg)
        whole = ctx.workspace_bytes()
        prev = 0
        for t_cnt in (1, 2, cfg.T // 2, cfg.T - 1, cfg.T, cfg.T + 1):
            for j_cnt in (1, max(cfg.n_g // 4, 1), max(cfg.n_g // 2, 1), cfg.n_g):
                b = ctx.workspace_bytes((0, t_cnt, 0, j_cnt))
                assert 0 < b <= whole, (cfg.name, t_cnt, j_cnt, b, whole)
            assert b >= prev, (cfg.name, t_cnt)  # full groups, growing time range
            prev = b
        ctx.close()


@pytest.mark.parametrize("over,code", [
    (dict(P=1), binding.ERR_SHAPE), (dict(P=3), binding.ERR_SHAPE), (dict(K=0), binding.ERR_SHAPE),
    (dict(T=0), binding.ERR_SHAPE), (dict(rank=-2), binding.ERR_SHAPE), (dict(K=17), binding.ERR_UNSUPPORTED),
    (dict(width=40), binding.ERR_UNSUPPORTED), (dict(act=2), binding.ERR_UNSUPPORTED),
    (dict(wdtype=3), binding.ERR_UNSUPPORTED), (dict(rank=64), binding.ERR_UNSUPPORTED),
    (dict(hyper_width=128), binding.ERR_UNSUPPORTED), (dict(n_hidden=9), binding.ERR_UNSUPPORTED),
    (dict(N=1 << 20, P=2, T=1023, obs_dim=1024), binding.ERR_UNSUPPORTED),      # observations beyond 32-bit offsets
    (dict(N=1 << 16, P=2, T=16383, width=2048), binding.ERR_UNSUPPORTED),       # one preference's activations too
    (dict(sigma_state=1, act_dim=9), binding.ERR_UNSUPPORTED),                  # 2A output columns must fit 16
    (dict(sigma_state=2), binding.ERR_UNSUPPORTED),
    (dict(P=65536, N=65536), binding.ERR_UNSUPPORTED),                          # the preference rides in gridDim.y / .z
])
def test_create_rejects_bad_dims(lib, over, code):
    d = configs.CONFIGS[1].dims_dict()
    d.update(over)
    with pytest.raises(binding.MorlaxError) as e:
        binding.Context(**d)
    assert e.value.code == code
    assert lib.morlax_last_error().decode() != ""


def test_ops_reject_bad_arguments_without_touching_the_gpu(lib):
    cfg = configs.CONFIGS[1]
    ctx = binding.Context.from_config(cfg)
    good = 0x10000  # aligned fake device address; never dereferenced because validation fails first
    with pytest.raises(binding.MorlaxError) as e:
        ctx.vec_gae(None, good, good, good, 0.99, 0.95, None, good, good, stream=0)
    assert e.value.code == binding.ERR_NULL
    with pytest.raises(binding.MorlaxError) as e:
        ctx.vec_gae(good + 4, good, good, good, 0.99, 0.95, None, good, good, stream=0)
    assert e.value.code == binding.ERR_SHAPE
    with pytest.raises(binding.MorlaxError) as e:
        ctx.vec_gae(good, good, good, good, 1.5, 0.95, None, good, good, stream=0)
    assert e.value.code == binding.ERR_SHAPE
    with pytest.raises(binding.MorlaxError) as e:
        ctx.hypernet_fwd(2, good, good, good, good, good, stream=0)
    assert e.value.code == binding.ERR_SHAPE
    with pytest.raises(binding.MorlaxError) as e:
        ctx.hypernet_bwd(0, good, good, None, good, good, good, stream=0)
    assert e.value.code == binding.ERR_NULL
    with pytest.raises(binding.MorlaxError) as e:
        ctx.hypernet_bwd_kept(0, good, good, good, good, good, None, stream=0)
    assert e.value.code == binding.ERR_NULL
    with pytest.raises(binding.MorlaxError) as e:
        ctx.hypernet_bwd_kept(3, good, good, good, good, good, good, stream=0)
    assert e.value.code == binding.ERR_SHAPE
    with pytest.raises(binding.MorlaxError) as e:      # actions, advantages and targets exist for t < T only
        ctx.ppo_loss_grad((0, cfg.T + 1, 0, cfg.n_g), good, good, 4, good, good, good, good, good, 0.2, 1, good, good,
                          good, good, good, stream=0)
    assert e.value.code == binding.ERR_SHAPE
    bad_rows = [(0, cfg.T + 2, 0, cfg.n_g), (0, 0, 0, 1), (0, 1, 0, cfg.n_g + 1), (-1, 1, 0, 1), (0, 1, cfg.n_g, 1)]
    for rows in bad_rows:
        with pytest.raises(binding.MorlaxError) as e:
            ctx.policy_fwd(0, good, good, good, rows, good, ws=good, stream=0)
        assert e.value.code == binding.ERR_SHAPE, rows
        with pytest.raises(binding.MorlaxError) as e:
            ctx.ppo_loss_grad(rows, good, good, 4, good, good, good, good, good, 0.2, 1, good, good, good, good,
                              good, stream=0)
        assert e.value.code == binding.ERR_SHAPE, rows
    with pytest.raises(binding.MorlaxError) as e:      # sampling outputs must come together
        ctx.policy_fwd(0, good, good, good, (0, 1, 0, 1), good, eps=good, ws=good, stream=0)
    assert e.value.code == binding.ERR_NULL
    with pytest.raises(binding.MorlaxError) as e:      # ... and only for the actor
        ctx.policy_fwd(1, good, good, good, (0, 1, 0, 1), good, eps=good, act=good, logp=good, ws=good, stream=0)
    assert e.value.code == binding.ERR_SHAPE
    with pytest.raises(binding.MorlaxError) as e:
        ctx.policy_bwd(1, good, good, good, (0, 1, 0, 1), good, good, good, good, good, good, stream=0)
    assert e.value.code == binding.ERR_SHAPE           # dlogsig is actor-only
    with pytest.raises(binding.MorlaxError) as e:
        ctx.ppo_loss_grad((0, 1, 0, 1), good, good, 1, good, good, good, good, good, 0.2, 1, good, good, good,
                          good, good, stream=0)
    assert e.value.code == binding.ERR_SHAPE           # logsig_stride < act_dim
    with pytest.raises(binding.MorlaxError) as e:      # the optimiser step counts from 1
        ctx.adam_step(0, good, good, good, good, 1e-3, 0.9, 0.999, 1e-8, 0, stream=0)
    assert e.value.code == binding.ERR_SHAPE
    with pytest.raises(binding.MorlaxError) as e:
        ctx.adam_step(0, good, good, good, good, 1e-3, 1.0, 0.999, 1e-8, 1, stream=0)
    assert e.value.code == binding.ERR_SHAPE
    with pytest.raises(binding.MorlaxError) as e:
        ctx.adam_step(1, good, good, None, good, 1e-3, 0.9, 0.999, 1e-8, 1, stream=0)
    assert e.value.code == binding.ERR_NULL
    with pytest.raises(binding.MorlaxError) as e:      # more extreme trade-offs than objectives
        ctx.sample_preferences(good, cfg.K + 1, good, stream=0)
    assert e.value.code == binding.ERR_SHAPE
    sctx = binding.Context.from_config(configs.scaled(cfg, name="sigma", sigma_state=1))
    with pytest.raises(binding.MorlaxError) as e:      # the log-sigma gradient is part of dout in this mode
        sctx.policy_bwd(0, good, good, good, (0, 1, 0, 1), good, good, good, good, good, good, stream=0)
    assert e.value.code == binding.ERR_SHAPE
    sctx.close()
    with pytest.raises(binding.MorlaxError) as e:      # the vector advantage has T rows, not T + 1
        ctx.scalarize_normalized((0, cfg.T + 1, 0, cfg.n_g), good, good, good, good, stream=0)
    assert e.value.code == binding.ERR_SHAPE
    with pytest.raises(binding.MorlaxError) as e:
        ctx.scalarize_normalized((0, 1, 0, 1), good, None, good, good, stream=0)
    assert e.value.code == binding.ERR_NULL
    with pytest.raises(binding.MorlaxError) as e:      # the truncation mask is not optional here
        ctx.vec_gae_trunc(good, good, good, None, good, 0.99, 0.95, None, good, good, stream=0)
    assert e.value.code == binding.ERR_NULL
    ctx.close()


def test_too_small_workspace_is_refused_before_any_launch(lib):
    """Every op that takes scratch checks its size on the host before anything is launched (the addresses here are
    fake: only a refused call is safe to make)."""
    cfg = configs.CONFIGS[1]
    ctx = binding.Context.from_config(cfg)
    good = 0x10000
    rows = (0, cfg.T, 0, cfg.n_g)
    calls = {
        "hypernet_fwd": lambda ws: ctx.hypernet_fwd(0, good, good, good, good, ws, stream=0),
        "hypernet_bwd": lambda ws: ctx.hypernet_bwd(0, good, good, good, good, good, ws, stream=0),
        "hypernet_bwd_kept": lambda ws: ctx.hypernet_bwd_kept(1, good, good, good, good, good, ws, stream=0),
        "policy_fwd": lambda ws: ctx.policy_fwd(0, good, good, good, rows, good, ws=ws, stream=0),
        "policy_bwd": lambda ws: ctx.policy_bwd(1, good, good, good, rows, good, good, None, good, good, ws, stream=0),
        "scalarize_normalized": lambda ws: ctx.scalarize_normalized(rows, good, good, good, ws, stream=0),
        "ppo_loss_grad": lambda ws: ctx.ppo_loss_grad(rows, good, good, 4, good, good, good, good, good, 0.2, 1, good,
                                                      good, good, good, ws, stream=0),
        "pareto_hypervolume": lambda ws: binding.pareto_hypervolume(good, good, 8, 3, good, good, ws, stream=0),
    }
    for name, call in calls.items():
        with pytest.raises(binding.MorlaxError) as e:
            call((good, 0))
        assert e.value.code == binding.ERR_WORKSPACE, name
        with pytest.raises(binding.MorlaxError) as e:
            call((good, 16))
        assert e.value.code == binding.ERR_WORKSPACE, name
        assert "needed" in str(e.value)
    hv_need = binding.hypervolume_workspace_bytes(8, 3)
    with pytest.raises(binding.MorlaxError) as e:
        binding.pareto_hypervolume(good, good, 8, 3, good, good, (good, hv_need - 1), stream=0)
    assert e.value.code == binding.ERR_WORKSPACE
    ctx.close()


def test_static_scratch_loss_refuses_what_does_not_fit(lib):
    # the per-block partial sums grow with the number of preferences: 16384 of them with 16 actions need 2.7 MB
    cfg = configs.scaled(configs.CONFIGS[1], name="too-many-preferences", P=16384, N=16384, act_dim=16)
    ctx = binding.Context.from_config(cfg)
    good = 0x10000
    with pytest.raises(binding.MorlaxError) as e:
        ctx.ppo_loss_grad_static((0, cfg.T, 0, cfg.n_g), good, good, cfg.act_dim, good, good, good, good, good, 0.2, 1,
                                 good, good, good, good, stream=0)
    assert e.value.code == binding.ERR_WORKSPACE and "static" in str(e.value)
    with pytest.raises(binding.MorlaxError) as e:      # the same argument checks as the workspace form
        ctx.ppo_loss_grad_static((0, cfg.T + 1, 0, 1), good, good, cfg.act_dim, good, good, good, good, good, 0.2, 1,
                                 good, good, good, good, stream=0)
    assert e.value.code == binding.ERR_SHAPE
    ctx.close()


def test_evaluation_entry_points_reject_bad_arguments(lib):
    cfg = configs.CONFIGS[1]
    ctx = binding.Context.from_config(cfg)
    good = 0x10000
    with pytest.raises(binding.MorlaxError) as e:
        ctx.eval_returns(good, None, 0.99, good, stream=0)
    assert e.value.code == binding.ERR_NULL
    for gamma in (0.0, 1.5, -0.1):
        with pytest.raises(binding.MorlaxError) as e:
            ctx.eval_returns(good, good, gamma, good, stream=0)
        assert e.value.code == binding.ERR_SHAPE
    # sizes the exact hypervolume serves: K <= 8, n <= 1024, n^(K-2) <= 2^32
    for n, K, ok in [(1, 1, True), (1024, 4, True), (256, 6, True), (257, 6, False), (1025, 2, False), (4, 9, False),
                     (0, 2, False), (40, 8, True), (41, 8, False)]:
        b = binding.hypervolume_workspace_bytes(n, K)
        assert (b > 0) == ok, (n, K, b)
        if not ok:
            with pytest.raises(binding.MorlaxError) as e:
                binding.pareto_hypervolume(good, good, n, K, good, good, good, stream=0)
            assert e.value.code == binding.ERR_SHAPE
    with pytest.raises(binding.MorlaxError) as e:
        binding.pareto_hypervolume(good, None, 4, 2, good, good, good, stream=0)
    assert e.value.code == binding.ERR_NULL


def test_bench_refuses_more_than_one_gpu():
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""
