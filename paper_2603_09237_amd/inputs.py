"""Seeded synthetic inputs for one MORLAX update step.

Stand-ins for the trajectories the paper collects from its MO-Playground
environments (Sec. III-D; Sec. III-C rollout phase): observations, vector
rewards, done flags and Gaussian action noise arrive as random tensors with the
shapes of `configs.CONFIGS`.  Physics is not simulated.

The module only draws random numbers and lays them out; it holds none of the
method's arithmetic.  The same host arrays are handed, byte for byte, to the
HIP path and to the CPU oracle.  Each tensor has its own stream
`numpy.random.default_rng([seed, tensor_id])`, so a tensor does not change when
another one is added or resized.
"""
from __future__ import annotations

import numpy as np

from .configs import Config, NET_ACTOR, NET_CRITIC

TID_W, TID_OBS, TID_REW, TID_DONE, TID_EPS, TID_HP_ACTOR, TID_HP_CRITIC = 0, 1, 2, 3, 4, 5, 6
TID_PERT_ACTOR, TID_PERT_CRITIC, TID_VALUES = 7, 8, 9


def _rng(seed: int, tid: int) -> np.random.Generator:
    return np.random.default_rng([int(seed), int(tid)])


def layer_shapes(cfg: Config, net: int):
    """(d_out, d_in) of every dense layer of a target network, input to output."""
    out = cfg.K
    if net == NET_ACTOR:    # means, and with a state-dependent standard deviation also the log sigmas
        out = 2 * cfg.act_dim if cfg.sigma_state else cfg.act_dim
    dims = [cfg.obs_dim] + [cfg.width] * cfg.n_hidden + [out]
    return [(dims[i + 1], dims[i]) for i in range(len(dims) - 1)]


def hparam_blocks(cfg: Config, net: int):
    """Flat order of a hypernetwork's parameter blocks: (name, shape, kind, scale).

    Order: trunk (Wh1, bh1, Wh2, bh2); per target layer (W0, b0, MA, cA, MB, cB,
    Mb) -- with rank < 0 (W0, b0, MW, Mb) --; for the actor finally (logsig0, Msig).  All blocks row-major.
    """
    K, F, r = cfg.K, cfg.hyper_width, cfg.rank
    blocks = [("Wh1", (F, K), "normal", K ** -0.5), ("bh1", (F,), "const", 0.0),
              ("Wh2", (F, F), "normal", F ** -0.5), ("bh2", (F,), "const", 0.0)]
    for l, (do, di) in enumerate(layer_shapes(cfg, net)):
        s = 0.3 * (max(r, 1) * di) ** -0.25
        blocks += [(f"W0_{l}", (do, di), "normal", di ** -0.5),
                   (f"b0_{l}", (do,), "const", 0.0)]
        if r < 0:   # strictly affine hypernetwork: a row of M per weight, sized so that |M f| ~ 0.13 |W0|
            blocks += [(f"MW_{l}", (do * di, F), "normal", 0.26 * di ** -0.5 * F ** -0.5)]
        else:
            blocks += [(f"MA_{l}", (do * r, F), "normal", s * F ** -0.5),
                       (f"cA_{l}", (do * r,), "normal", s),
                       (f"MB_{l}", (r * di, F), "normal", s * F ** -0.5),
                       (f"cB_{l}", (r * di,), "normal", s)]
        blocks += [(f"Mb_{l}", (do, F), "normal", 0.1 * F ** -0.5)]
    if net == NET_ACTOR and not cfg.sigma_state:
        blocks += [("logsig0", (cfg.act_dim,), "const", -0.5),
                   ("Msig", (cfg.act_dim, F), "normal", 0.1 * F ** -0.5)]
    return blocks


def hparam_count(cfg: Config, net: int) -> int:
    return sum(int(np.prod(shape)) for _, shape, _, _ in hparam_blocks(cfg, net))


def make_hparams(cfg: Config, net: int) -> np.ndarray:
    """Random initial hypernetwork parameters (Sec. III-C, initialisation)."""
    rng = _rng(cfg.seed, TID_HP_ACTOR if net == NET_ACTOR else TID_HP_CRITIC)
    parts = []
    for _, shape, kind, scale in hparam_blocks(cfg, net):
        n = int(np.prod(shape))
        if kind == "const":
            parts.append(np.full(n, scale, dtype=np.float32))
        else:
            parts.append((rng.standard_normal(n, dtype=np.float32) * np.float32(scale)))
    return np.concatenate(parts).astype(np.float32)


def perturb_hparams(cfg: Config, net: int, hparams: np.ndarray, rel: float = 0.05) -> np.ndarray:
    """Update-time parameters: every block moved by rel * RMS(block) * N(0,1).

    Makes the probability ratio differ from one so the clip branch is exercised: with rel = 0.05 between
    3 % and 10 % of the cells of every workload end up outside the clip range (0.02 leaves 0.1-0.5 %).
    """
    rng = _rng(cfg.seed, TID_PERT_ACTOR if net == NET_ACTOR else TID_PERT_CRITIC)
    out = hparams.astype(np.float32).copy()
    off = 0
    for _, shape, _, _ in hparam_blocks(cfg, net):
        n = int(np.prod(shape))
        blk = out[off:off + n]
        rms = float(np.sqrt(np.mean(blk.astype(np.float64) ** 2)))
        blk += np.float32(rel * rms) * rng.standard_normal(n, dtype=np.float32)
        off += n
    return out


def make_preferences(cfg: Config) -> np.ndarray:
    """P iid draws from a symmetric Dirichlet (Sec. III-C, sampling phase), [P, K] fp32."""
    rng = _rng(cfg.seed, TID_W)
    w = rng.dirichlet(np.full(cfg.K, cfg.dirichlet_alpha, dtype=np.float64), size=cfg.P)
    w = np.maximum(w, 0.0)
    w = w / w.sum(axis=1, keepdims=True)
    return w.astype(np.float32)


def reward_scales(cfg: Config) -> np.ndarray:
    if cfg.K == 3:
        return np.array([1.0, 0.1, 10.0], dtype=np.float32)
    if cfg.K == 1:
        return np.ones(1, dtype=np.float32)
    k = np.arange(cfg.K, dtype=np.float64)
    return (10.0 ** (2.0 * k / (cfg.K - 1) - 1.0)).astype(np.float32)


def make_rewards(cfg: Config) -> np.ndarray:
    """Vector rewards [T, N, K] fp32, one column per objective."""
    rng = _rng(cfg.seed, TID_REW)
    r = rng.standard_normal((cfg.T, cfg.N, cfg.K), dtype=np.float32)
    if cfg.K == 2 and cfg.obs_dim == 27:
        # quadruped-shaped: a forward-progress term and an energy-like penalty
        r[..., 0] = 1.0 + 0.5 * r[..., 0]
        r[..., 1] = -np.abs(r[..., 1])
    elif cfg.K == 2:
        pass
    else:
        r *= reward_scales(cfg)[None, None, :]
    return np.ascontiguousarray(r, dtype=np.float32)


def make_trajectory(cfg: Config) -> dict:
    """obs [T+1,N,O], rewards [T,N,K], dones [T,N] u8, eps [T,N,A], all host numpy."""
    obs = _rng(cfg.seed, TID_OBS).standard_normal((cfg.T + 1, cfg.N, cfg.obs_dim), dtype=np.float32)
    done = (_rng(cfg.seed, TID_DONE).random((cfg.T, cfg.N)) < cfg.p_done).astype(np.uint8)
    eps = _rng(cfg.seed, TID_EPS).standard_normal((cfg.T, cfg.N, cfg.act_dim), dtype=np.float32)
    return {"obs": obs, "rewards": make_rewards(cfg), "dones": done, "eps": eps}


def make_values(cfg: Config) -> np.ndarray:
    """Stand-alone critic values [T+1, N, K] for GAE unit tests."""
    return _rng(cfg.seed, TID_VALUES).standard_normal((cfg.T + 1, cfg.N, cfg.K), dtype=np.float32)


def make_all(cfg: Config) -> dict:
    """Every input of one update step."""
    d = make_trajectory(cfg)
    d["w"] = make_preferences(cfg)
    for net, key in ((NET_ACTOR, "actor"), (NET_CRITIC, "critic")):
        hp = make_hparams(cfg, net)
        d[f"hparams_{key}_old"] = hp
        d[f"hparams_{key}"] = perturb_hparams(cfg, net, hp)
    return d
