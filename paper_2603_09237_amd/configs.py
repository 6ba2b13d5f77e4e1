"""The five synthetic workloads this build is measured and checked on.

Each entry fixes the shapes of one MORLAX update step (Sec. III-C: sample,
rollout, update): K objectives, P trade-off vectors, N parallel environments
split into P contiguous groups of n_g = N / P, rollout horizon T, observation
and action widths, the target-network shape, the hypernetwork factor rank and
the PPO minibatch/epoch counts.  Symbols: the paper's `m` is `K` here and the
paper's `K` (number of distinct trade-offs) is `P`.

This module holds shapes and constants only; it contains none of the method's
arithmetic and is shared by the tests, the bench and the input generator.
"""
from __future__ import annotations

from dataclasses import dataclass, asdict

ACT_TANH = 0
ACT_SILU = 1
WDTYPE_F32 = 0
WDTYPE_BF16 = 1
NET_ACTOR = 0
NET_CRITIC = 1


@dataclass(frozen=True)
class Config:
    name: str
    K: int            # objectives (paper: m)
    P: int            # distinct trade-off vectors (paper: K)
    N: int            # parallel environments
    T: int            # rollout horizon
    obs_dim: int
    act_dim: int
    n_hidden: int     # hidden layers of the target nets
    width: int        # hidden width
    act: int          # ACT_TANH / ACT_SILU
    rank: int         # rank of the per-preference weight delta
    hyper_width: int  # F, feature width of the hypernet trunk
    wdtype: int       # WDTYPE_F32 / WDTYPE_BF16 (target-net weight + GEMM input type)
    mean_tanh: int    # 1: actor mean is tanh(z) (Sec. III-E)
    minibatches: int
    epochs: int
    dirichlet_alpha: float
    p_done: float
    gamma: float = 0.99
    lam: float = 0.95
    clip_eps: float = 0.2
    seed: int = 0
    sigma_state: int = 0   # 1: the actor network outputs its own log sigma (2A output columns)

    @property
    def n_g(self) -> int:
        return self.N // self.P

    def dims_dict(self) -> dict:
        keys = ("K", "P", "N", "T", "obs_dim", "act_dim", "n_hidden", "width", "act",
                "rank", "hyper_width", "wdtype", "mean_tanh", "sigma_state")
        d = asdict(self)
        return {k: d[k] for k in keys}


CONFIGS = {
    1: Config("cfg1-tiny-K2-P4-N64-T16-2x32-tanh-fp32", K=2, P=4, N=64, T=16, obs_dim=8, act_dim=2,
              n_hidden=2, width=32, act=ACT_TANH, rank=4, hyper_width=32, wdtype=WDTYPE_F32,
              mean_tanh=1, minibatches=1, epochs=1, dirichlet_alpha=1.0, p_done=0.02),
    2: Config("cfg2-quadruped-K2-P16-N4096-T32-3x256-silu-fp32", K=2, P=16, N=4096, T=32, obs_dim=27,
              act_dim=8, n_hidden=3, width=256, act=ACT_SILU, rank=8, hyper_width=32,
              wdtype=WDTYPE_F32, mean_tanh=1, minibatches=1, epochs=1, dirichlet_alpha=1.0,
              p_done=0.005),
    3: Config("cfg3-hopper-K3-P32-N8192-T32-3x256-silu-bf16", K=3, P=32, N=8192, T=32, obs_dim=11,
              act_dim=3, n_hidden=3, width=256, act=ACT_SILU, rank=8, hyper_width=32,
              wdtype=WDTYPE_BF16, mean_tanh=1, minibatches=1, epochs=1, dirichlet_alpha=1.0,
              p_done=0.01),
    4: Config("cfg4-humanoid-K6-P64-N8192-T32-4x512-silu-bf16", K=6, P=64, N=8192, T=32, obs_dim=64,
              act_dim=10, n_hidden=4, width=512, act=ACT_SILU, rank=16, hyper_width=32,
              wdtype=WDTYPE_BF16, mean_tanh=1, minibatches=1, epochs=1, dirichlet_alpha=0.5,
              p_done=0.005),
    5: Config("cfg5-largest-K6-P128-N16384-T64-4x512-silu-bf16-4mbx2ep", K=6, P=128, N=16384, T=64,
              obs_dim=64, act_dim=10, n_hidden=4, width=512, act=ACT_SILU, rank=16,
              hyper_width=32, wdtype=WDTYPE_BF16, mean_tanh=1, minibatches=4, epochs=2,
              dirichlet_alpha=0.5, p_done=0.005),
}


def scaled(cfg: Config, **over) -> Config:
    """A copy of `cfg` with some fields replaced (ragged / reduced test shapes)."""
    d = asdict(cfg)
    d.update(over)
    return Config(**d)
