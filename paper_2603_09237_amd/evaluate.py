"""Evaluation of a policy hypernetwork on the device (Fig. 2a): trade-offs -> actor family -> actions on the
roll-out's observations, and, once the roll-out is in, return vectors -> Pareto front -> hypervolume.

Argument marshalling only: every step runs in the library's kernels.  The environment itself is not part of this
package, so `actions` serves the caller's simulator and `score` takes the rewards and episode ends it produced.
"""
from __future__ import annotations

import torch

from . import binding
from .configs import Config, NET_ACTOR


class EvalSweep:
    def __init__(self, cfg: Config, device: str = "cuda"):
        self.cfg, self.dev = cfg, torch.device(device)
        self.ctx = binding.Context.from_config(cfg)
        P, K = cfg.P, cfg.K
        wdt = torch.bfloat16 if cfg.wdtype == 1 else torch.float32
        self.rows = (0, cfg.T + 1, 0, cfg.n_g)
        self.theta_mat = torch.empty(P, self.ctx.theta_mat_len(NET_ACTOR), dtype=wdt, device=self.dev)
        self.theta_vec = torch.empty(P, self.ctx.theta_vec_len(NET_ACTOR), device=self.dev)
        self.ws = torch.empty(self.ctx.workspace_bytes(self.rows), dtype=torch.uint8, device=self.dev)
        self.J = torch.empty(P, K, device=self.dev)
        self.front = torch.empty(P, dtype=torch.uint8, device=self.dev)
        self.hv = torch.empty(2, dtype=torch.float64, device=self.dev)
        self.ref = torch.zeros(16, device=self.dev)
        self.hv_ws = torch.empty(binding.hypervolume_workspace_bytes(P, K), dtype=torch.uint8, device=self.dev)

    def actions(self, hparams_actor, w, obs, out):
        """Mean actions of pi_p = H_pi(w_p) on every observation row: obs [T+1, N, O] -> out [T+1, N, A(, +A)]."""
        self.ctx.hypernet_fwd(NET_ACTOR, hparams_actor, w, self.theta_mat, self.theta_vec, self.ws)
        self.ctx.policy_fwd(NET_ACTOR, self.theta_mat, self.theta_vec, obs, self.rows, out, ws=self.ws)
        return out

    def score(self, rewards, dones, gamma, ref):
        """Return vectors J [P, K], front flags [P] and the hypervolume above ref [K] (device tensors; hv[0])."""
        self.ctx.eval_returns(rewards, dones, gamma, self.J)
        self.ref[: self.cfg.K] = ref
        binding.pareto_hypervolume(self.J, self.ref, self.cfg.P, self.cfg.K, self.front, self.hv, self.hv_ws)
        return self.J, self.front, self.hv
