"""Buffers and call sequence of one MORLAX update step on one GPU.

`UpdateStep` owns the device tensors (torch is used for memory and the stream only) and issues the
C-ABI calls in the order of the method (paper Sec. III-C): rollout forward of the actor and critic
families with the rollout-time hypernet parameters, vector GAE, then for every epoch and minibatch
hypernet forward, grouped forward, loss, grouped backward and hypernet backward for both nets.
No arithmetic happens here.
"""
from __future__ import annotations

import numpy as np

from . import binding
from .binding import ACTOR, CRITIC
from .configs import Config, WDTYPE_BF16


class UpdateStep:
    def __init__(self, cfg: Config, device: str = "cuda:0", keep_adv_vec: bool = False, two_streams: bool = False,
                 optimizer: dict | None = None, side_hypernet: bool = False, adv_norm: str = "scalar"):
        """optimizer = dict(lr_actor, lr_critic, beta1, beta2, eps): take one Adam step on either hypernet
        after every minibatch (a true PPO update); None: gradients only, parameters stay fixed.
        side_hypernet: the hypernet calls (backward, optimiser step, the next minibatch's forward) run on a second
        stream next to the grouped GEMMs of the other network / the next minibatch; the GEMM chain stays on the
        caller's stream.  two_streams: the older split, one stream per network family.
        adv_norm: "scalar" = the scalarised advantage is normalised over the minibatch (inside the loss call);
        "per_objective" = every objective is standardised over the minibatch before scalarisation
        (scalarize_normalized, then the loss without further normalisation)."""
        import torch
        self.torch = torch
        self.cfg = cfg
        self.dev = torch.device(device)
        self.ctx = binding.Context.from_config(cfg)
        c, ctx = cfg, self.ctx
        f32 = dict(dtype=torch.float32, device=self.dev)
        wdt = torch.bfloat16 if cfg.wdtype == WDTYPE_BF16 else torch.float32
        T, N, K, A, O, P = c.T, c.N, c.K, c.act_dim, c.obs_dim, c.P
        self.w = torch.empty(P, K, **f32)
        self.obs = torch.empty(T + 1, N, O, **f32)
        self.rewards = torch.empty(T, N, K, **f32)
        self.dones = torch.empty(T, N, dtype=torch.uint8, device=self.dev)
        self.eps = torch.empty(T, N, A, **f32)
        self.hp = {}
        self.hp_old = {}
        self.theta_mat, self.theta_vec, self.dtheta_mat, self.dtheta_vec, self.dhp = {}, {}, {}, {}, {}
        for net in (ACTOR, CRITIC):
            n = ctx.hparam_count(net)
            self.hp[net] = torch.empty(n, **f32)
            self.hp_old[net] = torch.empty(n, **f32)
            self.dhp[net] = torch.zeros(n, **f32)
            self.theta_mat[net] = torch.empty(P, ctx.theta_mat_len(net), dtype=wdt, device=self.dev)
            self.theta_vec[net] = torch.empty(P, ctx.theta_vec_len(net), **f32)
            self.dtheta_mat[net] = torch.empty(P, ctx.theta_mat_len(net), **f32)
            self.dtheta_vec[net] = torch.empty(P, ctx.theta_vec_len(net), **f32)
        AO = 2 * A if c.sigma_state else A   # actor output columns: means (+ state-dependent log sigmas)
        self.mu_old = torch.empty(T, N, AO, **f32)
        self.act = torch.empty(T, N, A, **f32)
        self.logp_old = torch.empty(T, N, **f32)
        self.v_roll = torch.empty(T + 1, N, K, **f32)
        self.vtarg = torch.empty(T, N, K, **f32)
        self.adv_s = torch.empty(T, N, **f32)
        assert adv_norm in ("scalar", "per_objective")
        self.adv_norm = adv_norm
        self.adv_vec = torch.empty(T, N, K, **f32) if (keep_adv_vec or adv_norm == "per_objective") else None
        self.adv_mb = torch.empty(T, N, **f32) if adv_norm == "per_objective" else None
        self.mu = torch.zeros(T, N, AO, **f32)
        self.v = torch.zeros(T, N, K, **f32)
        self.dmu = torch.zeros(T, N, AO, **f32)
        self.dv = torch.zeros(T, N, K, **f32)
        self.dlogsig = None if c.sigma_state else torch.zeros(P, A, **f32)
        self.stats = torch.zeros(8, **f32)
        if c.n_g % c.minibatches:
            raise ValueError("minibatches must divide n_g")
        self.mb_rows = [(0, T, b * (c.n_g // c.minibatches), c.n_g // c.minibatches)
                        for b in range(c.minibatches)]
        self.saved = {net: torch.empty(ctx.saved_bytes(net, self.mb_rows[0]), dtype=torch.uint8, device=self.dev)
                      for net in (ACTOR, CRITIC)}
        # one workspace and one stream per network family: the actor and critic chains are independent
        # between the loss (which needs both outputs) and the end of the minibatch
        self.wsn = {net: torch.empty(ctx.workspace_bytes(None), dtype=torch.uint8, device=self.dev)
                    for net in (ACTOR, CRITIC)}
        self.ws = self.wsn[ACTOR]
        self.streams = {net: torch.cuda.Stream(device=self.dev) for net in (ACTOR, CRITIC)} if two_streams else None
        self.side = torch.cuda.Stream(device=self.dev) if side_hypernet else None
        # a workspace per hypernetwork, touched by nothing but its forward and backward: the backward pass then
        # reads the trunk features and factors that the forward pass left there instead of computing them again
        self.hws = {net: torch.empty(ctx.workspace_bytes((0, 1, 0, 1)), dtype=torch.uint8, device=self.dev)
                    for net in (ACTOR, CRITIC)}
        self.optimizer = optimizer
        self.opt_step = 0
        if optimizer is not None:
            self.adam_m = {net: torch.zeros_like(self.hp[net]) for net in (ACTOR, CRITIC)}
            self.adam_v = {net: torch.zeros_like(self.hp[net]) for net in (ACTOR, CRITIC)}
        self.full_T = (0, T, 0, c.n_g)
        self.full_T1 = (0, T + 1, 0, c.n_g)
        self.logsig_off = ctx.theta_vec_len(ACTOR) - A

    def load_inputs(self, d: dict):
        t = self.torch
        put = lambda dst, src: dst.copy_(t.from_numpy(np.ascontiguousarray(src)))
        put(self.w, d["w"]); put(self.obs, d["obs"]); put(self.rewards, d["rewards"])
        put(self.dones, d["dones"]); put(self.eps, d["eps"])
        put(self.hp_old[ACTOR], d["hparams_actor_old"]); put(self.hp_old[CRITIC], d["hparams_critic_old"])
        put(self.hp[ACTOR], d["hparams_actor"]); put(self.hp[CRITIC], d["hparams_critic"])
        t.cuda.synchronize()

    def _per_net(self, fn):
        """Run fn(net, ws) for the actor and the critic, on their own streams when enabled; joins before returning."""
        t = self.torch
        if self.streams is None:
            for net in (ACTOR, CRITIC):
                fn(net, self.wsn[net])
            return
        main = t.cuda.current_stream()
        for net in (ACTOR, CRITIC):
            st = self.streams[net]
            st.wait_stream(main)
            with t.cuda.stream(st):
                fn(net, self.wsn[net])
        for net in (ACTOR, CRITIC):
            main.wait_stream(self.streams[net])

    def rollout(self):
        c, ctx = self.cfg, self.ctx

        def fwd(net, ws):
            ctx.hypernet_fwd(net, self.hp_old[net], self.w, self.theta_mat[net], self.theta_vec[net], ws)
            if net == ACTOR:
                ctx.policy_fwd(ACTOR, self.theta_mat[ACTOR], self.theta_vec[ACTOR], self.obs, self.full_T, self.mu_old,
                               eps=self.eps, act=self.act, logp=self.logp_old, saved=None, ws=ws)
            else:
                ctx.policy_fwd(CRITIC, self.theta_mat[CRITIC], self.theta_vec[CRITIC], self.obs, self.full_T1,
                               self.v_roll, saved=None, ws=ws)

        self._per_net(fwd)
        ctx.vec_gae(self.rewards, self.v_roll, self.dones, self.w, c.gamma, c.lam, self.adv_vec, self.vtarg,
                    self.adv_s)

    def minibatch(self, rows):
        c, ctx = self.cfg, self.ctx
        out = {ACTOR: self.mu, CRITIC: self.v}
        dout = {ACTOR: self.dmu, CRITIC: self.dv}

        def fwd(net, ws):
            ctx.hypernet_fwd(net, self.hp[net], self.w, self.theta_mat[net], self.theta_vec[net], self.hws[net])
            ctx.policy_fwd(net, self.theta_mat[net], self.theta_vec[net], self.obs, rows, out[net],
                           saved=self.saved[net], ws=ws)

        if self.optimizer is not None:
            self.opt_step += 1
        o = self.optimizer

        def bwd(net, ws):
            ctx.policy_bwd(net, self.theta_mat[net], self.theta_vec[net], self.obs, rows, self.saved[net], dout[net],
                           self.dlogsig if net == ACTOR else None, self.dtheta_mat[net], self.dtheta_vec[net], ws)
            ctx.hypernet_bwd_kept(net, self.hp[net], self.w, self.dtheta_mat[net], self.dtheta_vec[net], self.dhp[net],
                                  self.hws[net])
            if o is not None:
                ctx.adam_step(net, self.hp[net], self.dhp[net], self.adam_m[net], self.adam_v[net],
                              o["lr_actor"] if net == ACTOR else o["lr_critic"], o["beta1"], o["beta2"], o["eps"],
                              self.opt_step)

        self._per_net(fwd)
        logsig = None if c.sigma_state else self.theta_vec[ACTOR].data_ptr() + 4 * self.logsig_off
        self._loss(rows, logsig)
        self._per_net(bwd)

    def _loss(self, rows, logsig):
        c, ctx = self.cfg, self.ctx
        adv, norm = self.adv_s, 1
        if self.adv_norm == "per_objective":
            ctx.scalarize_normalized(rows, self.adv_vec, self.w, self.adv_mb, self.ws)
            adv, norm = self.adv_mb, 0
        ctx.ppo_loss_grad(rows, self.mu, logsig, ctx.theta_vec_len(ACTOR), self.act, self.logp_old, adv,
                          self.v, self.vtarg, c.clip_eps, norm, self.dmu, self.dlogsig, self.dv, self.stats, self.ws)

    def capture(self):
        """Record one whole update step into a HIP graph (the default one-stream schedule, no optimiser step: its step
        counter is a host-side argument).  The few hundred launches of a step then cost one submission; what they
        compute is unchanged.  One eager step runs first, so that one-time set-up inside the library (function
        attributes, device queries) happens outside the capture.  Nothing in the step allocates or clears memory
        with a memset node."""
        t = self.torch
        if self.optimizer is not None or self.streams is not None or self.side is not None:
            raise ValueError("capture() records the one-stream schedule without optimiser step")
        self.run()
        t.cuda.synchronize()
        g = t.cuda.CUDAGraph()
        with t.cuda.graph(g):
            self.run()
        self.graph = g
        return g

    def replay(self):
        """Submit the recorded step (capture() first) on the current stream."""
        self.graph.replay()

    def run(self, on_minibatch=None):
        """One whole update step.  `on_minibatch(e, b)` (optional) is called after each minibatch."""
        if self.side is not None:
            return self._run_side(on_minibatch)
        self.rollout()
        for e in range(self.cfg.epochs):
            for b, rows in enumerate(self.mb_rows):
                self.minibatch(rows)
                if on_minibatch is not None:
                    on_minibatch(e, b)

    def _run_side(self, on_minibatch):
        """The same calls with the hypernet work of one network overlapping the grouped GEMMs of the other:
        main stream = rollout, grouped forward / loss / grouped backward; side stream = hypernet backward,
        optimiser step and the hypernet forward of the next minibatch.  Events order every buffer hand-over:
        theta(net) is rewritten only after the main stream's last reader (grouped backward of net), dtheta(net)
        only after the side stream's hypernet backward has read it."""
        t, c, ctx = self.torch, self.cfg, self.ctx
        main, side = t.cuda.current_stream(), self.side
        nets = (ACTOR, CRITIC)
        out = {ACTOR: self.mu, CRITIC: self.v}
        dout = {ACTOR: self.dmu, CRITIC: self.dv}
        o = self.optimizer
        theta_ready = {n: t.cuda.Event() for n in nets}
        theta_free = {n: t.cuda.Event() for n in nets}
        dtheta_ready = {n: t.cuda.Event() for n in nets}
        dtheta_free = {n: None for n in nets}

        # rollout on the main stream; theta(net) is free for the update-time parameters after its forward
        for net in nets:
            ctx.hypernet_fwd(net, self.hp_old[net], self.w, self.theta_mat[net], self.theta_vec[net], self.wsn[net])
        ctx.policy_fwd(ACTOR, self.theta_mat[ACTOR], self.theta_vec[ACTOR], self.obs, self.full_T, self.mu_old,
                       eps=self.eps, act=self.act, logp=self.logp_old, saved=None, ws=self.ws)
        theta_free[ACTOR].record(main)
        ctx.policy_fwd(CRITIC, self.theta_mat[CRITIC], self.theta_vec[CRITIC], self.obs, self.full_T1, self.v_roll,
                       saved=None, ws=self.ws)
        theta_free[CRITIC].record(main)
        with t.cuda.stream(side):
            for net in nets:
                side.wait_event(theta_free[net])
                ctx.hypernet_fwd(net, self.hp[net], self.w, self.theta_mat[net], self.theta_vec[net], self.hws[net])
                theta_ready[net].record(side)
        ctx.vec_gae(self.rewards, self.v_roll, self.dones, self.w, c.gamma, c.lam, self.adv_vec, self.vtarg,
                    self.adv_s)

        steps = [(e, b) for e in range(c.epochs) for b in range(len(self.mb_rows))]
        for i, (e, b) in enumerate(steps):
            rows = self.mb_rows[b]
            last = i + 1 == len(steps)
            if o is not None:
                self.opt_step += 1
            for net in nets:
                main.wait_event(theta_ready[net])
                ctx.policy_fwd(net, self.theta_mat[net], self.theta_vec[net], self.obs, rows, out[net],
                               saved=self.saved[net], ws=self.ws)
            logsig = None if c.sigma_state else self.theta_vec[ACTOR].data_ptr() + 4 * self.logsig_off
            self._loss(rows, logsig)
            for net in nets:
                if dtheta_free[net] is not None:
                    main.wait_event(dtheta_free[net])
                ctx.policy_bwd(net, self.theta_mat[net], self.theta_vec[net], self.obs, rows, self.saved[net], dout[net],
                               self.dlogsig if net == ACTOR else None, self.dtheta_mat[net], self.dtheta_vec[net],
                               self.ws)
                dtheta_ready[net].record(main)
                with t.cuda.stream(side):
                    side.wait_event(dtheta_ready[net])
                    ctx.hypernet_bwd_kept(net, self.hp[net], self.w, self.dtheta_mat[net], self.dtheta_vec[net],
                                          self.dhp[net], self.hws[net])
                    dtheta_free[net] = t.cuda.Event()
                    dtheta_free[net].record(side)
                    if o is not None:
                        ctx.adam_step(net, self.hp[net], self.dhp[net], self.adam_m[net], self.adam_v[net],
                                      o["lr_actor"] if net == ACTOR else o["lr_critic"], o["beta1"], o["beta2"],
                                      o["eps"], self.opt_step)
                    if not last:
                        ctx.hypernet_fwd(net, self.hp[net], self.w, self.theta_mat[net], self.theta_vec[net],
                                         self.hws[net])
                        theta_ready[net] = t.cuda.Event()
                        theta_ready[net].record(side)
            if on_minibatch is not None:
                main.wait_stream(side)
                on_minibatch(e, b)
        main.wait_stream(side)
