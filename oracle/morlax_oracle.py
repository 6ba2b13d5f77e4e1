"""Plain CPU oracle for the MORLAX rollout-and-update step.  TEST INFRASTRUCTURE ONLY.

This file is the slow, obviously-correct definition that the HIP kernels are
checked against.  It may be imported only by `tests/`, by
`__graft_entry__.smoke()` and by the `cpu_baseline` leg of `bench.py`; the
product path never calls it and shares no code with it.

All arithmetic is numpy float64.  Inputs are whatever the caller passes (the
tests pass the float32 tensors of the seeded generator); outputs are float64
arrays which the tests compare with the GPU's float32 results.

Symbols: K objectives (paper: m), P distinct trade-off vectors (paper: K),
N environments in P contiguous groups of n_g = N / P (Sec. III-C, sampling
phase), T rollout horizon, O / A observation / action width, F hypernet
feature width, r factor rank.

Every function names the passage of the paper it follows.  Where the paper
is silent the reading taken is stated next to the code (and collected in the
design notes): the hypernet emits rank-r factors added to shared base
weights; the trunk f is a two-layer tanh MLP; the Gaussian log-std is state
independent and produced by the actor hypernet; the actor mean is tanh(z);
GAE is the textbook recursion with `done` as a select; advantages are
scalarised then normalised over the minibatch with population std + 1e-8;
losses carry no extra coefficients and no entropy term; the optimiser is Adam
with one learning rate per hypernet; a time-limit episode end bootstraps from
the next value but restarts the advantage sum.

Pinned by tests/test_oracle_*.py: closed forms and brute force for GAE,
float64 torch.autograd and central finite differences for every gradient,
library routines (torch linear/tanh/silu, torch Normal.log_prob) for the
forward pieces, structural invariants for the hypernet, closed forms and
torch.optim.Adam for the optimiser step, reduction to the untruncated recursion
on a cut trajectory for the truncation mask, Kolmogorov-Smirnov tests against the Beta marginals
of the uniform distribution on the simplex for the trade-off sampler.  Not pinned
("parity unpinned"): which of the readings above the authors' own code uses,
because that code is not available.
"""
from __future__ import annotations

import math
from collections import OrderedDict

import numpy as np

ACTOR, CRITIC = 0, 1
ACT_TANH, ACT_SILU = 0, 1


# --------------------------------------------------------------------------- shapes

def sigma_state(d):
    """True when the actor's standard deviation is an output of the network (state dependent) instead of
    a per-preference vector from the hypernetwork."""
    return bool(getattr(d, "sigma_state", 0))


def head_dim(d, net):
    """Width of a network's output layer: K values, or A means (+ A log sigmas when state dependent)."""
    if net != ACTOR:
        return d.K
    return 2 * d.act_dim if sigma_state(d) else d.act_dim


def layer_shapes(d, net):
    """(d_out, d_in) per dense layer: O -> W, (W -> W) x (L-1), W -> A or 2A (actor) or K (critic)."""
    out = head_dim(d, net)
    widths = [d.obs_dim] + [d.width] * d.n_hidden + [out]
    return [(widths[i + 1], widths[i]) for i in range(len(widths) - 1)]


def theta_mat_len(d, net):
    return sum(do * di for do, di in layer_shapes(d, net))


def theta_vec_len(d, net):
    n = sum(do for do, _ in layer_shapes(d, net))
    return n + (d.act_dim if (net == ACTOR and not sigma_state(d)) else 0)


def hparam_layout(d, net):
    """name -> (offset, shape) of each hypernet parameter block in the flat vector."""
    K, F, r = d.K, d.hyper_width, d.rank
    lay, off = OrderedDict(), 0

    def add(name, shape):
        nonlocal off
        lay[name] = (off, shape)
        off += int(np.prod(shape))

    add("Wh1", (F, K)); add("bh1", (F,)); add("Wh2", (F, F)); add("bh2", (F,))
    for l, (do, di) in enumerate(layer_shapes(d, net)):
        add(f"W0_{l}", (do, di)); add(f"b0_{l}", (do,))
        if r < 0:       # strictly affine: one row of M per weight
            add(f"MW_{l}", (do * di, F))
        else:
            add(f"MA_{l}", (do * r, F)); add(f"cA_{l}", (do * r,))
            add(f"MB_{l}", (r * di, F)); add(f"cB_{l}", (r * di,))
        add(f"Mb_{l}", (do, F))
    if net == ACTOR and not sigma_state(d):
        add("logsig0", (d.act_dim,)); add("Msig", (d.act_dim, F))
    lay["_total"] = (off, ())
    return lay


def hparam_count(d, net):
    return hparam_layout(d, net)["_total"][0]


def _unpack(d, net, flat):
    flat = np.asarray(flat, dtype=np.float64).reshape(-1)
    lay = hparam_layout(d, net)
    assert flat.size == lay["_total"][0], "hparams length"
    return {k: flat[o:o + int(np.prod(s))].reshape(s) for k, (o, s) in lay.items() if k != "_total"}


def env_pref_index(N, P):
    """g(n): index of the trade-off vector environment n rolls out (Sec. III-C, sampling phase:
    each of the P vectors is repeated N/P times in contiguous blocks).  P > 1 and P | N."""
    if not (P > 1 and N % P == 0):
        raise ValueError("need P > 1 and P | N")
    n_g = N // P
    return (np.arange(N, dtype=np.int64) // n_g).astype(np.int32)


def sample_preferences(u, kappa=0):
    """Trade-off vectors of one iteration (Sec. III-C, sampling phase): P - kappa draws from the
    symmetric Dirichlet distribution with all concentrations 1, i.e. uniform on the simplex, and kappa
    extreme points of the simplex.  u [P, K]: independent uniforms in (0, 1), supplied by the caller.
    A Dirichlet(1, ..., 1) vector is a vector of independent unit exponentials divided by its sum, and
    -ln(u) is a unit exponential, so w[p] = -ln(u[p]) / sum_k -ln(u[p, k]).  Reading taken for the
    extremes: the last kappa rows are the unit vectors e_0, ..., e_{kappa-1} (kappa <= min(P, K));
    their uniforms are ignored."""
    u = np.asarray(u, dtype=np.float64)
    P, K = u.shape
    if not (0 <= kappa <= min(P, K)):
        raise ValueError("kappa must lie in [0, min(P, K)]")
    e = -np.log(u)
    w = e / e.sum(axis=1, keepdims=True)
    for i in range(kappa):
        w[P - kappa + i] = 0.0
        w[P - kappa + i, i] = 1.0
    return w


def check_preferences(w, tol=1e-6):
    """Sec. III-A: every trade-off vector lies on the simplex."""
    w = np.asarray(w, dtype=np.float64)
    return bool(np.all(w >= 0.0) and np.all(np.abs(w.sum(axis=1) - 1.0) <= tol))


def round_bf16(x):
    """float -> nearest bfloat16 (ties to even), returned as float64."""
    f = np.ascontiguousarray(np.asarray(x, dtype=np.float32))
    u = f.view(np.uint32).astype(np.uint64)
    u = (u + np.uint64(0x7FFF) + ((u >> np.uint64(16)) & np.uint64(1))) & np.uint64(0xFFFF0000)
    out = u.astype(np.uint32).view(np.float32)
    out = np.where(np.isnan(f), f, out)
    return out.astype(np.float64)


def _act(z, kind):
    if kind == ACT_TANH:
        return np.tanh(z)
    return z / (1.0 + np.exp(-z))


def _dact(z, kind):
    if kind == ACT_TANH:
        return 1.0 - np.tanh(z) ** 2
    s = 1.0 / (1.0 + np.exp(-z))
    return s * (1.0 + z * (1.0 - s))


# --------------------------------------------------------------------------- hypernetwork

def _hyper_cache(d, net, hparams, w):
    hp = _unpack(d, net, hparams)
    w = np.asarray(w, dtype=np.float64)
    h1 = np.tanh(w @ hp["Wh1"].T + hp["bh1"])
    f = np.tanh(h1 @ hp["Wh2"].T + hp["bh2"])
    return hp, w, h1, f


def hypernet_fwd(d, net, hparams, w):
    """H(w) = M f(w) + b (Sec. III-B), read as: f a two-layer tanh MLP K -> F -> F; the affine map
    emits, per target layer l, factors A_l [d_out, r] and B_l [r, d_in] and a bias delta, and the
    layer's weights are W_l = W0_l + A_l B_l, b_l = b0_l + Mb_l f; the actor also gets
    log sigma = logsig0 + Msig f.  With d.rank < 0 the map is the strictly affine one of the section's
    equation, every weight its own row of M: W_l = W0_l + (MW_l f) reshaped to [d_out, d_in].
    Returns theta_mat [P, mat_len] (layers concatenated, each [d_out, d_in] row-major) and
    theta_vec [P, vec_len] (biases, then the actor's log sigma)."""
    hp, w, h1, f = _hyper_cache(d, net, hparams, w)
    P, r = w.shape[0], d.rank
    mats, vecs = [], []
    for l, (do, di) in enumerate(layer_shapes(d, net)):
        if r < 0:
            W = hp[f"W0_{l}"][None] + (f @ hp[f"MW_{l}"].T).reshape(P, do, di)
        else:
            A = (f @ hp[f"MA_{l}"].T + hp[f"cA_{l}"]).reshape(P, do, r)
            B = (f @ hp[f"MB_{l}"].T + hp[f"cB_{l}"]).reshape(P, r, di)
            W = hp[f"W0_{l}"][None] + np.einsum("pok,pki->poi", A, B)
        mats.append(W.reshape(P, do * di))
        vecs.append(hp[f"b0_{l}"][None] + f @ hp[f"Mb_{l}"].T)
    if net == ACTOR and not sigma_state(d):
        vecs.append(hp["logsig0"][None] + f @ hp["Msig"].T)
    return np.concatenate(mats, axis=1), np.concatenate(vecs, axis=1)


def hypernet_bwd(d, net, hparams, w, dtheta_mat, dtheta_vec):
    """Reverse mode of `hypernet_fwd`: gradient of a scalar with respect to the flat hypernet
    parameters, given its gradient with respect to every preference's theta (Sec. III-C update
    phase: the loss is differentiated back into the hypernetwork)."""
    hp, w, h1, f = _hyper_cache(d, net, hparams, w)
    P, r = w.shape[0], d.rank
    lay = hparam_layout(d, net)
    g = np.zeros(lay["_total"][0], dtype=np.float64)

    def put(name, val):
        o, s = lay[name]
        g[o:o + int(np.prod(s))] = np.asarray(val, dtype=np.float64).reshape(-1)

    dtheta_mat = np.asarray(dtheta_mat, dtype=np.float64)
    dtheta_vec = np.asarray(dtheta_vec, dtype=np.float64)
    df = np.zeros_like(f)
    moff = voff = 0
    for l, (do, di) in enumerate(layer_shapes(d, net)):
        dW = dtheta_mat[:, moff:moff + do * di].reshape(P, do, di)
        db = dtheta_vec[:, voff:voff + do]
        moff += do * di
        voff += do
        put(f"W0_{l}", dW.sum(axis=0))
        put(f"b0_{l}", db.sum(axis=0))
        if r < 0:
            dWf = dW.reshape(P, do * di)
            put(f"MW_{l}", dWf.T @ f)
            df += dWf @ hp[f"MW_{l}"]
        else:
            A = (f @ hp[f"MA_{l}"].T + hp[f"cA_{l}"]).reshape(P, do, r)
            B = (f @ hp[f"MB_{l}"].T + hp[f"cB_{l}"]).reshape(P, r, di)
            dA = np.einsum("poi,pki->pok", dW, B).reshape(P, do * r)
            dB = np.einsum("pok,poi->pki", A, dW).reshape(P, r * di)
            put(f"MA_{l}", dA.T @ f); put(f"cA_{l}", dA.sum(axis=0))
            put(f"MB_{l}", dB.T @ f); put(f"cB_{l}", dB.sum(axis=0))
            df += dA @ hp[f"MA_{l}"] + dB @ hp[f"MB_{l}"]
        put(f"Mb_{l}", db.T @ f)
        df += db @ hp[f"Mb_{l}"]
    if net == ACTOR and not sigma_state(d):
        dls = dtheta_vec[:, voff:voff + d.act_dim]
        put("logsig0", dls.sum(axis=0)); put("Msig", dls.T @ f)
        df += dls @ hp["Msig"]
    dz2 = df * (1.0 - f * f)
    put("Wh2", dz2.T @ h1); put("bh2", dz2.sum(axis=0))
    dz1 = (dz2 @ hp["Wh2"]) * (1.0 - h1 * h1)
    put("Wh1", dz1.T @ w); put("bh1", dz1.sum(axis=0))
    return g


# --------------------------------------------------------------------------- grouped target networks

def full_rows(d, t_cnt):
    return (0, int(t_cnt), 0, d.N // d.P)


def row_mask(d, rows, t_total):
    """Boolean [t_total, N]: the (t, n) cells a row selection covers.  rows = (t0, t_cnt, j0,
    j_cnt) selects times [t0, t0+t_cnt) and, in every preference group, the environments whose
    position inside the group lies in [j0, j0+j_cnt)."""
    t0, tc, j0, jc = rows
    n_g = d.N // d.P
    m = np.zeros((t_total, d.N), dtype=bool)
    j = np.arange(d.N) % n_g
    m[t0:t0 + tc, :] = ((j >= j0) & (j < j0 + jc))[None, :]
    return m


def _split_theta(d, net, theta_mat, theta_vec, p):
    Ws, bs, moff, voff = [], [], 0, 0
    for do, di in layer_shapes(d, net):
        Ws.append(np.asarray(theta_mat[p, moff:moff + do * di], dtype=np.float64).reshape(do, di))
        bs.append(np.asarray(theta_vec[p, voff:voff + do], dtype=np.float64))
        moff += do * di
        voff += do
    logsig = None
    if net == ACTOR and not sigma_state(d):
        logsig = np.asarray(theta_vec[p, voff:voff + d.act_dim], dtype=np.float64)
    return Ws, bs, logsig


def _group_env_index(d, rows, p):
    _, _, j0, jc = rows
    n_g = d.N // d.P
    return p * n_g + j0 + np.arange(jc)


def _mlp_forward(d, net, Ws, bs, X, emulate_bf16):
    """Sec. III-B / III-E: hidden layers h_l = act(W_l h_{l-1} + b_l); actor mean tanh(z) (actuator
    limits), critic output the K-vector z.  With emulate_bf16 every GEMM input activation is
    rounded to bfloat16 on entry (the weights arrive already rounded)."""
    hs, zs = [X], []
    nl = len(Ws)
    for l in range(nl):
        hin = round_bf16(hs[-1]) if emulate_bf16 else hs[-1]
        z = hin @ Ws[l].T + bs[l]
        zs.append(z)
        if l < nl - 1:
            hs.append(_act(z, d.act))
    z = zs[-1]
    out = z
    if net == ACTOR and d.mean_tanh:     # only the means are squashed, a state-dependent log sigma is not
        out = z.copy()
        out[:, :d.act_dim] = np.tanh(z[:, :d.act_dim])
    return hs, zs, out


def policy_fwd(d, net, theta_mat, theta_vec, x, rows, eps=None, emulate_bf16=False, prefs=None):
    """Rollout-phase forward of the family {pi_i} or {V_i} (Sec. III-C): environment n is served by
    the network of preference g(n).  x is [Tx, N, O]; returns `out` [Tx, N, A or K] (with a state-
    dependent standard deviation the actor's `out` is [Tx, N, 2A]: means, then log sigmas) and, when the
    Gaussian noise eps [Tx, N, A] is given (actor only), the sampled action a = mu + sigma * eps
    and its log-density log p = sum_j [ -((a_j - mu_j)/sigma_j)^2 / 2 - log sigma_j ] - (A/2) log 2 pi.
    Cells outside `rows` stay zero.  `prefs` (optional) restricts the work to those preference
    indices (the others' cells stay zero); preferences do not interact in this step."""
    x = np.asarray(x, dtype=np.float64)
    Tx = x.shape[0]
    t0, tc, j0, jc = rows
    odim = head_dim(d, net)
    out = np.zeros((Tx, d.N, odim))
    act = logp = None
    if eps is not None:
        assert net == ACTOR
        eps = np.asarray(eps, dtype=np.float64)
        act = np.zeros((Tx, d.N, d.act_dim))
        logp = np.zeros((Tx, d.N))
    for p in (range(d.P) if prefs is None else prefs):
        Ws, bs, logsig = _split_theta(d, net, theta_mat, theta_vec, p)
        idx = _group_env_index(d, rows, p)
        X = x[t0:t0 + tc][:, idx, :].reshape(tc * jc, d.obs_dim)
        _, _, o = _mlp_forward(d, net, Ws, bs, X, emulate_bf16)
        o = o.reshape(tc, jc, odim)
        out[t0:t0 + tc, idx[0]:idx[0] + jc, :] = o
        if eps is not None:
            mu = o[..., :d.act_dim]
            ls = o[..., d.act_dim:] if sigma_state(d) else logsig   # per state, or per preference
            e = eps[t0:t0 + tc, idx[0]:idx[0] + jc, :]
            a = mu + np.exp(ls) * e
            act[t0:t0 + tc, idx[0]:idx[0] + jc, :] = a
            logp[t0:t0 + tc, idx[0]:idx[0] + jc] = gaussian_logp(a, mu, ls)
    return out, act, logp


def gaussian_logp(a, mu, logsig):
    """Log-density of a diagonal Gaussian N(mu, diag(exp(logsig))^2) at a, summed over action dims."""
    sig = np.exp(logsig)
    q = (a - mu) / sig
    A = a.shape[-1]
    return (-0.5 * q * q - logsig).sum(axis=-1) - 0.5 * A * math.log(2.0 * math.pi)


def policy_bwd(d, net, theta_mat, theta_vec, x, rows, dout, dlogsig=None, emulate_bf16=False,
               want_dx=False, prefs=None):
    """Reverse mode through the grouped target networks: given dL/d(out) on the selected rows,
    returns dL/dtheta_mat [P, mat_len] and dL/dtheta_vec [P, vec_len] (bias gradients, then for the
    actor the given dL/dlogsig [P, A] copied through).  dW_l(p) = dZ_l^T H_{l-1} over the rows of
    preference p, db_l(p) = column sums of dZ_l, dH_{l-1} = dZ_l W_l(p), dZ = dH * act'(z).
    With emulate_bf16 both operands of every GEMM are rounded to bfloat16 on entry.  `prefs`
    (optional) restricts the work to those preference indices; the other rows stay zero."""
    x = np.asarray(x, dtype=np.float64)
    dout = np.asarray(dout, dtype=np.float64)
    t0, tc, j0, jc = rows
    odim = head_dim(d, net)
    dmat = np.zeros((d.P, theta_mat_len(d, net)))
    dvec = np.zeros((d.P, theta_vec_len(d, net)))
    dx = np.zeros_like(x) if want_dx else None
    rb = round_bf16 if emulate_bf16 else (lambda a: a)
    for p in (range(d.P) if prefs is None else prefs):
        Ws, bs, _ = _split_theta(d, net, theta_mat, theta_vec, p)
        idx = _group_env_index(d, rows, p)
        X = x[t0:t0 + tc][:, idx, :].reshape(tc * jc, d.obs_dim)
        hs, zs, o = _mlp_forward(d, net, Ws, bs, X, emulate_bf16)
        dz = dout[t0:t0 + tc][:, idx, :].reshape(tc * jc, odim)
        if net == ACTOR and d.mean_tanh:
            dz = dz.copy()
            dz[:, :d.act_dim] *= 1.0 - o[:, :d.act_dim] ** 2
        gW, gb = [None] * len(Ws), [None] * len(Ws)
        for l in range(len(Ws) - 1, -1, -1):
            gW[l] = rb(dz).T @ rb(hs[l])
            gb[l] = dz.sum(axis=0)
            if l > 0 or want_dx:
                dh = rb(dz) @ Ws[l]
                if l > 0:
                    dz = dh * _dact(zs[l - 1], d.act)
                else:
                    dx[t0:t0 + tc, idx[0]:idx[0] + jc, :] = dh.reshape(tc, jc, d.obs_dim)
        dmat[p] = np.concatenate([g.reshape(-1) for g in gW])
        vec = np.concatenate(gb)
        dvec[p, :vec.size] = vec
    if net == ACTOR and dlogsig is not None:
        assert not sigma_state(d), "a state-dependent log sigma is part of dout"
        dvec[:, -d.act_dim:] = np.asarray(dlogsig, dtype=np.float64)
    if want_dx:
        return dmat, dvec, dx
    return dmat, dvec


# --------------------------------------------------------------------------- advantage estimation

def vec_gae(r, v, done, w, gamma, lam, trunc=None):
    """Generalised advantage estimation applied to each objective on its own, then scalarised with
    the environment's trade-off vector (Sec. III-C, update phase).  r [T,N,K], v [T+1,N,K],
    done [T,N] (1: the transition at step t ended the episode), w [P,K].  Backward in time,
    per (n, k): if done: delta = r_t - V_t and the running sum restarts at delta; otherwise
    delta = r_t + gamma V_{t+1} - V_t and A_t = delta + gamma lam A_{t+1}; A_T = 0.
    Value target Vhat_t = A_t + V_t.  Scalar advantage A^s[t,n] = sum_k w[g(n),k] A_t[n,k].
    `done` acts as a select, so nothing after an episode end can reach the steps before it.

    trunc [T,N] (optional; Sec. III-E separates failures from time limits in value estimation):
    1 where the episode end at step t was a time limit.  Reading taken: a truncated step still
    bootstraps from V_{t+1}, which the caller supplies as the value of the state the episode was cut
    at, but like every episode end it restarts the running sum: delta = r_t + gamma V_{t+1} - V_t,
    A_t = delta.  A step with trunc = 1 counts as an episode end whatever `done` says."""
    r = np.asarray(r, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    done = np.asarray(done)
    w = np.asarray(w, dtype=np.float64)
    T, N, K = r.shape
    P = w.shape[0]
    g = env_pref_index(N, P)
    adv = np.zeros((T, N, K))
    acc = np.zeros((N, K))
    for t in range(T - 1, -1, -1):
        dn = (done[t] != 0)[:, None]
        delta_live = r[t] + gamma * v[t + 1] - v[t]
        delta_done = r[t] - v[t]
        acc = np.where(dn, delta_done, delta_live + gamma * lam * acc)
        if trunc is not None:
            tr = (np.asarray(trunc)[t] != 0)[:, None]
            acc = np.where(tr, delta_live, acc)
        adv[t] = acc
    vtarg = adv + v[:T]
    wn = w[g]                                  # [N, K]
    adv_s = np.zeros((T, N))
    for k in range(K):
        adv_s += adv[:, :, k] * wn[None, :, k]
    return adv, vtarg, adv_s


def adv_norm_stats(adv_s, mask):
    """Mean and population standard deviation of the scalarised advantage over the minibatch."""
    a = np.asarray(adv_s, dtype=np.float64)[mask]
    m = a.mean()
    s = math.sqrt(((a - m) ** 2).mean())
    return m, s


def scalarize_normalized(d, rows, adv_vec, w):
    """Per-objective normalisation before scalarisation -- the other reading of "normalised across the
    batch" in the update phase (Sec. III-C): every objective's advantages are standardised over the
    selected cells on their own (mean, population standard deviation, + 1e-8), and only then combined
    with the trade-off vector of the environment:
      Ahat[t, n] = sum_k w[g(n), k] (A_k[t, n] - mean_k) / (std_k + 1e-8).
    Objectives with very different reward scales then weigh in by w alone.  adv_vec [T, N, K],
    w [P, K]; returns [T, N] with zeros outside the selection."""
    a = np.asarray(adv_vec, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    T, N, K = a.shape
    mask = row_mask(d, rows, T)
    g = env_pref_index(N, w.shape[0])
    out = np.zeros((T, N))
    for k in range(K):
        sel = a[:, :, k][mask]
        mean = sel.mean()
        std = math.sqrt(((sel - mean) ** 2).mean())
        out += w[g, k][None, :] * (a[:, :, k] - mean) / (std + 1e-8)
    out[~mask] = 0.0
    return out


# --------------------------------------------------------------------------- losses

def ppo_loss_grad(d, rows, mu, logsig, act, logp_old, adv_s, v, vtarg, clip_eps, norm_adv=True):
    """Clipped PPO surrogate and vector value loss on one minibatch with their gradients
    (Sec. III-C, update phase).  With B the number of selected (t, n) cells:
      Ahat = (A^s - mean) / (std + 1e-8) over the minibatch (if norm_adv),
      rho  = exp(log pi_theta(a|s) - log pi_old(a|s)),
      L_pi = -(1/B) sum min(rho Ahat, clip(rho, 1-eps, 1+eps) Ahat),
      L_V  = (1/B) sum_rows sum_k (V_k - Vhat_k)^2.
    Ahat, Vhat, log pi_old and the actions are constants.  Gradients: the clipped branch is flat,
    so dL/dlogp = -(1/B) Ahat rho where (Ahat >= 0 and rho <= 1+eps) or (Ahat < 0 and rho >= 1-eps),
    else 0; dlogp/dmu_j = (a_j - mu_j)/sigma_j^2; dlogp/dlogsig_j = ((a_j-mu_j)/sigma_j)^2 - 1,
    summed over the rows of each preference; dL_V/dV_k = 2 (V_k - Vhat_k) / B.
    Returns dmu [Tx,N,A], dlogsig [P,A], dv [Tx,N,K] (zero outside the rows) and
    stats = [L_pi, L_V, clip fraction, mean(logp_old - logp), adv mean, adv std, mean rho, B].
    With a state-dependent standard deviation `mu` is the actor's whole output [Tx,N,2A] (means, then
    log sigmas), `logsig` is ignored, the first return value is the gradient of that output
    [Tx,N,2A] (the log-sigma gradients stay per cell) and the second is None."""
    mu = np.asarray(mu, dtype=np.float64); act = np.asarray(act, dtype=np.float64)
    logp_old = np.asarray(logp_old, dtype=np.float64); adv_s = np.asarray(adv_s, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64); vtarg = np.asarray(vtarg, dtype=np.float64)
    Tx = mu.shape[0]
    mask = row_mask(d, rows, Tx)
    B = int(mask.sum())
    g = env_pref_index(d.N, d.P)
    if sigma_state(d):
        mu, ls = mu[..., :d.act_dim], mu[..., d.act_dim:]           # [Tx, N, A] each
    else:
        ls = np.asarray(logsig, dtype=np.float64)[g][None, :, :]    # [1, N, A]
    sig = np.exp(ls)
    if norm_adv:
        m, s = adv_norm_stats(adv_s[:Tx], mask)
        ahat = (adv_s[:Tx] - m) / (s + 1e-8)
    else:
        m, s = adv_norm_stats(adv_s[:Tx], mask)
        ahat = adv_s[:Tx].copy()
    q = (act - mu) / sig
    logp = (-0.5 * q * q - ls).sum(axis=-1) - 0.5 * d.act_dim * math.log(2.0 * math.pi)
    rho = np.exp(logp - logp_old[:Tx])
    surr = np.minimum(rho * ahat, np.clip(rho, 1.0 - clip_eps, 1.0 + clip_eps) * ahat)
    L_pi = -(surr[mask].sum()) / B
    dv_all = v[:Tx] - vtarg[:Tx]
    L_V = (dv_all ** 2).sum(axis=-1)[mask].sum() / B
    live = np.where(ahat >= 0.0, rho <= 1.0 + clip_eps, rho >= 1.0 - clip_eps)
    dlogp = np.where(live & mask, -ahat * rho / B, 0.0)       # [Tx, N]
    dmu = np.where(mask[..., None], dlogp[..., None] * q / sig, 0.0)
    dls_rows = np.where(mask[..., None], dlogp[..., None] * (q * q - 1.0), 0.0)   # [Tx, N, A]
    if sigma_state(d):
        dmu = np.concatenate([dmu, dls_rows], axis=-1)
        dlogsig = None
    else:
        dlogsig = np.zeros((d.P, d.act_dim))
        for p in range(d.P):
            sel = (g == p)
            dlogsig[p] = dls_rows[:, sel, :].sum(axis=(0, 1))
    dv = np.where(mask[..., None], 2.0 * dv_all / B, 0.0)
    clipped = (np.abs(rho - 1.0) > clip_eps)
    stats = np.array([L_pi, L_V, clipped[mask].mean(), (logp_old[:Tx] - logp)[mask].mean(),
                      m, s, rho[mask].mean(), float(B)])
    return dmu, dlogsig, dv, stats


# --------------------------------------------------------------------------- one update step

def adam_step(theta, g, m, v, lr, beta1, beta2, eps, t):
    """One Adam step (Kingma & Ba 2015, Algorithm 1) on a flat parameter vector; t = 1 for the first
    step.  The paper updates the two hypernets separately so that they can learn at different rates
    (Sec. III-C, update phase) and does not name the optimiser; Adam is the reading taken.
      m <- beta1 m + (1 - beta1) g,  v <- beta2 v + (1 - beta2) g^2,
      theta <- theta - lr (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps).
    Returns (theta, m, v) as new float64 arrays."""
    theta = np.asarray(theta, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    m = beta1 * np.asarray(m, dtype=np.float64) + (1.0 - beta1) * g
    v = beta2 * np.asarray(v, dtype=np.float64) + (1.0 - beta2) * g * g
    m_hat = m / (1.0 - beta1 ** t)
    v_hat = v / (1.0 - beta2 ** t)
    return theta - lr * m_hat / (np.sqrt(v_hat) + eps), m, v


def minibatch_rows(d, T, b, MB):
    """Minibatch b of MB: every time step, and in each preference group the b-th slice of n_g / MB
    environments, so every minibatch holds every preference."""
    n_g = d.N // d.P
    if n_g % MB:
        raise ValueError("MB must divide n_g")
    return (0, T, b * (n_g // MB), n_g // MB)


def update_step(d, w, hp_actor_old, hp_critic_old, hp_actor, hp_critic, obs, rewards, dones, eps,
                gamma, lam, clip_eps, minibatches=1, epochs=1, emulate_bf16=False, keep=False, optimizer=None,
                adv_norm="scalar"):
    """One MORLAX iteration after the trade-offs are drawn (Sec. III-C): rollout forward of the
    actor family (sampling actions and their log-density) and of the critic family at every state,
    vector GAE, then for every epoch and minibatch the losses and their gradients with respect to
    both hypernets.  The actor loss reaches only the actor hypernet and the value loss only the
    critic hypernet (decoupled updates).  Without `optimizer` no parameter changes, so every
    minibatch is evaluated at the same update-time parameters.  With optimizer = dict(lr_actor,
    lr_critic, beta1, beta2, eps) each minibatch is followed by one Adam step on either hypernet with
    its own learning rate (moments start at zero, step counter t = 1, 2, ...), and the result holds
    the final parameters and moments.  adv_norm = "scalar": the scalarised advantage is normalised over
    the minibatch; "per_objective": scalarize_normalized() instead.  Returns a dict; with keep=True it also holds the intermediate
    tensors of the first minibatch."""
    T = rewards.shape[0]
    wq = (lambda m: round_bf16(m)) if (emulate_bf16 and d.wdtype == 1) else (lambda m: m)
    emu = bool(emulate_bf16 and d.wdtype == 1)
    res = {}
    tm_a0, tv_a0 = hypernet_fwd(d, ACTOR, hp_actor_old, w)
    tm_c0, tv_c0 = hypernet_fwd(d, CRITIC, hp_critic_old, w)
    tm_a0, tm_c0 = wq(tm_a0), wq(tm_c0)
    mu_old, act, logp_old = policy_fwd(d, ACTOR, tm_a0, tv_a0, obs[:T], full_rows(d, T), eps=eps,
                                       emulate_bf16=emu)
    v_roll, _, _ = policy_fwd(d, CRITIC, tm_c0, tv_c0, obs, full_rows(d, T + 1), emulate_bf16=emu)
    adv_vec, vtarg, adv_s = vec_gae(rewards, v_roll, dones, w, gamma, lam)
    grads = []
    if optimizer is not None:
        hp_actor = np.asarray(hp_actor, dtype=np.float64).copy()
        hp_critic = np.asarray(hp_critic, dtype=np.float64).copy()
        mom = {n: [np.zeros_like(h), np.zeros_like(h)] for n, h in ((ACTOR, hp_actor), (CRITIC, hp_critic))}
        t_opt = 0
    for e in range(epochs):
        for b in range(minibatches):
            rows = minibatch_rows(d, T, b, minibatches)
            tm_a, tv_a = hypernet_fwd(d, ACTOR, hp_actor, w)
            tm_c, tv_c = hypernet_fwd(d, CRITIC, hp_critic, w)
            tm_a, tm_c = wq(tm_a), wq(tm_c)
            mu, _, _ = policy_fwd(d, ACTOR, tm_a, tv_a, obs[:T], rows, emulate_bf16=emu)
            vv, _, _ = policy_fwd(d, CRITIC, tm_c, tv_c, obs[:T], rows, emulate_bf16=emu)
            logsig = None if sigma_state(d) else tv_a[:, -d.act_dim:]
            if adv_norm == "per_objective":
                dmu, dlogsig, dv, stats = ppo_loss_grad(d, rows, mu, logsig, act, logp_old,
                                                        scalarize_normalized(d, rows, adv_vec, w), vv, vtarg,
                                                        clip_eps, False)
            else:
                dmu, dlogsig, dv, stats = ppo_loss_grad(d, rows, mu, logsig, act, logp_old, adv_s, vv,
                                                        vtarg, clip_eps, True)
            dm_a, dvec_a = policy_bwd(d, ACTOR, tm_a, tv_a, obs[:T], rows, dmu, dlogsig, emulate_bf16=emu)
            dm_c, dvec_c = policy_bwd(d, CRITIC, tm_c, tv_c, obs[:T], rows, dv, None, emulate_bf16=emu)
            g_a = hypernet_bwd(d, ACTOR, hp_actor, w, dm_a, dvec_a)
            g_c = hypernet_bwd(d, CRITIC, hp_critic, w, dm_c, dvec_c)
            grads.append({"rows": rows, "dhp_actor": g_a, "dhp_critic": g_c, "stats": stats})
            if optimizer is not None:
                t_opt += 1
                o = optimizer
                hp_actor, mom[ACTOR][0], mom[ACTOR][1] = adam_step(hp_actor, g_a, mom[ACTOR][0], mom[ACTOR][1],
                                                                  o["lr_actor"], o["beta1"], o["beta2"], o["eps"], t_opt)
                hp_critic, mom[CRITIC][0], mom[CRITIC][1] = adam_step(hp_critic, g_c, mom[CRITIC][0], mom[CRITIC][1],
                                                                     o["lr_critic"], o["beta1"], o["beta2"], o["eps"], t_opt)
            if keep and e == 0 and b == 0:
                res.update(mu=mu, v=vv, dmu=dmu, dlogsig=dlogsig, dv=dv, dtheta_mat_actor=dm_a,
                           dtheta_vec_actor=dvec_a, dtheta_mat_critic=dm_c, dtheta_vec_critic=dvec_c,
                           theta_mat_actor=tm_a, theta_vec_actor=tv_a, theta_mat_critic=tm_c,
                           theta_vec_critic=tv_c)
    res["grads"] = grads
    if optimizer is not None:
        res.update(hp_actor=hp_actor, hp_critic=hp_critic, adam_m_actor=mom[ACTOR][0], adam_v_actor=mom[ACTOR][1],
                   adam_m_critic=mom[CRITIC][0], adam_v_critic=mom[CRITIC][1])
    if keep:
        res.update(mu_old=mu_old, act=act, logp_old=logp_old, v_roll=v_roll, adv_vec=adv_vec,
                   vtarg=vtarg, adv_s=adv_s)
    return res
