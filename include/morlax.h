/*
 * morlax.h -- C ABI of the MI355X (gfx950) hot path of MORLAX: the preference-conditioned
 * rollout-and-update step over N parallel environments (paper Sec. III-A..III-C, III-E).
 *
 * Symbols.  K objectives (the paper's m); P distinct trade-off vectors per iteration (the paper's
 * K); N environments split into P contiguous groups of n_g = N / P, environment n using trade-off
 * g(n) = n / n_g (Sec. III-C, sampling phase); T rollout horizon; O / A observation / action
 * width; target networks with L hidden layers of width W; F hypernet feature width; r factor rank.
 *
 * Conventions for every entry point
 *  - All tensor pointers are DEVICE pointers owned by the caller, contiguous, 16-byte aligned.
 *    The library allocates no device memory and frees none.  `ws` is caller-provided device
 *    scratch of `ws_bytes` bytes; morlax_workspace_bytes() is enough for every op on a selection,
 *    a smaller buffer is accepted when it covers what the called op needs, else the call fails
 *    with MORLAX_ERR_WORKSPACE.  Its contents are undefined between calls.
 *  - `stream` is a hipStream_t passed as void*.  Every op only enqueues kernels on it and returns;
 *    nothing synchronises.  Calls that share `ws`, `saved` or outputs must be stream-ordered.
 *  - Time-major layouts: x [Tx, N, O], out [Tx, N, A|K], r [T, N, K], done [T, N] ...; the row of
 *    (t, n) is t * N + n.
 *  - A row selection `morlax_rows` picks times [t0, t0+t_cnt) and, inside every preference group,
 *    the environments at positions [j0, j0+j_cnt): every selection holds every preference, so the
 *    per-preference (grouped) structure is kept.  Minibatch b of MB is {0, T, b*n_g/MB, n_g/MB}.
 *    Outputs are overwritten on the selected cells and not touched elsewhere.
 *  - Return value: MORLAX_OK or a negative morlax_status.  All argument checks run on the host
 *    before the first HIP call; a failed check launches nothing.  morlax_last_error() gives the
 *    message of the last failure on the calling thread.
 *  - theta layout (per preference): theta_mat = the layers' weight matrices concatenated, layer l
 *    stored [d_out, d_in] row-major (y = W x), element type fp32 or bf16 (dims.wdtype);
 *    theta_vec (fp32) = the layers' biases concatenated, then for the actor log sigma [A].
 *    Layers: O -> W, (W -> W) x (L-1), W -> A (actor) or K (critic).
 *  - hparams layout (fp32, flat, every block row-major): trunk Wh1 [F,K], bh1 [F], Wh2 [F,F],
 *    bh2 [F]; per target layer W0 [d_out,d_in], b0 [d_out], MA [d_out*r, F], cA [d_out*r],
 *    MB [r*d_in, F], cB [r*d_in], Mb [d_out, F]; actor only: logsig0 [A], Msig [A, F].
 */
#ifndef MORLAX_H
#define MORLAX_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct morlax_ctx morlax_ctx; /* opaque: dimensions and derived layouts, no device memory */

typedef enum { MORLAX_ACTOR = 0, MORLAX_CRITIC = 1 } morlax_net;

typedef enum {
    MORLAX_OK = 0,
    MORLAX_ERR_NULL = -1,        /* a required pointer is NULL */
    MORLAX_ERR_SHAPE = -2,       /* P < 2, P does not divide N, K < 1, bad row selection, misaligned pointer ... */
    MORLAX_ERR_UNSUPPORTED = -3, /* a size outside what the kernels are built for */
    MORLAX_ERR_WORKSPACE = -4,   /* ws_bytes is less than the op needs for these arguments */
    MORLAX_ERR_HIP = -5          /* a HIP runtime call failed */
} morlax_status;

typedef struct {
    int32_t K, P, N, T;
    int32_t obs_dim, act_dim;
    int32_t n_hidden, width;
    int32_t act;         /* hidden activation: 0 tanh, 1 SiLU */
    int32_t rank;        /* r >= 0: rank of the per-preference weight delta; -1: strictly affine hypernetwork */
    int32_t hyper_width; /* F */
    int32_t wdtype;      /* 0: fp32 weights and GEMM inputs; 1: bf16 weights and GEMM inputs, fp32 accumulate */
    int32_t mean_tanh;   /* 1: actor mean = tanh(z) (Sec. III-E); 0: mean = z */
    int32_t sigma_state; /* 0: log sigma [P, A] comes from the actor hypernetwork (theta_vec tail); 1: it is an output of
                            the actor network -- its output layer is 2A wide (means, then log sigmas), 2A <= 16 */
} morlax_dims;

typedef struct {
    int32_t t0, t_cnt;
    int32_t j0, j_cnt;
} morlax_rows;

/* Limits: 1 <= K <= 16, 1 <= act_dim <= 16, 1 <= obs_dim <= 1024, 1 <= n_hidden <= 8,
 * width a multiple of 16 in [16, 2048], -1 <= rank <= 32, 1 <= hyper_width <= 64, 2 <= P <= 65535, P | N. */
int morlax_create(const morlax_dims* dims, morlax_ctx** out);
void morlax_destroy(morlax_ctx* ctx);
const char* morlax_last_error(void); /* thread-local, never NULL */

int64_t morlax_hparam_count(const morlax_ctx* ctx, int net);   /* floats in a hypernet's flat parameter vector */
int64_t morlax_theta_mat_len(const morlax_ctx* ctx, int net);  /* weight elements per preference */
int64_t morlax_theta_vec_len(const morlax_ctx* ctx, int net);  /* fp32 elements per preference */
/* Bytes of the `saved` buffer policy_fwd fills for policy_bwd on this selection (rows NULL: all
 * n_g environments and T+1 times). */
int64_t morlax_saved_bytes(const morlax_ctx* ctx, int net, const morlax_rows* rows);
/* Bytes of scratch sufficient for every op on this selection (rows NULL: as above). */
int64_t morlax_workspace_bytes(const morlax_ctx* ctx, const morlax_rows* rows);

/* g(n) = n / n_g for n in [0, N): the environment -> trade-off map (Sec. III-C, sampling phase:
 * each trade-off repeated N/P times in contiguous blocks).  out [N] int32, device. */
int morlax_env_pref_index(const morlax_ctx* ctx, int32_t* out, void* stream);

/* Hypernetwork forward H(w) = M f(w) + b (Sec. III-B) for all P trade-offs: f is a two-layer tanh
 * MLP K -> F -> F; the affine map emits per target layer the factors A_l [d_out, r], B_l [r, d_in]
 * and a bias delta; W_l(p) = W0_l + A_l(p) B_l(p), b_l(p) = b0_l + Mb_l f(p); actor:
 * log sigma(p) = logsig0 + Msig f(p).  With dims.rank = -1 the map is the section's equation as it
 * stands: every weight has its own row of M, W_l(p) = W0_l + reshape(MW_l f(p)), MW_l [d_out * d_in, F]
 * stored in hparams where the factor maps would be (block order per layer: W0, b0, MW, Mb).
 * All arithmetic fp32; theta_mat rounded once (nearest even) when dims.wdtype is bf16.
 *   hparams [hparam_count] fp32, w [P, K] fp32 (rows on the simplex; not checked on the device)
 *   -> theta_mat [P, theta_mat_len] (wdtype), theta_vec [P, theta_vec_len] fp32. */
int morlax_hypernet_fwd(morlax_ctx* ctx, int net, const float* hparams, const float* w,
                        void* theta_mat, float* theta_vec, void* ws, int64_t ws_bytes, void* stream);

/* Reverse mode of morlax_hypernet_fwd (Sec. III-C, update phase: the losses are differentiated
 * back into each hypernetwork separately).  dtheta_mat [P, theta_mat_len] fp32 and dtheta_vec
 * [P, theta_vec_len] fp32 are the loss gradients w.r.t. every preference's parameters;
 * dhparams [hparam_count] fp32 is overwritten.  Reductions run in a fixed order (no atomics). */
int morlax_hypernet_bwd(morlax_ctx* ctx, int net, const float* hparams, const float* w,
                        const float* dtheta_mat, const float* dtheta_vec, float* dhparams,
                        void* ws, int64_t ws_bytes, void* stream);

/* The same reverse pass for a caller that kept the forward pass's workspace: ws_fwd must be the buffer the
 * last morlax_hypernet_fwd of this network ran in -- with these hparams and w -- and nothing may have
 * written to it since (give each network a workspace of its own, used by no other call).  The trunk
 * features and the factors are then read from it instead of being computed again; the result is bit for
 * bit that of morlax_hypernet_bwd.  The library cannot check the condition: a stale workspace gives wrong
 * gradients, not an error. */
int morlax_hypernet_bwd_kept(morlax_ctx* ctx, int net, const float* hparams, const float* w,
                             const float* dtheta_mat, const float* dtheta_vec, float* dhparams,
                             void* ws_fwd, int64_t ws_bytes, void* stream);

/* Grouped forward of the target-network family {pi_i} or {V_i} (Sec. III-C, rollout phase;
 * Sec. III-E for the tanh on the actor output): every selected (t, n) row of x goes through the
 * network of preference g(n).  Hidden layers h = act(W h + b); actor out = tanh(z) (or z when
 * mean_tanh = 0), critic out = z in R^K.  With dims.wdtype = bf16 every GEMM input is bf16 and
 * accumulation fp32; bias, activation and outputs are fp32.
 *   x [Tx, N, O] fp32; out [Tx, N, A] (actor) or [Tx, N, K] (critic) fp32.
 *   Actor only, all three or none: eps [Tx, N, A] standard normal noise -> act = out + sigma * eps
 *   and logp [Tx, N] = sum_j [ -((act_j - out_j)/sigma_j)^2 / 2 - log sigma_j ] - (A/2) log(2 pi).
 *   saved: NULL for inference/rollout, else morlax_saved_bytes() bytes that policy_bwd needs. */
int morlax_policy_fwd(morlax_ctx* ctx, int net, const void* theta_mat, const float* theta_vec,
                      const float* x, const morlax_rows* rows, float* out, const float* eps,
                      float* act, float* logp, void* saved, void* ws, int64_t ws_bytes, void* stream);

/* Grouped backward through the target networks (Sec. III-C, update phase).  dout [Tx, N, A|K] is
 * dL/d(out) on the selected rows; `saved` comes from the matching policy_fwd call (same ctx, net,
 * theta, x, rows).  Outputs, overwritten: dtheta_mat [P, theta_mat_len] fp32 with
 * dW_l(p) = sum over p's rows of dZ_l^T h_{l-1}, and dtheta_vec [P, theta_vec_len] fp32 with the
 * bias gradients followed (actor) by dlogsig [P, A] copied through (zeros when dlogsig is NULL). */
int morlax_policy_bwd(morlax_ctx* ctx, int net, const void* theta_mat, const float* theta_vec,
                      const float* x, const morlax_rows* rows, const void* saved, const float* dout,
                      const float* dlogsig, float* dtheta_mat, float* dtheta_vec, void* ws,
                      int64_t ws_bytes, void* stream);

/* Vector generalised advantage estimation, one reverse-time scan per (environment, objective),
 * then scalarisation with the environment's trade-off (Sec. III-C, update phase).
 *   r [T, N, K], v [T+1, N, K], done [T, N] u8 (non-zero: the transition at t ended the episode),
 *   w [P, K].  Backwards from t = T-1 with A_T = 0:
 *     done:  delta = r_t - V_t,                 A_t = delta
 *     else:  delta = r_t + gamma V_{t+1} - V_t, A_t = delta + gamma lambda A_{t+1}
 *   (`done` is a select: nothing after an episode end can influence the steps before it.)
 *   -> vtarg [T, N, K] = A_t + V_t, adv_s [T, N] = sum_k w[g(n), k] A_t[n, k],
 *      adv_vec [T, N, K] = A_t (optional, NULL to skip). */
int morlax_vec_gae(morlax_ctx* ctx, const float* r, const float* v, const uint8_t* done,
                   const float* w, float gamma, float lambda, float* adv_vec, float* vtarg,
                   float* adv_s, void* stream);

/* The same scan with time limits told apart from failures (Sec. III-E: terminations and truncations
 * are distinguished in value estimation).  trunc [T, N] u8, non-zero: the episode was cut by a time
 * limit at step t.  Such a step keeps the bootstrap, delta = r_t + gamma V_{t+1} - V_t with V_{t+1}
 * the value of the state the episode was cut at (the caller stores it in v[t+1]), and restarts the
 * sum like any episode end: A_t = delta.  A step with trunc != 0 is an episode end whatever done[t]
 * says; with trunc all zero the results equal morlax_vec_gae's bit for bit.  Other arguments,
 * layouts and errors as morlax_vec_gae; trunc is a device pointer and must not be NULL. */
int morlax_vec_gae_trunc(morlax_ctx* ctx, const float* r, const float* v, const uint8_t* done,
                         const uint8_t* trunc, const float* w, float gamma, float lambda,
                         float* adv_vec, float* vtarg, float* adv_s, void* stream);

/* Trade-off vectors of one iteration (Sec. III-C, sampling phase): P - kappa rows drawn from the
 * symmetric Dirichlet distribution with all concentrations 1 (uniform on the simplex) and kappa
 * extreme points.  u [P, K] (device): independent uniforms in (0, 1) supplied by the caller, so that
 * the draw is reproducible; w [P, K] (device, overwritten): w[p] = -ln u[p] / sum_k -ln u[p, k] for
 * p < P - kappa, and row P - kappa + i = unit vector e_i (reading taken for "the extreme endpoints
 * within the simplex"; their uniforms are ignored).  MORLAX_ERR_SHAPE unless 0 <= kappa <= min(P, K). */
int morlax_sample_preferences(morlax_ctx* ctx, const float* u, int32_t kappa, float* w, void* stream);

/* One Adam step on the hypernet parameters of `net` (Sec. III-C, update phase: the two hypernets are
 * updated separately so that they can learn at different rates; the paper does not name the
 * optimiser, Adam with bias correction is the reading taken).  All arrays are device pointers to
 * morlax_hparam_count(ctx, net) floats; hparams, m and v are updated in place, dhparams is read:
 *   m <- beta1 m + (1 - beta1) g,   v <- beta2 v + (1 - beta2) g^2,
 *   hparams <- hparams - lr (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps).
 * step counts from 1; the caller zeroes m and v before the first step and keeps one (m, v, step,
 * lr) per hypernet.  MORLAX_ERR_SHAPE for step < 1, betas outside [0, 1), eps <= 0 or lr < 0. */
int morlax_adam_step(morlax_ctx* ctx, int net, float* hparams, const float* dhparams, float* m,
                     float* v, float lr, float beta1, float beta2, float eps, int32_t step,
                     void* stream);

/* Per-objective advantage normalisation before scalarisation: the alternative reading of the update
 * phase's "normalised across the batch" (Sec. III-C).  Over the selected cells every objective k of the
 * vector advantage is standardised on its own (mean_k, population std_k) and the results are combined
 * with the trade-off vector of the environment:
 *   adv_out[t, n] = sum_k w[g(n), k] (adv_vec[t, n, k] - mean_k) / (std_k + 1e-8).
 * Feed adv_out to morlax_ppo_loss_grad with norm_adv = 0.  All pointers are DEVICE pointers:
 * adv_vec [T, N, K] (as written by morlax_vec_gae), w [P, K], adv_out [T, N] (only the selected cells are
 * written).  rows selects t in [0, T).  Sums in fp64 in a fixed
 * order: results are repeatable.  Errors: NULL arguments, invalid rows. */
int morlax_scalarize_normalized(morlax_ctx* ctx, const morlax_rows* rows, const float* adv_vec,
                                const float* w, float* adv_out, void* ws, int64_t ws_bytes, void* stream);

/* Clipped PPO surrogate and vector value loss with their gradients on one minibatch (Sec. III-C,
 * update phase).  B = selected cells.  Ahat = (adv_s - mean) / (std + 1e-8) over the selection
 * (population std) when norm_adv != 0, else adv_s.  logp = Gaussian log-density of act under
 * (mu, sigma = exp(logsig[g(n)])); rho = exp(logp - logp_old);
 *   L_pi = -(1/B) sum min(rho Ahat, clip(rho, 1-eps, 1+eps) Ahat);  L_V = (1/B) sum ||v - vtarg||^2.
 *   mu, act [T, N, A]; logsig [P, A] with row stride logsig_stride floats (pass the tail of the
 *   actor theta_vec and its row length); logp_old, adv_s [T, N]; v, vtarg [T, N, K]; rows selects
 *   t in [0, T) (the rollout's actions, advantages and targets exist for T steps, not T + 1).
 *   -> dmu [T, N, A], dv [T, N, K] on the selected cells; dlogsig [P, A] (summed over each
 *   preference's selected rows, fixed order); stats [8] fp32 on the device:
 *   L_pi, L_V, fraction with |rho-1| > eps, mean(logp_old - logp), adv mean, adv std, mean rho, B. */
int morlax_ppo_loss_grad(morlax_ctx* ctx, const morlax_rows* rows, const float* mu,
                         const float* logsig, int32_t logsig_stride, const float* act,
                         const float* logp_old, const float* adv_s, const float* v,
                         const float* vtarg, float clip_eps, int32_t norm_adv, float* dmu,
                         float* dlogsig, float* dv, float* stats, void* ws, int64_t ws_bytes, void* stream);

/* morlax_ppo_loss_grad for callers that cannot allocate device memory or hand over a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid allocation.  Same arguments (without ws),
 * same kernels, same results bit for bit; the partial sums live in a static device array inside the
 * library, MORLAX_STATIC_SCRATCH_BYTES bytes on every GPU the library runs on, held until the process
 * ends.  The call allocates and frees nothing.  The partial sums take 8 (5 + act_dim) bytes per block and
 * there are at most about 2048 + P blocks whatever the number of selected cells, so every selection of up to
 * some 10 000 trade-offs fits; one that does not is refused with MORLAX_ERR_WORKSPACE before anything is
 * launched.  All calls on one GPU share that GPU's array: calls that may overlap there (two
 * streams, two threads) race; order them.  Nothing in the array needs to survive or be cleared between
 * calls. */
#define MORLAX_STATIC_SCRATCH_BYTES (2 * 1024 * 1024)
int morlax_ppo_loss_grad_static(morlax_ctx* ctx, const morlax_rows* rows, const float* mu,
                                const float* logsig, int32_t logsig_stride, const float* act,
                                const float* logp_old, const float* adv_s, const float* v,
                                const float* vtarg, float clip_eps, int32_t norm_adv, float* dmu,
                                float* dlogsig, float* dv, float* stats, void* stream);

/* Evaluation side (Fig. 2a: a trade-off is picked, its policy rolled out, and the returns judged).
 * morlax_eval_returns: the return vector of every trade-off from a finished roll-out (Sec. II-A:
 * J = expected discounted return from the initial state): J[p, k] = mean over the n_g environments of
 * group p of sum_t gamma^t r[t, n, k] alive[t, n], alive = 1 up to and including the first done of
 * environment n and 0 after it.  r [T, N, K] fp32, done [T, N] u8 (device); J [P, K] fp32 (device,
 * overwritten).  Sums in fp64, fixed order.  MORLAX_ERR_SHAPE unless 0 < gamma <= 1. */
int morlax_eval_returns(morlax_ctx* ctx, const float* r, const uint8_t* done, float gamma, float* J,
                        void* stream);

/* Pareto front and hypervolume of n return vectors (Sec. II-A: j dominates i when it is at least as
 * good in every objective and differs from it; Sec. II-B: hypervolume = volume of objective space
 * dominated by the set).  The paper names no reference point: ref [K] is an input, and the volume is that
 * of the union of the boxes [ref, J[i]]; a point that is not above ref in every objective adds nothing.
 * The result is exact (no sampling): objectives 2 .. K-1 are cut into slabs at the points' coordinates
 * and every tuple of slabs contributes the area of a two-objective staircase, n^(K-2) tuples in all.
 *   J [n, K] fp32, ref [K] fp32 (device, read); front [n] u8 (device, written: 1 = not dominated by any
 *   other point; equal points do not dominate each other); hv [1] fp64 (device, written);
 *   ws: morlax_hypervolume_workspace_bytes(n, K) bytes of device scratch.
 * Independent of any morlax_ctx (an evaluation may use any number of trade-offs).  Sums in fp64 in a fixed
 * order.  MORLAX_ERR_SHAPE unless 1 <= K <= 8, 1 <= n <= 1024 and n^(K-2) <= 2^32;
 * morlax_hypervolume_workspace_bytes returns -1 for such sizes. */
int64_t morlax_hypervolume_workspace_bytes(int32_t n, int32_t K);
int morlax_pareto_hypervolume(const float* J, const float* ref, int32_t n, int32_t K, uint8_t* front,
                              double* hv, void* ws, int64_t ws_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MORLAX_H */
