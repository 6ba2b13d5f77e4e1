// Internal declarations shared by the translation units of libmorlax.so (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "morlax.h"

#define MORLAX_MAX_LAYERS 9   // n_hidden <= 8 -> at most 9 dense layers
#define MORLAX_MAX_OUT 16     // act_dim, K <= 16
#define MORLAX_MAX_F 64
#define MORLAX_MAX_RANK 32

// One dense layer of a target network and where its pieces live.
struct LayerDev {
    int32_t d_out, d_in;
    int64_t mat_off;  // offset of W_l inside one preference's theta_mat
    int64_t vec_off;  // offset of b_l inside one preference's theta_vec
    int64_t fac_a;    // offset of A_l [d_out, r] inside one preference's factor vector
    int64_t fac_b;    // offset of B_l [r, d_in]
    int64_t hp_w0, hp_b0, hp_ma, hp_ca, hp_mb, hp_cb, hp_mbias;  // offsets into hparams
};

// Rows q of the stacked affine map  out[p, q] = c[q] + sum_j M[q, j] f[p, j].
// Rows [0, fac_len) are the factor vector of a preference (A_0, B_0, A_1, B_1, ... in the order of
// LayerDev::fac_a / fac_b); rows [fac_len, fac_len + vec_len) are theta_vec (biases, then log sigma).
// Segment s covers rows [q0[s], q0[s+1]); row q of it reads M at hp_m[s] + (q - q0[s]) * F and c at
// hp_c[s] + (q - q0[s]) in the hypernet parameter vector.
#define MORLAX_MAX_SEG (3 * MORLAX_MAX_LAYERS + 1)
struct AffineTable {
    int32_t n_seg;
    int32_t q_total;
    int32_t q0[MORLAX_MAX_SEG + 1];
    int64_t hp_m[MORLAX_MAX_SEG];
    int64_t hp_c[MORLAX_MAX_SEG];
};

struct NetDev {
    int32_t n_layers, out_dim;
    int64_t mat_len, vec_len, fac_len, hp_count;
    int64_t hp_wh1, hp_bh1, hp_wh2, hp_bh2, hp_logsig0, hp_msig;
    LayerDev layer[MORLAX_MAX_LAYERS];
};

struct GemmProf;  // event pairs around grouped-GEMM launches (kernels_mlp.hip)

struct morlax_ctx {
    morlax_dims d;
    int32_t n_g;
    NetDev net[2];
    AffineTable aff[2];
    GemmProf* prof;  // NULL unless morlax_profile_begin() was called
};

#define MORLAX_GEMM_KINDS 6  // fwd first layer, fwd hidden, dX hidden, dW hidden, dW first layer, fused fwd
int prof_begin(morlax_ctx* c);
int prof_end(morlax_ctx* c, double* ms, int64_t* launches, double* flops);
void prof_free(morlax_ctx* c);

struct RowSel {  // a validated morlax_rows plus derived sizes
    int32_t t0, t_cnt, j0, j_cnt;
    int32_t M;  // rows per preference = t_cnt * j_cnt
};

// ---- launchers (each only enqueues kernels on `s`) ------------------------------------------
void launch_env_pref_index(const morlax_ctx* c, int32_t* out, hipStream_t s);

void launch_vec_gae(const morlax_ctx* c, const float* r, const float* v, const uint8_t* done,
                    const uint8_t* trunc, const float* w, float gamma, float lambda, float* adv_vec,
                    float* vtarg, float* adv_s, hipStream_t s);
void launch_sample_preferences(const morlax_ctx* c, const float* u, int kappa, float* w, hipStream_t s);
void launch_adam_step(float* theta, const float* g, float* m, float* v, int64_t n, float lr, float b1, float b2,
                      float eps, float c1, float c2, hipStream_t s);

int64_t loss_ws_bytes(const morlax_ctx* c, const RowSel& rs);
void launch_ppo_loss_grad(const morlax_ctx* c, const RowSel& rs, const float* mu, const float* logsig,
                          int logsig_stride, const float* act, const float* logp_old,
                          const float* adv_s, const float* v, const float* vtarg, float clip_eps,
                          int norm_adv, float* dmu, float* dlogsig, float* dv, float* stats,
                          void* ws, hipStream_t s);

// device address of this GPU's copy of the library's static scratch array (MORLAX_STATIC_SCRATCH_BYTES bytes);
// 0 on success.  Allocates nothing.
int loss_static_scratch(void** ptr);

int64_t advnorm_ws_bytes(const morlax_ctx* c, const RowSel& rs);
void launch_scalarize_normalized(const morlax_ctx* c, const RowSel& rs, const float* adv_vec, const float* w,
                                 float* adv_out, void* ws, hipStream_t s);

int64_t hyper_ws_bytes(const morlax_ctx* c);
void launch_hypernet_fwd(const morlax_ctx* c, int net, const float* hparams, const float* w,
                         void* theta_mat, float* theta_vec, void* ws, hipStream_t s);
void launch_hypernet_bwd(const morlax_ctx* c, int net, const float* hparams, const float* w,
                         const float* dtheta_mat, const float* dtheta_vec, float* dhparams,
                         void* ws, bool kept, hipStream_t s);

int64_t mlp_saved_bytes(const morlax_ctx* c, int net, const RowSel& rs);
int64_t mlp_ws_bytes(const morlax_ctx* c, const RowSel& rs);
void launch_policy_fwd(const morlax_ctx* c, int net, const void* theta_mat, const float* theta_vec,
                       const float* x, const RowSel& rs, float* out, const float* eps, float* act,
                       float* logp, void* saved, void* ws, hipStream_t s);
void launch_policy_bwd(const morlax_ctx* c, int net, const void* theta_mat, const float* theta_vec,
                       const float* x, const RowSel& rs, const void* saved, const float* dout,
                       const float* dlogsig, float* dtheta_mat, float* dtheta_vec, void* ws,
                       hipStream_t s);

void launch_eval_returns(const morlax_ctx* c, const float* r, const uint8_t* done, float gamma, float* J,
                         hipStream_t s);
int64_t hv_ws_bytes(int n, int K);
uint64_t hv_tuples(int n, int K);
void launch_pareto_hypervolume(const float* J, const float* ref, int n, int K, uint8_t* front, double* hv, void* ws,
                               hipStream_t s);

static inline int64_t align_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }
