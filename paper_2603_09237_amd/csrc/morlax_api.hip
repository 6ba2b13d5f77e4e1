// Host side of the C ABI declared in include/morlax.h: context construction (layouts of the
// hypernet parameter vector and of theta), argument validation (all of it before the first HIP
// call) and dispatch to the kernel launchers.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>

#include "morlax_internal.h"
#include "morlax_bench.h"

static thread_local char g_err[512] = "";

static int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

extern "C" const char* morlax_last_error(void) { return g_err; }

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static void build_net(const morlax_dims& d, int net, NetDev& nd, AffineTable& at) {
    // rank < 0: strictly affine hypernetwork -- every weight has its own row of M (stored where the factor maps
    // of the low-rank form would be) and W0 is its constant term; there are no factors
    const bool affine = d.rank < 0;
    const int64_t F = d.hyper_width, r = affine ? 0 : d.rank, K = d.K;
    // a state-dependent standard deviation doubles the actor's output layer: means, then log sigmas
    const int out = (net == MORLAX_ACTOR) ? (d.sigma_state ? 2 * d.act_dim : d.act_dim) : d.K;
    nd.n_layers = d.n_hidden + 1;
    nd.out_dim = out;
    int64_t hp = 0, mat = 0, vec = 0, fac = 0;
    nd.hp_wh1 = hp; hp += F * K;
    nd.hp_bh1 = hp; hp += F;
    nd.hp_wh2 = hp; hp += F * F;
    nd.hp_bh2 = hp; hp += F;
    for (int l = 0; l < nd.n_layers; ++l) {
        LayerDev& L = nd.layer[l];
        L.d_in = (l == 0) ? d.obs_dim : d.width;
        L.d_out = (l == nd.n_layers - 1) ? out : d.width;
        L.mat_off = mat; mat += (int64_t)L.d_out * L.d_in;
        L.vec_off = vec; vec += L.d_out;
        L.fac_a = fac; fac += (int64_t)L.d_out * r;
        L.fac_b = fac; fac += r * (int64_t)L.d_in;
        L.hp_w0 = hp; hp += (int64_t)L.d_out * L.d_in;
        L.hp_b0 = hp; hp += L.d_out;
        L.hp_ma = hp; hp += affine ? (int64_t)L.d_out * L.d_in * F : (int64_t)L.d_out * r * F;
        L.hp_ca = hp; hp += (int64_t)L.d_out * r;
        L.hp_mb = hp; hp += r * (int64_t)L.d_in * F;
        L.hp_cb = hp; hp += r * (int64_t)L.d_in;
        L.hp_mbias = hp; hp += (int64_t)L.d_out * F;
    }
    nd.hp_logsig0 = nd.hp_msig = -1;
    if (net == MORLAX_ACTOR && !d.sigma_state) {
        nd.hp_logsig0 = hp; hp += d.act_dim;
        nd.hp_msig = hp; hp += (int64_t)d.act_dim * F;
        vec += d.act_dim;
    }
    // stacked affine rows: factor rows first (in factor-vector order), then theta_vec rows
    at.n_seg = 0;
    int32_t q = 0;
    auto seg = [&](int64_t hp_m, int64_t hp_c, int32_t rows) {
        int s = at.n_seg++;
        at.q0[s] = q;
        at.hp_m[s] = hp_m;
        at.hp_c[s] = hp_c;
        q += rows;
        at.q0[s + 1] = q;
    };
    if (affine)
        for (int l = 0; l < nd.n_layers; ++l)  // the rows of theta_mat, in its own order
            seg(nd.layer[l].hp_ma, nd.layer[l].hp_w0, (int32_t)(nd.layer[l].d_out * nd.layer[l].d_in));
    if (r > 0)
        for (int l = 0; l < nd.n_layers; ++l) {
            const LayerDev& L = nd.layer[l];
            seg(L.hp_ma, L.hp_ca, (int32_t)(L.d_out * r));
            seg(L.hp_mb, L.hp_cb, (int32_t)(r * L.d_in));
        }
    for (int l = 0; l < nd.n_layers; ++l) seg(nd.layer[l].hp_mbias, nd.layer[l].hp_b0, nd.layer[l].d_out);
    if (net == MORLAX_ACTOR && !d.sigma_state) seg(nd.hp_msig, nd.hp_logsig0, d.act_dim);
    at.q_total = q;
    nd.mat_len = mat;
    nd.vec_len = vec;
    nd.fac_len = affine ? mat : fac;  // the leading rows of the stacked map: factor vector, or theta_mat itself
    nd.hp_count = hp;
}

extern "C" int morlax_create(const morlax_dims* dims, morlax_ctx** out) {
    if (!dims || !out) return fail(MORLAX_ERR_NULL, "morlax_create: NULL argument");
    *out = nullptr;
    const morlax_dims& d = *dims;
    if (d.K < 1 || d.T < 1 || d.N < 1 || d.obs_dim < 1 || d.act_dim < 1 || d.n_hidden < 1 ||
        d.width < 1 || d.rank < -1 || d.hyper_width < 1)
        return fail(MORLAX_ERR_SHAPE, "morlax_create: K, T, N, obs_dim, act_dim, n_hidden, width, hyper_width must be >= 1 and rank >= -1");
    if (d.P < 2) return fail(MORLAX_ERR_SHAPE, "morlax_create: need P > 1 trade-off vectors (got %d)", d.P);
    if (d.N % d.P != 0)
        return fail(MORLAX_ERR_SHAPE, "morlax_create: P = %d must divide N = %d", d.P, d.N);
    // several launches carry the preference in gridDim.y or gridDim.z
    if (d.P > 65535) return fail(MORLAX_ERR_UNSUPPORTED, "morlax_create: P must be <= 65535 (got %d)", d.P);
    if (d.K > MORLAX_MAX_OUT || d.act_dim > MORLAX_MAX_OUT)
        return fail(MORLAX_ERR_UNSUPPORTED, "morlax_create: K and act_dim must be <= %d", MORLAX_MAX_OUT);
    if (d.sigma_state != 0 && d.sigma_state != 1)
        return fail(MORLAX_ERR_UNSUPPORTED, "morlax_create: sigma_state must be 0 or 1");
    if (d.sigma_state && 2 * d.act_dim > MORLAX_MAX_OUT)
        return fail(MORLAX_ERR_UNSUPPORTED, "morlax_create: a state-dependent sigma needs 2 * act_dim <= %d", MORLAX_MAX_OUT);
    if (d.obs_dim > 1024) return fail(MORLAX_ERR_UNSUPPORTED, "morlax_create: obs_dim must be <= 1024");
    if (d.n_hidden > MORLAX_MAX_LAYERS - 1)
        return fail(MORLAX_ERR_UNSUPPORTED, "morlax_create: n_hidden must be <= %d", MORLAX_MAX_LAYERS - 1);
    if (d.width % 16 != 0 || d.width < 16 || d.width > 2048)
        return fail(MORLAX_ERR_UNSUPPORTED, "morlax_create: width must be a multiple of 16 in [16, 2048]");
    if (d.rank > MORLAX_MAX_RANK)
        return fail(MORLAX_ERR_UNSUPPORTED, "morlax_create: rank must be <= %d", MORLAX_MAX_RANK);
    if (d.hyper_width > MORLAX_MAX_F)
        return fail(MORLAX_ERR_UNSUPPORTED, "morlax_create: hyper_width must be <= %d", MORLAX_MAX_F);
    if (d.act != 0 && d.act != 1) return fail(MORLAX_ERR_UNSUPPORTED, "morlax_create: act must be 0 (tanh) or 1 (SiLU)");
    if (d.wdtype != 0 && d.wdtype != 1)
        return fail(MORLAX_ERR_UNSUPPORTED, "morlax_create: wdtype must be 0 (fp32) or 1 (bf16)");
    if (d.mean_tanh != 0 && d.mean_tanh != 1)
        return fail(MORLAX_ERR_UNSUPPORTED, "morlax_create: mean_tanh must be 0 or 1");
    if ((int64_t)(d.T + 1) * d.N >= (int64_t)1 << 31)
        return fail(MORLAX_ERR_UNSUPPORTED, "morlax_create: (T+1) * N must stay below 2^31");
    // the GEMM kernels address an operand with 32-bit byte offsets from a per-preference (activations) or
    // whole-tensor (observations) base
    if ((int64_t)(d.T + 1) * d.N * d.obs_dim * 4 >= (int64_t)1 << 32)
        return fail(MORLAX_ERR_UNSUPPORTED, "morlax_create: the observation tensor (T+1) * N * obs_dim must stay below 4 GiB");
    if ((int64_t)(d.T + 1) * (d.N / d.P) * d.width * 4 >= (int64_t)1 << 31)
        return fail(MORLAX_ERR_UNSUPPORTED,
                    "morlax_create: one preference's activations (T+1) * (N/P) * width must stay below 2 GiB");
    morlax_ctx* c = new (std::nothrow) morlax_ctx;
    if (!c) return fail(MORLAX_ERR_HIP, "morlax_create: out of host memory");
    memset(c, 0, sizeof(*c));
    c->d = d;
    c->n_g = d.N / d.P;
    build_net(d, MORLAX_ACTOR, c->net[0], c->aff[0]);
    build_net(d, MORLAX_CRITIC, c->net[1], c->aff[1]);
    if (c->net[0].hp_count >= ((int64_t)1 << 31) || c->net[1].hp_count >= ((int64_t)1 << 31)) {
        delete c;  // rows of the stacked affine matrix are addressed with 32-bit offsets into hparams
        return fail(MORLAX_ERR_UNSUPPORTED, "morlax_create: a hypernetwork with 2^31 or more parameters");
    }
    *out = c;
    return MORLAX_OK;
}

extern "C" void morlax_destroy(morlax_ctx* ctx) {
    if (!ctx) return;
    prof_free(ctx);
    delete ctx;
}

extern "C" int morlax_profile_begin(morlax_ctx* ctx) {
    if (!ctx) return fail(MORLAX_ERR_NULL, "morlax_profile_begin: ctx is NULL");
    if (prof_begin(ctx) != 0) return fail(MORLAX_ERR_HIP, "morlax_profile_begin: event creation failed");
    return MORLAX_OK;
}

extern "C" int morlax_profile_end(morlax_ctx* ctx, double* ms, int64_t* launches, double* flops) {
    if (!ctx || !ms || !launches || !flops) return fail(MORLAX_ERR_NULL, "morlax_profile_end: NULL argument");
    if (!ctx->prof) return fail(MORLAX_ERR_SHAPE, "morlax_profile_end: profiling was not started");
    if (prof_end(ctx, ms, launches, flops) != 0) return fail(MORLAX_ERR_HIP, "morlax_profile_end: event query failed");
    return MORLAX_OK;
}

static bool bad_net(int net) { return net != MORLAX_ACTOR && net != MORLAX_CRITIC; }

extern "C" int64_t morlax_hparam_count(const morlax_ctx* c, int net) {
    return (!c || bad_net(net)) ? -1 : c->net[net].hp_count;
}
extern "C" int64_t morlax_theta_mat_len(const morlax_ctx* c, int net) {
    return (!c || bad_net(net)) ? -1 : c->net[net].mat_len;
}
extern "C" int64_t morlax_theta_vec_len(const morlax_ctx* c, int net) {
    return (!c || bad_net(net)) ? -1 : c->net[net].vec_len;
}

// rows == NULL: the largest selection (all environments of a group, T+1 times).
static int resolve_rows(const morlax_ctx* c, const morlax_rows* rows, int t_max, RowSel& rs, const char* who) {
    if (!rows) {
        rs.t0 = 0; rs.t_cnt = t_max; rs.j0 = 0; rs.j_cnt = c->n_g;
    } else {
        rs.t0 = rows->t0; rs.t_cnt = rows->t_cnt; rs.j0 = rows->j0; rs.j_cnt = rows->j_cnt;
    }
    if (rs.t0 < 0 || rs.t_cnt < 1 || rs.t0 + (int64_t)rs.t_cnt > t_max)
        return fail(MORLAX_ERR_SHAPE, "%s: time slice [%d, %d+%d) outside [0, %d)", who, rs.t0, rs.t0, rs.t_cnt, t_max);
    if (rs.j0 < 0 || rs.j_cnt < 1 || rs.j0 + (int64_t)rs.j_cnt > c->n_g)
        return fail(MORLAX_ERR_SHAPE, "%s: group slice [%d, %d+%d) outside [0, n_g = %d)", who, rs.j0, rs.j0, rs.j_cnt, c->n_g);
    rs.M = rs.t_cnt * rs.j_cnt;
    return MORLAX_OK;
}

extern "C" int64_t morlax_saved_bytes(const morlax_ctx* c, int net, const morlax_rows* rows) {
    if (!c || bad_net(net)) return -1;
    RowSel rs;
    if (resolve_rows(c, rows, c->d.T + 1, rs, "morlax_saved_bytes") != MORLAX_OK) return -1;
    return mlp_saved_bytes(c, net, rs);
}

extern "C" int64_t morlax_workspace_bytes(const morlax_ctx* c, const morlax_rows* rows) {
    if (!c) return -1;
    RowSel rs;
    if (resolve_rows(c, rows, c->d.T + 1, rs, "morlax_workspace_bytes") != MORLAX_OK) return -1;
    int64_t b = hyper_ws_bytes(c);
    int64_t m = mlp_ws_bytes(c, rs);
    int64_t l = loss_ws_bytes(c, rs);
    int64_t n = advnorm_ws_bytes(c, rs);
    if (m > b) b = m;
    if (l > b) b = l;
    if (n > b) b = n;
    return b;
}

static int finish(const char* who) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(MORLAX_ERR_HIP, "%s: %s", who, hipGetErrorString(e));
    return MORLAX_OK;
}

#define REQ(ptr, who)                                                                   \
    do {                                                                                \
        if (!(ptr)) return fail(MORLAX_ERR_NULL, "%s: %s is NULL", who, #ptr);          \
        if (!aligned16(ptr)) return fail(MORLAX_ERR_SHAPE, "%s: %s is not 16-byte aligned", who, #ptr); \
    } while (0)
#define OPT(ptr, who)                                                                   \
    do {                                                                                \
        if ((ptr) && !aligned16(ptr)) return fail(MORLAX_ERR_SHAPE, "%s: %s is not 16-byte aligned", who, #ptr); \
    } while (0)

// caller-provided scratch: present, aligned and at least `need` bytes
#define WS(ptr, bytes, need, who)                                                                        \
    do {                                                                                                 \
        REQ(ptr, who);                                                                                   \
        if ((int64_t)(bytes) < (int64_t)(need))                                                          \
            return fail(MORLAX_ERR_WORKSPACE, "%s: workspace of %lld bytes, %lld needed", who,           \
                        (long long)(bytes), (long long)(need));                                          \
    } while (0)

extern "C" int morlax_env_pref_index(const morlax_ctx* ctx, int32_t* out, void* stream) {
    const char* who = "morlax_env_pref_index";
    if (!ctx) return fail(MORLAX_ERR_NULL, "%s: ctx is NULL", who);
    REQ(out, who);
    launch_env_pref_index(ctx, out, (hipStream_t)stream);
    return finish(who);
}

extern "C" int morlax_hypernet_fwd(morlax_ctx* ctx, int net, const float* hparams, const float* w,
                                   void* theta_mat, float* theta_vec, void* ws, int64_t ws_bytes, void* stream) {
    const char* who = "morlax_hypernet_fwd";
    if (!ctx) return fail(MORLAX_ERR_NULL, "%s: ctx is NULL", who);
    if (bad_net(net)) return fail(MORLAX_ERR_SHAPE, "%s: net must be 0 (actor) or 1 (critic)", who);
    REQ(hparams, who); REQ(w, who); REQ(theta_mat, who); REQ(theta_vec, who);
    WS(ws, ws_bytes, hyper_ws_bytes(ctx), who);
    launch_hypernet_fwd(ctx, net, hparams, w, theta_mat, theta_vec, ws, (hipStream_t)stream);
    return finish(who);
}

extern "C" int morlax_hypernet_bwd(morlax_ctx* ctx, int net, const float* hparams, const float* w,
                                   const float* dtheta_mat, const float* dtheta_vec, float* dhparams,
                                   void* ws, int64_t ws_bytes, void* stream) {
    const char* who = "morlax_hypernet_bwd";
    if (!ctx) return fail(MORLAX_ERR_NULL, "%s: ctx is NULL", who);
    if (bad_net(net)) return fail(MORLAX_ERR_SHAPE, "%s: net must be 0 (actor) or 1 (critic)", who);
    REQ(hparams, who); REQ(w, who); REQ(dtheta_mat, who); REQ(dtheta_vec, who); REQ(dhparams, who);
    WS(ws, ws_bytes, hyper_ws_bytes(ctx), who);
    launch_hypernet_bwd(ctx, net, hparams, w, dtheta_mat, dtheta_vec, dhparams, ws, false, (hipStream_t)stream);
    return finish(who);
}

extern "C" int morlax_hypernet_bwd_kept(morlax_ctx* ctx, int net, const float* hparams, const float* w,
                                        const float* dtheta_mat, const float* dtheta_vec, float* dhparams,
                                        void* ws_fwd, int64_t ws_bytes, void* stream) {
    const char* who = "morlax_hypernet_bwd_kept";
    if (!ctx) return fail(MORLAX_ERR_NULL, "%s: ctx is NULL", who);
    if (bad_net(net)) return fail(MORLAX_ERR_SHAPE, "%s: net must be 0 (actor) or 1 (critic)", who);
    REQ(hparams, who); REQ(w, who); REQ(dtheta_mat, who); REQ(dtheta_vec, who); REQ(dhparams, who);
    WS(ws_fwd, ws_bytes, hyper_ws_bytes(ctx), who);
    launch_hypernet_bwd(ctx, net, hparams, w, dtheta_mat, dtheta_vec, dhparams, ws_fwd, true, (hipStream_t)stream);
    return finish(who);
}

extern "C" int morlax_policy_fwd(morlax_ctx* ctx, int net, const void* theta_mat, const float* theta_vec,
                                 const float* x, const morlax_rows* rows, float* out, const float* eps,
                                 float* act, float* logp, void* saved, void* ws, int64_t ws_bytes, void* stream) {
    const char* who = "morlax_policy_fwd";
    if (!ctx) return fail(MORLAX_ERR_NULL, "%s: ctx is NULL", who);
    if (bad_net(net)) return fail(MORLAX_ERR_SHAPE, "%s: net must be 0 (actor) or 1 (critic)", who);
    REQ(theta_mat, who); REQ(theta_vec, who); REQ(x, who); REQ(out, who);
    OPT(eps, who); OPT(act, who); OPT(logp, who); OPT(saved, who);
    if (!rows) return fail(MORLAX_ERR_NULL, "%s: rows is NULL", who);
    const bool any = eps || act || logp, all = eps && act && logp;
    if (any && !all) return fail(MORLAX_ERR_NULL, "%s: eps, act and logp must be given together", who);
    if (any && net != MORLAX_ACTOR) return fail(MORLAX_ERR_SHAPE, "%s: sampling outputs are actor-only", who);
    RowSel rs;
    int rc = resolve_rows(ctx, rows, ctx->d.T + 1, rs, who);
    if (rc != MORLAX_OK) return rc;
    WS(ws, ws_bytes, mlp_ws_bytes(ctx, rs), who);
    launch_policy_fwd(ctx, net, theta_mat, theta_vec, x, rs, out, eps, act, logp, saved, ws, (hipStream_t)stream);
    return finish(who);
}

extern "C" int morlax_policy_bwd(morlax_ctx* ctx, int net, const void* theta_mat, const float* theta_vec,
                                 const float* x, const morlax_rows* rows, const void* saved,
                                 const float* dout, const float* dlogsig, float* dtheta_mat,
                                 float* dtheta_vec, void* ws, int64_t ws_bytes, void* stream) {
    const char* who = "morlax_policy_bwd";
    if (!ctx) return fail(MORLAX_ERR_NULL, "%s: ctx is NULL", who);
    if (bad_net(net)) return fail(MORLAX_ERR_SHAPE, "%s: net must be 0 (actor) or 1 (critic)", who);
    REQ(theta_mat, who); REQ(theta_vec, who); REQ(x, who); REQ(saved, who); REQ(dout, who);
    REQ(dtheta_mat, who); REQ(dtheta_vec, who);
    OPT(dlogsig, who);
    if (!rows) return fail(MORLAX_ERR_NULL, "%s: rows is NULL", who);
    if (dlogsig && net != MORLAX_ACTOR) return fail(MORLAX_ERR_SHAPE, "%s: dlogsig is actor-only", who);
    if (dlogsig && ctx->d.sigma_state)
        return fail(MORLAX_ERR_SHAPE, "%s: with a state-dependent sigma the log-sigma gradient is part of dout", who);
    RowSel rs;
    int rc = resolve_rows(ctx, rows, ctx->d.T + 1, rs, who);
    if (rc != MORLAX_OK) return rc;
    WS(ws, ws_bytes, mlp_ws_bytes(ctx, rs), who);
    launch_policy_bwd(ctx, net, theta_mat, theta_vec, x, rs, saved, dout, dlogsig, dtheta_mat, dtheta_vec,
                      ws, (hipStream_t)stream);
    return finish(who);
}

extern "C" int morlax_vec_gae(morlax_ctx* ctx, const float* r, const float* v, const uint8_t* done,
                              const float* w, float gamma, float lambda, float* adv_vec, float* vtarg,
                              float* adv_s, void* stream) {
    const char* who = "morlax_vec_gae";
    if (!ctx) return fail(MORLAX_ERR_NULL, "%s: ctx is NULL", who);
    REQ(r, who); REQ(v, who); REQ(done, who); REQ(w, who); REQ(vtarg, who); REQ(adv_s, who);
    OPT(adv_vec, who);
    if (!(gamma >= 0.f && gamma <= 1.f) || !(lambda >= 0.f && lambda <= 1.f))
        return fail(MORLAX_ERR_SHAPE, "%s: gamma and lambda must lie in [0, 1]", who);
    launch_vec_gae(ctx, r, v, done, nullptr, w, gamma, lambda, adv_vec, vtarg, adv_s, (hipStream_t)stream);
    return finish(who);
}

extern "C" int morlax_vec_gae_trunc(morlax_ctx* ctx, const float* r, const float* v, const uint8_t* done,
                                    const uint8_t* trunc, const float* w, float gamma, float lambda,
                                    float* adv_vec, float* vtarg, float* adv_s, void* stream) {
    const char* who = "morlax_vec_gae_trunc";
    if (!ctx) return fail(MORLAX_ERR_NULL, "%s: ctx is NULL", who);
    REQ(r, who); REQ(v, who); REQ(done, who); REQ(trunc, who); REQ(w, who); REQ(vtarg, who); REQ(adv_s, who);
    OPT(adv_vec, who);
    if (!(gamma >= 0.f && gamma <= 1.f) || !(lambda >= 0.f && lambda <= 1.f))
        return fail(MORLAX_ERR_SHAPE, "%s: gamma and lambda must lie in [0, 1]", who);
    launch_vec_gae(ctx, r, v, done, trunc, w, gamma, lambda, adv_vec, vtarg, adv_s, (hipStream_t)stream);
    return finish(who);
}

extern "C" int morlax_sample_preferences(morlax_ctx* ctx, const float* u, int32_t kappa, float* w, void* stream) {
    const char* who = "morlax_sample_preferences";
    if (!ctx) return fail(MORLAX_ERR_NULL, "%s: ctx is NULL", who);
    REQ(u, who); REQ(w, who);
    const int lim = ctx->d.P < ctx->d.K ? ctx->d.P : ctx->d.K;
    if (kappa < 0 || kappa > lim) return fail(MORLAX_ERR_SHAPE, "%s: kappa must lie in [0, min(P, K)]", who);
    launch_sample_preferences(ctx, u, kappa, w, (hipStream_t)stream);
    return finish(who);
}

extern "C" int morlax_eval_returns(morlax_ctx* ctx, const float* r, const uint8_t* done, float gamma, float* J,
                                   void* stream) {
    const char* who = "morlax_eval_returns";
    if (!ctx) return fail(MORLAX_ERR_NULL, "%s: ctx is NULL", who);
    REQ(r, who); REQ(done, who); REQ(J, who);
    if (!(gamma > 0.f && gamma <= 1.f)) return fail(MORLAX_ERR_SHAPE, "%s: gamma must lie in (0, 1]", who);
    launch_eval_returns(ctx, r, done, gamma, J, (hipStream_t)stream);
    return finish(who);
}

static bool hv_sizes_ok(int32_t n, int32_t K) {
    return K >= 1 && K <= 8 && n >= 1 && n <= 1024 && hv_tuples(n, K) <= (uint64_t(1) << 32);
}

extern "C" int64_t morlax_hypervolume_workspace_bytes(int32_t n, int32_t K) {
    return hv_sizes_ok(n, K) ? hv_ws_bytes(n, K) : -1;
}

extern "C" int morlax_pareto_hypervolume(const float* J, const float* ref, int32_t n, int32_t K, uint8_t* front,
                                         double* hv, void* ws, int64_t ws_bytes, void* stream) {
    const char* who = "morlax_pareto_hypervolume";
    REQ(J, who); REQ(ref, who); REQ(front, who); REQ(hv, who);
    if (!hv_sizes_ok(n, K))
        return fail(MORLAX_ERR_SHAPE, "%s: needs 1 <= K <= 8, 1 <= n <= 1024 and n^(K-2) <= 2^32 (n = %d, K = %d)", who,
                    (int)n, (int)K);
    WS(ws, ws_bytes, hv_ws_bytes(n, K), who);
    launch_pareto_hypervolume(J, ref, n, K, front, hv, ws, (hipStream_t)stream);
    return finish(who);
}

extern "C" int morlax_adam_step(morlax_ctx* ctx, int net, float* hparams, const float* dhparams, float* m, float* v,
                                float lr, float beta1, float beta2, float eps, int32_t step, void* stream) {
    const char* who = "morlax_adam_step";
    if (!ctx) return fail(MORLAX_ERR_NULL, "%s: ctx is NULL", who);
    if (bad_net(net)) return fail(MORLAX_ERR_SHAPE, "%s: net must be 0 (actor) or 1 (critic)", who);
    REQ(hparams, who); REQ(dhparams, who); REQ(m, who); REQ(v, who);
    if (step < 1) return fail(MORLAX_ERR_SHAPE, "%s: step counts from 1", who);
    if (!(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f))
        return fail(MORLAX_ERR_SHAPE, "%s: beta1 and beta2 must lie in [0, 1)", who);
    if (!(eps > 0.f) || !(lr >= 0.f)) return fail(MORLAX_ERR_SHAPE, "%s: eps must be positive and lr non-negative", who);
    const double c1 = 1.0 / (1.0 - std::pow((double)beta1, (double)step));
    const double c2 = 1.0 / (1.0 - std::pow((double)beta2, (double)step));
    launch_adam_step(hparams, dhparams, m, v, morlax_hparam_count(ctx, net), lr, beta1, beta2, eps, (float)c1,
                     (float)c2, (hipStream_t)stream);
    return finish(who);
}

extern "C" int morlax_scalarize_normalized(morlax_ctx* ctx, const morlax_rows* rows, const float* adv_vec,
                                           const float* w, float* adv_out, void* ws, int64_t ws_bytes,
                                           void* stream) {
    const char* who = "morlax_scalarize_normalized";
    if (!ctx) return fail(MORLAX_ERR_NULL, "%s: ctx is NULL", who);
    if (!rows) return fail(MORLAX_ERR_NULL, "%s: rows is NULL", who);
    REQ(adv_vec, who); REQ(w, who); REQ(adv_out, who);
    RowSel rs;
    int rc = resolve_rows(ctx, rows, ctx->d.T, rs, who);
    if (rc != MORLAX_OK) return rc;
    WS(ws, ws_bytes, advnorm_ws_bytes(ctx, rs), who);
    launch_scalarize_normalized(ctx, rs, adv_vec, w, adv_out, ws, (hipStream_t)stream);
    return finish(who);
}

// argument checks shared by the two forms of the loss call
static int check_loss_args(morlax_ctx* ctx, const morlax_rows* rows, const float* mu, const float* logsig,
                           int32_t logsig_stride, const float* act, const float* logp_old, const float* adv_s,
                           const float* v, const float* vtarg, float clip_eps, float* dmu, float* dlogsig, float* dv,
                           float* stats, RowSel& rs, const char* who) {
    if (!ctx) return fail(MORLAX_ERR_NULL, "%s: ctx is NULL", who);
    if (!rows) return fail(MORLAX_ERR_NULL, "%s: rows is NULL", who);
    REQ(mu, who); REQ(act, who); REQ(logp_old, who); REQ(adv_s, who); REQ(v, who);
    REQ(vtarg, who); REQ(dmu, who); REQ(dv, who); REQ(stats, who);
    if (ctx->d.sigma_state) {  // log sigma and its gradient travel inside mu / dmu (2 * act_dim columns)
        OPT(logsig, who); OPT(dlogsig, who);
    } else {
        REQ(dlogsig, who);
        if (!logsig) return fail(MORLAX_ERR_NULL, "%s: logsig is NULL", who);
        if ((reinterpret_cast<uintptr_t>(logsig) & 3u) != 0)
            return fail(MORLAX_ERR_SHAPE, "%s: logsig is not 4-byte aligned", who);
        if (logsig_stride < ctx->d.act_dim)
            return fail(MORLAX_ERR_SHAPE, "%s: logsig_stride %d < act_dim %d", who, logsig_stride, ctx->d.act_dim);
    }
    if (!(clip_eps >= 0.f)) return fail(MORLAX_ERR_SHAPE, "%s: clip_eps must be >= 0", who);
    // the advantages, targets and actions exist for t < T only
    return resolve_rows(ctx, rows, ctx->d.T, rs, who);
}

extern "C" int morlax_ppo_loss_grad(morlax_ctx* ctx, const morlax_rows* rows, const float* mu,
                                    const float* logsig, int32_t logsig_stride, const float* act,
                                    const float* logp_old, const float* adv_s, const float* v,
                                    const float* vtarg, float clip_eps, int32_t norm_adv, float* dmu,
                                    float* dlogsig, float* dv, float* stats, void* ws, int64_t ws_bytes,
                                    void* stream) {
    const char* who = "morlax_ppo_loss_grad";
    RowSel rs;
    int rc = check_loss_args(ctx, rows, mu, logsig, logsig_stride, act, logp_old, adv_s, v, vtarg, clip_eps, dmu,
                             dlogsig, dv, stats, rs, who);
    if (rc != MORLAX_OK) return rc;
    WS(ws, ws_bytes, loss_ws_bytes(ctx, rs), who);
    launch_ppo_loss_grad(ctx, rs, mu, logsig, logsig_stride, act, logp_old, adv_s, v, vtarg, clip_eps,
                         norm_adv, dmu, dlogsig, dv, stats, ws, (hipStream_t)stream);
    return finish(who);
}

extern "C" int morlax_ppo_loss_grad_static(morlax_ctx* ctx, const morlax_rows* rows, const float* mu,
                                           const float* logsig, int32_t logsig_stride, const float* act,
                                           const float* logp_old, const float* adv_s, const float* v,
                                           const float* vtarg, float clip_eps, int32_t norm_adv, float* dmu,
                                           float* dlogsig, float* dv, float* stats, void* stream) {
    const char* who = "morlax_ppo_loss_grad_static";
    RowSel rs;
    int rc = check_loss_args(ctx, rows, mu, logsig, logsig_stride, act, logp_old, adv_s, v, vtarg, clip_eps, dmu,
                             dlogsig, dv, stats, rs, who);
    if (rc != MORLAX_OK) return rc;
    const int64_t need = loss_ws_bytes(ctx, rs);
    if (need > (int64_t)MORLAX_STATIC_SCRATCH_BYTES)
        return fail(MORLAX_ERR_WORKSPACE,
                    "%s: this selection needs %lld bytes of scratch, the library's static array holds %lld; "
                    "use morlax_ppo_loss_grad with a workspace", who, (long long)need,
                    (long long)MORLAX_STATIC_SCRATCH_BYTES);
    void* ws = nullptr;
    if (loss_static_scratch(&ws) != 0)
        return fail(MORLAX_ERR_HIP, "%s: the address of the static scratch array is not available on this device", who);
    launch_ppo_loss_grad(ctx, rs, mu, logsig, logsig_stride, act, logp_old, adv_s, v, vtarg, clip_eps,
                         norm_adv, dmu, dlogsig, dv, stats, ws, (hipStream_t)stream);
    return finish(who);
}
