// Bandwidth-bound kernels of the update phase (paper Sec. III-C): the environment -> trade-off
// index map, the reverse-time vector GAE scan with scalarisation, the advantage statistics and the
// clipped-PPO / value loss with its gradients.  All reductions are two-stage and fixed-order.
#include "morlax_internal.h"

#define WAVE 64

// ------------------------------------------------------------------------------------------------
// g(n) = n / n_g  (Sec. III-C, sampling phase: contiguous blocks of N/P repeated trade-offs)
__global__ void k_env_pref_index(int32_t* __restrict__ out, int N, int n_g) {
    int n = blockIdx.x * blockDim.x + threadIdx.x;
    if (n < N) out[n] = n / n_g;
}

void launch_env_pref_index(const morlax_ctx* c, int32_t* out, hipStream_t s) {
    int N = c->d.N;
    k_env_pref_index<<<(N + 255) / 256, 256, 0, s>>>(out, N, c->n_g);
}

// ------------------------------------------------------------------------------------------------
// Vector GAE (Sec. III-C, update phase: the estimator applied to every objective on its own, then
// scalarised).  One lane per (environment, objective): a wave holds G = 64 / K environments with their
// K objectives in adjacent lanes, so every load of r[t] and v[t] is one contiguous run of G*K floats and
// the scalarisation sum_k w_k A_k is a K-lane shuffle reduction.
//
// The recursion over t, A_t = cut_t ? a_t : a_t + gl A_{t+1} (a_t = r_t - V_t at an episode end, else the
// TD error; cut_t = episode end or time limit), is a chain of affine maps, so the time axis is split as
// well: the four waves of a workgroup take four consecutive chunks of up to GAE_CH steps of the same
// lanes.  A wave requests all loads of its chunk at once, runs the recursion from zero (A'_t), and posts
// the value at its first step and whether its chunk holds a cut.  After a barrier it folds the posts of
// the later chunks into the advantage that enters its own chunk, x, and finishes
// A_t = (a cut between t and the chunk's end) ? A'_t : A'_t + gl^(steps to the chunk's end) x.
// Cuts stay selects throughout, so nothing behind an episode end -- NaN and Inf included -- reaches the
// steps before it.  Horizons above 4 * GAE_CH are walked in groups of four chunks, last group first.
template <int GAE_CH, int NW, int OCC>
__global__ __launch_bounds__(64 * NW, OCC) void k_vec_gae(const float* __restrict__ r, const float* __restrict__ v,
                                                const uint8_t* __restrict__ done,
                                                const uint8_t* __restrict__ trunc, const float* __restrict__ w,
                                                float gamma, float gl, float* __restrict__ adv_vec,
                                                float* __restrict__ vtarg, float* __restrict__ adv_s,
                                                int T, int N, int K, int n_g, int ch) {
    __shared__ float post_a[2][NW][WAVE];
    __shared__ uint8_t post_cut[2][NW][WAVE];
    __shared__ float carry[2][WAVE];
    // cw: chunk within the group; made visibly wave-uniform so that the step offsets stay in scalar registers
    const int lane = threadIdx.x & (WAVE - 1), cw = __builtin_amdgcn_readfirstlane(threadIdx.x / WAVE);
    const int G = WAVE / K;
    const int e = lane / K, k = lane - e * K;
    const int n = blockIdx.x * G + e;
    const bool live = (e < G) && (n < N);
    const int64_t NK = (int64_t)N * K;
    const int64_t idx = (int64_t)n * K + k;
    const float wk = live ? w[(n / n_g) * K + k] : 0.f;
    float gl_ch = 1.f;  // gl^ch: what a whole chunk without a cut multiplies the entering advantage by
    for (int m = 0; m < ch; ++m) gl_ch *= gl;

    const int n_chunks = (T + ch - 1) / ch, n_groups = (n_chunks + NW - 1) / NW;
    for (int g = n_groups - 1, it = 0; g >= 0; --g, ++it) {
        const int buf = it & 1;  // posts and carries alternate between two slots: one barrier per group
        const int c = NW * g + cw;
        const int t0 = c * ch;
        int len = T - t0;
        len = len < 0 ? 0 : (len > ch ? ch : len);
        // loads of the whole chunk
        float rt[GAE_CH], vt[GAE_CH + 1];
        uint32_t cutm = 0, donem = 0;
#pragma unroll
        for (int u = 0; u < GAE_CH; ++u) {
            const bool ok = live && u < len;
            const int64_t o = (int64_t)(t0 + u) * NK + idx;
            rt[u] = ok ? r[o] : 0.f;
            vt[u] = ok ? v[o] : 0.f;
            const uint32_t dn = ok ? done[(int64_t)(t0 + u) * N + n] : 0u;
            const uint32_t tr = (ok && trunc) ? trunc[(int64_t)(t0 + u) * N + n] : 0u;
            donem |= ((dn && !tr) ? 1u : 0u) << u;  // a time limit keeps the bootstrap whatever `done` says
            cutm |= ((dn | tr) ? 1u : 0u) << u;
        }
        // V after the chunk's last step (exists up to t = T)
        float vnext = (live && len > 0) ? v[(int64_t)(t0 + len) * NK + idx] : 0.f;
        // chunk-local recursion from zero, last step first
        float ap[GAE_CH];
        float acc = 0.f;
#pragma unroll
        for (int u = GAE_CH - 1; u >= 0; --u) {
            if (u < len) {
                const float vn = (u + 1 < len) ? vt[(u + 1) & (GAE_CH - 1)] : vnext;
                const float d_done = rt[u] - vt[u];
                const float d_live = rt[u] + gamma * vn - vt[u];
                const bool dn = (donem >> u) & 1u, ct = (cutm >> u) & 1u;
                acc = dn ? d_done : (ct ? d_live : d_live + gl * acc);
            }
            ap[u] = acc;
        }
        post_a[buf][cw][lane] = ap[0];
        post_cut[buf][cw][lane] = (uint8_t)(cutm != 0);
        __syncthreads();
        // advantage entering this chunk: later chunks of the group folded onto the group's carry-in
        float x = (it == 0) ? 0.f : carry[buf ^ 1][lane];
        for (int j = NW - 1; j > cw; --j) {
            int lj = T - (NW * g + j) * ch;
            lj = lj < 0 ? 0 : (lj > ch ? ch : lj);
            float f = gl_ch;
            if (lj < ch) {  // the last chunk of the horizon may be short (uniform)
                f = 1.f;
                for (int m = 0; m < lj; ++m) f *= gl;
            }
            if (lj > 0) x = post_cut[buf][j][lane] ? post_a[buf][j][lane] : post_a[buf][j][lane] + f * x;
        }
        // finish the chunk and write it out
        uint32_t cut_after = 0;  // a cut at or after step u, within the chunk
        float f = gl;            // gl^(steps from u to the chunk's end)
#pragma unroll
        for (int u = GAE_CH - 1; u >= 0; --u) {
            if (u < len) {
                cut_after |= (cutm >> u) & 1u;
                ap[u] = cut_after ? ap[u] : ap[u] + f * x;
                f *= gl;
            }
        }
        if (cw == 0) carry[buf][lane] = ap[0];  // read by every wave after the next group's barrier
#pragma unroll
        for (int u = 0; u < GAE_CH; ++u) {
            if (u < len) {  // uniform across the wave
                const float a = ap[u];
                const float sc = wk * a;
                float tot = sc;
                for (int j = 1; j < K; ++j) tot += __shfl_down(sc, j, WAVE);
                if (live) {
                    const int64_t o = (int64_t)(t0 + u) * NK + idx;
                    if (adv_vec) adv_vec[o] = a;
                    vtarg[o] = a + vt[u];
                    if (k == 0) adv_s[(int64_t)(t0 + u) * N + n] = tot;
                }
            }
        }
    }
}

void launch_vec_gae(const morlax_ctx* c, const float* r, const float* v, const uint8_t* done,
                    const uint8_t* trunc, const float* w, float gamma, float lambda, float* adv_vec,
                    float* vtarg, float* adv_s, hipStream_t s) {
    const int K = c->d.K, N = c->d.N, T = c->d.T;
    const int G = WAVE / K;
    const int blocks = (N + G - 1) / G;
    // the chunks of one group cover the horizon when it is short; CH steps each, in several groups, when it is long
    // eight chunks of up to eight steps, at most 64 registers per lane (eight waves per SIMD): the fastest of the
    // shapes tried at T = 64 (16 x 4: 36 us, 8 x 8: 30 us, 4 x 16: 33 us for 81 MB)
    constexpr int CH = 8, NW = 8;
    int ch = (T + NW - 1) / NW;
    ch = ch > CH ? CH : ch;
    k_vec_gae<CH, NW, 8><<<blocks, 64 * NW, 0, s>>>(r, v, done, trunc, w, gamma, gamma * lambda, adv_vec, vtarg, adv_s,
                                                   T, N, K, c->n_g, ch);
}

// ------------------------------------------------------------------------------------------------
// Loss.  Selected cells are enumerated per preference: cell m of preference p is time
// t0 + m / j_cnt, environment p * n_g + j0 + m % j_cnt.  A block handles 256 cells of one p.

__device__ inline double block_sum(double v, double* sh) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, WAVE);
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    if (lane == 0) sh[wv] = v;
    __syncthreads();
    double tot = sh[0] + sh[1] + sh[2] + sh[3];
    __syncthreads();
    return tot;
}

struct LossWs {
    double* adv_part;   // [nblk][2]
    double* adv_stat;   // [2]: mean, std
    double* stat_part;  // [nblk][5]
    double* dls_part;   // [nblk][A]
};

static LossWs loss_ws_layout(const morlax_ctx* c, const RowSel& rs, void* ws, int64_t* total) {
    const int64_t nbm = (rs.M + 255) / 256, nblk = nbm * c->d.P;
    LossWs L;
    double* p = reinterpret_cast<double*>(ws);
    L.adv_part = p; p += nblk * 2;
    L.adv_stat = p; p += 2;
    L.stat_part = p; p += nblk * 5;
    L.dls_part = p; p += nblk * c->d.act_dim;
    if (total) *total = (int64_t)((char*)p - (char*)ws);
    return L;
}

int64_t loss_ws_bytes(const morlax_ctx* c, const RowSel& rs) {
    int64_t tot = 0;
    loss_ws_layout(c, rs, nullptr, &tot);
    return align_up(tot, 256);
}

__device__ inline int64_t cell_row(const RowSel& rs, int p, int m, int N, int n_g) {
    const int t = rs.t0 + m / rs.j_cnt;
    const int j = rs.j0 + m % rs.j_cnt;
    return (int64_t)t * N + (int64_t)p * n_g + j;
}

__global__ __launch_bounds__(256) void k_adv_partial(RowSel rs, const float* __restrict__ adv_s,
                                                    double* __restrict__ part, int N, int n_g) {
    __shared__ double sh[4];
    const int p = blockIdx.y, m = blockIdx.x * 256 + threadIdx.x;
    double a = 0.0;
    if (m < rs.M) a = (double)adv_s[cell_row(rs, p, m, N, n_g)];
    const double s1 = block_sum(a, sh);
    const double s2 = block_sum(a * a, sh);
    if (threadIdx.x == 0) {
        const int64_t b = (int64_t)p * gridDim.x + blockIdx.x;
        part[b * 2] = s1;
        part[b * 2 + 1] = s2;
    }
}

__global__ __launch_bounds__(256) void k_adv_final(const double* __restrict__ part, int64_t nblk, double cnt,
                                                  double* __restrict__ stat) {
    __shared__ double sh[4];
    double s1 = 0.0, s2 = 0.0;
    for (int64_t b = threadIdx.x; b < nblk; b += 256) {
        s1 += part[b * 2];
        s2 += part[b * 2 + 1];
    }
    s1 = block_sum(s1, sh);
    s2 = block_sum(s2, sh);
    if (threadIdx.x == 0) {
        const double mean = s1 / cnt;
        double var = s2 / cnt - mean * mean;
        if (var < 0.0) var = 0.0;
        stat[0] = mean;
        stat[1] = sqrt(var);
    }
}

template <int A_MAX>
__global__ __launch_bounds__(256) void k_ppo_loss_grad(
    RowSel rs, const float* __restrict__ mu, const float* __restrict__ logsig, int ls_stride,
    const float* __restrict__ act, const float* __restrict__ logp_old, const float* __restrict__ adv_s,
    const float* __restrict__ v, const float* __restrict__ vtarg, const double* __restrict__ adv_stat,
    float clip_eps, int norm_adv, float inv_B, float* __restrict__ dmu, float* __restrict__ dv,
    double* __restrict__ stat_part, double* __restrict__ dls_part, int N, int n_g, int A, int K, int sig_state) {
    // sig_state: mu and dmu have 2A columns per cell -- means, then log sigmas (state dependent) / their gradients
    __shared__ float red[5 + A_MAX][256 + 16];
    __shared__ float s_ls[A_MAX], s_isig[A_MAX];
    const int p = blockIdx.y, m = blockIdx.x * 256 + threadIdx.x;
    const int mus = sig_state ? 2 * A : A;  // row stride of mu and dmu
    if (threadIdx.x < A && !sig_state) {
        const float ls = logsig[(int64_t)p * ls_stride + threadIdx.x];
        s_ls[threadIdx.x] = ls;
        s_isig[threadIdx.x] = expf(-ls);
    }
    __syncthreads();
    const bool ok = m < rs.M;
    float l_pi = 0.f, l_v = 0.f, clipped = 0.f, kl = 0.f, rho_s = 0.f;
    float dls[A_MAX];
#pragma unroll
    for (int a = 0; a < A_MAX; ++a) dls[a] = 0.f;
    if (ok) {
        const int64_t row = cell_row(rs, p, m, N, n_g);
        float ahat = adv_s[row];
        if (norm_adv) ahat = (float)(((double)ahat - adv_stat[0]) / (adv_stat[1] + 1e-8));
        float q[A_MAX], isig[A_MAX];
        float logp = -0.918938533204672742f * (float)A;  // -(A/2) log(2 pi)
#pragma unroll
        for (int a = 0; a < A_MAX; ++a) {
            if (a < A) {
                float ls = 0.f;
                if (sig_state) {
                    ls = mu[row * mus + A + a];
                    isig[a] = expf(-ls);
                } else {
                    ls = s_ls[a];
                    isig[a] = s_isig[a];
                }
                q[a] = (act[row * A + a] - mu[row * mus + a]) * isig[a];
                logp += -0.5f * q[a] * q[a] - ls;
            }
        }
        const float lpo = logp_old[row];
        const float rho = expf(logp - lpo);
        const float rc = fminf(fmaxf(rho, 1.f - clip_eps), 1.f + clip_eps);
        l_pi = -fminf(rho * ahat, rc * ahat);
        const bool pass = (ahat >= 0.f) ? (rho <= 1.f + clip_eps) : (rho >= 1.f - clip_eps);
        const float dlogp = pass ? (-ahat * rho * inv_B) : 0.f;
        clipped = (fabsf(rho - 1.f) > clip_eps) ? 1.f : 0.f;
        kl = lpo - logp;
        rho_s = rho;
#pragma unroll
        for (int a = 0; a < A_MAX; ++a) {
            if (a < A) {
                dmu[row * mus + a] = dlogp * q[a] * isig[a];
                const float g = dlogp * (q[a] * q[a] - 1.f);
                if (sig_state) dmu[row * mus + A + a] = g;  // stays per cell: it flows back through the network
                else dls[a] = g;
            }
        }
        for (int k = 0; k < K; ++k) {
            const float dd = v[row * K + k] - vtarg[row * K + k];
            l_v += dd * dd;
            dv[row * K + k] = 2.f * dd * inv_B;
        }
    }
    // block sums of the 5 statistics and the A log-sigma terms: the per-cell values go to LDS (one padded row
    // per quantity), then 16 lanes add up each row in fp64 -- 16 values each in ascending order, then four
    // exchange steps -- so the whole reduction costs two barriers and has a fixed order
    const int64_t b = (int64_t)p * gridDim.x + blockIdx.x;
    const int nq = 5 + A;
    red[0][threadIdx.x] = l_pi; red[1][threadIdx.x] = l_v; red[2][threadIdx.x] = clipped;
    red[3][threadIdx.x] = kl; red[4][threadIdx.x] = rho_s;
#pragma unroll
    for (int a = 0; a < A_MAX; ++a)
        if (a < A) red[5 + a][threadIdx.x] = dls[a];
    __syncthreads();
    const int qi = threadIdx.x >> 4, li = threadIdx.x & 15;
    for (int q = qi; q < nq; q += 16) {  // (a wave's four groups of 16 lanes take the same number of turns)
        double t = 0.0;
#pragma unroll
        for (int j = 0; j < 16; ++j) t += (double)red[q][16 * j + li];
        t += __shfl_xor(t, 8, WAVE);
        t += __shfl_xor(t, 4, WAVE);
        t += __shfl_xor(t, 2, WAVE);
        t += __shfl_xor(t, 1, WAVE);
        if (li == 0) {
            if (q < 5) stat_part[b * 5 + q] = t;
            else dls_part[b * A + (q - 5)] = t;
        }
    }
}

// blocks 0..P-1: dlogsig[p][:]; block P: stats
__global__ __launch_bounds__(256) void k_loss_final(const double* __restrict__ stat_part,
                                                   const double* __restrict__ dls_part,
                                                   const double* __restrict__ adv_stat, int nbm, int P, int A,
                                                   double cnt, float* __restrict__ dlogsig,
                                                   float* __restrict__ stats) {
    __shared__ double sh[4];
    const int p = blockIdx.x;
    if (p < P) {
        if (!dlogsig) return;  // (state-dependent sigma: there is no per-preference log-sigma gradient)
        for (int a = 0; a < A; ++a) {
            double s = 0.0;
            for (int b = threadIdx.x; b < nbm; b += 256) s += dls_part[((int64_t)p * nbm + b) * A + a];
            s = block_sum(s, sh);
            if (threadIdx.x == 0) dlogsig[p * A + a] = (float)s;
        }
    } else {
        const int64_t nblk = (int64_t)nbm * P;
        double acc[5];
        for (int i = 0; i < 5; ++i) {
            double s = 0.0;
            for (int64_t b = threadIdx.x; b < nblk; b += 256) s += stat_part[b * 5 + i];
            acc[i] = block_sum(s, sh);
        }
        if (threadIdx.x == 0) {
            stats[0] = (float)(acc[0] / cnt);
            stats[1] = (float)(acc[1] / cnt);
            stats[2] = (float)(acc[2] / cnt);
            stats[3] = (float)(acc[3] / cnt);
            stats[4] = (float)adv_stat[0];
            stats[5] = (float)adv_stat[1];
            stats[6] = (float)(acc[4] / cnt);
            stats[7] = (float)cnt;
        }
    }
}

void launch_ppo_loss_grad(const morlax_ctx* c, const RowSel& rs, const float* mu, const float* logsig,
                          int logsig_stride, const float* act, const float* logp_old,
                          const float* adv_s, const float* v, const float* vtarg, float clip_eps,
                          int norm_adv, float* dmu, float* dlogsig, float* dv, float* stats, void* ws,
                          hipStream_t s) {
    const int P = c->d.P, N = c->d.N, A = c->d.act_dim, K = c->d.K;
    LossWs L = loss_ws_layout(c, rs, ws, nullptr);
    const int nbm = (rs.M + 255) / 256;
    const dim3 grid(nbm, P);
    const double cnt = (double)rs.M * P;
    k_adv_partial<<<grid, 256, 0, s>>>(rs, adv_s, L.adv_part, N, c->n_g);
    k_adv_final<<<1, 256, 0, s>>>(L.adv_part, (int64_t)nbm * P, cnt, L.adv_stat);
    k_ppo_loss_grad<MORLAX_MAX_OUT><<<grid, 256, 0, s>>>(rs, mu, logsig, logsig_stride, act, logp_old, adv_s, v,
                                                        vtarg, L.adv_stat, clip_eps, norm_adv,
                                                        (float)(1.0 / cnt), dmu, dv, L.stat_part, L.dls_part,
                                                        N, c->n_g, A, K, c->d.sigma_state);
    k_loss_final<<<P + 1, 256, 0, s>>>(L.stat_part, L.dls_part, L.adv_stat, nbm, P, A, cnt, dlogsig, stats);
}

// The same call on scratch that lives in the library's own image, for callers that cannot allocate: a
// file-scope device array, one copy per GPU at an address of its own, which host code learns once per
// device from hipGetSymbolAddress (the array's name itself is not a device address on the host side).
static __device__ __align__(256) unsigned char scratch[MORLAX_STATIC_SCRATCH_BYTES];

#include <mutex>
#define MORLAX_MAX_DEVICES 64
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[MORLAX_MAX_DEVICES];  // per device, filled on the first call with that device current

int loss_static_scratch(void** ptr) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MORLAX_MAX_DEVICES) return -1;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return -1;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return 0;
}

// ------------------------------------------------------------------------------------------------
// Per-objective advantage normalisation before scalarisation (the other reading of "normalised across
// the batch" in the update phase, Sec. III-C): every objective is standardised over the selected cells
// on its own, then the objectives are combined with the trade-off vector of the environment.
// Workspace: [nblk][2K] partial sums, then [2K] (mean_k, std_k), all fp64; fixed summation order.
int64_t advnorm_ws_bytes(const morlax_ctx* c, const RowSel& rs) {
    const int64_t nblk = (int64_t)((rs.M + 255) / 256) * c->d.P;
    return align_up((nblk * 2 * c->d.K + 2 * c->d.K) * 8, 256);
}

__global__ __launch_bounds__(256) void k_advk_partial(RowSel rs, const float* __restrict__ adv_vec,
                                                     double* __restrict__ part, int N, int n_g, int K) {
    __shared__ double sh[4];
    const int p = blockIdx.y, m = blockIdx.x * 256 + threadIdx.x;
    const float* a = (m < rs.M) ? adv_vec + cell_row(rs, p, m, N, n_g) * K : nullptr;
    const int64_t b = (int64_t)p * gridDim.x + blockIdx.x;
    for (int k = 0; k < K; ++k) {
        const double x = a ? (double)a[k] : 0.0;
        const double s1 = block_sum(x, sh);
        const double s2 = block_sum(x * x, sh);
        if (threadIdx.x == 0) {
            part[(b * K + k) * 2] = s1;
            part[(b * K + k) * 2 + 1] = s2;
        }
    }
}

__global__ __launch_bounds__(256) void k_advk_final(const double* __restrict__ part, int64_t nblk, int K, double cnt,
                                                   double* __restrict__ stat) {
    __shared__ double sh[4];
    const int k = blockIdx.x;
    double s1 = 0.0, s2 = 0.0;
    for (int64_t b = threadIdx.x; b < nblk; b += 256) {
        s1 += part[(b * K + k) * 2];
        s2 += part[(b * K + k) * 2 + 1];
    }
    s1 = block_sum(s1, sh);
    s2 = block_sum(s2, sh);
    if (threadIdx.x == 0) {
        const double mean = s1 / cnt;
        double var = s2 / cnt - mean * mean;
        if (var < 0.0) var = 0.0;
        stat[2 * k] = mean;
        stat[2 * k + 1] = sqrt(var);
    }
}

__global__ __launch_bounds__(256) void k_advk_apply(RowSel rs, const float* __restrict__ adv_vec,
                                                   const float* __restrict__ w, const double* __restrict__ stat,
                                                   float* __restrict__ out, int N, int n_g, int K) {
    const int p = blockIdx.y, m = blockIdx.x * 256 + threadIdx.x;
    if (m >= rs.M) return;
    const int64_t row = cell_row(rs, p, m, N, n_g);
    const float* a = adv_vec + row * K;
    double acc = 0.0;
    for (int k = 0; k < K; ++k)
        acc += (double)w[(int64_t)p * K + k] * (((double)a[k] - stat[2 * k]) / (stat[2 * k + 1] + 1e-8));
    out[row] = (float)acc;
}

void launch_scalarize_normalized(const morlax_ctx* c, const RowSel& rs, const float* adv_vec, const float* w,
                                 float* adv_out, void* ws, hipStream_t s) {
    const int P = c->d.P, N = c->d.N, K = c->d.K;
    const int nbm = (rs.M + 255) / 256;
    const int64_t nblk = (int64_t)nbm * P;
    double* part = reinterpret_cast<double*>(ws);
    double* stat = part + nblk * 2 * K;
    const dim3 grid(nbm, P);
    k_advk_partial<<<grid, 256, 0, s>>>(rs, adv_vec, part, N, c->n_g, K);
    k_advk_final<<<K, 256, 0, s>>>(part, nblk, K, (double)rs.M * P, stat);
    k_advk_apply<<<grid, 256, 0, s>>>(rs, adv_vec, w, stat, adv_out, N, c->n_g, K);
}

// ------------------------------------------------------------------------------------------------
// Adam step on a flat parameter vector (optimiser of the decoupled hypernet updates, Sec. III-C):
//   m <- b1 m + (1 - b1) g,  v <- b2 v + (1 - b2) g^2,
//   theta <- theta - lr (m c1) / (sqrt(v c2) + eps),  c1 = 1 / (1 - b1^t), c2 = 1 / (1 - b2^t)
// (the host computes c1 and c2 in double precision).  Four elements per thread; bound: HBM, 28 bytes
// per parameter (theta, g, m, v read; theta, m, v written).
__global__ __launch_bounds__(256) void k_adam_step(float* __restrict__ theta, const float* __restrict__ g,
                                                  float* __restrict__ m, float* __restrict__ v, int64_t n,
                                                  float lr, float b1, float b2, float eps, float c1, float c2) {
    const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i >= n) return;
    float th[4], gg[4], mm[4], vv[4];
    const bool full = i + 4 <= n;
    if (full) {
        const float4 a = *reinterpret_cast<const float4*>(theta + i), b = *reinterpret_cast<const float4*>(g + i);
        const float4 c = *reinterpret_cast<const float4*>(m + i), d = *reinterpret_cast<const float4*>(v + i);
        th[0] = a.x; th[1] = a.y; th[2] = a.z; th[3] = a.w;
        gg[0] = b.x; gg[1] = b.y; gg[2] = b.z; gg[3] = b.w;
        mm[0] = c.x; mm[1] = c.y; mm[2] = c.z; mm[3] = c.w;
        vv[0] = d.x; vv[1] = d.y; vv[2] = d.z; vv[3] = d.w;
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const bool ok = i + e < n;
            th[e] = ok ? theta[i + e] : 0.f; gg[e] = ok ? g[i + e] : 0.f;
            mm[e] = ok ? m[i + e] : 0.f; vv[e] = ok ? v[i + e] : 0.f;
        }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        mm[e] = b1 * mm[e] + (1.f - b1) * gg[e];
        vv[e] = b2 * vv[e] + (1.f - b2) * gg[e] * gg[e];
        th[e] -= lr * (mm[e] * c1) / (sqrtf(vv[e] * c2) + eps);
    }
    if (full) {
        *reinterpret_cast<float4*>(theta + i) = make_float4(th[0], th[1], th[2], th[3]);
        *reinterpret_cast<float4*>(m + i) = make_float4(mm[0], mm[1], mm[2], mm[3]);
        *reinterpret_cast<float4*>(v + i) = make_float4(vv[0], vv[1], vv[2], vv[3]);
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (i + e < n) { theta[i + e] = th[e]; m[i + e] = mm[e]; v[i + e] = vv[e]; }
    }
}

void launch_adam_step(float* theta, const float* g, float* m, float* v, int64_t n, float lr, float b1, float b2,
                      float eps, float c1, float c2, hipStream_t s) {
    const int64_t blocks = (n + 1023) / 1024;
    k_adam_step<<<(unsigned)blocks, 256, 0, s>>>(theta, g, m, v, n, lr, b1, b2, eps, c1, c2);
}

// ------------------------------------------------------------------------------------------------
// Trade-off vectors of one iteration (Sec. III-C, sampling phase): P - kappa rows uniform on the simplex
// (unit exponentials -ln u divided by their sum) and, in the last kappa rows, the unit vectors e_0 ..
// e_{kappa-1}.  One thread per row; K <= 16.
__global__ __launch_bounds__(256) void k_sample_preferences(const float* __restrict__ u, float* __restrict__ w,
                                                           int P, int K, int kappa) {
    const int p = blockIdx.x * 256 + threadIdx.x;
    if (p >= P) return;
    if (p >= P - kappa) {
        for (int k = 0; k < K; ++k) w[p * K + k] = (k == p - (P - kappa)) ? 1.f : 0.f;
        return;
    }
    float e[MORLAX_MAX_OUT];
    float sum = 0.f;
#pragma unroll
    for (int k = 0; k < MORLAX_MAX_OUT; ++k) {
        e[k] = (k < K) ? -logf(u[p * K + k]) : 0.f;
        sum += e[k];
    }
    const float inv = 1.f / sum;
#pragma unroll
    for (int k = 0; k < MORLAX_MAX_OUT; ++k)
        if (k < K) w[p * K + k] = e[k] * inv;
}

void launch_sample_preferences(const morlax_ctx* c, const float* u, int kappa, float* w, hipStream_t s) {
    k_sample_preferences<<<(c->d.P + 255) / 256, 256, 0, s>>>(u, w, c->d.P, c->d.K, kappa);
}
