// Bandwidth-bound kernels of the update phase (paper Sec. III-C): the environment -> trade-off
// index map, the reverse-time vector GAE scan with scalarisation, the advantage statistics and the
// clipped-PPO / value loss with its gradients.  All reductions are two-stage and fixed-order.
#include "morlax_internal.h"
#include "numeric.h"

#include <type_traits>

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
// scalarised).  A workgroup owns GAE_E = 32 consecutive environments: their (environment, objective)
// pairs are F = 32 K consecutive floats of every time row of r, v and vtarg -- a whole number of 128-byte
// lines starting on a line, whatever K is -- and lane f of the row takes pair f, so every load and store of a
// wave is one aligned run of 256 bytes.
//
// The recursion over t, A_t = cut_t ? a_t : a_t + gl A_{t+1} (a_t = r_t - V_t at an episode end, else the
// TD error; cut_t = episode end or time limit), is a chain of affine maps, so the time axis is split as
// well: the LW = ceil(F / 64) waves that cover a row exist NC times, copy c taking chunk c of up to GAE_CH
// steps.  A wave requests all loads of its chunk at once -- unconditionally, with clamped addresses, so that they
// leave back to back, and one group of chunks ahead: the next group's values arrive while this one is finished,
// scalarised and written --, runs the recursion from zero (A'_t), and posts
// the value at its first step and whether its chunk holds a cut.  After a barrier it folds the posts of
// the later chunks into the advantage that enters its own chunk, x, and finishes
// A_t = (a cut between t and the chunk's end) ? A'_t : A'_t + gl^(steps to the chunk's end) x.
// Cuts stay selects throughout, so nothing behind an episode end -- NaN and Inf included -- reaches the
// steps before it.  Horizons above NC * GAE_CH are walked in groups of NC chunks, last group first.
// The scalarisation sum_k w_k A_k goes through LDS: every lane leaves w_k A_t there, and after a second
// barrier the workgroup adds the K terms of a cell in ascending k and writes adv_s as 128-byte runs.
#define GAE_E 32
// results that this kernel does not read again leave with non-temporal stores (measured: +4 % bandwidth on the
// T = 256, N = 65536 shape; the same mark on the loads of r and v gained nothing and cost 5 % at workload 5)
__device__ inline void st_stream(float* p, float v) { __builtin_nontemporal_store(v, p); }

template <int GAE_CH, bool TRUNC>
__global__ __launch_bounds__(768, 6) void k_vec_gae(const float* __restrict__ r, const float* __restrict__ v,
                                                     const uint8_t* __restrict__ done,
                                                     const uint8_t* __restrict__ trunc, const float* __restrict__ w,
                                                     float gamma, float gl, float* __restrict__ adv_vec,
                                                     float* __restrict__ vtarg, float* __restrict__ adv_s,
                                                     int T, int N, int K, int n_g, int ch, int LW, int NC) {
    __shared__ float post_a[2][1024];     // [slot][chunk copy][pair]: NC * F <= 1024
    __shared__ uint8_t post_cut[2][1024];
    __shared__ float carry[2][512];
    __shared__ float sc[GAE_CH * 1024];   // [chunk copy][step][pair]: w_k A_t of the group being written
    const int F = GAE_E * K;
    const int lane = threadIdx.x & (WAVE - 1);
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x / WAVE);
    const int cw = wv / LW, lw = wv - cw * LW;  // chunk copy, wave within the row (both wave-uniform)
    const int f = lw * WAVE + lane;
    const int e = f / K, k = f - e * K;
    // workgroups are dealt to the chip's eight dies in turn; the block of environments follows the die, so that
    // neighbouring blocks -- which share the 128-byte lines of `done` -- meet in one die's L2
    const int nb = gridDim.x, xq = nb / 8, xr = nb % 8, xd = blockIdx.x % 8;
    const int blk = xd * xq + (xd < xr ? xd : xr) + blockIdx.x / 8;
    const int n0 = blk * GAE_E, n = n0 + e;
    const bool live = (f < F) && (n < N);
    const int64_t NK = (int64_t)N * K;
    const float wk = live ? w[(n / n_g) * K + k] : 0.f;
    float gl_ch = 1.f;  // gl^ch: what a whole chunk without a cut multiplies the entering advantage by
    for (int m = 0; m < ch; ++m) gl_ch *= gl;

    const int n_chunks = (T + ch - 1) / ch, n_groups = (n_chunks + NC - 1) / NC;
    // the loads of a group's chunk: requested while the group before it (later in time) is finished and written
    float rt_n[GAE_CH], vt_n[GAE_CH], vnext_n;
    uint32_t cutm_n, donem_n;
    // addresses = a wave-uniform row start (scalar registers) + the lane's pair or environment
    const int64_t pair0 = (int64_t)n0 * K;
    // Every load is issued whatever the lane or the step: rows past the chunk repeat the horizon's last row and idle
    // lanes read the block's first pair, so the requests of a chunk leave back to back with no branch between them;
    // what they return is discarded below.
    // (a scalar row start plus an unsigned 32-bit byte offset of the lane: one address register per lane)
    const uint32_t fs = live ? 4u * f : 0u, es = live ? e : 0u;
    auto at = [](const float* row, uint32_t byte_off) {
        return reinterpret_cast<const float*>(reinterpret_cast<const char*>(row) + byte_off);
    };
    auto request = [&](int g) {
        const int t0 = (NC * g + cw) * ch;
        int len = T - t0;
        len = len < 0 ? 0 : (len > ch ? ch : len);
        uint32_t dn[GAE_CH], tr[GAE_CH];
#pragma unroll
        for (int u = 0; u < GAE_CH; ++u) {  // the bytes first: the masks below then wait for these loads only
            const int t = t0 + u < T ? t0 + u : T - 1;
            dn[u] = (done + (int64_t)t * N + n0)[es];
            tr[u] = TRUNC ? (trunc + (int64_t)t * N + n0)[es] : 0u;
        }
#pragma unroll
        for (int u = 0; u < GAE_CH; ++u) {
            const int t = t0 + u < T ? t0 + u : T - 1;
            rt_n[u] = *at(r + ((int64_t)t * NK + pair0), fs);
            vt_n[u] = *at(v + ((int64_t)t * NK + pair0), fs);
        }
        // V after the chunk's last step (exists up to t = T)
        const int tl = t0 + len < T ? t0 + len : T;
        vnext_n = *at(v + ((int64_t)tl * NK + pair0), fs);
        cutm_n = 0;
        donem_n = 0;
#pragma unroll
        for (int u = 0; u < GAE_CH; ++u) {
            const bool ok = live && u < len;
            donem_n |= ((ok && dn[u] && !tr[u]) ? 1u : 0u) << u;  // a time limit keeps the bootstrap whatever `done` says
            cutm_n |= ((ok && (dn[u] | tr[u])) ? 1u : 0u) << u;
        }
    };
    request(n_groups - 1);
    for (int g = n_groups - 1, it = 0; g >= 0; --g, ++it) {
        const int buf = it & 1;  // posts and carries alternate between two slots
        const int c = NC * g + cw;
        const int t0 = c * ch;
        int len = T - t0;
        len = len < 0 ? 0 : (len > ch ? ch : len);
        float rt[GAE_CH], vt[GAE_CH];
#pragma unroll
        for (int u = 0; u < GAE_CH; ++u) {
            const bool ok = live && u < len;
            rt[u] = ok ? rt_n[u] : 0.f;
            vt[u] = ok ? vt_n[u] : 0.f;
        }
        const float vnext = (live && len > 0) ? vnext_n : 0.f;
        const uint32_t cutm = cutm_n, donem = donem_n;
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
        if (f < F) {
            post_a[buf][cw * F + f] = ap[0];
            post_cut[buf][cw * F + f] = (uint8_t)(cutm != 0);
        }
        __syncthreads();  // (also: every wave is done reading the previous group's scalarisation terms)
        if (g > 0) request(g - 1);
        // advantage entering this chunk: later chunks of the group folded onto the group's carry-in
        float x = (it == 0 || f >= F) ? 0.f : carry[buf ^ 1][f];
        for (int j = NC - 1; j > cw; --j) {
            int lj = T - (NC * g + j) * ch;
            lj = lj < 0 ? 0 : (lj > ch ? ch : lj);
            float fj = gl_ch;
            if (lj < ch) {  // the last chunk of the horizon may be short (uniform)
                fj = 1.f;
                for (int m = 0; m < lj; ++m) fj *= gl;
            }
            if (lj > 0 && f < F) x = post_cut[buf][j * F + f] ? post_a[buf][j * F + f] : post_a[buf][j * F + f] + fj * x;
        }
        // finish the chunk and write it out
        uint32_t cut_after = 0;  // a cut at or after step u, within the chunk
        float fu = gl;           // gl^(steps from u to the chunk's end)
#pragma unroll
        for (int u = GAE_CH - 1; u >= 0; --u) {
            if (u < len) {
                cut_after |= (cutm >> u) & 1u;
                ap[u] = cut_after ? ap[u] : ap[u] + fu * x;
                fu *= gl;
            }
        }
        if (cw == 0 && f < F) carry[buf][f] = ap[0];  // read by every wave after the next group's first barrier
#pragma unroll
        for (int u = 0; u < GAE_CH; ++u) {
            if (u < len) {  // uniform across the wave
                const float a = ap[u];
                if (f < F) sc[(cw * GAE_CH + u) * F + f] = wk * a;
                if (live) {
                    const int64_t o = (int64_t)(t0 + u) * NK + pair0;  // wave-uniform
                    if (adv_vec) st_stream(adv_vec + o + f, a);
                    st_stream(vtarg + o + f, a + vt[u]);
                }
            }
        }
        __syncthreads();
        // scalarised advantage of the group's cells: 32 environments of a step per half-wave
        for (int q = threadIdx.x; q < NC * GAE_CH * GAE_E; q += blockDim.x) {
            const int cu = q / GAE_E, ee = q % GAE_E;       // (chunk copy, step), environment
            const int cj = cu / GAE_CH, u = cu % GAE_CH;
            const int t = (NC * g + cj) * ch + u;
            if (u < ch && t < T && n0 + ee < N) {
                const float* term = sc + cu * F + ee * K;
                float tot = term[0];
                for (int j = 1; j < K; ++j) tot += term[j];
                st_stream(adv_s + (int64_t)t * N + n0 + ee, tot);
            }
        }
    }
}

void launch_vec_gae(const morlax_ctx* c, const float* r, const float* v, const uint8_t* done,
                    const uint8_t* trunc, const float* w, float gamma, float lambda, float* adv_vec,
                    float* vtarg, float* adv_s, hipStream_t s) {
    const int K = c->d.K, N = c->d.N, T = c->d.T;
    const int blocks = (N + GAE_E - 1) / GAE_E;
    // chunks of up to eight steps; a workgroup of at most twelve waves (two or three of them share a CU at six waves
    // and 80 registers per SIMD: the chunk being finished and the next one's loads are both held in registers); the
    // chunk copies: the largest power of two that keeps it within that, at most eight (K = 6: four copies of three
    // waves; five measured slower at T = 64 and T = 256), then no more than evens out the groups of chunks
    constexpr int CH = 8;
    const int LW = (GAE_E * K + WAVE - 1) / WAVE;
    int NC = 8;
    while (NC * LW > 12) NC >>= 1;
    int ch = (T + NC - 1) / NC;
    ch = ch > CH ? CH : ch;
    const int n_chunks = (T + ch - 1) / ch, n_groups = (n_chunks + NC - 1) / NC;
    NC = (n_chunks + n_groups - 1) / n_groups;
    if (trunc)
        k_vec_gae<CH, true><<<blocks, WAVE * LW * NC, 0, s>>>(r, v, done, trunc, w, gamma, gamma * lambda, adv_vec, vtarg,
                                                             adv_s, T, N, K, c->n_g, ch, LW, NC);
    else
        k_vec_gae<CH, false><<<blocks, WAVE * LW * NC, 0, s>>>(r, v, done, trunc, w, gamma, gamma * lambda, adv_vec, vtarg,
                                                              adv_s, T, N, K, c->n_g, ch, LW, NC);
}

// ------------------------------------------------------------------------------------------------
// Loss.  Selected cells are enumerated per preference: cell m of preference p is time
// t0 + m / j_cnt, environment p * n_g + j0 + m % j_cnt.  A block handles G consecutive groups of 256 cells
// of one p, one group after the other; a group is up to 256 / j_cnt + 2 runs of consecutive rows of the
// time-major tensors.  The runs of mu, act, v and vtarg go from global memory straight into LDS as they lie in
// memory (direct-to-LDS loads, 256 contiguous bytes per wave instruction, all of a group's requests in flight
// at once), a thread then works on its cell out of LDS, leaves the gradients there, and the block writes
// them back run by run -- every global access of the kernel is a contiguous run instead of one 4-byte piece
// per 40-byte row and lane.
//
// Three launches per call.  k_adv_partial adds up the scalar advantage of the selection into at most
// LOSS_MAX_ADV_PART fixed partial sums; every block of k_ppo_loss_grad adds those partials in the same fixed
// order and so knows mean and standard deviation without a launch in between.  The block sums of the
// statistics and of the log-sigma gradients are written per block (G is chosen so that there are about
// LOSS_TARGET_BLOCKS of them, few enough for one workgroup to add up) and k_loss_final adds them in block order:
// fixed orders throughout, no atomics, results repeatable bit for bit.  (Finishing inside the loss kernel, by
// whichever block comes last, needs a device-scope release in every block; on this chip that is a write-back of
// the whole L2 and made the call three times slower.)

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

#define LOSS_NT 128              // cells per group = threads per block of the loss kernel
#define LOSS_MAX_ADV_PART 512
#define LOSS_TARGET_BLOCKS 2048

struct LossPlan {
    int nbm;     // groups of LOSS_NT cells per preference
    int G;       // groups per block
    int nbx;     // blocks per preference
    int nb256;   // groups of 256 cells per preference (the advantage statistics pass)
    int n_adv;   // partial sums of the advantage statistics
    int per;     // 256-cell groups (over all preferences) per advantage partial
};

static LossPlan loss_plan(const morlax_ctx* c, const RowSel& rs) {
    LossPlan L;
    L.nbm = (rs.M + LOSS_NT - 1) / LOSS_NT;
    const int64_t ngrp = (int64_t)L.nbm * c->d.P;
    int G = (int)((ngrp + LOSS_TARGET_BLOCKS - 1) / LOSS_TARGET_BLOCKS);
    L.G = G < 1 ? 1 : G;
    L.nbx = (L.nbm + L.G - 1) / L.G;
    L.nb256 = (rs.M + 255) / 256;
    const int64_t n256 = (int64_t)L.nb256 * c->d.P;
    const int64_t cap = n256 < LOSS_MAX_ADV_PART ? n256 : LOSS_MAX_ADV_PART;
    L.per = (int)((n256 + cap - 1) / cap);
    L.n_adv = (int)((n256 + L.per - 1) / L.per);
    return L;
}

struct LossWs {
    double* adv_part;   // [n_adv][2]
    double* stat_part;  // [P * nbx][5]
    double* dls_part;   // [P * nbx][A]
};

static LossWs loss_ws_layout(const morlax_ctx* c, const RowSel& rs, void* ws, int64_t* total) {
    const LossPlan pl = loss_plan(c, rs);
    const int64_t nblk = (int64_t)pl.nbx * c->d.P;
    LossWs L;
    double* p = reinterpret_cast<double*>(ws);
    L.adv_part = p; p += (int64_t)pl.n_adv * 2;
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

// partial b covers the 256-cell groups [b * per, (b + 1) * per) of the (preference, group) enumeration; the
// loads of sixteen groups are issued together.  V4 (every run of selected cells starts on a 16-byte boundary
// and holds a multiple of four cells): a group is 64 threads x four consecutive cells, 16 bytes per load.
template <bool V4>
__global__ __launch_bounds__(256) void k_adv_partial(RowSel rs, const float* __restrict__ adv_s,
                                                    double* __restrict__ part, int N, int n_g, int nbm, int ngrp,
                                                    int per) {
    __shared__ double sh[4];
    double s1 = 0.0, s2 = 0.0;
    const int lo = blockIdx.x * per, hi = (lo + per < ngrp) ? lo + per : ngrp;
    if (V4) {
        // the block's 256 threads take four groups at a time: wave w group cb + w, lane l its cells 4 l .. 4 l + 3
        const int wv = threadIdx.x >> 6, lane = threadIdx.x & 63;
        for (int cb = lo; cb < hi; cb += 16) {
            float4 a[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int g = cb + 4 * u + wv, p = g / nbm, m = (g - p * nbm) * 256 + 4 * lane;
                a[u] = (g < hi && m < rs.M) ? *reinterpret_cast<const float4*>(adv_s + cell_row(rs, p, m, N, n_g))
                                            : make_float4(0.f, 0.f, 0.f, 0.f);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const double x0 = a[u].x, x1 = a[u].y, x2 = a[u].z, x3 = a[u].w;
                s1 += (x0 + x1) + (x2 + x3);
                s2 += (x0 * x0 + x1 * x1) + (x2 * x2 + x3 * x3);
            }
        }
    } else {
        for (int cb = lo; cb < hi; cb += 16) {
            float a[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int g = cb + u, p = g / nbm, m = (g - p * nbm) * 256 + threadIdx.x;
                a[u] = (g < hi && m < rs.M) ? adv_s[cell_row(rs, p, m, N, n_g)] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                s1 += (double)a[u];
                s2 += (double)a[u] * (double)a[u];
            }
        }
    }
    s1 = block_sum(s1, sh);
    s2 = block_sum(s2, sh);
    if (threadIdx.x == 0) {
        part[2 * blockIdx.x] = s1;
        part[2 * blockIdx.x + 1] = s2;
    }
}

// One array of a group's cells between global memory and LDS.  The group's cells [m0, m1) of preference p
// fall into runs of consecutive rows, one per time step touched; a run holds ncell * C consecutive floats.
struct CellRuns {
    int m0, m1, j_cnt, tA, tB;
    int64_t row00;  // row of (time step t0, position j0) of this preference
    int64_t N;
    __device__ inline void run(int tt, int& cell0, int& ncell, int64_t& row) const {
        const int a = tt * j_cnt, b = a + j_cnt;
        const int cA = m0 > a ? m0 : a, cB = m1 < b ? m1 : b;
        cell0 = cA - m0;
        ncell = cB - cA;
        row = row00 + (int64_t)tt * N + (cA - a);
    }
};

// V4: every run starts on a 16-byte boundary and holds a multiple of four floats (the launcher checks the
// selection), so a lane moves 16 bytes at a time.  The loads are marked non-temporal (each byte is read once;
// +6 % bandwidth measured on the T = 256, N = 65536 shape; the same mark on the stores gained nothing).
template <bool V4, int NT>
__device__ inline void runs_to_lds(const CellRuns& cr, const float* __restrict__ X, int C, uint32_t lds_addr) {
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    for (int tt = cr.tA; tt <= cr.tB; ++tt) {
        int cell0, ncell;
        int64_t row;
        cr.run(tt, cell0, ncell, row);
        const float* src = X + row * C;
        if (V4) {
            const int count = ncell * C / 4;
            for (int c0 = wave * 64; c0 < count; c0 += NT)
                if (c0 + lane < count)
                    dma16_nt(src + 4 * c0, (uint32_t)lane * 16u,
                          __builtin_amdgcn_readfirstlane(lds_addr + (uint32_t)(cell0 * C + 4 * c0) * 4u));
        } else {
            const int count = ncell * C;
            for (int c0 = wave * 64; c0 < count; c0 += NT)
                if (c0 + lane < count)
                    dma4_nt(src + c0, (uint32_t)lane * 4u,
                         __builtin_amdgcn_readfirstlane(lds_addr + (uint32_t)(cell0 * C + c0) * 4u));
        }
    }
}

template <bool V4, int NT>
__device__ inline void lds_to_runs(const CellRuns& cr, float* __restrict__ X, int C, const float* lds) {
    for (int tt = cr.tA; tt <= cr.tB; ++tt) {
        int cell0, ncell;
        int64_t row;
        cr.run(tt, cell0, ncell, row);
        float* dst = X + row * C;
        const float* src = lds + cell0 * C;
        if (V4) {
            const int count = ncell * C / 4;
            for (int i = threadIdx.x; i < count; i += NT)
                reinterpret_cast<float4*>(dst)[i] = reinterpret_cast<const float4*>(src)[i];
        } else {
            const int count = ncell * C;
            for (int i = threadIdx.x; i < count; i += NT) dst[i] = src[i];
        }
    }
}

// sum over the block's NT / 64 waves, fixed order
template <int NT>
__device__ inline double block_sum_nt(double v, double* sh) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, WAVE);
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    if (lane == 0) sh[wv] = v;
    __syncthreads();
    double tot = sh[0];
#pragma unroll
    for (int i = 1; i < NT / 64; ++i) tot += sh[i];
    __syncthreads();
    return tot;
}

// NT threads work on groups of NT cells
template <int A_MAX, int NT, bool V4>
__global__ __launch_bounds__(NT, 8) void k_ppo_loss_grad(
    RowSel rs, const float* __restrict__ mu, const float* __restrict__ logsig, int ls_stride,
    const float* __restrict__ act, const float* __restrict__ logp_old, const float* __restrict__ adv_s,
    const float* __restrict__ v, const float* __restrict__ vtarg, const double* __restrict__ adv_part, int n_adv,
    float clip_eps, int norm_adv, double cnt_cells, float* __restrict__ dmu, float* __restrict__ dv,
    double* __restrict__ stat_part, double* __restrict__ dls_part, int N, int n_g, int A, int K, int G,
    int sig_state) {
    // sig_state: mu and dmu have 2A columns per cell -- means, then log sigmas (state dependent) / their gradients
    extern __shared__ __align__(16) float lds[];
    __shared__ float s_ls[A_MAX], s_isig[A_MAX];
    __shared__ double sh[4];
    constexpr int RP = NT + 16;  // pitch of a reduction row
    const int p = blockIdx.y, tid = threadIdx.x;
    const int mus = sig_state ? 2 * A : A;  // row stride of mu and dmu
    // LDS: mu (dmu) | v (dv) | act | vtarg, cell-major as in memory; the reduction rows later reuse act | vtarg.
    // (Two such buffers, the next group arriving while this one is worked on, halve the blocks per CU and
    // measured a quarter slower: the kernel lives on many independent blocks, eight per CU.)
    float* l_mu = lds;
    float* l_v = l_mu + NT * mus;
    float* l_act = l_v + NT * K;
    float* l_vt = l_act + NT * A;
    const uint32_t lbase = (uint32_t)(size_t)lds;
    CellRuns cr;
    cr.j_cnt = rs.j_cnt;
    cr.N = N;
    cr.row00 = (int64_t)rs.t0 * N + (int64_t)p * n_g + rs.j0;
    auto request = [&](int grp) {  // a group's runs of the four arrays, on their way into LDS
        cr.m0 = grp * NT;
        cr.m1 = cr.m0 + NT < rs.M ? cr.m0 + NT : rs.M;
        cr.tA = cr.m0 / rs.j_cnt;
        cr.tB = (cr.m1 - 1) / rs.j_cnt;
        runs_to_lds<V4, NT>(cr, mu, mus, lbase);
        runs_to_lds<V4, NT>(cr, v, K, lbase + (uint32_t)(NT * mus) * 4u);
        runs_to_lds<V4, NT>(cr, act, A, lbase + (uint32_t)(NT * (mus + K)) * 4u);
        runs_to_lds<V4, NT>(cr, vtarg, K, lbase + (uint32_t)(NT * (mus + K + A)) * 4u);
    };
    const int nbm = (rs.M + NT - 1) / NT;
    const int g_lo = blockIdx.x * G, g_hi = (g_lo + G < nbm) ? g_lo + G : nbm;
    request(g_lo);
    if (tid < A && !sig_state) {
        const float ls = logsig[(int64_t)p * ls_stride + tid];
        s_ls[tid] = ls;
        s_isig[tid] = expf(-ls);
    }
    // mean and standard deviation of the selection's advantage from the fixed partial sums
    double s1 = 0.0, s2 = 0.0;
    for (int i = tid; i < n_adv; i += NT) {
        s1 += adv_part[2 * i];
        s2 += adv_part[2 * i + 1];
    }
    s1 = block_sum_nt<NT>(s1, sh);
    s2 = block_sum_nt<NT>(s2, sh);
    const double a_mean = s1 / cnt_cells;
    double a_var = s2 / cnt_cells - a_mean * a_mean;
    a_var = a_var < 0.0 ? 0.0 : a_var;
    const double a_std = sqrt(a_var);
    const float inv_B = (float)(1.0 / cnt_cells);
    const double inv_std = 1.0 / (a_std + 1e-8);

    float l_pi = 0.f, l_val = 0.f, clipped = 0.f, kl = 0.f, rho_s = 0.f;
    float dls[A_MAX];
#pragma unroll
    for (int a = 0; a < A_MAX; ++a) dls[a] = 0.f;
    for (int grp = g_lo; grp < g_hi; ++grp) {
        const int m = grp * NT + tid;
        const bool ok = m < rs.M;
        float ahat = 0.f, lpo = 0.f;
        if (ok) {
            const int64_t row = cell_row(rs, p, m, N, n_g);
            ahat = adv_s[row];
            lpo = logp_old[row];
        }
        wait_vm<0>();
        __syncthreads();  // the group's runs are in LDS
        if (ok) {
            if (norm_adv) ahat = (float)(((double)ahat - a_mean) * inv_std);
            float* c_mu = l_mu + tid * mus;
            const float* c_act = l_act + tid * A;
            // two passes over the action components (the second forms q again from LDS) instead of per-component
            // register arrays: 64 registers per lane, eight waves per SIMD
            float logp = -0.918938533204672742f * (float)A;  // -(A/2) log(2 pi)
#pragma unroll
            for (int a = 0; a < A_MAX; ++a) {
                if (a < A) {
                    const float ls = sig_state ? c_mu[A + a] : s_ls[a];
                    const float is = sig_state ? expf(-ls) : s_isig[a];
                    const float q = (c_act[a] - c_mu[a]) * is;
                    logp += -0.5f * q * q - ls;
                }
            }
            const float rho = expf(logp - lpo);
            const float rc = fminf(fmaxf(rho, 1.f - clip_eps), 1.f + clip_eps);
            l_pi += -fminf(rho * ahat, rc * ahat);
            const bool pass = (ahat >= 0.f) ? (rho <= 1.f + clip_eps) : (rho >= 1.f - clip_eps);
            const float dlogp = pass ? (-ahat * rho * inv_B) : 0.f;
            clipped += (fabsf(rho - 1.f) > clip_eps) ? 1.f : 0.f;
            kl += lpo - logp;
            rho_s += rho;
#pragma unroll
            for (int a = 0; a < A_MAX; ++a) {
                if (a < A) {
                    const float is = sig_state ? expf(-c_mu[A + a]) : s_isig[a];
                    const float q = (c_act[a] - c_mu[a]) * is;
                    c_mu[a] = dlogp * q * is;
                    const float g = dlogp * (q * q - 1.f);
                    if (sig_state) c_mu[A + a] = g;  // stays per cell: it flows back through the network
                    else dls[a] += g;
                }
            }
            float* c_v = l_v + tid * K;
            const float* c_vt = l_vt + tid * K;
            for (int k = 0; k < K; ++k) {
                const float dd = c_v[k] - c_vt[k];
                l_val += dd * dd;
                c_v[k] = 2.f * dd * inv_B;
            }
        }
        __syncthreads();  // gradients complete in LDS; act and vtarg no longer needed
        lds_to_runs<V4, NT>(cr, dmu, mus, l_mu);
        lds_to_runs<V4, NT>(cr, dv, K, l_v);
        if (grp + 1 < g_hi) {
            __syncthreads();  // every thread has read what it stores before the next group's runs arrive
            request(grp + 1);
        }
    }
    // block sums of the 5 statistics and the A log-sigma terms: the per-cell values go to LDS (one padded row
    // per quantity), then 16 lanes add up each row in fp64 -- NT / 16 values each in ascending order, then four
    // exchange steps -- so the whole reduction costs two barriers and has a fixed order
    float* red = l_act;
    const int64_t b = (int64_t)p * gridDim.x + blockIdx.x;
    const int nq = 5 + (sig_state ? 0 : A);
    red[0 * RP + tid] = l_pi; red[1 * RP + tid] = l_val; red[2 * RP + tid] = clipped;
    red[3 * RP + tid] = kl; red[4 * RP + tid] = rho_s;
    if (!sig_state) {
#pragma unroll
        for (int a = 0; a < A_MAX; ++a)
            if (a < A) red[(5 + a) * RP + tid] = dls[a];
    }
    __syncthreads();
    const int qi = tid >> 4, li = tid & 15;
    for (int q = qi; q < nq; q += NT / 16) {  // (a wave's four groups of 16 lanes take the same number of turns)
        double t = 0.0;
#pragma unroll
        for (int j = 0; j < NT / 16; ++j) t += (double)red[q * RP + 16 * j + li];
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

// blocks 0 .. P-1: dlogsig[p][:] (the preference's block partials in block order); block P: the statistics.
// 1024 threads, so that the one block that adds up the statistics has enough loads in flight.
__device__ inline double block_sum16(double v, double* sh) {  // 16 waves, fixed order
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, WAVE);
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    if (lane == 0) sh[wv] = v;
    __syncthreads();
    double tot = sh[0];
#pragma unroll
    for (int i = 1; i < 16; ++i) tot += sh[i];
    __syncthreads();
    return tot;
}

__global__ __launch_bounds__(1024) void k_loss_final(const double* __restrict__ stat_part,
                                                    const double* __restrict__ dls_part,
                                                    const double* __restrict__ adv_part, int n_adv, int nbx, int P,
                                                    int A, double cnt, float* __restrict__ dlogsig,
                                                    float* __restrict__ stats) {
    __shared__ double sh[16];
    const int p = blockIdx.x;
    if (p < P) {
        if (!dlogsig) return;  // (state-dependent sigma: there is no per-preference log-sigma gradient)
        // thread (a, i) adds the partials i, i + 64, ... of component a; then the 64 shares of a component in order
        __shared__ double part[MORLAX_MAX_OUT][64];
        const int a = threadIdx.x >> 6, i = threadIdx.x & 63;
        double s = 0.0;
        if (a < A)
            for (int b = i; b < nbx; b += 64) s += dls_part[((int64_t)p * nbx + b) * A + a];
        part[a][i] = s;
        __syncthreads();
        if (threadIdx.x < A) {
            double t = 0.0;
            for (int j = 0; j < 64; ++j) t += part[threadIdx.x][j];
            dlogsig[p * A + threadIdx.x] = (float)t;
        }
    } else {
        const int64_t nblk = (int64_t)nbx * P;
        double s[7] = {0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0};
        for (int64_t b = threadIdx.x; b < nblk; b += 1024) {
#pragma unroll
            for (int i = 0; i < 5; ++i) s[i] += stat_part[b * 5 + i];
        }
        for (int b = threadIdx.x; b < n_adv; b += 1024) {
            s[5] += adv_part[2 * b];
            s[6] += adv_part[2 * b + 1];
        }
        double acc[7];
        for (int i = 0; i < 7; ++i) acc[i] = block_sum16(s[i], sh);
        if (threadIdx.x == 0) {
            const double mean = acc[5] / cnt;
            double var = acc[6] / cnt - mean * mean;
            var = var < 0.0 ? 0.0 : var;
            stats[0] = (float)(acc[0] / cnt);
            stats[1] = (float)(acc[1] / cnt);
            stats[2] = (float)(acc[2] / cnt);
            stats[3] = (float)(acc[3] / cnt);
            stats[4] = (float)mean;
            stats[5] = (float)sqrt(var);
            stats[6] = (float)(acc[4] / cnt);
            stats[7] = (float)cnt;
        }
    }
}

static int64_t loss_lds_floats(int mus, int A, int K, int nq) {
    const int64_t dead = LOSS_NT * (int64_t)(A + K), red = (int64_t)(LOSS_NT + 16) * nq;
    return LOSS_NT * (int64_t)(mus + K) + (dead > red ? dead : red);
}

// every run of every array starts on a 16-byte boundary and is a multiple of 16 bytes long
static bool loss_vec4_ok(const morlax_ctx* c, const RowSel& rs, int mus) {
    const int A = c->d.act_dim, K = c->d.K;
    const int cs[3] = {mus, A, K};
    for (int C : cs) {
        if (((int64_t)c->d.N * C) % 4 || ((int64_t)c->n_g * C) % 4 || ((int64_t)rs.j0 * C) % 4 ||
            ((int64_t)rs.j_cnt * C) % 4 || ((int64_t)LOSS_NT * C) % 4)
            return false;
    }
    return true;
}

void launch_ppo_loss_grad(const morlax_ctx* c, const RowSel& rs, const float* mu, const float* logsig,
                          int logsig_stride, const float* act, const float* logp_old,
                          const float* adv_s, const float* v, const float* vtarg, float clip_eps,
                          int norm_adv, float* dmu, float* dlogsig, float* dv, float* stats, void* ws,
                          hipStream_t s) {
    const int P = c->d.P, N = c->d.N, A = c->d.act_dim, K = c->d.K, sig = c->d.sigma_state;
    const LossPlan pl = loss_plan(c, rs);
    LossWs L = loss_ws_layout(c, rs, ws, nullptr);
    const double cnt = (double)rs.M * P;
    if (N % 4 == 0 && c->n_g % 4 == 0 && rs.j0 % 4 == 0 && rs.j_cnt % 4 == 0)
        k_adv_partial<true><<<pl.n_adv, 256, 0, s>>>(rs, adv_s, L.adv_part, N, c->n_g, pl.nb256, pl.nb256 * P, pl.per);
    else
        k_adv_partial<false><<<pl.n_adv, 256, 0, s>>>(rs, adv_s, L.adv_part, N, c->n_g, pl.nb256, pl.nb256 * P, pl.per);
    const int mus = sig ? 2 * A : A;
    const size_t lds_bytes = (size_t)loss_lds_floats(mus, A, K, 5 + (sig ? 0 : A)) * 4;
    auto launch = [&](auto v4) {
        constexpr bool V4 = decltype(v4)::value;
        k_ppo_loss_grad<MORLAX_MAX_OUT, LOSS_NT, V4><<<dim3(pl.nbx, P), LOSS_NT, lds_bytes, s>>>(
            rs, mu, logsig, logsig_stride, act, logp_old, adv_s, v, vtarg, L.adv_part, pl.n_adv, clip_eps, norm_adv,
            cnt, dmu, dv, L.stat_part, L.dls_part, N, c->n_g, A, K, pl.G, sig);
    };
    if (loss_vec4_ok(c, rs, mus)) launch(std::true_type{}); else launch(std::false_type{});
    k_loss_final<<<P + 1, 1024, 0, s>>>(L.stat_part, L.dls_part, L.adv_part, pl.n_adv, pl.nbx, P, A, cnt, dlogsig, stats);
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
