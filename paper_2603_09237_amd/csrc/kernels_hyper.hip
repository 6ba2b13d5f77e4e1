// Hypernetwork forward and backward (paper Sec. III-B: H(w) = M f(w) + b, read as rank-r factors on
// shared base weights; with rank < 0 the strictly affine form, every weight its own row of M, which runs
// entirely through the stacked affine map below).  fp32 arithmetic; theta_mat is rounded to bf16 (nearest even) on store when
// the target networks run in bf16.  Every reduction is fixed-order.
#include "morlax_internal.h"
#include "numeric.h"

#define QW 64  // stacked-affine rows per wave of the df partial kernel (at least)
#define DAB_COLS 128  // columns of dW one block of the fused dA/dB kernel walks
#define DAB_NCT (DAB_COLS / 64)
#define DAB_MAX_CS (2048 / DAB_COLS)  // column runs of the widest layer

struct HyperWs {
    float *h1, *f, *fac, *dfac, *df_part, *df, *dz2, *dz1, *vecs, *da_part;
    int32_t* mrow;  // [q_total] offset of row q of the stacked affine matrix inside hparams
    int n_chunk, n_cs;
};

// stacked-affine rows per wave of the df partial kernel: QW, more when there are very many rows (strictly
// affine hypernetwork), so that the partials stay a few thousand chunks
static int df_chunk_rows(int64_t q_total) {
    int qw = QW;
    while ((q_total + qw - 1) / qw > 4096) qw *= 2;
    return qw;
}

static HyperWs hyper_ws_layout(const morlax_ctx* c, void* ws, int64_t* total) {
    const int64_t P = c->d.P, F = c->d.hyper_width;
    const bool affine = c->d.rank < 0;  // no factor vector: the leading stacked rows are theta_mat itself
    int64_t fac = affine ? 0 : (c->net[0].fac_len > c->net[1].fac_len ? c->net[0].fac_len : c->net[1].fac_len);
    int64_t q = c->aff[0].q_total > c->aff[1].q_total ? c->aff[0].q_total : c->aff[1].q_total;
    HyperWs L;
    float* p = reinterpret_cast<float*>(ws);
    auto take = [&](int64_t n) { float* r = p; p += align_up(n, 64); return r; };
    L.h1 = take(P * F);
    L.f = take(P * F);
    L.df = take(P * F);
    L.dz2 = take(P * F);
    L.dz1 = take(P * F);
    {
        int64_t vl = c->net[0].vec_len > c->net[1].vec_len ? c->net[0].vec_len : c->net[1].vec_len;
        L.vecs = take(P * vl);
    }
    L.fac = take(P * fac);
    L.dfac = take(P * fac);
    {  // chunks of the df partials: each network with its own rows per chunk
        L.n_chunk = 0;
        for (int n = 0; n < 2; ++n) {
            const int64_t qn = c->aff[n].q_total;
            const int qw = df_chunk_rows(qn);
            const int nc = (int)((qn + qw - 1) / qw);
            L.n_chunk = nc > L.n_chunk ? nc : L.n_chunk;
        }
    }
    L.df_part = take((int64_t)L.n_chunk * P * F);
    L.mrow = reinterpret_cast<int32_t*>(take(q));
    {
        int wmax = c->d.width > c->d.obs_dim ? c->d.width : c->d.obs_dim;
        L.n_cs = (wmax + DAB_COLS - 1) / DAB_COLS;
        L.da_part = L.n_cs > 1 ? take((int64_t)L.n_cs * P * fac) : nullptr;
    }
    if (total) *total = (int64_t)((char*)p - (char*)ws);
    return L;
}

int64_t hyper_ws_bytes(const morlax_ctx* c) {
    int64_t t = 0;
    hyper_ws_layout(c, nullptr, &t);
    return align_up(t, 256);
}

// ------------------------------------------------------------------------------------------------
// Trunk f(w): h1 = tanh(Wh1 w + bh1), f = tanh(Wh2 h1 + bh2).  One block per preference.
__global__ __launch_bounds__(64) void k_hyper_trunk(const float* __restrict__ hp, const float* __restrict__ w,
                                                   float* __restrict__ h1, float* __restrict__ f, int K, int F,
                                                   int64_t o_wh1, int64_t o_bh1, int64_t o_wh2, int64_t o_bh2) {
    __shared__ float sh[MORLAX_MAX_F];
    const int p = blockIdx.x, j = threadIdx.x;
    if (j < F) {
        float a = hp[o_bh1 + j];
        for (int k = 0; k < K; ++k) a += hp[o_wh1 + (int64_t)j * K + k] * w[p * K + k];
        a = tanhf(a);
        sh[j] = a;
        h1[p * F + j] = a;
    }
    __syncthreads();
    if (j < F) {
        float a = hp[o_bh2 + j];
        for (int i = 0; i < F; ++i) a += hp[o_wh2 + (int64_t)j * F + i] * sh[i];
        f[p * F + j] = tanhf(a);
    }
}

__device__ inline int find_seg(const AffineTable& at, int q) {
    int s = 0;
    while (s + 1 < at.n_seg && q >= at.q0[s + 1]) ++s;
    return s;
}

// Stacked affine map: row q for every preference.  Thread per row with its M row in registers; f[p, :]
// is read through wave-uniform addresses (scalar loads), so the inner product costs no LDS traffic.
template <typename TF>  // type of the leading rows' destination: float factors, or theta_mat (strictly affine form)
__global__ __launch_bounds__(256) void k_hyper_affine(AffineTable at, const float* __restrict__ hp,
                                                     const float* __restrict__ f, TF* __restrict__ fac,
                                                     float* __restrict__ theta_vec, int P, int F,
                                                     int64_t fac_len, int64_t vec_len) {
    const int q = blockIdx.x * 256 + threadIdx.x;
    if (q >= at.q_total) return;
    float m[MORLAX_MAX_F];
    const int s = find_seg(at, q);
    const int64_t loc = q - at.q0[s];
    const float c = hp[at.hp_c[s] + loc];
    const float* mr = hp + at.hp_m[s] + loc * F;
#pragma unroll
    for (int j = 0; j < MORLAX_MAX_F; ++j) m[j] = (j < F) ? mr[j] : 0.f;
    const bool lead = q < fac_len;
    TF* dst_f = fac + q;
    float* dst_v = theta_vec + (q - fac_len);
    auto put = [&](int p, float a) {
        if (lead) dst_f[(int64_t)p * fac_len] = cvt<TF>(a);
        else dst_v[(int64_t)p * vec_len] = a;
    };
    // blockIdx.y takes a run of preferences (one run: more did not pay, the per-thread row of M is reloaded)
    const int per = (P + gridDim.y - 1) / gridDim.y;
    const int p_lo = blockIdx.y * per, p_hi = (p_lo + per < P) ? (p_lo + per) : P;
    if (F == 32) {
        // four preferences per batch: their feature rows (wave-uniform loads) are requested together
        int p = p_lo;
        for (; p + 4 <= p_hi; p += 4) {
            float a[4] = {c, c, c, c};
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float* fp = f + (int64_t)(p + u) * 32;
#pragma unroll
                for (int j = 0; j < 32; ++j) a[u] += m[j] * fp[j];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) put(p + u, a[u]);
        }
        for (; p < p_hi; ++p) {
            const float* fp = f + (int64_t)p * 32;
            float a = c;
#pragma unroll
            for (int j = 0; j < 32; ++j) a += m[j] * fp[j];
            put(p, a);
        }
    } else {
        for (int p = p_lo; p < p_hi; ++p) {
            const float* fp = f + (int64_t)p * F;
            float a = c;
#pragma unroll
            for (int j = 0; j < MORLAX_MAX_F; ++j)
                if (j < F) a += m[j] * fp[j];
            put(p, a);
        }
    }
}

// W_l(p) = W0_l + A_l(p) B_l(p).  A block makes a 64 (d_out) x 128 (d_in) tile of one layer of one
// preference; each thread 4 x 8 outputs with the factor tiles in LDS.
struct MatTiles {
    int32_t tile0[MORLAX_MAX_LAYERS + 1];  // first tile id of each layer
    int32_t tiles_i[MORLAX_MAX_LAYERS];    // tiles along d_in
};

template <typename T>
__global__ __launch_bounds__(256) void k_hyper_materialize(NetDev nd, MatTiles mt, const float* __restrict__ hp,
                                                          const float* __restrict__ fac,
                                                          T* __restrict__ theta_mat, int r) {
    __shared__ float sA[64][MORLAX_MAX_RANK + 1];
    __shared__ float sB[MORLAX_MAX_RANK][128];
    const int p = blockIdx.y;
    int l = 0;
    while (l + 1 < nd.n_layers && (int)blockIdx.x >= mt.tile0[l + 1]) ++l;
    const LayerDev L = nd.layer[l];
    const int tl = blockIdx.x - mt.tile0[l];
    const int o0 = (tl / mt.tiles_i[l]) * 64, i0 = (tl % mt.tiles_i[l]) * 128;
    const float* fp = fac + (int64_t)p * nd.fac_len;
    for (int idx = threadIdx.x; idx < 64 * r; idx += 256) {
        const int oo = idx / r, k = idx % r;
        sA[oo][k] = (o0 + oo < L.d_out) ? fp[L.fac_a + (int64_t)(o0 + oo) * r + k] : 0.f;
    }
    for (int idx = threadIdx.x; idx < r * 128; idx += 256) {
        const int k = idx / 128, ii = idx % 128;
        sB[k][ii] = (i0 + ii < L.d_in) ? fp[L.fac_b + (int64_t)k * L.d_in + i0 + ii] : 0.f;
    }
    __syncthreads();
    const int to = (threadIdx.x / 16) * 4, ti = (threadIdx.x % 16) * 8;
    float acc[4][8];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 8; ++b) acc[a][b] = 0.f;
    for (int k = 0; k < r; ++k) {
        float bv[8], av[4];
#pragma unroll
        for (int b = 0; b < 8; ++b) bv[b] = sB[k][ti + b];
#pragma unroll
        for (int a = 0; a < 4; ++a) av[a] = sA[to + a][k];
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = 0; b < 8; ++b) acc[a][b] += av[a] * bv[b];
    }
    T* dst = theta_mat + (int64_t)p * nd.mat_len + L.mat_off;
    const float* w0 = hp + L.hp_w0;
    const bool vec = (L.d_in % 8 == 0);
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const int o = o0 + to + a;
        if (o >= L.d_out) continue;
        const int64_t base = (int64_t)o * L.d_in + i0 + ti;
        if (vec && i0 + ti + 8 <= L.d_in) {
            float v[8];
#pragma unroll
            for (int b = 0; b < 8; ++b) v[b] = w0[base + b] + acc[a][b];
            store8(dst + base, v);
        } else {
#pragma unroll
            for (int b = 0; b < 8; ++b)
                if (i0 + ti + b < L.d_in) dst[base + b] = cvt<T>(w0[base + b] + acc[a][b]);
        }
    }
}

static void run_trunk_and_affine(const morlax_ctx* c, int net, const float* hp, const float* w,
                                 const HyperWs& L, float* theta_vec_or_null, float* vec_scratch, hipStream_t s) {
    const NetDev& nd = c->net[net];
    const AffineTable& at = c->aff[net];
    const int P = c->d.P, F = c->d.hyper_width;
    k_hyper_trunk<<<P, 64, 0, s>>>(hp, w, L.h1, L.f, c->d.K, F, nd.hp_wh1, nd.hp_bh1, nd.hp_wh2, nd.hp_bh2);
    float* tv = theta_vec_or_null ? theta_vec_or_null : vec_scratch;
    k_hyper_affine<float><<<dim3((at.q_total + 255) / 256, 1), 256, 0, s>>>(at, hp, L.f, L.fac, tv, P, F, nd.fac_len,
                                                                            nd.vec_len);
}

static MatTiles mat_tiles(const NetDev& nd) {
    MatTiles mt;
    int t = 0;
    for (int l = 0; l < nd.n_layers; ++l) {
        mt.tile0[l] = t;
        mt.tiles_i[l] = (nd.layer[l].d_in + 127) / 128;
        t += mt.tiles_i[l] * ((nd.layer[l].d_out + 63) / 64);
    }
    mt.tile0[nd.n_layers] = t;
    return mt;
}

void launch_hypernet_fwd(const morlax_ctx* c, int net, const float* hparams, const float* w,
                         void* theta_mat, float* theta_vec, void* ws, hipStream_t s) {
    const NetDev& nd = c->net[net];
    HyperWs L = hyper_ws_layout(c, ws, nullptr);
    if (c->d.rank < 0) {
        // strictly affine form (Sec. III-B as written): the stacked map writes theta_mat and theta_vec directly
        const AffineTable& at = c->aff[net];
        const int P = c->d.P, F = c->d.hyper_width;
        k_hyper_trunk<<<P, 64, 0, s>>>(hparams, w, L.h1, L.f, c->d.K, F, nd.hp_wh1, nd.hp_bh1, nd.hp_wh2, nd.hp_bh2);
        const dim3 grid((at.q_total + 255) / 256, 1);
        if (c->d.wdtype == 1)
            k_hyper_affine<bf16_t><<<grid, 256, 0, s>>>(at, hparams, L.f, (bf16_t*)theta_mat, theta_vec, P, F, nd.fac_len,
                                                        nd.vec_len);
        else
            k_hyper_affine<float><<<grid, 256, 0, s>>>(at, hparams, L.f, (float*)theta_mat, theta_vec, P, F, nd.fac_len,
                                                       nd.vec_len);
        return;
    }
    run_trunk_and_affine(c, net, hparams, w, L, theta_vec, nullptr, s);
    MatTiles mt = mat_tiles(nd);
    const dim3 grid(mt.tile0[nd.n_layers], c->d.P);
    if (c->d.wdtype == 1)
        k_hyper_materialize<bf16_t><<<grid, 256, 0, s>>>(nd, mt, hparams, L.fac, (bf16_t*)theta_mat, c->d.rank);
    else
        k_hyper_materialize<float><<<grid, 256, 0, s>>>(nd, mt, hparams, L.fac, (float*)theta_mat, c->d.rank);
}

// ------------------------------------------------------------------------------------------------
// Backward.

// dW0_l = sum_p dW_l(p): four consecutive elements per thread, p ascending.
__global__ __launch_bounds__(256) void k_hyper_dbase(NetDev nd, const float* __restrict__ dmat,
                                                    float* __restrict__ dhp, int P) {
    const int64_t e = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (e >= nd.mat_len) return;
    int l = 0;
    while (l + 1 < nd.n_layers && e >= nd.layer[l + 1].mat_off) ++l;
    float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int p = 0; p < P; ++p) {
        const float4 v = *reinterpret_cast<const float4*>(dmat + (int64_t)p * nd.mat_len + e);
        a.x += v.x; a.y += v.y; a.z += v.z; a.w += v.w;
    }
    float* d = dhp + nd.layer[l].hp_w0 + (e - nd.layer[l].mat_off);
    d[0] = a.x; d[1] = a.y; d[2] = a.z; d[3] = a.w;
}

// Fused dA / dB on fp32 MFMA, one pass over dW:
//   dA_l(p)[o, k] = sum_i dW_l(p)[o, i] B_l(p)[k, i],   dB_l(p)[k, i] = sum_o A_l(p)[o, k] dW_l(p)[o, i].
// A block owns (p, layer, a run of <= DAB_COLS columns).  It walks the 64 x 64 tiles of dW row block by row
// block: wave w multiplies rows 16 w .. of the tile by B^T (dA, finished after the columns of a row block)
// and A^T by columns 16 w .. of the tile (dB, accumulated over all row blocks in registers).
struct DabWork {
    int32_t n;
    int16_t layer[DAB_MAX_CS * MORLAX_MAX_LAYERS];
    int16_t cs[DAB_MAX_CS * MORLAX_MAX_LAYERS];
};

template <int RT>
__global__ __launch_bounds__(256) void k_hyper_dAB(NetDev nd, DabWork wk, const float* __restrict__ dmat,
                                                  const float* __restrict__ fac, float* __restrict__ dfac,
                                                  float* __restrict__ da_part, int r, int P) {
    constexpr int AP = 16 * RT + 4;
    __shared__ __align__(16) float sW[64][68];
    __shared__ float sA[64][AP];
    __shared__ float sB[DAB_NCT][16 * RT][68];
    const int p = blockIdx.y;
    const LayerDev L = nd.layer[wk.layer[blockIdx.x]];
    const int cs = wk.cs[blockIdx.x];
    const int c_lo = cs * DAB_COLS;
    const int c_hi = (L.d_in < c_lo + DAB_COLS) ? L.d_in : (c_lo + DAB_COLS);
    const int nct = (c_hi - c_lo + 63) / 64;
    const int n_cs = (L.d_in + DAB_COLS - 1) / DAB_COLS;
    const float* dW = dmat + (int64_t)p * nd.mat_len + L.mat_off;
    const float* Ap = fac + (int64_t)p * nd.fac_len + L.fac_a;
    const float* Bp = fac + (int64_t)p * nd.fac_len + L.fac_b;
    float* dAp = (n_cs > 1 ? da_part + ((int64_t)cs * P + p) * nd.fac_len : dfac + (int64_t)p * nd.fac_len) + L.fac_a;
    float* dBp = dfac + (int64_t)p * nd.fac_len + L.fac_b;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, ln = lane & 15, kg = lane >> 4;
    const bool vec = (L.d_in % 4 == 0);
    float4_t accB[DAB_NCT][RT];
#pragma unroll
    for (int ct = 0; ct < DAB_NCT; ++ct)
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) accB[ct][rt] = float4_t{0.f, 0.f, 0.f, 0.f};
    // The tiles are walked row block by row block; the next tile of dW is fetched into registers while the
    // current one is multiplied out of LDS.
    const int nrb = (L.d_out + 63) / 64, ntile = nrb * nct;
    auto fetch = [&](int tile, float4 (&regs)[4]) {
        const int o0 = (tile / nct) * 64, i0 = c_lo + (tile % nct) * 64;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int idx = threadIdx.x + 256 * q, row = idx / 16, c4 = (idx % 16) * 4;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (o0 + row < L.d_out) {
                const float* src = dW + (int64_t)(o0 + row) * L.d_in + i0 + c4;
                if (vec && i0 + c4 + 4 <= c_hi) {
                    v = *reinterpret_cast<const float4*>(src);
                } else {
                    if (i0 + c4 < c_hi) v.x = src[0];
                    if (i0 + c4 + 1 < c_hi) v.y = src[1];
                    if (i0 + c4 + 2 < c_hi) v.z = src[2];
                    if (i0 + c4 + 3 < c_hi) v.w = src[3];
                }
            }
            regs[q] = v;
        }
    };
    // the block's columns of B(p): the same for every row block
    for (int idx = threadIdx.x; idx < DAB_NCT * 16 * RT * 64; idx += 256) {
        const int ct = idx / (16 * RT * 64), k = (idx / 64) % (16 * RT), cc = idx % 64, i = c_lo + ct * 64 + cc;
        sB[ct][k][cc] = (k < r && i < c_hi) ? Bp[(int64_t)k * L.d_in + i] : 0.f;
    }
    // a row block's rows of A(p), requested one row block ahead
    constexpr int APT = 64 * 16 * RT / 256;
    float anx[APT];
    auto fetch_a = [&](int rb) {
#pragma unroll
        for (int q = 0; q < APT; ++q) {
            const int idx = threadIdx.x + 256 * q, row = idx / (16 * RT), k = idx % (16 * RT);
            anx[q] = (rb * 64 + row < L.d_out && k < r) ? Ap[(int64_t)(rb * 64 + row) * r + k] : 0.f;
        }
    };
    float4 nxt[4];
    fetch(0, nxt);
    fetch_a(0);
    for (int rb = 0; rb < nrb; ++rb) {
        const int o0 = rb * 64;
        __syncthreads();
#pragma unroll
        for (int q = 0; q < APT; ++q) {
            const int idx = threadIdx.x + 256 * q;
            sA[idx / (16 * RT)][idx % (16 * RT)] = anx[q];
        }
        if (rb + 1 < nrb) fetch_a(rb + 1);
        float4_t accA[RT];
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) accA[rt] = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ct = 0; ct < DAB_NCT; ++ct) {
            if (ct < nct) {
                __syncthreads();
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int idx = threadIdx.x + 256 * q;
                    *reinterpret_cast<float4*>(&sW[idx / 16][(idx % 16) * 4]) = nxt[q];
                }
                if (rb * nct + ct + 1 < ntile) fetch(rb * nct + ct + 1, nxt);
                __syncthreads();
#pragma unroll
                for (int kk = 0; kk < 16; ++kk) {
                    const float a = sW[16 * wave + ln][4 * kk + kg];
#pragma unroll
                    for (int rt = 0; rt < RT; ++rt)
                        accA[rt] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, sB[ct][16 * rt + ln][4 * kk + kg], accA[rt], 0, 0, 0);
                }
#pragma unroll
                for (int kk = 0; kk < 16; ++kk) {
                    const int row = 16 * (kk >> 2) + (kk & 3) + 4 * kg;
                    const float b = sW[row][16 * wave + ln];
#pragma unroll
                    for (int rt = 0; rt < RT; ++rt)
                        accB[ct][rt] = __builtin_amdgcn_mfma_f32_16x16x4f32(sA[row][16 * rt + ln], b, accB[ct][rt], 0, 0, 0);
                }
            }
        }
        // dA tile: lane holds factor index 16 rt + ln of rows o0 + 16 wave + 4 kg + e
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int o = o0 + 16 * wave + 4 * kg + e, k = 16 * rt + ln;
                if (o < L.d_out && k < r) dAp[(int64_t)o * r + k] = accA[rt][e];
            }
    }
    // dB tiles: lane holds column i of factor rows 16 rt + 4 kg + e
#pragma unroll
    for (int ct = 0; ct < DAB_NCT; ++ct)
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int i = c_lo + ct * 64 + 16 * wave + ln, k = 16 * rt + 4 * kg + e;
                if (ct < nct && i < c_hi && k < r) dBp[(int64_t)k * L.d_in + i] = accB[ct][rt][e];
            }
}

// dA of layers wider than one column run: add the column-run partials in order.
__global__ __launch_bounds__(256) void k_hyper_dA_merge(NetDev nd, const float* __restrict__ da_part,
                                                       float* __restrict__ dfac, int r, int P) {
    const int p = blockIdx.y;
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    for (int l = 0; l < nd.n_layers; ++l) {
        const LayerDev L = nd.layer[l];
        const int n_cs = (L.d_in + DAB_COLS - 1) / DAB_COLS;
        if (n_cs > 1 && e >= L.fac_a && e < L.fac_a + (int64_t)L.d_out * r) {
            float a = 0.f;
            for (int cs = 0; cs < n_cs; ++cs) a += da_part[((int64_t)cs * P + p) * nd.fac_len + e];
            dfac[(int64_t)p * nd.fac_len + e] = a;
        }
    }
}

__device__ inline float grad_row(const float* __restrict__ dfac, const float* __restrict__ dvec, int64_t p, int q,
                                 int64_t fac_len, int64_t vec_len) {
    return (q < fac_len) ? dfac[p * fac_len + q] : dvec[p * vec_len + (q - fac_len)];
}

// dM[q, :] = sum_p g[p, q] f[p, :],  dc[q] = sum_p g[p, q]  (g: gradient of the stacked affine rows).
// Thread per row, p ascending, f[p, :] through wave-uniform (scalar) loads.
__global__ __launch_bounds__(256) void k_hyper_dM(AffineTable at, const float* __restrict__ f,
                                                 const float* __restrict__ dfac, const float* __restrict__ dvec,
                                                 float* __restrict__ dhp, int P, int F, int64_t fac_len,
                                                 int64_t vec_len) {
    const int q = blockIdx.x * 256 + threadIdx.x;
    if (q >= at.q_total) return;
    float acc[MORLAX_MAX_F];
#pragma unroll
    for (int j = 0; j < MORLAX_MAX_F; ++j) acc[j] = 0.f;
    float dc = 0.f;
    const float* src = (q < fac_len) ? (dfac + q) : (dvec + (q - fac_len));
    const int64_t stride = (q < fac_len) ? fac_len : vec_len;
    if (F == 32) {
        // eight preferences per batch: their (strided, independent) loads are in flight together
        int p = 0;
        for (; p + 8 <= P; p += 8) {
            float g[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) g[u] = src[(int64_t)(p + u) * stride];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const float* fp = f + (int64_t)(p + u) * 32;
                dc += g[u];
#pragma unroll
                for (int j = 0; j < 32; ++j) acc[j] += g[u] * fp[j];
            }
        }
        for (; p < P; ++p) {
            const float g = src[(int64_t)p * stride];
            const float* fp = f + (int64_t)p * 32;
            dc += g;
#pragma unroll
            for (int j = 0; j < 32; ++j) acc[j] += g * fp[j];
        }
    } else {
        for (int p = 0; p < P; ++p) {
            const float g = src[(int64_t)p * stride];
            const float* fp = f + (int64_t)p * F;
            dc += g;
#pragma unroll
            for (int j = 0; j < MORLAX_MAX_F; ++j)
                if (j < F) acc[j] += g * fp[j];
        }
    }
    const int s = find_seg(at, q);
    const int64_t loc = q - at.q0[s];
    dhp[at.hp_c[s] + loc] = dc;
    float* mr = dhp + at.hp_m[s] + loc * F;
#pragma unroll
    for (int j = 0; j < MORLAX_MAX_F; ++j)
        if (j < F) mr[j] = acc[j];
}

// Offset inside hparams of every row of the stacked affine matrix (built once per call).
__global__ __launch_bounds__(256) void k_hyper_mrow(AffineTable at, int32_t* __restrict__ mrow, int F) {
    const int q = blockIdx.x * 256 + threadIdx.x;
    if (q >= at.q_total) return;
    const int s = find_seg(at, q);
    mrow[q] = (int32_t)(at.hp_m[s] + (int64_t)(q - at.q0[s]) * F);
}

// df partials on fp32 MFMA: part[chunk, p, j] = sum over the chunk's qw stacked rows q of g[p, q] M[q, j].
// One wave per chunk; lane (ln, kg) feeds rows p = 16 pt + ln of g and columns j = 16 jt + ln of M for the
// contraction indices q0 + 4 kg + e, e = 0..3 (one MFMA per e).
template <int JT>
__global__ __launch_bounds__(256) void k_hyper_df_part(const float* __restrict__ hp, const int32_t* __restrict__ mrow,
                                                      const float* __restrict__ dfac,
                                                      const float* __restrict__ dvec, float* __restrict__ part,
                                                      int P, int F, int64_t fac_len, int64_t vec_len, int q_total,
                                                      int n_chunk, int qw) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, ln = lane & 15, kg = lane >> 4;
    const int chunk = blockIdx.x * 4 + wave;
    if (chunk >= n_chunk) return;
    const int qa = chunk * qw;
    const int qb = (qa + qw < q_total) ? (qa + qw) : q_total;
    for (int p0 = 0; p0 < P; p0 += 128) {
        float4_t acc[8][JT];
#pragma unroll
        for (int pt = 0; pt < 8; ++pt)
#pragma unroll
            for (int jt = 0; jt < JT; ++jt) acc[pt][jt] = float4_t{0.f, 0.f, 0.f, 0.f};
        for (int q0 = qa; q0 < qb; q0 += 16) {
            float b[JT][4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int q = q0 + 4 * kg + e;
                const int off = (q < qb) ? mrow[q] : 0;
#pragma unroll
                for (int jt = 0; jt < JT; ++jt) {
                    const int j = 16 * jt + ln;
                    b[jt][e] = (q < qb && j < F) ? hp[off + j] : 0.f;
                }
            }
#pragma unroll
            for (int pt = 0; pt < 8; ++pt) {
                const int pp = p0 + 16 * pt + ln;
                if (p0 + 16 * pt < P) {  // uniform
                    float a[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int q = q0 + 4 * kg + e;
                        a[e] = (pp < P && q < qb) ? grad_row(dfac, dvec, pp, q, fac_len, vec_len) : 0.f;
                    }
#pragma unroll
                    for (int e = 0; e < 4; ++e)
#pragma unroll
                        for (int jt = 0; jt < JT; ++jt)
                            acc[pt][jt] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[e], b[jt][e], acc[pt][jt], 0, 0, 0);
                }
            }
        }
        // lane holds column j = 16 jt + ln of rows p = p0 + 16 pt + 4 kg + e
#pragma unroll
        for (int pt = 0; pt < 8; ++pt)
#pragma unroll
            for (int jt = 0; jt < JT; ++jt)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int pp = p0 + 16 * pt + 4 * kg + e, j = 16 * jt + ln;
                    if (pp < P && j < F) part[((int64_t)chunk * P + pp) * F + j] = acc[pt][jt][e];
                }
    }
}

// dM, dc and the df partials in one pass over the gradient g of the stacked affine rows (P <= 128):
//   dM[q, :] = sum_p g[p, q] f[p, :],  dc[q] = sum_p g[p, q] (four interleaved shares of the preferences, each in
//   order, added in a fixed order),  part[wg, p, j] = sum over the workgroup's rows q of g[p, q] M[q, j].
// A workgroup walks DMF_TPW-or-more tiles of 64 rows.  The tile of g (all P preferences x 64 rows, every
// preference's 64 values one 256-byte run) and the tile of M go through LDS and feed fp32 MFMAs twice: wave w
// forms dM of rows 16 w .. 16 w + 15 (contraction over p), and accumulates, across the tiles, the df partial of
// preferences 32 w .. 32 w + 31 (contraction over the tile's rows).  The next tiles of g and M are in flight in
// registers meanwhile.  LDS pitches: g 68 floats (the df read, lane -> preference, is conflict free; the dM read
// shares banks four ways), f and M 16 JT + 16 (conflict free).
#define DMF_Q 64
template <int JT>
__global__ __launch_bounds__(256) void k_hyper_dM_df(AffineTable at, const float* __restrict__ hp,
                                                    const int32_t* __restrict__ mrow, const float* __restrict__ f,
                                                    const float* __restrict__ dfac, const float* __restrict__ dvec,
                                                    float* __restrict__ dhp, float* __restrict__ part, int P, int F,
                                                    int64_t fac_len, int64_t vec_len, int q_total, int n_tiles, int tpw) {
    constexpr int PD = 68, PJ = 16 * JT + 16, PP = 128;
    __shared__ float Dl[PP][PD];
    __shared__ float Fl[PP][PJ];
    __shared__ float Ml[DMF_Q][PJ];
    __shared__ float Cl[4][DMF_Q];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, ln = lane & 15, kg = lane >> 4;
    const int t_lo = blockIdx.x * tpw, t_hi = (t_lo + tpw < n_tiles) ? (t_lo + tpw) : n_tiles;
    // f, zero-padded to 128 preferences and 16 JT features
    for (int idx = threadIdx.x; idx < PP * 16 * JT; idx += 256) {
        const int pp = idx / (16 * JT), j = idx % (16 * JT);
        Fl[pp][j] = (pp < P && j < F) ? f[(int64_t)pp * F + j] : 0.f;
    }
    // a thread's share of a tile of g (row qq = lane of preferences wave, wave + 4, ...) and of the tile of M
    // (piece idx = thread + 256 i of the 64 x 16 JT values), requested one tile ahead
    constexpr int MPT = DMF_Q * 16 * JT / 256;
    float nxt[PP / 4], mnx[MPT];
    auto fetch = [&](int tile) {
        const int q = tile * DMF_Q + lane;
#pragma unroll
        for (int i = 0; i < PP / 4; ++i) {
            const int pp = wave + 4 * i;
            nxt[i] = (pp < P && q < q_total) ? grad_row(dfac, dvec, pp, q, fac_len, vec_len) : 0.f;
        }
#pragma unroll
        for (int i = 0; i < MPT; ++i) {
            const int idx = threadIdx.x + 256 * i, qq = idx / (16 * JT), j = idx % (16 * JT), qm = tile * DMF_Q + qq;
            mnx[i] = (qm < q_total && j < F) ? hp[mrow[qm] + j] : 0.f;
        }
    };
    float4_t accF[2][JT];
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int jt = 0; jt < JT; ++jt) accF[u][jt] = float4_t{0.f, 0.f, 0.f, 0.f};
    if (t_lo < t_hi) fetch(t_lo);
    for (int tile = t_lo; tile < t_hi; ++tile) {
        const int q0 = tile * DMF_Q;
        __syncthreads();  // the previous tile's readers are done (first pass: orders nothing that matters)
        {
            float c = 0.f;  // this wave's share of dc: its preferences in order
#pragma unroll
            for (int i = 0; i < PP / 4; ++i) {
                Dl[wave + 4 * i][lane] = nxt[i];
                c += nxt[i];
            }
            Cl[wave][lane] = c;
        }
#pragma unroll
        for (int i = 0; i < MPT; ++i) {
            const int idx = threadIdx.x + 256 * i;
            Ml[idx / (16 * JT)][idx % (16 * JT)] = mnx[i];
        }
        if (tile + 1 < t_hi) fetch(tile + 1);
        __syncthreads();
        // dM of rows q0 + 16 wave + (0..15): contraction over the preferences
        {
            float4_t accM[JT];
#pragma unroll
            for (int jt = 0; jt < JT; ++jt) accM[jt] = float4_t{0.f, 0.f, 0.f, 0.f};
            const int kmax = (P + 3) / 4;
            for (int kk = 0; kk < kmax; ++kk) {
                const float a = Dl[4 * kk + kg][16 * wave + ln];
#pragma unroll
                for (int jt = 0; jt < JT; ++jt)
                    accM[jt] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, Fl[4 * kk + kg][16 * jt + ln], accM[jt], 0, 0, 0);
            }
            // lane holds feature j = 16 jt + ln of rows q0 + 16 wave + 4 kg + e
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int q = q0 + 16 * wave + 4 * kg + e;
                if (q < q_total) {
                    float* mr = dhp + mrow[q];
#pragma unroll
                    for (int jt = 0; jt < JT; ++jt)
                        if (16 * jt + ln < F) mr[16 * jt + ln] = accM[jt][e];
                }
            }
        }
        // dc: the four waves' shares, in wave order
        if (threadIdx.x < DMF_Q && q0 + (int)threadIdx.x < q_total) {
            const int q = q0 + threadIdx.x;
            const int sg = find_seg(at, q);
            dhp[at.hp_c[sg] + (q - at.q0[sg])] =
                (Cl[0][threadIdx.x] + Cl[1][threadIdx.x]) + (Cl[2][threadIdx.x] + Cl[3][threadIdx.x]);
        }
        // df partial of preferences 32 wave + (0..31): contraction over the tile's rows
#pragma unroll
        for (int kk = 0; kk < DMF_Q / 4; ++kk) {
            float b[JT];
#pragma unroll
            for (int jt = 0; jt < JT; ++jt) b[jt] = Ml[4 * kk + kg][16 * jt + ln];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const float a = Dl[32 * wave + 16 * u + ln][4 * kk + kg];
#pragma unroll
                for (int jt = 0; jt < JT; ++jt)
                    accF[u][jt] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b[jt], accF[u][jt], 0, 0, 0);
            }
        }
    }
    // lane holds feature j = 16 jt + ln of preferences 32 wave + 16 u + 4 kg + e
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int jt = 0; jt < JT; ++jt)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int pp = 32 * wave + 16 * u + 4 * kg + e, j = 16 * jt + ln;
                if (pp < P && j < F) part[((int64_t)blockIdx.x * P + pp) * F + j] = accF[u][jt][e];
            }
}

// df[p, j] = sum_chunk part; dz2 = df * (1 - f^2).  64 outputs per block; the four thread groups take the
// chunks c = g, g + 4, ... and are merged in group order.
__global__ __launch_bounds__(256) void k_hyper_df_final(const float* __restrict__ part, int n_chunk,
                                                       const float* __restrict__ f, float* __restrict__ dz2,
                                                       int PF) {
    __shared__ float red[4][64];
    const int o = threadIdx.x & 63, g = threadIdx.x >> 6;
    const int i = blockIdx.x * 64 + o;
    float a = 0.f;
    if (i < PF) {
        int c = g;
        for (; c + 28 < n_chunk; c += 32) {  // eight chunks of this group per batch, loads in flight together
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = part[(int64_t)(c + 4 * u) * PF + i];
#pragma unroll
            for (int u = 0; u < 8; ++u) a += v[u];
        }
        for (; c < n_chunk; c += 4) a += part[(int64_t)c * PF + i];
    }
    red[g][o] = a;
    __syncthreads();
    if (g == 0 && i < PF) {
        const float fv = f[i];
        dz2[i] = (red[0][o] + red[1][o] + red[2][o] + red[3][o]) * (1.f - fv * fv);
    }
}

// Trunk backward, stage 1: dWh2, dbh2 (sums over p ascending) and dz1 = (dz2 Wh2) * (1 - h1^2).
// One thread per output element.
__global__ __launch_bounds__(256) void k_hyper_trunk_bwd_a(const float* __restrict__ hp, const float* __restrict__ h1,
                                                          const float* __restrict__ dz2, float* __restrict__ dz1,
                                                          float* __restrict__ dhp, int P, int F, int64_t o_wh2,
                                                          int64_t o_bh2) {
    int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx < F * F) {
        const int j = idx / F, i = idx % F;
        float a = 0.f;
        int p = 0;
        for (; p + 8 <= P; p += 8) {
            float x[8], y[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) { x[u] = dz2[(p + u) * F + j]; y[u] = h1[(p + u) * F + i]; }
#pragma unroll
            for (int u = 0; u < 8; ++u) a += x[u] * y[u];
        }
        for (; p < P; ++p) a += dz2[p * F + j] * h1[p * F + i];
        dhp[o_wh2 + idx] = a;
        return;
    }
    idx -= F * F;
    if (idx < F) {
        float a = 0.f;
        int p = 0;
        for (; p + 8 <= P; p += 8) {
            float x[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) x[u] = dz2[(p + u) * F + idx];
#pragma unroll
            for (int u = 0; u < 8; ++u) a += x[u];
        }
        for (; p < P; ++p) a += dz2[p * F + idx];
        dhp[o_bh2 + idx] = a;
        return;
    }
    idx -= F;
    if (idx < P * F) {
        const int p = idx / F, i = idx % F;
        float a = 0.f;
        for (int j = 0; j < F; ++j) a += dz2[p * F + j] * hp[o_wh2 + (int64_t)j * F + i];
        const float h = h1[idx];
        dz1[idx] = a * (1.f - h * h);
    }
}

// Stage 2: dWh1, dbh1 (sums over p ascending).
__global__ __launch_bounds__(256) void k_hyper_trunk_bwd_b(const float* __restrict__ w, const float* __restrict__ dz1,
                                                          float* __restrict__ dhp, int P, int K, int F, int64_t o_wh1,
                                                          int64_t o_bh1) {
    int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx < F * K) {
        const int i = idx / K, k = idx % K;
        float a = 0.f;
        int p = 0;
        for (; p + 8 <= P; p += 8) {
            float x[8], y[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) { x[u] = dz1[(p + u) * F + i]; y[u] = w[(p + u) * K + k]; }
#pragma unroll
            for (int u = 0; u < 8; ++u) a += x[u] * y[u];
        }
        for (; p < P; ++p) a += dz1[p * F + i] * w[p * K + k];
        dhp[o_wh1 + idx] = a;
        return;
    }
    idx -= F * K;
    if (idx < F) {
        float a = 0.f;
        int p = 0;
        for (; p + 8 <= P; p += 8) {
            float x[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) x[u] = dz1[(p + u) * F + idx];
#pragma unroll
            for (int u = 0; u < 8; ++u) a += x[u];
        }
        for (; p < P; ++p) a += dz1[p * F + idx];
        dhp[o_bh1 + idx] = a;
    }
}

void launch_hypernet_bwd(const morlax_ctx* c, int net, const float* hparams, const float* w,
                         const float* dtheta_mat, const float* dtheta_vec, float* dhparams, void* ws,
                         bool kept, hipStream_t s) {
    const NetDev& nd = c->net[net];
    const AffineTable& at = c->aff[net];
    const int P = c->d.P, F = c->d.hyper_width, r = c->d.rank, K = c->d.K;
    HyperWs L = hyper_ws_layout(c, ws, nullptr);
    const bool affine = r < 0;
    // the gradient of the leading stacked rows: of the factor vector, or (strictly affine form) of theta_mat itself
    const float* dlead = affine ? dtheta_mat : L.dfac;
    // kept: the workspace still holds what the forward pass of this network left there (h1, f, the factors)
    if (affine) {
        // only f is needed again; dW0 and dMW come out of the dM pass below (W0 is the constant term of those rows)
        if (!kept)
            k_hyper_trunk<<<P, 64, 0, s>>>(hparams, w, L.h1, L.f, K, F, nd.hp_wh1, nd.hp_bh1, nd.hp_wh2, nd.hp_bh2);
    } else {
        // recompute f and the factors; the theta_vec rows of the affine map land in a scratch nobody reads
        if (!kept) run_trunk_and_affine(c, net, hparams, w, L, nullptr, L.vecs, s);
        k_hyper_dbase<<<(int)((nd.mat_len / 4 + 255) / 256), 256, 0, s>>>(nd, dtheta_mat, dhparams, P);
    }
    if (r > 0) {
        DabWork wk;
        wk.n = 0;
        bool split = false;
        for (int l = 0; l < nd.n_layers; ++l) {
            const int n_cs = (nd.layer[l].d_in + DAB_COLS - 1) / DAB_COLS;
            split |= n_cs > 1;
            for (int cs = 0; cs < n_cs; ++cs) {
                wk.layer[wk.n] = (int16_t)l;
                wk.cs[wk.n] = (int16_t)cs;
                ++wk.n;
            }
        }
        if (r <= 16) k_hyper_dAB<1><<<dim3(wk.n, P), 256, 0, s>>>(nd, wk, dtheta_mat, L.fac, L.dfac, L.da_part, r, P);
        else k_hyper_dAB<2><<<dim3(wk.n, P), 256, 0, s>>>(nd, wk, dtheta_mat, L.fac, L.dfac, L.da_part, r, P);
        if (split)
            k_hyper_dA_merge<<<dim3((int)((nd.fac_len + 255) / 256), P), 256, 0, s>>>(nd, L.da_part, L.dfac, r, P);
    }
    k_hyper_mrow<<<(at.q_total + 255) / 256, 256, 0, s>>>(at, L.mrow, F);
    int n_chunk;
    if (P <= 128) {
        // one pass over the gradient of the stacked rows; at least four tiles per workgroup, about a thousand
        // workgroups at most (never more partial slots than the layout holds)
        const int n_tiles = (at.q_total + DMF_Q - 1) / DMF_Q;
        int tpw = (n_tiles + 1023) / 1024;
        if (tpw < 4) tpw = 4;
        n_chunk = (n_tiles + tpw - 1) / tpw;
        if (F <= 32)
            k_hyper_dM_df<2><<<n_chunk, 256, 0, s>>>(at, hparams, L.mrow, L.f, dlead, dtheta_vec, dhparams, L.df_part, P, F,
                                                     nd.fac_len, nd.vec_len, at.q_total, n_tiles, tpw);
        else
            k_hyper_dM_df<4><<<n_chunk, 256, 0, s>>>(at, hparams, L.mrow, L.f, dlead, dtheta_vec, dhparams, L.df_part, P, F,
                                                     nd.fac_len, nd.vec_len, at.q_total, n_tiles, tpw);
    } else {
        k_hyper_dM<<<(at.q_total + 255) / 256, 256, 0, s>>>(at, L.f, dlead, dtheta_vec, dhparams, P, F, nd.fac_len,
                                                           nd.vec_len);
        const int qw = df_chunk_rows(at.q_total);
        n_chunk = (at.q_total + qw - 1) / qw;
        if (F <= 32)
            k_hyper_df_part<2><<<(n_chunk + 3) / 4, 256, 0, s>>>(hparams, L.mrow, dlead, dtheta_vec, L.df_part, P, F,
                                                                nd.fac_len, nd.vec_len, at.q_total, n_chunk, qw);
        else
            k_hyper_df_part<4><<<(n_chunk + 3) / 4, 256, 0, s>>>(hparams, L.mrow, dlead, dtheta_vec, L.df_part, P, F,
                                                                nd.fac_len, nd.vec_len, at.q_total, n_chunk, qw);
    }
    k_hyper_df_final<<<(P * F + 63) / 64, 256, 0, s>>>(L.df_part, n_chunk, L.f, L.dz2, P * F);
    k_hyper_trunk_bwd_a<<<(F * F + F + P * F + 255) / 256, 256, 0, s>>>(hparams, L.h1, L.dz2, L.dz1, dhparams, P, F,
                                                                       nd.hp_wh2, nd.hp_bh2);
    k_hyper_trunk_bwd_b<<<(F * K + F + 255) / 256, 256, 0, s>>>(w, L.dz1, dhparams, P, K, F, nd.hp_wh1, nd.hp_bh1);
}
