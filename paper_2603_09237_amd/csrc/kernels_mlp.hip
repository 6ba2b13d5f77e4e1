// Grouped target-network forward and backward (paper Sec. III-C rollout and update phases,
// Sec. III-E for the tanh head): every preference p applies its own weights W_l(p) to its own rows.
//
// Rows of preference p in a selection {t0, t_cnt, j0, j_cnt} are numbered m = (t - t0) * j_cnt +
// (j - j0); their home in the time-major tensors is row (t * N + p * n_g + j).  Hidden activations
// live in compact [P][M][W] buffers of the GEMM input type T (fp32 or bf16).
//
// Hidden layers run on MFMA: a 256-thread workgroup owns a 128 x 128 output tile of one preference,
// both operands are staged through LDS as rows of four 16-byte chunks along the contraction axis
// (32 bf16 or 16 fp32 values per step) and each of the four waves accumulates a 64 x 64 sub-tile with
// v_mfma_f32_32x32x16_bf16 / v_mfma_f32_32x32x2_f32.  Operands whose contraction axis is the slow
// axis in memory (W in the dX product, both operands of the dW product) are transposed on the way
// into LDS.  The skinny output layer (<= 16 columns) uses 16x16 MFMA tiles straight from global
// memory in the forward pass and plain vector code in the backward pass.
#include "morlax_internal.h"
#include "numeric.h"

#define BM 128
#define BN 128
#define PITCH 80           // bytes per LDS tile row: four 16-byte chunks + 16 bytes of padding
#define TILE_BYTES (128 * PITCH)
#define OUT_PITCH 16       // floats per row of the saved head output

enum { SRC_KCONTIG = 0, SRC_KSTRIDED = 1, SRC_X_KCONTIG = 2, SRC_X_KSTRIDED = 3 };

struct RowMap {  // compact row m of preference p -> row of a time-major tensor
    int32_t t0, j0, j_cnt, N, n_g;
    __device__ inline int64_t row(int p, int m) const {
        return (int64_t)(t0 + m / j_cnt) * N + (int64_t)p * n_g + j0 + m % j_cnt;
    }
};

template <typename T> struct Elems { static constexpr int VE = 16 / sizeof(T); };

__device__ inline uint32_t pack2(bf16_t a, bf16_t b) {
    return (uint32_t)__builtin_bit_cast(uint16_t, a) | ((uint32_t)__builtin_bit_cast(uint16_t, b) << 16);
}

template <typename T> __device__ inline uint4 pack_chunk(const float* v);
template <> __device__ inline uint4 pack_chunk<float>(const float* v) {
    return make_uint4(__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3]));
}
template <> __device__ inline uint4 pack_chunk<bf16_t>(const float* v) {
    return make_uint4(pack2((bf16_t)v[0], (bf16_t)v[1]), pack2((bf16_t)v[2], (bf16_t)v[3]),
                      pack2((bf16_t)v[4], (bf16_t)v[5]), pack2((bf16_t)v[6], (bf16_t)v[7]));
}

// One GEMM operand: a [rows x Kdim] matrix of which a workgroup stages 128 rows x (4 chunks) per step.
template <typename T, int KIND>
struct Operand {
    const void* base;  // T* (compact kinds) or float* (x kinds), already offset to preference p
    int64_t ld;        // compact: elements between consecutive slow-axis indices; x: obs_dim
    int rows, kdim;    // valid extent
    RowMap rm;
    int p;
    bool vec_ok;       // 16-byte loads allowed (alignment)

    static constexpr int VE = Elems<T>::VE;

    // element (row r of the operand, contraction index k), zero outside the valid extent
    __device__ inline float elem(int r, int k) const {
        if (r >= rows || k >= kdim) return 0.f;
        if (KIND == SRC_KCONTIG) return to_f(reinterpret_cast<const T*>(base)[(int64_t)r * ld + k]);
        if (KIND == SRC_KSTRIDED) return to_f(reinterpret_cast<const T*>(base)[(int64_t)k * ld + r]);
        if (KIND == SRC_X_KCONTIG) return reinterpret_cast<const float*>(base)[rm.row(p, r) * ld + k];
        return reinterpret_cast<const float*>(base)[rm.row(p, k) * ld + r];
    }

    // Stage the tile rows [r0, r0+128) x contraction [k0, k0 + 4*VE) into registers (two chunks).
    __device__ inline void load(int r0, int k0, uint4 regs[2]) const {
        const int tid = threadIdx.x;
        if (KIND == SRC_KCONTIG || KIND == SRC_X_KCONTIG) {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int c = tid + 256 * i, r = r0 + c / 4, k = k0 + (c % 4) * VE;
                if (KIND == SRC_KCONTIG && vec_ok && r < rows && k + VE <= kdim) {
                    regs[i] = *reinterpret_cast<const uint4*>(reinterpret_cast<const T*>(base) + (int64_t)r * ld + k);
                } else if (KIND == SRC_X_KCONTIG && vec_ok && r < rows && k + VE <= kdim) {
                    const float4* src = reinterpret_cast<const float4*>(reinterpret_cast<const float*>(base) +
                                                                        rm.row(p, r) * ld + k);
                    float v[8];
#pragma unroll
                    for (int q = 0; q < VE / 4; ++q) {
                        const float4 f = src[q];
                        v[4 * q] = f.x; v[4 * q + 1] = f.y; v[4 * q + 2] = f.z; v[4 * q + 3] = f.w;
                    }
                    regs[i] = pack_chunk<T>(v);
                } else {
                    float v[8];
#pragma unroll
                    for (int e = 0; e < VE; ++e) v[e] = elem(r, k + e);
                    regs[i] = pack_chunk<T>(v);
                }
            }
        } else if (KIND == SRC_KSTRIDED && sizeof(T) == 2 && vec_ok) {
            // bf16: a thread reads a pair of adjacent rows for 8 consecutive k and splits it into two chunks
            const int r = r0 + 2 * (tid % 64), k = k0 + (tid / 64) * 8;
            uint32_t d[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                d[e] = 0u;
                if (r < rows && k + e < kdim)
                    d[e] = *reinterpret_cast<const uint32_t*>(reinterpret_cast<const T*>(base) + (int64_t)(k + e) * ld + r);
            }
            regs[0] = make_uint4((d[0] & 0xffffu) | (d[1] << 16), (d[2] & 0xffffu) | (d[3] << 16),
                                 (d[4] & 0xffffu) | (d[5] << 16), (d[6] & 0xffffu) | (d[7] << 16));
            regs[1] = make_uint4((d[0] >> 16) | (d[1] & 0xffff0000u), (d[2] >> 16) | (d[3] & 0xffff0000u),
                                 (d[4] >> 16) | (d[5] & 0xffff0000u), (d[6] >> 16) | (d[7] & 0xffff0000u));
        } else {
            // a thread builds chunk (row r, 16 bytes of k) from VE strided loads; adjacent lanes -> adjacent rows
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int r = r0 + tid % 128, k = k0 + (tid / 128 + 2 * i) * VE;
                float v[8];
#pragma unroll
                for (int e = 0; e < VE; ++e) v[e] = elem(r, k + e);
                regs[i] = pack_chunk<T>(v);
            }
        }
    }

    __device__ inline void store(unsigned char* tile, const uint4 regs[2]) const {
        const int tid = threadIdx.x;
        if (KIND == SRC_KCONTIG || KIND == SRC_X_KCONTIG) {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int c = tid + 256 * i;
                *reinterpret_cast<uint4*>(tile + (c / 4) * PITCH + (c % 4) * 16) = regs[i];
            }
        } else if (KIND == SRC_KSTRIDED && sizeof(T) == 2 && vec_ok) {
            const int r = 2 * (tid % 64), kc = tid / 64;
            *reinterpret_cast<uint4*>(tile + r * PITCH + kc * 16) = regs[0];
            *reinterpret_cast<uint4*>(tile + (r + 1) * PITCH + kc * 16) = regs[1];
        } else {
#pragma unroll
            for (int i = 0; i < 2; ++i)
                *reinterpret_cast<uint4*>(tile + (tid % 128) * PITCH + (tid / 128 + 2 * i) * 16) = regs[i];
        }
    }
};

template <typename T> struct Mma32;
template <> struct Mma32<bf16_t> {
    static __device__ inline void run(const uint4& a, const uint4& b, float16_t& c) {
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c,
                                                    0, 0, 0);
    }
};
template <> struct Mma32<float> {
    static __device__ inline void run(const uint4& a, const uint4& b, float16_t& c) {
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), c, 0, 0, 0);
    }
};

__device__ inline float act_fn(float z, int kind) {
    if (kind == 0) return tanhf(z);
    return z / (1.f + expf(-z));
}
__device__ inline float act_grad(float z, int kind) {
    if (kind == 0) {
        const float t = tanhf(z);
        return 1.f - t * t;
    }
    const float s = 1.f / (1.f + expf(-z));
    return s * (1.f + z * (1.f - s));
}

// ---- epilogues: called once per accumulator element with its tile-global (row, col) ------------
template <typename T>
struct EpiFwd {  // h = act(z + b), optionally also act'(z); compact [M][n_cols] stores
    const float* bias;  // [n_cols] of preference p
    T* H;               // compact, offset to p
    typename GradT<T>::type* G;  // nullable
    int ld, act;
    static constexpr bool kColSum = false;
    float* part;  // unused
    __device__ inline float operator()(int r, int c, float v) const {
        const float z = v + bias[c];
        const float h = act_fn(z, act);
        H[(int64_t)r * ld + c] = cvt<T>(h);
        if (G) G[(int64_t)r * ld + c] = cvt<typename GradT<T>::type>(act_grad(z, act));
        return h;
    }
};
template <typename T>
struct EpiDx {  // dZ_{l-1} = (dZ_l W_l) * act'(z_{l-1})
    const typename GradT<T>::type* G;
    T* dZ;
    int ld;
    static constexpr bool kColSum = true;  // column sums of the unrounded dZ feed the bias gradient
    float* part;                           // [P][tiles_m][ld] partial column sums
    __device__ inline float operator()(int r, int c, float v) const {
        const float d = v * to_f(G[(int64_t)r * ld + c]);
        dZ[(int64_t)r * ld + c] = cvt<T>(d);
        return d;
    }
};
struct EpiDw {  // dW_l(p)[o, i]
    float* dW;
    int ld;
    static constexpr bool kColSum = false;
    float* part;  // unused
    __device__ inline float operator()(int r, int c, float v) const {
        dW[(int64_t)r * ld + c] = v;
        return v;
    }
};

template <typename T> __device__ inline void shift_epi(EpiFwd<T>& e, int p, int64_t s0, int64_t s1, int64_t) {
    e.bias += (int64_t)p * s0;
    e.H += (int64_t)p * s1;
    if (e.G) e.G += (int64_t)p * s1;
}
template <typename T> __device__ inline void shift_epi(EpiDx<T>& e, int p, int64_t s0, int64_t, int64_t) {
    e.G += (int64_t)p * s0;
    e.dZ += (int64_t)p * s0;
}
__device__ inline void shift_epi(EpiDw& e, int p, int64_t s0, int64_t, int64_t) { e.dW += (int64_t)p * s0; }

// Logical tile id so that consecutive ids run on the same XCD (workgroups are dealt round-robin to
// the 8 XCDs by hardware id): the tiles of one preference then share that XCD's L2 copy of W(p).
__device__ inline int xcd_remap(int bid, int nb) {
    const int q = nb / 8, rem = nb % 8, x = bid % 8, pos = bid / 8;
    return x * q + (x < rem ? x : rem) + pos;
}

template <typename T, int KA, int KB, class Epi>
struct GemmArgs {
    Operand<T, KA> a;
    Operand<T, KB> b;
    Epi epi;
    int64_t a_pstride, b_pstride;  // per-preference strides (elements of the operand's storage type)
    int64_t e0_pstride, e1_pstride, e2_pstride;
    int tiles_m, tiles_n;
};

// C[rows_a x rows_b] = A[rows_a x K] * B[rows_b x K]^T for every preference.
template <typename T, int KA, int KB, class Epi>
__global__ __launch_bounds__(256) void k_grouped_gemm(GemmArgs<T, KA, KB, Epi> g) {
    __shared__ __align__(16) unsigned char lds[2][2][TILE_BYTES];
    constexpr int VE = Elems<T>::VE;
    constexpr int BK = 4 * VE;
    const int id = xcd_remap(blockIdx.x, gridDim.x);
    const int per_p = g.tiles_m * g.tiles_n;
    const int p = id / per_p, tm = (id % per_p) / g.tiles_n, tn = id % g.tiles_n;

    Operand<T, KA> A = g.a;
    Operand<T, KB> B = g.b;
    A.p = p; B.p = p;
    if (KA == SRC_KCONTIG || KA == SRC_KSTRIDED)
        A.base = reinterpret_cast<const T*>(A.base) + (int64_t)p * g.a_pstride;
    if (KB == SRC_KCONTIG || KB == SRC_KSTRIDED)
        B.base = reinterpret_cast<const T*>(B.base) + (int64_t)p * g.b_pstride;
    Epi epi = g.epi;
    // epilogue pointers are shifted by the caller-provided strides through the specialisations below
    shift_epi(epi, p, g.e0_pstride, g.e1_pstride, g.e2_pstride);

    const int r0 = tm * BM, c0 = tn * BN;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
    const int lr = lane & 31, lg = lane >> 5;

    float16_t acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const int kdim = A.kdim;
    const int nk = (kdim + BK - 1) / BK;
    uint4 ra[2], rb[2];
    A.load(r0, 0, ra);
    B.load(c0, 0, rb);
    A.store(lds[0][0], ra);
    B.store(lds[0][1], rb);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < nk) {
            A.load(r0, (kt + 1) * BK, ra);
            B.load(c0, (kt + 1) * BK, rb);
        }
        const unsigned char* ta = lds[cur][0];
        const unsigned char* tb = lds[cur][1];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const int ch = (2 * ks + lg) * 16;
            uint4 fa[2], fb[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) fa[i] = *reinterpret_cast<const uint4*>(ta + (wm + 32 * i + lr) * PITCH + ch);
#pragma unroll
            for (int j = 0; j < 2; ++j) fb[j] = *reinterpret_cast<const uint4*>(tb + (wn + 32 * j + lr) * PITCH + ch);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) Mma32<T>::run(fa[i], fb[j], acc[i][j]);
        }
        if (kt + 1 < nk) {
            A.store(lds[cur ^ 1][0], ra);
            B.store(lds[cur ^ 1][1], rb);
        }
        __syncthreads();
    }
    // accumulator element e of lane: row 8*(e/4) + 4*(lane/32) + e%4, column lane%32 of its 32x32 tile
    const int rows = A.rows, cols = B.rows;
    float cs[2] = {0.f, 0.f};
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int c = c0 + wn + 32 * j + lr;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int r = r0 + wm + 32 * i + 8 * (e / 4) + 4 * lg + (e % 4);
                if (r < rows && c < cols) cs[j] += epi(r, c, acc[i][j][e]);
            }
        }
    if (Epi::kColSum) {
        // column sums over this tile's 128 rows in a fixed order: lane pair, then the two row waves
        float* red = reinterpret_cast<float*>(&lds[0][0][0]);  // the staging tiles are no longer read
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            cs[j] += __shfl_xor(cs[j], 32, 64);
            if (lg == 0) red[wave * 64 + 32 * j + lr] = cs[j];
        }
        __syncthreads();
        if (threadIdx.x < 128) {
            const int wsel = threadIdx.x >> 6, col = threadIdx.x & 63;
            const float v = red[wsel * 64 + col] + red[(2 + wsel) * 64 + col];
            if (c0 + threadIdx.x < cols)
                epi.part[((int64_t)p * g.tiles_m + tm) * epi.ld + c0 + threadIdx.x] = v;
        }
    }
}

// ---- optional event timing of the GEMM launches ------------------------------------------------
#include <vector>
struct GemmProf {
    struct Rec { hipEvent_t a, b; int kind; double flops; };
    std::vector<Rec> recs;
    size_t used = 0;
    bool on = false;
};

int prof_begin(morlax_ctx* c) {
    if (!c->prof) c->prof = new GemmProf;
    c->prof->used = 0;
    c->prof->on = true;
    return 0;
}

void prof_free(morlax_ctx* c) {
    if (!c->prof) return;
    for (auto& r : c->prof->recs) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
    delete c->prof;
    c->prof = nullptr;
}

int prof_end(morlax_ctx* c, double* ms, int64_t* launches, double* flops) {
    GemmProf* pr = c->prof;
    pr->on = false;
    for (int k = 0; k < MORLAX_GEMM_KINDS; ++k) { ms[k] = 0.0; launches[k] = 0; flops[k] = 0.0; }
    if (pr->used == 0) return 0;
    if (hipEventSynchronize(pr->recs[pr->used - 1].b) != hipSuccess) return -1;
    for (size_t i = 0; i < pr->used; ++i) {
        float t = 0.f;
        if (hipEventElapsedTime(&t, pr->recs[i].a, pr->recs[i].b) != hipSuccess) return -1;
        ms[pr->recs[i].kind] += t;
        launches[pr->recs[i].kind] += 1;
        flops[pr->recs[i].kind] += pr->recs[i].flops;
    }
    pr->used = 0;
    return 0;
}

static GemmProf::Rec* prof_take(const morlax_ctx* c, int kind, double flops) {
    GemmProf* pr = c->prof;
    if (!pr || !pr->on) return nullptr;
    if (pr->used == pr->recs.size()) {
        GemmProf::Rec r;
        if (hipEventCreate(&r.a) != hipSuccess || hipEventCreate(&r.b) != hipSuccess) return nullptr;
        pr->recs.push_back(r);
    }
    GemmProf::Rec* r = &pr->recs[pr->used++];
    r->kind = kind;
    r->flops = flops;
    return r;
}

template <typename T, int KA, int KB, class Epi>
static void run_gemm(const morlax_ctx* c, int kind, GemmArgs<T, KA, KB, Epi>& g, int P, hipStream_t s) {
    g.tiles_m = (g.a.rows + BM - 1) / BM;
    g.tiles_n = (g.b.rows + BN - 1) / BN;
    const int nb = g.tiles_m * g.tiles_n * P;
    GemmProf::Rec* r = prof_take(c, kind, 2.0 * g.a.rows * (double)g.b.rows * g.a.kdim * P);
    if (r) (void)hipEventRecord(r->a, s);
    k_grouped_gemm<T, KA, KB, Epi><<<nb, 256, 0, s>>>(g);
    if (r) (void)hipEventRecord(r->b, s);
}

// ---- output layer ------------------------------------------------------------------------------
template <typename T> struct Mma16;
template <> struct Mma16<bf16_t> {
    static __device__ inline void run(const uint4& a, const uint4& b, float4_t& c) {
        c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c,
                                                    0, 0, 0);
    }
};
template <> struct Mma16<float> {
    static __device__ inline void run(const uint4& a, const uint4& b, float4_t& c) {
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.x), __uint_as_float(b.x), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.y), __uint_as_float(b.y), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.z), __uint_as_float(b.z), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.w), __uint_as_float(b.w), c, 0, 0, 0);
    }
};

// out = head(h W_L(p)^T + b_L(p)); actor: optional sampling a = mu + sigma eps and its log-density.
// A wave owns 16 rows; lane (row = lane % 16, chunk = lane / 16) feeds 16x16 MFMA tiles from global.
template <typename T>
__global__ __launch_bounds__(256) void k_head_fwd(const T* __restrict__ Hin, const T* __restrict__ theta_mat,
                                                 const float* __restrict__ theta_vec, int64_t mat_len,
                                                 int64_t vec_len, int64_t mat_off, int64_t vec_off, int W,
                                                 int out_dim, int M, RowMap rm, int tanh_head,
                                                 float* __restrict__ out, float* __restrict__ saved_out,
                                                 const float* __restrict__ eps, float* __restrict__ act,
                                                 float* __restrict__ logp, int64_t logsig_off) {
    constexpr int VE = Elems<T>::VE;
    const int p = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m0 = (blockIdx.x * 4 + wave) * 16;
    if (m0 >= M) return;
    const int lr = lane & 15, lg = lane >> 4;
    const T* hrow = Hin + ((int64_t)p * M + (m0 + lr)) * W;
    const T* wrow = theta_mat + (int64_t)p * mat_len + mat_off + (int64_t)lr * W;
    const bool a_ok = (m0 + lr) < M, b_ok = lr < out_dim;
    float4_t c = {0.f, 0.f, 0.f, 0.f};
    for (int k0 = 0; k0 < W; k0 += 4 * VE) {
        const int k = k0 + lg * VE;
        uint4 fa = make_uint4(0, 0, 0, 0), fb = make_uint4(0, 0, 0, 0);
        if (a_ok && k < W) fa = *reinterpret_cast<const uint4*>(hrow + k);
        if (b_ok && k < W) fb = *reinterpret_cast<const uint4*>(wrow + k);
        Mma16<T>::run(fa, fb, c);
    }
    // lane holds column lr of rows m0 + 4*lg + e
    const float bias = b_ok ? theta_vec[(int64_t)p * vec_len + vec_off + lr] : 0.f;
    float ls = 0.f, sg = 0.f;
    if (eps && b_ok) {
        ls = theta_vec[(int64_t)p * vec_len + logsig_off + lr];
        sg = expf(ls);
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int m = m0 + 4 * lg + e;
        const bool ok = (m < M) && b_ok;
        const float z = c[e] + bias;
        const float o = tanh_head ? tanhf(z) : z;
        int64_t row = 0;
        if (m < M) row = rm.row(p, m);
        float term = 0.f;
        if (ok) {
            out[row * out_dim + lr] = o;
            if (saved_out) saved_out[((int64_t)p * M + m) * OUT_PITCH + lr] = o;
            if (eps) {
                const float ep = eps[row * out_dim + lr];
                act[row * out_dim + lr] = o + sg * ep;
                term = -0.5f * ep * ep - ls;
            }
        }
        if (eps) {
            term += __shfl_xor(term, 8, 64);
            term += __shfl_xor(term, 4, 64);
            term += __shfl_xor(term, 2, 64);
            term += __shfl_xor(term, 1, 64);
            if (m < M && lr == 0) logp[row] = term - 0.918938533204672742f * (float)out_dim;
        }
    }
}

// dZ_{L-1}[m, i] = (sum_j dz_L[m, j] W_L(p)[j, i]) * act'(z_{L-1})[m, i], dz_L = dout * (1 - mu^2) for the
// tanh head.  Block: 64 rows x 128 columns of one preference; thread: 4 rows x 8 columns.
template <typename T>
__global__ __launch_bounds__(256) void k_head_bwd_dz(const float* __restrict__ dout,
                                                    const float* __restrict__ saved_out,
                                                    const T* __restrict__ theta_mat, int64_t mat_len,
                                                    int64_t mat_off,
                                                    const typename GradT<T>::type* __restrict__ G,
                                                    T* __restrict__ dZ, float* __restrict__ part,
                                                    int W, int out_dim, int M, RowMap rm, int tanh_head) {
    __shared__ float sdz[64][MORLAX_MAX_OUT];
    __shared__ float red[16][128];
    const int p = blockIdx.z, m0 = blockIdx.y * 64, i0 = blockIdx.x * 128;
    for (int idx = threadIdx.x; idx < 64 * MORLAX_MAX_OUT; idx += 256) {
        const int mm = idx / MORLAX_MAX_OUT, j = idx % MORLAX_MAX_OUT;
        float d = 0.f;
        if (m0 + mm < M && j < out_dim) {
            d = dout[rm.row(p, m0 + mm) * out_dim + j];
            if (tanh_head) {
                const float mu = saved_out[((int64_t)p * M + m0 + mm) * OUT_PITCH + j];
                d *= (1.f - mu * mu);
            }
            d = to_f(cvt<T>(d));  // GEMM input rounding
        }
        sdz[mm][j] = d;
    }
    __syncthreads();
    const int tr = (threadIdx.x / 16) * 4, ti = i0 + (threadIdx.x % 16) * 8;
    const bool live = ti < W;
    float acc[4][8];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 8; ++b) acc[a][b] = 0.f;
    const T* wl = theta_mat + (int64_t)p * mat_len + mat_off;
    for (int j = 0; j < out_dim && live; ++j) {
        float wv[8];
#pragma unroll
        for (int b = 0; b < 8; ++b) wv[b] = to_f(wl[(int64_t)j * W + ti + b]);
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const float d = sdz[tr + a][j];
#pragma unroll
            for (int b = 0; b < 8; ++b) acc[a][b] += d * wv[b];
        }
    }
    float cs[8];
#pragma unroll
    for (int b = 0; b < 8; ++b) cs[b] = 0.f;
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const int m = m0 + tr + a;
        if (m >= M || !live) continue;
        const int64_t o = ((int64_t)p * M + m) * W + ti;
        float v[8];
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            v[b] = acc[a][b] * to_f(G[o + b]);
            cs[b] += v[b];
        }
        store8(dZ + o, v);
    }
    // partial column sums of the unrounded dZ over this block's 64 rows (row groups in fixed order)
#pragma unroll
    for (int b = 0; b < 8; ++b) red[threadIdx.x / 16][(threadIdx.x % 16) * 8 + b] = cs[b];
    __syncthreads();
    if (threadIdx.x < 128 && i0 + threadIdx.x < W) {
        float v = 0.f;
#pragma unroll
        for (int q = 0; q < 16; ++q) v += red[q][threadIdx.x];
        part[((int64_t)p * gridDim.y + blockIdx.y) * W + i0 + threadIdx.x] = v;
    }
}

// dW_L(p)[j, i] = sum_m dz_L[m, j] h_{L-1}[m, i] and db_L(p)[j] = sum_m dz_L[m, j].
// Block: 64 columns i of one preference, 4 waves taking rows m = wave, wave + 4, ...; fixed-order merge.
template <typename T>
__global__ __launch_bounds__(256) void k_head_bwd_dw(const float* __restrict__ dout,
                                                    const float* __restrict__ saved_out,
                                                    const T* __restrict__ Hin, float* __restrict__ dtheta_mat,
                                                    float* __restrict__ dtheta_vec, int64_t mat_len,
                                                    int64_t vec_len, int64_t mat_off, int64_t vec_off, int W,
                                                    int out_dim, int M, RowMap rm, int tanh_head) {
    __shared__ float sdr[256][MORLAX_MAX_OUT];  // rounded dz (GEMM input)
    __shared__ float sdu[256][MORLAX_MAX_OUT];  // unrounded dz (bias gradient)
    __shared__ float red[4][MORLAX_MAX_OUT][64];
    const int p = blockIdx.y;
    const int col = threadIdx.x & 63, sub = threadIdx.x >> 6;
    const int i = blockIdx.x * 64 + col;
    float acc[MORLAX_MAX_OUT];
#pragma unroll
    for (int j = 0; j < MORLAX_MAX_OUT; ++j) acc[j] = 0.f;
    float bsum = 0.f;  // thread (j = tid % 16, part = tid / 16) of block x = 0
    for (int m0 = 0; m0 < M; m0 += 256) {
        __syncthreads();
        {
            const int mm = threadIdx.x;
#pragma unroll
            for (int j = 0; j < MORLAX_MAX_OUT; ++j) {
                float d = 0.f;
                if (m0 + mm < M && j < out_dim) {
                    d = dout[rm.row(p, m0 + mm) * out_dim + j];
                    if (tanh_head) {
                        const float mu = saved_out[((int64_t)p * M + m0 + mm) * OUT_PITCH + j];
                        d *= (1.f - mu * mu);
                    }
                }
                sdu[mm][j] = d;
                sdr[mm][j] = to_f(cvt<T>(d));
            }
        }
        __syncthreads();
        if (i < W) {
            for (int mm = sub; mm < 256 && m0 + mm < M; mm += 4) {
                const float h = to_f(Hin[((int64_t)p * M + m0 + mm) * W + i]);
#pragma unroll
                for (int j = 0; j < MORLAX_MAX_OUT; ++j)
                    if (j < out_dim) acc[j] += sdr[mm][j] * h;
            }
        }
        if (blockIdx.x == 0) {
            const int j = threadIdx.x & 15, part = threadIdx.x >> 4;
            for (int mm = part * 16; mm < part * 16 + 16; ++mm) bsum += sdu[mm][j];
        }
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < MORLAX_MAX_OUT; ++j) red[sub][j][col] = acc[j];
    __syncthreads();
    if (sub == 0 && i < W) {
        for (int j = 0; j < out_dim; ++j) {
            const float v = red[0][j][col] + red[1][j][col] + red[2][j][col] + red[3][j][col];
            dtheta_mat[(int64_t)p * mat_len + mat_off + (int64_t)j * W + i] = v;
        }
    }
    if (blockIdx.x == 0) {
        __syncthreads();
        float* r2 = &red[0][0][0];
        r2[threadIdx.x] = bsum;
        __syncthreads();
        if (threadIdx.x < out_dim) {
            float v = 0.f;
            for (int part = 0; part < 16; ++part) v += r2[part * 16 + threadIdx.x];
            dtheta_vec[(int64_t)p * vec_len + vec_off + threadIdx.x] = v;
        }
    }
}

// db_l(p)[o] = sum over the row blocks of the partial column sums of dZ_l, in block order.
__global__ __launch_bounds__(256) void k_colsum_final(const float* __restrict__ part, int n_part,
                                                     float* __restrict__ dtheta_vec, int64_t vec_len,
                                                     int64_t vec_off, int W) {
    const int p = blockIdx.y, i = blockIdx.x * 256 + threadIdx.x;
    if (i >= W) return;
    float a = 0.f;
    for (int q = 0; q < n_part; ++q) a += part[((int64_t)p * n_part + q) * W + i];
    dtheta_vec[(int64_t)p * vec_len + vec_off + i] = a;
}

__global__ void k_copy_dlogsig(const float* __restrict__ dlogsig, float* __restrict__ dtheta_vec, int64_t vec_len,
                               int64_t off, int P, int A) {
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= P * A) return;
    const int p = idx / A, a = idx % A;
    dtheta_vec[(int64_t)p * vec_len + off + a] = dlogsig ? dlogsig[idx] : 0.f;
}

// ---- host side ---------------------------------------------------------------------------------
static int64_t esize(const morlax_ctx* c) { return c->d.wdtype == 1 ? 2 : 4; }
static int64_t act_elems(const morlax_ctx* c, const RowSel& rs) {
    return align_up((int64_t)c->d.P * rs.M * c->d.width, 64);
}

int64_t mlp_saved_bytes(const morlax_ctx* c, int net, const RowSel& rs) {
    (void)net;
    return 2 * (int64_t)c->d.n_hidden * act_elems(c, rs) * esize(c) +
           align_up((int64_t)c->d.P * rs.M * OUT_PITCH * 4, 256);
}
static int64_t part_elems(const morlax_ctx* c, const RowSel& rs) {
    return align_up((int64_t)c->d.P * ((rs.M + 63) / 64) * c->d.width, 64);
}
int64_t mlp_ws_bytes(const morlax_ctx* c, const RowSel& rs) {
    return 2 * act_elems(c, rs) * esize(c) + part_elems(c, rs) * 4;
}

static RowMap make_rowmap(const morlax_ctx* c, const RowSel& rs) {
    RowMap rm;
    rm.t0 = rs.t0; rm.j0 = rs.j0; rm.j_cnt = rs.j_cnt; rm.N = c->d.N; rm.n_g = c->n_g;
    return rm;
}

template <typename T>
static void policy_fwd_t(const morlax_ctx* c, int net, const T* theta_mat, const float* theta_vec, const float* x,
                         const RowSel& rs, float* out, const float* eps, float* act, float* logp, void* saved,
                         void* ws, hipStream_t s) {
    const NetDev& nd = c->net[net];
    const int P = c->d.P, W = c->d.width, M = rs.M, L = c->d.n_hidden, O = c->d.obs_dim;
    const int64_t ae = act_elems(c, rs);
    const RowMap rm = make_rowmap(c, rs);
    T* sv = reinterpret_cast<T*>(saved);
    T* wsT = reinterpret_cast<T*>(ws);
    auto Hbuf = [&](int l) { return sv ? sv + (int64_t)(2 * l) * ae : wsT + (int64_t)(l & 1) * ae; };
    typedef typename GradT<T>::type GT;
    auto Gbuf = [&](int l) { return sv ? reinterpret_cast<GT*>(sv + (int64_t)(2 * l + 1) * ae) : (GT*)nullptr; };
    float* saved_out = sv ? reinterpret_cast<float*>(sv + (int64_t)2 * L * ae) : nullptr;
    constexpr int VE = Elems<T>::VE;
    for (int l = 0; l < L; ++l) {
        const LayerDev& Ld = nd.layer[l];
        EpiFwd<T> ep;
        ep.bias = theta_vec + Ld.vec_off;
        ep.H = Hbuf(l);
        ep.G = Gbuf(l);
        ep.ld = W;
        ep.act = c->d.act;
        if (l == 0) {
            GemmArgs<T, SRC_X_KCONTIG, SRC_KCONTIG, EpiFwd<T>> g;
            g.a.base = x; g.a.ld = O; g.a.rows = M; g.a.kdim = O; g.a.rm = rm; g.a.vec_ok = (O % 4 == 0);
            g.b.base = theta_mat + Ld.mat_off; g.b.ld = O; g.b.rows = W; g.b.kdim = O; g.b.rm = rm;
            g.b.vec_ok = (O % VE == 0);
            g.a_pstride = 0; g.b_pstride = nd.mat_len;
            g.epi = ep; g.e0_pstride = nd.vec_len; g.e1_pstride = (int64_t)M * W; g.e2_pstride = 0;
            run_gemm(c, 0, g, P, s);
        } else {
            GemmArgs<T, SRC_KCONTIG, SRC_KCONTIG, EpiFwd<T>> g;
            g.a.base = Hbuf(l - 1); g.a.ld = W; g.a.rows = M; g.a.kdim = W; g.a.rm = rm; g.a.vec_ok = true;
            g.b.base = theta_mat + Ld.mat_off; g.b.ld = W; g.b.rows = W; g.b.kdim = W; g.b.rm = rm; g.b.vec_ok = true;
            g.a_pstride = (int64_t)M * W; g.b_pstride = nd.mat_len;
            g.epi = ep; g.e0_pstride = nd.vec_len; g.e1_pstride = (int64_t)M * W; g.e2_pstride = 0;
            run_gemm(c, 1, g, P, s);
        }
    }
    const LayerDev& Lh = nd.layer[L];
    const int tanh_head = (net == MORLAX_ACTOR && c->d.mean_tanh) ? 1 : 0;
    const dim3 grid((M + 63) / 64, P);
    k_head_fwd<T><<<grid, 256, 0, s>>>(Hbuf(L - 1), theta_mat, theta_vec, nd.mat_len, nd.vec_len, Lh.mat_off,
                                       Lh.vec_off, W, nd.out_dim, M, rm, tanh_head, out, saved_out, eps, act, logp,
                                       Lh.vec_off + Lh.d_out);
}

template <typename T>
static void policy_bwd_t(const morlax_ctx* c, int net, const T* theta_mat, const float* theta_vec, const float* x,
                         const RowSel& rs, const void* saved, const float* dout, const float* dlogsig,
                         float* dtheta_mat, float* dtheta_vec, void* ws, hipStream_t s) {
    (void)theta_vec;
    const NetDev& nd = c->net[net];
    const int P = c->d.P, W = c->d.width, M = rs.M, L = c->d.n_hidden, O = c->d.obs_dim;
    const int64_t ae = act_elems(c, rs);
    const RowMap rm = make_rowmap(c, rs);
    const T* sv = reinterpret_cast<const T*>(saved);
    T* wsT = reinterpret_cast<T*>(ws);
    auto Hbuf = [&](int l) { return sv + (int64_t)(2 * l) * ae; };
    typedef typename GradT<T>::type GT;
    auto Gbuf = [&](int l) { return reinterpret_cast<const GT*>(sv + (int64_t)(2 * l + 1) * ae); };
    auto dZbuf = [&](int l) { return wsT + (int64_t)(l & 1) * ae; };
    float* part = reinterpret_cast<float*>(wsT + 2 * ae);
    int n_part = (M + 63) / 64;  // row blocks of whichever kernel produced the current dZ
    const float* saved_out = reinterpret_cast<const float*>(sv + (int64_t)2 * L * ae);
    const int tanh_head = (net == MORLAX_ACTOR && c->d.mean_tanh) ? 1 : 0;
    constexpr int VE = Elems<T>::VE;
    const LayerDev& Lh = nd.layer[L];
    // output layer
    k_head_bwd_dw<T><<<dim3((W + 63) / 64, P), 256, 0, s>>>(dout, saved_out, Hbuf(L - 1), dtheta_mat, dtheta_vec,
                                                           nd.mat_len, nd.vec_len, Lh.mat_off, Lh.vec_off, W,
                                                           nd.out_dim, M, rm, tanh_head);
    k_head_bwd_dz<T><<<dim3((W + 127) / 128, (M + 63) / 64, P), 256, 0, s>>>(
        dout, saved_out, theta_mat, nd.mat_len, Lh.mat_off, Gbuf(L - 1), dZbuf(L - 1), part, W, nd.out_dim, M, rm,
        tanh_head);
    for (int l = L - 1; l >= 0; --l) {
        const LayerDev& Ld = nd.layer[l];
        k_colsum_final<<<dim3((W + 255) / 256, P), 256, 0, s>>>(part, n_part, dtheta_vec, nd.vec_len, Ld.vec_off, W);
        EpiDw ew;
        ew.dW = dtheta_mat + Ld.mat_off;
        ew.ld = Ld.d_in;
        if (l > 0) {
            GemmArgs<T, SRC_KSTRIDED, SRC_KSTRIDED, EpiDw> g;
            g.a.base = dZbuf(l); g.a.ld = W; g.a.rows = W; g.a.kdim = M; g.a.rm = rm; g.a.vec_ok = true;
            g.b.base = Hbuf(l - 1); g.b.ld = W; g.b.rows = W; g.b.kdim = M; g.b.rm = rm; g.b.vec_ok = true;
            g.a_pstride = (int64_t)M * W; g.b_pstride = (int64_t)M * W;
            g.epi = ew; g.e0_pstride = nd.mat_len; g.e1_pstride = 0; g.e2_pstride = 0;
            run_gemm(c, 3, g, P, s);
            GemmArgs<T, SRC_KCONTIG, SRC_KSTRIDED, EpiDx<T>> h;
            h.a.base = dZbuf(l); h.a.ld = W; h.a.rows = M; h.a.kdim = W; h.a.rm = rm; h.a.vec_ok = true;
            h.b.base = theta_mat + Ld.mat_off; h.b.ld = W; h.b.rows = W; h.b.kdim = W; h.b.rm = rm; h.b.vec_ok = true;
            h.a_pstride = (int64_t)M * W; h.b_pstride = nd.mat_len;
            h.epi.G = Gbuf(l - 1); h.epi.dZ = dZbuf(l - 1); h.epi.ld = W; h.epi.part = part;
            h.e0_pstride = (int64_t)M * W; h.e1_pstride = 0; h.e2_pstride = 0;
            run_gemm(c, 2, h, P, s);
            n_part = (M + BM - 1) / BM;
        } else {
            GemmArgs<T, SRC_KSTRIDED, SRC_X_KSTRIDED, EpiDw> g;
            g.a.base = dZbuf(0); g.a.ld = W; g.a.rows = W; g.a.kdim = M; g.a.rm = rm; g.a.vec_ok = true;
            g.b.base = x; g.b.ld = O; g.b.rows = O; g.b.kdim = M; g.b.rm = rm; g.b.vec_ok = false;
            g.a_pstride = (int64_t)M * W; g.b_pstride = 0;
            g.epi = ew; g.e0_pstride = nd.mat_len; g.e1_pstride = 0; g.e2_pstride = 0;
            run_gemm(c, 4, g, P, s);
        }
    }
    (void)VE;
    if (net == MORLAX_ACTOR) {
        const int n = P * c->d.act_dim;
        k_copy_dlogsig<<<(n + 255) / 256, 256, 0, s>>>(dlogsig, dtheta_vec, nd.vec_len, Lh.vec_off + Lh.d_out, P,
                                                      c->d.act_dim);
    }
}

void launch_policy_fwd(const morlax_ctx* c, int net, const void* theta_mat, const float* theta_vec,
                       const float* x, const RowSel& rs, float* out, const float* eps, float* act,
                       float* logp, void* saved, void* ws, hipStream_t s) {
    if (c->d.wdtype == 1)
        policy_fwd_t<bf16_t>(c, net, (const bf16_t*)theta_mat, theta_vec, x, rs, out, eps, act, logp, saved, ws, s);
    else
        policy_fwd_t<float>(c, net, (const float*)theta_mat, theta_vec, x, rs, out, eps, act, logp, saved, ws, s);
}

void launch_policy_bwd(const morlax_ctx* c, int net, const void* theta_mat, const float* theta_vec,
                       const float* x, const RowSel& rs, const void* saved, const float* dout,
                       const float* dlogsig, float* dtheta_mat, float* dtheta_vec, void* ws,
                       hipStream_t s) {
    if (c->d.wdtype == 1)
        policy_bwd_t<bf16_t>(c, net, (const bf16_t*)theta_mat, theta_vec, x, rs, saved, dout, dlogsig, dtheta_mat,
                             dtheta_vec, ws, s);
    else
        policy_bwd_t<float>(c, net, (const float*)theta_mat, theta_vec, x, rs, saved, dout, dlogsig, dtheta_mat,
                            dtheta_vec, ws, s);
}
