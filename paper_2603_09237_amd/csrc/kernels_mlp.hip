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
#include <type_traits>

#include "morlax_internal.h"
#include "numeric.h"

#define BM 128
#define BN 128
#define GEMM_NCH 4         // 16-byte chunks of the contraction axis staged per step and operand row
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

// One GEMM operand: a [rows x kdim] matrix of which a workgroup stages 128 rows x NCH 16-byte chunks of
// the contraction axis per step.  FAST = every access is a full, aligned vector (the launcher checks
// the shapes): loads are branch-free, out-of-range rows are clamped to a valid row (their results are
// never stored) and out-of-range contraction indices are masked to zero.  !FAST = element-wise loads
// with bounds checks, used only where a dimension is odd (first layer with an odd observation width).
template <typename T, int KIND, bool FAST, int NCH>
struct Operand {
    const void* base;  // T* (compact kinds) or float* (x kinds), already offset to preference p
    int64_t ld;        // compact: elements between consecutive slow-axis indices; x: obs_dim
    int rows, kdim;    // valid extent
    RowMap rm;
    int p;

    static constexpr int VE = Elems<T>::VE;
    static constexpr int PITCH = NCH * 16 + 16;
    static constexpr int CPT = NCH / 2;  // chunks per thread (128 * NCH / 256)
    static constexpr bool PAIR = (KIND == SRC_KSTRIDED && sizeof(T) == 2 && FAST);

    // FAST: byte offset of the thread's chunk i at contraction index 0, relative to `base`.  Per-preference
    // tensors stay far below 4 GiB (checked by the launcher), so 32-bit offsets on a wave-uniform base do.
    uint32_t voff[CPT];

    __device__ inline float elem(int r, int k) const {
        if (r >= rows || k >= kdim) return 0.f;
        if (KIND == SRC_KCONTIG) return to_f(reinterpret_cast<const T*>(base)[(int64_t)r * ld + k]);
        if (KIND == SRC_KSTRIDED) return to_f(reinterpret_cast<const T*>(base)[(int64_t)k * ld + r]);
        if (KIND == SRC_X_KCONTIG) return reinterpret_cast<const float*>(base)[rm.row(p, r) * ld + k];
        return reinterpret_cast<const float*>(base)[rm.row(p, k) * ld + r];
    }

    // thread -> (tile row, chunk) of its i-th chunk
    __device__ static inline int trow(int i) {
        const int tid = threadIdx.x;
        if (KIND == SRC_KCONTIG || KIND == SRC_X_KCONTIG) return (tid + 256 * i) / NCH;
        if (PAIR) return 2 * (tid % 64);
        return tid % 128;
    }
    __device__ static inline int tchunk(int i) {
        const int tid = threadIdx.x;
        if (KIND == SRC_KCONTIG || KIND == SRC_X_KCONTIG) return (tid + 256 * i) % NCH;
        if (PAIR) return tid / 64 + 4 * (i / 2);  // chunks 2i and 2i+1 of a pair thread share the k range
        return tid / 128 + 2 * i;
    }

    __device__ inline void init(int r0) {
        if (!FAST) return;
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            int r = r0 + trow(i);
            const int lim = PAIR ? rows - 2 : rows - 1;
            r = r < lim ? r : lim;
            if (KIND == SRC_KCONTIG) voff[i] = (uint32_t)((r * (int)ld + tchunk(i) * VE) * (int)sizeof(T));
            else if (KIND == SRC_X_KCONTIG) voff[i] = (uint32_t)((rm.row(p, r) * ld + tchunk(i) * VE) * 4);
            else if (KIND == SRC_KSTRIDED) voff[i] = (uint32_t)((tchunk(i) * VE * (int)ld + r) * (int)sizeof(T));
            else voff[i] = (uint32_t)(r * 4);
        }
    }

    // Raw staging registers per thread: the loads of step k+1 are issued before the products of step k
    // and nothing touches the loaded values until store(), so the load latency overlaps the MFMAs.
    static constexpr bool XSRC = (KIND == SRC_X_KCONTIG || KIND == SRC_X_KSTRIDED);
    static constexpr int RPC = (XSRC && sizeof(T) == 2) ? 2 : 1;  // uint4 registers per chunk (fp32 source of bf16)
    static constexpr int NRAW = FAST ? CPT * RPC : CPT;

    // Issue the loads of contraction range [k0, k0 + NCH * VE).  TAIL = the range may cross kdim: indices
    // are clamped (and the values masked in store()); otherwise addresses are base + uniform + voff.
    template <bool TAIL>
    __device__ inline void load(int r0, int k0, uint4 raw[NRAW]) const {
        if (!FAST) {
#pragma unroll
            for (int i = 0; i < CPT; ++i) {
                const int r = r0 + trow(i), k = k0 + tchunk(i) * VE;
                float v[8];
#pragma unroll
                for (int e = 0; e < VE; ++e) v[e] = elem(r, k + e);
                raw[i] = pack_chunk<T>(v);
            }
            return;
        }
        const char* b = reinterpret_cast<const char*>(base);
        if (KIND == SRC_KCONTIG || KIND == SRC_X_KCONTIG) {
            constexpr int ES = (KIND == SRC_KCONTIG) ? (int)sizeof(T) : 4;
            const char* bk = b + (int64_t)k0 * ES;
#pragma unroll
            for (int i = 0; i < CPT; ++i) {
                const char* src = bk + voff[i];
                if (TAIL && !(k0 + tchunk(i) * VE < kdim)) src = b + voff[i];  // any valid address; masked later
#pragma unroll
                for (int q = 0; q < RPC; ++q) raw[i * RPC + q] = reinterpret_cast<const uint4*>(src)[q];
            }
        } else if (KIND == SRC_KSTRIDED) {
            const int64_t rstep = ld * (int64_t)sizeof(T);  // bytes between consecutive k
            const char* bk = b + (int64_t)k0 * rstep;
#pragma unroll
            for (int i = 0; i < CPT; i += (PAIR ? 2 : 1)) {
                uint32_t d[8];
#pragma unroll
                for (int e = 0; e < (PAIR ? 8 : 4); ++e) {
                    const char* src = bk + e * rstep + voff[i];
                    if (TAIL) {
                        const int kk = k0 + tchunk(i) * VE + e;
                        if (kk >= kdim) src = b + (int64_t)(kdim - 1) * rstep + (voff[i] - (uint32_t)(tchunk(i) * VE) * (uint32_t)rstep);
                    }
                    d[e] = *reinterpret_cast<const uint32_t*>(src);
                }
                raw[i] = make_uint4(d[0], d[1], d[2], d[3]);
                if (PAIR) raw[i + 1] = make_uint4(d[4], d[5], d[6], d[7]);
            }
        } else {
            // x, contraction over rows of the selection: VE consecutive selected rows share one time step
            // (the launcher checks j_cnt % VE == 0), so one row lookup serves the chunk
#pragma unroll
            for (int i = 0; i < CPT; ++i) {
                const int k = k0 + tchunk(i) * VE;
                const int64_t rb = rm.row(p, k < kdim ? k : 0);
                uint32_t d[8];
#pragma unroll
                for (int e = 0; e < VE; ++e)
                    d[e] = *reinterpret_cast<const uint32_t*>(b + (rb + e) * ld * 4 + voff[i]);
                raw[i * RPC] = make_uint4(d[0], d[1], d[2], d[3]);
                if (RPC == 2) raw[i * RPC + 1] = make_uint4(d[4], d[5], d[6], d[7]);
            }
        }
    }

    __device__ static inline uint4 mask4(const uint4& u, bool ok) {
        const uint32_t m = ok ? 0xffffffffu : 0u;
        return make_uint4(u.x & m, u.y & m, u.z & m, u.w & m);
    }

    // Convert / transpose (and with TAIL mask) the staged values of range k0 and write them to the LDS tile.
    template <bool TAIL>
    __device__ inline void store(unsigned char* tile, const uint4 raw[NRAW], int k0) const {
        if (!FAST || KIND == SRC_KCONTIG) {
#pragma unroll
            for (int i = 0; i < CPT; ++i) {
                const bool ok = !FAST || !TAIL || (k0 + tchunk(i) * VE < kdim);
                *reinterpret_cast<uint4*>(tile + trow(i) * PITCH + tchunk(i) * 16) = mask4(raw[i], ok);
            }
        } else if (PAIR) {
#pragma unroll
            for (int i = 0; i < CPT; i += 2) {
                const int k = k0 + tchunk(i) * 8;
                uint32_t d[8] = {raw[i].x, raw[i].y, raw[i].z, raw[i].w, raw[i + 1].x, raw[i + 1].y, raw[i + 1].z, raw[i + 1].w};
                if (TAIL) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) d[e] = (k + e < kdim) ? d[e] : 0u;
                }
                const uint4 lo = make_uint4((d[0] & 0xffffu) | (d[1] << 16), (d[2] & 0xffffu) | (d[3] << 16),
                                            (d[4] & 0xffffu) | (d[5] << 16), (d[6] & 0xffffu) | (d[7] << 16));
                const uint4 hi = make_uint4((d[0] >> 16) | (d[1] & 0xffff0000u), (d[2] >> 16) | (d[3] & 0xffff0000u),
                                            (d[4] >> 16) | (d[5] & 0xffff0000u), (d[6] >> 16) | (d[7] & 0xffff0000u));
                *reinterpret_cast<uint4*>(tile + trow(i) * PITCH + tchunk(i) * 16) = lo;
                *reinterpret_cast<uint4*>(tile + (trow(i) + 1) * PITCH + tchunk(i) * 16) = hi;
            }
        } else if (KIND == SRC_KSTRIDED) {  // fp32, element-wise mask of the contraction tail
#pragma unroll
            for (int i = 0; i < CPT; ++i) {
                const int k = k0 + tchunk(i) * 4;
                uint4 u = raw[i];
                if (TAIL)
                    u = make_uint4(k < kdim ? u.x : 0u, k + 1 < kdim ? u.y : 0u, k + 2 < kdim ? u.z : 0u,
                                   k + 3 < kdim ? u.w : 0u);
                *reinterpret_cast<uint4*>(tile + trow(i) * PITCH + tchunk(i) * 16) = u;
            }
        } else {  // x sources: fp32 -> T, whole chunks in or out of the contraction range
#pragma unroll
            for (int i = 0; i < CPT; ++i) {
                const bool ok = !TAIL || (k0 + tchunk(i) * VE < kdim);
                float v[8];
#pragma unroll
                for (int q = 0; q < RPC; ++q) {
                    const uint4 u = raw[i * RPC + q];
                    v[4 * q] = __uint_as_float(u.x); v[4 * q + 1] = __uint_as_float(u.y);
                    v[4 * q + 2] = __uint_as_float(u.z); v[4 * q + 3] = __uint_as_float(u.w);
                }
                *reinterpret_cast<uint4*>(tile + trow(i) * PITCH + tchunk(i) * 16) = mask4(pack_chunk<T>(v), ok);
            }
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
// h = act(z) and g = act'(z).  SiLU uses the hardware exp2 / reciprocal approximations (about 1 ulp
// each): s = 1 / (1 + e^-z), h = z s, g = s (1 + z - h).  tanh keeps the library routine.
template <int ACT>
__device__ inline void act_pair(float z, float& h, float& g) {
    if (ACT == 0) {
        h = tanhf(z);
        g = 1.f - h * h;
    } else {
        const float e = __expf(-z);
        const float s = __builtin_amdgcn_rcpf(1.f + e);
        h = z * s;
        g = s * (1.f + z - h);
    }
}

// eight consecutive elements of type T / of the saved-derivative type: packing and 16-byte accesses
struct Pack8 { uint4 lo, hi; };  // bf16 / fixed point use lo only; fp32 uses both
__device__ inline Pack8 pack8(const float v[8], const float*) {
    Pack8 r;
    r.lo = make_uint4(__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3]));
    r.hi = make_uint4(__float_as_uint(v[4]), __float_as_uint(v[5]), __float_as_uint(v[6]), __float_as_uint(v[7]));
    return r;
}
__device__ inline Pack8 pack8(const float v[8], const bf16_t*) {
    Pack8 r;
    r.lo = pack_chunk<bf16_t>(v);
    r.hi = make_uint4(0, 0, 0, 0);
    return r;
}
__device__ inline Pack8 pack8(const float v[8], const gfix16_t*) {
    // round(v / step + 1/8 / step); values are in (-0.125, 1.125) so the conversion cannot overflow
    uint32_t q[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) q[i] = (uint32_t)(v[i] * (1.0f / GFIX_STEP) + (0.125f / GFIX_STEP + 0.5f));
    Pack8 r;
    r.lo = make_uint4(q[0] | (q[1] << 16), q[2] | (q[3] << 16), q[4] | (q[5] << 16), q[6] | (q[7] << 16));
    r.hi = make_uint4(0, 0, 0, 0);
    return r;
}
__device__ inline void put8(float* dst, const Pack8& pk) {
    reinterpret_cast<uint4*>(dst)[0] = pk.lo;
    reinterpret_cast<uint4*>(dst)[1] = pk.hi;
}
__device__ inline void put8(bf16_t* dst, const Pack8& pk) { *reinterpret_cast<uint4*>(dst) = pk.lo; }
__device__ inline void put8(gfix16_t* dst, const Pack8& pk) { *reinterpret_cast<uint4*>(dst) = pk.lo; }
__device__ inline void get8(const float* src, float v[8]) {
    const float4 a = reinterpret_cast<const float4*>(src)[0], b = reinterpret_cast<const float4*>(src)[1];
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
__device__ inline void unpack8(const uint4& u, float v[8]) {  // eight fixed-point derivatives
    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        v[2 * i] = (float)(w[i] & 0xffffu) * GFIX_STEP - 0.125f;
        v[2 * i + 1] = (float)(w[i] >> 16) * GFIX_STEP - 0.125f;
    }
}
__device__ inline void get8(const gfix16_t* src, float v[8]) {
    const uint4 u = *reinterpret_cast<const uint4*>(src);
    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        v[2 * i] = (float)(w[i] & 0xffffu) * GFIX_STEP - 0.125f;
        v[2 * i + 1] = (float)(w[i] >> 16) * GFIX_STEP - 0.125f;
    }
}

// ---- epilogues.  A lane owns, for each of its 8 "octets", row r and the eight consecutive columns
// c .. c+7 (c a multiple of 8).  compute() turns the accumulators into results (left in v[], used for
// the column sums) and packs what will be stored; flush() issues the stores.  The kernel calls
// compute() for all octets first and then all flush()es back to back, so that the pieces of a cache
// line leave the wave together. ---------------------------------------------------------------------
template <typename T, int ACT, bool SAVE>
struct EpiFwd {  // h = act(z + b) and, when SAVE, act'(z); compact [M][ld] stores
    const float* bias;  // [ld] of preference p
    T* H;               // compact, offset to p
    typename GradT<T>::type* G;  // used when SAVE
    int ld;
    static constexpr bool kColSum = false;
    float* part;  // unused
    struct Out { Pack8 h, g; };
    __device__ inline void compute(int r, int c, int n, float v[8], Out& o) const {
        (void)r; (void)n;  // ld is a multiple of 16, so an octet is never cut
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] += bias[c + i];
        compute_biased(v, o);
    }
    __device__ inline void compute_biased(float v[8], Out& o) const {  // v already holds z + b
        float g[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) act_pair<ACT>(v[i], v[i], g[i]);
        o.h = pack8(v, (const T*)nullptr);
        if (SAVE) o.g = pack8(g, (const typename GradT<T>::type*)nullptr);
    }
    static constexpr bool kBias = true;  // the persistent kernel stages the tile's bias slice in LDS
    static constexpr bool kPrefetch = false;
    __device__ inline void flush(int r, int c, int n, const Out& o) const {
        (void)n;
        put8(H + (int64_t)r * ld + c, o.h);
        if (SAVE) put8(G + (int64_t)r * ld + c, o.g);
    }
    // row-contiguous stores through an LDS patch (see the kernel): arrays, element size, row-0 address
    static constexpr bool kStage = true;
    static constexpr bool kStagePers = true;
    static constexpr int kArrays = SAVE ? 2 : 1;
    static constexpr int kES = (int)sizeof(T);
    __device__ inline char* arr(int a) const { return a == 0 ? reinterpret_cast<char*>(H) : reinterpret_cast<char*>(G); }
    __device__ static inline const Pack8& pk(const Out& o, int a) { return a == 0 ? o.h : o.g; }
};
template <typename T>
struct EpiDx {  // dZ_{l-1} = (dZ_l W_l) * act'(z_{l-1})
    const typename GradT<T>::type* G;
    T* dZ;
    int ld;
    static constexpr bool kColSum = true;  // column sums of the unrounded dZ feed the bias gradient
    float* part;                           // [P][tiles_m][ld] partial column sums
    struct Out { Pack8 d; };
    __device__ inline void compute(int r, int c, int n, float v[8], Out& o) const {
        (void)n;
        float g[8];
        get8(G + (int64_t)r * ld + c, g);
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] *= g[i];
        o.d = pack8(v, (const T*)nullptr);
    }
    __device__ inline void flush(int r, int c, int n, const Out& o) const {
        (void)n;
        put8(dZ + (int64_t)r * ld + c, o.d);
    }
    // the persistent kernel (bf16) fetches the derivatives of a 32-row block one block ahead of their use
    static constexpr bool kPrefetch = std::is_same<T, bf16_t>::value;
    __device__ inline uint4 fetch(int r, int c) const { return *reinterpret_cast<const uint4*>(G + (int64_t)r * ld + c); }
    __device__ inline void compute_fetched(const uint4& gq, float v[8], Out& o) const {
        float g[8];
        unpack8(gq, g);
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] *= g[i];
        o.d = pack8(v, (const T*)nullptr);
    }
    static constexpr bool kStage = false;  // direct 16-byte stores measured faster in the 128 x 128 kernels,
    static constexpr bool kStagePers = true;  // row-contiguous staged stores in the persistent one
    static constexpr bool kBias = false;
    static constexpr int kArrays = 1;
    static constexpr int kES = (int)sizeof(T);
    __device__ inline char* arr(int) const { return reinterpret_cast<char*>(dZ); }
    __device__ static inline const Pack8& pk(const Out& o, int) { return o.d; }
};
struct EpiDw {  // dW_l(p)[o, i]
    float* dW;
    int ld;
    static constexpr bool kColSum = false;
    float* part;  // unused
    struct Out { Pack8 w; };
    __device__ inline void compute(int r, int c, int n, float v[8], Out& o) const {
        (void)r; (void)c; (void)n;
        o.w = pack8(v, (const float*)nullptr);
    }
    __device__ inline void flush(int r, int c, int n, const Out& o) const {
        float* d = dW + (int64_t)r * ld + c;
        if (n == 8 && (ld & 3) == 0) {
            put8(d, o.w);
        } else {
            const uint32_t w[8] = {o.w.lo.x, o.w.lo.y, o.w.lo.z, o.w.lo.w, o.w.hi.x, o.w.hi.y, o.w.hi.z, o.w.hi.w};
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (i < n) d[i] = __uint_as_float(w[i]);
        }
    }
    static constexpr bool kStage = false;
    static constexpr bool kStagePers = false;
    static constexpr bool kBias = false;
    static constexpr bool kPrefetch = false;
    static constexpr int kArrays = 1;
    static constexpr int kES = 4;
    __device__ inline char* arr(int) const { return reinterpret_cast<char*>(dW); }
    __device__ static inline const Pack8& pk(const Out& o, int) { return o.w; }
};

template <typename T, int ACT, bool SAVE>
__device__ inline void shift_epi(EpiFwd<T, ACT, SAVE>& e, int p, int64_t s0, int64_t s1, int64_t) {
    e.bias += (int64_t)p * s0;
    e.H += (int64_t)p * s1;
    if (SAVE) e.G += (int64_t)p * s1;
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

// One step of the pairwise fold of per-lane slot arrays: lanes whose bit H of lr is set keep the upper H
// slots, the others the lower H, and each adds what its partner (lr ^ H) held for the kept slots.
template <int H>
__device__ inline void fold_slots(float* cs, int lr) {
    const bool up = (lr & H) != 0;
#pragma unroll
    for (int t = 0; t < H; ++t) {
        const float send = up ? cs[t] : cs[t + H];
        const float keep = up ? cs[t + H] : cs[t];
        cs[t] = keep + __shfl_xor(send, H, 64);
    }
}

// ---- epilogue shared by the grouped GEMM kernels.  `lds0` is the workgroup's LDS, free for reuse (at
// least 36 KB); all four waves call this after a barrier.
template <class Epi>
__device__ inline void gemm_epilogue(const Epi& epi, float16_t (&acc)[2][2], unsigned char* lds0, int p, int tm,
                                     int tiles_m, int r0, int c0, int rows, int cols) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
    const int lr = lane & 31, lg = lane >> 5;
    // The products were issued with the operands swapped, so each 32x32 accumulator holds the transposed
    // tile: lane (lr, lg) owns output row lr; with the row permutation of the B fragments its 16 values
    // are the columns 16 h + 8 lg + 0..7 for h = 0, 1 (accumulator elements 8 h .. 8 h + 7) -- one 16-byte
    // bf16 access per octet, and the two lane groups of a row together fill 32 contiguous bytes.
    float cs[Epi::kColSum ? 32 : 1];
    // kStage epilogues send their stores through a per-wave LDS patch (32 rows x 64 columns) so that every
    // store instruction writes whole 128-byte (bf16) or 256-byte (fp32) row segments instead of 32 bytes in
    // each of 32 rows; with two output arrays per tile that measured faster, with one it did not.
    constexpr int ES = Epi::kES;
    constexpr int WP = 64 * ES + 16;            // patch pitch in bytes
    constexpr int PPR = 64 * ES / 16;           // 16-byte pieces per patch row
    constexpr int NB = Epi::kStage ? 4 : 2;     // octets computed before their stores are issued
    unsigned char* patch = lds0 + wave * (32 * WP);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int r = r0 + wm + 32 * i + lr;
#pragma unroll
        for (int jb = 0; jb < 4 / NB; ++jb) {
            typename Epi::Out outs[NB];
#pragma unroll
            for (int o = 0; o < NB; ++o) {
                const int j = (NB == 4) ? (o >> 1) : jb, h = o & 1;
                const int c = c0 + wn + 32 * j + 16 * h + 8 * lg;
                float v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) v[u] = acc[i][j][8 * h + u];
                const bool ok = (r < rows) && (c < cols);
                // out-of-range octets are computed on a clamped, valid position and not stored
                const int rc = r < rows ? r : rows - 1;
                const int cc = c < cols ? c : 0;
                epi.compute(rc, cc, 8, v, outs[o]);
                if (Epi::kColSum) {
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const int t = Epi::kColSum ? (16 * j + 8 * h + u) : 0;
                        cs[t] = (i == 0 ? 0.f : cs[t]) + (ok ? v[u] : 0.f);
                    }
                }
            }
            if (Epi::kStage) {
#pragma unroll
                for (int a = 0; a < Epi::kArrays; ++a) {
#pragma unroll
                    for (int o = 0; o < NB; ++o) {
                        unsigned char* dst = patch + lr * WP + (32 * (o >> 1) + 16 * (o & 1) + 8 * lg) * ES;
                        const Pack8& pk = Epi::pk(outs[o], a);
                        *reinterpret_cast<uint4*>(dst) = pk.lo;
                        if (ES == 4) *reinterpret_cast<uint4*>(dst + 16) = pk.hi;
                    }
                    __builtin_amdgcn_wave_barrier();
                    char* base = epi.arr(a);
#pragma unroll
                    for (int it = 0; it < 32 * PPR / 64; ++it) {
                        const int q = it * 64 + lane, prow = q / PPR, pc = q % PPR;
                        const uint4 u = *reinterpret_cast<const uint4*>(patch + prow * WP + pc * 16);
                        const int gr = r0 + wm + 32 * i + prow, gc = c0 + wn + pc * (16 / ES);
                        if (gr < rows && gc < cols)
                            *reinterpret_cast<uint4*>(base + ((int64_t)gr * epi.ld + gc) * ES) = u;
                    }
                    __builtin_amdgcn_wave_barrier();
                }
            } else {
#pragma unroll
                for (int o = 0; o < NB; ++o) {
                    const int c = c0 + wn + 32 * jb + 16 * (o & 1) + 8 * lg;
                    if (r < rows && c < cols) epi.flush(r, c, (cols - c < 8) ? (cols - c) : 8, outs[o]);
                }
            }
        }
    }
    if (Epi::kColSum) {
        // Column sums over the tile's 128 rows, fixed order.  Slot t = 16 j + 8 h + u of a lane is column
        // wn + 32 j + 16 h + 8 lg + u; the 32 lanes of a half-wave (same lg) fold their 32 slots pairwise so
        // that lane lr ends up with the half-wave total of slot lr.
        fold_slots<16>(cs, lr);
        fold_slots<8>(cs, lr);
        fold_slots<4>(cs, lr);
        fold_slots<2>(cs, lr);
        fold_slots<1>(cs, lr);
        float* red = reinterpret_cast<float*>(lds0 + 4 * 32 * WP);  // behind the store patches
        {
            const int j = lr >> 4, h = (lr >> 3) & 1, u = lr & 7;
            red[wave * 64 + 32 * j + 16 * h + 8 * lg + u] = cs[0];
        }
        __syncthreads();
        if (threadIdx.x < 128) {
            const int wsel = threadIdx.x >> 6, col = threadIdx.x & 63;
            const float v = red[wsel * 64 + col] + red[(2 + wsel) * 64 + col];
            if (c0 + threadIdx.x < cols)
                epi.part[((int64_t)p * tiles_m + tm) * epi.ld + c0 + threadIdx.x] = v;
        }
    }
}

template <typename T, int KA, int KB, class Epi, bool FAST, int NCH>
struct GemmArgs {
    Operand<T, KA, FAST, NCH> a;
    Operand<T, KB, FAST, NCH> b;
    Epi epi;
    int64_t a_pstride, b_pstride;  // per-preference strides (elements of the operand's storage type)
    int64_t e0_pstride, e1_pstride, e2_pstride;
    int tiles_m, tiles_n;
};

// C[rows_a x rows_b] = A[rows_a x K] * B[rows_b x K]^T for every preference.
template <typename T, int KA, int KB, class Epi, bool FAST, int NCH>
__global__ __launch_bounds__(256) void k_grouped_gemm(GemmArgs<T, KA, KB, Epi, FAST, NCH> g) {
    constexpr int PITCH = NCH * 16 + 16;
    constexpr int TILE = 128 * PITCH;
    constexpr int CPT = NCH / 2;
    __shared__ __align__(16) unsigned char lds[2][2][TILE];
    constexpr int VE = Elems<T>::VE;
    constexpr int BK = NCH * VE;
    const int id = xcd_remap(blockIdx.x, gridDim.x);
    const int per_p = g.tiles_m * g.tiles_n;
    const int p = id / per_p, tm = (id % per_p) / g.tiles_n, tn = id % g.tiles_n;

    Operand<T, KA, FAST, NCH> A = g.a;
    Operand<T, KB, FAST, NCH> B = g.b;
    A.p = p; B.p = p;
    if (KA == SRC_KCONTIG || KA == SRC_KSTRIDED)
        A.base = reinterpret_cast<const T*>(A.base) + (int64_t)p * g.a_pstride;
    if (KB == SRC_KCONTIG || KB == SRC_KSTRIDED)
        B.base = reinterpret_cast<const T*>(B.base) + (int64_t)p * g.b_pstride;
    Epi epi = g.epi;
    shift_epi(epi, p, g.e0_pstride, g.e1_pstride, g.e2_pstride);

    const int r0 = tm * BM, c0 = tn * BN;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
    const int lr = lane & 31, lg = lane >> 5;
    // B rows are fed to the MFMA with bits 2 and 3 of the row index swapped, which makes every lane's
    // accumulators cover two runs of eight consecutive output columns (see the epilogue)
    const int lrp = (lr & 0x13) | ((lr & 4) << 1) | ((lr & 8) >> 1);
    A.init(r0);
    B.init(c0);

    float16_t acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const int kdim = A.kdim;
    const int nk = (kdim + BK - 1) / BK;
    // Register stage + two LDS stages: the loads of step kt+1 are in flight while step kt is multiplied
    // out of LDS; they are converted and written to the other LDS stage after the products.  Only the last
    // step can cross the end of the contraction range; it alone runs the clamped / masked loader.
    constexpr int NRA = Operand<T, KA, FAST, NCH>::NRAW, NRB = Operand<T, KB, FAST, NCH>::NRAW;
    uint4 ra[NRA], rb[NRB];
    const int nfull = kdim / BK;  // steps [0, nfull) are entirely inside the contraction range
    if (nfull > 0) {
        A.template load<false>(r0, 0, ra);
        B.template load<false>(c0, 0, rb);
        A.template store<false>(lds[0][0], ra, 0);
        B.template store<false>(lds[0][1], rb, 0);
    } else {
        A.template load<true>(r0, 0, ra);
        B.template load<true>(c0, 0, rb);
        A.template store<true>(lds[0][0], ra, 0);
        B.template store<true>(lds[0][1], rb, 0);
    }
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        const bool more = kt + 1 < nk, full = kt + 1 < nfull;
        if (full) {
            A.template load<false>(r0, (kt + 1) * BK, ra);
            B.template load<false>(c0, (kt + 1) * BK, rb);
        } else if (more) {
            A.template load<true>(r0, (kt + 1) * BK, ra);
            B.template load<true>(c0, (kt + 1) * BK, rb);
        }
        const unsigned char* ta = lds[cur][0] + (wm + lr) * PITCH + lg * 16;
        const unsigned char* tb = lds[cur][1] + (wn + lrp) * PITCH + lg * 16;
#pragma unroll
        for (int ks = 0; ks < NCH / 2; ++ks) {
            uint4 fa[2], fb[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) fa[i] = *reinterpret_cast<const uint4*>(ta + 32 * i * PITCH + ks * 32);
#pragma unroll
            for (int j = 0; j < 2; ++j) fb[j] = *reinterpret_cast<const uint4*>(tb + 32 * j * PITCH + ks * 32);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) Mma32<T>::run(fb[j], fa[i], acc[i][j]);  // transposed tile
        }
        if (full) {
            A.template store<false>(lds[cur ^ 1][0], ra, (kt + 1) * BK);
            B.template store<false>(lds[cur ^ 1][1], rb, (kt + 1) * BK);
        } else if (more) {
            A.template store<true>(lds[cur ^ 1][0], ra, (kt + 1) * BK);
            B.template store<true>(lds[cur ^ 1][1], rb, (kt + 1) * BK);
        }
        __syncthreads();
    }
    gemm_epilogue(epi, acc, &lds[0][0][0], p, tm, g.tiles_m, r0, c0, A.rows, B.rows);
}

// ---- bf16 grouped GEMM with direct-to-LDS loads ------------------------------------------------
// Same tiles, wave layout and epilogues as k_grouped_gemm, for bf16 operands whose shapes need no
// masking (the launcher checks them).  Operand tiles go from global memory straight into LDS, 16 bytes
// per lane, DMA_NST - 1 contraction steps ahead of the products, so that the latency of a load from HBM
// is covered by several steps of MFMAs instead of one.  A DMA instruction fills 1 KB of LDS, lane l
// writing bytes 16 l .. 16 l + 15 of it; which global chunk a lane fetches is free, and that is where
// the bank swizzles below are applied.
//   SRC_KCONTIG  operand, stage = 128 rows x 4 chunks (8 contraction indices each): chunk (r, c) sits at
//                position 4 r + (c ^ swz(r)); fragments are read with one 16-byte LDS read.
//   SRC_KSTRIDED operand (global [k][row]), stage = 32 k x 16 chunks (8 rows each): chunk (k, ic) sits at
//                position 16 k + (ic ^ 4 (k & 3)); fragments are read with two transposing 8-byte reads,
//                each of which hands lane b of a 16-lane group the elements [k0 .. k0+3][row b] of the
//                4 x 16 block whose 64-bit words the lanes 4 e + c (k = k0 + e, rows 4 c .. 4 c + 3) address.
#define DMA_NST 4
#define DMA_STAGE_BYTES 16384  // A tile 8 KB, then B tile 8 KB

typedef short short4_t __attribute__((ext_vector_type(4)));

// The LDS has 64 banks of 4 bytes: it serves 16 lanes of a 16-byte read, or 32 lanes of an 8-byte read,
// per cycle, and the lanes of such a group must touch distinct slots modulo 256 bytes.  With 64-byte rows,
// rows r .. r+3 fill one 256-byte window, so the chunk index is XORed with bits 2, 3 of the row; the
// K-strided tiles XOR bits 2, 3 of the chunk index with the contraction index modulo 4.
__device__ inline int swz_rk(int r) { return (r >> 2) & 3; }

template <int KIND>
struct DmaOperand {
    const char* base;   // per-preference base, bytes
    uint32_t voff[2];   // lane offsets of its two DMA instructions per stage
    int64_t kstep;      // bytes per contraction step (32 indices)
    uint32_t roff;      // lane's LDS byte offset of fragment (block 0, ks 0) within the operand's stage tile

    __device__ inline void init(const bf16_t* b, int ld, int rows, int t0, int wbase, bool brole) {
        base = reinterpret_cast<const char*>(b);
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int j = 2 * wave + i;
            if (KIND == SRC_KCONTIG) {
                const int row = 16 * j + lane / 4, c = (lane % 4) ^ swz_rk(row);
                int gr = t0 + row;
                gr = gr < rows ? gr : rows - 1;
                voff[i] = (uint32_t)((gr * ld + 8 * c) * 2);
            } else {
                const int k = 4 * j + lane / 16, ic = (lane % 16) ^ (4 * (k & 3));
                int gr = t0 + 8 * ic;
                gr = gr < rows - 8 ? gr : rows - 8;
                voff[i] = (uint32_t)((k * ld + gr) * 2);
            }
        }
        kstep = (KIND == SRC_KCONTIG) ? 64 : (int64_t)64 * ld;
        const int lr = lane & 31, lg = lane >> 5;
        if (KIND == SRC_KCONTIG) {
            const int rr = brole ? ((lr & 0x13) | ((lr & 4) << 1) | ((lr & 8) >> 1)) : lr;
            const int row = wbase + rr;
            roff = (uint32_t)(row * 64 + ((lg ^ swz_rk(row)) * 16));
        } else {
            const int a = lane & 15, q0 = (lane >> 4) & 1, e = a >> 2, c = a & 3;
            const int cs = brole ? (((c & 1) << 1) | (c >> 1)) : c;
            const int col = wbase + 16 * q0 + 4 * cs, k = 8 * lg + e;
            roff = (uint32_t)((k * 16 + ((col >> 3) ^ (4 * (k & 3)))) * 16 + ((col >> 2) & 1) * 8);
        }
    }
    // issue the loads of contraction step kt into the stage tile at LDS address `tile`
    __device__ inline void issue(int kt, uint32_t tile) const {
        const char* b = base + (int64_t)kt * kstep;
        const int wave = threadIdx.x >> 6;
#pragma unroll
        for (int i = 0; i < 2; ++i)
            dma16(b, voff[i], __builtin_amdgcn_readfirstlane(tile + (uint32_t)(2 * wave + i) * 1024u));
    }
    // fragment of 32-row block `blk` (0, 1) for the 16 contraction indices ks (0, 1) of the stage
    __device__ inline uint4 frag(const unsigned char* tile, int blk, int ks) const {
        if (KIND == SRC_KCONTIG) {
            // chunk 2 ks + lg: the swizzle only touches the low two bits, so ks selects the upper half
            return *reinterpret_cast<const uint4*>(tile + ((roff + blk * 2048) ^ (uint32_t)(ks * 32)));
        } else {
            typedef __attribute__((address_space(3))) short4_t lds_s4;
            const uint32_t o = (roff ^ (uint32_t)(blk * 64)) + ks * 4096;
            const short4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4*)(tile + o));
            const short4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4*)(tile + o + 1024));
            uint2 a = __builtin_bit_cast(uint2, lo), b2 = __builtin_bit_cast(uint2, hi);
            return make_uint4(a.x, a.y, b2.x, b2.y);
        }
    }
};

template <int KA, int KB, class Epi>
__global__ __launch_bounds__(256) void k_gemm_dma(GemmArgs<bf16_t, KA, KB, Epi, true, GEMM_NCH> g) {
    extern __shared__ __align__(16) unsigned char dlds[];
    const int id = xcd_remap(blockIdx.x, gridDim.x);
    const int per_p = g.tiles_m * g.tiles_n;
    const int p = id / per_p, tm = (id % per_p) / g.tiles_n, tn = id % g.tiles_n;
    Epi epi = g.epi;
    shift_epi(epi, p, g.e0_pstride, g.e1_pstride, g.e2_pstride);
    const int r0 = tm * BM, c0 = tn * BN;
    const int wave = threadIdx.x >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
    DmaOperand<KA> A;
    DmaOperand<KB> B;
    A.init(reinterpret_cast<const bf16_t*>(g.a.base) + (int64_t)p * g.a_pstride, (int)g.a.ld, g.a.rows, r0, wm, false);
    B.init(reinterpret_cast<const bf16_t*>(g.b.base) + (int64_t)p * g.b_pstride, (int)g.b.ld, g.b.rows, c0, wn, true);

    float16_t acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const int nk = g.a.kdim / 32;
    const uint32_t lbase = (uint32_t)(size_t)dlds;
#pragma unroll
    for (int st = 0; st < DMA_NST - 1; ++st)
        if (st < nk) {
            A.issue(st, lbase + st * DMA_STAGE_BYTES);
            B.issue(st, lbase + st * DMA_STAGE_BYTES + 8192);
        }
    for (int kt = 0; kt < nk; ++kt) {
        // each wave has 4 loads per stage in flight; the oldest stage is the one multiplied next
        const int ahead = nk - 1 - kt;
        if (ahead >= 2) wait_vm<8>();
        else if (ahead == 1) wait_vm<4>();
        else wait_vm<0>();
        __syncthreads();  // stage kt has landed for every wave, and everyone is done with stage kt - 1
        if (kt + DMA_NST - 1 < nk) {
            const uint32_t tile = lbase + (uint32_t)((kt + DMA_NST - 1) % DMA_NST) * DMA_STAGE_BYTES;
            A.issue(kt + DMA_NST - 1, tile);
            B.issue(kt + DMA_NST - 1, tile + 8192);
        }
        const unsigned char* ta = dlds + (kt % DMA_NST) * DMA_STAGE_BYTES;
        const unsigned char* tb = ta + 8192;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            uint4 fa[2], fb[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) fa[i] = A.frag(ta, i, ks);
#pragma unroll
            for (int j = 0; j < 2; ++j) fb[j] = B.frag(tb, j, ks);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) Mma32<bf16_t>::run(fb[j], fa[i], acc[i][j]);  // transposed tile
        }
    }
    __syncthreads();
    gemm_epilogue(epi, acc, dlds, p, tm, g.tiles_m, r0, c0, g.a.rows, g.b.rows);
}

// ---- persistent bf16 grouped GEMM, 256 x TN tiles -----------------------------------------------
// Resident workgroups walk over the tiles; a wave owns 128 x 64 outputs (4 x 2 blocks of 32 x 32, 128
// accumulator registers), which reads three quarters of the LDS bytes per product that the 64 x 64 wave
// tiles above read.  Operand stages (A 16 KB, B TN * 64 bytes) are filled by direct-to-LDS loads two
// contraction steps ahead, and the first two stages of a workgroup's next tile are requested before the
// epilogue of the current one, so that their latency is covered by the epilogue's arithmetic.  The
// layouts inside a stage follow DmaOperand; a row of a K-strided tile has ROWS / 8 chunks.
#define PG_NST 3
#define PG_A_BYTES 16384
#define PG_TM 256
// TN = 128: four waves (2 x 2), two workgroups per CU.  TN = 256: eight waves (2 x 4), one workgroup per CU;
// a third fewer operand bytes per product travel from the L2 into LDS.
template <int TN> struct PgShape {
    static constexpr int kWaves = TN / 32;                 // 128 x 64 outputs per wave
    static constexpr int kBBytes = TN * 64;
    static constexpr int kStage = PG_A_BYTES + kBBytes;
    static constexpr int kLds = PG_NST * kStage;
    static constexpr int kLoads = (PG_A_BYTES + kBBytes) / 1024 / kWaves;  // DMA instructions per wave and stage
};

template <int KIND, int ROWS, int MBLK, int NW>
struct DmaTile {
    static constexpr int NI = ROWS / 16 / NW;  // DMA instructions per wave and stage
    static constexpr int CPR = ROWS / 8;   // chunks per contraction index (K-strided layout)
    const char* base;
    uint32_t voff[NI];
    int64_t kstep;
    uint32_t roff[MBLK];  // LDS byte offset of the lane's fragment of block b, ks 0

    __device__ inline void set_tile(const bf16_t* b, int ld, int rows, int t0) {
        base = reinterpret_cast<const char*>(b);
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int j = NI * wave + i;
            if (KIND == SRC_KCONTIG) {
                const int row = 16 * j + lane / 4, c = (lane % 4) ^ swz_rk(row);
                int gr = t0 + row;
                gr = gr < rows ? gr : rows - 1;
                voff[i] = (uint32_t)((gr * ld + 8 * c) * 2);
            } else {
                const int pos = 64 * j + lane, k = pos / CPR, ic = (pos % CPR) ^ (4 * (k & 3));
                int gr = t0 + 8 * ic;
                gr = gr < rows - 8 ? gr : rows - 8;
                voff[i] = (uint32_t)((k * ld + gr) * 2);
            }
        }
        kstep = (KIND == SRC_KCONTIG) ? 64 : (int64_t)64 * ld;
    }
    __device__ inline void set_lane(int wbase, bool brole) {
        const int lane = threadIdx.x & 63, lr = lane & 31, lg = lane >> 5;
#pragma unroll
        for (int b = 0; b < MBLK; ++b) {
            if (KIND == SRC_KCONTIG) {
                const int rr = brole ? ((lr & 0x13) | ((lr & 4) << 1) | ((lr & 8) >> 1)) : lr;
                const int row = wbase + 32 * b + rr;
                roff[b] = (uint32_t)(row * 64 + ((lg ^ swz_rk(row)) * 16));
            } else {
                const int a = lane & 15, q0 = (lane >> 4) & 1, e = a >> 2, c = a & 3;
                const int cs = brole ? (((c & 1) << 1) | (c >> 1)) : c;
                const int col = wbase + 32 * b + 16 * q0 + 4 * cs, k = 8 * lg + e;
                roff[b] = (uint32_t)((k * CPR + ((col >> 3) ^ (4 * (k & 3)))) * 16 + ((col >> 2) & 1) * 8);
            }
        }
    }
    __device__ inline void issue(int kt, uint32_t tile) const {
        const char* b = base + (int64_t)kt * kstep;
        const int wave = threadIdx.x >> 6;
#pragma unroll
        for (int i = 0; i < NI; ++i)
            dma16(b, voff[i], __builtin_amdgcn_readfirstlane(tile + (uint32_t)(NI * wave + i) * 1024u));
    }
    __device__ inline uint4 frag(const unsigned char* tile, int blk, int ks) const {
        if (KIND == SRC_KCONTIG) {
            return *reinterpret_cast<const uint4*>(tile + (roff[blk] ^ (uint32_t)(ks * 32)));
        } else {
            typedef __attribute__((address_space(3))) short4_t lds_s4;
            const uint32_t o = roff[blk] + ks * (16 * CPR * 16);
            const short4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4*)(tile + o));
            const short4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4*)(tile + o + 4 * CPR * 16));
            uint2 a = __builtin_bit_cast(uint2, lo), b2 = __builtin_bit_cast(uint2, hi);
            return make_uint4(a.x, a.y, b2.x, b2.y);
        }
    }
};

// Epilogue of a 128 x 64 wave tile.  `lds_free` is LDS no load is in flight to (4 KB per wave) for the
// staged stores; `red` (64 floats per wave) takes the column sums and is the space of the bias slices, which
// an epilogue with column sums does not use.
template <class Epi, int MB, int TN>
__device__ inline void tile_epilogue(const Epi& epi, float16_t (&acc)[MB][2], unsigned char* lds_free,
                                     const float* lds_bias, float* red, const uint4 (&first)[4], int p, int tm,
                                     int tiles_m, int r0, int c0, int rows, int cols, int wm, int wn) {
    static_assert(!(Epi::kBias && Epi::kColSum), "the bias slice and the column sums share LDS");
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lr = lane & 31, lg = lane >> 5;
    float cs[Epi::kColSum ? 32 : 1];
    // staged stores: a per-wave patch of 32 rows x 128 bytes whose 16-byte chunks are XOR-swizzled by the
    // row, written by the lanes that own the values and read back as whole 128-byte row segments
    unsigned char* patch = lds_free + wave * 4096;
    uint4 cur[4];
#pragma unroll
    for (int o = 0; o < 4; ++o) cur[o] = first[o];
#pragma unroll
    for (int i = 0; i < MB; ++i) {
        const int r = r0 + wm + 32 * i + lr;
        const int rc = r < rows ? r : rows - 1;
        if (Epi::kStagePers) {
            static_assert(!Epi::kStagePers || Epi::kES == 2, "staged stores are for 2-byte outputs");
            uint4 second[4];
            uint4 nxt[4];
            if constexpr (Epi::kPrefetch) {  // operands of block i + 1 are requested before block i is worked on
                if (i + 1 < MB) {
                    const int rn = r0 + wm + 32 * (i + 1) + lr, rnc = rn < rows ? rn : rows - 1;
#pragma unroll
                    for (int o = 0; o < 4; ++o) {
                        const int c = c0 + wn + 16 * o + 8 * lg;
                        nxt[o] = epi.fetch(rnc, c < cols ? c : 0);
                    }
                }
            }
#pragma unroll
            for (int o = 0; o < 4; ++o) {
                const int j = o >> 1, h = o & 1;
                const int c = c0 + wn + 32 * j + 16 * h + 8 * lg;
                float v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) v[u] = acc[i][j][8 * h + u];
                typename Epi::Out out;
                if constexpr (Epi::kBias) {
                    // lds_bias holds the bias of the tile's columns (clamped at the matrix edge)
                    const float4 b0 = *reinterpret_cast<const float4*>(lds_bias + wn + 32 * j + 16 * h + 8 * lg);
                    const float4 b1 = *reinterpret_cast<const float4*>(lds_bias + wn + 32 * j + 16 * h + 8 * lg + 4);
                    v[0] += b0.x; v[1] += b0.y; v[2] += b0.z; v[3] += b0.w;
                    v[4] += b1.x; v[5] += b1.y; v[6] += b1.z; v[7] += b1.w;
                    epi.compute_biased(v, out);
                } else if constexpr (Epi::kPrefetch) {
                    epi.compute_fetched(cur[o], v, out);
                } else {
                    epi.compute(rc, c < cols ? c : 0, 8, v, out);
                }
                if (Epi::kColSum) {
                    const bool ok = (r < rows) && (c < cols);
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const int t = Epi::kColSum ? (8 * o + u) : 0;
                        cs[t] = (i == 0 ? 0.f : cs[t]) + (ok ? v[u] : 0.f);
                    }
                }
                const int cch = 4 * j + 2 * h + lg;
                *reinterpret_cast<uint4*>(patch + lr * 128 + ((cch ^ (lr & 7)) * 16)) = Epi::pk(out, 0).lo;
                if (Epi::kArrays == 2) second[o] = Epi::pk(out, 1).lo;
            }
#pragma unroll
            for (int a = 0; a < Epi::kArrays; ++a) {
                if (a == 1) {
                    __builtin_amdgcn_wave_barrier();
#pragma unroll
                    for (int o = 0; o < 4; ++o) {
                        const int cch = 4 * (o >> 1) + 2 * (o & 1) + lg;
                        *reinterpret_cast<uint4*>(patch + lr * 128 + ((cch ^ (lr & 7)) * 16)) = second[o];
                    }
                }
                __builtin_amdgcn_wave_barrier();
                char* base = epi.arr(a);
#pragma unroll
                for (int it = 0; it < 4; ++it) {
                    const int q = it * 64 + lane, prow = q >> 3, pc = q & 7;
                    const uint4 u = *reinterpret_cast<const uint4*>(patch + prow * 128 + ((pc ^ (prow & 7)) * 16));
                    const int gr = r0 + wm + 32 * i + prow, gc = c0 + wn + pc * 8;
                    if (gr < rows && gc < cols) *reinterpret_cast<uint4*>(base + ((int64_t)gr * epi.ld + gc) * 2) = u;
                }
            }
            __builtin_amdgcn_wave_barrier();
            if constexpr (Epi::kPrefetch) {
#pragma unroll
                for (int o = 0; o < 4; ++o) cur[o] = nxt[o];
            }
        } else {
            // `first` holds the prefetched operands of block 0 (four octets per lane); those of block
            // i + 1 are requested before block i is worked on
            uint4 nxt[4];
            if constexpr (Epi::kPrefetch) {
                if (i + 1 < MB) {
                    const int rn = r0 + wm + 32 * (i + 1) + lr, rnc = rn < rows ? rn : rows - 1;
#pragma unroll
                    for (int o = 0; o < 4; ++o) {
                        const int c = c0 + wn + 16 * o + 8 * lg;
                        nxt[o] = epi.fetch(rnc, c < cols ? c : 0);
                    }
                }
            }
#pragma unroll
            for (int jb = 0; jb < 2; ++jb) {
                typename Epi::Out outs[2];
#pragma unroll
                for (int o = 0; o < 2; ++o) {
                    const int c = c0 + wn + 32 * jb + 16 * o + 8 * lg;
                    float v[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) v[u] = acc[i][jb][8 * o + u];
                    const bool ok = (r < rows) && (c < cols);
                    if constexpr (Epi::kPrefetch) epi.compute_fetched(cur[2 * jb + o], v, outs[o]);
                    else epi.compute(rc, c < cols ? c : 0, 8, v, outs[o]);
                    if (Epi::kColSum) {
#pragma unroll
                        for (int u = 0; u < 8; ++u) {
                            const int t = Epi::kColSum ? (16 * jb + 8 * o + u) : 0;
                            cs[t] = (i == 0 ? 0.f : cs[t]) + (ok ? v[u] : 0.f);
                        }
                    }
                }
#pragma unroll
                for (int o = 0; o < 2; ++o) {
                    const int c = c0 + wn + 32 * jb + 16 * o + 8 * lg;
                    if (r < rows && c < cols) epi.flush(r, c, (cols - c < 8) ? (cols - c) : 8, outs[o]);
                }
            }
            if constexpr (Epi::kPrefetch) {
#pragma unroll
                for (int o = 0; o < 4; ++o) cur[o] = nxt[o];
            }
        }
    }
    if (Epi::kColSum) {
        // as in gemm_epilogue, over the 128 rows of the wave tile and then over the two waves of a column half
        fold_slots<16>(cs, lr);
        fold_slots<8>(cs, lr);
        fold_slots<4>(cs, lr);
        fold_slots<2>(cs, lr);
        fold_slots<1>(cs, lr);
        {
            const int j = lr >> 4, h = (lr >> 3) & 1, u = lr & 7;
            red[wave * 64 + 32 * j + 16 * h + 8 * lg + u] = cs[0];
        }
        __syncthreads();
        if (threadIdx.x < TN) {  // the two waves of a 64-column strip: wave ids s and s + TN / 64
            const int strip = threadIdx.x >> 6, col = threadIdx.x & 63;
            const float v = red[strip * 64 + col] + red[(TN / 64 + strip) * 64 + col];
            if (c0 + threadIdx.x < cols) epi.part[((int64_t)p * tiles_m + tm) * epi.ld + c0 + threadIdx.x] = v;
        }
    }
}

template <int KA, int KB, class Epi, int TN>
__global__ __launch_bounds__(2 * TN, 2) void k_gemm_pers(GemmArgs<bf16_t, KA, KB, Epi, true, GEMM_NCH> g, int n_tiles) {
    typedef PgShape<TN> S;
    extern __shared__ __align__(16) unsigned char dlds[];
    const int wave = threadIdx.x >> 6;
    const int wm = (wave / (TN / 64)) * 128, wn = (wave % (TN / 64)) * 64;
    const int per_p = g.tiles_m * g.tiles_n;
    const int nk = g.a.kdim / 32;
    const uint32_t lbase = (uint32_t)(size_t)dlds;
    DmaTile<KA, PG_TM, 4, S::kWaves> A;
    DmaTile<KB, TN, 2, S::kWaves> B;
    A.set_lane(wm, false);
    B.set_lane(wn, true);

    // tile ids of this workgroup: blockIdx.x, + gridDim.x, ...; the XCD remap keeps the tiles that the
    // workgroups of one XCD work on at the same time next to each other (same preference, same W(p))
    auto locate = [&](int vid, int& p, int& tm, int& tn) {
        const int id = xcd_remap(vid, n_tiles);
        p = id / per_p;
        tm = (id % per_p) / g.tiles_n;
        tn = id % g.tiles_n;
    };
    int bslot = 0;
    auto request = [&](int p, int tm, int tn) {  // first stages of a tile (and its bias slice)
        if constexpr (Epi::kBias) {
            bslot ^= 1;
            if (wave < TN / 64) {
                int c = tn * TN + 64 * wave + (threadIdx.x & 63);
                c = c < g.b.rows ? c : g.b.rows - 1;
                dma4(g.epi.bias + (int64_t)p * g.e0_pstride, (uint32_t)c * 4u,
                     __builtin_amdgcn_readfirstlane(lbase + S::kLds + (uint32_t)(bslot * (4 * TN) + wave * 256)));
            }
        }
        A.set_tile(reinterpret_cast<const bf16_t*>(g.a.base) + (int64_t)p * g.a_pstride, (int)g.a.ld, g.a.rows, tm * PG_TM);
        B.set_tile(reinterpret_cast<const bf16_t*>(g.b.base) + (int64_t)p * g.b_pstride, (int)g.b.ld, g.b.rows, tn * TN);
#pragma unroll
        for (int st = 0; st < PG_NST - 1; ++st)
            if (st < nk) {
                A.issue(st, lbase + st * S::kStage);
                B.issue(st, lbase + st * S::kStage + PG_A_BYTES);
            }
    };

    int vid = blockIdx.x;
    if (vid >= n_tiles) return;
    int p, tm, tn;
    locate(vid, p, tm, tn);
    request(p, tm, tn);
    for (;;) {
        float16_t acc[4][2];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
        uint4 first[4] = {};
        for (int kt = 0; kt < nk; ++kt) {
            // a wave has kLoads loads per stage in flight.  At the first step of a tile the stores of the
            // previous epilogue may still be counted as well, so everything is waited for.
            if (kt == 0 || kt == nk - 1) wait_vm<0>();
            else wait_vm<S::kLoads>();
            __syncthreads();  // stage kt is complete, and stage kt - 1 (or the last epilogue's patch) is free
            if constexpr (Epi::kPrefetch) {
                // the epilogue's first block of act'(z): requested behind the tile's last operand stage, during the
                // last contraction step (after the products it cost 0.2 ms more per step of workload 5; two or four
                // steps earlier measured no better)
                if (kt == nk - 1) {
                    Epi epi0 = g.epi;
                    shift_epi(epi0, p, g.e0_pstride, g.e1_pstride, g.e2_pstride);
                    const int r = tm * PG_TM + wm + (threadIdx.x & 31), rc = r < g.a.rows ? r : g.a.rows - 1;
#pragma unroll
                    for (int o = 0; o < 4; ++o) {
                        const int c = tn * TN + wn + 16 * o + 8 * ((threadIdx.x & 63) >> 5);
                        first[o] = epi0.fetch(rc, c < g.b.rows ? c : 0);
                    }
                }
            }
            if (kt + PG_NST - 1 < nk) {
                const uint32_t tile = lbase + (uint32_t)((kt + PG_NST - 1) % PG_NST) * S::kStage;
                A.issue(kt + PG_NST - 1, tile);
                B.issue(kt + PG_NST - 1, tile + PG_A_BYTES);
            }
            const unsigned char* ta = dlds + (kt % PG_NST) * S::kStage;
            const unsigned char* tb = ta + PG_A_BYTES;
            // all fragments of the stage are requested before the first product, so that one LDS latency is
            // exposed per step instead of one per pair of products
            uint4 fa[2][4], fb[2][2];
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
                for (int j = 0; j < 2; ++j) fb[ks][j] = B.frag(tb, j, ks);
#pragma unroll
                for (int i = 0; i < 4; ++i) fa[ks][i] = A.frag(ta, i, ks);
            }
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j) Mma32<bf16_t>::run(fb[ks][j], fa[ks][i], acc[i][j]);  // transposed tile
            constexpr int kReads = ((KA == SRC_KCONTIG) ? 8 : 16) + ((KB == SRC_KCONTIG) ? 4 : 8);
            __builtin_amdgcn_sched_group_barrier(0x100, kReads, 0);  // LDS reads
            __builtin_amdgcn_sched_group_barrier(0x008, 16, 0);      // MFMAs
        }
        __syncthreads();  // every wave is done with the stages
        const int pc = p, tmc = tm, tnc = tn;
        const float* lds_bias = reinterpret_cast<const float*>(dlds + S::kLds + bslot * (4 * TN));
        Epi epi = g.epi;
        shift_epi(epi, pc, g.e0_pstride, g.e1_pstride, g.e2_pstride);
        vid += gridDim.x;
        const bool more = vid < n_tiles;
        if (more) {
            locate(vid, p, tm, tn);
            request(p, tm, tn);  // stages 0 and 1; the epilogue below stages its stores in the third
        }
        tile_epilogue<Epi, 4, TN>(epi, acc, dlds + (PG_NST - 1) * S::kStage, lds_bias,
                                  reinterpret_cast<float*>(dlds + S::kLds), first, pc, tmc, g.tiles_m, tmc * PG_TM, tnc * TN,
                              g.a.rows, g.b.rows, wm, wn);
        if (!more) break;
    }
}

// ---- fused forward: observations -> every hidden layer -> output layer (bf16, width 512 or 256) -------
// (paper Sec. III-C: the target network of a preference applied to that preference's environments, in the
// rollout and in the update.)  One workgroup of W / 64 waves carries 128 rows of one preference through the
// whole network, tile after tile (width 512: eight waves, one workgroup per CU; width 256: four waves and half the
// tile, two per CU).  The activations of the tile live in LDS (128 rows x 2 W bytes, 16-byte chunks XOR-swizzled by
// the row) and are rewritten in place layer after layer; HBM sees the observations once, the outputs once
// and, in the saving variant, the stores of h and act'(z) that the backward pass reads -- never a load of
// an activation.
// Wave w owns output features [64 w, 64 w + 64) of every layer for all 128 rows: its slice of W_l(p) is
// used by no other wave, so the W fragments go from global memory (they sit in L2: 64 tiles share one
// W(p)) straight into registers, requested half a super-step ("unit": 16 products, 32 contraction indices
// per lane group) ahead of their use.  The kernel reads them from a copy of the matrices in fragment order
// (k_theta_fragment_order, made by the same call): every load instruction then covers 1 KB of consecutive
// addresses.  Read from the row-major matrices the same stream takes 32 bytes from each of 32 rows per
// instruction, and the workgroups of a CU, 64 KB of such lines in flight against its vector cache, fetch
// lines from L2 more than once: streamed alone, without the products, W moved at 9.7 TB/s row-major and
// 15.3 TB/s in fragment order, and a launch of workload 5 spends most of its time on exactly this stream.
// Inside a super-step lane group g
// of product jj covers contraction indices 64 s + 32 g + 8 jj .. + 8 for both operands.  The bias enters
// as the initial value of the accumulators.  A layer ends with a barrier, the epilogue (activation, its
// derivative, the in-place rewrite of the tile, the stores of the saving variant) and a second barrier;
// the products and the epilogue of a workgroup do not overlap, and with 128 KB of LDS for the tile there is
// one workgroup per CU.  Measured on workload 5 the time of a launch splits, additively, into the W
// requests, the products, the epilogue arithmetic and a fixed part per tile (observation gather, first
// requests, barriers).
#define FF_ROWS 128

struct FusedFwdArgs {
    const float* x;           // observations, time-major rows of O values
    bf16_t* x0;               // saving: receives the gathered observations, compact [P][M][O] bf16
    const bf16_t* theta_mat;  // [P][mat_len]: the output layer's matrix is read from here
    const bf16_t* theta_frag; // [P][mat_len]: the first and the hidden layers' matrices in fragment order
    const float* theta_vec;   // [P][vec_len]
    int64_t mat_len, vec_len;
    int64_t mat_off[MORLAX_MAX_LAYERS], vec_off[MORLAX_MAX_LAYERS];
    int64_t frag_len, frag_off[MORLAX_MAX_LAYERS];  // the fragment-order copy: elements per preference, layer starts
    int32_t Opad;  // O rounded up to a multiple of 64: the first layer's contraction, zero-filled beyond O
    bf16_t* H;    // saving: h of layer l at H + l * lstride; else the last layer's h only
    gfix16_t* G;  // saving: act'(z) of layer l at G + l * lstride
    int64_t lstride;
    int32_t L, O, M, tiles_m, n_tiles;
    // output layer (applied to the tile's last hidden activations while they are still in LDS)
    int64_t head_mat_off, head_vec_off, logsig_off;
    int32_t out_dim, tanh_cols;  // leading output columns that are squashed by tanh (the actor's means)
    int32_t adim, sig_state;     // action width; 1: log sigma = output columns [adim, 2 adim) of the same row
    RowMap rm;
    float* out;        // time-major [.., N, out_dim]
    float* saved_out;  // saving: compact [P][M][OUT_PITCH]
    const float* eps;  // actor with sampling: noise, and the two outputs below
    float* act;
    float* logp;
};

__device__ inline int swap_bits23(int i) { return (i & 0x13) | ((i & 4) << 1) | ((i & 8) >> 1); }

// Fragment order of a [W][K] bf16 matrix (K a multiple of 64): the 16-byte pieces of W in the order in
// which the fused forward requests them, so that each of its load instructions reads 1 KB of consecutive
// addresses (eight whole cache lines) instead of 32 bytes from each of 32 rows.  Wave v of the forward owns
// output features [64 v, 64 v + 64); its stream is K / 32 units of 4 KB; unit u holds four 1 KB blocks
// (j, e), j = feature half, e = which 16 bytes; lane (lg, lr) of a block holds, for feature
// 64 v + 32 j + swap_bits23(lr), the contraction indices 64 (u / 2) + 32 lg + 16 (u % 2) + 8 e + [0, 8).
// One workgroup moves a super-step pair of units of one j: 32 rows x 128 bytes, whole lines in and out.
struct FragOrderArgs {
    const bf16_t* src;  // [P][mat_len] row-major matrices
    bf16_t* dst;        // [P][frag_len]
    int64_t mat_len, frag_len;
    int64_t mat_off[MORLAX_MAX_LAYERS], frag_off[MORLAX_MAX_LAYERS];
    int32_t K[MORLAX_MAX_LAYERS];     // contraction length in the copy (a multiple of 64)
    int32_t Ksrc[MORLAX_MAX_LAYERS];  // columns of the row-major matrix; the copy is zero beyond them
    int32_t g0[MORLAX_MAX_LAYERS + 1];  // first workgroup of layer l; g0[L] = workgroups per preference
    int32_t L;
};

__global__ __launch_bounds__(256) void k_theta_fragment_order(FragOrderArgs a) {
    const int p = blockIdx.y;
    int l = 0;
    while (l + 1 < a.L && (int)blockIdx.x >= a.g0[l + 1]) ++l;
    const int K = a.K[l], g = blockIdx.x - a.g0[l];
    const int per_wave = 2 * (K >> 6);
    const int v = g / per_wave, r = g % per_wave, sstep = r >> 1, j = r & 1;
    const int wq = threadIdx.x >> 6, ln = threadIdx.x & 63, ub = wq >> 1, e = wq & 1, lg = ln >> 5, lr = ln & 31;
    const int u = 2 * sstep + ub;
    const bf16_t* Wsrc = a.src + (int64_t)p * a.mat_len + a.mat_off[l];
    char* D = reinterpret_cast<char*>(a.dst + (int64_t)p * a.frag_len + a.frag_off[l]);
    const int f = 64 * v + 32 * j + swap_bits23(lr);
    const int k0 = (sstep * 128 + ub * 32 + lg * 64 + e * 16) >> 1, Ks = a.Ksrc[l];
    uint4 q;
    if (Ks == K) {
        q = *reinterpret_cast<const uint4*>(Wsrc + (int64_t)f * K + k0);
    } else {  // an observation width that is no multiple of 64: element by element, zeros beyond it
        const unsigned short* row = reinterpret_cast<const unsigned short*>(Wsrc) + (int64_t)f * Ks;
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t lo = (k0 + 2 * i < Ks) ? row[k0 + 2 * i] : 0u, hi = (k0 + 2 * i + 1 < Ks) ? row[k0 + 2 * i + 1] : 0u;
            w[i] = lo | (hi << 16);
        }
        q = make_uint4(w[0], w[1], w[2], w[3]);
    }
    *reinterpret_cast<uint4*>(D + (int64_t)v * (K >> 5) * 4096 + u * 4096 + j * 2048 + e * 1024 + ln * 16) = q;
}

// a value the compiler can no longer trace back to its source: address arithmetic derived from it stays
// where it is written instead of being hoisted out of the layer loop into registers held across the products
__device__ inline int opaque(int v) {
    asm volatile("" : "+v"(v));
    return v;
}

template <int ACT, bool SAVE, int WD>
__global__ __launch_bounds__(WD, 2) void k_mlp_fused_fwd(FusedFwdArgs a) {
    constexpr int RB = 2 * WD;           // bytes of a tile row
    constexpr int NW = WD / 64;          // waves: 64 output features each
    constexpr int TILE_BYTES = FF_ROWS * RB;
    extern __shared__ __align__(16) unsigned char dlds[];
    // One workgroup per CU walks the tiles (no launch gap, no register spill in the saving variant).  Everything
    // derived from the lane is formed again for every tile behind opaque(): kept across tiles it would occupy
    // registers that the products and the epilogue need.
    for (int vt = blockIdx.x; vt < a.n_tiles; vt += gridDim.x) {
        const int lane = opaque((int)(threadIdx.x & 63)), lr = lane & 31, lg = lane >> 5;
        const int wave = __builtin_amdgcn_readfirstlane(opaque((int)(threadIdx.x >> 6)));
        const int tile = xcd_remap(vt, a.n_tiles);
        const int p = tile / a.tiles_m, m0 = (tile % a.tiles_m) * FF_ROWS;
        const int rows = a.M - m0 < FF_ROWS ? a.M - m0 : FF_ROWS;
        const int wn = wave * 64;

        const bf16_t* Wp = a.theta_frag + (int64_t)p * a.frag_len;
        const float* bp = a.theta_vec + (int64_t)p * a.vec_len;
        auto w_rows = [&](int l, const char* (&w)[2]) {  // the lane's place in the wave's stream of W_l(p), per feature half
            const int K = l == 0 ? a.Opad : WD;
#pragma unroll
            for (int j = 0; j < 2; ++j)
                w[j] = reinterpret_cast<const char*>(Wp + a.frag_off[l]) + (int64_t)wave * (K >> 5) * 4096 + j * 2048 +
                       lane * 16;
        };
        // unit u of a layer = 32 contraction indices per lane group, 4 KB of the wave's stream (fragment order)
        auto load_w = [&](uint4 (&wf)[2][2], const char* w0, const char* w1, int u) {
            const int off = u * 4096;
            wf[0][0] = *reinterpret_cast<const uint4*>(w0 + off);
            wf[0][1] = *reinterpret_cast<const uint4*>(w0 + off + 1024);
            wf[1][0] = *reinterpret_cast<const uint4*>(w1 + off);
            wf[1][1] = *reinterpret_cast<const uint4*>(w1 + off + 1024);
        };
        // W fragments: two buffers, a unit's request one unit ahead of its use (a longer distance with four
        // buffers measured slower: the registers it takes spill in the epilogue)
        const char* wp[2];
        uint4 wfa[2][2], wfb[2][2];
        float16_t acc[4][2];
        w_rows(0, wp);
        load_w(wfa, wp[0], wp[1], 0);

        {  // the tile's observations, gathered from the time-major tensor and rounded to bf16; rows past the end
           // repeat the last row (their results are never stored).  The saving variant keeps the compact copy
           // that the first layer's dW product reads.
            const int cpr = a.Opad >> 3;
            const bool whole = (a.O & 7) == 0;  // rows of whole 8-value pieces (16-byte aligned: the launcher checks x)
            for (int id = threadIdx.x; id < FF_ROWS * cpr; id += WD) {
                const int r = id / cpr, c = id % cpr, rc = r < rows ? r : rows - 1;
                const float* xr = a.x + a.rm.row(p, m0 + rc) * a.O;
                float v[8];
                if (whole && 8 * c < a.O) {
                    get8(xr + 8 * c, v);
                } else {  // a width that is no multiple of 8, or the zero fill up to Opad
#pragma unroll
                    for (int e = 0; e < 8; ++e) v[e] = (8 * c + e < a.O) ? xr[8 * c + e] : 0.f;
                }
                const uint4 q = pack_chunk<bf16_t>(v);
                *reinterpret_cast<uint4*>(dlds + r * RB + ((c ^ (r & 15)) * 16)) = q;
                if (SAVE && a.x0 && r < rows && 8 * c < a.O)
                    *reinterpret_cast<uint4*>(a.x0 + ((int64_t)p * a.M + m0 + r) * a.O + 8 * c) = q;
            }
        }
        // fragment addresses: row 32 i + lr, chunk (8 s + 4 lg + jj) ^ (lr & 15)
        const int x = lr & 15;
        const unsigned char* arow = dlds + lr * RB;
        uint32_t aoff[4];
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) aoff[jj] = (uint32_t)(((4 * lg + jj) ^ (x & 7)) * 16);
        const int sflip = x >> 3;

        // one unit: 16 products; HALF = u & 1 picks the chunks 2 HALF, 2 HALF + 1 of the super-step
        auto unit = [&](const uint4 (&wf)[2][2], int u, auto half_tag) {
            constexpr int HALF = decltype(half_tag)::value;
            const unsigned char* as = arow + ((u >> 1) ^ sflip) * 128;
            uint4 fa[2][4];
#pragma unroll
            for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                for (int i = 0; i < 4; ++i) fa[jj][i] = *reinterpret_cast<const uint4*>(as + i * (32 * RB) + aoff[2 * HALF + jj]);
#pragma unroll
            for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j) Mma32<bf16_t>::run(wf[j][jj], fa[jj][i], acc[i][j]);
        };
        // lane n of `bias` holds b_l[wn + n]; every accumulator of a lane's octet o starts from its feature's bias
        auto init_acc = [&](float bias) {
#pragma unroll
            for (int o = 0; o < 4; ++o)
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const float b = __shfl(bias, 16 * o + 8 * lg + u, 64);
#pragma unroll
                    for (int i = 0; i < 4; ++i) acc[i][o >> 1][8 * (o & 1) + u] = b;
                }
        };
        auto load_bias = [&](int l) { return bp[a.vec_off[l] + wn + lane]; };

        init_acc(load_bias(0));
        __syncthreads();
        for (int l = 0; l < a.L; ++l) {
            const bool more = l + 1 < a.L;
            // the last request of a layer fetches the first unit of the next one (of this one again after the last
            // layer: a harmless, valid load), so that every pass through the loop has the same loads in flight
            const char* wq[2];
            w_rows(more ? l + 1 : l, wq);
            const int nU = l == 0 ? a.Opad >> 5 : WD / 32;
            for (int u = 0; u < nU; u += 2) {
                load_w(wfb, wp[0], wp[1], u + 1);
                __builtin_amdgcn_sched_barrier(0);  // the requests stay ahead of the products they overlap with
                unit(wfa, u, std::integral_constant<int, 0>{});
                const bool last = u + 2 == nU;
                load_w(wfa, last ? wq[0] : wp[0], last ? wq[1] : wp[1], last ? 0 : u + 2);
                __builtin_amdgcn_sched_barrier(0);
                unit(wfb, u + 1, std::integral_constant<int, 1>{});
            }
            wp[0] = wq[0];
            wp[1] = wq[1];
            __syncthreads();  // every wave has read the layer's input for the last time
            const float bnext = load_bias(more ? l + 1 : l);
            {
                const int ol = opaque(lane), olr = ol & 31, olg = ol >> 5, ox = ol & 15;
                unsigned char* hrow = dlds + olr * RB;
                unsigned char* patch = dlds + TILE_BYTES + wave * 4096;
                gfix16_t* Gl = SAVE ? a.G + (int64_t)l * a.lstride + ((int64_t)p * a.M + m0) * WD + wn : nullptr;
                bf16_t* Hl = SAVE ? a.H + (int64_t)l * a.lstride + ((int64_t)p * a.M + m0) * WD + wn : nullptr;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    uint4 gq[4], hq[4];
#pragma unroll
                    for (int o = 0; o < 4; ++o) {
                        const int j = o >> 1, h = o & 1;
                        float v[8], g[8];
#pragma unroll
                        for (int u = 0; u < 8; ++u) act_pair<ACT>(acc[i][j][8 * h + u], v[u], g[u]);
                        const int cc = 8 * wave + 4 * j + 2 * h + olg;
                        hq[o] = pack_chunk<bf16_t>(v);
                        *reinterpret_cast<uint4*>(hrow + i * (32 * RB) + ((cc ^ ox) * 16)) = hq[o];
                        if (SAVE) gq[o] = pack8(g, (const gfix16_t*)nullptr).lo;
                    }
                    // act'(z) and h leave through the wave's patch as whole 128-byte row segments, row block by row
                    // block between the epilogue's arithmetic (h read back from the tile after the closing barrier and
                    // stored as whole rows cost 1 ms more per step of workload 5: those stores sat in front of the
                    // next layer's first requests)
                    if (SAVE) {
#pragma unroll
                        for (int arr = 0; arr < 2; ++arr) {
#pragma unroll
                            for (int o = 0; o < 4; ++o) {
                                const int cch = 4 * (o >> 1) + 2 * (o & 1) + olg;
                                *reinterpret_cast<uint4*>(patch + olr * 128 + ((cch ^ (olr & 7)) * 16)) = arr ? hq[o] : gq[o];
                            }
                            __builtin_amdgcn_wave_barrier();
                            char* dst = arr ? reinterpret_cast<char*>(Hl) : reinterpret_cast<char*>(Gl);
#pragma unroll
                            for (int it = 0; it < 4; ++it) {
                                const int prow = it * 8 + (ol >> 3), pc = ol & 7;
                                const uint4 u = *reinterpret_cast<const uint4*>(patch + prow * 128 + ((pc ^ (prow & 7)) * 16));
                                const int gr = 32 * i + prow;
                                if (gr < rows) *reinterpret_cast<uint4*>(dst + ((int64_t)gr * WD + pc * 8) * 2) = u;
                            }
                            __builtin_amdgcn_wave_barrier();
                        }
                    }
                }
            }
            __syncthreads();  // the layer's output is complete in LDS
            if (more) init_acc(bnext);
        }

        // output layer: wave w takes rows 16 w .. 16 w + 15 of the tile with 16x16x32 products; lane (hl, hg)
        // supplies row hl / output hl at contraction chunk 4 u + hg and receives output hl of rows 4 hg + e
        // (width 256: four waves, two passes of 64 rows)
#pragma unroll
        for (int pass = 0; pass < 8 / NW; ++pass) {
            const int hl = lane & 15, hg = lane >> 4;
            const int wv = wave + NW * pass;
            const int r = 16 * wv + hl;
            const unsigned char* hrow = dlds + r * RB;
            const bf16_t* wrow = a.theta_mat + (int64_t)p * a.mat_len + a.head_mat_off + (int64_t)hl * WD;
            const bool b_ok = hl < a.out_dim;
            float4_t c = {0.f, 0.f, 0.f, 0.f}, c2 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int half = 0; half < WD / 256; ++half) {
                uint4 fa[8], fb[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int ch = 32 * half + 4 * u + hg;
                    fa[u] = *reinterpret_cast<const uint4*>(hrow + ((ch ^ (r & 15)) * 16));
                    fb[u] = make_uint4(0, 0, 0, 0);
                    if (b_ok) fb[u] = *reinterpret_cast<const uint4*>(wrow + 8 * ch);
                }
#pragma unroll
                for (int u = 0; u < 8; u += 2) {
                    Mma16<bf16_t>::run(fa[u], fb[u], c);
                    Mma16<bf16_t>::run(fa[u + 1], fb[u + 1], c2);
                }
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) c[e] += c2[e];
            const float bias = b_ok ? bp[a.head_vec_off + hl] : 0.f;
            const bool a_ok = hl < a.adim;  // lanes that hold an action mean
            float ls_p = 0.f;
            if (a.eps && a_ok && !a.sig_state) ls_p = bp[a.logsig_off + hl];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int tr = 16 * wv + 4 * hg + e, m = m0 + tr;
                const bool ok = (tr < rows) && b_ok;
                const float z = c[e] + bias;
                const float o = (hl < a.tanh_cols) ? tanhf(z) : z;
                int64_t row = 0;
                if (tr < rows) row = a.rm.row(p, m);
                float term = 0.f;
                // a state-dependent log sigma sits adim columns to the right, in the same group of 16 lanes
                const float ls_s = __shfl(o, (lane & 48) | ((hl + a.adim) & 15), 64);
                if (ok) {
                    a.out[row * a.out_dim + hl] = o;
                    if (SAVE) a.saved_out[((int64_t)p * a.M + m) * OUT_PITCH + hl] = o;
                    if (a.eps && a_ok) {
                        const float ls = a.sig_state ? ls_s : ls_p;
                        const float ep = a.eps[row * a.adim + hl];
                        a.act[row * a.adim + hl] = o + expf(ls) * ep;
                        term = -0.5f * ep * ep - ls;
                    }
                }
                if (a.eps) {
                    term += __shfl_xor(term, 8, 64);
                    term += __shfl_xor(term, 4, 64);
                    term += __shfl_xor(term, 2, 64);
                    term += __shfl_xor(term, 1, 64);
                    if (tr < rows && hl == 0) a.logp[row] = term - 0.918938533204672742f * (float)a.adim;
                }
            }
        }
        __syncthreads();  // the tile's last readers are done before the next tile is gathered
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

// the launches since the last record's end belong to it too (a merge after a split GEMM)
static void prof_extend(const morlax_ctx* c, hipStream_t s) {
    GemmProf* pr = c->prof;
    if (pr && pr->on && pr->used > 0) (void)hipEventRecord(pr->recs[pr->used - 1].b, s);
}

// The direct-to-LDS kernel serves bf16 GEMMs of compact operands whose contraction length is a multiple
// of 32 and whose addresses are 16-byte aligned; everything else runs k_grouped_gemm.
template <int KIND>
static bool dma_operand_ok(const void* base, int64_t ld, int rows, int kdim, int64_t pstride) {
    if ((reinterpret_cast<uintptr_t>(base) & 15) || (ld & 7) || (pstride & 7)) return false;
    if (KIND == SRC_KCONTIG) return rows >= 1 && (int64_t)rows * ld * 2 < (int64_t(1) << 31);
    return rows >= 8 && (rows & 7) == 0 && (64 * ld + rows) * 2 < (int64_t(1) << 31);
}
static int resident_slots() {  // workgroups of the persistent kernel: two per CU
    static int n = 0;
    if (n == 0) {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
            cus = 256;
        n = 2 * cus;
    }
    return n;
}

template <typename T, int KA, int KB, class Epi, bool FAST, int NCH>
static bool launch_dma(GemmArgs<T, KA, KB, Epi, FAST, NCH>& g, int P, int nb, hipStream_t s) {
    if constexpr (std::is_same<T, bf16_t>::value && FAST && (KA == SRC_KCONTIG || KA == SRC_KSTRIDED) &&
                  (KB == SRC_KCONTIG || KB == SRC_KSTRIDED)) {
        if (g.a.kdim < 32 || (g.a.kdim & 31)) return false;
        if (!dma_operand_ok<KA>(g.a.base, g.a.ld, g.a.rows, g.a.kdim, g.a_pstride)) return false;
        if (!dma_operand_ok<KB>(g.b.base, g.b.ld, g.b.rows, g.b.kdim, g.b_pstride)) return false;
        // large problems: persistent kernel, 256 x 256 tiles (one workgroup of eight waves per CU) when the
        // output is at least that wide and there is a tile for every CU, else 256 x 128 tiles (two workgroups
        // of four waves per CU) as soon as those fill the resident workgroups
        const int ptm = (g.a.rows + PG_TM - 1) / PG_TM;
        auto launch_pers = [&](auto tn_tag, int slots) {
            constexpr int TN = decltype(tn_tag)::value;
            const int ptn = (g.b.rows + TN - 1) / TN, pnt = ptm * ptn * P;
            static bool pattr_set = false;
            constexpr int plds = PgShape<TN>::kLds + 8 * TN;
            if (!pattr_set) {
                (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_pers<KA, KB, Epi, TN>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, plds);
                pattr_set = true;
            }
            g.tiles_m = ptm;
            g.tiles_n = ptn;
            const int grid = pnt < slots ? pnt : slots;
            k_gemm_pers<KA, KB, Epi, TN><<<grid, 2 * TN, plds, s>>>(g, pnt);
        };
        if (g.a.rows >= 64) {
            const int slots = resident_slots();
            // (the wide shape as soon as there is a tile per CU: a third fewer operand bytes per product through the
            // vector cache, whose requests in flight are what the products wait for; dW at W = 512 with two tiles per
            // workgroup: 8.3 -> 7.9 ms per step of workload 5, with one tile per workgroup at workload 4: 0.945 -> 0.915)
            if (g.b.rows >= 256 && ptm * ((g.b.rows + 255) / 256) * P >= slots / 2) {
                launch_pers(std::integral_constant<int, 256>{}, slots / 2);
                return true;
            }
            if (ptm * ((g.b.rows + 127) / 128) * P >= slots) {
                launch_pers(std::integral_constant<int, 128>{}, slots);
                return true;
            }
        }
        static bool attr_set = false;
        constexpr int lds_bytes = DMA_NST * DMA_STAGE_BYTES;
        if (!attr_set) {
            (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_dma<KA, KB, Epi>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
            attr_set = true;
        }
        k_gemm_dma<KA, KB, Epi><<<nb, 256, lds_bytes, s>>>(g);
        return true;
    } else {
        (void)g; (void)nb; (void)s;
        return false;
    }
}

template <typename T, int KA, int KB, class Epi, bool FAST, int NCH>
static void run_gemm(const morlax_ctx* c, int kind, GemmArgs<T, KA, KB, Epi, FAST, NCH>& g, int P, hipStream_t s) {
    g.tiles_m = (g.a.rows + BM - 1) / BM;
    g.tiles_n = (g.b.rows + BN - 1) / BN;
    const int nb = g.tiles_m * g.tiles_n * P;
    GemmProf::Rec* r = prof_take(c, kind, 2.0 * g.a.rows * (double)g.b.rows * g.a.kdim * P);
    if (r) (void)hipEventRecord(r->a, s);
    if (!launch_dma(g, P, nb, s)) k_grouped_gemm<T, KA, KB, Epi, FAST, NCH><<<nb, 256, 0, s>>>(g);
    if (r) (void)hipEventRecord(r->b, s);
}

// ---- output layer ------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_head_fwd(const T* __restrict__ Hin, const T* __restrict__ theta_mat,
                                                 const float* __restrict__ theta_vec, int64_t mat_len,
                                                 int64_t vec_len, int64_t mat_off, int64_t vec_off, int W,
                                                 int out_dim, int M, RowMap rm, int tanh_cols,
                                                 float* __restrict__ out, float* __restrict__ saved_out,
                                                 const float* __restrict__ eps, float* __restrict__ act,
                                                 float* __restrict__ logp, int64_t logsig_off, int adim,
                                                 int sig_state) {
    constexpr int VE = Elems<T>::VE;
    const int p = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m0 = (blockIdx.x * 4 + wave) * 16;
    if (m0 >= M) return;
    const int lr = lane & 15, lg = lane >> 4;
    const T* hrow = Hin + ((int64_t)p * M + (m0 + lr)) * W;
    const T* wrow = theta_mat + (int64_t)p * mat_len + mat_off + (int64_t)lr * W;
    const bool a_ok = (m0 + lr) < M, b_ok = lr < out_dim;
    // eight contraction steps per batch: their loads are issued together, and two accumulators alternate so
    // that consecutive MFMAs do not wait for each other
    float4_t c = {0.f, 0.f, 0.f, 0.f}, c2 = {0.f, 0.f, 0.f, 0.f};
    for (int k0 = 0; k0 < W; k0 += 32 * VE) {
        uint4 fa[8], fb[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int k = k0 + (4 * u + lg) * VE;
            fa[u] = make_uint4(0, 0, 0, 0);
            fb[u] = make_uint4(0, 0, 0, 0);
            if (a_ok && k < W) fa[u] = *reinterpret_cast<const uint4*>(hrow + k);
            if (b_ok && k < W) fb[u] = *reinterpret_cast<const uint4*>(wrow + k);
        }
#pragma unroll
        for (int u = 0; u < 8; u += 2) {
            Mma16<T>::run(fa[u], fb[u], c);
            Mma16<T>::run(fa[u + 1], fb[u + 1], c2);
        }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) c[e] += c2[e];
    // lane holds column lr of rows m0 + 4*lg + e
    const float bias = b_ok ? theta_vec[(int64_t)p * vec_len + vec_off + lr] : 0.f;
    const bool mean_lane = lr < adim;  // lanes that hold an action mean
    float ls_p = 0.f;
    if (eps && mean_lane && !sig_state) ls_p = theta_vec[(int64_t)p * vec_len + logsig_off + lr];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int m = m0 + 4 * lg + e;
        const bool ok = (m < M) && b_ok;
        const float z = c[e] + bias;
        const float o = (lr < tanh_cols) ? tanhf(z) : z;
        int64_t row = 0;
        if (m < M) row = rm.row(p, m);
        float term = 0.f;
        // a state-dependent log sigma sits adim columns to the right, in the same group of 16 lanes
        const float ls_s = __shfl(o, (lane & 48) | ((lr + adim) & 15), 64);
        if (ok) {
            out[row * out_dim + lr] = o;
            if (saved_out) saved_out[((int64_t)p * M + m) * OUT_PITCH + lr] = o;
            if (eps && mean_lane) {
                const float ls = sig_state ? ls_s : ls_p;
                const float ep = eps[row * adim + lr];
                act[row * adim + lr] = o + expf(ls) * ep;
                term = -0.5f * ep * ep - ls;
            }
        }
        if (eps) {
            term += __shfl_xor(term, 8, 64);
            term += __shfl_xor(term, 4, 64);
            term += __shfl_xor(term, 2, 64);
            term += __shfl_xor(term, 1, 64);
            if (m < M && lr == 0) logp[row] = term - 0.918938533204672742f * (float)adim;
        }
    }
}

// dz_L = dout * (1 - mu^2) for the tanh head (else dout), gathered once per call into compact rows
// dzh[p][m][0..15] (unrounded, zero beyond out_dim) for the two kernels below; the bias gradient
// db_L(p)[j] = sum_m dz_L[m, j] leaves as per-block partials pb[p][block][j] (256 rows per block, summed in a
// fixed order).
template <typename T>
__global__ __launch_bounds__(256) void k_head_dzh(const float* __restrict__ dout, const float* __restrict__ saved_out,
                                                 float* __restrict__ dzh, float* __restrict__ pb, int out_dim, int M,
                                                 RowMap rm, int tanh_cols) {
    __shared__ float red[4][MORLAX_MAX_OUT];
    const int p = blockIdx.y, m = blockIdx.x * 256 + threadIdx.x;
    float d[MORLAX_MAX_OUT];
#pragma unroll
    for (int j = 0; j < MORLAX_MAX_OUT; ++j) d[j] = 0.f;
    if (m < M) {
        const int64_t row = rm.row(p, m);
#pragma unroll
        for (int j = 0; j < MORLAX_MAX_OUT; ++j) {
            if (j < out_dim) {
                d[j] = dout[row * out_dim + j];
                if (j < tanh_cols) {
                    const float mu = saved_out[((int64_t)p * M + m) * OUT_PITCH + j];
                    d[j] *= (1.f - mu * mu);
                }
            }
        }
        float4* dst = reinterpret_cast<float4*>(dzh + ((int64_t)p * M + m) * MORLAX_MAX_OUT);
#pragma unroll
        for (int q = 0; q < MORLAX_MAX_OUT / 4; ++q) dst[q] = make_float4(d[4 * q], d[4 * q + 1], d[4 * q + 2], d[4 * q + 3]);
    }
    // bias partials: butterfly inside each wave, then the four waves in order
#pragma unroll
    for (int j = 0; j < MORLAX_MAX_OUT; ++j) {
        float v = d[j];
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6][j] = v;
    }
    __syncthreads();
    if (threadIdx.x < MORLAX_MAX_OUT)
        pb[((int64_t)p * gridDim.x + blockIdx.x) * MORLAX_MAX_OUT + threadIdx.x] =
            (red[0][threadIdx.x] + red[1][threadIdx.x]) + (red[2][threadIdx.x] + red[3][threadIdx.x]);
}

// dZ_{L-1}[m, i] = (sum_j dz_L[m, j] W_L(p)[j, i]) * act'(z_{L-1})[m, i].  Block: 64 rows x 128 columns of
// one preference; thread: 4 rows x 8 columns.
template <typename T>
__global__ __launch_bounds__(256) void k_head_bwd_dz(const float* __restrict__ dzh,
                                                    const T* __restrict__ theta_mat, int64_t mat_len,
                                                    int64_t mat_off,
                                                    const typename GradT<T>::type* __restrict__ G,
                                                    T* __restrict__ dZ, float* __restrict__ part,
                                                    int W, int out_dim, int M) {
    __shared__ float sdz[64][MORLAX_MAX_OUT];
    __shared__ float red[16][128];
    const int p = blockIdx.z, m0 = blockIdx.y * 64, i0 = blockIdx.x * 128;
    for (int idx = threadIdx.x; idx < 64 * MORLAX_MAX_OUT; idx += 256) {
        const int mm = idx / MORLAX_MAX_OUT, j = idx % MORLAX_MAX_OUT;
        float d = 0.f;
        if (m0 + mm < M) d = to_f(cvt<T>(dzh[((int64_t)p * M + m0 + mm) * MORLAX_MAX_OUT + j]));  // GEMM input rounding
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

// Transposing 8-byte LDS read: the 16 lanes of a group address the 64-bit words of a 4 x 16 block of 16-bit values
// -- lane 4 e + c the word of contraction index e that holds columns 4 c .. 4 c + 3 -- and lane b of the group
// receives the four contraction indices of column b: the B operand of a 16x16x16 MFMA read from a row-major tile.
template <typename E>
__device__ inline short4_t lds_tr4(const E* word) {
    typedef __attribute__((address_space(3))) short4_t lds_s4;
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4*)(word));
}

// dW_L(p)[j, i] = sum_m dz_L[m, j] h_{L-1}[m, i] in two stages.  Stage 1: a block takes one of HB_SPLIT row
// ranges of one preference and 128 columns, and walks its rows 128 at a time: the dz rows (rounded to the
// GEMM input type) and the h tile sit in LDS, the next h tile is already on its way in registers; wave w
// multiplies dz^T [16 x 128] by h [128 x columns 32 w .. 32 w + 31]: bf16 networks with 16x16x16 bf16 MFMAs (dz^T
// staged with the contraction contiguous, h read through transposing LDS reads), fp32 ones with 16x16x4 MFMAs.  Partials go to pw[p][range][j][i]; stage 2
// (k_head_bwd_dw_final) adds the ranges, and the bias partials of k_head_dzh, in order.
#define HB_ROWS 128
#define HB_SPLIT 4
template <typename T>
__global__ __launch_bounds__(256) void k_head_bwd_dw(const float* __restrict__ dzh, const T* __restrict__ Hin,
                                                    float* __restrict__ pw, int W, int M) {
    constexpr int VE = Elems<T>::VE;
    constexpr int HP = 128 + VE;                           // h tile pitch in elements (16 bytes of padding)
    constexpr int CPR = 128 / VE;                          // 16-byte pieces per tile row
    constexpr int NPT = HB_ROWS * CPR / 256;               // pieces per thread
    constexpr bool kBf = std::is_same<T, bf16_t>::value;
    __shared__ __align__(16) float sdr[kBf ? 1 : HB_ROWS][MORLAX_MAX_OUT];        // fp32: dz rows as they lie
    __shared__ __align__(16) bf16_t sdT[kBf ? MORLAX_MAX_OUT : 1][HB_ROWS + 8];  // bf16: dz^T, contraction contiguous
    __shared__ __align__(16) T sh[HB_ROWS][HP];
    const int p = blockIdx.z, rs = blockIdx.y, i0 = blockIdx.x * 128;
    const int per = ((M + HB_SPLIT - 1) / HB_SPLIT + HB_ROWS - 1) / HB_ROWS * HB_ROWS;  // rows per range
    const int m_lo = rs * per, m_hi = (m_lo + per < M) ? (m_lo + per) : M;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int ln = lane & 15, kg = lane >> 4;
    float4_t acc[2][2];
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int q = 0; q < 2; ++q) acc[c][q] = float4_t{0.f, 0.f, 0.f, 0.f};
    uint4 nxt[NPT];
    auto fetch = [&](int m0) {
#pragma unroll
        for (int q = 0; q < NPT; ++q) {
            const int idx = threadIdx.x + 256 * q, mm = idx / CPR, cc = (idx % CPR) * VE;
            uint4 u = make_uint4(0, 0, 0, 0);
            if (m0 + mm < m_hi && i0 + cc < W)
                u = *reinterpret_cast<const uint4*>(Hin + ((int64_t)p * M + m0 + mm) * W + i0 + cc);
            nxt[q] = u;
        }
    };
    if (m_lo < m_hi) fetch(m_lo);
    for (int m0 = m_lo; m0 < m_hi; m0 += HB_ROWS) {
        __syncthreads();  // the previous tile has been multiplied
#pragma unroll
        for (int q = 0; q < NPT; ++q) {
            const int idx = threadIdx.x + 256 * q;
            *reinterpret_cast<uint4*>(&sh[idx / CPR][(idx % CPR) * VE]) = nxt[q];
        }
        for (int idx = threadIdx.x; idx < HB_ROWS * (MORLAX_MAX_OUT / 4); idx += 256) {
            const int mm = idx / (MORLAX_MAX_OUT / 4), q = idx % (MORLAX_MAX_OUT / 4);
            float4 d = make_float4(0.f, 0.f, 0.f, 0.f);
            if (m0 + mm < m_hi) d = *reinterpret_cast<const float4*>(dzh + ((int64_t)p * M + m0 + mm) * MORLAX_MAX_OUT + 4 * q);
            if constexpr (kBf) {
                sdT[4 * q][mm] = cvt<T>(d.x); sdT[4 * q + 1][mm] = cvt<T>(d.y);
                sdT[4 * q + 2][mm] = cvt<T>(d.z); sdT[4 * q + 3][mm] = cvt<T>(d.w);
            } else {
                sdr[mm][4 * q] = to_f(cvt<T>(d.x)); sdr[mm][4 * q + 1] = to_f(cvt<T>(d.y));
                sdr[mm][4 * q + 2] = to_f(cvt<T>(d.z)); sdr[mm][4 * q + 3] = to_f(cvt<T>(d.w));
            }
        }
        if (m0 + HB_ROWS < m_hi) fetch(m0 + HB_ROWS);
        __syncthreads();
        if constexpr (kBf) {
            // both operands are bf16 values: 16x16x16 bf16 MFMAs, eight times the fp32 rate for the same sums
#pragma unroll
            for (int ks = 0; ks < HB_ROWS / 16; ++ks) {
                const short4_t a = *reinterpret_cast<const short4_t*>(&sdT[ln][16 * ks + 4 * kg]);  // dz^T[j = ln][4 m]
#pragma unroll
                for (int c = 0; c < 2; ++c)
                    acc[c][ks & 1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(
                        a, lds_tr4(&sh[16 * ks + 4 * kg + (ln >> 2)][32 * wave + 16 * c + 4 * (ln & 3)]), acc[c][ks & 1], 0, 0, 0);
            }
        } else {
#pragma unroll
            for (int kk = 0; kk < HB_ROWS / 4; ++kk) {
                const int m = 4 * kk + kg;
                const float a = sdr[m][ln];                              // dz^T[j = ln][m]
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    const float b = to_f(sh[m][32 * wave + 16 * c + ln]);  // h[m][column]
                    acc[c][kk & 1] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[c][kk & 1], 0, 0, 0);
                }
            }
        }
    }
    // lane holds column ln of rows j = 4 kg + e
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        const int col = i0 + 32 * wave + 16 * c + ln;
        if (col < W) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                pw[(((int64_t)p * HB_SPLIT + rs) * MORLAX_MAX_OUT + 4 * kg + e) * W + col] = acc[c][0][e] + acc[c][1][e];
        }
    }
}

// ---- dW of a W x W layer with few preferences: contraction split into ranges ---------------------------------
// dW_l(p) has (W/128)^2 tiles per preference and the whole selection as its contraction; with few preferences that
// is a few dozen workgroups walking thousands of rows each.  The selection is cut into S equal ranges that run as
// P S groups of the same grouped GEMM into partial matrices, and the ranges are added in order.
#ifndef DW_SPLIT_TARGET
#define DW_SPLIT_TARGET 512
#endif
__global__ __launch_bounds__(256) void k_dw_split_final(const float* __restrict__ pw, int S, int64_t WW,
                                                       float* __restrict__ dtheta_mat, int64_t mat_len, int64_t mat_off) {
    const int p = blockIdx.y;
    const int64_t i4 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i4 >= WW) return;
    float4 v = *reinterpret_cast<const float4*>(pw + (int64_t)p * S * WW + i4);
    for (int c = 1; c < S; ++c) {
        const float4 u = *reinterpret_cast<const float4*>(pw + ((int64_t)p * S + c) * WW + i4);
        v.x += u.x; v.y += u.y; v.z += u.z; v.w += u.w;
    }
    // W is a multiple of 16, so every matrix starts on a 16-byte boundary of the row
    *reinterpret_cast<float4*>(dtheta_mat + (int64_t)p * mat_len + mat_off + i4) = v;
}

// ---- forward of the first layer with a narrow observation (O <= 32) ---------------------------------------
// h = act(x W0(p)^T + b0(p)) is, per output, an inner product of O terms: too short to fill GEMM tiles (the tiled
// kernel pads the contraction to 32 and loads the odd-width rows element by element) and bound by the stores of h
// and act'(z).  A block of 256 threads takes FN_ROWS rows of one preference with W0(p) in LDS, transposed to
// [i][o] in fp32 (exact for bf16 weights), and the rows' observations rounded to the network's type as the GEMM
// rounds them; a thread owns eight consecutive outputs of FN_ROWS / RPT rows, walks the contraction once with its
// eight weights of the step in registers, and stores 16- or 32-byte pieces that the threads of a row join to whole
// rows.  Sums run in ascending i in fp32, as one accumulator per output.
#define FN_ROWS 64
template <typename T, int ACT, bool SAVE>
__global__ __launch_bounds__(256) void k_first_fwd_narrow(const float* __restrict__ x, const T* __restrict__ theta_mat,
                                                         const float* __restrict__ theta_vec, int64_t mat_len,
                                                         int64_t vec_len, int64_t mat_off, int64_t vec_off, int O, int W,
                                                         int M, RowMap rm, T* __restrict__ H,
                                                         typename GradT<T>::type* __restrict__ G) {
    extern __shared__ __align__(16) float fn_lds[];
    const int WP = W + 4;  // pitch of a row of W0^T: keeps 16-byte alignment, shifts the banks from row to row
    float* sw = fn_lds;               // [O][WP]
    float* sb = sw + O * WP;          // [W]
    float* sx = sb + W;               // [FN_ROWS][O]
    const int p = blockIdx.y, m0 = blockIdx.x * FN_ROWS;
    const T* w0 = theta_mat + (int64_t)p * mat_len + mat_off;
    for (int idx = threadIdx.x; idx < W * O; idx += 256) {
        const int o = idx / O, i = idx - o * O;
        sw[i * WP + o] = to_f(w0[idx]);
    }
    for (int o = threadIdx.x; o < W; o += 256) sb[o] = theta_vec[(int64_t)p * vec_len + vec_off + o];
    for (int idx = threadIdx.x; idx < FN_ROWS * O; idx += 256) {
        const int r = idx / O, i = idx - r * O;
        const int m = m0 + r < M ? m0 + r : M - 1;
        sx[idx] = to_f(cvt<T>(x[rm.row(p, m) * O + i]));
    }
    __syncthreads();
    const int CH = W >> 3;        // pieces of eight outputs per row (at most 256)
    const int RPT = 256 / CH;     // rows in work at a time
    const int chunk = threadIdx.x % CH, slot = threadIdx.x / CH;
    if (slot >= RPT) return;
    constexpr int TURNS = 8;      // rows per thread and pass
    for (int r0 = 0; r0 < FN_ROWS; r0 += RPT * TURNS) {
        float acc[TURNS][8];
        const float4 b0 = *reinterpret_cast<const float4*>(sb + 8 * chunk), b1 = *reinterpret_cast<const float4*>(sb + 8 * chunk + 4);
        const float* xr[TURNS];
#pragma unroll
        for (int t = 0; t < TURNS; ++t) {
            acc[t][0] = b0.x; acc[t][1] = b0.y; acc[t][2] = b0.z; acc[t][3] = b0.w;
            acc[t][4] = b1.x; acc[t][5] = b1.y; acc[t][6] = b1.z; acc[t][7] = b1.w;
            const int r = r0 + slot + t * RPT;
            xr[t] = sx + (r < FN_ROWS ? r : FN_ROWS - 1) * O;
        }
        for (int i = 0; i < O; ++i) {  // (the observation values read four steps at a time measured no faster)
            const float4 wa = *reinterpret_cast<const float4*>(sw + i * WP + 8 * chunk);
            const float4 wb = *reinterpret_cast<const float4*>(sw + i * WP + 8 * chunk + 4);
#pragma unroll
            for (int t = 0; t < TURNS; ++t) {
                const float xv = xr[t][i];
                acc[t][0] += xv * wa.x; acc[t][1] += xv * wa.y; acc[t][2] += xv * wa.z; acc[t][3] += xv * wa.w;
                acc[t][4] += xv * wb.x; acc[t][5] += xv * wb.y; acc[t][6] += xv * wb.z; acc[t][7] += xv * wb.w;
            }
        }
#pragma unroll
        for (int t = 0; t < TURNS; ++t) {
            const int r = r0 + slot + t * RPT, m = m0 + r;
            if (r < FN_ROWS && m < M) {
                float g[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) act_pair<ACT>(acc[t][u], acc[t][u], g[u]);
                const int64_t at = ((int64_t)p * M + m) * W + 8 * chunk;
                put8(H + at, pack8(acc[t], (const T*)nullptr));
                if (SAVE) put8(G + at, pack8(g, (const typename GradT<T>::type*)nullptr));
            }
        }
    }
}
static int64_t first_fwd_narrow_lds(const morlax_ctx* c) {
    return ((int64_t)(c->d.width + 4) * c->d.obs_dim + c->d.width + (int64_t)FN_ROWS * c->d.obs_dim) * 4;
}
static bool first_fwd_narrow_ok(const morlax_ctx* c) {
    // bf16 networks only: with fp32 outputs (twice the bytes per store) the tiled kernel measured faster
    return c->d.wdtype == 1 && c->d.obs_dim <= 32 && c->d.width % 8 == 0 && c->d.width <= 2048 &&
           first_fwd_narrow_lds(c) <= 64 * 1024;
}

// ---- first layer with a narrow observation (O <= 32) and few preferences ----------------------------------
// dW_0(p)[o, i] = sum_m dZ_0[m, o] x[m, i] has W x O outputs and the whole selection as its contraction: as a tiled
// GEMM it is two or three tiles per preference walking thousands of rows each (workload 2: 32 workgroups on 256 CUs).
// It is the output layer's dW with the roles exchanged, so it takes the same streaming form: the observation rows
// are gathered once into compact fp32 rows padded to 16 JB columns, a block takes one of n_split row ranges of one
// preference and 128 columns of dZ_0, and the ranges are added in order by k_first_dw_final.
template <typename T>
__global__ __launch_bounds__(256) void k_gather_x_pad(const float* __restrict__ x, float* __restrict__ xz, int O, int OP,
                                                     int M, RowMap rm) {
    const int p = blockIdx.y;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)M * OP) return;
    const int m = (int)(idx / OP), c = (int)(idx % OP);
    xz[((int64_t)p * M + m) * OP + c] = c < O ? x[rm.row(p, m) * O + c] : 0.f;
}

template <typename T, int JB>
__global__ __launch_bounds__(256) void k_first_bwd_dw(const float* __restrict__ xz, const T* __restrict__ dZ,
                                                     float* __restrict__ pw, int W, int M, int n_split) {
    constexpr int VE = Elems<T>::VE;
    constexpr int HP = 128 + VE;
    constexpr int CPR = 128 / VE;
    constexpr int NPT = HB_ROWS * CPR / 256;
    constexpr int OP = 16 * JB;
    constexpr bool kBf = std::is_same<T, bf16_t>::value;
    __shared__ __align__(16) float sdr[kBf ? 1 : HB_ROWS][OP];        // fp32: observation rows as they lie
    __shared__ __align__(16) bf16_t sdT[kBf ? OP : 1][HB_ROWS + 8];  // bf16: x^T, contraction contiguous
    __shared__ __align__(16) T sh[HB_ROWS][HP];
    const int p = blockIdx.z, rs = blockIdx.y, i0 = blockIdx.x * 128;
    const int per = ((M + n_split - 1) / n_split + HB_ROWS - 1) / HB_ROWS * HB_ROWS;  // rows per range
    const int m_lo = rs * per, m_hi = (m_lo + per < M) ? (m_lo + per) : M;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int ln = lane & 15, kg = lane >> 4;
    float4_t acc[JB][2][2];
#pragma unroll
    for (int jb = 0; jb < JB; ++jb)
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int q = 0; q < 2; ++q) acc[jb][c][q] = float4_t{0.f, 0.f, 0.f, 0.f};
    uint4 nxt[NPT];
    auto fetch = [&](int m0) {
#pragma unroll
        for (int q = 0; q < NPT; ++q) {
            const int idx = threadIdx.x + 256 * q, mm = idx / CPR, cc = (idx % CPR) * VE;
            uint4 u = make_uint4(0, 0, 0, 0);
            if (m0 + mm < m_hi && i0 + cc < W)
                u = *reinterpret_cast<const uint4*>(dZ + ((int64_t)p * M + m0 + mm) * W + i0 + cc);
            nxt[q] = u;
        }
    };
    if (m_lo < m_hi) fetch(m_lo);
    for (int m0 = m_lo; m0 < m_hi; m0 += HB_ROWS) {
        __syncthreads();  // the previous tile has been multiplied
#pragma unroll
        for (int q = 0; q < NPT; ++q) {
            const int idx = threadIdx.x + 256 * q;
            *reinterpret_cast<uint4*>(&sh[idx / CPR][(idx % CPR) * VE]) = nxt[q];
        }
        for (int idx = threadIdx.x; idx < HB_ROWS * (OP / 4); idx += 256) {
            const int mm = idx / (OP / 4), q = idx % (OP / 4);
            float4 d = make_float4(0.f, 0.f, 0.f, 0.f);
            if (m0 + mm < m_hi) d = *reinterpret_cast<const float4*>(xz + ((int64_t)p * M + m0 + mm) * OP + 4 * q);
            if constexpr (kBf) {  // GEMM input rounding
                sdT[4 * q][mm] = cvt<T>(d.x); sdT[4 * q + 1][mm] = cvt<T>(d.y);
                sdT[4 * q + 2][mm] = cvt<T>(d.z); sdT[4 * q + 3][mm] = cvt<T>(d.w);
            } else {
                sdr[mm][4 * q] = to_f(cvt<T>(d.x)); sdr[mm][4 * q + 1] = to_f(cvt<T>(d.y));
                sdr[mm][4 * q + 2] = to_f(cvt<T>(d.z)); sdr[mm][4 * q + 3] = to_f(cvt<T>(d.w));
            }
        }
        if (m0 + HB_ROWS < m_hi) fetch(m0 + HB_ROWS);
        __syncthreads();
        if constexpr (kBf) {
#pragma unroll
            for (int ks = 0; ks < HB_ROWS / 16; ++ks) {
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    const short4_t b = lds_tr4(&sh[16 * ks + 4 * kg + (ln >> 2)][32 * wave + 16 * c + 4 * (ln & 3)]);
#pragma unroll
                    for (int jb = 0; jb < JB; ++jb)
                        acc[jb][c][ks & 1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(
                            *reinterpret_cast<const short4_t*>(&sdT[16 * jb + ln][16 * ks + 4 * kg]), b, acc[jb][c][ks & 1], 0, 0, 0);
                }
            }
        } else {
#pragma unroll
            for (int kk = 0; kk < HB_ROWS / 4; ++kk) {
                const int m = 4 * kk + kg;
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    const float b = to_f(sh[m][32 * wave + 16 * c + ln]);  // dZ_0[m][column]
#pragma unroll
                    for (int jb = 0; jb < JB; ++jb)
                        acc[jb][c][kk & 1] = __builtin_amdgcn_mfma_f32_16x16x4f32(sdr[m][16 * jb + ln], b, acc[jb][c][kk & 1], 0, 0, 0);
                }
            }
        }
    }
    // lane holds column ln of observation components 16 jb + 4 kg + e
#pragma unroll
    for (int jb = 0; jb < JB; ++jb)
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const int col = i0 + 32 * wave + 16 * c + ln;
            if (col < W) {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    pw[(((int64_t)p * n_split + rs) * OP + 16 * jb + 4 * kg + e) * W + col] = acc[jb][c][0][e] + acc[jb][c][1][e];
            }
        }
}

// dW_0(p)[o, i] = the ranges' partials [i][o] added in order
__global__ __launch_bounds__(256) void k_first_dw_final(const float* __restrict__ pw, int n_split, int OP,
                                                       float* __restrict__ dtheta_mat, int64_t mat_len, int64_t mat_off,
                                                       int W, int O) {
    const int p = blockIdx.y, idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= W * O) return;
    const int o = idx / O, i = idx % O;
    float v = 0.f;
    for (int c = 0; c < n_split; ++c) v += pw[(((int64_t)p * n_split + c) * OP + i) * W + o];
    dtheta_mat[(int64_t)p * mat_len + mat_off + idx] = v;
}

__global__ __launch_bounds__(256) void k_head_bwd_dw_final(const float* __restrict__ pw, const float* __restrict__ pb,
                                                          int n_chunk_w, int n_chunk_b, float* __restrict__ dtheta_mat,
                                                          float* __restrict__ dtheta_vec, int64_t mat_len,
                                                          int64_t vec_len, int64_t mat_off, int64_t vec_off, int W,
                                                          int out_dim) {
    const int p = blockIdx.y, idx = blockIdx.x * 256 + threadIdx.x;
    if (idx < out_dim * W) {
        const int j = idx / W, i = idx % W;
        float v = 0.f;
        for (int c = 0; c < n_chunk_w; ++c) v += pw[(((int64_t)p * n_chunk_w + c) * MORLAX_MAX_OUT + j) * W + i];
        dtheta_mat[(int64_t)p * mat_len + mat_off + idx] = v;
    }
    if (idx < out_dim) {
        float v = 0.f;
        for (int c = 0; c < n_chunk_b; ++c) v += pb[((int64_t)p * n_chunk_b + c) * MORLAX_MAX_OUT + idx];
        dtheta_vec[(int64_t)p * vec_len + vec_off + idx] = v;
    }
}

// db_l(p)[o] = sum over the row blocks of the partial column sums of dZ_l.  A block takes 32 columns of one
// preference; its eight groups of 32 threads each add a contiguous eighth of the row blocks in order, and the eight
// sums are added in group order (a fixed association: results repeat bit for bit).
__global__ __launch_bounds__(256) void k_colsum_final(const float* __restrict__ part, int n_part,
                                                     float* __restrict__ dtheta_vec, int64_t vec_len,
                                                     int64_t vec_off, int W) {
    __shared__ float sg[8][32];
    const int p = blockIdx.y, c = threadIdx.x & 31, g = threadIdx.x >> 5, i = blockIdx.x * 32 + c;
    const int per = (n_part + 7) / 8, q_lo = g * per, q_hi = (q_lo + per < n_part) ? q_lo + per : n_part;
    float a = 0.f;
    if (i < W)
        for (int q = q_lo; q < q_hi; ++q) a += part[((int64_t)p * n_part + q) * W + i];
    sg[g][c] = a;
    __syncthreads();
    if (g == 0 && i < W) {
        float t = sg[0][c];
#pragma unroll
        for (int k = 1; k < 8; ++k) t += sg[k][c];
        dtheta_vec[(int64_t)p * vec_len + vec_off + i] = t;
    }
}

__global__ void k_copy_dlogsig(const float* __restrict__ dlogsig, float* __restrict__ dtheta_vec, int64_t vec_len,
                               int64_t off, int P, int A) {
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= P * A) return;
    const int p = idx / A, a = idx % A;
    dtheta_vec[(int64_t)p * vec_len + off + a] = dlogsig ? dlogsig[idx] : 0.f;
}

// Rows of the fp32 observation tensor picked by the row map, rounded to the GEMM input type, as compact
// [P][M][O] rows (O a multiple of 8): the first layer's GEMMs then run on the direct-to-LDS kernels.
template <typename T>
__global__ __launch_bounds__(256) void k_gather_x(const float* __restrict__ x, T* __restrict__ xc, int O, int M,
                                                 RowMap rm) {
    const int p = blockIdx.y;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;  // one 8-element piece
    const int per_row = O / 8;
    if (idx >= (int64_t)M * per_row) return;
    const int m = (int)(idx / per_row), c = (int)(idx % per_row) * 8;
    const float* src = x + rm.row(p, m) * O + c;
    float v[8];
    get8(src, v);
    store8(xc + ((int64_t)p * M + m) * O + c, v);
}

// ---- host side ---------------------------------------------------------------------------------
static int64_t esize(const morlax_ctx* c) { return c->d.wdtype == 1 ? 2 : 4; }
static int64_t act_elems(const morlax_ctx* c, const RowSel& rs) {
    return align_up((int64_t)c->d.P * rs.M * c->d.width, 64);
}

static int64_t x0_elems(const morlax_ctx* c, const RowSel& rs) {
    return align_up((int64_t)c->d.P * rs.M * c->d.obs_dim, 64);
}
// compact first-layer input: bf16 networks whose observation width suits the direct-to-LDS GEMMs
static bool use_x0(const morlax_ctx* c) { return c->d.wdtype == 1 && c->d.obs_dim % 32 == 0; }
// saved: per hidden layer h and act', then the head's output rows, then (when used) the gathered observations
int64_t mlp_saved_bytes(const morlax_ctx* c, int net, const RowSel& rs) {
    (void)net;
    return 2 * (int64_t)c->d.n_hidden * act_elems(c, rs) * esize(c) +
           align_up((int64_t)c->d.P * rs.M * OUT_PITCH * 4, 256) + (use_x0(c) ? x0_elems(c, rs) * esize(c) : 0);
}
// fp32 scratch behind the two activation buffers: [0, head_lo): partial column sums of dZ, or the output
// layer's dW partials followed by its bias partials; [head_lo, ..): the compact dz rows of the output layer
// (still read while the column sums of the layer below are written).
static int64_t head_pw_elems(const morlax_ctx* c) { return (int64_t)c->d.P * HB_SPLIT * MORLAX_MAX_OUT * c->d.width; }
static int64_t head_lo_elems(const morlax_ctx* c, const RowSel& rs) {
    const int64_t colsum = (int64_t)c->d.P * ((rs.M + 63) / 64) * c->d.width;
    const int64_t head = head_pw_elems(c) + (int64_t)c->d.P * ((rs.M + 255) / 256) * MORLAX_MAX_OUT;
    return align_up(colsum > head ? colsum : head, 64);
}
// the first layer's dW as a streaming split-K kernel: narrow observations and too few GEMM tiles to fill the chip
static bool first_skinny(const morlax_ctx* c) {
    return c->d.obs_dim <= 32 && ((c->d.width + 127) / 128) * c->d.P < 256;
}
static int first_split(const morlax_ctx* c, const RowSel& rs) {
    const int tiles = ((c->d.width + 127) / 128) * c->d.P;
    int n = (1024 + tiles - 1) / tiles;
    const int cap = (rs.M + HB_ROWS - 1) / HB_ROWS;
    n = n > 64 ? 64 : n;
    n = n > cap ? cap : n;
    return n < 1 ? 1 : n;
}
static int64_t first_skinny_elems(const morlax_ctx* c, const RowSel& rs) {  // padded rows, then the ranges' partials
    if (!first_skinny(c)) return 0;
    const int OP = c->d.obs_dim <= 16 ? 16 : 32;
    return align_up((int64_t)c->d.P * rs.M * OP, 64) + align_up((int64_t)c->d.P * first_split(c, rs) * OP * c->d.width, 64);
}
// ranges the contraction of a hidden layer's dW is cut into (1 = the plain grouped GEMM)
static int dw_split(const morlax_ctx* c, const RowSel& rs) {
    const int t = (c->d.width + 127) / 128, tiles = t * t * c->d.P;
    int S = 1;
    while (S < 16 && tiles * S < DW_SPLIT_TARGET && rs.M % (2 * S * 64) == 0 && rs.M / (2 * S) >= 256) S *= 2;
    return S;
}
// room for the partial matrices: sized by the most ranges any selection of at most this many rows can be cut
// into, so that the workspace of a selection also serves every smaller one
static int64_t dw_split_elems(const morlax_ctx* c, const RowSel& rs) {
    const int t = (c->d.width + 127) / 128, tiles = t * t * c->d.P;
    int S = 1;
    while (S < 16 && tiles * S < DW_SPLIT_TARGET && rs.M / (2 * S) >= 256) S *= 2;
    return S > 1 ? align_up((int64_t)c->d.P * S * c->d.width * c->d.width, 64) : 0;
}
static int64_t part_elems(const morlax_ctx* c, const RowSel& rs) {
    return head_lo_elems(c, rs) + align_up((int64_t)c->d.P * rs.M * MORLAX_MAX_OUT, 64) + first_skinny_elems(c, rs) +
           dw_split_elems(c, rs);
}
static bool fused_fwd_dims_ok(const morlax_ctx* c) {
    return c->d.wdtype == 1 && (c->d.width == 512 || c->d.width == 256) && c->d.obs_dim <= c->d.width &&
           c->d.n_hidden >= 1;
}
// elements per preference of the fused forward's copy of the matrices: the first layer's rows padded to a multiple of 64
static int64_t fused_frag_len(const morlax_ctx* c, int net) {
    const int Opad = (c->d.obs_dim + 63) & ~63;
    return c->net[net].mat_len + (int64_t)c->d.width * (Opad - c->d.obs_dim);
}

int64_t mlp_ws_bytes(const morlax_ctx* c, const RowSel& rs) {
    int64_t b = 2 * act_elems(c, rs) * esize(c) + part_elems(c, rs) * 4 + (use_x0(c) ? x0_elems(c, rs) * esize(c) : 0);
    if (fused_fwd_dims_ok(c)) {  // the fused forward's copy of the matrices in fragment order
        for (int net = 0; net < 2; ++net) {
            const int64_t f = align_up((int64_t)c->d.P * fused_frag_len(c, net) * 2, 256);
            if (f > b) b = f;
        }
    }
    return b;
}

static RowMap make_rowmap(const morlax_ctx* c, const RowSel& rs) {
    RowMap rm;
    rm.t0 = rs.t0; rm.j0 = rs.j0; rm.j_cnt = rs.j_cnt; rm.N = c->d.N; rm.n_g = c->n_g;
    return rm;
}

// The fused forward serves bf16 networks of width 512 or 256 (the observation is zero-filled to a multiple of 64 in LDS).
static bool fused_fwd_ok(const morlax_ctx* c, const NetDev& nd, const void* theta_mat) {
    if (!fused_fwd_dims_ok(c)) return false;
    if ((reinterpret_cast<uintptr_t>(theta_mat) & 15) || (nd.mat_len & 7)) return false;
    for (int l = 0; l <= c->d.n_hidden; ++l)
        if (nd.layer[l].mat_off & 7) return false;
    return true;
}

template <int ACT, bool SAVE, int WD>
static void launch_fused_fwd_w(const morlax_ctx* c, const FusedFwdArgs& a, hipStream_t s) {
    constexpr int lds = FF_ROWS * WD * 2 + (SAVE ? (WD / 64) * 4096 : 0);
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_mlp_fused_fwd<ACT, SAVE, WD>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        attr_set = true;
    }
    const double per_row = 2.0 * WD * ((double)a.O + (double)(a.L - 1) * WD);
    GemmProf::Rec* r = prof_take(c, 5, per_row * a.M * c->d.P);
    if (r) (void)hipEventRecord(r->a, s);
    // width 512: one workgroup per CU (the tile fills its LDS); width 256: half the tile and half the waves, two per CU
    const int slots = resident_slots() / 2 * (512 / WD);
    k_mlp_fused_fwd<ACT, SAVE, WD><<<a.n_tiles < slots ? a.n_tiles : slots, WD, lds, s>>>(a);
    if (r) (void)hipEventRecord(r->b, s);
}
template <int ACT, bool SAVE>
static void launch_fused_fwd(const morlax_ctx* c, const FusedFwdArgs& a, hipStream_t s) {
    if (c->d.width == 256) launch_fused_fwd_w<ACT, SAVE, 256>(c, a, s);
    else launch_fused_fwd_w<ACT, SAVE, 512>(c, a, s);
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
    auto layer = [&](int l, auto act_tag, auto save_tag) {
        constexpr int ACT = decltype(act_tag)::value;
        constexpr bool SAVE = decltype(save_tag)::value;
        const LayerDev& Ld = nd.layer[l];
        EpiFwd<T, ACT, SAVE> ep;
        ep.bias = theta_vec + Ld.vec_off;
        ep.H = Hbuf(l);
        ep.G = Gbuf(l);
        ep.ld = W;
        ep.part = nullptr;
        if (l == 0 && use_x0(c)) {
            if constexpr (std::is_same<T, bf16_t>::value) {
                T* x0 = sv ? reinterpret_cast<T*>(reinterpret_cast<char*>(sv) + (int64_t)2 * L * ae * sizeof(T) +
                                                  align_up((int64_t)P * M * OUT_PITCH * 4, 256))
                           : reinterpret_cast<T*>(reinterpret_cast<float*>(wsT + 2 * ae) + part_elems(c, rs));
                const int64_t pieces = (int64_t)M * (O / 8);
                k_gather_x<T><<<dim3((unsigned)((pieces + 255) / 256), P), 256, 0, s>>>(x, x0, O, M, rm);
                GemmArgs<T, SRC_KCONTIG, SRC_KCONTIG, EpiFwd<T, ACT, SAVE>, true, GEMM_NCH> g;
                g.a.base = x0; g.a.ld = O; g.a.rows = M; g.a.kdim = O; g.a.rm = rm;
                g.b.base = theta_mat + Ld.mat_off; g.b.ld = O; g.b.rows = W; g.b.kdim = O; g.b.rm = rm;
                g.a_pstride = (int64_t)M * O; g.b_pstride = nd.mat_len;
                g.epi = ep; g.e0_pstride = nd.vec_len; g.e1_pstride = (int64_t)M * W; g.e2_pstride = 0;
                run_gemm(c, 0, g, P, s);
            }
        } else if (l == 0 && first_fwd_narrow_ok(c)) {
            const int lds = (int)first_fwd_narrow_lds(c);
            static bool attr_set = false;
            if (!attr_set) {
                (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_first_fwd_narrow<T, ACT, SAVE>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, 64 * 1024);
                attr_set = true;
            }
            GemmProf::Rec* r = prof_take(c, 0, 2.0 * M * (double)W * O * P);
            if (r) (void)hipEventRecord(r->a, s);
            k_first_fwd_narrow<T, ACT, SAVE><<<dim3((M + FN_ROWS - 1) / FN_ROWS, P), 256, lds, s>>>(
                x, theta_mat, theta_vec, nd.mat_len, nd.vec_len, Ld.mat_off, Ld.vec_off, O, W, M, rm, Hbuf(0), Gbuf(0));
            if (r) (void)hipEventRecord(r->b, s);
        } else if (l == 0) {
            auto launch = [&](auto fast) {
                constexpr bool F = decltype(fast)::value;
                GemmArgs<T, SRC_X_KCONTIG, SRC_KCONTIG, EpiFwd<T, ACT, SAVE>, F, GEMM_NCH> g;
                g.a.base = x; g.a.ld = O; g.a.rows = M; g.a.kdim = O; g.a.rm = rm;
                g.b.base = theta_mat + Ld.mat_off; g.b.ld = O; g.b.rows = W; g.b.kdim = O; g.b.rm = rm;
                g.a_pstride = 0; g.b_pstride = nd.mat_len;
                g.epi = ep; g.e0_pstride = nd.vec_len; g.e1_pstride = (int64_t)M * W; g.e2_pstride = 0;
                run_gemm(c, 0, g, P, s);
            };
            if (O % VE == 0) launch(std::true_type{}); else launch(std::false_type{});
        } else {
            GemmArgs<T, SRC_KCONTIG, SRC_KCONTIG, EpiFwd<T, ACT, SAVE>, true, GEMM_NCH> g;
            g.a.base = Hbuf(l - 1); g.a.ld = W; g.a.rows = M; g.a.kdim = W; g.a.rm = rm;
            g.b.base = theta_mat + Ld.mat_off; g.b.ld = W; g.b.rows = W; g.b.kdim = W; g.b.rm = rm;
            g.a_pstride = (int64_t)M * W; g.b_pstride = nd.mat_len;
            g.epi = ep; g.e0_pstride = nd.vec_len; g.e1_pstride = (int64_t)M * W; g.e2_pstride = 0;
            run_gemm(c, 1, g, P, s);
        }
    };
    bool fused = false;
    if constexpr (std::is_same<T, bf16_t>::value) {
        if (fused_fwd_ok(c, nd, theta_mat)) {
            FusedFwdArgs a;
            a.x = x;
            a.x0 = (sv && use_x0(c)) ? reinterpret_cast<T*>(reinterpret_cast<char*>(sv) + (int64_t)2 * L * ae * sizeof(T) +
                                                            align_up((int64_t)P * M * OUT_PITCH * 4, 256))
                                     : nullptr;
            a.theta_mat = theta_mat; a.theta_vec = theta_vec;
            a.Opad = (O + 63) & ~63;
            a.frag_len = fused_frag_len(c, net);
            a.mat_len = nd.mat_len; a.vec_len = nd.vec_len;
            for (int l = 0; l < L; ++l) { a.mat_off[l] = nd.layer[l].mat_off; a.vec_off[l] = nd.layer[l].vec_off; }
            {  // the matrices the kernel streams, once more in the order of its requests
                FragOrderArgs fo;
                fo.src = theta_mat; fo.dst = reinterpret_cast<bf16_t*>(ws); fo.mat_len = nd.mat_len; fo.L = L;
                fo.frag_len = a.frag_len;
                int g = 0;
                for (int l = 0; l < L; ++l) {
                    fo.mat_off[l] = nd.layer[l].mat_off;
                    fo.frag_off[l] = a.frag_off[l] = nd.layer[l].mat_off + (l > 0 ? (int64_t)W * (a.Opad - O) : 0);
                    fo.K[l] = l == 0 ? a.Opad : W;
                    fo.Ksrc[l] = l == 0 ? O : W;
                    fo.g0[l] = g;
                    g += (W / 64) * 2 * (fo.K[l] >> 6);
                }
                fo.g0[L] = g;
                k_theta_fragment_order<<<dim3(g, P), 256, 0, s>>>(fo);
                a.theta_frag = fo.dst;
            }
            a.H = sv;
            a.G = sv ? reinterpret_cast<gfix16_t*>(sv + ae) : nullptr;
            a.lstride = 2 * ae;
            a.L = L; a.O = O; a.M = M;
            a.tiles_m = (M + FF_ROWS - 1) / FF_ROWS;
            a.n_tiles = a.tiles_m * P;
            const LayerDev& Lo = nd.layer[L];
            a.head_mat_off = Lo.mat_off; a.head_vec_off = Lo.vec_off; a.logsig_off = Lo.vec_off + Lo.d_out;
            a.out_dim = nd.out_dim;
            a.tanh_cols = (net == MORLAX_ACTOR && c->d.mean_tanh) ? c->d.act_dim : 0;
            a.adim = c->d.act_dim;
            a.sig_state = (net == MORLAX_ACTOR && c->d.sigma_state) ? 1 : 0;
            a.rm = rm; a.out = out; a.saved_out = saved_out; a.eps = eps; a.act = act; a.logp = logp;
            if (c->d.act == 0) {
                if (sv) launch_fused_fwd<0, true>(c, a, s); else launch_fused_fwd<0, false>(c, a, s);
            } else {
                if (sv) launch_fused_fwd<1, true>(c, a, s); else launch_fused_fwd<1, false>(c, a, s);
            }
            fused = true;
        }
    }
    for (int l = 0; l < L && !fused; ++l) {
        const bool save = sv != nullptr;
        if (c->d.act == 0) {
            if (save) layer(l, std::integral_constant<int, 0>{}, std::true_type{});
            else layer(l, std::integral_constant<int, 0>{}, std::false_type{});
        } else {
            if (save) layer(l, std::integral_constant<int, 1>{}, std::true_type{});
            else layer(l, std::integral_constant<int, 1>{}, std::false_type{});
        }
    }
    if (fused) return;  // the fused kernel applies the output layer as well
    const LayerDev& Lh = nd.layer[L];
    const int tanh_cols = (net == MORLAX_ACTOR && c->d.mean_tanh) ? c->d.act_dim : 0;
    const dim3 grid((M + 63) / 64, P);
    k_head_fwd<T><<<grid, 256, 0, s>>>(Hbuf(L - 1), theta_mat, theta_vec, nd.mat_len, nd.vec_len, Lh.mat_off,
                                       Lh.vec_off, W, nd.out_dim, M, rm, tanh_cols, out, saved_out, eps, act, logp,
                                       Lh.vec_off + Lh.d_out, c->d.act_dim,
                                       (net == MORLAX_ACTOR && c->d.sigma_state) ? 1 : 0);
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
    const int tanh_cols = (net == MORLAX_ACTOR && c->d.mean_tanh) ? c->d.act_dim : 0;
    constexpr int VE = Elems<T>::VE;
    const LayerDev& Lh = nd.layer[L];
    // output layer
    {
        const int n_chunk_b = (M + 255) / 256;
        float* pw = part;
        float* pb = part + head_pw_elems(c);
        float* dzh = part + head_lo_elems(c, rs);
        k_head_dzh<T><<<dim3(n_chunk_b, P), 256, 0, s>>>(dout, saved_out, dzh, pb, nd.out_dim, M, rm, tanh_cols);
        k_head_bwd_dw<T><<<dim3((W + 127) / 128, HB_SPLIT, P), 256, 0, s>>>(dzh, Hbuf(L - 1), pw, W, M);
        k_head_bwd_dw_final<<<dim3((nd.out_dim * W + 255) / 256, P), 256, 0, s>>>(
            pw, pb, HB_SPLIT, n_chunk_b, dtheta_mat, dtheta_vec, nd.mat_len, nd.vec_len, Lh.mat_off, Lh.vec_off, W,
            nd.out_dim);
        k_head_bwd_dz<T><<<dim3((W + 127) / 128, (M + 63) / 64, P), 256, 0, s>>>(
            dzh, theta_mat, nd.mat_len, Lh.mat_off, Gbuf(L - 1), dZbuf(L - 1), part, W, nd.out_dim, M);
    }
    for (int l = L - 1; l >= 0; --l) {
        const LayerDev& Ld = nd.layer[l];
        k_colsum_final<<<dim3((W + 31) / 32, P), 256, 0, s>>>(part, n_part, dtheta_vec, nd.vec_len, Ld.vec_off, W);
        EpiDw ew;
        ew.dW = dtheta_mat + Ld.mat_off;
        ew.ld = Ld.d_in;
        if (l > 0) {
            GemmArgs<T, SRC_KSTRIDED, SRC_KSTRIDED, EpiDw, true, GEMM_NCH> g;
            g.a.base = dZbuf(l); g.a.ld = W; g.a.rows = W; g.a.kdim = M; g.a.rm = rm;
            g.b.base = Hbuf(l - 1); g.b.ld = W; g.b.rows = W; g.b.kdim = M; g.b.rm = rm;
            g.a_pstride = (int64_t)M * W; g.b_pstride = (int64_t)M * W;
            g.epi = ew; g.e0_pstride = nd.mat_len; g.e1_pstride = 0; g.e2_pstride = 0;
            const int S = dw_split(c, rs);
            if (S > 1) {
                float* pws = part + head_lo_elems(c, rs) + align_up((int64_t)P * M * MORLAX_MAX_OUT, 64) +
                             first_skinny_elems(c, rs);
                const int64_t WW = (int64_t)W * W;
                g.a.kdim = g.b.kdim = M / S;
                g.a_pstride = g.b_pstride = (int64_t)(M / S) * W;
                g.epi.dW = pws; g.epi.ld = W; g.e0_pstride = WW;
                run_gemm(c, 3, g, P * S, s);
                k_dw_split_final<<<dim3((unsigned)((WW / 4 + 255) / 256), P), 256, 0, s>>>(pws, S, WW, dtheta_mat, nd.mat_len,
                                                                                        Ld.mat_off);
                prof_extend(c, s);
            } else {
                run_gemm(c, 3, g, P, s);
            }
            GemmArgs<T, SRC_KCONTIG, SRC_KSTRIDED, EpiDx<T>, true, GEMM_NCH> h;
            h.a.base = dZbuf(l); h.a.ld = W; h.a.rows = M; h.a.kdim = W; h.a.rm = rm;
            h.b.base = theta_mat + Ld.mat_off; h.b.ld = W; h.b.rows = W; h.b.kdim = W; h.b.rm = rm;
            h.a_pstride = (int64_t)M * W; h.b_pstride = nd.mat_len;
            h.epi.G = Gbuf(l - 1); h.epi.dZ = dZbuf(l - 1); h.epi.ld = W; h.epi.part = part;
            h.e0_pstride = (int64_t)M * W; h.e1_pstride = 0; h.e2_pstride = 0;
            run_gemm(c, 2, h, P, s);
            n_part = h.tiles_m;  // row tiles of the kernel that ran (128 or 256 rows)
        } else if (first_skinny(c)) {
            const int OP = O <= 16 ? 16 : 32, ns = first_split(c, rs);
            float* xz = part + head_lo_elems(c, rs) + align_up((int64_t)P * M * MORLAX_MAX_OUT, 64);
            float* pw1 = xz + align_up((int64_t)P * M * OP, 64);
            const int64_t n = (int64_t)M * OP;
            GemmProf::Rec* r = prof_take(c, 4, 2.0 * W * (double)O * M * P);
            if (r) (void)hipEventRecord(r->a, s);
            k_gather_x_pad<T><<<dim3((unsigned)((n + 255) / 256), P), 256, 0, s>>>(x, xz, O, OP, M, rm);
            const dim3 grid((W + 127) / 128, ns, P);
            if (OP == 16) k_first_bwd_dw<T, 1><<<grid, 256, 0, s>>>(xz, dZbuf(0), pw1, W, M, ns);
            else k_first_bwd_dw<T, 2><<<grid, 256, 0, s>>>(xz, dZbuf(0), pw1, W, M, ns);
            k_first_dw_final<<<dim3((W * O + 255) / 256, P), 256, 0, s>>>(pw1, ns, OP, dtheta_mat, nd.mat_len, Ld.mat_off, W, O);
            if (r) (void)hipEventRecord(r->b, s);
        } else if (use_x0(c)) {
            if constexpr (std::is_same<T, bf16_t>::value) {
                // the rows gathered by the forward pass
                const T* x0 = reinterpret_cast<const T*>(reinterpret_cast<const char*>(sv) + (int64_t)2 * L * ae * sizeof(T) +
                                                         align_up((int64_t)P * M * OUT_PITCH * 4, 256));
                GemmArgs<T, SRC_KSTRIDED, SRC_KSTRIDED, EpiDw, true, GEMM_NCH> g;
                g.a.base = dZbuf(0); g.a.ld = W; g.a.rows = W; g.a.kdim = M; g.a.rm = rm;
                g.b.base = x0; g.b.ld = O; g.b.rows = O; g.b.kdim = M; g.b.rm = rm;
                g.a_pstride = (int64_t)M * W; g.b_pstride = (int64_t)M * O;
                g.epi = ew; g.e0_pstride = nd.mat_len; g.e1_pstride = 0; g.e2_pstride = 0;
                run_gemm(c, 4, g, P, s);
            }
        } else {
            auto launch = [&](auto fast) {
                constexpr bool F = decltype(fast)::value;
                GemmArgs<T, SRC_KSTRIDED, SRC_X_KSTRIDED, EpiDw, F, GEMM_NCH> g;
                g.a.base = dZbuf(0); g.a.ld = W; g.a.rows = W; g.a.kdim = M; g.a.rm = rm;
                g.b.base = x; g.b.ld = O; g.b.rows = O; g.b.kdim = M; g.b.rm = rm;
                g.a_pstride = (int64_t)M * W; g.b_pstride = 0;
                g.epi = ew; g.e0_pstride = nd.mat_len; g.e1_pstride = 0; g.e2_pstride = 0;
                run_gemm(c, 4, g, P, s);
            };
            if (rs.j_cnt % VE == 0) launch(std::true_type{}); else launch(std::false_type{});
        }
    }
    (void)VE;
    if (net == MORLAX_ACTOR && !c->d.sigma_state) {  // (a state-dependent log sigma is part of dout)
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
