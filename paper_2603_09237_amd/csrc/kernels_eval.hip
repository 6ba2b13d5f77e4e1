// Evaluation side of MORLAX (Fig. 2a; Sec. II-A: returns and Pareto dominance; Sec. II-B: hypervolume):
// the return vector of every trade-off from a finished roll-out, the Pareto-optimal subset of a set of
// return vectors, and the hypervolume that set dominates above a reference point.  gfx950 only.
#include "morlax_internal.h"

// ------------------------------------------------------------------------------------------------
// Return vectors.  J[p, k] = mean over the n_g environments of group p of
//   sum_t gamma^t r[t, n, k] alive[t, n],  alive = 1 up to and including the first done of n.
// One workgroup per preference, JL x K threads: thread (j, k) walks environments j, j + JL, ... of the group
// through time for objective k (the threads of a step read consecutive floats), every step's loads independent
// of the episode ends (the cells of an ended episode are deselected), sums in fp64; the JL partial sums of an
// objective are added in a fixed tree.
__global__ __launch_bounds__(1024) void k_eval_returns(const float* __restrict__ r, const uint8_t* __restrict__ done,
                                                      double gamma, int T, int N, int K, int n_g, int JL,
                                                      float* __restrict__ J) {
    __shared__ double red[1024];
    const int p = blockIdx.x, tid = threadIdx.x, k = tid % K, j0 = tid / K;
    double acc = 0.0;
    for (int j = j0; j < n_g; j += JL) {
        const int n = p * n_g + j;
        double disc = 1.0;
        bool alive = true;
#pragma unroll 8
        for (int t = 0; t < T; ++t) {
            const double rv = (double)r[((int64_t)t * N + n) * K + k];
            const bool d = done[(int64_t)t * N + n] != 0;
            acc += alive ? disc * rv : 0.0;   // a select: values after the end of the episode never enter
            alive = alive && !d;
            disc *= gamma;
        }
    }
    red[tid] = acc;
    __syncthreads();
    for (int s = JL / 2; s > 0; s >>= 1) {   // lanes j0 and j0 + s of the same objective
        if (j0 < s) red[tid] += red[tid + s * K];
        __syncthreads();
    }
    if (j0 == 0) J[p * K + k] = (float)(red[tid] / (double)n_g);
}

void launch_eval_returns(const morlax_ctx* c, const float* r, const uint8_t* done, float gamma, float* J,
                         hipStream_t s) {
    int JL = 64;  // environment lanes: a power of two, JL * K threads
    while (2 * JL * c->d.K <= 1024 && JL < c->n_g) JL *= 2;
    k_eval_returns<<<c->d.P, JL * c->d.K, 0, s>>>(r, done, (double)gamma, c->d.T, c->d.N, c->d.K, c->n_g, JL, J);
}

// ------------------------------------------------------------------------------------------------
// Pareto front and hypervolume of n points in K objectives above a reference point.
//
// With V[i] = max(J[i] - ref, 0) the hypervolume is the measure of the union of the boxes [0, V[i]].  Cut
// objectives 2 .. K-1 at the coordinates of the points: between two neighbouring cuts of objective d (a slab
// of thickness delta_d[j], j counting the cuts from the top) the boxes that reach into the slab are those of
// the j + 1 points with the largest coordinate d.  For a tuple of slabs (j_2 .. j_{K-1}) the cross-section in
// objectives 0, 1 is the staircase of the points that are in every one of those prefixes, and
//   HV = sum over tuples of prod_d delta_d[j_d] * area(staircase of the tuple's points).
// Prefix sets are bit masks over the points in the order of decreasing objective 0, so a tuple's set is the
// AND of K - 2 masks and its staircase one pass over the set bits: a point adds x * (y - top) when its y is
// above the top so far.  All sums are fp64 in a fixed order (per thread by ascending tuple, then a fixed
// tree per workgroup, then a fixed tree over the workgroups): results are repeatable.
#define HV_MAX_N 1024
#define HV_MAX_K 8
#define HV_BLOCKS 1024
#define HV_THREADS 256

struct HvWs {
    double* xs;      // [n] objective 0 in decreasing order
    double* ys;      // [n] objective 1 of the same points
    double* delta;   // [K - 2][n]
    uint64_t* mask;  // [K - 2][n][W]
    double* part;    // [HV_BLOCKS]
    uint16_t* pr0;   // [n] position (in the order of objective 0) of the point of rank j in objective 2
};

static HvWs hv_layout(void* ws, int n, int K) {
    const int S = K > 2 ? K - 2 : 0, W = (n + 63) / 64;
    char* b = reinterpret_cast<char*>(ws);
    HvWs h;
    h.xs = reinterpret_cast<double*>(b); b += align_up((int64_t)n * 8, 256);
    h.ys = reinterpret_cast<double*>(b); b += align_up((int64_t)n * 8, 256);
    h.delta = reinterpret_cast<double*>(b); b += align_up((int64_t)S * n * 8 + 8, 256);
    h.mask = reinterpret_cast<uint64_t*>(b); b += align_up((int64_t)S * n * W * 8 + 8, 256);
    h.part = reinterpret_cast<double*>(b); b += align_up((int64_t)HV_BLOCKS * 8, 256);
    h.pr0 = reinterpret_cast<uint16_t*>(b);
    return h;
}

int64_t hv_ws_bytes(int n, int K) {
    const int S = K > 2 ? K - 2 : 0, W = (n + 63) / 64;
    return 2 * align_up((int64_t)n * 8, 256) + align_up((int64_t)S * n * 8 + 8, 256) +
           align_up((int64_t)S * n * W * 8 + 8, 256) + align_up((int64_t)HV_BLOCKS * 8, 256) +
           align_up((int64_t)n * 2, 256);
}

// One workgroup: shifted coordinates, dominance flags, the order by objective 0, and per cut objective the
// slab thicknesses and prefix masks.  lds: V [K][n] doubles, then rank-by-position [n] uint16.
__global__ __launch_bounds__(1024) void k_hv_prepare(const float* __restrict__ J, const float* __restrict__ ref, int n,
                                                    int K, uint8_t* __restrict__ front, HvWs h, double* __restrict__ hv) {
    extern __shared__ __align__(16) unsigned char hv_lds[];
    double* V = reinterpret_cast<double*>(hv_lds);
    uint16_t* posof = reinterpret_cast<uint16_t*>(V + (size_t)K * n);  // point -> position in the objective-0 order
    uint16_t* rpos = posof + n;                                        // position -> rank in the current cut objective
    double* cut = reinterpret_cast<double*>(rpos + n + ((4 - ((2 * n) & 3)) & 3));  // sorted coordinates of the current objective
    const int tid = threadIdx.x, W = (n + 63) / 64;
    for (int i = tid; i < n; i += blockDim.x)
        for (int k = 0; k < K; ++k) {
            const double v = (double)J[(int64_t)i * K + k] - (double)ref[k];
            V[(size_t)k * n + i] = v > 0.0 ? v : 0.0;
        }
    // Pareto dominance on the values as given (Sec. II-A): j dominates i when it is at least as good in every
    // objective and the two differ
    for (int i = tid; i < n; i += blockDim.x) {
        bool dominated = false;
        for (int j = 0; j < n && !dominated; ++j) {
            bool ge = true, gt = false;
            for (int k = 0; k < K; ++k) {
                const float a = J[(int64_t)j * K + k], b = J[(int64_t)i * K + k];
                ge = ge && (a >= b);
                gt = gt || (a > b);
            }
            dominated = ge && gt;
        }
        front[i] = dominated ? 0 : 1;
    }
    __syncthreads();
    // rank of point i in objective d: points with a larger coordinate, or an equal one and a smaller index
    auto rank_in = [&](int d, int i) {
        const double* c = V + (size_t)d * n;
        const double vi = c[i];
        int rk = 0;
        for (int j = 0; j < n; ++j) rk += (c[j] > vi) || (c[j] == vi && j < i);
        return rk;
    };
    for (int i = tid; i < n; i += blockDim.x) {
        const int pos = rank_in(0, i);
        posof[i] = (uint16_t)pos;
        h.xs[pos] = V[i];
        h.ys[pos] = K > 1 ? V[(size_t)n + i] : 1.0;
    }
    __syncthreads();
    if (K == 1 && tid == 0) {
        double m = 0.0;
        for (int i = 0; i < n; ++i) m = V[i] > m ? V[i] : m;
        hv[0] = m;
    }
    for (int d = 2; d < K; ++d) {
        for (int i = tid; i < n; i += blockDim.x) {
            const int rk = rank_in(d, i);
            rpos[posof[i]] = (uint16_t)rk;
            cut[rk] = V[(size_t)d * n + i];
            if (d == 2) h.pr0[rk] = posof[i];
        }
        __syncthreads();
        double* dl = h.delta + (size_t)(d - 2) * n;
        for (int j = tid; j < n; j += blockDim.x) dl[j] = cut[j] - (j + 1 < n ? cut[j + 1] : 0.0);
        uint64_t* mk = h.mask + (size_t)(d - 2) * n * W;
        for (int id = tid; id < n * W; id += blockDim.x) {
            const int j = id / W, wd = id % W;
            uint64_t m = 0;
            for (int b = 0; b < 64; ++b) {
                const int pos = 64 * wd + b;
                if (pos < n && rpos[pos] <= j) m |= (uint64_t)1 << b;
            }
            mk[id] = m;
        }
        __syncthreads();
    }
}

// Work item = the slabs of objectives 3 .. K-1 (the "outer" tuple: its weight and the AND of its masks are
// formed once) x a run of consecutive slabs of objective 2.  Going down the slabs of objective 2 the set gains
// the point of rank j at slab j: the staircase is recomputed only when that point belongs to the outer set,
// otherwise the slab repeats the area of the one above.
#define HV_MAX_W (HV_MAX_N / 64)
// WB: compile-time bound on the mask words, ceil(n / 64) <= WB.  The staircase coordinates, the thicknesses and
// ranks of objective 2 and (up to 256 points) its prefix masks sit in LDS: the passes over the set bits are
// chains of dependent reads.
template <int WB>
__global__ __launch_bounds__(HV_THREADS) void k_hv_slices(int n, int K, HvWs h, uint64_t items, int runs, int run_len) {
    constexpr bool MASK_LDS = WB <= 4;
    __shared__ double red[HV_THREADS];
    __shared__ double2 xy[64 * WB];
    __shared__ double d0[64 * WB];
    __shared__ uint16_t pr0[64 * WB];
    __shared__ uint64_t m0[MASK_LDS ? 64 * WB * WB : 1];
    const int S = K - 2 > 0 ? K - 2 : 0, W = (n + 63) / 64;
    for (int i = threadIdx.x; i < n; i += HV_THREADS) {
        xy[i] = make_double2(h.xs[i], h.ys[i]);
        if (S > 0) {
            d0[i] = h.delta[i];
            pr0[i] = h.pr0[i];
        }
    }
    if (MASK_LDS && S > 0)
        for (int i = threadIdx.x; i < n * W; i += HV_THREADS) m0[i] = h.mask[i];
    __syncthreads();
    const uint64_t* mask0 = MASK_LDS ? m0 : h.mask;
    const uint64_t stride = (uint64_t)gridDim.x * HV_THREADS;
    double sum = 0.0;
    for (uint64_t it = (uint64_t)blockIdx.x * HV_THREADS + threadIdx.x; it < items; it += stride) {
        uint32_t q = (uint32_t)it;
        const int run = (int)(q % (uint32_t)runs);
        q /= (uint32_t)runs;
        uint64_t mo[WB];
#pragma unroll
        for (int wd = 0; wd < WB; ++wd) {
            uint64_t m = 0;
            if (wd < W) {
                m = ~(uint64_t)0;
                if (64 * (wd + 1) > n) m = ((uint64_t)1 << (n - 64 * wd)) - 1;  // n - 64 wd is in [1, 63] here
            }
            mo[wd] = m;
        }
        double wout = 1.0;
        for (int s = 1; s < S; ++s) {
            const int j = (int)(q % (uint32_t)n);
            q /= (uint32_t)n;
            wout *= h.delta[(size_t)s * n + j];
            const uint64_t* mk = h.mask + ((size_t)s * n + j) * W;
#pragma unroll
            for (int wd = 0; wd < WB; ++wd)
                if (wd < W) mo[wd] &= mk[wd];
        }
        if (wout == 0.0) continue;
        // area of the staircase of the outer set's points inside prefix j of objective 2 (j < 0: the outer set)
        auto staircase = [&](int j) {
            const uint64_t* mk = mask0 + (size_t)(j < 0 ? 0 : j) * W;
            double area = 0.0, top = 0.0;
#pragma unroll
            for (int wd = 0; wd < WB; ++wd) {
                uint64_t m = mo[wd];
                if (j >= 0 && wd < W) m &= mk[wd];
                while (m) {
                    const int pos = 64 * wd + __builtin_ctzll(m);
                    m &= m - 1;
                    const double2 c = xy[pos];
                    if (c.y > top) {
                        area += c.x * (c.y - top);
                        top = c.y;
                    }
                }
            }
            return area;
        };
        if (S == 0) {
            sum += staircase(-1);
            continue;
        }
        const int j_lo = run * run_len, j_hi = j_lo + run_len < n ? j_lo + run_len : n;
        if (j_lo >= j_hi) continue;
        double cur = j_lo > 0 ? staircase(j_lo - 1) : 0.0, acc = 0.0;
        for (int j = j_lo; j < j_hi; ++j) {
            const int pos = (int)pr0[j];
            uint64_t word = 0;
#pragma unroll
            for (int wd = 0; wd < WB; ++wd)
                if (wd == (pos >> 6)) word = mo[wd];
            if ((word >> (pos & 63)) & 1) cur = staircase(j);
            acc += d0[j] * cur;
        }
        sum += wout * acc;
    }
    red[threadIdx.x] = sum;
    __syncthreads();
    for (int s = HV_THREADS / 2; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) h.part[blockIdx.x] = red[0];
}

// the workgroups' sums: thread t adds partials t, t + 64, ... in order, then a fixed tree over the 64 threads
__global__ __launch_bounds__(64) void k_hv_final(const double* __restrict__ part, int nb, double* __restrict__ hv) {
    __shared__ double red[64];
    double s = 0.0;
    for (int b = threadIdx.x; b < nb; b += 64) s += part[b];
    red[threadIdx.x] = s;
    __syncthreads();
    for (int w = 32; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) hv[0] = red[0];
}

uint64_t hv_tuples(int n, int K) {  // n^(K-2), saturating at 2^63
    uint64_t t = 1;
    for (int s = 0; s < K - 2; ++s) {
        if (t > (uint64_t(1) << 62) / (uint64_t)n) return uint64_t(1) << 63;
        t *= (uint64_t)n;
    }
    return t;
}

void launch_pareto_hypervolume(const float* J, const float* ref, int n, int K, uint8_t* front, double* hv, void* ws,
                               hipStream_t s) {
    const HvWs h = hv_layout(ws, n, K);
    const size_t lds = (size_t)K * n * 8 + (size_t)2 * n * 2 + 8 + (size_t)n * 8;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_hv_prepare),
                                  hipFuncAttributeMaxDynamicSharedMemorySize,
                                  HV_MAX_K * HV_MAX_N * 8 + 4 * HV_MAX_N + 8 + HV_MAX_N * 8);
        attr_set = true;
    }
    k_hv_prepare<<<1, 1024, lds, s>>>(J, ref, n, K, front, h, hv);
    if (K == 1) return;
    // enough work items for every lane of the chip: the outer tuples, split along objective 2 when they are few
    const uint64_t outer = K > 3 ? hv_tuples(n, K - 1) : 1;
    int runs = 1;
    if (K > 2 && outer < 262144) {
        const uint64_t want_runs = (262144 + outer - 1) / outer;
        const int max_runs = (n + 7) / 8;
        runs = want_runs < (uint64_t)max_runs ? (int)want_runs : max_runs;
    }
    const int run_len = (n + runs - 1) / runs;
    const uint64_t items = outer * (uint64_t)runs;  // below 2^32
    const uint64_t want = (items + HV_THREADS - 1) / HV_THREADS;
    const int nb = want < HV_BLOCKS ? (int)want : HV_BLOCKS;
    const int W = (n + 63) / 64;
    if (W <= 1) k_hv_slices<1><<<nb, HV_THREADS, 0, s>>>(n, K, h, items, runs, run_len);
    else if (W <= 2) k_hv_slices<2><<<nb, HV_THREADS, 0, s>>>(n, K, h, items, runs, run_len);
    else if (W <= 4) k_hv_slices<4><<<nb, HV_THREADS, 0, s>>>(n, K, h, items, runs, run_len);
    else k_hv_slices<HV_MAX_W><<<nb, HV_THREADS, 0, s>>>(n, K, h, items, runs, run_len);
    k_hv_final<<<1, 64, 0, s>>>(h.part, nb, hv);
}
