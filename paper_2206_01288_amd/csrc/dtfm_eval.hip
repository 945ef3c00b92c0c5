// General-shape kernels for the cost model (any N <= 1024, D_dp <= 64, D_pp <= 16):
//   k_weights     Sec. 2 symmetrisation + the per-link terms of Eqs. 2 and 3
//   k_datap       Eq. 2 per stage and the max over stages (Sec. 3.2)
//   k_match       Eq. 3: bottleneck perfect matching of one stage pair per wavefront
//   k_held_karp   Eq. 4: open-loop TSP over the coarsened graph, exact, by subset dynamic
//                 programming; adds the two parts (Eq. 1)
// All arithmetic is fp64 with one rounding per operation (compiled with -ffp-contract=off; the
// sums that define the result's bits use __dadd_rn explicitly).
#include "dtfm_internal.h"

#include <math.h>

// ------------------------------------------------------------------------------------------------
// a0: W_dp[d][d'] = 2 (alpha + shard / beta), W_pp[d][d'] = 2 (alpha + c_pp / beta) with
// alpha, beta the averages of the two directions (communication graph G of Sec. 2).
__global__ void k_weights(const double *__restrict__ lat, const double *__restrict__ bw, int N,
                          double shard, double c_pp, double *__restrict__ W_dp,
                          double *__restrict__ W_pp)
{
    int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= N * N) return;
    int d = idx / N, e = idx - d * N;
    if (d == e) {
        W_dp[idx] = 0.0;
        W_pp[idx] = 0.0;
        return;
    }
    double alpha = __dmul_rn(0.5, __dadd_rn(lat[idx], lat[e * N + d]));
    double beta = __dmul_rn(0.5, __dadd_rn(bw[idx], bw[e * N + d]));
    W_dp[idx] = __dmul_rn(2.0, __dadd_rn(alpha, __ddiv_rn(shard, beta)));
    W_pp[idx] = __dmul_rn(2.0, __dadd_rn(alpha, __ddiv_rn(c_pp, beta)));
}

int dtfm_weights_enqueue(const double *lat_dev, const double *bw_dev, int N, double shard,
                         double c_pp, double *W_dp, double *W_pp, hipStream_t st)
{
    int total = N * N;
    hipLaunchKernelGGL(k_weights, dim3((total + 255) / 256), dim3(256), 0, st, lat_dev, bw_dev, N,
                       shard, c_pp, W_dp, W_pp);
    DTFM_HIP(hipGetLastError());
    return DTFM_OK;
}

// ------------------------------------------------------------------------------------------------
// a2/a3: one workgroup per candidate, one thread per position q (device d = perm[q], stage
// j = q / D_dp, slot i = q % D_dp). The row sum runs over the stage's slots in order, skipping the
// device's own slot, starting from +0.0; max over the devices of all stages is exact in any order.
// Also zeroes the diagonal of the candidate's coarsened graph.
__global__ void k_datap(const double *__restrict__ W_dp, const int32_t *__restrict__ perm, int N,
                        int D_dp, int D_pp, double *__restrict__ datap, double *__restrict__ ghat)
{
    extern __shared__ int32_t s_perm[];
    __shared__ double s_red[16];
    size_t p = blockIdx.x;
    const int32_t *row = perm + p * N;
    for (int q = threadIdx.x; q < N; q += blockDim.x) s_perm[q] = row[q];
    if (ghat != nullptr)
        for (int j = threadIdx.x; j < D_pp; j += blockDim.x) ghat[(p * D_pp + j) * D_pp + j] = 0.0;
    __syncthreads();
    double worst = 0.0;  // all weights are >= 0, so every row sum is >= +0.0
    for (int q = threadIdx.x; q < N; q += blockDim.x) {
        int j = q / D_dp, i = q - j * D_dp;
        const double *wr = W_dp + (size_t)s_perm[q] * N;
        const int32_t *C = s_perm + j * D_dp;
        double sum = 0.0;
        for (int k = 0; k < D_dp; k++)
            if (k != i) sum = __dadd_rn(sum, wr[C[k]]);
        worst = fmax(worst, sum);
    }
    for (int o = 32; o >= 1; o >>= 1) worst = fmax(worst, __shfl_xor(worst, o));
    int wave = threadIdx.x / DTFM_WAVE, nw = (blockDim.x + DTFM_WAVE - 1) / DTFM_WAVE;
    if ((threadIdx.x & (DTFM_WAVE - 1)) == 0) s_red[wave] = worst;
    __syncthreads();
    if (threadIdx.x == 0) {
        double m = s_red[0];
        for (int w = 1; w < nw; w++) m = fmax(m, s_red[w]);
        datap[p] = m;
    }
}

// ------------------------------------------------------------------------------------------------
// a4: bottleneck assignment for one (candidate, stage pair) per wavefront, lane c = column c
// (device at slot c of the second stage). Rows (slots of the first stage) are inserted one at a
// time; for each, the alternating path to a free column that minimises its largest edge is found
// by a Dijkstra-style search in which `dist[c]` is the smallest achievable largest-edge of an
// alternating path from the new row to column c. The optimum of Eq. 3 is the largest of these
// path values over all insertions: a perfect matching within threshold T exists iff every
// insertion finds a path within T (Berge), and the matching kept so far never uses an edge above
// the running maximum. The value is one of the block's entries, so no rounding is involved.
__device__ __forceinline__ double wave_min_f64(double v)
{
    for (int o = 32; o >= 1; o >>= 1) v = fmin(v, __shfl_xor(v, o));
    return v;
}

__global__ void k_match(const double *__restrict__ W_pp, const int32_t *__restrict__ perm, int N,
                        int D_dp, int D_pp, int npairs, size_t total, double *__restrict__ ghat)
{
    const int lane = threadIdx.x & (DTFM_WAVE - 1);
    size_t item = (size_t)blockIdx.x * (blockDim.x / DTFM_WAVE) + threadIdx.x / DTFM_WAVE;
    if (item >= total) return;  // whole wavefront leaves together
    size_t p = item / npairs;
    int t = (int)(item - p * npairs);
    // t-th stage pair (j1 < j2) in lexicographic order
    int j1 = 0, rem = t;
    while (rem >= D_pp - 1 - j1) {
        rem -= D_pp - 1 - j1;
        j1++;
    }
    int j2 = j1 + 1 + rem;
    const int32_t *row = perm + p * N;
    const int32_t *Ca = row + j1 * D_dp;
    const bool active = lane < D_dp;
    const int coldev = active ? row[j2 * D_dp + lane] : 0;

    int match_row = -1;  // row currently matched to this lane's column
    double T = 0.0;      // weights are >= 0
    for (int r0 = 0; r0 < D_dp; r0++) {
        double dist = active ? W_pp[(size_t)Ca[r0] * N + coldev] : INFINITY;
        int prev = -1;       // previous column on the best path to this column, -1: straight from r0
        bool visited = !active;
        double dmin = INFINITY;
        int cmin = 0;
        // at most r0 matched columns are visited before a free one; the bound also ends the search
        // on malformed input (non-finite weights), leaving T = inf
        for (int step = 0; step <= r0; step++) {
            double key = visited ? INFINITY : dist;
            dmin = wave_min_f64(key);
            unsigned long long hit = __ballot(!visited && key == dmin);
            if (hit == 0ull) {
                dmin = INFINITY;
                break;
            }
            cmin = __ffsll((long long)hit) - 1;
            if (lane == cmin) visited = true;
            int mr = __shfl(match_row, cmin);
            if (mr < 0) break;  // free column reached
            double w = active ? W_pp[(size_t)Ca[mr] * N + coldev] : INFINITY;
            double nd = fmax(dmin, w);
            if (!visited && nd < dist) {
                dist = nd;
                prev = cmin;
            }
        }
        T = fmax(T, dmin);
        // flip the path: column c takes the row of its predecessor column; the first column takes r0
        int c = cmin;
        for (int step = 0; step <= r0; step++) {  // a path has at most r0 + 1 columns
            int pc = __shfl(prev, c);
            int prow = __shfl(match_row, pc < 0 ? 0 : pc);
            int newrow = (pc < 0) ? r0 : prow;
            if (lane == c) match_row = newrow;
            if (pc < 0) break;
            c = pc;
        }
    }
    if (lane == 0) {
        double *G = ghat + p * D_pp * D_pp;
        G[j1 * D_pp + j2] = T;
        G[j2 * D_pp + j1] = T;
    }
}

// ------------------------------------------------------------------------------------------------
// a5/a6: Held-Karp. tab[S*n + v] = cheapest path visiting exactly the stage set S and ending in v,
// each candidate value formed as fl(tab[S \ v][u] + Ghat[u][v]). Subsets are processed in layers
// of equal size (list `subsets` ordered by popcount), one (S, v) item per thread, with a workgroup
// barrier between layers. The table is in LDS when it fits, else in this workgroup's slice of an
// HBM scratch area. One workgroup walks over candidates p = blockIdx.x, += gridDim.x.
template <bool LDS_TABLE>
__global__ void k_held_karp(const double *__restrict__ ghat, const double *__restrict__ datap, int n,
                            const uint32_t *__restrict__ subsets, dtfm_layer_off lo,
                            double *__restrict__ tab_global, double *__restrict__ cost, size_t P)
{
    extern __shared__ double smem[];
    double *G = smem;
    double *tab = LDS_TABLE ? smem + n * n : tab_global + (size_t)blockIdx.x * ((size_t)n << n);
    const uint32_t full = (1u << n) - 1u;
    for (size_t p = blockIdx.x; p < P; p += gridDim.x) {
        for (int e = threadIdx.x; e < n * n; e += blockDim.x) G[e] = ghat[p * n * n + e];
        for (int v = threadIdx.x; v < n; v += blockDim.x) tab[((size_t)1 << v) * n + v] = 0.0;
        __syncthreads();
        for (int k = 2; k <= n; k++) {
            int first = lo.off[k], items = (lo.off[k + 1] - first) * k;
            for (int it = threadIdx.x; it < items; it += blockDim.x) {
                int si = it / k, tv = it - si * k;
                uint32_t S = subsets[first + si];
                uint32_t m = S;
                for (int z = 0; z < tv; z++) m &= m - 1;
                int v = __ffs((int)m) - 1;
                uint32_t rest = S ^ (1u << v);
                const double *src = tab + (size_t)rest * n;
                double best = INFINITY;
                for (uint32_t r = rest; r; r &= r - 1) {
                    int u = __ffs((int)r) - 1;
                    best = fmin(best, __dadd_rn(src[u], G[u * n + v]));
                }
                tab[(size_t)S * n + v] = best;
            }
            __syncthreads();
        }
        if (threadIdx.x == 0) {
            double m = INFINITY;
            for (int v = 0; v < n; v++) m = fmin(m, tab[(size_t)full * n + v]);
            cost[p] = __dadd_rn(datap[p], m);
        }
        __syncthreads();
    }
}

// a5/a6 for D_pp above the LDS limit: the table [S][16] lives in HBM and is walked source-side.
// tab[T][v] depends only on the row of S = T \ v: tab[T][v] = min_{u in S} fl(tab[S][u] + Ghat[u][v]).
// So a group of 16 lanes takes one source set S, reads its row (128 contiguous bytes; lane u holds
// tab[S][u], or +inf when u is not in S), rotates the row through the group with DPP so that every
// lane v meets every u, keeps min_u (tab[S][u] + Ghat[u][v]) and, for v not in S, stores it as
// tab[S + v][v]: every entry is written exactly once and every row is read exactly once, layer by
// layer (workgroup barrier between layers). Per candidate 8 MiB of rows are read and 4 MiB of
// entries written, instead of one 8-byte read per relaxation.
template <int R>
__device__ __forceinline__ int dpp_ror_i32(int x)
{
    return __builtin_amdgcn_update_dpp(0, x, 0x120 + R, 0xf, 0xf, false);   // row_ror:R within 16 lanes
}
template <int R>
__device__ __forceinline__ double dpp_ror_f64(double x)
{
    union {
        double d;
        int i[2];
    } a, b;
    a.d = x;
    b.i[0] = dpp_ror_i32<R>(a.i[0]);
    b.i[1] = dpp_ror_i32<R>(a.i[1]);
    return b.d;
}

template <int R>
struct hk_push_rot {
    // Gc[R-1] = Ghat[u][v] for the lane u that rotation R brings to lane v
    static __device__ __forceinline__ void setup(const double *G, int v, double *Gc)
    {
        const int u = dpp_ror_i32<R>(v);
        Gc[R - 1] = G[u * 16 + v];
        hk_push_rot<R - 1>::setup(G, v, Gc);
    }
    static __device__ __forceinline__ double relax(double x, const double *Gc, double y)
    {
        y = hk_push_rot<R - 1>::relax(x, Gc, y);
        return fmin(y, __dadd_rn(dpp_ror_f64<R>(x), Gc[R - 1]));
    }
};
template <>
struct hk_push_rot<0> {
    static __device__ __forceinline__ void setup(const double *, int, double *) {}
    static __device__ __forceinline__ double relax(double, const double *, double y) { return y; }
};

__global__ void __launch_bounds__(1024)
k_held_karp_push(const double *__restrict__ ghat, const double *__restrict__ datap, int n,
                 const uint32_t *__restrict__ subsets, dtfm_layer_off lo, double *__restrict__ tab_global,
                 double *__restrict__ cost, size_t P)
{
    __shared__ double G[16 * 16];
    double *tab = tab_global + (size_t)blockIdx.x * ((size_t)16 << n);
    const int v = threadIdx.x & 15, grp = threadIdx.x >> 4, ngrp = blockDim.x >> 4;
    const uint32_t full = (1u << n) - 1u;
    for (size_t p = blockIdx.x; p < P; p += gridDim.x) {
        for (int e = threadIdx.x; e < 256; e += blockDim.x) {
            const int a = e >> 4, b = e & 15;
            G[e] = (a < n && b < n) ? ghat[p * n * n + a * n + b] : INFINITY;
        }
        if ((int)threadIdx.x < n) tab[((size_t)1 << threadIdx.x) * 16 + threadIdx.x] = 0.0;
        __syncthreads();
        double Gc[15];
        hk_push_rot<15>::setup(G, v, Gc);
        for (int k = 1; k < n; k++) {
            const int first = lo.off[k], cnt = lo.off[k + 1] - first;
            for (int i = grp; i < cnt; i += ngrp) {
                const uint32_t S = subsets[first + i];
                const bool in = (S >> v) & 1u;
                const double x = in ? tab[(size_t)S * 16 + v] : INFINITY;
                const double y = hk_push_rot<15>::relax(x, Gc, INFINITY);
                if (!in && v < n) tab[(size_t)(S | (1u << v)) * 16 + v] = y;
            }
            __syncthreads();
        }
        if (threadIdx.x == 0) {
            double m = INFINITY;
            for (int u = 0; u < n; u++) m = fmin(m, tab[(size_t)full * 16 + u]);
            cost[p] = __dadd_rn(datap[p], m);
        }
        __syncthreads();
    }
}

dtfm_eval_bufs dtfm_eval_carve(const dtfm_problem *pr, dtfm_arena &ar, size_t rows)
{
    dtfm_eval_bufs b;
    size_t n = pr->D_pp;
    b.datap = ar.take<double>(rows);
    b.ghat = ar.take<double>(rows * n * n);
    b.hk_tab = nullptr;
    if (pr->D_pp > DTFM_HK_LDS_MAX_DPP) {
        size_t grid = rows < DTFM_HK_GLOBAL_GRID ? rows : DTFM_HK_GLOBAL_GRID;
        b.hk_tab = ar.take<double>(grid * ((size_t)16 << n));
    }
    return b;
}

int dtfm_eval_enqueue(const dtfm_problem *pr, const dtfm_eval_bufs &b, const int32_t *perm,
                      size_t rows, double *cost, hipStream_t st)
{
    if (rows == 0) return DTFM_OK;
    if (pr->fast64)
        return cost != nullptr ? dtfm_fast64_enqueue(pr, perm, rows, cost, nullptr, nullptr, st)
                               : dtfm_fast64_enqueue(pr, perm, rows, nullptr, b.ghat, b.datap, st);
    const int N = pr->N, n = pr->D_pp;
    int threads = ((N + DTFM_WAVE - 1) / DTFM_WAVE) * DTFM_WAVE;
    if (threads > 1024) threads = 1024;
    hipLaunchKernelGGL(k_datap, dim3((unsigned)rows), dim3(threads), N * sizeof(int32_t), st, pr->W_dp,
                       perm, N, pr->D_dp, n, b.datap, b.ghat);
    DTFM_HIP(hipGetLastError());
    if (pr->npairs > 0) {
        size_t total = rows * (size_t)pr->npairs;
        const int waves_per_block = 4;
        size_t blocks = (total + waves_per_block - 1) / waves_per_block;
        hipLaunchKernelGGL(k_match, dim3((unsigned)blocks), dim3(waves_per_block * DTFM_WAVE), 0, st,
                           pr->W_pp, perm, N, pr->D_dp, n, pr->npairs, total, b.ghat);
        DTFM_HIP(hipGetLastError());
    }
    if (cost == nullptr) return DTFM_OK;
    if (n <= DTFM_HK_LDS_MAX_DPP) {
        size_t lds = ((size_t)n * n + ((size_t)n << n)) * sizeof(double);
        int bt = n <= 6 ? 64 : 256;
        if (lds > 48 * 1024)  // above the default dynamic-LDS limit: raise it for this kernel
            DTFM_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_held_karp<true>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        hipLaunchKernelGGL(k_held_karp<true>, dim3((unsigned)rows), dim3(bt), lds, st, b.ghat, b.datap, n,
                           pr->hk_subsets, pr->hk_off, (double *)nullptr, cost, rows);
    } else {
        size_t grid = rows < DTFM_HK_GLOBAL_GRID ? rows : DTFM_HK_GLOBAL_GRID;
        hipLaunchKernelGGL(k_held_karp_push, dim3((unsigned)grid), dim3(1024), 0, st, b.ghat, b.datap, n,
                           pr->hk_subsets, pr->hk_off, b.hk_tab, cost, rows);
    }
    DTFM_HIP(hipGetLastError());
    return DTFM_OK;
}
