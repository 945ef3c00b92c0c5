// Assignment extraction: the stage order and the pipelines behind a candidate's cost (Sec. 2,
// "Pipeline parallel": P_i = { sigma_{i,j} }; Sec. 3.3: devices matched between adjacent stage
// groups handle the same micro-batch, the groups are ordered by the open-loop tour).
// Neither optimum is unique and the paper names no choice; the canonical choices are:
//   order     Held-Karp back-tracking: the path ends in the lowest-numbered node attaining the
//             minimum; the node before v in a path over S is the lowest-numbered u in S \ v with
//             fl(tab[S \ v][u] + Ghat[u][v]) == tab[S][v];
//   matching  for adjacent groups (A, B) with optimum T = Ghat[A][B]: the lexicographically smallest
//             vector (slot of B matched to slot 0 of A, to slot 1, ...) among the perfect matchings
//             within W_pp <= T;
//   pipeline  P_i starts at slot i of the first group of the order and follows the matchings.
//   k_hk_path        one workgroup per candidate: full Held-Karp table in a scratch slice, then the
//                    back-tracking by one thread
//   k_lexmin_match   one wavefront per (candidate, adjacent pair): bit-mask augmenting paths
//   k_chain          composes the matchings into pipelines
#include "dtfm_internal.h"

#include <math.h>

namespace {

constexpr int HKP_THREADS = 256;
// concurrently live Held-Karp tables: as many as fit 256 MiB of scratch (32 of 8 MiB at D_pp = 16),
// at most 2048
static size_t hkp_grid(int n, size_t rows)
{
    size_t g = ((size_t)256 << 20) / (((size_t)n << n) * sizeof(double));
    if (g > 2048) g = 2048;
    return rows < g ? rows : g;
}

__global__ void __launch_bounds__(HKP_THREADS)
k_hk_path(const double *__restrict__ ghat, int n, const uint32_t *__restrict__ subsets, dtfm_layer_off lo,
          double *__restrict__ tab_global, int32_t *__restrict__ order, size_t P)
{
    __shared__ double G[DTFM_MAX_DPP * DTFM_MAX_DPP];
    double *tab = tab_global + (size_t)blockIdx.x * ((size_t)n << n);
    const uint32_t full = (1u << n) - 1u;
    for (size_t p = blockIdx.x; p < P; p += gridDim.x) {
        for (int e = threadIdx.x; e < n * n; e += blockDim.x) G[e] = ghat[p * n * n + e];
        for (int v = threadIdx.x; v < n; v += blockDim.x) tab[((size_t)1 << v) * n + v] = 0.0;
        __syncthreads();
        for (int k = 2; k <= n; k++) {
            const int first = lo.off[k], items = (lo.off[k + 1] - first) * k;
            for (int it = threadIdx.x; it < items; it += blockDim.x) {
                const int si = it / k, tv = it - si * k;
                const uint32_t S = subsets[first + si];
                uint32_t m = S;
                for (int z = 0; z < tv; z++) m &= m - 1;
                const int v = __ffs((int)m) - 1;
                const uint32_t rest = S ^ (1u << v);
                const double *src = tab + (size_t)rest * n;
                double best = INFINITY;
                for (uint32_t r = rest; r; r &= r - 1) {
                    const int u = __ffs((int)r) - 1;
                    best = fmin(best, __dadd_rn(src[u], G[u * n + v]));
                }
                tab[(size_t)S * n + v] = best;
            }
            __syncthreads();   // the layer just written is read by the next one (same workgroup)
        }
        if (threadIdx.x == 0) {
            int32_t *ord = order + p * n;
            int v = 0;
            for (int x = 1; x < n; x++)
                if (tab[(size_t)full * n + x] < tab[(size_t)full * n + v]) v = x;
            uint32_t S = full;
            for (int pos = n - 1; pos >= 0; pos--) {
                ord[pos] = v;
                const uint32_t rest = S ^ (1u << v);
                if (rest == 0u) break;
                int pred = -1;
                for (int u = 0; u < n && pred < 0; u++)
                    if (((rest >> u) & 1u) && __dadd_rn(tab[(size_t)rest * n + u], G[u * n + v]) == tab[(size_t)S * n + v])
                        pred = u;
                if (pred < 0) pred = __ffs((int)rest) - 1;   // cannot happen for finite weights; keeps the walk inside S
                S = rest;
                v = pred;
            }
        }
        __syncthreads();
    }
}

// Alternating-path search on bit masks, one wavefront. Lane x plays row x and column x.
//   coladj  (lane c) rows allowed for column c          mcol (lane r) column matched to row r
//   mrow    (lane c) row matched to column c, -1: free
// Looks for an augmenting path from row `start` (treated as unmatched) to a column of `target`,
// entering only columns of `cols` and continuing only through rows of `rows`; on success flips the
// path (the start row and every row on it move one column along) and returns the column reached,
// else returns -1 and changes nothing. At most D columns are visited, one or more per pass.
__device__ __forceinline__ int augment(int lane, int D, uint64_t coladj, int &mcol, int &mrow, int start,
                                       uint64_t rows, uint64_t cols, uint64_t target)
{
    uint64_t frontier = 1ull << start, visited = 0ull;
    int parent = -1;
    int reached = -1;
    for (int pass = 0; pass <= D && reached < 0; pass++) {
        const uint64_t via = coladj & frontier;
        const bool newly = ((cols >> lane) & 1ull) != 0ull && ((visited >> lane) & 1ull) == 0ull && via != 0ull;
        const uint64_t reach = __ballot(newly);
        if (reach == 0ull) return -1;
        if (newly) parent = __builtin_ctzll(via);
        visited |= reach;
        const uint64_t hit = reach & target;
        if (hit != 0ull) {
            reached = __builtin_ctzll(hit);
            break;
        }
        // every column reached here is matched (the free ones are in `target`): their rows go on
        frontier = __ballot(lane != start && mcol >= 0 && ((rows >> lane) & 1ull) != 0ull && ((reach >> mcol) & 1ull) != 0ull);
        if (frontier == 0ull) return -1;
    }
    if (reached < 0) return -1;
    int c = reached;
    for (int step = 0; step <= D; step++) {
        const int r = __builtin_amdgcn_readlane(parent, c);
        const int prevc = __builtin_amdgcn_readlane(mcol, r);
        if (lane == r) mcol = c;
        if (lane == c) mrow = r;
        if (r == start) break;
        c = prevc;
    }
    return reached;
}

__global__ void __launch_bounds__(256)
k_lexmin_match(const double *__restrict__ W_pp, const int32_t *__restrict__ perm, const double *__restrict__ ghat,
               const int32_t *__restrict__ order, int N, int D, int n, size_t total, int32_t *__restrict__ mates)
{
    const int lane = threadIdx.x & (DTFM_WAVE - 1);
    const size_t item = (size_t)blockIdx.x * (blockDim.x / DTFM_WAVE) + threadIdx.x / DTFM_WAVE;
    if (item >= total) return;   // whole wavefront leaves together
    const size_t p = item / (size_t)(n - 1);
    const int k = (int)(item - p * (size_t)(n - 1));
    const int A = order[p * n + k], B = order[p * n + k + 1];
    const double T = ghat[p * n * n + A * n + B];
    const int32_t *row = perm + p * N;
    const bool active = lane < D;
    const uint64_t all = D >= 64 ? ~0ull : ((1ull << D) - 1ull);
    uint64_t coladj = 0ull;
    {
        const double *wcol = W_pp + (active ? row[B * D + lane] : 0);
        for (int i = 0; i < D; i++) {
            const double w = wcol[(size_t)row[A * D + i] * N];
            if (active && w <= T) coladj |= 1ull << i;
        }
    }
    int mcol = -1, mrow = -1;
    // any perfect matching within the threshold: one augmenting path per row
    uint64_t freecols = all;
    bool ok = true;
    for (int r = 0; r < D && ok; r++) {
        const int c = augment(lane, D, coladj, mcol, mrow, r, all, all, freecols);
        if (c < 0) ok = false;
        else freecols &= ~(1ull << c);
    }
    // row by row, move the row to the smallest column that still leaves the later rows a perfect matching
    uint64_t fixed = 0ull;
    for (int i = 0; i < D && ok; i++) {
        const int cur = __builtin_amdgcn_readlane(mcol, i);
        const uint64_t rowadj = __ballot(active && ((coladj >> i) & 1ull) != 0ull);
        uint64_t cand = rowadj & ~fixed & ((1ull << cur) - 1ull);
        const uint64_t later = i >= 63 ? 0ull : (all & ~((2ull << i) - 1ull));   // rows after i
        while (cand != 0ull) {
            const int c = __builtin_ctzll(cand);
            cand &= cand - 1ull;
            // forcing (i, c) frees column `cur` and unseats the row at c, which must reach `cur`
            const int other = __builtin_amdgcn_readlane(mrow, c);
            const int got = augment(lane, D, coladj, mcol, mrow, other, later, all & ~fixed & ~(1ull << c), 1ull << cur);
            if (got >= 0) {
                if (lane == i) mcol = c;
                if (lane == c) mrow = i;
                break;
            }
        }
        fixed |= 1ull << __builtin_amdgcn_readlane(mcol, i);
    }
    if (active) mates[item * D + lane] = ok ? mcol : -1;
}

// sigma[p][i][k]: pipeline i at position k. One thread per (candidate, pipeline).
__global__ void k_chain(const int32_t *__restrict__ perm, const int32_t *__restrict__ order,
                        const int32_t *__restrict__ mates, int N, int D, int n, size_t P, int32_t *__restrict__ sigma)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= P * (size_t)D) return;
    const size_t p = idx / D;
    const int i = (int)(idx - p * D);
    const int32_t *row = perm + p * N, *ord = order + p * n;
    int32_t *out = sigma + (p * D + i) * n;
    int slot = i;
    out[0] = row[ord[0] * D + slot];
    for (int k = 0; k + 1 < n; k++) {
        const int m = mates[(p * (size_t)(n - 1) + k) * D + slot];
        slot = m < 0 ? slot : m;   // m < 0 only for malformed input
        out[k + 1] = row[ord[k + 1] * D + slot];
    }
}

}  // namespace

dtfm_assign_bufs dtfm_assign_carve(const dtfm_problem *pr, dtfm_arena &ar, size_t rows)
{
    dtfm_assign_bufs b;
    const size_t n = pr->D_pp;
    b.ev = dtfm_eval_carve(pr, ar, rows);
    const size_t grid = hkp_grid(pr->D_pp, rows);
    b.tab = ar.take<double>(grid * (n << n));
    b.mates = ar.take<int32_t>(rows * (n > 1 ? n - 1 : 1) * (size_t)pr->D_dp);
    return b;
}

int dtfm_assign_enqueue(const dtfm_problem *pr, const dtfm_assign_bufs &b, const int32_t *perm, size_t rows,
                        int32_t *stage_order, int32_t *sigma, hipStream_t st)
{
    if (rows == 0) return DTFM_OK;
    const int n = pr->D_pp, D = pr->D_dp, N = pr->N;
    int rc = dtfm_eval_enqueue(pr, b.ev, perm, rows, nullptr, st);   // coarsened graphs only
    if (rc != DTFM_OK) return rc;
    const size_t grid = hkp_grid(n, rows);
    hipLaunchKernelGGL(k_hk_path, dim3((unsigned)grid), dim3(HKP_THREADS), 0, st, b.ev.ghat, n, pr->hk_subsets,
                       pr->hk_off, b.tab, stage_order, rows);
    DTFM_HIP(hipGetLastError());
    if (n > 1) {
        const size_t total = rows * (size_t)(n - 1);
        hipLaunchKernelGGL(k_lexmin_match, dim3((unsigned)((total + 3) / 4)), dim3(256), 0, st, pr->W_pp, perm,
                           b.ev.ghat, stage_order, N, D, n, total, b.mates);
        DTFM_HIP(hipGetLastError());
    }
    const size_t threads = rows * (size_t)D;
    hipLaunchKernelGGL(k_chain, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, perm, stage_order, b.mates,
                       N, D, n, rows, sigma);
    DTFM_HIP(hipGetLastError());
    return DTFM_OK;
}
