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

// Eq. 2 when W_dp does not fit the 4 MiB L2 of an XCD (N = 1024: 8 MiB), so that k_datap's gathers miss
// it eight times out of nine. Workgroups are handed to the 8 XCDs round robin, so workgroup b runs on XCD
// b mod 8; it takes, of its candidates, only the positions whose DEVICE d has d mod 8 = b mod 8: every
// XCD then gathers from one eighth of the rows of W_dp (1 MiB), which stays in its L2. A candidate holds
// every device once, so a slice is exactly the devices x, x + 8, ..: its positions are compacted into
// LDS and each thread sums one row (slot order, own slot skipped). The slices' maxima meet in datap[p]
// through an atomic max on the bit pattern (weights are >= +0.0, so the order of the bits is the order
// of the values); datap must be zero on entry. Only the mapping of work to XCDs is an assumption
// about the hardware; the result does not depend on it.
#define DTFM_XCDS 8
__global__ void k_datap_sliced(const double *__restrict__ W_dp, const int32_t *__restrict__ perm, int N,
                               int D_dp, int D_pp, size_t P, size_t stride, double *__restrict__ datap,
                               double *__restrict__ ghat)
{
    extern __shared__ int32_t s_all[];
    int32_t *s_perm = s_all, *s_list = s_all + N;   // the row; the positions of this slice
    __shared__ int s_count;
    __shared__ double s_red[16];
    const int x = blockIdx.x % DTFM_XCDS;
    for (size_t p = blockIdx.x / DTFM_XCDS; p < P; p += stride) {
        __syncthreads();
        if (threadIdx.x == 0) s_count = 0;
        const int32_t *row = perm + p * N;
        for (int q = threadIdx.x; q < N; q += blockDim.x) s_perm[q] = row[q];
        if (ghat != nullptr && x == 0)
            for (int j = threadIdx.x; j < D_pp; j += blockDim.x) ghat[(p * D_pp + j) * D_pp + j] = 0.0;
        __syncthreads();
        for (int q = threadIdx.x; q < N; q += blockDim.x)
            if ((s_perm[q] % DTFM_XCDS) == x) s_list[atomicAdd(&s_count, 1)] = q;
        __syncthreads();
        const int cnt = s_count;
        double worst = 0.0;   // all weights are >= 0, so every row sum is >= +0.0
        for (int t = threadIdx.x; t < cnt; t += blockDim.x) {
            const int q = s_list[t], j = q / D_dp, i = q - j * D_dp;
            const double *wr = W_dp + (size_t)s_perm[q] * N;
            const int32_t *C = s_perm + j * D_dp;
            double sum = 0.0;
            for (int k = 0; k < D_dp; k++)
                if (k != i) sum = __dadd_rn(sum, wr[C[k]]);
            worst = fmax(worst, sum);
        }
        for (int o = 32; o >= 1; o >>= 1) worst = fmax(worst, __shfl_xor(worst, o));
        const int wave = threadIdx.x / DTFM_WAVE, nw = (blockDim.x + DTFM_WAVE - 1) / DTFM_WAVE;
        if ((threadIdx.x & (DTFM_WAVE - 1)) == 0) s_red[wave] = worst;
        __syncthreads();
        if (threadIdx.x == 0) {
            double m = s_red[0];
            for (int w = 1; w < nw; w++) m = fmax(m, s_red[w]);
            atomicMax(reinterpret_cast<unsigned long long *>(datap + p), (unsigned long long)__double_as_longlong(m));
        }
    }
}

__global__ void k_zero_f64(double *__restrict__ dst, size_t n)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = 0.0;
}

// ------------------------------------------------------------------------------------------------
// a4: bottleneck assignment for one (candidate, stage pair) per wavefront, lane c = column c (device
// at slot c of the second stage). The optimum of Eq. 3 is one of the block's entries and depends
// only on their order, so the search runs on `Wr`, the dense ranks of W_pp (equal weights share a
// rank), and the result is mapped back through `rank_val`: no rounding is involved.
// Lane c keeps its column of the block, E[r] = Wr[C_j1[r]][C_j2[c]], in registers; every row index
// used below is wavefront-uniform, so E is read by register-relative moves and the search touches
// no memory. Rows are inserted one at a time. For row r0 the alternating-path search grows a set of
// reached rows; dist[c] is the smallest edge from a reached row to column c, and every unvisited
// column with dist <= theta is reachable within the threshold theta. theta starts at the optimum T
// of the rows inserted so far and is raised, only when the search is stuck, to the smallest dist of
// an unvisited column: a perfect matching of rows 0..r0 within theta exists iff an alternating path
// from r0 to a free column exists within theta (Berge), so the final theta is the new optimum.
typedef uint32_t dtfm_u32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t dtfm_u32x32 __attribute__((ext_vector_type(32)));

template <int NB>  // number of 16-row register blocks: D_dp <= 16 * NB
__global__ void __launch_bounds__(256)
k_match(const uint32_t *__restrict__ Wr, const double *__restrict__ rank_val,
        const int32_t *__restrict__ perm, int N, int D_dp, int D_pp, int npairs, size_t total,
        double *__restrict__ ghat, int inc_j, int inc_jp)
{
    const int lane = threadIdx.x & (DTFM_WAVE - 1);
    size_t item = (size_t)blockIdx.x * (blockDim.x / DTFM_WAVE) + threadIdx.x / DTFM_WAVE;
    if (item >= total) return;  // whole wavefront leaves together
    size_t p = item / npairs;
    int t = (int)(item - p * npairs);
    int j1, j2;
    if (inc_j < 0) {
        // t-th stage pair (j1 < j2) in lexicographic order
        int rem = t;
        j1 = 0;
        while (rem >= D_pp - 1 - j1) {
            rem -= D_pp - 1 - j1;
            j1++;
        }
        j2 = j1 + 1 + rem;
    } else {
        // only the npairs = 2 D_pp - 3 pairs that contain stage inc_j or inc_jp (inc_j < inc_jp): (inc_j, k) for
        // the D_pp - 1 stages k != inc_j, then (inc_jp, k) for the D_pp - 2 others
        int a, k;
        if (t < D_pp - 1) {
            a = inc_j;
            k = t + (t >= inc_j ? 1 : 0);
        } else {
            a = inc_jp;
            k = t - (D_pp - 1);
            k += k >= inc_j ? 1 : 0;
            k += k >= inc_jp ? 1 : 0;
        }
        j1 = a < k ? a : k;
        j2 = a < k ? k : a;
    }
    const int32_t *row = perm + p * N;
    const int32_t *Ca = row + j1 * D_dp;
    const bool active = lane < D_dp;
    const uint32_t *col = Wr + (active ? row[j2 * D_dp + lane] : 0);

    // The block's column for this lane in registers: 16 entries (NB = 1), 32 (NB = 2) or two vectors of 32.
    dtfm_u32x16 E0;
    dtfm_u32x32 F0, F1;
#pragma unroll
    for (int r = 0; r < 16; r++) {
        if (NB == 1) E0[r] = r < D_dp ? col[(size_t)Ca[r] * N] : 0xffffffffu;
    }
#pragma unroll
    for (int r = 0; r < 32; r++) {
        if (NB > 1) F0[r] = r < D_dp ? col[(size_t)Ca[r] * N] : 0xffffffffu;
        if (NB > 2) F1[r] = r + 32 < D_dp ? col[(size_t)Ca[r + 32] * N] : 0xffffffffu;
    }
    // E[r] for a wavefront-uniform r. The empty asm statements keep the two register-relative
    // reads apart (merged into one 64-entry access they would go through scratch memory).
    auto entry = [&](int r) -> uint32_t {
        if (NB == 1) return E0[r & 15];
        const int lo = r & 31, hi = r >> 5;
        uint32_t w = F0[lo];
        if (NB > 2) {
            asm volatile("" : "+v"(w));
            uint32_t x = F1[lo];
            asm volatile("" : "+v"(x));
            w = hi == 1 ? x : w;
        }
        return w;
    };

    const uint64_t allcols = D_dp >= 64 ? ~0ull : ((1ull << D_dp) - 1ull);
    uint64_t freecols = allcols;  // columns not matched yet
    int match_row = 0;            // row matched to this lane's column (meaningful when not free)
    uint32_t T = 0;
    for (int r0 = 0; r0 < D_dp; r0++) {
        uint32_t dist = entry(r0);
        int prev = -1;  // column whose matched row gave `dist`; -1: the inserted row itself
        uint64_t visited = 0;
        uint32_t theta = T;
        int cfin = -1;
        // every pass visits at least one new column, ends the search, or follows a raise of theta
        // that makes the next pass do so: at most 2 (r0 + 1) passes
        for (int pass = 0; pass < 2 * 16 * NB + 2; pass++) {
            uint64_t reach = __ballot(dist <= theta) & ~visited & allcols;
            if (reach == 0ull) {
                // smallest dist of an unvisited column: prefix minima inside each row of 16 lanes by data-parallel
                // shifts (a lane without a source keeps its own value), then the four row results
                uint32_t k = (((visited >> lane) & 1ull) != 0ull || !active) ? 0xffffffffu : dist;
                k = min(k, (uint32_t)__builtin_amdgcn_update_dpp((int)k, (int)k, 0x111, 0xF, 0xF, false));   // row_shr:1
                k = min(k, (uint32_t)__builtin_amdgcn_update_dpp((int)k, (int)k, 0x112, 0xF, 0xF, false));   // row_shr:2
                k = min(k, (uint32_t)__builtin_amdgcn_update_dpp((int)k, (int)k, 0x114, 0xF, 0xF, false));   // row_shr:4
                k = min(k, (uint32_t)__builtin_amdgcn_update_dpp((int)k, (int)k, 0x118, 0xF, 0xF, false));   // row_shr:8
                const uint32_t m0 = (uint32_t)__builtin_amdgcn_readlane((int)k, 15), m1 = (uint32_t)__builtin_amdgcn_readlane((int)k, 31);
                const uint32_t m2 = (uint32_t)__builtin_amdgcn_readlane((int)k, 47), m3 = (uint32_t)__builtin_amdgcn_readlane((int)k, 63);
                theta = min(min(m0, m1), min(m2, m3));
                continue;
            }
            uint64_t hit = reach & freecols;
            if (hit != 0ull) {
                cfin = __builtin_ctzll(hit);
                break;
            }
            visited |= reach;
            const bool open = ((visited >> lane) & 1ull) == 0ull;  // a visited column keeps its path
            while (reach != 0ull) {  // the rows matched to the newly reached columns join the search
                const int c = __builtin_ctzll(reach);
                reach &= reach - 1ull;
                const int mr = __builtin_amdgcn_readlane(match_row, c);
                const uint32_t w = entry(mr);
                if (open && w < dist) {
                    dist = w;
                    prev = c;
                }
            }
        }
        if (cfin < 0) {  // cannot happen for a finite block; leaves +inf rather than a wrong value
            T = 0xffffffffu;
            break;
        }
        T = theta;
        // flip the path: column c takes the row of its predecessor column; the first column takes r0
        int c = cfin;
        for (int step = 0; step <= r0; step++) {  // a path has at most r0 + 1 columns
            const int pc = __builtin_amdgcn_readlane(prev, c);
            const int prow = __builtin_amdgcn_readlane(match_row, pc < 0 ? 0 : pc);
            if (lane == c) match_row = pc < 0 ? r0 : prow;
            if (pc < 0) break;
            c = pc;
        }
        freecols &= ~(1ull << cfin);
    }
    if (lane == 0) {
        const double v = T == 0xffffffffu ? INFINITY : rank_val[T];
        double *G = ghat + p * D_pp * D_pp;
        G[j1 * D_pp + j2] = v;
        G[j2 * D_pp + j1] = v;
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
                            double *__restrict__ tab_global, double *__restrict__ cost, size_t P,
                            const int32_t *__restrict__ list, const int32_t *__restrict__ count,
                            double *__restrict__ pp_out)
{
    extern __shared__ double smem[];
    double *G = smem;
    double *tab = LDS_TABLE ? smem + n * n : tab_global + (size_t)blockIdx.x * ((size_t)n << n);
    const uint32_t full = (1u << n) - 1u;
    // with a list: only the rows list[0 .. *count)
    const size_t todo = list != nullptr ? (size_t)*count : P;
    for (size_t idx = blockIdx.x; idx < todo; idx += gridDim.x) {
        const size_t p = list != nullptr ? (size_t)list[idx] : idx;
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
            if (pp_out != nullptr) pp_out[p] = m;
        }
        __syncthreads();
    }
}

// a5/a6 for D_pp above the LDS limit: the table is walked source-side, in blocks that live in LDS.
// tab[T][v] depends only on the row of S = T \ v: tab[T][v] = min_{u in S} fl(tab[S][u] + Ghat[u][v]).
// Rows have 16 slots; the slot of a stage that is not in the set holds +inf. A group of 16 lanes
// takes one source set S; all its lanes read the whole row (128-bit LDS reads of one address per
// group, served as broadcasts), lane v keeps min_u (tab[S][u] + Ghat[u][v]) with its column of
// Ghat in registers and, for v not in S, stores it as tab[S + v][v]: every entry is written
// exactly once and every row is read exactly once.
// A set S is split into its high part H (stages >= NL) and its low part L (stages < NL). All 2^NL
// rows that share H form a block [L][16] in LDS; the blocks are processed in increasing H (every
// subset of H before H), and inside a block the rows go in layers of |L| with a workgroup barrier
// between layers. A push to a low stage v stays in the block. A push to a high stage v belongs to
// the later block H + v: it goes to the workgroup's exchange area X[H + v][v][L] in HBM and is
// loaded, contiguously, when that block starts. Only these n - NL of every 16 entries cross HBM.
// C(b, i) for b <= 10
__device__ const unsigned char dtfm_binom10[11][11] = {
    {1, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0},   {1, 1, 0, 0, 0, 0, 0, 0, 0, 0, 0},    {1, 2, 1, 0, 0, 0, 0, 0, 0, 0, 0},
    {1, 3, 3, 1, 0, 0, 0, 0, 0, 0, 0},   {1, 4, 6, 4, 1, 0, 0, 0, 0, 0, 0},    {1, 5, 10, 10, 5, 1, 0, 0, 0, 0, 0},
    {1, 6, 15, 20, 15, 6, 1, 0, 0, 0, 0}, {1, 7, 21, 35, 35, 21, 7, 1, 0, 0, 0}, {1, 8, 28, 56, 70, 56, 28, 8, 1, 0, 0},
    {1, 9, 36, 84, 126, 126, 84, 36, 9, 1, 0}, {1, 10, 45, 120, 210, 252, 210, 120, 45, 10, 1}};

constexpr int dtfm_binom(int n, int k)
{
    int r = 1;
    for (int i = 1; i <= k; i++) r = r * (n - k + i) / i;
    return r;
}
// first position of the sets with k elements in the (popcount, value) order of the subsets of NL stages
constexpr int dtfm_layer_first(int NL, int k)
{
    int f = 0;
    for (int j = 0; j < k; j++) f += dtfm_binom(NL, j);
    return f;
}

// The layers of one block of the blocked Held-Karp kernel (see k_held_karp_blocked); HM, a compile-time
// constant, says which pairs of high-stage slots hold a stage of the block's set H. The loop over the layers is
// unrolled: their sizes are compile-time constants, and the low part L of a group's next row (a table look-up
// in LDS) is fetched one row ahead, across the barrier too. The barrier after the last layer also completes
// the block's stores to the exchange area.
template <int NL, int NPAIR, uint32_t HM>
__device__ __forceinline__ void hk_block_layers(double *tab, const uint16_t *lsub, const double (&Gc)[16],
                                                double *X, uint32_t H, int nh, int n, int v, int grp)
{
    static_assert(NL % 2 == 0 && 16 - NL <= 6, "slot pairs (NL + 2 q, NL + 2 q + 1), q < 3");
    constexpr int GROUPS = (1 << NL) / 16, RS = DTFM_HK_ROW_STRIDE;
    uint32_t Lnext = 0;   // layer 0 is the empty low part alone (group 0)
#pragma unroll
    for (int k = 0; k <= NL; k++) {
        const int first = dtfm_layer_first(NL, k), cnt = dtfm_binom(NL, k);
        for (int i = grp; i < cnt; i += GROUPS) {
            const uint32_t L = Lnext;
            if (i + GROUPS < cnt) Lnext = lsub[first + i + GROUPS];
            const uint32_t S = (H << NL) | L;
            const bool in = (S >> v) & 1u;
            const double2 *row = reinterpret_cast<const double2 *>(tab + L * RS);
            double y = INFINITY;
#pragma unroll
            for (int h = 0; h < NPAIR; h++) {
                // HM: bit q set = the pair of slots NL + 2 q, NL + 2 q + 1 holds a stage of H
                const bool present = 2 * h >= NL ? ((HM >> ((2 * h - NL) / 2)) & 1u) != 0u : true;
                if (!present) continue;
                const double2 x = row[h];
                y = fmin(y, __dadd_rn(x.x, Gc[2 * h]));
                y = fmin(y, __dadd_rn(x.y, Gc[2 * h + 1]));
            }
            if (!in && v < n && S != 0u) {
                if (v < NL)
                    tab[(L | (1u << v)) * RS + v] = y;
                else
                    X[(((size_t)(H | (1u << (v - NL))) * nh + (v - NL)) << NL) + L] = y;
            }
        }
        if (k < NL) {
            if (grp < dtfm_binom(NL, k + 1)) Lnext = lsub[dtfm_layer_first(NL, k + 1) + grp];
            DTFM_LDS_BARRIER();
        } else {
            __syncthreads();
        }
    }
}

// NL: low stages per block (the workgroup has 2^NL threads); NPAIR: pairs of row slots that can hold a stage
// (ceil(D_pp / 2): the slots beyond D_pp are +inf in every row and are not read)
template <int NL, int NPAIR>
__global__ void __launch_bounds__(1 << NL)
k_held_karp_blocked(const double *__restrict__ ghat, const double *__restrict__ datap, int n,
                    double *__restrict__ xchg, double *__restrict__ cost, size_t P,
                    const int32_t *__restrict__ list, const int32_t *__restrict__ count, double *__restrict__ pp_out)
{
    // rows are RS = 18 doubles apart (144 B = 36 banks): the same slot of 16 consecutive rows falls
    // into 16 different bank pairs, and the 128-bit row reads stay aligned
    constexpr int ROWS = 1 << NL, THREADS = 1 << NL, RS = DTFM_HK_ROW_STRIDE;
    extern __shared__ double smem[];
    double *tab = smem;                                           // [ROWS][RS], 16 slots used
    double *G = smem + ROWS * RS;                                 // [16][16], +inf outside n x n
    uint16_t *lsub = reinterpret_cast<uint16_t *>(G + 256);       // low parts ordered by popcount
    __shared__ unsigned char horder[1 << (16 - NL)];              // the sets H ordered by popcount
    constexpr int NHMAX = 16 - NL;
    const int nh = n - NL;
    double *X = xchg + (size_t)blockIdx.x * (((size_t)nh << nh) << NL);   // [H][high stage][L]
    const int v = threadIdx.x & 15, grp = threadIdx.x >> 4;
    const int Lt = threadIdx.x;   // the row this thread prepares at the start of a block

    {   // position of L = threadIdx.x in the (popcount, value) order: combinatorial number system
        const int L = threadIdx.x, k = __popc(L);
        int rank = 0, i = 0;
        for (int m = L; m; m &= m - 1) {
            i++;
            rank += dtfm_binom10[__ffs(m) - 1][i];
        }
        int first = 0;
        for (int j = 0; j < k; j++) first += dtfm_binom10[NL][j];
        lsub[first + rank] = (uint16_t)L;
        if (L < (1 << nh)) {   // the same order for the sets H of the nh high stages
            int hfirst = 0;
            for (int j = 0; j < k; j++) hfirst += dtfm_binom10[nh][j];
            horder[hfirst + rank] = (unsigned char)L;
        }
    }
    const int nblocks = 1 << nh;
    const size_t todo = list != nullptr ? (size_t)*count : P;   // with a list: only the rows list[0 .. *count)
    for (size_t idx = blockIdx.x; idx < todo; idx += gridDim.x) {
        const size_t p = list != nullptr ? (size_t)list[idx] : idx;
        __syncthreads();   // the tables above; the previous candidate's result has been read
        for (int e = threadIdx.x; e < 256; e += THREADS) {
            const int a = e >> 4, b = e & 15;
            G[e] = (a < n && b < n) ? ghat[p * n * n + a * n + b] : INFINITY;
        }
        __syncthreads();
        double Gc[16];   // column v of Ghat
#pragma unroll
        for (int u = 0; u < 16; u++) Gc[u] = G[u * 16 + v];
        // entries of block Hq that end in a high stage: pushed by the blocks Hq - h (a single high
        // stage alone is a path of one node); +inf for the high stages outside Hq
        auto fetch = [&](uint32_t Hq, double (&xv)[NHMAX]) {
#pragma unroll
            for (int hi = 0; hi < NHMAX; hi++) {
                double val = INFINITY;
                if (hi < nh && ((Hq >> hi) & 1u))
                    val = (Hq == (1u << hi) && Lt == 0) ? 0.0 : X[(((size_t)Hq * nh + hi) << NL) + Lt];
                xv[hi] = val;
            }
        };
        // The blocks go by popcount of H (every subset of H before H). Two consecutive blocks of the same
        // popcount do not depend on each other, so the exchanged entries of the next block are loaded while this
        // one is computed; the first block of a popcount loads its own after the barrier that ends the one before.
        double xv[NHMAX];
#pragma unroll
        for (int hi = 0; hi < NHMAX; hi++) xv[hi] = INFINITY;   // block H = 0
        bool have = true;
        for (int bi = 0; bi < nblocks; bi++) {
            const uint32_t H = horder[bi];
            // this thread's row of the new block: the previous block is done (barrier after its last layer). Low slots
            // +inf (block 0: a single low stage alone is a path of one node), high slots as exchanged.
            if (!have) fetch(H, xv);
            {
                double2 *mine = reinterpret_cast<double2 *>(tab + Lt * RS);
                const bool single = H == 0u && __popc(Lt) == 1;
                const int one = __ffs(Lt) - 1;
#pragma unroll
                for (int h = 0; h < NL / 2; h++)
                    mine[h] = make_double2(single && one == 2 * h ? 0.0 : INFINITY, single && one == 2 * h + 1 ? 0.0 : INFINITY);
#pragma unroll
                for (int h = NL / 2; h < 8; h++)
                    mine[h] = make_double2(xv[2 * h - NL], 2 * h - NL + 1 < NHMAX ? xv[2 * h - NL + 1] : INFINITY);
            }
            have = false;
            if (bi + 1 < nblocks) {
                const uint32_t Hn = horder[bi + 1];
                if (__popc(Hn) == __popc(H)) {
                    fetch(Hn, xv);
                    have = true;
                }
            }
            DTFM_LDS_BARRIER();
            // The slots of high stages outside H are +inf in every row of the block. One copy of the layer
            // loops per set of empty slot pairs (NL, NL+1), (NL+2, NL+3), (NL+4, NL+5): a copy neither reads nor
            // relaxes its empty pairs. (A copy per set H, 64 of them, outgrows the instruction cache.)
#define DTFM_HK_CASE(m) \
    case m: hk_block_layers<NL, NPAIR, m>(tab, lsub, Gc, X, H, nh, n, v, grp); break;
            switch (((H & 3u) != 0u ? 1u : 0u) | ((H & 12u) != 0u ? 2u : 0u) | ((H & 48u) != 0u ? 4u : 0u)) {
                DTFM_HK_CASE(0) DTFM_HK_CASE(1) DTFM_HK_CASE(2) DTFM_HK_CASE(3)
                DTFM_HK_CASE(4) DTFM_HK_CASE(5) DTFM_HK_CASE(6) DTFM_HK_CASE(7)
            default: break;
            }
#undef DTFM_HK_CASE
        }
        if (threadIdx.x == 0) {   // the block of H = all high stages came last and is still in LDS; its last row is the full set
            double m = INFINITY;
            for (int u = 0; u < n; u++) m = fmin(m, tab[(ROWS - 1) * RS + u]);
            cost[p] = __dadd_rn(datap[p], m);
            if (pp_out != nullptr) pp_out[p] = m;
        }
    }
}

// Trial evaluations of the local search (Sec. 3.4): settles, without Held-Karp, the trials whose coarsened graph
// says enough. Eq. 4 depends on the graph only, so a trial whose graph equals its current row's has the same
// PipelineP-Cost: cost = fl(DataP' + pp_cur), the bits Held-Karp would give. Every path sum is monotone in every
// edge (fl(x + w) is), hence so is Eq. 4: a trial whose graph is nowhere below the current one has
// PipelineP >= pp_cur, and if fl(DataP' + pp_cur) already reaches the current cost the trial cannot be strictly
// cheaper: it is rejected, which is all the search needs of it (its cost is set to +inf). The other trials go on the
// list for Held-Karp. One wavefront per trial; *count must be zero on entry.
__global__ void k_trial_shortcut(const double *__restrict__ ghat, const double *__restrict__ datap, int nn,
                                 const double *__restrict__ ghat_cur, const double *__restrict__ pp_cur,
                                 const double *__restrict__ cur, double *__restrict__ cost, double *__restrict__ pp_out,
                                 int32_t *__restrict__ list, int32_t *__restrict__ count, size_t rows, int trials_per_row)
{
    const size_t p = (size_t)blockIdx.x * (blockDim.x / DTFM_WAVE) + threadIdx.x / DTFM_WAVE;
    if (p >= rows) return;   // whole wavefront
    const size_t c = p / (size_t)trials_per_row;   // the current row this trial was made from
    const int lane = threadIdx.x & (DTFM_WAVE - 1);
    bool differs = false, below = false;
    for (int e = lane; e < nn; e += DTFM_WAVE) {
        const double a = ghat[p * nn + e], b = ghat_cur[c * nn + e];
        differs |= a != b;
        below |= a < b;
    }
    const bool any_differs = __ballot(differs) != 0ull, any_below = __ballot(below) != 0ull;
    if (lane != 0) return;
    const double with_cur = __dadd_rn(datap[p], pp_cur[c]);
    if (!any_differs) {
        cost[p] = with_cur;
        pp_out[p] = pp_cur[c];
    } else if (!any_below && with_cur >= cur[c]) {
        cost[p] = INFINITY;
    } else {
        list[atomicAdd(count, 1)] = (int32_t)p;
    }
}

__global__ void k_zero_count(int32_t *count) { *count = 0; }

size_t dtfm_hk_exchange_bytes(const dtfm_problem *pr)
{
    if (pr->D_pp <= DTFM_HK_LDS_MAX_DPP) return 0;
    size_t nh = (size_t)pr->D_pp - DTFM_HK_BLOCK_LOW;
    return ((nh << nh) << DTFM_HK_BLOCK_LOW) * sizeof(double);
}

dtfm_eval_bufs dtfm_eval_carve(const dtfm_problem *pr, dtfm_arena &ar, size_t rows, size_t hk_grid_cap)
{
    dtfm_eval_bufs b;
    size_t n = pr->D_pp;
    b.datap = ar.take<double>(rows);
    b.ghat = ar.take<double>(rows * n * n);
    b.hk_tab = nullptr;
    b.hk_grid = 0;
    if (pr->D_pp > DTFM_HK_LDS_MAX_DPP) {
        size_t cap = hk_grid_cap != 0 && hk_grid_cap < DTFM_HK_GLOBAL_GRID ? hk_grid_cap : DTFM_HK_GLOBAL_GRID;
        b.hk_grid = rows < cap ? rows : cap;
        b.hk_tab = ar.take<double>(b.hk_grid * (dtfm_hk_exchange_bytes(pr) / sizeof(double)));
    }
    b.pp = ar.take<double>(rows);
    b.list = ar.take<int32_t>(rows);
    b.count = ar.take<int32_t>(1);
    return b;
}

int dtfm_eval_enqueue(const dtfm_problem *pr, const dtfm_eval_bufs &b, const int32_t *perm,
                      size_t rows, double *cost, hipStream_t st)
{
    return dtfm_eval_inc_enqueue(pr, b, perm, rows, cost, -1, -1, st);
}

// As dtfm_eval_enqueue; with inc_j >= 0 (inc_j < inc_jp) b.ghat already holds the coarsened graphs of rows
// that differ from `perm` only in stages inc_j and inc_jp: only the edges of those two stages are matched again.
int dtfm_eval_inc_enqueue(const dtfm_problem *pr, const dtfm_eval_bufs &b, const int32_t *perm, size_t rows,
                          double *cost, int inc_j, int inc_jp, hipStream_t st, const dtfm_trial_ref *ref)
{
    if (rows == 0) return DTFM_OK;
    if (pr->fast64)
        return cost != nullptr ? dtfm_fast64_enqueue(pr, perm, rows, cost, nullptr, nullptr, st)
                               : dtfm_fast64_enqueue(pr, perm, rows, nullptr, b.ghat, b.datap, st);
    const int N = pr->N, n = pr->D_pp;
    int threads = ((N + DTFM_WAVE - 1) / DTFM_WAVE) * DTFM_WAVE;
    if (threads > 1024) threads = 1024;
    if ((size_t)N * N * sizeof(double) > ((size_t)2 << 20) && N % DTFM_XCDS == 0) {
        // W_dp larger than half an XCD's L2: one slice of its rows per XCD
        hipLaunchKernelGGL(k_zero_f64, dim3((unsigned)((rows + 255) / 256)), dim3(256), 0, st, b.datap, rows);
        DTFM_HIP(hipGetLastError());
        size_t per_slice = rows < 512 ? rows : 512;   // workgroups per slice; each strides over the candidates
        int slice_threads = ((N / DTFM_XCDS + DTFM_WAVE - 1) / DTFM_WAVE) * DTFM_WAVE;
        hipLaunchKernelGGL(k_datap_sliced, dim3((unsigned)(per_slice * DTFM_XCDS)), dim3(slice_threads),
                           2 * N * sizeof(int32_t), st, pr->W_dp, perm, N, pr->D_dp, n, rows, per_slice, b.datap, b.ghat);
    } else {
        hipLaunchKernelGGL(k_datap, dim3((unsigned)rows), dim3(threads), N * sizeof(int32_t), st, pr->W_dp,
                           perm, N, pr->D_dp, n, b.datap, b.ghat);
    }
    DTFM_HIP(hipGetLastError());
    if (pr->npairs > 0) {
        const int match_pairs = inc_j >= 0 ? 2 * n - 3 : pr->npairs;
        size_t total = rows * (size_t)match_pairs;
        const int waves_per_block = 4;
        size_t blocks = (total + waves_per_block - 1) / waves_per_block;
        auto kern = pr->D_dp <= 16 ? k_match<1> : pr->D_dp <= 32 ? k_match<2> : pr->D_dp <= 48 ? k_match<3> : k_match<4>;
        hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(waves_per_block * DTFM_WAVE), 0, st,
                           pr->W_rank, pr->rank_val, perm, N, pr->D_dp, n, match_pairs, total, b.ghat, inc_j, inc_jp);
        DTFM_HIP(hipGetLastError());
    }
    if (cost == nullptr) return DTFM_OK;
    const int32_t *list = nullptr, *count = nullptr;
    if (ref != nullptr) {   // trials of the local search: Held-Karp only where the coarsened graph does not settle the trial
        hipLaunchKernelGGL(k_zero_count, dim3(1), dim3(1), 0, st, b.count);
        DTFM_HIP(hipGetLastError());
        hipLaunchKernelGGL(k_trial_shortcut, dim3((unsigned)((rows + 3) / 4)), dim3(4 * DTFM_WAVE), 0, st, b.ghat, b.datap,
                           n * n, ref->ghat_cur, ref->pp_cur, ref->cur, cost, b.pp, b.list, b.count, rows, ref->trials_per_row);
        DTFM_HIP(hipGetLastError());
        list = b.list;
        count = b.count;
    }
    if (n <= DTFM_HK_LDS_MAX_DPP) {
        size_t lds = ((size_t)n * n + ((size_t)n << n)) * sizeof(double);
        int bt = n <= 6 ? 64 : 256;
        if (lds > 48 * 1024)  // above the default dynamic-LDS limit: raise it for this kernel
            DTFM_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_held_karp<true>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        hipLaunchKernelGGL(k_held_karp<true>, dim3((unsigned)rows), dim3(bt), lds, st, b.ghat, b.datap, n,
                           pr->hk_subsets, pr->hk_off, (double *)nullptr, cost, rows, list, count, b.pp);
    } else {
        size_t grid = b.hk_grid;
        constexpr int NL = DTFM_HK_BLOCK_LOW;
        size_t lds = ((size_t)(DTFM_HK_ROW_STRIDE << NL) + 256) * sizeof(double) + ((size_t)sizeof(uint16_t) << NL);
        auto kern = n <= 12 ? k_held_karp_blocked<NL, 6> : n <= 14 ? k_held_karp_blocked<NL, 7> : k_held_karp_blocked<NL, 8>;
        DTFM_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                     (int)lds));
        hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(1 << NL), lds, st, b.ghat, b.datap, n, b.hk_tab, cost, rows, list,
                           count, b.pp);
    }
    DTFM_HIP(hipGetLastError());
    return DTFM_OK;
}
