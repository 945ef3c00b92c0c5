// Search kernels (Sec. 3.4): swap-move local search (exhaustive and the paper's four-candidate
// neighbourhood) and the generation-wise genetic loop (selection, crossover, mutation,
// replacement), general shapes. Every cost they compare is the full cost of Eq. 1 as produced by
// the evaluation kernels, so a move's cost is bit-identical to evaluating the swapped allocation.
#include "dtfm_internal.h"
#include "dtfm_philox.h"

#include <math.h>

// Rows evaluated per call while enumerating the exhaustive neighbourhood.
#define DTFM_LS_ROWS_MAX ((size_t)1 << 18)

// ------------------------------------------------------------------------------------------------
// index <-> pair (a < b) among n items in lexicographic order (0,1),(0,2),...,(0,n-1),(1,2),...
__device__ __forceinline__ long long pair_base(int n, int a)
{
    return (long long)a * n - (long long)a * (a + 1) / 2;
}

__device__ __forceinline__ void pair_decode(int n, long long m, int &a, int &b)
{
    double disc = (2.0 * n - 1.0) * (2.0 * n - 1.0) - 8.0 * (double)m;
    int g = (int)(((2.0 * n - 1.0) - sqrt(disc > 0.0 ? disc : 0.0)) * 0.5);
    if (g < 0) g = 0;
    if (g > n - 2) g = n - 2;
    while (g > 0 && pair_base(n, g) > m) g--;
    while (g < n - 2 && pair_base(n, g + 1) <= m) g++;
    a = g;
    b = g + 1 + (int)(m - pair_base(n, g));
}

__device__ __forceinline__ long long pair_encode(int n, int a, int b)
{
    return pair_base(n, a) + (b - a - 1);
}

// ------------------------------------------------------------------------------------------------
// ALL_PAIRS: materialise, for candidates p0 .. p0+cp-1, every allocation one swap away
// (row (p - p0) * M + m = candidate p with the positions of move m exchanged).
__global__ void k_make_swapped(const int32_t *__restrict__ perm, int N, long long M, size_t p0,
                               int32_t *__restrict__ tmp_perm)
{
    size_t rowi = blockIdx.x;
    size_t pc = rowi / (size_t)M;
    long long m = (long long)(rowi - pc * (size_t)M);
    int a, b;
    pair_decode(N, m, a, b);
    const int32_t *src = perm + (p0 + pc) * N;
    int32_t *dst = tmp_perm + rowi * N;
    for (int q = threadIdx.x; q < N; q += blockDim.x) {
        int s = q == a ? b : (q == b ? a : q);
        dst[q] = src[s];
    }
}

// ALL_PAIRS by stage pair (general shapes): the swaps between a slot of stage j and a slot of stage jp (j < jp:
// D_dp^2 of them; j = jp: the D_dp (D_dp - 1) / 2 swaps inside the stage), in the order of their move index.
// Trial g of group (j, jp) exchanges positions a < b:
__device__ __forceinline__ void group_move(int D_dp, int j, int jp, long long g, int &a, int &b)
{
    if (j == jp) {
        int i, k;
        pair_decode(D_dp, g, i, k);
        a = j * D_dp + i;
        b = j * D_dp + k;
    } else {
        a = j * D_dp + (int)(g / D_dp);
        b = jp * D_dp + (int)(g % D_dp);
    }
}

// row (p - p0) * G + g = candidate p with trial g of the group applied
__global__ void k_make_swapped_group(const int32_t *__restrict__ perm, int N, int D_dp, int j, int jp, long long G,
                                     size_t p0, int32_t *__restrict__ tmp_perm)
{
    const size_t rowi = blockIdx.x;
    const size_t pc = rowi / (size_t)G;
    int a, b;
    group_move(D_dp, j, jp, (long long)(rowi - pc * (size_t)G), a, b);
    const int32_t *src = perm + (p0 + pc) * N;
    int32_t *dst = tmp_perm + rowi * N;
    for (int q = threadIdx.x; q < N; q += blockDim.x) {
        const int s = q == a ? b : (q == b ? a : q);
        dst[q] = src[s];
    }
}

// the group's costs to their places among all N (N - 1) / 2 moves of their candidate
__global__ void k_scatter_group(const double *__restrict__ group_cost, size_t T, int N, int D_dp, int j, int jp,
                                long long G, long long M, double *__restrict__ all_cost)
{
    const size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= T) return;
    const size_t pc = t / (size_t)G;
    int a, b;
    group_move(D_dp, j, jp, (long long)(t - pc * (size_t)G), a, b);
    all_cost[pc * (size_t)M + (size_t)pair_encode(N, a, b)] = group_cost[t];
}

// ALL_PAIRS: per candidate, the cheapest move (lowest index on ties); applied only if strictly
// cheaper than the current cost.
__global__ void k_pick_apply(int32_t *__restrict__ perm, int N, long long M, size_t p0,
                             const double *__restrict__ tmp_cost, double *__restrict__ cur,
                             int64_t *__restrict__ applied, int moves, int r)
{
    __shared__ double s_c[256];
    __shared__ long long s_i[256];
    size_t pc = blockIdx.x, p = p0 + pc;
    const double *c = tmp_cost + pc * (size_t)M;
    double best = INFINITY;
    long long bi = -1;
    for (long long m = threadIdx.x; m < M; m += blockDim.x) {
        double v = c[m];
        if (v < best) {  // ascending m within a thread: first minimiser kept
            best = v;
            bi = m;
        }
    }
    s_c[threadIdx.x] = best;
    s_i[threadIdx.x] = bi;
    __syncthreads();
    for (int o = blockDim.x / 2; o >= 1; o >>= 1) {
        if ((int)threadIdx.x < o) {
            double oc = s_c[threadIdx.x + o];
            long long oi = s_i[threadIdx.x + o];
            bool take = oi >= 0 && (s_i[threadIdx.x] < 0 || oc < s_c[threadIdx.x] ||
                                    (oc == s_c[threadIdx.x] && oi < s_i[threadIdx.x]));
            if (take) {
                s_c[threadIdx.x] = oc;
                s_i[threadIdx.x] = oi;
            }
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        long long mv = -1;
        if (s_i[0] >= 0 && s_c[0] < cur[p]) {
            int a, b;
            pair_decode(N, s_i[0], a, b);
            int32_t *row = perm + p * N;
            int32_t t = row[a];
            row[a] = row[b];
            row[b] = t;
            cur[p] = s_c[0];
            mv = s_i[0];
        }
        if (applied != nullptr) applied[p * (size_t)moves + r] = mv;
    }
}

// ------------------------------------------------------------------------------------------------
// GAIN4 proposal for round r, one wavefront per candidate. Stage pair (j, j') = pair number
// r mod D_pp(D_pp-1)/2; fastest link inside each stage = lexicographically first minimiser of W_pp
// over slot pairs; the four end-point swaps ranked by the paper's Gain (sums over the pre-swap
// sets in slot order from +0.0, divided by D_dp, four terms combined left to right), first
// maximiser wins. Writes the swapped allocation and the two positions.
__global__ void k_gain4_propose(const double *__restrict__ W_pp, const int32_t *__restrict__ perm,
                                int N, int D_dp, int D_pp, int r, int32_t *__restrict__ tmp_perm,
                                int32_t *__restrict__ move_ab)
{
    const int lane = threadIdx.x;
    size_t p = blockIdx.x;
    int npairs = D_pp * (D_pp - 1) / 2;
    int j, jp;
    pair_decode(D_pp, r % npairs, j, jp);
    const int32_t *row = perm + p * N;
    const int32_t *Cs[2] = {row + j * D_dp, row + jp * D_dp};
    int slot[2][2];
    double link[2];
    long long E = (long long)D_dp * (D_dp - 1) / 2;
    for (int s = 0; s < 2; s++) {
        const int32_t *C = Cs[s];
        double best = INFINITY;
        long long be = E;
        for (long long e = lane; e < E; e += DTFM_WAVE) {
            int i, k;
            pair_decode(D_dp, e, i, k);
            double w = W_pp[(size_t)C[i] * N + C[k]];
            if (w < best) {
                best = w;
                be = e;
            }
        }
        for (int o = 32; o >= 1; o >>= 1) {
            double ow = __shfl_xor(best, o);
            long long oe = __shfl_xor(be, o);
            if (ow < best || (ow == best && oe < be)) {
                best = ow;
                be = oe;
            }
        }
        if (be >= E) be = 0;  // only on malformed (non-finite) weights
        pair_decode(D_dp, be, slot[s][0], slot[s][1]);
        link[s] = best;
    }
    // lanes 0,1: mean over C_j' of w[x][.] for x = d1, d2; lanes 2,3: mean over C_j of w[y][.]
    double mean = 0.0;
    if (lane < 4) {
        int s = lane >> 1;                      // which stage the moving device is in
        int dev = Cs[s][slot[s][lane & 1]];
        const int32_t *other = Cs[1 - s];
        double sum = 0.0;
        for (int i = 0; i < D_dp; i++) sum = __dadd_rn(sum, W_pp[(size_t)dev * N + other[i]]);
        mean = __ddiv_rn(sum, (double)D_dp);
    }
    double mx[2] = {__shfl(mean, 0), __shfl(mean, 1)};
    double my[2] = {__shfl(mean, 2), __shfl(mean, 3)};
    double bestg = 0.0;
    int bk = -1;
    for (int k = 0; k < 4; k++) {
        double g = mx[k >> 1];
        g = __dadd_rn(g, -link[0]);   // w[x][mate(x)]: the fast link inside C_j
        g = __dadd_rn(g, my[k & 1]);
        g = __dadd_rn(g, -link[1]);   // w[y][mate(y)]: the fast link inside C_j'
        if (bk < 0 || g > bestg) {
            bestg = g;
            bk = k;
        }
    }
    int a = j * D_dp + slot[0][bk >> 1], b = jp * D_dp + slot[1][bk & 1];
    int32_t *dst = tmp_perm + p * N;
    for (int q = lane; q < N; q += DTFM_WAVE) {
        int s = q == a ? b : (q == b ? a : q);
        dst[q] = row[s];
    }
    if (lane == 0) {
        move_ab[2 * p] = a;
        move_ab[2 * p + 1] = b;
    }
}

// BEST4 (the four candidates of the paper's neighbourhood judged by the cost): one wavefront per candidate writes
// the four swapped allocations of round r, rows 4 p .. 4 p + 3 of tmp_perm in the order (d1,d1'), (d1,d2'), (d2,d1'),
// (d2,d2'), and their positions. The fastest link of a stage as in k_gain4_propose.
__global__ void k_best4_propose(const double *__restrict__ W_pp, const int32_t *__restrict__ perm,
                                int N, int D_dp, int D_pp, int r, int32_t *__restrict__ tmp_perm,
                                int32_t *__restrict__ move_ab)
{
    const int lane = threadIdx.x;
    size_t p = blockIdx.x;
    int npairs = D_pp * (D_pp - 1) / 2;
    int j, jp;
    pair_decode(D_pp, r % npairs, j, jp);
    const int32_t *row = perm + p * N;
    const int32_t *Cs[2] = {row + j * D_dp, row + jp * D_dp};
    int slot[2][2];
    long long E = (long long)D_dp * (D_dp - 1) / 2;
    for (int s = 0; s < 2; s++) {
        const int32_t *C = Cs[s];
        double best = INFINITY;
        long long be = E;
        for (long long e = lane; e < E; e += DTFM_WAVE) {
            int i, k;
            pair_decode(D_dp, e, i, k);
            double w = W_pp[(size_t)C[i] * N + C[k]];
            if (w < best) {
                best = w;
                be = e;
            }
        }
        for (int o = 32; o >= 1; o >>= 1) {
            double ow = __shfl_xor(best, o);
            long long oe = __shfl_xor(be, o);
            if (ow < best || (ow == best && oe < be)) {
                best = ow;
                be = oe;
            }
        }
        if (be >= E) be = 0;  // only on malformed (non-finite) weights
        pair_decode(D_dp, be, slot[s][0], slot[s][1]);
    }
    for (int k = 0; k < 4; k++) {
        const int a = j * D_dp + slot[0][k >> 1], b = jp * D_dp + slot[1][k & 1];
        int32_t *dst = tmp_perm + (4 * p + k) * N;
        for (int q = lane; q < N; q += DTFM_WAVE) {
            int s = q == a ? b : (q == b ? a : q);
            dst[q] = row[s];
        }
        if (lane == 0) {
            move_ab[2 * (4 * p + k)] = a;
            move_ab[2 * (4 * p + k) + 1] = b;
        }
    }
}

// BEST4: the cheapest of the candidate's four trials (the first on ties) is applied iff strictly cheaper than the
// current row; its coarsened graph and PipelineP-Cost then become the current ones (ghat_cur may be null).
__global__ void k_best4_pick(int32_t *__restrict__ perm, int N, const double *__restrict__ tmp_cost,
                             double *__restrict__ cur, const int32_t *__restrict__ move_ab, int64_t *__restrict__ applied,
                             int moves, int r, int nn, const double *__restrict__ ghat_trial, double *__restrict__ ghat_cur,
                             const double *__restrict__ pp_trial, double *__restrict__ pp_cur)
{
    const size_t p = blockIdx.x;
    int bk = 0;
    double bc = tmp_cost[4 * p];
    for (int k = 1; k < 4; k++) {
        const double c = tmp_cost[4 * p + k];
        if (c < bc) {
            bc = c;
            bk = k;
        }
    }
    const bool take = bc < cur[p];   // uniform over the workgroup
    if (take && ghat_cur != nullptr)
        for (int e = threadIdx.x; e < nn; e += blockDim.x) ghat_cur[p * nn + e] = ghat_trial[(4 * p + bk) * nn + e];
    if (threadIdx.x != 0) return;
    long long mv = -1;
    if (take) {
        const int a = move_ab[2 * (4 * p + bk)], b = move_ab[2 * (4 * p + bk) + 1];
        int32_t *row = perm + p * N;
        const int32_t t = row[a];
        row[a] = row[b];
        row[b] = t;
        cur[p] = bc;
        if (pp_cur != nullptr) pp_cur[p] = pp_trial[4 * p + bk];
        mv = pair_encode(N, a, b);
    }
    if (applied != nullptr) applied[p * (size_t)moves + r] = mv;
}

// dst[(reps c + k) * nn + e] = src[c * nn + e]: the current rows' coarsened graphs under each of their trial rows
__global__ void k_replicate_f64(const double *__restrict__ src, double *__restrict__ dst, int nn, int reps, size_t total)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const size_t row = i / nn, e = i - row * nn;
    dst[i] = src[(row / reps) * nn + e];
}

// KL neighbourhood (Sec. 3.4 "Existing Local Search Strategy", the strategy the paper compares with):
// one wavefront per candidate; round r looks at the same stage pair as the four-candidate
// neighbourhood and proposes, among all D_dp^2 swaps between the two stages, the one of largest
//   gain_KL = sum_{C_j'} w[x][.] - sum_{C_j - x} w[x][.] + sum_{C_j} w[y][.] - sum_{C_j' - y} w[y][.] - 2 w[x][y]
// (w = W_pp; each sum in slot order from +0.0, the five terms combined left to right; the first
// maximiser in (slot of C_j, slot of C_j') order wins). Writes the swapped allocation and the positions.
__global__ void k_kl_propose(const double *__restrict__ W_pp, const int32_t *__restrict__ perm, int N,
                             int D_dp, int D_pp, int r, int32_t *__restrict__ tmp_perm,
                             int32_t *__restrict__ move_ab)
{
    __shared__ double S[4][DTFM_MAX_DDP];   // the four sums per slot: [0],[1] for x = C_j[slot]; [2],[3] for y = C_j'[slot]
    const int lane = threadIdx.x;
    size_t p = blockIdx.x;
    int npairs = D_pp * (D_pp - 1) / 2;
    int j, jp;
    pair_decode(D_pp, r % npairs, j, jp);
    const int32_t *row = perm + p * N;
    const int32_t *Cj = row + j * D_dp, *Cjp = row + jp * D_dp;
    if (lane < D_dp) {
        const double *wx = W_pp + (size_t)Cj[lane] * N, *wy = W_pp + (size_t)Cjp[lane] * N;
        double s1 = 0.0, s2 = 0.0, s3 = 0.0, s4 = 0.0;
        for (int i = 0; i < D_dp; i++) s1 = __dadd_rn(s1, wx[Cjp[i]]);
        for (int i = 0; i < D_dp; i++)
            if (i != lane) s2 = __dadd_rn(s2, wx[Cj[i]]);
        for (int i = 0; i < D_dp; i++) s3 = __dadd_rn(s3, wy[Cj[i]]);
        for (int i = 0; i < D_dp; i++)
            if (i != lane) s4 = __dadd_rn(s4, wy[Cjp[i]]);
        S[0][lane] = s1;
        S[1][lane] = s2;
        S[2][lane] = s3;
        S[3][lane] = s4;
    }
    __syncthreads();
    double bestg = 0.0;
    int be = -1;
    for (int e = lane; e < D_dp * D_dp; e += DTFM_WAVE) {   // e = sx * D_dp + sy, increasing per lane
        const int sx = e / D_dp, sy = e - sx * D_dp;
        double g = __dadd_rn(S[0][sx], -S[1][sx]);
        g = __dadd_rn(g, S[2][sy]);
        g = __dadd_rn(g, -S[3][sy]);
        g = __dadd_rn(g, -__dmul_rn(2.0, W_pp[(size_t)Cj[sx] * N + Cjp[sy]]));
        if (be < 0 || g > bestg) {
            bestg = g;
            be = e;
        }
    }
    for (int o = 32; o >= 1; o >>= 1) {
        const double og = __shfl_xor(bestg, o);
        const int oe = __shfl_xor(be, o);
        if (oe >= 0 && (be < 0 || og > bestg || (og == bestg && oe < be))) {
            bestg = og;
            be = oe;
        }
    }
    if (be < 0) be = 0;   // only on malformed (NaN) weights
    const int a = j * D_dp + be / D_dp, b = jp * D_dp + be % D_dp;
    int32_t *dst = tmp_perm + p * N;
    for (int q = lane; q < N; q += DTFM_WAVE) {
        int s = q == a ? b : (q == b ? a : q);
        dst[q] = row[s];
    }
    if (lane == 0) {
        move_ab[2 * p] = a;
        move_ab[2 * p + 1] = b;
    }
}

// GAIN4 and KL: accept the proposed swap iff its cost is strictly lower.
// GAIN4 / KL rounds: the coarsened graph of an accepted trial row becomes the candidate's current one
// (runs before k_accept, on the same condition)
__global__ void k_keep_ghat(const double *__restrict__ tmp_cost, const double *__restrict__ cur, int nn,
                            const double *__restrict__ ghat_trial, double *__restrict__ ghat_cur,
                            const double *__restrict__ pp_trial, double *__restrict__ pp_cur)
{
    const size_t p = blockIdx.x;
    if (!(tmp_cost[p] < cur[p])) return;
    for (int e = threadIdx.x; e < nn; e += blockDim.x) ghat_cur[p * nn + e] = ghat_trial[p * nn + e];
    if (threadIdx.x == 0) pp_cur[p] = pp_trial[p];
}

__global__ void k_accept(int32_t *__restrict__ perm, int N, const double *__restrict__ tmp_cost,
                         double *__restrict__ cur, const int32_t *__restrict__ move_ab,
                         int64_t *__restrict__ applied, int moves, int r, size_t P)
{
    size_t p = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= P) return;
    long long mv = -1;
    if (tmp_cost[p] < cur[p]) {
        int a = move_ab[2 * p], b = move_ab[2 * p + 1];
        int32_t *row = perm + p * N;
        int32_t t = row[a];
        row[a] = row[b];
        row[b] = t;
        cur[p] = tmp_cost[p];
        mv = pair_encode(N, a, b);
    }
    if (applied != nullptr) applied[p * (size_t)moves + r] = mv;
}

__global__ void k_copy_f64(const double *__restrict__ src, double *__restrict__ dst, size_t n)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = src[i];
}

__global__ void k_copy_i32(const int32_t *__restrict__ src, int32_t *__restrict__ dst, size_t n)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = src[i];
}

__global__ void k_fill_i64(int64_t *__restrict__ dst, int64_t v, size_t n)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = v;
}

// ALL_PAIRS of the local search on general shapes goes by stage pair (see dtfm_ls_enqueue) when there are at least
// three stages; pricing (dtfm_move_costs) and the other cases materialise every swap of a chunk of candidates
static bool all_pairs_by_group(const dtfm_problem *pr) { return !pr->fast64 && pr->D_pp >= 3; }

dtfm_ls_bufs dtfm_ls_carve(const dtfm_problem *pr, dtfm_arena &ar, size_t P, int neighbourhood, bool pricing)
{
    dtfm_ls_bufs b;
    size_t N = pr->N, M = N * (N - 1) / 2;
    b.cur = ar.take<double>(P);
    b.all_cost = nullptr;
    b.group_chunk = 0;
    if (neighbourhood == DTFM_ALL_PAIRS && M > 0) {
        size_t chunk = DTFM_LS_ROWS_MAX / M;
        if (chunk < 1) chunk = 1;
        if (chunk > P) chunk = P;
        b.chunk = chunk;
        b.rows = chunk * M > P ? chunk * M : P;
        if (!pricing && all_pairs_by_group(pr)) {
            const size_t G = (size_t)pr->D_dp * pr->D_dp;   // the largest group: swaps between two stages
            size_t gc = DTFM_LS_ROWS_MAX / G;
            if (gc < 1) gc = 1;
            if (gc > P) gc = P;
            b.group_chunk = gc;
            b.rows = gc * G > P ? gc * G : P;
            b.all_cost = ar.take<double>(gc * M);
        }
    } else {
        b.chunk = P;
        b.rows = neighbourhood == DTFM_BEST4 ? 4 * P : P;   // BEST4 prices four trials per candidate
    }
    b.move_ab = ar.take<int32_t>(2 * b.rows);
    b.tmp_perm = ar.take<int32_t>(b.rows * N);
    b.tmp_cost = ar.take<double>(b.rows);
    b.ghat_cur = ar.take<double>(P * (size_t)pr->D_pp * pr->D_pp);
    b.pp_cur = ar.take<double>(P);
    b.ev = dtfm_eval_carve(pr, ar, b.rows);
    return b;
}

int dtfm_move_costs_enqueue(const dtfm_problem *pr, const dtfm_ls_bufs &b, const int32_t *perm, size_t P, double *out,
                            hipStream_t st)
{
    const int N = pr->N;
    const long long M = (long long)N * (N - 1) / 2;
    if (P == 0 || M == 0) return DTFM_OK;
    if (pr->fast64) return dtfm_fast64_move_costs_enqueue(pr, perm, P, out, st);
    for (size_t p0 = 0; p0 < P; p0 += b.chunk) {
        size_t cp = P - p0 < b.chunk ? P - p0 : b.chunk;
        size_t rows = cp * (size_t)M;
        hipLaunchKernelGGL(k_make_swapped, dim3((unsigned)rows), dim3(DTFM_WAVE), 0, st, perm, N, M, p0, b.tmp_perm);
        DTFM_HIP(hipGetLastError());
        int rc = dtfm_eval_enqueue(pr, b.ev, b.tmp_perm, rows, out + p0 * (size_t)M, st);
        if (rc != DTFM_OK) return rc;
    }
    return DTFM_OK;
}

int dtfm_ls_enqueue(const dtfm_problem *pr, const dtfm_ls_bufs &b, int32_t *perm, size_t P, int moves,
                    int neighbourhood, double *cost, int64_t *applied, hipStream_t st)
{
    if (P == 0) return DTFM_OK;
    if (pr->fast64 && neighbourhood == DTFM_GAIN4)
        return dtfm_fast64_ls_gain4_enqueue(pr, perm, P, moves, cost, applied, st);
    if (pr->fast64 && neighbourhood == DTFM_ALL_PAIRS && moves > 0)
        return dtfm_fast64_ls_allpairs_enqueue(pr, perm, P, moves, cost, applied, st);
    const int N = pr->N;
    const long long M = (long long)N * (N - 1) / 2;
    int rc = dtfm_eval_enqueue(pr, b.ev, perm, P, b.cur, st);
    if (rc != DTFM_OK) return rc;
    for (int r = 0; r < moves; r++) {
        if (neighbourhood == DTFM_ALL_PAIRS) {
            if (M == 0) {
                if (applied != nullptr) {
                    size_t n = P * (size_t)moves;
                    hipLaunchKernelGGL(k_fill_i64, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, applied,
                                       (int64_t)-1, n);
                    DTFM_HIP(hipGetLastError());
                }
                break;
            }
            if (b.all_cost != nullptr) {
                // By stage pair: the swaps between two stages leave every other stage's DataP rows and every
                // coarsened edge outside those two stages as they are, so a group's trial rows start from their
                // current row's graph, match again only the 2 D_pp - 3 edges of the two stages (none for swaps
                // inside a stage) and skip Held-Karp where the graph settles the trial (k_trial_shortcut: a trial
                // it rejects gets +inf, which is never picked: it is not below the current cost).
                const int n = pr->D_pp, nn = n * n, D = pr->D_dp;
                if (r > 0) {   // graphs and PipelineP of the rows as they are now (round 0: just evaluated)
                    rc = dtfm_eval_enqueue(pr, b.ev, perm, P, b.cur, st);
                    if (rc != DTFM_OK) return rc;
                }
                hipLaunchKernelGGL(k_copy_f64, dim3((unsigned)((P * nn + 255) / 256)), dim3(256), 0, st, b.ev.ghat, b.ghat_cur,
                                   P * nn);
                DTFM_HIP(hipGetLastError());
                hipLaunchKernelGGL(k_copy_f64, dim3((unsigned)((P + 255) / 256)), dim3(256), 0, st, b.ev.pp, b.pp_cur, P);
                DTFM_HIP(hipGetLastError());
                for (size_t p0 = 0; p0 < P; p0 += b.group_chunk) {
                    const size_t cp = P - p0 < b.group_chunk ? P - p0 : b.group_chunk;
                    for (int j = 0; j < n; j++) {
                        for (int jp = j; jp < n; jp++) {
                            const long long G = j == jp ? (long long)D * (D - 1) / 2 : (long long)D * D;
                            if (G == 0) continue;
                            const size_t T = cp * (size_t)G;
                            hipLaunchKernelGGL(k_make_swapped_group, dim3((unsigned)T), dim3(DTFM_WAVE), 0, st, perm, N, D, j, jp,
                                               G, p0, b.tmp_perm);
                            DTFM_HIP(hipGetLastError());
                            hipLaunchKernelGGL(k_replicate_f64, dim3((unsigned)((T * nn + 255) / 256)), dim3(256), 0, st,
                                               b.ghat_cur + p0 * nn, b.ev.ghat, nn, (int)G, T * nn);
                            DTFM_HIP(hipGetLastError());
                            const dtfm_trial_ref ref = {b.ghat_cur + p0 * nn, b.pp_cur + p0, b.cur + p0, (int)G};
                            rc = dtfm_eval_inc_enqueue(pr, b.ev, b.tmp_perm, T, b.tmp_cost, j, jp, st, &ref);
                            if (rc != DTFM_OK) return rc;
                            hipLaunchKernelGGL(k_scatter_group, dim3((unsigned)((T + 255) / 256)), dim3(256), 0, st, b.tmp_cost, T,
                                               N, D, j, jp, G, M, b.all_cost);
                            DTFM_HIP(hipGetLastError());
                        }
                    }
                    hipLaunchKernelGGL(k_pick_apply, dim3((unsigned)cp), dim3(256), 0, st, perm, N, M, p0, b.all_cost, b.cur,
                                       applied, moves, r);
                    DTFM_HIP(hipGetLastError());
                }
                continue;
            }
            for (size_t p0 = 0; p0 < P; p0 += b.chunk) {
                size_t cp = P - p0 < b.chunk ? P - p0 : b.chunk;
                size_t rows = cp * (size_t)M;
                hipLaunchKernelGGL(k_make_swapped, dim3((unsigned)rows), dim3(DTFM_WAVE), 0, st, perm, N, M, p0,
                                   b.tmp_perm);
                DTFM_HIP(hipGetLastError());
                rc = dtfm_eval_enqueue(pr, b.ev, b.tmp_perm, rows, b.tmp_cost, st);
                if (rc != DTFM_OK) return rc;
                hipLaunchKernelGGL(k_pick_apply, dim3((unsigned)cp), dim3(256), 0, st, perm, N, M, p0, b.tmp_cost,
                                   b.cur, applied, moves, r);
                DTFM_HIP(hipGetLastError());
            }
        } else {
            // A round's trial rows differ from the current rows in the round's two stages only: with three or
            // more stages the trial evaluation starts from the current rows' coarsened graphs and matches
            // again only the 2 D_pp - 3 edges of those two stages.
            const int n = pr->D_pp, nn = n * n;
            const bool inc = n >= 3 && !pr->fast64;   // the 64-device shape prices rows with its own fused kernel
            const int tpr = neighbourhood == DTFM_BEST4 ? 4 : 1;   // trial rows per candidate
            const size_t T = P * (size_t)tpr;
            int j = -1, jp = -1;
            if (inc) {
                int t = r % pr->npairs;   // the round's stage pair, lexicographic order
                j = 0;
                while (t >= n - 1 - j) {
                    t -= n - 1 - j;
                    j++;
                }
                jp = j + 1 + t;
                if (r == 0) {   // the evaluation above left the current rows' graphs and PipelineP-Costs in b.ev
                    hipLaunchKernelGGL(k_copy_f64, dim3((unsigned)((P * nn + 255) / 256)), dim3(256), 0, st, b.ev.ghat,
                                       b.ghat_cur, P * nn);
                    DTFM_HIP(hipGetLastError());
                    hipLaunchKernelGGL(k_copy_f64, dim3((unsigned)((P + 255) / 256)), dim3(256), 0, st, b.ev.pp, b.pp_cur, P);
                    DTFM_HIP(hipGetLastError());
                }
                if (r > 0 || tpr > 1) {   // every trial row starts from its current row's graph
                    hipLaunchKernelGGL(k_replicate_f64, dim3((unsigned)((T * nn + 255) / 256)), dim3(256), 0, st, b.ghat_cur,
                                       b.ev.ghat, nn, tpr, T * nn);
                    DTFM_HIP(hipGetLastError());
                }
            }
            hipLaunchKernelGGL(neighbourhood == DTFM_KL ? k_kl_propose : neighbourhood == DTFM_BEST4 ? k_best4_propose : k_gain4_propose,
                               dim3((unsigned)P), dim3(DTFM_WAVE), 0, st, pr->W_pp, perm, N, pr->D_dp, pr->D_pp, r, b.tmp_perm,
                               b.move_ab);
            DTFM_HIP(hipGetLastError());
            const dtfm_trial_ref ref = {b.ghat_cur, b.pp_cur, b.cur, tpr};
            rc = dtfm_eval_inc_enqueue(pr, b.ev, b.tmp_perm, T, b.tmp_cost, j, jp, st, inc ? &ref : nullptr);
            if (rc != DTFM_OK) return rc;
            if (neighbourhood == DTFM_BEST4) {
                hipLaunchKernelGGL(k_best4_pick, dim3((unsigned)P), dim3(DTFM_WAVE), 0, st, perm, N, b.tmp_cost, b.cur, b.move_ab,
                                   applied, moves, r, nn, b.ev.ghat, inc ? b.ghat_cur : (double *)nullptr, b.ev.pp,
                                   inc ? b.pp_cur : (double *)nullptr);
                DTFM_HIP(hipGetLastError());
                continue;
            }
            if (inc) {
                hipLaunchKernelGGL(k_keep_ghat, dim3((unsigned)P), dim3(DTFM_WAVE), 0, st, b.tmp_cost, b.cur, nn, b.ev.ghat,
                                   b.ghat_cur, b.ev.pp, b.pp_cur);
                DTFM_HIP(hipGetLastError());
            }
            hipLaunchKernelGGL(k_accept, dim3((unsigned)((P + 255) / 256)), dim3(256), 0, st, perm, N, b.tmp_cost,
                               b.cur, b.move_ab, applied, moves, r, P);
            DTFM_HIP(hipGetLastError());
        }
    }
    hipLaunchKernelGGL(k_copy_f64, dim3((unsigned)((P + 255) / 256)), dim3(256), 0, st, b.cur, cost, P);
    DTFM_HIP(hipGetLastError());
    return DTFM_OK;
}

// ------------------------------------------------------------------------------------------------
__global__ void k_philox_blocks(uint32_t k0, uint32_t k1, uint32_t stream, uint32_t g, uint32_t k,
                                uint32_t first_block, int n_blocks, uint32_t *__restrict__ out)
{
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= n_blocks) return;
    philox_out o = philox4x32_10(first_block + (uint32_t)b, k, g, stream, k0, k1);
    for (int i = 0; i < 4; i++) out[4 * b + i] = o.w[i];
}

int dtfm_philox_enqueue(uint64_t seed, uint32_t stream, uint32_t g, uint32_t k, uint32_t first_block,
                        int n_blocks, uint32_t *out, hipStream_t st)
{
    if (n_blocks == 0) return DTFM_OK;
    hipLaunchKernelGGL(k_philox_blocks, dim3((n_blocks + 63) / 64), dim3(64), 0, st, (uint32_t)seed,
                       (uint32_t)(seed >> 32), stream, g, k, first_block, n_blocks, out);
    DTFM_HIP(hipGetLastError());
    return DTFM_OK;
}

// Initial population: candidate k = Fisher-Yates shuffle of the identity, i = N-1 .. 1,
// j = randint(i+1) from draw number N-1-i of stream INIT. The draws are generated by all lanes,
// the dependent swaps by lane 0.
__global__ void k_init_population(uint32_t k0, uint32_t k1, int N, int32_t *__restrict__ pop)
{
    extern __shared__ int32_t sm[];
    int32_t *perm = sm, *jd = sm + N;
    uint32_t k = blockIdx.x;
    for (int q = threadIdx.x; q < N; q += blockDim.x) perm[q] = q;
    for (int blk = threadIdx.x; 4 * blk < N - 1; blk += blockDim.x) {
        philox_out o = philox4x32_10((uint32_t)blk, k, 0u, STREAM_INIT, k0, k1);
        for (int i = 0; i < 4; i++) {
            int t = 4 * blk + i;
            if (t < N - 1) jd[t] = (int32_t)randint(o.w[i], (uint32_t)(N - t));  // i+1 = N-1-t+1
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int t = 0; t < N - 1; t++) {
            int i = N - 1 - t, j = jd[t];
            int32_t x = perm[i];
            perm[i] = perm[j];
            perm[j] = x;
        }
    }
    __syncthreads();
    for (int q = threadIdx.x; q < N; q += blockDim.x) pop[(size_t)k * N + q] = perm[q];
}

// One offspring per workgroup: selection (two uniform parents), crossover (child = parent 1; m_x
// times a random device that parent 2 keeps in another stage is swapped with the device at a
// random slot of that stage), mutation (m_m random transpositions). Copies, inversions and the
// random draws (two steps per Philox block) are done by all lanes, DTFM_DRAW_CHUNK steps at a time;
// the dependent swaps by lane 0 in LDS.
#define DTFM_DRAW_CHUNK 128
__global__ void k_make_offspring(uint32_t k0, uint32_t k1, uint32_t g, const int32_t *__restrict__ pop,
                                 int P, int N, int D_dp, int m_x, int m_m, int32_t *__restrict__ off)
{
    extern __shared__ int32_t sm[];
    int32_t *child = sm, *pos_child = sm + N, *pos_par2 = sm + 2 * N, *stage_of = sm + 3 * N;
    int32_t *draw_a = sm + 4 * N, *draw_b = draw_a + DTFM_DRAW_CHUNK;
    uint32_t k = blockIdx.x;
    philox_out sel = philox4x32_10(0u, k, g, STREAM_SELECT, k0, k1);
    int p1 = (int)randint(sel.w[0], (uint32_t)P), p2 = (int)randint(sel.w[1], (uint32_t)P);
    const int32_t *par1 = pop + (size_t)p1 * N, *par2 = pop + (size_t)p2 * N;
    for (int q = threadIdx.x; q < N; q += blockDim.x) {
        int32_t d = par1[q];
        child[q] = d;
        pos_child[d] = q;
        pos_par2[par2[q]] = q;
        stage_of[q] = q / D_dp;
    }
    for (int t0 = 0; t0 < m_x; t0 += DTFM_DRAW_CHUNK) {
        const int steps = min(DTFM_DRAW_CHUNK, m_x - t0);   // t0 is even: step t0 + 2 b + h uses words 2 h, 2 h + 1 of block (t0 / 2 + b)
        __syncthreads();
        for (int blk = threadIdx.x; 2 * blk < steps; blk += blockDim.x) {
            const philox_out o = philox4x32_10((uint32_t)(t0 / 2 + blk), k, g, STREAM_CROSSOVER, k0, k1);
            for (int h = 0; h < 2; h++) {
                // the device, and the position it would go to: the drawn slot of the stage parent 2 keeps it in
                // (parent 2 does not change, so this is known before the dependent steps)
                const int d = (int)randint(o.w[2 * h], (uint32_t)N);
                const int slot = (int)randint(o.w[2 * h + 1], (uint32_t)D_dp);
                draw_a[2 * blk + h] = d;
                draw_b[2 * blk + h] = stage_of[pos_par2[d]] * D_dp + slot;
            }
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            for (int t = 0; t < steps; t++) {
                const int d = draw_a[t], qb = draw_b[t];
                const int qa = pos_child[d];
                const int e = child[qb];
                if (stage_of[qa] == stage_of[qb]) continue;
                child[qa] = e;
                child[qb] = d;
                pos_child[e] = qa;
                pos_child[d] = qb;
            }
        }
    }
    for (int t0 = 0; t0 < m_m; t0 += DTFM_DRAW_CHUNK) {
        const int steps = min(DTFM_DRAW_CHUNK, m_m - t0);
        __syncthreads();
        for (int blk = threadIdx.x; 2 * blk < steps; blk += blockDim.x) {
            const philox_out o = philox4x32_10((uint32_t)(t0 / 2 + blk), k, g, STREAM_MUTATION, k0, k1);
            for (int h = 0; h < 2; h++) {
                draw_a[2 * blk + h] = (int32_t)randint(o.w[2 * h], (uint32_t)N);
                draw_b[2 * blk + h] = (int32_t)randint(o.w[2 * h + 1], (uint32_t)N);
            }
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            for (int t = 0; t < steps; t++) {
                const int a = draw_a[t], b = draw_b[t];
                const int32_t x = child[a];
                child[a] = child[b];
                child[b] = x;
            }
        }
    }
    __syncthreads();
    for (int q = threadIdx.x; q < N; q += blockDim.x) off[(size_t)k * N + q] = child[q];
}

// Replacement: rank of element i among parents (origin 0..P-1) and offspring (origin P..P+L-1)
// under the order (cost, origin); the P lowest survive, placed at their rank. The count over the
// P+L keys is split: block (x, y) counts, for 256 elements i, the keys of chunk y that precede them,
// and adds the partial count to rank[i]. A wavefront walks its chunk in dependent steps of sixteen
// keys, each a round trip to the scalar cache: short chunks (many blocks) keep that chain short.
#define DTFM_RANK_CHUNK 64
// counts the keys key[0..m) that precede element (ci, i); j_first = index of key[0] among all keys.
// MODE 0: key <= ci (the keys all have lower indices), 1: key < ci (all higher), 2: index compared.
// The key address is the same for every lane: the loads go through the scalar cache, sixteen keys at a time.
template <int MODE>
__device__ __forceinline__ int count_before(const double *__restrict__ key, int m, int j_first, double ci, int i)
{
    int cnt = 0, t = 0;
    for (; t + 16 <= m; t += 16) {
        double k8[16];
#pragma unroll
        for (int e = 0; e < 16; e++) k8[e] = key[t + e];
#pragma unroll
        for (int e = 0; e < 16; e++)
            cnt += MODE == 0 ? (k8[e] <= ci ? 1 : 0)
                 : MODE == 1 ? (k8[e] < ci ? 1 : 0)
                             : ((k8[e] < ci || (k8[e] == ci && j_first + t + e < i)) ? 1 : 0);
    }
    for (; t < m; t++) {
        const double kj = key[t];
        cnt += MODE == 0 ? (kj <= ci ? 1 : 0) : MODE == 1 ? (kj < ci ? 1 : 0) : ((kj < ci || (kj == ci && j_first + t < i)) ? 1 : 0);
    }
    return cnt;
}

// With parents_sorted the parents are in (cost, origin) order already (every generation but the first:
// the previous replacement placed them by rank): parent i has i parents before it, an offspring as
// many as have a cost <= its own (binary search), and only the offspring keys are counted.
__global__ void k_rank_count(const double *__restrict__ cost, const double *__restrict__ off_cost, int P, int L,
                             int parents_sorted, int chunk, int32_t *__restrict__ rank)
{
    const int n = P + L;
    const int j0 = blockIdx.y * chunk;
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int j1 = j0 + chunk < n ? j0 + chunk : n;
    if (parents_sorted && blockIdx.y != 0 && j1 <= P) return;
    const double ci = i < P ? cost[i] : off_cost[i - P];
    // the chunk's keys: [ja, jb) among the parents, [jc, jd) among the offspring
    int ja = j0 < P ? j0 : P, jb = j1 < P ? j1 : P;
    const int jc = j0 > P ? j0 : P, jd = j1 > P ? j1 : P;
    int base = 0;
    if (parents_sorted) {
        if (blockIdx.y == 0) {
            if (i < P) {
                base = i;
            } else {
                int lo = 0, hi = P;
                while (lo < hi) {
                    const int mid = (lo + hi) >> 1;
                    if (cost[mid] <= ci) lo = mid + 1;
                    else hi = mid;
                }
                base = lo;
            }
        }
        ja = jb = P;   // no parent keys
    }
    // A chunk that lies wholly before (after) this block's elements needs no index comparison: ties go
    // to the key (to the element).
    const int i0 = blockIdx.x * blockDim.x;
    int cnt;
    if (j1 <= i0)
        cnt = count_before<0>(cost + ja, jb - ja, ja, ci, i) + count_before<0>(off_cost + (jc - P), jd - jc, jc, ci, i);
    else if (j0 >= i0 + (int)blockDim.x)
        cnt = count_before<1>(cost + ja, jb - ja, ja, ci, i) + count_before<1>(off_cost + (jc - P), jd - jc, jc, ci, i);
    else
        cnt = count_before<2>(cost + ja, jb - ja, ja, ci, i) + count_before<2>(off_cost + (jc - P), jd - jc, jc, ci, i);
    cnt += base;
    if (cnt) atomicAdd(&rank[i], cnt);
}

// Replacement, second step: one workgroup per element; an element whose rank is below P is a survivor:
// its row and cost go to position `rank` of the next population, the lowest to the trace. The element's
// rank counter is cleared for the next generation.
__global__ void k_rank_place(const int32_t *__restrict__ pop, const int32_t *__restrict__ off,
                             const double *__restrict__ cost, const double *__restrict__ off_cost, int P, int L, int N,
                             int32_t *__restrict__ rank, int32_t *__restrict__ next, double *__restrict__ next_cost,
                             double *__restrict__ trace_slot)
{
    const int i = blockIdx.x;
    const int r = rank[i];
    __syncthreads();   // every thread has read the counter before thread 0 clears it
    if (threadIdx.x == 0) rank[i] = 0;
    if (r >= P) return;
    const int32_t *s = i < P ? pop + (size_t)i * N : off + (size_t)(i - P) * N;
    for (int q = threadIdx.x; q < N; q += blockDim.x) next[(size_t)r * N + q] = s[q];
    if (threadIdx.x == 0) {
        const double ci = i < P ? cost[i] : off_cost[i - P];
        next_cost[r] = ci;
        if (r == 0) *trace_slot = ci;
    }
}

__global__ void k_fill_i32(int32_t *__restrict__ dst, int32_t v, size_t n)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = v;
}

dtfm_ga_bufs dtfm_ga_carve(const dtfm_problem *pr, dtfm_arena &ar, const dtfm_ga_params &prm)
{
    dtfm_ga_bufs b;
    size_t P = prm.P, L = prm.lambda, N = pr->N;
    b.off = ar.take<int32_t>(L * N);
    b.off_cost = ar.take<double>(L);
    b.next = ar.take<int32_t>(P * N);
    b.next_cost = ar.take<double>(P);
    b.rank = ar.take<int32_t>(P + L);
    b.ls = dtfm_ls_carve(pr, ar, P > L ? P : L, prm.neighbourhood);
    return b;
}

int dtfm_ga_enqueue(const dtfm_problem *pr, const dtfm_ga_bufs &b, uint64_t seed, int generations,
                    const dtfm_ga_params &prm, int32_t *population, double *cost, double *best_trace,
                    hipStream_t st)
{
    const int N = pr->N, P = prm.P, L = prm.lambda;
    const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    if (!prm.warm_start) {
        hipLaunchKernelGGL(k_init_population, dim3(P), dim3(DTFM_WAVE), 2 * N * sizeof(int32_t), st, k0, k1, N,
                           population);
        DTFM_HIP(hipGetLastError());
    }
    int rc = dtfm_eval_enqueue(pr, b.ls.ev, population, P, cost, st);
    if (rc != DTFM_OK) return rc;
    const int nk = P + L;
    hipLaunchKernelGGL(k_fill_i32, dim3((nk + 255) / 256), dim3(256), 0, st, b.rank, 0, (size_t)nk);
    DTFM_HIP(hipGetLastError());
    // the population alternates between the caller's buffers and the arena's
    int32_t *pop_cur = population, *pop_next = b.next;
    double *cost_cur = cost, *cost_next = b.next_cost;
    for (int g = 0; g < generations; g++) {
        if (pr->fast64 && prm.neighbourhood == DTFM_GAIN4 && dtfm_fast64_ls_makes_offspring(pr, L, prm.ls_moves)) {
            // one launch makes the offspring and carries them through the local search
            const dtfm_offspring_src src = {k0, k1, (uint32_t)g, pop_cur, P, prm.m_x, prm.m_m};
            rc = dtfm_fast64_offspring_ls_gain4_enqueue(pr, src, b.off, L, prm.ls_moves, b.off_cost, st);
            if (rc != DTFM_OK) return rc;
        } else {
            hipLaunchKernelGGL(k_make_offspring, dim3(L), dim3(DTFM_WAVE), (4 * N + 2 * DTFM_DRAW_CHUNK) * sizeof(int32_t), st,
                               k0, k1, (uint32_t)g, pop_cur, P, N, pr->D_dp, prm.m_x, prm.m_m, b.off);
            DTFM_HIP(hipGetLastError());
            rc = dtfm_ls_enqueue(pr, b.ls, b.off, L, prm.ls_moves, prm.neighbourhood, b.off_cost, nullptr, st);
            if (rc != DTFM_OK) return rc;
        }
        int chunk = DTFM_RANK_CHUNK;   // longer chunks when the grid's second dimension would not hold the short ones
        while ((nk + chunk - 1) / chunk > 65535) chunk *= 2;
        hipLaunchKernelGGL(k_rank_count, dim3((nk + 255) / 256, (nk + chunk - 1) / chunk), dim3(256), 0,
                           st, cost_cur, b.off_cost, P, L, g > 0 ? 1 : 0, chunk, b.rank);
        DTFM_HIP(hipGetLastError());
        hipLaunchKernelGGL(k_rank_place, dim3(nk), dim3(DTFM_WAVE), 0, st, pop_cur, b.off, cost_cur, b.off_cost, P, L, N,
                           b.rank, pop_next, cost_next, best_trace + g);
        DTFM_HIP(hipGetLastError());
        int32_t *tp = pop_cur;
        pop_cur = pop_next;
        pop_next = tp;
        double *tc = cost_cur;
        cost_cur = cost_next;
        cost_next = tc;
    }
    if (pop_cur != population) {
        size_t n = (size_t)P * N;
        hipLaunchKernelGGL(k_copy_i32, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, pop_cur, population, n);
        DTFM_HIP(hipGetLastError());
        hipLaunchKernelGGL(k_copy_f64, dim3((P + 255) / 256), dim3(256), 0, st, cost_cur, cost, (size_t)P);
        DTFM_HIP(hipGetLastError());
    }
    return DTFM_OK;
}

// ------------------------------------------------------------------------------------------------
// Validity of an allocation (Sec. 2): every device exactly once.
__global__ void k_validate(const int32_t *__restrict__ perm, int N, int32_t *__restrict__ bad_rows)
{
    extern __shared__ int32_t seen[];
    __shared__ int bad;
    size_t p = blockIdx.x;
    if (threadIdx.x == 0) bad = 0;
    for (int q = threadIdx.x; q < N; q += blockDim.x) seen[q] = 0;
    __syncthreads();
    for (int q = threadIdx.x; q < N; q += blockDim.x) {
        int d = perm[p * N + q];
        if (d < 0 || d >= N) bad = 1;
        else if (atomicAdd(&seen[d], 1) != 0) bad = 1;
    }
    __syncthreads();
    if (threadIdx.x == 0 && bad) atomicAdd(bad_rows, 1);
}

__global__ void k_zero_i32(int32_t *p) { *p = 0; }

int dtfm_validate_enqueue(const dtfm_problem *pr, const int32_t *perm, size_t P, int32_t *bad_rows,
                          hipStream_t st)
{
    hipLaunchKernelGGL(k_zero_i32, dim3(1), dim3(1), 0, st, bad_rows);
    DTFM_HIP(hipGetLastError());
    if (P == 0) return DTFM_OK;
    hipLaunchKernelGGL(k_validate, dim3((unsigned)P), dim3(DTFM_WAVE), pr->N * sizeof(int32_t), st, perm, pr->N,
                       bad_rows);
    DTFM_HIP(hipGetLastError());
    return DTFM_OK;
}
