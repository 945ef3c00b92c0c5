// General-shape kernels for the cost model (any N <= 1024, D_dp <= 64, D_pp <= 16):
//   k_weights     Sec. 2 symmetrisation + the per-link terms of Eqs. 2 and 3
//   k_datap       Eq. 2 per stage and the max over stages (Sec. 3.2); for matrices beyond an XCD's L2
//                 k_datap_sliced (by slice of devices) or k_positions + k_datap_rows + k_datap_reduce (by device)
//   k_match       Eq. 3: bottleneck perfect matching of one stage pair per wavefront
//   k_held_karp   Eq. 4: open-loop TSP over the coarsened graph, exact, by subset dynamic
//                 programming; adds the two parts (Eq. 1); k_held_karp_blocked from 11 stages on
//   k_trial_shortcut   trials of the local search that the coarsened graph settles without Eq. 4
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

// Eq. 2 by device, for the same large matrices as k_datap_sliced, when a stage is a whole number of 16-byte pieces of
// the row (D_dp a multiple of 4, rows 16-byte aligned). A gather of W_dp from L2 moves a cache sector per 8 bytes
// used; here every workgroup keeps DTFM_DATAP_DPW rows of W_dp in LDS and sums, for each candidate of its share,
// the row sums of those devices: the device's position comes from the inverse of the row (k_positions), the
// members of its stage are read as contiguous 16-byte pieces, and the entries come from LDS. The sum runs over
// the stage's slots in order from +0.0; the device's own slot adds W_dp[d][d] = +0.0, which leaves the (non-
// negative) sum as it is, so the bits are those of the sum that skips it. Row sums go to rowsum[p][position];
// k_datap_reduce takes the maximum per candidate.
#define DTFM_DATAP_DPW 4
#define DTFM_DATAP_SPLIT 4   // workgroups that share a group of devices; each takes every SPLIT-th pass of candidates

__global__ void k_positions(const int32_t *__restrict__ perm, int N, size_t total, int32_t *__restrict__ pos)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const size_t p = i / (size_t)N;
    const uint32_t d = (uint32_t)perm[i];
    if (d < (uint32_t)N) pos[p * N + d] = (int32_t)(i - p * N);
}

__global__ void __launch_bounds__(256)
k_datap_rows(const double *__restrict__ W_dp, const int32_t *__restrict__ perm, const int32_t *__restrict__ pos, int N,
             int D_dp, size_t P, double *__restrict__ rowsum)
{
    extern __shared__ double s_W[];   // DTFM_DATAP_DPW rows of W_dp
    const int d0 = (int)(blockIdx.x / DTFM_DATAP_SPLIT) * DTFM_DATAP_DPW, share = (int)(blockIdx.x % DTFM_DATAP_SPLIT);
    for (int e = threadIdx.x; e < DTFM_DATAP_DPW * N; e += blockDim.x) s_W[e] = W_dp[(size_t)d0 * N + e];
    __syncthreads();
    const int r = threadIdx.x % DTFM_DATAP_DPW;
    const size_t per = blockDim.x / DTFM_DATAP_DPW;   // candidates per pass
    const double *wr = s_W + r * N;
    const uint32_t last = (uint32_t)N - 1u;
    for (size_t p = (size_t)share * per + threadIdx.x / DTFM_DATAP_DPW; p < P; p += per * DTFM_DATAP_SPLIT) {
        // a row that is not a permutation leaves positions unwritten: any value is kept inside the row
        const uint32_t q = min((uint32_t)pos[p * N + d0 + r], last);
        const uint32_t j = q / (uint32_t)D_dp;
        const int4 *C = reinterpret_cast<const int4 *>(perm + p * N + (size_t)j * D_dp);
        double sum = 0.0;
        for (int k4 = 0; k4 < D_dp / 4; k4++) {
            const int4 c = C[k4];
            sum = __dadd_rn(sum, wr[min((uint32_t)c.x, last)]);
            sum = __dadd_rn(sum, wr[min((uint32_t)c.y, last)]);
            sum = __dadd_rn(sum, wr[min((uint32_t)c.z, last)]);
            sum = __dadd_rn(sum, wr[min((uint32_t)c.w, last)]);
        }
        rowsum[p * N + q] = sum;
    }
}

// max over a candidate's row sums (all weights are >= 0, so every row sum is >= +0.0); also zeroes the diagonal
// of the candidate's coarsened graph
__global__ void __launch_bounds__(256)
k_datap_reduce(const double *__restrict__ rowsum, int N, int D_pp, double *__restrict__ datap, double *__restrict__ ghat)
{
    __shared__ double s_red[4];
    const size_t p = blockIdx.x;
    double worst = 0.0;
    for (int q = threadIdx.x; q < N; q += blockDim.x) worst = fmax(worst, rowsum[p * N + q]);
    if (ghat != nullptr)
        for (int j = threadIdx.x; j < D_pp; j += blockDim.x) ghat[(p * D_pp + j) * D_pp + j] = 0.0;
    for (int o = 32; o >= 1; o >>= 1) worst = fmax(worst, __shfl_xor(worst, o));
    if ((threadIdx.x & (DTFM_WAVE - 1)) == 0) s_red[threadIdx.x / DTFM_WAVE] = worst;
    __syncthreads();
    if (threadIdx.x == 0) datap[p] = fmax(fmax(s_red[0], s_red[1]), fmax(s_red[2], s_red[3]));
}

__global__ void k_zero_f64(double *__restrict__ dst, size_t n)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = 0.0;
}

// ------------------------------------------------------------------------------------------------
// a4: bottleneck assignment for one (candidate, stage pair) per wavefront (one wavefront per workgroup),
// lane c = column c (device at slot c of the second stage). The optimum of Eq. 3 is one of the block's
// entries and depends only on their order, so the search runs on the dense ranks of W_pp (equal weights share
// a rank), and the result is mapped back through `rank_val`: no rounding is involved.
//
// Invariant: a matching of some of the rows within the threshold theta, and theta <= the optimum T*.
//  1. theta starts at the largest column minimum (every column is matched through one of its entries).
//  2. Greedy pass, rows in order: a row takes the first free column it reaches within theta. A row with
//     no entry within theta at all raises theta to its own minimum first (it too is matched through one
//     of its entries). Rows that find no free column are left pending.
//  3. Every pending row r0 is inserted by an alternating-path search: dist[c] is the smallest entry from a
//     reached row to column c, every unvisited column with dist <= theta is reachable within theta, and
//     the rows matched to the newly reached columns join the search. When the search is stuck, the reached
//     rows X own one column fewer than they need among the visited ones, so some row of X is matched
//     outside them in every perfect matching: T* >= the smallest dist of an unvisited column, and theta is
//     raised to exactly that. An alternating path to a free column exists within theta iff a larger
//     matching does (Berge), so after the last insertion theta = T*.
// The order in which rows are inserted and ties between paths do not change the value.
//
// Lane c keeps its column of the block in registers for the steps whose row index is known at compile time
// (1 and 2). For the search, where the row comes from a lane, the wavefront keeps the block in LDS,
// s_E[r * 64 + c] (all lanes read one row: no bank conflicts); 8 KiB per wavefront, and the number of resident
// wavefronts is what this latency-bound search lives on. Registers and LDS hold 16-bit codes, order-preserving
// images of the ranks:
//  - first solve: the entries are gathered from `Wcode`, 2 + (rank >> shift) with the `shift` that fits the
//    problem's largest rank (0 up to 65,532 distinct weights), pad 0xffff: the result is the exact optimum when
//    shift = 0, else the bucket of 2^shift ranks that holds it (a matching within a bucket exists iff one
//    exists within the bucket's largest rank);
//  - if the block holds more than one distinct rank of that bucket (looked up in `Wrank`, only by the lanes that
//    hold an entry of the bucket), a second solve on 1 (ranks below the bucket: all "within"), 2 + rank - the
//    bucket's first rank (inside), 0xffff (above: never needed) separates them.
// dist carries, in its low 7 bits, the column whose matched row gave it (127: the inserted row), so relaxing is
// one shift-OR and one unsigned minimum; a visited column parks that field in `parked` and holds dist = 0 from
// then on, which no minimum changes. Lanes c >= D_dp hold the pad code and never take part.
__device__ __forceinline__ uint32_t dtfm_wave_min_u32(uint32_t k)
{
    // prefix minima inside each row of 16 lanes by data-parallel shifts (a lane without a source keeps its own
    // value), then the four row results
    k = min(k, (uint32_t)__builtin_amdgcn_update_dpp((int)k, (int)k, 0x111, 0xF, 0xF, false));   // row_shr:1
    k = min(k, (uint32_t)__builtin_amdgcn_update_dpp((int)k, (int)k, 0x112, 0xF, 0xF, false));   // row_shr:2
    k = min(k, (uint32_t)__builtin_amdgcn_update_dpp((int)k, (int)k, 0x114, 0xF, 0xF, false));   // row_shr:4
    k = min(k, (uint32_t)__builtin_amdgcn_update_dpp((int)k, (int)k, 0x118, 0xF, 0xF, false));   // row_shr:8
    const uint32_t m0 = (uint32_t)__builtin_amdgcn_readlane((int)k, 15), m1 = (uint32_t)__builtin_amdgcn_readlane((int)k, 31);
    const uint32_t m2 = (uint32_t)__builtin_amdgcn_readlane((int)k, 47), m3 = (uint32_t)__builtin_amdgcn_readlane((int)k, 63);
    return min(min(m0, m1), min(m2, m3));
}

// Scalar bit scans of a 64-bit mask in one instruction each: the index of the lowest set bit (-1 for an empty
// mask), and the mask with one bit cleared.
__device__ __forceinline__ int dtfm_first_bit(uint64_t m)
{
    int c;
    asm("s_ff1_i32_b64 %0, %1" : "=s"(c) : "s"(m));
    return c;
}
__device__ __forceinline__ uint64_t dtfm_clear_bit(uint64_t m, int bit)
{
    asm("s_bitset0_b64 %0, %1" : "+s"(m) : "s"(bit));
    return m;
}

#define DTFM_MATCH_ROOT 127u   // `via` field of a dist that comes from the inserted row itself

// Steps 2 and 3 and the second solve for one block, by one wavefront. E: the lane's column as codes (pad 0xffff for the
// rows and lanes outside the block); tile: room for the block's LDS copy, entry (row r, this lane) at tile[r * 64] (the
// caller passes its lane's base). rank_of(r): the rank of the lane's entry in row r (looked up only inside the
// optimum's bucket). Returns the optimum's rank, or 0xffffffff if a search fails (cannot happen for a finite block).
template <int NB, typename RankOf>
__device__ __forceinline__ uint32_t match_block(uint16_t *tile, uint32_t (&E)[16 * NB], int lane, bool active, int D_dp,
                                                int shift0, RankOf rank_of)
{
    constexpr int R = 16 * NB, RS = R - 16;   // rows below RS exist for every D_dp this instance is launched for
    uint32_t colmin = 0xffffu;
#pragma unroll
    for (int r = 0; r < R; r++) colmin = min(colmin, E[r]);
    // the largest column minimum = ~ the smallest of the complements (idle lanes: complement of 0)
    uint32_t theta = ~dtfm_wave_min_u32(active ? ~colmin : 0xffffffffu);   // the threshold, as a code

    const uint64_t allcols = D_dp >= 64 ? ~0ull : ((1ull << D_dp) - 1ull);
    uint32_t base = 0u;              // second solve: first rank of the bucket
    uint32_t result = 0xffffffffu;
    for (int solve = 0; solve < 2; solve++) {
        {
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int r = 0; r < R; r++) tile[r * DTFM_WAVE] = (uint16_t)E[r];
            __builtin_amdgcn_wave_barrier();   // one wavefront: its LDS accesses are executed in order
        }
        uint32_t thr = (theta << 7) | 127u;   // a key (code << 7 | via) is within theta iff key <= thr

        // step 2
        uint64_t freecols = allcols, pending = 0ull;
        int match_row = 0;   // row matched to this lane's column (meaningful when not free)
#pragma unroll
        for (int r = 0; r < R; r++) {
            if (r < RS || r < D_dp) {
                uint64_t m = __ballot(E[r] <= theta);
                if (m == 0ull) {
                    theta = dtfm_wave_min_u32(E[r]);
                    thr = (theta << 7) | 127u;
                    m = __ballot(E[r] <= theta);
                }
                m &= freecols;
                if (m != 0ull) {
                    const int c = dtfm_first_bit(m);
                    freecols = dtfm_clear_bit(freecols, c);
                    if (lane == c) match_row = r;
                } else {
                    pending |= 1ull << r;
                }
            }
        }

        // step 3
        bool failed = false;
        while (pending != 0ull) {
            const int r0 = dtfm_first_bit(pending);
            pending = dtfm_clear_bit(pending, r0);
            uint32_t dist = ((uint32_t)tile[r0 * DTFM_WAVE] << 7) | DTFM_MATCH_ROOT;
            uint32_t parked = 0u;
            int cfin = -1;
            uint64_t reach = __ballot(dist - 1u < thr);   // unvisited (dist != 0) and within theta
            // every turn parks at least one column or ends the search: at most D_dp turns
            for (int turn = 0; turn <= R; turn++) {
                if (reach == 0ull) {
                    // stuck: the smallest dist of an unvisited column; dist - 1 sends the visited ones (0) to the top
                    const uint32_t k = dtfm_wave_min_u32(dist - 1u);
                    if (k >= (0xffffu << 7) - 1u) break;   // no unvisited column with an entry of the block
                    thr = (k + 1u) | 127u;
                    reach = __ballot(dist - 1u < thr);
                }
                const uint64_t hit = reach & freecols;
                if (hit != 0ull) {
                    cfin = dtfm_first_bit(hit);
                    break;
                }
                if (dist - 1u < thr) {
                    parked = dist & 127u;
                    dist = 0u;
                }
                do {   // the rows matched to the newly reached columns join the search, two per turn
                    const int c0 = dtfm_first_bit(reach);
                    reach = dtfm_clear_bit(reach, c0);
                    const int c1 = max(dtfm_first_bit(reach), c0);   // none left: c0 once more
                    reach = dtfm_clear_bit(reach, c1);
                    const int m0 = __builtin_amdgcn_readlane(match_row, c0), m1 = __builtin_amdgcn_readlane(match_row, c1);
                    const uint32_t w0 = ((uint32_t)tile[m0 * DTFM_WAVE] << 7) | (uint32_t)c0;
                    const uint32_t w1 = ((uint32_t)tile[m1 * DTFM_WAVE] << 7) | (uint32_t)c1;
                    dist = min(dist, min(w0, w1));
                } while (reach != 0ull);
                reach = __ballot(dist - 1u < thr);
            }
            if (cfin < 0) {
                failed = true;
                break;
            }
            // flip the path: column c takes the row of its predecessor column; the first column takes r0
            const int via = (int)(dist == 0u ? parked : (dist & 127u));
            int c = cfin;
            for (int step = 0; step <= D_dp; step++) {  // a path has at most D_dp columns
                const int pc = __builtin_amdgcn_readlane(via, c);
                const int prow = __builtin_amdgcn_readlane(match_row, pc & 63);
                if (lane == c) match_row = pc == (int)DTFM_MATCH_ROOT ? r0 : prow;
                if (pc == (int)DTFM_MATCH_ROOT) break;
                c = pc;
            }
            freecols = dtfm_clear_bit(freecols, cfin);
        }
        theta = thr >> 7;   // >= 2: the first solve has no code below 2, the second no matching below its bucket
        if (failed || theta < 2u) break;
        if (solve > 0) {
            result = base + theta - 2u;
            break;
        }
        if (shift0 == 0) {
            result = theta - 2u;
            break;
        }
        // The optimum lies in the bucket of 2^shift0 ranks with code theta. The block's entries with that code, as
        // ranks (few: they are looked up one row at a time, and only by the lanes that hold one): if they are one
        // rank, that is the optimum; else they are told apart by a second solve on 1 (below the bucket),
        // 2 + rank - first rank of the bucket (inside), 0xffff (above it: never needed).
        base = (theta - 2u) << shift0;
        uint32_t lo = 0xffffffffu, hi = 0u;
#pragma unroll
        for (int r = 0; r < R; r++) {
            const bool inside = E[r] == theta;
            if (__ballot(inside) != 0ull) {   // wavefront-uniform
                uint32_t code2 = E[r] < theta ? 1u : 0xffffu;
                if (inside) {
                    const uint32_t rk = rank_of(r);
                    lo = min(lo, rk);
                    hi = max(hi, rk);
                    code2 = 2u + (rk - base);
                }
                E[r] = code2;
            } else {
                E[r] = E[r] < theta ? 1u : 0xffffu;
            }
        }
        lo = dtfm_wave_min_u32(lo);
        hi = ~dtfm_wave_min_u32(~hi);
        if (lo == hi) {
            result = lo;
            break;
        }
        // theta of the second solve starts at the largest column minimum again
        uint32_t cm = 0xffffu;
#pragma unroll
        for (int r = 0; r < R; r++) cm = min(cm, E[r]);
        theta = ~dtfm_wave_min_u32(active ? ~cm : 0xffffffffu);
    }
    return result;
}

// One wavefront (= one workgroup) per (candidate, stage pair): the lane gathers its column of the block from the
// table of codes, 2 bytes an entry (pad 0xffff outside the block), and keeps the block's LDS copy as s_E[r * 64 + c].
template <int NB>  // number of 16-row blocks: D_dp <= 16 * NB
__global__ void __launch_bounds__(DTFM_WAVE) __attribute__((amdgpu_waves_per_eu(5)))
k_match(const uint16_t *__restrict__ Wcode, const uint32_t *__restrict__ Wrank, const double *__restrict__ rank_val, int shift0,
        const int32_t *__restrict__ perm, int N, int D_dp, int D_pp,
        double *__restrict__ ghat, int inc_j, int inc_jp)
{
    constexpr int R = 16 * NB, RS = R - 16;
    extern __shared__ uint16_t s_E[];   // R x 64 codes
    const int lane = threadIdx.x;
    const bool active = lane < D_dp;
    const size_t p = blockIdx.x;   // candidate
    const int t = (int)blockIdx.y; // stage pair
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
        // only the 2 D_pp - 3 pairs that contain stage inc_j or inc_jp (inc_j < inc_jp): (inc_j, k) for
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
    const int32_t *Ca = row + j1 * D_dp;   // wavefront-uniform: read through the scalar cache
    const uint32_t coldev = active ? (uint32_t)row[j2 * D_dp + lane] : 0u;
    uint32_t E[R];
#pragma unroll
    for (int r = 0; r < R; r++) {
        const bool real = r < RS || r < D_dp;
        const uint32_t v = Wcode[(uint32_t)Ca[real ? r : 0] * (uint32_t)N + coldev];
        E[r] = (active && real) ? v : 0xffffu;
    }
    const uint32_t result = match_block<NB>(s_E + lane, E, lane, active, D_dp, shift0, [&](int r) {
        return Wrank[(uint32_t)Ca[r] * (uint32_t)N + coldev];
    });
    if (lane == 0) {
        const double v = result == 0xffffffffu ? INFINITY : rank_val[result];
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
__device__ __forceinline__ void hk_block_layers(double *tab, const uint32_t *lsub, const double (&Gc)[16],
                                                double *X, uint32_t H, int nh, int n, int v, int grp)
{
    static_assert(NL % 2 == 0 && 16 - NL <= 6, "slot pairs (NL + 2 q, NL + 2 q + 1), q < 3");
    constexpr int GROUPS = (1 << NL) / 16, RS = DTFM_HK_ROW_STRIDE;
    uint32_t Lnext = 0;   // layer 0 is the empty low part alone (group 0)
    const bool can_push = v < n;
#pragma unroll
    for (int k = 0; k <= NL; k++) {
        const int first = dtfm_layer_first(NL, k), cnt = dtfm_binom(NL, k);
        const int turns = (cnt + GROUPS - 1) / GROUPS;   // every group takes part in all turns but, maybe, the last
        const uint32_t *next = lsub + first + grp + GROUPS;
#pragma nounroll
        for (int t = 0; t < turns; t++) {
            const uint32_t L = Lnext;
            Lnext = next[t * GROUPS];   // lsub is padded: the read behind the layer's last row stays inside it
            if (t + 1 < turns || grp + (turns - 1) * GROUPS < cnt) {
                const uint32_t S = (H << NL) | L;
                const bool in = (S >> v) & 1u;
                const double2 *row = reinterpret_cast<const double2 *>(tab + L * RS);
                // HM: bit q set = the pair of slots NL + 2 q, NL + 2 q + 1 holds a stage of H. All reads of the row
                // are issued before the first relaxation (left to itself the compiler reuses the registers of the
                // first four and waits for LDS three times per turn).
                double2 x[NPAIR];
#pragma unroll
                for (int h = 0; h < NPAIR; h++) {
                    const bool present = 2 * h >= NL ? ((HM >> ((2 * h - NL) / 2)) & 1u) != 0u : true;
                    if (present) x[h] = row[h];
                }
                __builtin_amdgcn_sched_barrier(0);
                double y = fmin(__dadd_rn(x[0].x, Gc[0]), __dadd_rn(x[0].y, Gc[1]));
#pragma unroll
                for (int h = 1; h < NPAIR; h++) {
                    const bool present = 2 * h >= NL ? ((HM >> ((2 * h - NL) / 2)) & 1u) != 0u : true;
                    if (!present) continue;
                    y = fmin(y, __dadd_rn(x[h].x, Gc[2 * h]));
                    y = fmin(y, __dadd_rn(x[h].y, Gc[2 * h + 1]));
                }
                // the empty set (layer 0 of block 0) pushes nothing: a single stage alone is a path of one node
                if (!in && can_push && (k > 0 || H != 0u)) {
                    if (v < NL)
                        tab[L * RS + ((1u << v) * RS + v)] = y;   // v is not in L: L | 1 << v = L + (1 << v)
                    else
                        X[(((size_t)(H | (1u << (v - NL))) * nh + (v - NL)) << NL) + L] = y;
                }
            }
        }
        if (k < NL) {
            Lnext = lsub[dtfm_layer_first(NL, k + 1) + grp];
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
    uint32_t *lsub = reinterpret_cast<uint32_t *>(G + 256);       // low parts ordered by popcount
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
        lsub[first + rank] = (uint32_t)L;
        if (L < 2 * (THREADS / 16)) lsub[(1 << NL) + L] = 0;   // the entries read ahead behind the last layer
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

// DataP by device (k_datap_rows) pays when W_dp is too large for an XCD's L2; it needs D_dp a multiple of 4
static bool datap_by_device(const dtfm_problem *pr)
{
    return (size_t)pr->N * pr->N * sizeof(double) > ((size_t)2 << 20) && pr->D_dp % 4 == 0 && pr->N % DTFM_DATAP_DPW == 0;
}

dtfm_eval_bufs dtfm_eval_carve(const dtfm_problem *pr, dtfm_arena &ar, size_t rows, size_t hk_grid_cap, bool lean)
{
    dtfm_eval_bufs b;
    size_t n = pr->D_pp;
    b.pos = nullptr;
    b.rowsum = nullptr;
    if (!lean && datap_by_device(pr)) {
        b.pos = ar.take<int32_t>(rows * pr->N);
        b.rowsum = ar.take<double>(rows * pr->N);
    }
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
    if (b.pos != nullptr && rows >= 64 && (reinterpret_cast<uintptr_t>(perm) & 15u) == 0) {
        // W_dp larger than half an XCD's L2 and stages made of 16-byte pieces: rows of W_dp in LDS, by device
        const size_t total = rows * (size_t)N;
        hipLaunchKernelGGL(k_positions, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, perm, N, total, b.pos);
        DTFM_HIP(hipGetLastError());
        hipLaunchKernelGGL(k_datap_rows, dim3((unsigned)(N / DTFM_DATAP_DPW * DTFM_DATAP_SPLIT)), dim3(256),
                           (size_t)DTFM_DATAP_DPW * N * sizeof(double), st, pr->W_dp, perm, b.pos, N, pr->D_dp, rows, b.rowsum);
        DTFM_HIP(hipGetLastError());
        hipLaunchKernelGGL(k_datap_reduce, dim3((unsigned)rows), dim3(256), 0, st, b.rowsum, N, n, b.datap, b.ghat);
    } else if ((size_t)N * N * sizeof(double) > ((size_t)2 << 20) && N % DTFM_XCDS == 0) {
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
        // trial rows that differ from their current rows inside one stage only (inc_j = inc_jp) keep every edge
        const int match_pairs = inc_j >= 0 ? (inc_j == inc_jp ? 0 : 2 * n - 3) : pr->npairs;
        const int nb = (pr->D_dp + 15) / 16;
        if (rows > 0x7fffffffu) return DTFM_ERR_ARG;
        if (match_pairs > 0) {
        auto kern = nb <= 1 ? k_match<1> : nb == 2 ? k_match<2> : nb == 3 ? k_match<3> : k_match<4>;
        // one wavefront per (candidate, stage pair)
        hipLaunchKernelGGL(kern, dim3((unsigned)rows, (unsigned)match_pairs), dim3(DTFM_WAVE),
                           (size_t)16 * nb * DTFM_WAVE * sizeof(uint16_t), st, pr->W_code, pr->W_rank, pr->rank_val, pr->rank_shift, perm, N, pr->D_dp, n,
                           b.ghat, inc_j, inc_jp);
        DTFM_HIP(hipGetLastError());
        }
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
        // rows, Ghat, and the low parts in layer order with two more turns of entries behind them (read ahead, never used)
        size_t lds = ((size_t)(DTFM_HK_ROW_STRIDE << NL) + 256) * sizeof(double) + sizeof(uint32_t) * (((size_t)1 << NL) + 2 * (((size_t)1 << NL) / 16));
        auto kern = n <= 12 ? k_held_karp_blocked<NL, 6> : n <= 14 ? k_held_karp_blocked<NL, 7> : k_held_karp_blocked<NL, 8>;
        DTFM_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                     (int)lds));
        hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(1 << NL), lds, st, b.ghat, b.datap, n, b.hk_tab, cost, rows, list,
                           count, b.pp);
    }
    DTFM_HIP(hipGetLastError());
    return DTFM_OK;
}
