// Fused population-evaluation kernel for the 64-device shape (N = 64, D_dp = 8, D_pp = 8): one
// wavefront evaluates four candidates end to end (Eqs. 1-4).
//
//   Matching (Eq. 3)   The bottleneck value of a block depends only on the ORDER of its entries,
//                      so the kernel works on 16-bit ranks of W_pp (rank table in LDS, built once
//                      per problem) and maps the winning rank back to its fp64 weight at the end:
//                      bit-identical to working on the doubles. Per stage pair a min-max dynamic
//                      programme over column subsets, row by row:
//                          g[S] = min_{c in S} max(g[S \ c], w[|S|-1][c]),   g[all] = optimum.
//                      Lane = (candidate 0..3, couple of stage pairs 0..13): two pairs packed in
//                      one 32-bit register, 16-bit packed max/min. Every lane walks the subsets in
//                      the same order, so the whole table lives in registers with compile-time
//                      indices: no table traffic, no index arithmetic, 2 ALU ops per transition.
//   Held-Karp (Eq. 4)  per candidate, fp64 table [v][S] in LDS, one lane per (S, v) item, layers
//                      of equal |S|; which item a lane owns in each step is fixed and comes from a
//                      small table built with the problem (held in registers).
//   DataP (Eq. 2)      lane = position; 8 gathers of W_dp (L2-resident 32 KiB table) summed in
//                      slot order (the device's own slot adds the zero diagonal), wave max.
#include "dtfm_internal.h"

#include <math.h>

#include <utility>
#include <vector>

namespace {

constexpr int NDEV = 64, CANDS = 4;   // candidates per wavefront pass
constexpr int BINOM8[9] = {1, 8, 28, 56, 70, 56, 28, 8, 1};

// the subsets of {0..7} grouped by size: LAYER.s[k][i] = i-th subset with k elements, ascending
struct layer_table {
    unsigned char s[9][70];
};
constexpr layer_table make_layers()
{
    layer_table t = {};
    for (int k = 0; k <= 8; k++) {
        int n = 0;
        for (int S = 0; S < 256; S++) {
            int pc = 0;
            for (int b = 0; b < 8; b++) pc += (S >> b) & 1;
            if (pc == k) t.s[k][n++] = (unsigned char)S;
        }
    }
    return t;
}
constexpr layer_table LAYER = make_layers();

constexpr int hk_steps(int k) { return (BINOM8[k] * k + 63) / 64; }
constexpr int hk_first(int k)
{
    int o = 0;
    for (int i = 2; i < k; i++) o += hk_steps(i);
    return o;
}
constexpr int N_HSTEP = hk_first(9);   // 19

// LDS: shared rank table, then one slice per wavefront
constexpr int LDS_RANK_BYTES = NDEV * NDEV * 2;        // 8 KiB
constexpr int OFF_HK = 0;                              // fp64 [8 end nodes][256 subsets]   16 KiB
constexpr int OFF_GHAT = 16384;                        // fp64 [4 candidates][8][8]          2 KiB
constexpr int OFF_PB = OFF_GHAT + CANDS * 512;         // u8 [4 candidates][64] perm, stage-major
constexpr int WAVE_LDS_BYTES = OFF_PB + CANDS * 64;    // 18688
constexpr int WAVES_PER_BLOCK = 8;
constexpr int LDS_TOTAL = LDS_RANK_BYTES + WAVES_PER_BLOCK * WAVE_LDS_BYTES;   // 157696 <= 160 KiB

typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pk_max(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(u16x2, a),
                                                                  __builtin_bit_cast(u16x2, b)));
}
__device__ __forceinline__ uint32_t pk_min(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_min(__builtin_bit_cast(u16x2, a),
                                                                  __builtin_bit_cast(u16x2, b)));
}

// Orders this wavefront's earlier LDS writes before its later LDS reads as seen by other lanes.
// The LDS unit serves one wavefront's requests in order; this only stops the compiler from moving
// accesses across the point.
#define WAVE_LDS_SYNC()                                         \
    do {                                                        \
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");  \
        __builtin_amdgcn_wave_barrier();                        \
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");  \
    } while (0)

struct hk_consts {
    uint32_t nib[N_HSTEP], a[N_HSTEP], b[N_HSTEP];
};

// One layer of Held-Karp: every lane owns (S, v) items with |S| = K. ghat_off: byte offset of this
// candidate's coarsened graph inside the wavefront's LDS slice.
template <int K>
__device__ __forceinline__ void hk_layer(unsigned char *wl, const hk_consts &hc, uint32_t ghat_off)
{
#pragma unroll
    for (int s = 0; s < hk_steps(K); s++) {
        const uint32_t nib = hc.nib[hk_first(K) + s], a = hc.a[hk_first(K) + s], b = hc.b[hk_first(K) + s];
        const uint32_t rest8 = a & 0xFFFFu;            // byte offset of tab[0][S \ v]
        const uint32_t gcol = (a >> 16) + ghat_off;    // byte offset of ghat[0][v]
        double best = INFINITY;
#pragma unroll
        for (int t = 0; t < K - 1; t++) {
            const uint32_t u = (nib >> (4 * t)) & 15u;
            const double x = *reinterpret_cast<const double *>(wl + OFF_HK + rest8 + u * 2048u);
            const double e = *reinterpret_cast<const double *>(wl + gcol + u * 64u);
            best = fmin(best, __dadd_rn(x, e));
        }
        if (b >> 31) *reinterpret_cast<double *>(wl + OFF_HK + (b & 0xFFFFu)) = best;
        __builtin_amdgcn_sched_barrier(0);   // keep one step's loads in flight, not the whole layer's
    }
    WAVE_LDS_SYNC();
}

// byte k (0..7) of a 64-bit value held as two dwords
__device__ __forceinline__ uint32_t byte_of(uint2 v, int k) { return ((k < 4 ? v.x : v.y) >> (8 * (k & 3))) & 0xFFu; }

__global__ void __launch_bounds__(WAVES_PER_BLOCK * 64)
k_eval_fast64(const double *__restrict__ W_dp, const uint16_t *__restrict__ rank_tab,
              const double *__restrict__ rank_val, const uint32_t *__restrict__ step_tab,
              const int32_t *__restrict__ perm, size_t P, double *__restrict__ cost,
              double *__restrict__ ghat_out, double *__restrict__ datap_out)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint16_t *R = reinterpret_cast<const uint16_t *>(smem);
    unsigned char *wl = smem + LDS_RANK_BYTES + wave * WAVE_LDS_BYTES;

    // rank table -> LDS (8 KiB, 16 bytes per thread per pass)
    for (int i = threadIdx.x; i < LDS_RANK_BYTES / 16; i += blockDim.x)
        reinterpret_cast<uint4 *>(smem)[i] = reinterpret_cast<const uint4 *>(rank_tab)[i];
    // zero diagonals of the four coarsened graphs (never overwritten)
    if (lane < CANDS * 8) *reinterpret_cast<double *>(wl + OFF_GHAT + (lane >> 3) * 512 + (lane & 7) * 72) = 0.0;
    // matching role of this lane: candidate slot and the couple of stage pairs (2q, 2q+1) in
    // lexicographic pair order; lanes with q = 14, 15 repeat couple 13 and write nothing
    const int mc = lane >> 4, q = (lane & 15) < 14 ? (lane & 15) : 13;
    const bool couple_valid = (lane & 15) < 14;
    int j1[2], j2[2];
#pragma unroll
    for (int h = 0; h < 2; h++) {
        int t = 2 * q + h, a = 0;
        while (t >= 7 - a) {
            t -= 7 - a;
            a++;
        }
        j1[h] = a;
        j2[h] = a + 1 + t;
    }
    __syncthreads();

    const size_t nwaves = (size_t)gridDim.x * WAVES_PER_BLOCK;
    const size_t nquads = (P + CANDS - 1) / CANDS;
    for (size_t quad = (size_t)blockIdx.x * WAVES_PER_BLOCK + wave; quad < nquads; quad += nwaves) {
        // ---- a1: four candidate rows; position = lane: stage = lane / 8, slot = lane % 8 ----
        int dev[CANDS];
#pragma unroll
        for (int c = 0; c < CANDS; c++) {
            size_t cand = quad * CANDS + c;
            if (cand >= P) cand = P - 1;   // ragged tail: recompute the last row, never stored
            dev[c] = perm[cand * NDEV + lane];
            wl[OFF_PB + c * 64 + lane] = (unsigned char)dev[c];
        }
        WAVE_LDS_SYNC();

        // ---- a4: bottleneck matchings of this lane's two stage pairs, as ranks ----
        uint32_t gfull;
        {
            const unsigned char *pb = wl + OFF_PB + mc * 64;
            uint2 rowdev[2], coldev[2];
            uint32_t coloff[2][8];
#pragma unroll
            for (int h = 0; h < 2; h++) {
                rowdev[h] = *reinterpret_cast<const uint2 *>(pb + 8 * j1[h]);   // devices of stage j1, slots 0..7
                coldev[h] = *reinterpret_cast<const uint2 *>(pb + 8 * j2[h]);   // devices of stage j2
#pragma unroll
                for (int c = 0; c < 8; c++) coloff[h][c] = byte_of(coldev[h], c);
            }
            uint32_t G[256];
            // rows are gathered one layer ahead of their use; the scheduling barriers keep the
            // register footprint to two rows plus two layers of the table
            uint32_t wnext[8];
            {
                const uint32_t rb0 = byte_of(rowdev[0], 0) * NDEV, rb1 = byte_of(rowdev[1], 0) * NDEV;
#pragma unroll
                for (int c = 0; c < 8; c++)
                    wnext[c] = (uint32_t)R[rb0 + coloff[0][c]] | ((uint32_t)R[rb1 + coloff[1][c]] << 16);
            }
#pragma unroll
            for (int r = 0; r < 8; r++) {
                // row r of both blocks: w[c] = (rank of pair-0 entry (r,c)) | (rank of pair-1 entry) << 16
                uint32_t w[8];
#pragma unroll
                for (int c = 0; c < 8; c++) w[c] = wnext[c];
                if (r < 7) {
                    const uint32_t rb0 = byte_of(rowdev[0], r + 1) * NDEV, rb1 = byte_of(rowdev[1], r + 1) * NDEV;
#pragma unroll
                    for (int c = 0; c < 8; c++)
                        wnext[c] = (uint32_t)R[rb0 + coloff[0][c]] | ((uint32_t)R[rb1 + coloff[1][c]] << 16);
                }
#pragma unroll
                for (int i = 0; i < BINOM8[r + 1]; i++) {
                    const int S = LAYER.s[r + 1][i];
                    uint32_t acc = 0;
                    bool first = true;
#pragma unroll
                    for (int c = 0; c < 8; c++) {
                        if (!(S & (1 << c))) continue;
                        const uint32_t m = (r == 0) ? w[c] : pk_max(G[S ^ (1 << c)], w[c]);
                        acc = first ? m : pk_min(acc, m);
                        first = false;
                    }
                    G[S] = acc;
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            gfull = G[255];
        }
        // ---- winning ranks -> fp64 weights -> coarsened graphs in LDS ----
        {
            const double e0 = rank_val[gfull & 0xFFFFu], e1 = rank_val[gfull >> 16];
            if (couple_valid) {
                double *gh = reinterpret_cast<double *>(wl + OFF_GHAT + mc * 512);
                gh[j1[0] * 8 + j2[0]] = e0;
                gh[j2[0] * 8 + j1[0]] = e0;
                gh[j1[1] * 8 + j2[1]] = e1;
                gh[j2[1] * 8 + j1[1]] = e1;
            }
        }
        WAVE_LDS_SYNC();

        // per-lane Held-Karp item tables (L2-resident, reloaded per pass so that they do not occupy
        // registers during the matching programme; the asm keeps the loads from being hoisted)
        hk_consts hc;
        {
            const uint32_t *st = step_tab;
            asm volatile("" : "+s"(st));
#pragma unroll
            for (int i = 0; i < N_HSTEP; i++) {
                hc.nib[i] = st[(0 * N_HSTEP + i) * 64 + lane];
                hc.a[i] = st[(1 * N_HSTEP + i) * 64 + lane];
                hc.b[i] = st[(2 * N_HSTEP + i) * 64 + lane];
            }
        }
        // ---- per candidate: a5 Held-Karp, a2/a3 DataP, a6 total ----
#pragma nounroll
        for (int c = 0; c < CANDS; c++) {
            // hide the tables' loop invariance: addresses derived from them must not be hoisted
#pragma unroll
            for (int i = 0; i < N_HSTEP; i++) {
                asm volatile("" : "+v"(hc.nib[i]));
                asm volatile("" : "+v"(hc.a[i]));
                asm volatile("" : "+v"(hc.b[i]));
            }
            const size_t cand = quad * CANDS + c;
            const bool live = cand < P;   // wave-uniform
            const int d = c == 0 ? dev[0] : c == 1 ? dev[1] : c == 2 ? dev[2] : dev[3];
            // DataP gathers first: their latency hides behind Held-Karp
            const uint2 mates = *reinterpret_cast<const uint2 *>(wl + OFF_PB + c * 64 + (lane & ~7));
            const double *wrow = W_dp + d * NDEV;
            double wv[8];
#pragma unroll
            for (int k = 0; k < 8; k++) wv[k] = wrow[byte_of(mates, k)];   // own slot: the zero diagonal
            const uint32_t ghat_off = OFF_GHAT + c * 512;
            if (ghat_out != nullptr && live)
                ghat_out[cand * 64 + lane] = *reinterpret_cast<const double *>(wl + ghat_off + lane * 8);

            if (lane < 8) *reinterpret_cast<double *>(wl + OFF_HK + (lane * 256 + (1 << lane)) * 8) = 0.0;
            WAVE_LDS_SYNC();
            hk_layer<2>(wl, hc, ghat_off);
            hk_layer<3>(wl, hc, ghat_off);
            hk_layer<4>(wl, hc, ghat_off);
            hk_layer<5>(wl, hc, ghat_off);
            hk_layer<6>(wl, hc, ghat_off);
            hk_layer<7>(wl, hc, ghat_off);
            hk_layer<8>(wl, hc, ghat_off);
            double pp = *reinterpret_cast<const double *>(wl + OFF_HK + ((lane & 7) * 256 + 255) * 8);
            pp = fmin(pp, __shfl_xor(pp, 1));
            pp = fmin(pp, __shfl_xor(pp, 2));
            pp = fmin(pp, __shfl_xor(pp, 4));

            double sum = 0.0;
#pragma unroll
            for (int k = 0; k < 8; k++) sum = __dadd_rn(sum, wv[k]);
#pragma unroll
            for (int o = 32; o >= 1; o >>= 1) sum = fmax(sum, __shfl_xor(sum, o));
            if (lane == 0 && live) {
                if (cost != nullptr) cost[cand] = __dadd_rn(sum, pp);
                if (datap_out != nullptr) datap_out[cand] = sum;
            }
            WAVE_LDS_SYNC();   // the next candidate reuses the table
        }
    }
}

// rank of every W_pp entry among all off-diagonal entries (number of strictly smaller ones): equal
// weights get equal ranks, the order is preserved, and N*N <= 4096 values fit 16 bits. rank_val
// maps a rank back to the weight.
__global__ void k_rank_weights(const double *__restrict__ W_pp, int N, uint16_t *__restrict__ rank_tab,
                               double *__restrict__ rank_val)
{
    int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= N * N) return;
    int d = idx / N, e = idx - d * N;
    if (d == e) {
        rank_tab[idx] = 0;
        return;
    }
    double w = W_pp[idx];
    int r = 0;
    for (int i = 0; i < N * N; i++) {
        int x = i / N, y = i - x * N;
        r += (x != y && W_pp[i] < w) ? 1 : 0;
    }
    rank_tab[idx] = (uint16_t)r;
    rank_val[r] = w;   // equal weights write equal bits
}

}  // namespace

bool dtfm_fast64_applicable(const dtfm_problem *pr) { return pr->N == 64 && pr->D_dp == 8 && pr->D_pp == 8; }

// Builds the rank tables and the per-lane Held-Karp item tables of a 64-device problem.
int dtfm_fast64_prepare(dtfm_problem *pr)
{
    const int N = pr->N;
    DTFM_HIP(hipMalloc((void **)&pr->f64_rank, (size_t)N * N * sizeof(uint16_t)));
    DTFM_HIP(hipMalloc((void **)&pr->f64_rank_val, (size_t)N * N * sizeof(double)));
    DTFM_HIP(hipMemset(pr->f64_rank_val, 0, (size_t)N * N * sizeof(double)));
    hipLaunchKernelGGL(k_rank_weights, dim3((N * N + 255) / 256), dim3(256), 0, (hipStream_t) nullptr, pr->W_pp, N,
                       pr->f64_rank, pr->f64_rank_val);
    DTFM_HIP(hipGetLastError());

    std::vector<uint32_t> tab((size_t)(3 * N_HSTEP) * 64, 0u);
    uint32_t *h_nib = tab.data(), *h_a = h_nib + N_HSTEP * 64, *h_b = h_a + N_HSTEP * 64;
    int hs = 0;
    for (int k = 2; k <= 8; k++) {
        // Held-Karp items of layer k: (subset, end node v in it), subsets ascending, v ascending
        std::vector<std::pair<uint32_t, int>> items;
        for (uint32_t S = 1; S < 256; S++)
            if (__builtin_popcount(S) == k)
                for (int v = 0; v < 8; v++)
                    if (S & (1u << v)) items.push_back({S, v});
        for (int s = 0; s < hk_steps(k); s++, hs++)
            for (int lane = 0; lane < 64; lane++) {
                int i = s * 64 + lane;
                if (i >= (int)items.size()) continue;
                uint32_t S = items[i].first, v = items[i].second, rest = S ^ (1u << v), nib = 0;
                int t = 0;
                for (int u = 0; u < 8; u++)
                    if (rest & (1u << u)) nib |= (uint32_t)u << (4 * t++);
                h_nib[hs * 64 + lane] = nib;
                h_a[hs * 64 + lane] = (rest * 8) | ((v * 8) << 16);
                h_b[hs * 64 + lane] = ((v * 256 + S) * 8) | 0x80000000u;
            }
    }
    DTFM_HIP(hipMalloc((void **)&pr->f64_steps, tab.size() * sizeof(uint32_t)));
    DTFM_HIP(hipMemcpy(pr->f64_steps, tab.data(), tab.size() * sizeof(uint32_t), hipMemcpyHostToDevice));
    DTFM_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_eval_fast64),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, LDS_TOTAL));
    hipDeviceProp_t prop;
    DTFM_HIP(hipGetDeviceProperties(&prop, pr->device));
    pr->f64_grid = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    DTFM_HIP(hipDeviceSynchronize());
    return DTFM_OK;
}

void dtfm_fast64_release(dtfm_problem *pr)
{
    if (pr->f64_rank) (void)hipFree(pr->f64_rank);
    if (pr->f64_rank_val) (void)hipFree(pr->f64_rank_val);
    if (pr->f64_steps) (void)hipFree(pr->f64_steps);
}

int dtfm_fast64_enqueue(const dtfm_problem *pr, const int32_t *perm, size_t rows, double *cost, double *ghat,
                        double *datap, hipStream_t st)
{
    if (rows == 0) return DTFM_OK;
    size_t quads = (rows + CANDS - 1) / CANDS;
    size_t blocks = (quads + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK;
    if (blocks > (size_t)pr->f64_grid) blocks = pr->f64_grid;
    hipLaunchKernelGGL(k_eval_fast64, dim3((unsigned)blocks), dim3(WAVES_PER_BLOCK * 64), LDS_TOTAL, st, pr->W_dp,
                       pr->f64_rank, pr->f64_rank_val, pr->f64_steps, perm, rows, cost, ghat, datap);
    DTFM_HIP(hipGetLastError());
    return DTFM_OK;
}
