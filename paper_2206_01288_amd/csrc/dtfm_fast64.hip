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
//   Held-Karp (Eq. 4)  two candidates at a time, their fp64 values side by side in 128-bit LDS
//                      entries; one lane per (S, v) item, layers of equal |S| kept in two
//                      alternating compact buffers. Which item a lane owns in each step, and the
//                      byte offsets of the entries it reads, are fixed: they come from a table built
//                      once (LDS-resident) whose slot assignment avoids LDS bank conflicts.
//   DataP (Eq. 2)      lane = position; 8 gathers of W_dp (L2-resident 32 KiB table) summed in
//                      slot order (the device's own slot adds the zero diagonal), wave max.
#include "dtfm_internal.h"

#include <math.h>

#include <mutex>
#include <utility>
#include <vector>

namespace {

constexpr int NDEV = 64, CANDS = 4;   // most candidates per wavefront pass (kernels are built for 4 and 2)
// Row stride of the rank table in LDS, in 16-bit entries. 66 instead of 64 skews consecutive rows by
// one 4-byte bank, so that lanes reading the same column of different rows hit different banks.
constexpr int RSTRIDE = 66;
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

constexpr int hk_steps(int k) { return (BINOM8[k] * k + 63) / 64; }    // 64-lane steps of layer k
constexpr int hk_words4(int k) { return (k + 3) / 4; }                 // 128-bit table words per item
constexpr int hk_tab_first(int k)                                       // first table word of layer k
{
    int o = 0;
    for (int i = 2; i < k; i++) o += hk_steps(i) * hk_words4(i);
    return o;
}
constexpr int HK_TAB_WORDS4 = hk_tab_first(9);          // 29 (x 64 lanes x 16 B = 29696 B)
constexpr int HK_BUF_ENTRIES = 5 * 64;                  // largest layer: 5 steps of 64 lanes

// LDS: rank table and Held-Karp item table shared by the workgroup, then one slice per wavefront
constexpr int LDS_RANK_BYTES = ((NDEV * RSTRIDE * 2 + 15) / 16) * 16;   // 8.25 KiB
constexpr int LDS_HKTAB_BYTES = HK_TAB_WORDS4 * 64 * 16;           // 29 KiB
constexpr int OFF_BUF0 = 0;                                        // double2 [320]: even layers
constexpr int OFF_BUF1 = OFF_BUF0 + HK_BUF_ENTRIES * 16;           // double2 [320]: odd layers
// Coarsened graphs, one 2 KiB block per candidate pair: double2 [u][16]: column s of row u holds
// ghat[u][s % 8] (both candidates), so a lane of pass-lane s whose item ends in v = s % 8 always reads
// its own column: the 16 lanes of a 128-bit read pass never share a bank group.
constexpr int GHAT_PAIR_BYTES = 8 * 16 * 16;
constexpr int OFF_GHAT = OFF_BUF1 + HK_BUF_ENTRIES * 16;
constexpr int OFF_PB = OFF_GHAT + 2 * GHAT_PAIR_BYTES;             // u8 [4 candidates][64] perm, stage-major
constexpr int OFF_PBCUR = OFF_PB + CANDS * 64;                     // u8 [4][64]: current rows (local search)
constexpr int WAVE_LDS_BYTES = OFF_PBCUR + CANDS * 64;             // 14848
constexpr int WAVES_PER_BLOCK = 8;
constexpr int LDS_TOTAL = LDS_RANK_BYTES + LDS_HKTAB_BYTES + WAVES_PER_BLOCK * WAVE_LDS_BYTES;

typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) u32x4 lds_u32x4;   // explicitly LDS-qualified

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

// One layer of Held-Karp for a pair of candidates: every lane owns (S, v) items with |S| = K.
// Item table (128-bit words, lane-major): word 0 = byte offset of the item's own entry in this
// layer's buffer | valid << 31; words 1..K-1 = one per predecessor u in S \ v:
// (byte offset of tab[S \ v][u] in the previous layer's buffer) | (byte offset of ghat[u][v]) << 16.
template <int K>
__device__ __forceinline__ double2 hk_layer(unsigned char *wl, const unsigned char *hktab, uint32_t ghat_off,
                                            int lane)
{
    constexpr int PREV = (K & 1) ? OFF_BUF0 : OFF_BUF1, CUR = (K & 1) ? OFF_BUF1 : OFF_BUF0;
    constexpr int STEPS = hk_steps(K), W4 = hk_words4(K);
    // all item words of the layer first, then all reads and arithmetic, then all writes: with no
    // store between the loads of different steps the compiler may overlap their LDS latencies
    uint32_t word[STEPS][4 * W4];
#pragma unroll
    for (int s = 0; s < STEPS; s++)
#pragma unroll
        for (int i = 0; i < W4; i++) {
            // volatile: keep this one dense 128-bit read per lane (the compiler would otherwise narrow
            // it to the words actually used, which at a 16-byte lane stride conflicts heavily)
            const u32x4 t = *(const volatile lds_u32x4 *)(hktab + ((hk_tab_first(K) + s * W4 + i) * 64 + lane) * 16);
            word[s][4 * i + 0] = t.x;
            word[s][4 * i + 1] = t.y;
            word[s][4 * i + 2] = t.z;
            word[s][4 * i + 3] = t.w;
        }
    double2 best[STEPS];
#pragma unroll
    for (int s = 0; s < STEPS; s++) {
        best[s] = make_double2(INFINITY, INFINITY);
#pragma unroll
        for (int t = 1; t < K; t++) {
            const double2 x = *reinterpret_cast<const double2 *>(wl + PREV + (word[s][t] & 0xFFFFu));
            const double2 e = *reinterpret_cast<const double2 *>(wl + ghat_off + (word[s][t] >> 16));
            best[s].x = fmin(best[s].x, __dadd_rn(x.x, e.x));
            best[s].y = fmin(best[s].y, __dadd_rn(x.y, e.y));
        }
    }
#pragma unroll
    for (int s = 0; s < STEPS; s++) {
        if (word[s][0] >> 31) *reinterpret_cast<double2 *>(wl + CUR + (word[s][0] & 0xFFFFu)) = best[s];
        else best[s] = make_double2(INFINITY, INFINITY);
    }
    WAVE_LDS_SYNC();
    return best[STEPS - 1];
}

// byte k (0..7) of a 64-bit value held as two dwords
__device__ __forceinline__ uint32_t byte_of(uint2 v, int k) { return ((k < 4 ? v.x : v.y) >> (8 * (k & 3))) & 0xFFu; }

// Per-wavefront context: LDS pointers and the lane's fixed role in the matching programme.
struct wave_ctx {
    unsigned char *wl;            // this wavefront's LDS slice
    const uint16_t *R;            // rank table (LDS)
    const unsigned char *hktab;   // Held-Karp item table (LDS)
    int lane;
    int mc;                       // candidate slot 0..3 whose matchings this lane computes
    bool couple_valid;            // lanes 14, 15 of each 16 repeat couple 13 and write nothing
    int j1[2], j2[2];             // the lane's two stage pairs (j1 < j2)
};

// Loads the workgroup's tables into LDS and derives the lane roles. Ends with a workgroup barrier.
template <int NC>
__device__ __forceinline__ wave_ctx wave_setup(unsigned char *smem, const uint16_t *rank_tab, const uint32_t *step_tab)
{
    wave_ctx cx;
    cx.lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    cx.R = reinterpret_cast<const uint16_t *>(smem);
    cx.hktab = smem + LDS_RANK_BYTES;
    cx.wl = smem + LDS_RANK_BYTES + LDS_HKTAB_BYTES + wave * WAVE_LDS_BYTES;
    // rank table -> LDS, rows re-strided (two entries per thread per pass)
    for (int i = threadIdx.x; i < NDEV * NDEV / 2; i += blockDim.x) {
        const int row = i / (NDEV / 2), col2 = i - row * (NDEV / 2);
        reinterpret_cast<uint32_t *>(smem)[row * (RSTRIDE / 2) + col2] = reinterpret_cast<const uint32_t *>(rank_tab)[i];
    }
    // Held-Karp item table -> LDS
    for (int i = threadIdx.x; i < LDS_HKTAB_BYTES / 16; i += blockDim.x)
        reinterpret_cast<uint4 *>(smem + LDS_RANK_BYTES)[i] = reinterpret_cast<const uint4 *>(step_tab)[i];
    // zero diagonals of the four coarsened graphs (never overwritten): [pair][j][column j][cand & 1]
    if (cx.lane < CANDS * 8)
        *reinterpret_cast<double *>(cx.wl + OFF_GHAT + (cx.lane >> 4) * GHAT_PAIR_BYTES +
                                    ((cx.lane & 7) * 16 + (cx.lane & 7)) * 16 + ((cx.lane >> 3) & 1) * 8) = 0.0;
    // matching role: candidate slot and the couple of stage pairs (2q, 2q+1) in lexicographic order
    // (with NC = 2 the upper half of the wavefront repeats the lower half's work and writes nothing)
    cx.mc = (cx.lane >> 4) % NC;
    const int q = (cx.lane & 15) < 14 ? (cx.lane & 15) : 13;
    cx.couple_valid = (cx.lane & 15) < 14 && cx.lane < NC * 16;
#pragma unroll
    for (int h = 0; h < 2; h++) {
        int t = 2 * q + h, a = 0;
        while (t >= 7 - a) {
            t -= 7 - a;
            a++;
        }
        cx.j1[h] = a;
        cx.j2[h] = a + 1 + t;
    }
    __syncthreads();
    return cx;
}

// Evaluates the NC (4 or 2) candidates whose rows are in the wavefront's LDS slice at OFF_PB (stage-major
// bytes, already visible to all lanes); dev[c] = device at position `lane` of candidate c.
// On return total[c] (Eq. 1) and datap[c] (Eq. 2 + max) are held by every lane. ghat_out, if not
// null, receives the coarsened graphs of candidates cand0 .. cand0+3 that are < P.
template <int NC>
__device__ __forceinline__ void eval_quad(const wave_ctx &cx, const double *__restrict__ W_dp,
                                          const double *__restrict__ rank_val, const int (&dev)[CANDS],
                                          double (&total)[CANDS], double (&datap)[CANDS],
                                          double *__restrict__ ghat_out, size_t cand0, size_t P)
{
    unsigned char *wl = cx.wl;
    const uint16_t *R = cx.R;
    const int lane = cx.lane;
    // ---- a4: bottleneck matchings of this lane's two stage pairs, as ranks ----
    uint32_t gfull;
    {
        const unsigned char *pb = wl + OFF_PB + cx.mc * 64;
        uint2 rowdev[2], coldev[2];
        uint32_t coloff[2][8];
#pragma unroll
        for (int h = 0; h < 2; h++) {
            rowdev[h] = *reinterpret_cast<const uint2 *>(pb + 8 * cx.j1[h]);   // devices of stage j1, slots 0..7
            coldev[h] = *reinterpret_cast<const uint2 *>(pb + 8 * cx.j2[h]);   // devices of stage j2
#pragma unroll
            for (int c = 0; c < 8; c++) coloff[h][c] = byte_of(coldev[h], c);
        }
        uint32_t G[256];
        // rows are gathered one layer ahead of their use; the scheduling barriers keep the
        // register footprint to two rows plus two layers of the table
        uint32_t wnext[8];
        {
            const uint32_t rb0 = byte_of(rowdev[0], 0) * RSTRIDE, rb1 = byte_of(rowdev[1], 0) * RSTRIDE;
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
                const uint32_t rb0 = byte_of(rowdev[0], r + 1) * RSTRIDE, rb1 = byte_of(rowdev[1], r + 1) * RSTRIDE;
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
        if (cx.couple_valid) {   // entries [candidate pair][u][columns v and v + 8][candidate & 1]
            double *gh = reinterpret_cast<double *>(wl + OFF_GHAT + (cx.mc >> 1) * GHAT_PAIR_BYTES) + (cx.mc & 1);
#pragma unroll
            for (int h = 0; h < 2; h++) {
                const double e = h == 0 ? e0 : e1;
                const int a = cx.j1[h], b = cx.j2[h];
                gh[(a * 16 + b) * 2] = e;
                gh[(a * 16 + b + 8) * 2] = e;
                gh[(b * 16 + a) * 2] = e;
                gh[(b * 16 + a + 8) * 2] = e;
            }
        }
    }
    WAVE_LDS_SYNC();

    // ---- per candidate pair: a5 Held-Karp, a2/a3 DataP, a6 total ----
#pragma nounroll
    for (int pr = 0; pr < NC / 2; pr++) {
        // DataP gathers first: their latency hides behind Held-Karp
        double wv[2][8];
#pragma unroll
        for (int h = 0; h < 2; h++) {
            const int d = pr == 0 ? dev[h] : dev[2 + h];
            const uint2 mates = *reinterpret_cast<const uint2 *>(wl + OFF_PB + (2 * pr + h) * 64 + (lane & ~7));
            const double *wrow = W_dp + d * NDEV;
#pragma unroll
            for (int k = 0; k < 8; k++) wv[h][k] = wrow[byte_of(mates, k)];   // own slot: the zero diagonal
        }
        const uint32_t ghat_off = OFF_GHAT + pr * GHAT_PAIR_BYTES;
        if (ghat_out != nullptr) {
            const double2 g2 = *reinterpret_cast<const double2 *>(wl + ghat_off + ((lane >> 3) * 16 + (lane & 7)) * 16);
            if (cand0 + 2 * pr < P) ghat_out[(cand0 + 2 * pr) * 64 + lane] = g2.x;
            if (cand0 + 2 * pr + 1 < P) ghat_out[(cand0 + 2 * pr + 1) * 64 + lane] = g2.y;
        }
        // layer 1: tab[{v}][v] = 0, kept twice (entries v and v + 8 of the odd buffer)
        if (lane < 16) *reinterpret_cast<double2 *>(wl + OFF_BUF1 + lane * 16) = make_double2(0.0, 0.0);
        WAVE_LDS_SYNC();
        hk_layer<2>(wl, cx.hktab, ghat_off, lane);
        hk_layer<3>(wl, cx.hktab, ghat_off, lane);
        hk_layer<4>(wl, cx.hktab, ghat_off, lane);
        hk_layer<5>(wl, cx.hktab, ghat_off, lane);
        hk_layer<6>(wl, cx.hktab, ghat_off, lane);
        hk_layer<7>(wl, cx.hktab, ghat_off, lane);
        // the 8 items of the last layer sit in lanes 0..7 (others hold +inf): PP = min over them
        double2 pp = hk_layer<8>(wl, cx.hktab, ghat_off, lane);
#pragma unroll
        for (int o = 1; o <= 4; o <<= 1) {
            pp.x = fmin(pp.x, __shfl_xor(pp.x, o));
            pp.y = fmin(pp.y, __shfl_xor(pp.y, o));
        }
        pp.x = __shfl(pp.x, 0);
        pp.y = __shfl(pp.y, 0);
        double res[2], dpv[2];
#pragma unroll
        for (int h = 0; h < 2; h++) {
            double sum = 0.0;
#pragma unroll
            for (int k = 0; k < 8; k++) sum = __dadd_rn(sum, wv[h][k]);
#pragma unroll
            for (int o = 32; o >= 1; o >>= 1) sum = fmax(sum, __shfl_xor(sum, o));
            dpv[h] = sum;
            res[h] = __dadd_rn(sum, h == 0 ? pp.x : pp.y);
        }
        if (pr == 0) {
            total[0] = res[0]; total[1] = res[1]; datap[0] = dpv[0]; datap[1] = dpv[1];
            if (NC == 2) { total[2] = total[3] = datap[2] = datap[3] = 0.0; }
        } else {
            total[2] = res[0]; total[3] = res[1]; datap[2] = dpv[0]; datap[3] = dpv[1];
        }
        WAVE_LDS_SYNC();   // the next pair reuses the buffers
    }
}

template <int NC>
__global__ void __launch_bounds__(WAVES_PER_BLOCK * 64)
k_eval_fast64(const double *__restrict__ W_dp, const uint16_t *__restrict__ rank_tab,
              const double *__restrict__ rank_val, const uint32_t *__restrict__ step_tab,
              const int32_t *__restrict__ perm, size_t P, double *__restrict__ cost,
              double *__restrict__ ghat_out, double *__restrict__ datap_out)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const wave_ctx cx = wave_setup<NC>(smem, rank_tab, step_tab);
    const int lane = cx.lane, wave = threadIdx.x >> 6;
    const size_t nwaves = (size_t)gridDim.x * WAVES_PER_BLOCK;
    const size_t nquads = (P + NC - 1) / NC;
    for (size_t quad = (size_t)blockIdx.x * WAVES_PER_BLOCK + wave; quad < nquads; quad += nwaves) {
        // ---- a1: NC candidate rows; position = lane: stage = lane / 8, slot = lane % 8 ----
        int dev[CANDS] = {0, 0, 0, 0};
#pragma unroll
        for (int c = 0; c < NC; c++) {
            size_t cand = quad * NC + c;
            if (cand >= P) cand = P - 1;   // ragged tail: recompute the last row, never stored
            dev[c] = perm[cand * NDEV + lane];
            cx.wl[OFF_PB + c * 64 + lane] = (unsigned char)dev[c];
        }
        WAVE_LDS_SYNC();
        double total[CANDS], datap[CANDS];
        eval_quad<NC>(cx, W_dp, rank_val, dev, total, datap, ghat_out, quad * NC, P);
        if (lane < NC) {
            const size_t cand = quad * NC + lane;
            const double t = lane == 0 ? total[0] : lane == 1 ? total[1] : lane == 2 ? total[2] : total[3];
            const double d = lane == 0 ? datap[0] : lane == 1 ? datap[1] : lane == 2 ? datap[2] : datap[3];
            if (cand < P) {
                if (cost != nullptr) cost[cand] = t;
                if (datap_out != nullptr) datap_out[cand] = d;
            }
        }
    }
}

// ---- Sec. 3.4 local search with the paper's four-candidate neighbourhood, all rounds in one launch
// Each wavefront carries its four candidates through every round: propose a swap (fastest link inside
// each of the round's two stages, the four end-point swaps ranked by the paper's Gain), evaluate the
// swapped allocation with eval_quad, keep it iff strictly cheaper. The fastest link is found on the
// ranks (same order and same ties as the weights); the Gain sums use the fp64 weights in slot order.
__device__ __forceinline__ void pair8_decode(int e, int &i, int &k)
{
    int a = 0;
    while (e >= 7 - a) {
        e -= 7 - a;
        a++;
    }
    i = a;
    k = a + 1 + e;
}

template <int NC>
__global__ void __launch_bounds__(WAVES_PER_BLOCK * 64)
k_ls_gain4_fast64(const double *__restrict__ W_dp, const double *__restrict__ W_pp,
                  const uint16_t *__restrict__ rank_tab, const double *__restrict__ rank_val,
                  const uint32_t *__restrict__ step_tab, int32_t *__restrict__ perm, size_t P, int moves,
                  double *__restrict__ cost, int64_t *__restrict__ applied)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const wave_ctx cx = wave_setup<NC>(smem, rank_tab, step_tab);
    const int lane = cx.lane, wave = threadIdx.x >> 6;
    unsigned char *wl = cx.wl;
    const int grp = (lane >> 4) % NC, sub = lane & 15;   // proposal role: 16 lanes per candidate
    const size_t nwaves = (size_t)gridDim.x * WAVES_PER_BLOCK;
    const size_t nquads = (P + NC - 1) / NC;
    for (size_t quad = (size_t)blockIdx.x * WAVES_PER_BLOCK + wave; quad < nquads; quad += nwaves) {
        int cur[CANDS] = {0, 0, 0, 0};   // current allocation: device at position `lane`
        double cur_cost[CANDS], unused[CANDS];
#pragma unroll
        for (int c = 0; c < NC; c++) {
            size_t cand = quad * NC + c;
            if (cand >= P) cand = P - 1;
            cur[c] = perm[cand * NDEV + lane];
            wl[OFF_PB + c * 64 + lane] = (unsigned char)cur[c];
            wl[OFF_PBCUR + c * 64 + lane] = (unsigned char)cur[c];
        }
        WAVE_LDS_SYNC();
        eval_quad<NC>(cx, W_dp, rank_val, cur, cur_cost, unused, nullptr, quad * NC, P);
#pragma nounroll
        for (int r = 0; r < moves; r++) {
            // ---- proposal for candidate `grp` by its 16 lanes ----
            int j, jp;
            {
                int t = r % 28, a = 0;
                while (t >= 7 - a) {
                    t -= 7 - a;
                    a++;
                }
                j = a;
                jp = a + 1 + t;
            }
            const unsigned char *pc = wl + OFF_PBCUR + grp * 64;
            int slot[2][2];
#pragma unroll
            for (int s = 0; s < 2; s++) {
                const unsigned char *C = pc + 8 * (s == 0 ? j : jp);
                uint32_t key = 0xFFFFFFFFu;   // (rank << 8) | pair index: first minimiser wins
#pragma unroll
                for (int e0 = 0; e0 < 32; e0 += 16) {
                    const int e = e0 + sub;
                    if (e < 28) {
                        int i, k;
                        pair8_decode(e, i, k);
                        const uint32_t kk = ((uint32_t)cx.R[(int)C[i] * RSTRIDE + C[k]] << 8) | (uint32_t)e;
                        key = kk < key ? kk : key;
                    }
                }
#pragma unroll
                for (int o = 1; o <= 8; o <<= 1) {
                    const uint32_t ok = __shfl_xor(key, o);
                    key = ok < key ? ok : key;
                }
                pair8_decode((int)(key & 0xFFu), slot[s][0], slot[s][1]);
            }
            const int Cj = 8 * j, Cjp = 8 * jp;
            // lanes 0,1 of the group: mean over C_j' of w[x][.] for x = d1, d2; lanes 2,3: mean over C_j of w[y][.]
            double mean = 0.0;
            {
                const int side = (sub >> 1) & 1;
                const int dv = pc[(side == 0 ? Cj : Cjp) + slot[side][sub & 1]];
                const unsigned char *other = pc + (side == 0 ? Cjp : Cj);
                double sum = 0.0;
                if (sub < 4) {
#pragma unroll
                    for (int i = 0; i < 8; i++) sum = __dadd_rn(sum, W_pp[dv * NDEV + other[i]]);
                }
                mean = __ddiv_rn(sum, 8.0);
            }
            const double link0 = W_pp[(int)pc[Cj + slot[0][0]] * NDEV + pc[Cj + slot[0][1]]];
            const double link1 = W_pp[(int)pc[Cjp + slot[1][0]] * NDEV + pc[Cjp + slot[1][1]]];
            const int base = lane & ~15;
            const double mx[2] = {__shfl(mean, base + 0), __shfl(mean, base + 1)};
            const double my[2] = {__shfl(mean, base + 2), __shfl(mean, base + 3)};
            double bestg = 0.0;
            int bk = -1;
#pragma unroll
            for (int k = 0; k < 4; k++) {
                double g = mx[k >> 1];
                g = __dadd_rn(g, -link0);
                g = __dadd_rn(g, my[k & 1]);
                g = __dadd_rn(g, -link1);
                if (bk < 0 || g > bestg) {
                    bestg = g;
                    bk = k;
                }
            }
            const int pa = Cj + slot[0][bk >> 1], pb_ = Cjp + slot[1][bk & 1];   // positions, pa < pb_
            // ---- trial rows: every lane needs each candidate's swap ----
            int trial[CANDS] = {0, 0, 0, 0}, ta[CANDS], tb[CANDS];
#pragma unroll
            for (int c = 0; c < NC; c++) {
                ta[c] = __shfl(pa, c * 16);
                tb[c] = __shfl(pb_, c * 16);
                const int src = lane == ta[c] ? tb[c] : (lane == tb[c] ? ta[c] : lane);
                trial[c] = wl[OFF_PBCUR + c * 64 + src];
            }
            WAVE_LDS_SYNC();
#pragma unroll
            for (int c = 0; c < NC; c++) wl[OFF_PB + c * 64 + lane] = (unsigned char)trial[c];
            WAVE_LDS_SYNC();
            double tcost[CANDS];
            eval_quad<NC>(cx, W_dp, rank_val, trial, tcost, unused, nullptr, quad * NC, P);
            // ---- accept iff strictly cheaper ----
#pragma unroll
            for (int c = 0; c < NC; c++) {
                const bool take = tcost[c] < cur_cost[c];   // wave-uniform
                if (take) {
                    cur[c] = trial[c];
                    cur_cost[c] = tcost[c];
                    wl[OFF_PBCUR + c * 64 + lane] = (unsigned char)trial[c];
                }
                const size_t cand = quad * NC + c;
                if (applied != nullptr && lane == 0 && cand < P)
                    applied[cand * (size_t)moves + r] =
                        take ? (long long)ta[c] * NDEV - (long long)ta[c] * (ta[c] + 1) / 2 + (tb[c] - ta[c] - 1) : -1ll;
            }
            WAVE_LDS_SYNC();
        }
#pragma unroll
        for (int c = 0; c < NC; c++) {
            const size_t cand = quad * NC + c;
            if (cand < P) {
                perm[cand * NDEV + lane] = cur[c];
                if (lane == 0) cost[cand] = cur_cost[c];
            }
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

// ---- Held-Karp item table (problem independent, built once per process) ------------------------
// A 128-bit LDS read is served 16 lanes at a time and is fastest when those 16 lanes hit 16 different
// bank groups (address / 16 mod 16) - lanes that share an address are only free when adjacent. The
// items are therefore laid out by a cyclic structure that makes this true by construction:
//  * item (S, v) with S = v + ({0} u D) (mod 8) belongs to class D, a (k-1)-subset of {1..7}; the 8
//    items of a class are the rotations v = 0..7 and occupy 8 consecutive lanes (lane % 8 = v);
//  * a pass of 16 lanes holds two classes (halves h = 0, 1); the item's entry index in its layer's
//    buffer is pass*16 + h*8 + v, so writes are dense and an entry's bank group is h*8 + v;
//  * every class visits its predecessors in an order (d_1 .. d_{k-1}) of D: at step t all 8 lanes read
//    u = v + d_t, i.e. the 8 rotations of ONE source class D' = (D \ d_t) - d_t of the previous layer:
//    8 different bank groups, all in the half h(D') where that class was placed;
//  * the read of a pass is conflict free when its two classes read from opposite halves; class
//    placement and visiting orders are chosen by a small deterministic search to make that so;
//  * ghat[u][v] is read from the lane's own column (see GHAT_PAIR_BYTES): never a conflict.
struct hk_class {
    uint8_t D;        // difference set as a bit mask over {1..7} (bit d set = d in D)
    uint8_t ord[7];   // visiting order of D's elements
};

inline uint8_t hk_source_class(uint8_t D, int d)   // (D \ d) - d (mod 8), as a mask over {1..7}
{
    uint8_t out = 0;
    for (int e = 1; e < 8; e++)
        if (e != d && (D & (1 << e))) out |= (uint8_t)(1 << ((e - d + 8) & 7));
    return out;
}

const std::vector<uint32_t> &hk_item_table()
{
    static std::vector<uint32_t> tab;
    static std::once_flag once;
    std::call_once(once, [] {
        tab.assign((size_t)HK_TAB_WORDS4 * 64 * 4, 0u);
        // half[D] (0/1) and pass[D] of every class of the previous layer, indexed by mask; -1: none
        int prev_half[256], prev_pass[256], cur_half[256], cur_pass[256];
        for (int i = 0; i < 256; i++) prev_half[i] = prev_pass[i] = -1;
        uint64_t rng = 0x2545F4914F6CDD1Dull;
        auto next = [&rng](uint32_t n) {
            rng = rng * 6364136223846793005ull + 1442695040888963407ull;
            return (uint32_t)((rng >> 33) % n);
        };
        for (int k = 2; k <= 8; k++) {
            std::vector<hk_class> cls;
            for (int D = 0; D < 256; D += 2)
                if (__builtin_popcount(D) == k - 1) {
                    hk_class c = {};
                    c.D = (uint8_t)D;
                    int t = 0;
                    for (int d = 1; d < 8; d++)
                        if (D & (1 << d)) c.ord[t++] = (uint8_t)d;
                    cls.push_back(c);
                }
            const int nc = (int)cls.size(), np = (nc + 1) / 2;
            // position i of `cls` = (pass i / 2, half i % 2). Cost: number of (pass, step) whose two
            // classes read from the same half of the previous layer (layer 1 is kept in both halves).
            auto pass_cost = [&](int p) {
                if (2 * p + 1 >= nc || k == 2) return 0;
                int c = 0;
                for (int t = 0; t < k - 1; t++) {
                    int ha = prev_half[hk_source_class(cls[2 * p].D, cls[2 * p].ord[t])];
                    int hb = prev_half[hk_source_class(cls[2 * p + 1].D, cls[2 * p + 1].ord[t])];
                    c += ha == hb;
                }
                return c;
            };
            std::vector<int> cost(np);
            int total = 0;
            for (int p = 0; p < np; p++) total += cost[p] = pass_cost(p);
            for (int it = 0; it < 60000 && total > 0; it++) {
                int a = (int)next(nc);
                if (next(2) == 0 && k > 2) {
                    int x = (int)next(k - 1), y = (int)next(k - 1);
                    if (x == y) continue;
                    std::swap(cls[a].ord[x], cls[a].ord[y]);
                    int c = pass_cost(a / 2);
                    if (c <= cost[a / 2]) {
                        total += c - cost[a / 2];
                        cost[a / 2] = c;
                    } else
                        std::swap(cls[a].ord[x], cls[a].ord[y]);
                } else {
                    int b = (int)next(nc);
                    if (a / 2 == b / 2) continue;
                    std::swap(cls[a], cls[b]);
                    int ca = pass_cost(a / 2), cb = pass_cost(b / 2);
                    if (ca + cb <= cost[a / 2] + cost[b / 2]) {
                        total += ca + cb - cost[a / 2] - cost[b / 2];
                        cost[a / 2] = ca;
                        cost[b / 2] = cb;
                    } else
                        std::swap(cls[a], cls[b]);
                }
            }
            for (int i = 0; i < 256; i++) cur_half[i] = cur_pass[i] = -1;
            for (int i = 0; i < nc; i++) {
                cur_pass[cls[i].D] = i / 2;
                cur_half[cls[i].D] = i % 2;
            }
            // emit: item (S, v) of class i sits at step (i/2)/4, lane ((i/2)%4)*16 + (i%2)*8 + v
            for (int i = 0; i < nc; i++)
                for (int v = 0; v < 8; v++) {
                    const int pass = i / 2, half = i % 2, s = pass / 4, lane = (pass % 4) * 16 + half * 8 + v;
                    uint32_t word[8] = {0};
                    word[0] = (uint32_t)((pass * 16 + half * 8 + v) * 16) | 0x80000000u;
                    for (int t = 0; t < k - 1; t++) {
                        const int d = cls[i].ord[t], u = (v + d) & 7;
                        int src;   // entry index of (S \ v, u) in the previous layer's buffer
                        if (k == 2)
                            src = half * 8 + u;   // layer 1 is stored in both halves
                        else {
                            const uint8_t Ds = hk_source_class(cls[i].D, d);
                            src = prev_pass[Ds] * 16 + prev_half[Ds] * 8 + u;
                        }
                        word[1 + t] = (uint32_t)(src * 16) | ((uint32_t)((u * 16 + half * 8 + v) * 16) << 16);
                    }
                    for (int w = 0; w < hk_words4(k) * 4; w++) {
                        size_t word4 = (size_t)hk_tab_first(k) + (size_t)s * hk_words4(k) + w / 4;
                        tab[(word4 * 64 + lane) * 4 + w % 4] = word[w];
                    }
                }
            // lanes without an item still execute the reads: point them at their own bank group
            for (int s = 0; s < hk_steps(k); s++)
                for (int lane = 0; lane < 64; lane++) {
                    size_t word4 = (size_t)hk_tab_first(k) + (size_t)s * hk_words4(k);
                    if (tab[(word4 * 64 + lane) * 4] >> 31) continue;
                    for (int w = 1; w < hk_words4(k) * 4; w++)
                        tab[((word4 + w / 4) * 64 + lane) * 4 + w % 4] =
                            (uint32_t)((lane & 15) * 16) | ((uint32_t)((lane & 15) * 16) << 16);
                }
            for (int i = 0; i < 256; i++) {
                prev_half[i] = cur_half[i];
                prev_pass[i] = cur_pass[i];
            }
        }
    });
    return tab;
}

}  // namespace

bool dtfm_fast64_applicable(const dtfm_problem *pr) { return pr->N == 64 && pr->D_dp == 8 && pr->D_pp == 8; }

// Builds the rank tables of a 64-device problem and uploads the Held-Karp item table.
int dtfm_fast64_prepare(dtfm_problem *pr)
{
    const int N = pr->N;
    DTFM_HIP(hipMalloc((void **)&pr->f64_rank, (size_t)N * N * sizeof(uint16_t)));
    DTFM_HIP(hipMalloc((void **)&pr->f64_rank_val, (size_t)N * N * sizeof(double)));
    DTFM_HIP(hipMemset(pr->f64_rank_val, 0, (size_t)N * N * sizeof(double)));
    hipLaunchKernelGGL(k_rank_weights, dim3((N * N + 255) / 256), dim3(256), 0, (hipStream_t) nullptr, pr->W_pp, N,
                       pr->f64_rank, pr->f64_rank_val);
    DTFM_HIP(hipGetLastError());

    const std::vector<uint32_t> &tab = hk_item_table();
    DTFM_HIP(hipMalloc((void **)&pr->f64_steps, tab.size() * sizeof(uint32_t)));
    DTFM_HIP(hipMemcpy(pr->f64_steps, tab.data(), tab.size() * sizeof(uint32_t), hipMemcpyHostToDevice));
    DTFM_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_eval_fast64<4>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, LDS_TOTAL));
    DTFM_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_eval_fast64<2>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, LDS_TOTAL));
    DTFM_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_ls_gain4_fast64<4>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, LDS_TOTAL));
    DTFM_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_ls_gain4_fast64<2>),
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

// Four candidates per wavefront give the best throughput; when there are too few candidates to
// give every wavefront slot of the chip a pass that way, two per wavefront halve the latency.
static bool use_two(const dtfm_problem *pr, size_t rows)
{
    return (rows + 3) / 4 < 2 * (size_t)pr->f64_grid * WAVES_PER_BLOCK;
}

int dtfm_fast64_enqueue(const dtfm_problem *pr, const int32_t *perm, size_t rows, double *cost, double *ghat,
                        double *datap, hipStream_t st)
{
    if (rows == 0) return DTFM_OK;
    const int nc = use_two(pr, rows) ? 2 : 4;
    size_t passes = (rows + nc - 1) / nc;
    size_t blocks = (passes + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK;
    if (blocks > (size_t)pr->f64_grid) blocks = pr->f64_grid;
    if (nc == 2)
        hipLaunchKernelGGL(k_eval_fast64<2>, dim3((unsigned)blocks), dim3(WAVES_PER_BLOCK * 64), LDS_TOTAL, st, pr->W_dp,
                           pr->f64_rank, pr->f64_rank_val, pr->f64_steps, perm, rows, cost, ghat, datap);
    else
        hipLaunchKernelGGL(k_eval_fast64<4>, dim3((unsigned)blocks), dim3(WAVES_PER_BLOCK * 64), LDS_TOTAL, st, pr->W_dp,
                           pr->f64_rank, pr->f64_rank_val, pr->f64_steps, perm, rows, cost, ghat, datap);
    DTFM_HIP(hipGetLastError());
    return DTFM_OK;
}

int dtfm_fast64_ls_gain4_enqueue(const dtfm_problem *pr, int32_t *perm, size_t rows, int moves, double *cost,
                                 int64_t *applied, hipStream_t st)
{
    if (rows == 0) return DTFM_OK;
    const int nc = use_two(pr, rows) ? 2 : 4;
    size_t passes = (rows + nc - 1) / nc;
    size_t blocks = (passes + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK;
    if (blocks > (size_t)pr->f64_grid) blocks = pr->f64_grid;
    if (nc == 2)
        hipLaunchKernelGGL(k_ls_gain4_fast64<2>, dim3((unsigned)blocks), dim3(WAVES_PER_BLOCK * 64), LDS_TOTAL, st,
                           pr->W_dp, pr->W_pp, pr->f64_rank, pr->f64_rank_val, pr->f64_steps, perm, rows, moves, cost,
                           applied);
    else
        hipLaunchKernelGGL(k_ls_gain4_fast64<4>, dim3((unsigned)blocks), dim3(WAVES_PER_BLOCK * 64), LDS_TOTAL, st,
                           pr->W_dp, pr->W_pp, pr->f64_rank, pr->f64_rank_val, pr->f64_steps, perm, rows, moves, cost,
                           applied);
    DTFM_HIP(hipGetLastError());
    return DTFM_OK;
}
