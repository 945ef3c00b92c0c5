// Fused population-evaluation kernel for the 64-device shape (N = 64, D_dp = 8, D_pp = 8): one
// wavefront evaluates eight candidates end to end (Eqs. 1-4); apart from the table gathers the whole
// evaluation is register arithmetic.
//
//   Matching (Eq. 3)   The bottleneck value of a block depends only on the ORDER of its entries,
//                      so the kernel works on 16-bit ranks of W_pp (rank table in LDS, built once
//                      per problem) and maps the winning rank back to its fp64 weight at the end:
//                      bit-identical to working on the doubles. Per stage pair a min-max dynamic
//                      programme over column subsets, row by row:
//                          g[S] = min_{c in S} max(g[S \ c], w[|S|-1][c]),   g[all] = optimum.
//                      Lane = (candidate 0..3, couple of stage pairs 0..13), two passes for the eight
//                      candidates: two pairs packed in one 32-bit register, 16-bit packed max/min.
//                      Every lane walks the subsets in the same order, so the whole table lives in
//                      registers with compile-time indices: no table traffic, no index arithmetic,
//                      2 ALU ops per transition.
//   Held-Karp (Eq. 4)  lane = (candidate 0..7, stage v 0..7). The stages are taken as the group
//                      Z_2^3: item (S, v) with S = v xor ({0} u D) belongs to class D (a subset of
//                      {1..7}), and lane v holds the items (class D, v) of ALL classes, one register
//                      pair per class. The relaxation tab[S][v] = min_u tab[S \ v][u] + Ghat[u][v] with
//                      u = v xor d reads class (D \ d) xor d at lane v xor d: a compile-time register
//                      and a lane exchange within the 8 lanes of the candidate, done by data-parallel
//                      primitive moves (xor 1, 2, 3: quad permutations; xor 7: mirror of the 8 lanes;
//                      xor 4, 5, 6: mirror, then a quad permutation). No memory traffic at all.
//   DataP (Eq. 2)      lane = (candidate, stage): the 8 x 8 entries of W_dp (LDS copy) of the stage's
//                      devices summed in slot order (the device's own slot adds the zero diagonal),
//                      max over the stage, then over the 8 lanes of the candidate.
#include "dtfm_internal.h"

#include <math.h>

namespace {

constexpr int NDEV = 64;
// Row stride of the rank table in LDS, in 16-bit entries. 66 instead of 64 skews consecutive rows by
// one 4-byte bank, so that lanes reading the same column of different rows hit different banks.
constexpr int RSTRIDE = 66;
constexpr int BINOM8[9] = {1, 8, 28, 56, 70, 56, 28, 8, 1};
constexpr int BINOM7[8] = {1, 7, 21, 35, 35, 21, 7, 1};

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

// Held-Karp classes: D as a bit mask over {1..7} (bit d set = d in D; bit 0 never set).
// HKC.cls[j][i] = i-th class with j elements (ascending masks), HKC.idx[D] = its index i.
struct hk_class_table {
    unsigned char cls[8][35];
    unsigned char idx[256];
};
constexpr hk_class_table make_hk_classes()
{
    hk_class_table t = {};
    for (int j = 0; j <= 7; j++) {
        int n = 0;
        for (int D = 0; D < 256; D += 2) {
            int pc = 0;
            for (int b = 1; b < 8; b++) pc += (D >> b) & 1;
            if (pc == j) {
                t.cls[j][n] = (unsigned char)D;
                t.idx[D] = (unsigned char)n;
                n++;
            }
        }
    }
    return t;
}
constexpr hk_class_table HKC = make_hk_classes();

// class reached from source class Ds by the relaxation through d (d not in Ds): (Ds xor d) u {d}
constexpr int hk_dest_class(int Ds, int d)
{
    int out = 1 << d;
    for (int e = 1; e < 8; e++)
        if ((Ds >> e) & 1) out |= 1 << (e ^ d);
    return out;
}
// source class of class D through d (d in D): (D \ d) xor d
constexpr int hk_source_class(int D, int d)
{
    int out = 0;
    for (int e = 1; e < 8; e++)
        if (e != d && ((D >> e) & 1)) out |= 1 << (e ^ d);
    return out;
}
// true when, walking the source classes of a layer in ascending index and d ascending within a source,
// (source of D through d) is the first relaxation into D: it initialises D's register instead of
// taking a min. (Two different d can have the same source class, e.g. D = {d, e} through d and e.)
constexpr bool hk_first_into(int D, int d)
{
    const int mine = HKC.idx[hk_source_class(D, d)];
    for (int e = 1; e < 8; e++) {
        if (e == d || !((D >> e) & 1)) continue;
        const int other = HKC.idx[hk_source_class(D, e)];
        if (other < mine || (other == mine && e < d)) return false;
    }
    return true;
}
// The relaxation programme: HKP.step[J][s][d] for source class s of layer J - 1 and d = 1..7:
// 0xFF when d is in the source class (no relaxation), else (index of the destination class in layer
// J) | 0x80 when this relaxation is the first into its destination.
struct hk_program {
    unsigned char step[8][35][8];
};
constexpr hk_program make_hk_program()
{
    hk_program p = {};
    for (int J = 1; J <= 7; J++)
        for (int s = 0; s < BINOM7[J - 1]; s++)
            for (int d = 1; d < 8; d++) {
                const int Ds = HKC.cls[J - 1][s];
                if ((Ds >> d) & 1) {
                    p.step[J][s][d] = 0xFF;
                    continue;
                }
                const int D = hk_dest_class(Ds, d);
                p.step[J][s][d] = (unsigned char)(HKC.idx[D] | (hk_first_into(D, d) ? 0x80 : 0));
            }
    return p;
}
constexpr hk_program HKP = make_hk_program();

// ---- LDS layout: three tables shared by the workgroup, then one slice per wavefront ----
constexpr int MAXC = 8;                                                 // candidates per wavefront pass
constexpr int LDS_RANK_BYTES = ((NDEV * RSTRIDE * 2 + 15) / 16) * 16;   // 8.25 KiB: u16 rank of W_pp
constexpr int LDS_RVAL_BYTES = NDEV * NDEV * 8;                         // 32 KiB: rank -> weight
constexpr int LDS_WDP_BYTES = NDEV * NDEV * 8;                          // 32 KiB: W_dp
constexpr int OFF_PB = 0;                                // u8 [8 candidates][64]: rows under evaluation, stage-major
constexpr int OFF_PBCUR = OFF_PB + MAXC * 64;            // u8 [8][64]: current rows (local search)
// coarsened graphs, double [candidate][u][v] with rows padded to 9 and candidates to 73 entries
constexpr int GH_ROW = 9, GH_CAND = 73;
constexpr int OFF_GHAT = OFF_PBCUR + MAXC * 64;
constexpr int WAVE_LDS_BYTES = ((OFF_GHAT + MAXC * GH_CAND * 8 + 15) / 16) * 16;
constexpr int WAVES_PER_BLOCK = 8;
constexpr int LDS_TOTAL = LDS_RANK_BYTES + LDS_RVAL_BYTES + LDS_WDP_BYTES + WAVES_PER_BLOCK * WAVE_LDS_BYTES;

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

// ---- lane exchanges inside the 8 lanes of a candidate (data-parallel primitive moves) ----
constexpr int DPP_XOR1 = 0xB1;          // quad permutation [1,0,3,2]
constexpr int DPP_XOR2 = 0x4E;          // quad permutation [2,3,0,1]
constexpr int DPP_XOR3 = 0x1B;          // quad permutation [3,2,1,0]
constexpr int DPP_HALF_MIRROR = 0x141;  // lane i of every 8 takes lane 7 - i: xor 7

template <int CTRL>
__device__ __forceinline__ double dpp_move(double x)
{
    const uint64_t b = __builtin_bit_cast(uint64_t, x);
    const int lo = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)b, CTRL, 0xF, 0xF, true);
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)(b >> 32), CTRL, 0xF, 0xF, true);
    return __builtin_bit_cast(double, ((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo);
}
// value of x at lane (lane xor d), d = 1, 2, 3, 7
__device__ __forceinline__ double lane_xor_direct(double x, int d)
{
    switch (d) {
    case 1: return dpp_move<DPP_XOR1>(x);
    case 2: return dpp_move<DPP_XOR2>(x);
    case 3: return dpp_move<DPP_XOR3>(x);
    default: return dpp_move<DPP_HALF_MIRROR>(x);
    }
}

// One layer of Held-Karp: classes with J elements from the classes with J - 1. Source-major order, so
// that the mirrored copy of a source serves all its relaxations through d = 4, 5, 6.
template <int J>
__device__ __forceinline__ void hk_layer(const double (&prev)[35], double (&cur)[35], const double (&G)[8])
{
#pragma unroll
    for (int s = 0; s < BINOM7[J - 1]; s++) {
        const double x = prev[s];
        double xm = 0.0;
        if (HKP.step[J][s][4] != 0xFF || HKP.step[J][s][5] != 0xFF || HKP.step[J][s][6] != 0xFF)
            xm = dpp_move<DPP_HALF_MIRROR>(x);
#pragma unroll
        for (int d = 1; d < 8; d++) {
            const int step = HKP.step[J][s][d];
            if (step == 0xFF) continue;
            const int i = step & 0x7F;
            // tab[S \ v][u] at u = v xor d, then + Ghat[u][v]
            const double moved = (d >= 4 && d <= 6) ? lane_xor_direct(xm, d ^ 7) : lane_xor_direct(x, d);
            const double t = __dadd_rn(moved, G[d]);
            cur[i] = (step & 0x80) ? t : fmin(cur[i], t);
        }
    }
}

// Eq. 4 for the candidate of this lane's 8-lane group; G[d] = Ghat[v][v xor d] of the lane's stage v.
// Every lane of the group returns the optimum.
__device__ __forceinline__ double hk_registers(const double (&G)[8])
{
    double a[35], b[35];
    // one stage: 0; two stages {v, v xor d}: 0 + Ghat
#pragma unroll
    for (int d = 1; d < 8; d++) b[HKC.idx[1 << d]] = G[d];
    hk_layer<2>(b, a, G);
    hk_layer<3>(a, b, G);
    hk_layer<4>(b, a, G);
    hk_layer<5>(a, b, G);
    hk_layer<6>(b, a, G);
    hk_layer<7>(a, b, G);
    double pp = b[0];   // all eight stages, ending in v: min over v
    pp = fmin(pp, dpp_move<DPP_XOR1>(pp));
    pp = fmin(pp, dpp_move<DPP_XOR2>(pp));
    pp = fmin(pp, dpp_move<DPP_HALF_MIRROR>(pp));
    return pp;
}

// byte k (0..7) of a 64-bit value held as two dwords
__device__ __forceinline__ uint32_t byte_of(uint2 v, int k) { return ((k < 4 ? v.x : v.y) >> (8 * (k & 3))) & 0xFFu; }

// Per-wavefront context: LDS pointers and the lane's fixed roles.
struct wave_ctx {
    unsigned char *wl;       // this wavefront's LDS slice
    const uint16_t *R;       // rank table (LDS)
    const double *rank_val;  // rank -> weight (LDS)
    const double *Wdp;       // W_dp (LDS)
    int lane;
    int mslot;               // matching role: candidate slot 0..3 within a matching pass
    bool couple_valid;       // lanes 14, 15 of each 16 repeat couple 13 and write nothing
    int j1[2], j2[2];        // the lane's two stage pairs (j1 < j2)
    int hc, hv;              // Held-Karp / DataP role: candidate slot, stage
};

// Loads the workgroup's tables into LDS and derives the lane roles. Ends with a workgroup barrier.
template <int NC>
__device__ __forceinline__ wave_ctx wave_setup(unsigned char *smem, const uint16_t *rank_tab,
                                               const double *rank_val, const double *W_dp)
{
    wave_ctx cx;
    cx.lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    cx.R = reinterpret_cast<const uint16_t *>(smem);
    cx.rank_val = reinterpret_cast<const double *>(smem + LDS_RANK_BYTES);
    cx.Wdp = reinterpret_cast<const double *>(smem + LDS_RANK_BYTES + LDS_RVAL_BYTES);
    cx.wl = smem + LDS_RANK_BYTES + LDS_RVAL_BYTES + LDS_WDP_BYTES + wave * WAVE_LDS_BYTES;
    // rank table -> LDS, rows re-strided (two entries per thread per pass)
    for (int i = threadIdx.x; i < NDEV * NDEV / 2; i += blockDim.x) {
        const int row = i / (NDEV / 2), col2 = i - row * (NDEV / 2);
        reinterpret_cast<uint32_t *>(smem)[row * (RSTRIDE / 2) + col2] = reinterpret_cast<const uint32_t *>(rank_tab)[i];
    }
    for (int i = threadIdx.x; i < NDEV * NDEV / 2; i += blockDim.x) {
        reinterpret_cast<double2 *>(smem + LDS_RANK_BYTES)[i] = reinterpret_cast<const double2 *>(rank_val)[i];
        reinterpret_cast<double2 *>(smem + LDS_RANK_BYTES + LDS_RVAL_BYTES)[i] = reinterpret_cast<const double2 *>(W_dp)[i];
    }
    // zero diagonals of the eight coarsened graphs (never overwritten)
    *reinterpret_cast<double *>(cx.wl + OFF_GHAT + ((cx.lane >> 3) * GH_CAND + (cx.lane & 7) * (GH_ROW + 1)) * 8) = 0.0;
    // matching role: candidate slot and the couple of stage pairs (2q, 2q+1) in lexicographic order
    cx.mslot = cx.lane >> 4;
    const int q = (cx.lane & 15) < 14 ? (cx.lane & 15) : 13;
    cx.couple_valid = (cx.lane & 15) < 14;
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
    // with NC = 4 the upper half of the wavefront repeats the lower half's Held-Karp and DataP
    cx.hc = (cx.lane >> 3) % NC;
    cx.hv = cx.lane & 7;
    __syncthreads();
    return cx;
}

// a4 for one pass of four candidates: the bottleneck matchings of this lane's two stage pairs of the
// candidate whose row is at pb, as two packed ranks.
__device__ __forceinline__ uint32_t match_couple(const wave_ctx &cx, const unsigned char *pb)
{
    const uint16_t *R = cx.R;
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
    return G[255];
}

// Evaluates the NC (8 or 4) candidates whose rows are in the wavefront's LDS slice at OFF_PB (stage-major
// bytes, already visible to all lanes). On return every lane holds total (Eq. 1) and datap (Eq. 2 + max)
// of candidate slot cx.hc. ghat_out, if not null, receives the coarsened graphs of candidates
// cand0 .. cand0 + NC - 1 that are < P.
template <int NC>
__device__ __forceinline__ void eval_group(const wave_ctx &cx, double &total, double &datap,
                                           double *__restrict__ ghat_out, size_t cand0, size_t P)
{
    unsigned char *wl = cx.wl;
    const int lane = cx.lane;
    double *gh = reinterpret_cast<double *>(wl + OFF_GHAT);
    // ---- a4: matchings on ranks; winning ranks -> fp64 weights -> coarsened graphs in LDS ----
#pragma nounroll
    for (int pass = 0; pass < NC / 4; pass++) {
        const int mc = 4 * pass + cx.mslot;
        const uint32_t gfull = match_couple(cx, wl + OFF_PB + mc * 64);
        const double e0 = cx.rank_val[gfull & 0xFFFFu], e1 = cx.rank_val[gfull >> 16];
        if (cx.couple_valid) {
            double *g = gh + mc * GH_CAND;
            g[cx.j1[0] * GH_ROW + cx.j2[0]] = e0;
            g[cx.j2[0] * GH_ROW + cx.j1[0]] = e0;
            g[cx.j1[1] * GH_ROW + cx.j2[1]] = e1;
            g[cx.j2[1] * GH_ROW + cx.j1[1]] = e1;
        }
    }
    WAVE_LDS_SYNC();
    if (ghat_out != nullptr) {
#pragma unroll
        for (int c = 0; c < NC; c++)
            if (cand0 + c < P) ghat_out[(cand0 + c) * 64 + lane] = gh[c * GH_CAND + (lane >> 3) * GH_ROW + (lane & 7)];
    }
    // ---- a5: Held-Karp in registers ----
    double G[8];
    G[0] = 0.0;
#pragma unroll
    for (int d = 1; d < 8; d++) G[d] = gh[cx.hc * GH_CAND + cx.hv * GH_ROW + (cx.hv ^ d)];
    const double pp = hk_registers(G);
    // ---- a2/a3: DataP of stage hv of candidate hc, then max over the candidate's 8 lanes ----
    const uint2 devs = *reinterpret_cast<const uint2 *>(wl + OFF_PB + cx.hc * 64 + 8 * cx.hv);
    uint32_t dv[8];
#pragma unroll
    for (int k = 0; k < 8; k++) dv[k] = byte_of(devs, k);
    double dp = 0.0;
#pragma unroll
    for (int i = 0; i < 8; i++) {
        const double *wrow = cx.Wdp + dv[i] * NDEV;
        double sum = 0.0;
#pragma unroll
        for (int k = 0; k < 8; k++) sum = __dadd_rn(sum, wrow[dv[k]]);   // own slot: the zero diagonal
        dp = i == 0 ? sum : fmax(dp, sum);
    }
    dp = fmax(dp, dpp_move<DPP_XOR1>(dp));
    dp = fmax(dp, dpp_move<DPP_XOR2>(dp));
    dp = fmax(dp, dpp_move<DPP_HALF_MIRROR>(dp));
    datap = dp;
    total = __dadd_rn(dp, pp);   // a6
    WAVE_LDS_SYNC();             // the next group reuses the slice
}

template <int NC>
__global__ void __launch_bounds__(WAVES_PER_BLOCK * 64)
k_eval_fast64(const double *__restrict__ W_dp, const uint16_t *__restrict__ rank_tab,
              const double *__restrict__ rank_val, const int32_t *__restrict__ perm, size_t P,
              double *__restrict__ cost, double *__restrict__ ghat_out, double *__restrict__ datap_out)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const wave_ctx cx = wave_setup<NC>(smem, rank_tab, rank_val, W_dp);
    const int lane = cx.lane, wave = threadIdx.x >> 6;
    const size_t nwaves = (size_t)gridDim.x * WAVES_PER_BLOCK;
    const size_t ngroups = (P + NC - 1) / NC;
    for (size_t grp = (size_t)blockIdx.x * WAVES_PER_BLOCK + wave; grp < ngroups; grp += nwaves) {
        // ---- a1: NC candidate rows; position = lane: stage = lane / 8, slot = lane % 8 ----
#pragma unroll
        for (int c = 0; c < NC; c++) {
            size_t cand = grp * NC + c;
            if (cand >= P) cand = P - 1;   // ragged tail: recompute the last row, never stored
            cx.wl[OFF_PB + c * 64 + lane] = (unsigned char)perm[cand * NDEV + lane];
        }
        WAVE_LDS_SYNC();
        double total, datap;
        eval_group<NC>(cx, total, datap, ghat_out, grp * NC, P);
        const size_t cand = grp * NC + (lane >> 3);
        if ((lane & 7) == 0 && lane < NC * 8 && cand < P) {
            if (cost != nullptr) cost[cand] = total;
            if (datap_out != nullptr) datap_out[cand] = datap;
        }
    }
}

// ---- Sec. 3.4 local search with the paper's four-candidate neighbourhood, all rounds in one launch
// Each wavefront carries its candidates through every round: propose a swap (fastest link inside
// each of the round's two stages, the four end-point swaps ranked by the paper's Gain), evaluate the
// swapped allocation with eval_group, keep it iff strictly cheaper. The fastest link is found on the
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
                  int32_t *__restrict__ perm, size_t P, int moves, double *__restrict__ cost,
                  int64_t *__restrict__ applied)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const wave_ctx cx = wave_setup<NC>(smem, rank_tab, rank_val, W_dp);
    const int lane = cx.lane, wave = threadIdx.x >> 6;
    unsigned char *wl = cx.wl;
    const int sub = lane & 15;   // proposal role: 16 lanes per candidate, four candidates per pass
    const size_t nwaves = (size_t)gridDim.x * WAVES_PER_BLOCK;
    const size_t ngroups = (P + NC - 1) / NC;
    for (size_t grp = (size_t)blockIdx.x * WAVES_PER_BLOCK + wave; grp < ngroups; grp += nwaves) {
#pragma unroll
        for (int c = 0; c < NC; c++) {
            size_t cand = grp * NC + c;
            if (cand >= P) cand = P - 1;
            const unsigned char d = (unsigned char)perm[cand * NDEV + lane];
            wl[OFF_PB + c * 64 + lane] = d;
            wl[OFF_PBCUR + c * 64 + lane] = d;
        }
        WAVE_LDS_SYNC();
        double cur_cost, unused;   // of candidate slot cx.hc
        eval_group<NC>(cx, cur_cost, unused, nullptr, grp * NC, P);
#pragma nounroll
        for (int r = 0; r < moves; r++) {
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
            const int Cj = 8 * j, Cjp = 8 * jp;
            int ta[NC], tb[NC];   // proposed positions of every candidate slot, ta < tb
#pragma unroll
            for (int pass = 0; pass < NC / 4; pass++) {
                // ---- proposal for candidate slot 4 * pass + lane / 16 by its 16 lanes ----
                const unsigned char *pc = wl + OFF_PBCUR + (4 * pass + (lane >> 4)) * 64;
                int slot[2][2];
#pragma unroll
                for (int s = 0; s < 2; s++) {
                    const unsigned char *C = pc + (s == 0 ? Cj : Cjp);
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
#pragma unroll
                for (int c = 0; c < 4; c++) {
                    ta[4 * pass + c] = __shfl(pa, c * 16);
                    tb[4 * pass + c] = __shfl(pb_, c * 16);
                }
            }
            // ---- trial rows ----
#pragma unroll
            for (int c = 0; c < NC; c++) {
                const int src = lane == ta[c] ? tb[c] : (lane == tb[c] ? ta[c] : lane);
                wl[OFF_PB + c * 64 + lane] = wl[OFF_PBCUR + c * 64 + src];
            }
            WAVE_LDS_SYNC();
            double tcost;
            eval_group<NC>(cx, tcost, unused, nullptr, grp * NC, P);
            // ---- accept iff strictly cheaper ----
            const bool mine = tcost < cur_cost;   // uniform over the 8 lanes of a candidate slot
            const uint64_t takes = __ballot(mine);
            if (mine) cur_cost = tcost;
#pragma unroll
            for (int c = 0; c < NC; c++) {
                const bool take = (takes >> (8 * c)) & 1;   // wave-uniform
                if (take) wl[OFF_PBCUR + c * 64 + lane] = wl[OFF_PB + c * 64 + lane];
                const size_t cand = grp * NC + c;
                if (applied != nullptr && lane == 0 && cand < P)
                    applied[cand * (size_t)moves + r] =
                        take ? (long long)ta[c] * NDEV - (long long)ta[c] * (ta[c] + 1) / 2 + (tb[c] - ta[c] - 1) : -1ll;
            }
            WAVE_LDS_SYNC();
        }
#pragma unroll
        for (int c = 0; c < NC; c++) {
            const size_t cand = grp * NC + c;
            if (cand < P) perm[cand * NDEV + lane] = wl[OFF_PBCUR + c * 64 + lane];
        }
        const size_t cand = grp * NC + (lane >> 3);
        if ((lane & 7) == 0 && lane < NC * 8 && cand < P) cost[cand] = cur_cost;
        WAVE_LDS_SYNC();
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

// Builds the rank tables of a 64-device problem.
int dtfm_fast64_prepare(dtfm_problem *pr)
{
    const int N = pr->N;
    DTFM_HIP(hipMalloc((void **)&pr->f64_rank, (size_t)N * N * sizeof(uint16_t)));
    DTFM_HIP(hipMalloc((void **)&pr->f64_rank_val, (size_t)N * N * sizeof(double)));
    DTFM_HIP(hipMemset(pr->f64_rank_val, 0, (size_t)N * N * sizeof(double)));
    hipLaunchKernelGGL(k_rank_weights, dim3((N * N + 255) / 256), dim3(256), 0, (hipStream_t) nullptr, pr->W_pp, N,
                       pr->f64_rank, pr->f64_rank_val);
    DTFM_HIP(hipGetLastError());
    DTFM_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_eval_fast64<8>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, LDS_TOTAL));
    DTFM_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_eval_fast64<4>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, LDS_TOTAL));
    DTFM_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_ls_gain4_fast64<8>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, LDS_TOTAL));
    DTFM_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_ls_gain4_fast64<4>),
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
}

// Eight candidates per wavefront give the best throughput (every lane busy in Held-Karp); when there
// are too few candidates to give every SIMD of the chip a wavefront that way, four per wavefront
// shorten the pass.
static bool use_four(const dtfm_problem *pr, size_t rows) { return rows <= 4 * 4 * (size_t)pr->f64_grid; }

int dtfm_fast64_enqueue(const dtfm_problem *pr, const int32_t *perm, size_t rows, double *cost, double *ghat,
                        double *datap, hipStream_t st)
{
    if (rows == 0) return DTFM_OK;
    const int nc = use_four(pr, rows) ? 4 : 8;
    size_t passes = (rows + nc - 1) / nc;
    size_t blocks = (passes + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK;
    if (blocks > (size_t)pr->f64_grid) blocks = pr->f64_grid;
    if (nc == 4)
        hipLaunchKernelGGL(k_eval_fast64<4>, dim3((unsigned)blocks), dim3(WAVES_PER_BLOCK * 64), LDS_TOTAL, st, pr->W_dp,
                           pr->f64_rank, pr->f64_rank_val, perm, rows, cost, ghat, datap);
    else
        hipLaunchKernelGGL(k_eval_fast64<8>, dim3((unsigned)blocks), dim3(WAVES_PER_BLOCK * 64), LDS_TOTAL, st, pr->W_dp,
                           pr->f64_rank, pr->f64_rank_val, perm, rows, cost, ghat, datap);
    DTFM_HIP(hipGetLastError());
    return DTFM_OK;
}

int dtfm_fast64_ls_gain4_enqueue(const dtfm_problem *pr, int32_t *perm, size_t rows, int moves, double *cost,
                                 int64_t *applied, hipStream_t st)
{
    if (rows == 0) return DTFM_OK;
    const int nc = use_four(pr, rows) ? 4 : 8;
    size_t passes = (rows + nc - 1) / nc;
    size_t blocks = (passes + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK;
    if (blocks > (size_t)pr->f64_grid) blocks = pr->f64_grid;
    if (nc == 4)
        hipLaunchKernelGGL(k_ls_gain4_fast64<4>, dim3((unsigned)blocks), dim3(WAVES_PER_BLOCK * 64), LDS_TOTAL, st,
                           pr->W_dp, pr->W_pp, pr->f64_rank, pr->f64_rank_val, perm, rows, moves, cost, applied);
    else
        hipLaunchKernelGGL(k_ls_gain4_fast64<8>, dim3((unsigned)blocks), dim3(WAVES_PER_BLOCK * 64), LDS_TOTAL, st,
                           pr->W_dp, pr->W_pp, pr->f64_rank, pr->f64_rank_val, perm, rows, moves, cost, applied);
    DTFM_HIP(hipGetLastError());
    return DTFM_OK;
}
