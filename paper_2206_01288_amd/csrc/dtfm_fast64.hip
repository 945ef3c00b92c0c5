// Fused population-evaluation kernel for the 64-device shape (N = 64, D_dp = 8, D_pp = 8): one
// wavefront evaluates a group of 4, 8 or 32 candidates end to end (Eqs. 1-4); apart from the table
// gathers the whole evaluation is register arithmetic.
//
//   Matching (Eq. 3)   The bottleneck value of a block depends only on the ORDER of its entries,
//                      so the kernel works on 16-bit ranks of W_pp (rank table in LDS, built once
//                      per problem) and maps the winning rank back to its fp64 weight at the end:
//                      bit-identical to working on the doubles. Per stage pair a min-max dynamic
//                      programme over column subsets, row by row:
//                          g[S] = min_{c in S} max(g[S \ c], w[|S|-1][c]),   g[all] = optimum.
//                      A lane takes a couple of stage pairs of one candidate: two pairs packed in
//                      one 32-bit register, 16-bit packed max/min. The work items are the 14 x NC
//                      (candidate, couple) combinations, 64 per pass. Every lane walks the subsets
//                      in the same order, so the whole table lives in registers with compile-time
//                      indices: no table traffic, no index arithmetic, 2 ALU ops per transition.
//   Held-Karp (Eq. 4)  lane = (candidate 0..7, stage v 0..7). The stages are taken as the group
//                      Z_2^3: item (S, v) with S = v xor ({0} u D) belongs to class D (a subset of
//                      {1..7}), and lane v holds the items (class D, v) of ALL classes, one register
//                      pair per class. The relaxation tab[S][v] = min_u tab[S \ v][u] + Ghat[u][v] with
//                      u = v xor d reads class (D \ d) xor d at lane v xor d: a compile-time register
//                      and a lane exchange within the 8 lanes of the candidate (xor 1, 2, 3: DPP quad
//                      permutations; xor 7: DPP mirror of the 8 lanes; xor 4, 5, 6: through the LDS
//                      crossbar, no memory access). No table traffic at all.
//   DataP (Eq. 2)      lane = (candidate, stage): the 8 x 8 entries of W_dp (LDS copy) of the stage's
//                      devices summed in slot order (the device's own slot adds the zero diagonal),
//                      max over the stage, then over the 8 lanes of the candidate.
#include "dtfm_fast64_device.h"
#include "dtfm_philox.h"

namespace {

// ---- LDS layout: tables shared by the workgroup, then one slice per wavefront ----
constexpr int MAXC = 32;                                                // most candidates per wavefront pass
constexpr int OFF_PB = 0;                        // u8 [NC candidates][64]: rows under evaluation, stage-major
// coarsened graphs as winning ranks: u16 [candidate][stage pair 0..27, lexicographic]; the couple
// (pairs 2q, 2q+1) of candidate c is the 32-bit word 14 c + q
constexpr int off_ghr(int nc) { return OFF_PB + nc * 64; }
constexpr int off_res(int nc) { return (off_ghr(nc) + nc * 28 * 2 + 7) / 8 * 8; }   // double [2][NC]: total, DataP
constexpr int off_curc(int nc) { return off_res(nc) + 2 * nc * 8; }            // double [NC]: current costs (local search)
constexpr int off_pbcur(int nc) { return off_curc(nc) + nc * 8; }              // u8 [NC][64]: current rows (local search)
constexpr int off_prop(int nc) { return off_pbcur(nc) + nc * 64; }             // u8 [NC][2]: proposed positions (local search)
constexpr int off_ghrcur(int nc) { return (off_prop(nc) + nc * 2 + 3) / 4 * 4; }   // u16 [NC][28]: coarsened graphs of the current rows
// with 4 candidates the local-search kernel can make its rows itself (offspring of the evolutionary search):
// u8 [4][64] position of each device in the child, u8 [4][64] the same in parent 2, u8 [2][4][32] draws
constexpr int MK_STEPS = 32;                                                    // crossover / mutation steps drawn at a time
constexpr int off_mk(int nc) { return (off_ghrcur(nc) + nc * 28 * 2 + 3) / 4 * 4; }
constexpr int mk_bytes(int nc) { return nc == 4 ? 2 * nc * 64 + 2 * nc * MK_STEPS : 0; }
constexpr int wave_lds_bytes(int nc, bool ls) { return ((ls ? off_mk(nc) + mk_bytes(nc) : off_curc(nc)) + 15) / 16 * 16; }
// the local-search kernels also keep W_pp in LDS (for the proposals), except with 32 candidates per
// wavefront, where the slices need the room and the proposals go through the rank tables instead
constexpr bool wpp_in_lds(int nc, bool ls) { return ls && nc < 32; }
constexpr int lds_total(int nc, bool ls, int waves = WAVES_PER_BLOCK) { return LDS_TABLES + (wpp_in_lds(nc, ls) ? LDS_WDP_BYTES : 0) + waves * wave_lds_bytes(nc, ls); }
static_assert(lds_total(MAXC, true) <= 160 * 1024, "LDS budget of a CU");

// Per-wavefront context: LDS pointers and the lane's fixed roles.
struct wave_ctx {
    unsigned char *wl;       // this wavefront's LDS slice
    const uint16_t *R;       // rank table (LDS)
    const double *rank_val;  // rank -> weight (LDS)
    const double *Wdp;       // W_dp (LDS)
    const double *Wpp;       // W_pp (local-search kernels with fewer than 32 candidates per wavefront: LDS copy)
    int lane;
    int hv;                  // Held-Karp / DataP role: stage; the candidate slot is 8 * pass + lane / 8
};

// Loads the workgroup's tables into LDS and derives the lane roles. Ends with a workgroup barrier.
template <int NC, bool LS>
__device__ __forceinline__ wave_ctx wave_setup(unsigned char *smem, const uint16_t *rank_tab,
                                               const double *rank_val, const double *W_dp, const double *W_pp)
{
    wave_ctx cx;
    cx.lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    cx.R = reinterpret_cast<const uint16_t *>(smem);
    cx.rank_val = reinterpret_cast<const double *>(smem + LDS_RANK_BYTES);
    cx.Wdp = reinterpret_cast<const double *>(smem + LDS_RANK_BYTES + LDS_RVAL_BYTES);
    cx.Wpp = wpp_in_lds(NC, LS) ? reinterpret_cast<const double *>(smem + LDS_TABLES) : nullptr;
    cx.wl = smem + LDS_TABLES + (wpp_in_lds(NC, LS) ? LDS_WDP_BYTES : 0) + wave * wave_lds_bytes(NC, LS);
    stage_tables<(NC < 32)>(smem, rank_tab, rank_val, W_dp);
    if (wpp_in_lds(NC, LS))   // NC < 32
#pragma unroll 8
        for (int i = threadIdx.x; i < NDEV * NDEV / 2; i += blockDim.x)
            reinterpret_cast<double2 *>(smem + LDS_TABLES)[i] = reinterpret_cast<const double2 *>(W_pp)[i];
    cx.hv = cx.lane & 7;
    __syncthreads();
    return cx;
}

// a4 for one lane: the bottleneck matchings of the stage pairs (j1[0], j2[0]) and (j1[1], j2[1]) of the
// candidate whose row is at pb, as two packed ranks.
__device__ __forceinline__ uint32_t match_couple(const wave_ctx &cx, const unsigned char *pb, const int (&j1)[2],
                                                 const int (&j2)[2])
{
    uint2 rowdev[2], coldev[2];
#pragma unroll
    for (int h = 0; h < 2; h++) {
        rowdev[h] = *reinterpret_cast<const uint2 *>(pb + 8 * j1[h]);   // devices of stage j1, slots 0..7
        coldev[h] = *reinterpret_cast<const uint2 *>(pb + 8 * j2[h]);   // devices of stage j2
    }
    uint32_t G[256];
    match_rows<8, true>(cx.R, rowdev, coldev, G);
    return G[255];
}

// The same two matchings shared by a pair of neighbouring lanes: lane parity 0 matches rows 0..3 of each
// block into every 4-column subset S, parity 1 rows 4..7; the optimum is the minimum over S of
// max(first half into S, second half into the other four columns). 1,070 dependent-chain
// instructions instead of 1,790: for wavefronts with at most 32 couples to match. Both lanes return
// the result.
__device__ __forceinline__ uint32_t match_couple_halves(const wave_ctx &cx, const unsigned char *pb, const int (&j1)[2],
                                                        const int (&j2)[2])
{
    const bool upper = (cx.lane & 1) != 0;
    uint2 rowdev[2], coldev[2];
#pragma unroll
    for (int h = 0; h < 2; h++) {
        rowdev[h].x = *reinterpret_cast<const uint32_t *>(pb + 8 * j1[h] + (upper ? 4 : 0));   // slots 0..3 or 4..7
        rowdev[h].y = 0;
        coldev[h] = *reinterpret_cast<const uint2 *>(pb + 8 * j2[h]);
    }
    uint32_t G[256];
    match_rows<4, false>(cx.R, rowdev, coldev, G);
    uint32_t best = 0;
#pragma unroll
    for (int i = 0; i < BINOM8[4]; i++) {
        const int S = LAYER.s[4][i];
        const uint32_t other = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)G[255 ^ S], DPP_XOR1, 0xF, 0xF, true);
        const uint32_t m = pk_max(G[S], other);
        best = i == 0 ? m : pk_min(best, m);
    }
    return best;
}

// Evaluates the NC (4, 8 or 32) candidates whose rows are in the wavefront's LDS slice at OFF_PB
// (stage-major bytes, already visible to all lanes). The work items of the matching phase are the
// NC * 14 (candidate, couple of stage pairs) combinations, 64 per pass: with NC = 32 every lane of all
// seven passes is busy. Held-Karp and DataP then run NC / 8 passes of eight candidates (with NC = 4 the
// upper half of the wavefront repeats the lower half). On return the slice holds, visible to all
// lanes, total (Eq. 1) of candidate slot c at res[c] and DataP (Eq. 2 + max) at res[NC + c]. ghat_out,
// if not null, receives the coarsened graphs of candidates cand0 .. cand0 + NC - 1 that are < P.
// With INC and sj >= 0 (sj < sjp) the rows differ from rows whose winning ranks are already in the
// slice only in stages sj and sjp: only the 13 stage pairs that contain one of them are matched
// again (7 couples per candidate, the last with its second pair repeated).
template <int NC, bool INC>
__device__ __forceinline__ void eval_group(const wave_ctx &cx, double *__restrict__ ghat_out, size_t cand0, size_t P,
                                           int sj, int sjp)
{
    unsigned char *wl = cx.wl;
    const int lane = cx.lane;
    constexpr int HPASSES = (NC + 7) / 8;
    uint16_t *ghr16 = reinterpret_cast<uint16_t *>(wl + off_ghr(NC));
    double *res = reinterpret_cast<double *>(wl + off_res(NC));
    // ---- a4: matchings on ranks; the winning ranks of stage pair (a, b) of candidate c go to [c][index of (a, b)] ----
    const bool inc = INC && sj >= 0;
    // a pass with 32 couples or fewer (the only pass with 4 candidates, the last of four with 32):
    // two lanes per couple, each matching half of the rows
    constexpr bool HALVES = INC && (NC * 7) % 64 != 0 && (NC * 7) % 64 <= 32;
    const int per_cand = inc ? 7 : 14, items = NC * per_cand, mpasses = (items + 63) / 64;
#pragma nounroll
    for (int pass = 0; pass < mpasses; pass++) {
        const bool halves = HALVES && inc && items - pass * 64 <= 32;   // wave-uniform
        int t = pass * 64 + (halves ? lane >> 1 : lane);
        const bool valid = t < items && !(halves && (lane & 1));
        if (t >= items) t = items - 1;   // idle lanes repeat the last item and write nothing
        const int mc = t / per_cand, q = t - per_cand * mc;
        int j1[2], j2[2];
        if (!inc) {
            pair8_decode(2 * q, j1[0], j2[0]);
            pair8_decode(2 * q + 1, j1[1], j2[1]);
        } else {
#pragma unroll
            for (int h = 0; h < 2; h++) {
                // changed pair number e = 0..12: (sj, k) for the 7 stages k != sj, then (sjp, k) for the 6 others
                const int e = 2 * q + h < 12 ? 2 * q + h : 12;
                int a, k;
                if (e < 7) {
                    a = sj;
                    k = e + (e >= sj ? 1 : 0);
                } else {
                    a = sjp;
                    k = e - 7;
                    k += k >= sj ? 1 : 0;
                    k += k >= sjp ? 1 : 0;
                }
                j1[h] = a < k ? a : k;
                j2[h] = a < k ? k : a;
            }
        }
        uint32_t gfull;
        if (HALVES && halves) gfull = match_couple_halves(cx, wl + OFF_PB + mc * 64, j1, j2);
        else gfull = match_couple(cx, wl + OFF_PB + mc * 64, j1, j2);
        if (valid) {
            ghr16[mc * 28 + pair_index(j1[0], j2[0])] = (uint16_t)gfull;
            ghr16[mc * 28 + pair_index(j1[1], j2[1])] = (uint16_t)(gfull >> 16);
        }
    }
    WAVE_LDS_SYNC();
    if (ghat_out != nullptr) {
        const int u = lane >> 3, v = lane & 7;
        const int pi = pair_index(u < v ? u : v, u < v ? v : u);
#pragma nounroll
        for (int c = 0; c < NC; c++)
            if (cand0 + c < P) ghat_out[(cand0 + c) * 64 + lane] = u == v ? 0.0 : cx.rank_val[ghr16[c * 28 + pi]];
    }
#pragma nounroll
    for (int h = 0; h < HPASSES; h++) {
        const int hc = (8 * h + (lane >> 3)) % NC;
        // ---- a5: winning ranks -> fp64 weights; Held-Karp in registers ----
        // With four candidates the upper half of the wavefront shares the work of the lower half: its
        // lanes stand for the stages with bits 0 and 1 swapped (see hk_registers).
        constexpr bool SPLIT = NC == 4;
        const bool relabel = SPLIT && lane >= 32;
        const int v = relabel ? hk_swap01(cx.hv) : cx.hv;
        double G[8];
        G[0] = 0.0;
#pragma unroll
        for (int d = 1; d < 8; d++) {
            const int u = v ^ (relabel ? hk_swap01(d) : d);
            G[d] = cx.rank_val[ghr16[hc * 28 + pair_index(u < v ? u : v, u < v ? v : u)]];
        }
        const double pp = hk_registers<SPLIT>(G, lane);
        // ---- a2/a3: DataP of stage hv of candidate hc, then max over the candidate's 8 lanes ----
        double dp = stage_datap(cx.Wdp, *reinterpret_cast<const uint2 *>(wl + OFF_PB + hc * 64 + 8 * cx.hv));
        dp = fmax(dp, dpp_move<DPP_XOR1>(dp));
        dp = fmax(dp, dpp_move<DPP_XOR2>(dp));
        dp = fmax(dp, dpp_move<DPP_HALF_MIRROR>(dp));
        if (cx.hv == 0 && lane < NC * 8) {
            res[hc] = __dadd_rn(dp, pp);   // a6
            res[NC + hc] = dp;
        }
    }
    WAVE_LDS_SYNC();
}

template <int NC>
__global__ void __launch_bounds__(WAVES_PER_BLOCK * 64)
k_eval_fast64(const double *__restrict__ W_dp, const uint16_t *__restrict__ rank_tab,
              const double *__restrict__ rank_val, const int32_t *__restrict__ perm, size_t P,
              double *__restrict__ cost, double *__restrict__ ghat_out, double *__restrict__ datap_out)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const wave_ctx cx = wave_setup<NC, false>(smem, rank_tab, rank_val, W_dp, nullptr);
    const int lane = cx.lane, wave = threadIdx.x >> 6;
    const int wpb = blockDim.x >> 6;   // wavefronts per workgroup: WAVES_PER_BLOCK, fewer for small populations
    const size_t nwaves = (size_t)gridDim.x * wpb;
    const size_t ngroups = (P + NC - 1) / NC;
    for (size_t grp = (size_t)blockIdx.x * wpb + wave; grp < ngroups; grp += nwaves) {
        // ---- a1: NC candidate rows; position = lane: stage = lane / 8, slot = lane % 8 ----
#pragma unroll 8
        for (int c = 0; c < NC; c++) {
            size_t cand = grp * NC + c;
            if (cand >= P) cand = P - 1;   // ragged tail: recompute the last row, never stored
            cx.wl[OFF_PB + c * 64 + lane] = (unsigned char)perm[cand * NDEV + lane];
        }
        WAVE_LDS_SYNC();
        eval_group<NC, false>(cx, ghat_out, grp * NC, P, -1, -1);
        const double *res = reinterpret_cast<const double *>(cx.wl + off_res(NC));
        const size_t cand = grp * NC + lane;
        if (lane < NC && cand < P) {
            if (cost != nullptr) cost[cand] = res[lane];
            if (datap_out != nullptr) datap_out[cand] = res[NC + lane];
        }
        WAVE_LDS_SYNC();   // the next group reuses the slice
    }
}

// Population evaluation for populations so small that every SIMD has one group of four candidates and the launch
// is as long as one wavefront's instruction stream: the group gets a PAIR of wavefronts (w and w + cw of the
// workgroup, which share a SIMD). Both match: each takes two of the four candidates, two lanes per couple of stage
// pairs (28 couples, 56 lanes, the programme of match_couple_halves, 1,070 instructions instead of 1,790), and the
// two streams fill each other's wait states. Then the first runs Held-Karp for all four candidates (64 lanes,
// hk_registers<true>) while the second computes their DataP straight from the global W_dp (no LDS copy of it).
// Workgroup barriers: after the table set-up, after the matching, before the final sum.
__global__ void __launch_bounds__(WAVES_PER_BLOCK * 64)
k_eval_fast64_paired(const double *__restrict__ W_dp, const uint16_t *__restrict__ rank_tab,
                     const double *__restrict__ rank_val, const int32_t *__restrict__ perm, size_t P,
                     double *__restrict__ cost, double *__restrict__ ghat_out, double *__restrict__ datap_out)
{
    constexpr int NC = 4;
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int cw = blockDim.x >> 7;            // groups of the workgroup; wavefronts g and g + cw work on group g
    const bool second = wave >= cw;
    const int slice = second ? wave - cw : wave;
    wave_ctx cx;
    cx.lane = lane;
    cx.hv = lane & 7;
    cx.R = reinterpret_cast<const uint16_t *>(smem);
    cx.rank_val = reinterpret_cast<const double *>(smem + LDS_RANK_BYTES);
    cx.Wdp = nullptr;
    cx.Wpp = nullptr;
    cx.wl = smem + LDS_TABLES + slice * wave_lds_bytes(NC, false);
    unsigned char *wl = cx.wl;
    const size_t grp = (size_t)blockIdx.x * cw + slice;
    // ---- set-up: rank table and rank values by all; a1: the group's rows by its first wavefront ----
#pragma unroll 2
    for (int i = threadIdx.x; i < NDEV * NDEV / 2; i += blockDim.x) {
        const int row = i / (NDEV / 2), col2 = i - row * (NDEV / 2);
        reinterpret_cast<uint32_t *>(smem)[row * (RSTRIDE / 2) + col2] = reinterpret_cast<const uint32_t *>(rank_tab)[i];
    }
#pragma unroll 4
    for (int i = threadIdx.x; i < NDEV * NDEV / 2; i += blockDim.x)
        reinterpret_cast<double2 *>(smem + LDS_RANK_BYTES)[i] = reinterpret_cast<const double2 *>(rank_val)[i];
    if (!second) {
#pragma unroll
        for (int c = 0; c < NC; c++) {
            size_t cand = grp * NC + c;
            if (cand >= P) cand = P - 1;   // ragged tail: recompute the last row, never stored
            wl[OFF_PB + c * 64 + lane] = (unsigned char)perm[cand * NDEV + lane];
        }
    }
    __syncthreads();
    uint16_t *ghr16 = reinterpret_cast<uint16_t *>(wl + off_ghr(NC));
    double *res = reinterpret_cast<double *>(wl + off_res(NC));
    {   // ---- a4: candidates 0, 1 by the first wavefront, 2, 3 by the second; lanes 2 t, 2 t + 1 share couple t ----
        int t = lane >> 1;
        const bool valid = t < 28 && !(lane & 1);
        if (t >= 28) t = 27;   // idle lanes repeat the last item and write nothing
        const int mc = (second ? 2 : 0) + t / 14, q = t % 14;
        int j1[2], j2[2];
        pair8_decode(2 * q, j1[0], j2[0]);
        pair8_decode(2 * q + 1, j1[1], j2[1]);
        const uint32_t gfull = match_couple_halves(cx, wl + OFF_PB + mc * 64, j1, j2);
        if (valid) {
            ghr16[mc * 28 + pair_index(j1[0], j2[0])] = (uint16_t)gfull;
            ghr16[mc * 28 + pair_index(j1[1], j2[1])] = (uint16_t)(gfull >> 16);
        }
    }
    __syncthreads();
    const int hc = (lane >> 3) & 3;
    if (second) {
        // ---- a2/a3: DataP of the four candidates, lane = (candidate, stage) ----
        double dp = stage_datap(W_dp, *reinterpret_cast<const uint2 *>(wl + OFF_PB + hc * 64 + 8 * cx.hv));
        dp = fmax(dp, dpp_move<DPP_XOR1>(dp));
        dp = fmax(dp, dpp_move<DPP_XOR2>(dp));
        dp = fmax(dp, dpp_move<DPP_HALF_MIRROR>(dp));
        if (cx.hv == 0 && lane < NC * 8) res[NC + hc] = dp;
        if (ghat_out != nullptr) {
            const int u = lane >> 3, v = lane & 7;
            const int pi = pair_index(u < v ? u : v, u < v ? v : u);
#pragma nounroll
            for (int c = 0; c < NC; c++)
                if (grp * NC + c < P) ghat_out[(grp * NC + c) * 64 + lane] = u == v ? 0.0 : cx.rank_val[ghr16[c * 28 + pi]];
        }
        __syncthreads();
        return;
    }
    // ---- a5: Held-Karp in registers, the two halves of the wavefront sharing each candidate (see hk_registers) ----
    const bool relabel = lane >= 32;
    const int v = relabel ? hk_swap01(cx.hv) : cx.hv;
    double G[8];
    G[0] = 0.0;
#pragma unroll
    for (int d = 1; d < 8; d++) {
        const int u = v ^ (relabel ? hk_swap01(d) : d);
        G[d] = cx.rank_val[ghr16[hc * 28 + pair_index(u < v ? u : v, u < v ? v : u)]];
    }
    const double pp = hk_registers<true>(G, lane);
    __syncthreads();
    // ---- a6 ----
    const size_t cand = grp * NC + hc;
    if (cx.hv == 0 && lane < NC * 8 && cand < P) {
        const double dp = res[NC + hc];
        if (cost != nullptr) cost[cand] = __dadd_rn(dp, pp);
        if (datap_out != nullptr) datap_out[cand] = dp;
    }
}

// W_pp[a][b], a != b, for the proposals: from the LDS copy where there is one; with 32 candidates per
// wavefront (no room for it) through the rank tables, rank_val[rank[a][b]] being the same bits.
template <int NC>
__device__ __forceinline__ double wpp(const wave_ctx &cx, uint32_t a, uint32_t b)
{
    if (wpp_in_lds(NC, true)) return cx.Wpp[a * NDEV + b];
    return cx.rank_val[cx.R[a * RSTRIDE + b]];
}

// The round's proposal for every candidate slot (Sec. 3.4, "Improving Local Search Strategy"): the fastest
// link inside stage j and inside stage jp of the current row, and of the four swaps of their end points
// the one of largest Gain; its two positions (first < second) go to prop[2 c], prop[2 c + 1].
template <int NC>
__device__ __forceinline__ void propose_gain4(const wave_ctx &cx, const unsigned char *pbcur, unsigned char *prop, int j,
                                              int jp)
{
    const int lane = cx.lane, sub = lane & 15;   // 16 lanes per candidate, four candidates per pass
    int ea_i, ea_k, eb_i, eb_k;                  // the two slot pairs this lane looks at when the fastest link is sought
    pair8_decode(sub, ea_i, ea_k);
    pair8_decode(sub < 12 ? sub + 16 : sub, eb_i, eb_k);
    const int Cj = 8 * j, Cjp = 8 * jp;
#pragma nounroll
    for (int pass = 0; pass < NC / 4; pass++) {
        // ---- proposal for candidate slot 4 * pass + lane / 16 by its 16 lanes: registers and
        // lane exchanges only, apart from the table gathers ----
        const int pslot = 4 * pass + (lane >> 4);
        const unsigned char *pc = pbcur + pslot * 64;
        const uint2 cdev[2] = {*reinterpret_cast<const uint2 *>(pc + Cj), *reinterpret_cast<const uint2 *>(pc + Cjp)};
        int slot[2][2];
#pragma unroll
        for (int s = 0; s < 2; s++) {
            // fastest link inside the stage: key = (rank << 8) | pair index, first minimiser wins;
            // this lane looks at slot pairs `sub` and `sub + 16`
            uint32_t key = ((uint32_t)cx.R[byte_at(cdev[s], ea_i) * RSTRIDE + byte_at(cdev[s], ea_k)] << 8) | (uint32_t)sub;
            const uint32_t kb = ((uint32_t)cx.R[byte_at(cdev[s], eb_i) * RSTRIDE + byte_at(cdev[s], eb_k)] << 8) | (uint32_t)(sub + 16);
            if (sub < 12 && kb < key) key = kb;
            key = min(key, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)key, 0x128, 0xF, 0xF, true));   // row_ror:8
            key = min(key, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)key, 0x124, 0xF, 0xF, true));   // row_ror:4
            key = min(key, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)key, 0x122, 0xF, 0xF, true));   // row_ror:2
            key = min(key, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)key, 0x121, 0xF, 0xF, true));   // row_ror:1
            pair8_decode((int)(key & 0xFFu), slot[s][0], slot[s][1]);
        }
        // every quad of lanes computes the four means itself: lanes 0,1 the mean over C_j' of w[x][.] for
        // x = d1, d2; lanes 2,3 the mean over C_j of w[y][.] for y = d1', d2'
        double mean;
        {
            const int side = (lane >> 1) & 1, which = lane & 1;
            const uint32_t dv = byte_at(cdev[side], side == 0 ? slot[0][which] : slot[1][which]);
            const uint2 other = cdev[side ^ 1];
            double sum = 0.0;
#pragma unroll
            for (int i = 0; i < 8; i++) sum = __dadd_rn(sum, wpp<NC>(cx, dv, byte_of(other, i)));
            mean = sum * 0.125;   // the mean over 8 entries; exact scaling, the same bits as the division
        }
        const double link0 = wpp<NC>(cx, byte_at(cdev[0], slot[0][0]), byte_at(cdev[0], slot[0][1]));
        const double link1 = wpp<NC>(cx, byte_at(cdev[1], slot[1][0]), byte_at(cdev[1], slot[1][1]));
        const double mx[2] = {dpp_move<0x00>(mean), dpp_move<0x55>(mean)};   // lane 0 / lane 1 of the quad
        const double my[2] = {dpp_move<0xAA>(mean), dpp_move<0xFF>(mean)};   // lane 2 / lane 3
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
        if (sub == 0) {   // positions, first < second
            prop[2 * pslot] = (unsigned char)(Cj + slot[0][bk >> 1]);
            prop[2 * pslot + 1] = (unsigned char)(Cjp + slot[1][bk & 1]);
        }
    }
}

// ---- offspring of the evolutionary search made inside the local-search kernel (4 candidates per wavefront)
// The lane's share of the two parents' rows (positions sub, sub + 16, sub + 32, sub + 48 of the lane's
// candidate): loaded ahead of the table set-up, which hides the selection draw and the loads.
struct parent_rows {
    int d1[4], d2[4];
};
__device__ __forceinline__ parent_rows load_parents4(const dtfm_offspring_src &src, size_t cand0, size_t L, int lane)
{
    size_t kk = cand0 + (lane >> 4);
    if (kk >= L) kk = L - 1;
    const philox_out sel = philox4x32_10(0u, (uint32_t)kk, src.g, STREAM_SELECT, src.k0, src.k1);
    const int32_t *par1 = src.pop + (size_t)randint(sel.w[0], (uint32_t)src.P) * NDEV;
    const int32_t *par2 = src.pop + (size_t)randint(sel.w[1], (uint32_t)src.P) * NDEV;
    parent_rows r;
#pragma unroll
    for (int i = 0; i < 4; i++) {
        r.d1[i] = par1[(lane & 15) + 16 * i];
        r.d2[i] = par2[(lane & 15) + 16 * i];
    }
    return r;
}

// Sec. 3.4 selection, crossover and mutation for the four offspring cand0 .. cand0 + 3 of a wavefront (16
// lanes each), the rows left as bytes at `rows` (4 x 64, stage-major). Same draws and steps as
// k_make_offspring: two uniform parents; the child starts as parent 1; m_x times a random device that parent
// 2 keeps in another stage is swapped with the device at a random slot of that stage; m_m random
// transpositions. The draws of MK_STEPS steps are made by the 16 lanes (two steps per Philox block), the
// dependent swaps by the first lane of each candidate.
__device__ __forceinline__ void make_offspring4(const wave_ctx &cx, const dtfm_offspring_src &src, const parent_rows &par,
                                                size_t cand0, size_t L, unsigned char *rows, unsigned char *scratch)
{
    const int lane = cx.lane, c = lane >> 4, sub = lane & 15;
    size_t kk = cand0 + c;
    if (kk >= L) kk = L - 1;   // ragged tail: the last offspring again, never stored
    const uint32_t k = (uint32_t)kk;
    unsigned char *child = rows + c * 64, *pos_child = scratch + c * 64, *pos_par2 = scratch + 4 * 64 + c * 64;
    unsigned char *draw_a = scratch + 8 * 64 + c * MK_STEPS, *draw_b = draw_a + 4 * MK_STEPS;
#pragma unroll
    for (int i = 0; i < 4; i++) {
        const int q = sub + 16 * i;
        const int d = par.d1[i];
        child[q] = (unsigned char)d;
        pos_child[d] = (unsigned char)q;
        pos_par2[par.d2[i]] = (unsigned char)q;
    }
    WAVE_LDS_SYNC();
    for (int t0 = 0; t0 < src.m_x; t0 += MK_STEPS) {
        const int steps = min(MK_STEPS, src.m_x - t0);
        if (2 * sub < steps) {
            const philox_out o = philox4x32_10((uint32_t)(t0 / 2 + sub), k, src.g, STREAM_CROSSOVER, src.k0, src.k1);
#pragma unroll
            for (int h = 0; h < 2; h++) {
                const int d = (int)randint(o.w[2 * h], (uint32_t)NDEV);
                const int slot = (int)randint(o.w[2 * h + 1], 8u);
                draw_a[2 * sub + h] = (unsigned char)d;
                draw_b[2 * sub + h] = (unsigned char)((pos_par2[d] & ~7) + slot);   // the slot of the stage parent 2 keeps d in
            }
        }
        WAVE_LDS_SYNC();
        if (sub == 0) {
            // all draws of the chunk into registers first: a step then waits for one LDS round trip only
            uint32_t da[MK_STEPS / 4], db[MK_STEPS / 4];
#pragma unroll
            for (int w = 0; w < MK_STEPS / 4; w++) {
                da[w] = reinterpret_cast<const uint32_t *>(draw_a)[w];
                db[w] = reinterpret_cast<const uint32_t *>(draw_b)[w];
            }
#pragma unroll
            for (int t = 0; t < MK_STEPS; t++) {
                if (t < steps) {
                    const int d = (da[t >> 2] >> (8 * (t & 3))) & 0xFF, qb = (db[t >> 2] >> (8 * (t & 3))) & 0xFF;
                    const int qa = pos_child[d];
                    const int e = child[qb];
                    if ((qa >> 3) != (qb >> 3)) {
                        child[qa] = (unsigned char)e;
                        child[qb] = (unsigned char)d;
                        pos_child[e] = (unsigned char)qa;
                        pos_child[d] = (unsigned char)qb;
                    }
                }
            }
        }
        WAVE_LDS_SYNC();
    }
    for (int t0 = 0; t0 < src.m_m; t0 += MK_STEPS) {
        const int steps = min(MK_STEPS, src.m_m - t0);
        if (2 * sub < steps) {
            const philox_out o = philox4x32_10((uint32_t)(t0 / 2 + sub), k, src.g, STREAM_MUTATION, src.k0, src.k1);
#pragma unroll
            for (int h = 0; h < 2; h++) {
                draw_a[2 * sub + h] = (unsigned char)randint(o.w[2 * h], (uint32_t)NDEV);
                draw_b[2 * sub + h] = (unsigned char)randint(o.w[2 * h + 1], (uint32_t)NDEV);
            }
        }
        WAVE_LDS_SYNC();
        if (sub == 0) {
            for (int t = 0; t < steps; t++) {
                const int a = draw_a[t], b = draw_b[t];
                const unsigned char x = child[a];
                child[a] = child[b];
                child[b] = x;
            }
        }
        WAVE_LDS_SYNC();
    }
}

// ---- Sec. 3.4 local search with the paper's four-candidate neighbourhood, all rounds in one launch
// Each wavefront carries its candidates through every round: propose a swap (fastest link inside
// each of the round's two stages, the four end-point swaps ranked by the paper's Gain), evaluate the
// swapped allocation with eval_group, keep it iff strictly cheaper. The fastest link is found on the
// ranks (same order and same ties as the weights); the Gain sums use the fp64 weights in slot order.
// With MAKE (4 candidates per wavefront) the rows are not read but made here: the offspring of `src`.
template <int NC, bool MAKE>
__global__ void __launch_bounds__(WAVES_PER_BLOCK * 64)
k_ls_gain4_fast64(const double *__restrict__ W_dp, const double *__restrict__ W_pp,
                  const uint16_t *__restrict__ rank_tab, const double *__restrict__ rank_val,
                  int32_t *__restrict__ perm, size_t P, int moves, double *__restrict__ cost,
                  int64_t *__restrict__ applied, dtfm_offspring_src src)
{
    extern __shared__ __align__(16) unsigned char smem[];
    parent_rows par = {};
    if (MAKE && NC == 4)   // the first group's parents, in flight during the table set-up
        par = load_parents4(src, ((size_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6)) * NC, P, threadIdx.x & 63);
    const wave_ctx cx = wave_setup<NC, true>(smem, rank_tab, rank_val, W_dp, W_pp);
    const int lane = cx.lane, wave = threadIdx.x >> 6;
    unsigned char *wl = cx.wl;
    unsigned char *pbcur = wl + off_pbcur(NC), *prop = wl + off_prop(NC);
    const double *res = reinterpret_cast<const double *>(wl + off_res(NC));
    double *curc = reinterpret_cast<double *>(wl + off_curc(NC));
    uint32_t *ghr32 = reinterpret_cast<uint32_t *>(wl + off_ghr(NC)), *ghrcur32 = reinterpret_cast<uint32_t *>(wl + off_ghrcur(NC));
    const int wpb = blockDim.x >> 6;   // wavefronts per workgroup: WAVES_PER_BLOCK, fewer for small populations
    const size_t nwaves = (size_t)gridDim.x * wpb;
    const size_t ngroups = (P + NC - 1) / NC;
    for (size_t grp = (size_t)blockIdx.x * wpb + wave; grp < ngroups; grp += nwaves) {
        if (MAKE && NC == 4) {
            if (grp >= nwaves) par = load_parents4(src, grp * NC, P, lane);   // later groups of a wavefront
            make_offspring4(cx, src, par, grp * NC, P, wl + OFF_PB, wl + off_mk(NC));
#pragma unroll
            for (int c = 0; c < NC; c++) pbcur[c * 64 + lane] = wl[OFF_PB + c * 64 + lane];
        } else {
#pragma unroll 8
            for (int c = 0; c < NC; c++) {
                size_t cand = grp * NC + c;
                if (cand >= P) cand = P - 1;
                const unsigned char d = (unsigned char)perm[cand * NDEV + lane];
                wl[OFF_PB + c * 64 + lane] = d;
                pbcur[c * 64 + lane] = d;
            }
        }
        WAVE_LDS_SYNC();
        // round -1 prices the rows as they are; each later round prices the rows with the proposed swap
#pragma nounroll
        for (int r = -1; r < moves; r++) {
            int j = -1, jp = -1;
            if (r >= 0) {
                pair8_decode(r % 28, j, jp);
                propose_gain4<NC>(cx, pbcur, prop, j, jp);
                WAVE_LDS_SYNC();
                // ---- trial rows; the evaluation starts from the current rows' coarsened graphs ----
#pragma unroll 8
                for (int c = 0; c < NC; c++) {
                    const int ta = prop[2 * c], tb = prop[2 * c + 1];
                    const int src = lane == ta ? tb : (lane == tb ? ta : lane);
                    wl[OFF_PB + c * 64 + lane] = pbcur[c * 64 + src];
                }
                for (int w = lane; w < NC * 14; w += 64) ghr32[w] = ghrcur32[w];
                WAVE_LDS_SYNC();
            }
            eval_group<NC, true>(cx, nullptr, grp * NC, P, j, jp);
            if (r < 0) {
                if (lane < NC) curc[lane] = res[lane];
                for (int w = lane; w < NC * 14; w += 64) ghrcur32[w] = ghr32[w];
                WAVE_LDS_SYNC();
                continue;
            }
            // ---- accept iff strictly cheaper ----
            bool mine = false;
            if (lane < NC) {
                const double t = res[lane];
                mine = t < curc[lane];
                if (mine) curc[lane] = t;
            }
            const uint64_t takes = __ballot(mine);
#pragma unroll 8
            for (int c = 0; c < NC; c++) {
                const bool take = (takes >> c) & 1;   // wave-uniform
                if (take) pbcur[c * 64 + lane] = wl[OFF_PB + c * 64 + lane];
            }
            for (int w = lane; w < NC * 14; w += 64)
                if ((takes >> (w / 14)) & 1) ghrcur32[w] = ghr32[w];
            if (applied != nullptr && lane < NC && grp * NC + lane < P) {
                const long long ta = prop[2 * lane], tb = prop[2 * lane + 1];
                applied[(grp * NC + lane) * (size_t)moves + r] = mine ? ta * NDEV - ta * (ta + 1) / 2 + (tb - ta - 1) : -1ll;
            }
            WAVE_LDS_SYNC();
        }
#pragma unroll 8
        for (int c = 0; c < NC; c++) {
            const size_t cand = grp * NC + c;
            if (cand < P) perm[cand * NDEV + lane] = pbcur[c * 64 + lane];
        }
        if (lane < NC && grp * NC + lane < P) cost[grp * NC + lane] = curc[lane];
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
    DTFM_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_eval_fast64<32>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, lds_total(32, false)));
    DTFM_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_eval_fast64<8>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, lds_total(8, false)));
    DTFM_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_eval_fast64<4>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, lds_total(4, false)));
    DTFM_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_eval_fast64_paired),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, lds_total(4, false)));
    DTFM_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_ls_gain4_fast64<32, false>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, lds_total(32, true)));
    DTFM_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_ls_gain4_fast64<8, false>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, lds_total(8, true)));
    DTFM_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_ls_gain4_fast64<4, false>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, lds_total(4, true)));
    DTFM_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_ls_gain4_fast64<4, true>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, lds_total(4, true)));
    int rc = dtfm_fast64_allpairs_prepare();
    if (rc != DTFM_OK) return rc;
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

// Candidates per wavefront pass. 32 keep every lane of the matching phase busy (32 * 14 couples = 7
// full passes) and are used once that still gives every wavefront slot of the chip a pass; 8 fill
// Held-Karp's lanes. Up to two wavefronts per SIMD of 4 candidates each (8192 candidates) the shorter
// passes of 4 win: their matching and Held-Karp programmes use the idle lanes to split the work.
static int group_size(const dtfm_problem *pr, size_t rows)
{
    const size_t simds = 4 * (size_t)pr->f64_grid;
    if (rows >= 32 * 2 * simds) return 32;
    return rows <= 8 * simds ? 4 : 8;
}

// Wavefronts per workgroup. The LDS tables allow one workgroup per CU, so a launch with fewer
// workgroups than CUs leaves CUs idle: the workgroups get as few wavefronts (two at least, which
// still load the tables in reasonable time) as give every pass a wavefront of its own on the chip's
// CUs; beyond 8 per CU the wavefronts take several passes each.
static int waves_per_block(const dtfm_problem *pr, size_t passes)
{
    int w = 2;
    while (w < WAVES_PER_BLOCK && (passes + w - 1) / w > (size_t)pr->f64_grid) w <<= 1;
    return w;
}

template <int NC>
static void launch_eval(const dtfm_problem *pr, const int32_t *perm, size_t rows, double *cost, double *ghat,
                        double *datap, hipStream_t st)
{
    size_t passes = (rows + NC - 1) / NC;
    const int wpb = waves_per_block(pr, passes);
    size_t blocks = (passes + wpb - 1) / wpb;
    if (blocks > (size_t)pr->f64_grid) blocks = pr->f64_grid;
    hipLaunchKernelGGL(k_eval_fast64<NC>, dim3((unsigned)blocks), dim3(wpb * 64), lds_total(NC, false, wpb), st,
                       pr->W_dp, pr->f64_rank, pr->f64_rank_val, perm, rows, cost, ghat, datap);
}

// With 32 candidates per pass the chip's wavefront slots (two per SIMD) take 65,536 candidates per
// round of passes. What is left after the last full round, if it is not nearly a round itself, goes to
// a launch of its own with a smaller group size instead of costing a whole further round.
static size_t full_rounds_rows(const dtfm_problem *pr, size_t rows)
{
    const size_t round = 32 * 2 * 4 * (size_t)pr->f64_grid;
    const size_t rest = rows % round;
    return (rows >= round && rest != 0 && rest <= round * 3 / 4) ? rows - rest : rows;
}

int dtfm_fast64_enqueue(const dtfm_problem *pr, const int32_t *perm, size_t rows, double *cost, double *ghat,
                        double *datap, hipStream_t st)
{
    if (rows == 0) return DTFM_OK;
    const size_t head = full_rounds_rows(pr, rows);
    if (head < rows) {
        int rc = dtfm_fast64_enqueue(pr, perm, head, cost, ghat, datap, st);
        if (rc != DTFM_OK) return rc;
        return dtfm_fast64_enqueue(pr, perm + head * NDEV, rows - head, cost ? cost + head : nullptr,
                                   ghat ? ghat + head * 64 : nullptr, datap ? datap + head : nullptr, st);
    }
    const size_t passes4 = (rows + 3) / 4;
    if (group_size(pr, rows) == 4 && passes4 <= 4 * (size_t)pr->f64_grid) {
        // one group of four per SIMD at most: a pair of wavefronts per group
        const int cw = passes4 > 2 * (size_t)pr->f64_grid ? 4 : 2;
        hipLaunchKernelGGL(k_eval_fast64_paired, dim3((unsigned)((passes4 + cw - 1) / cw)), dim3(2 * cw * 64),
                           lds_total(4, false, cw), st, pr->W_dp, pr->f64_rank, pr->f64_rank_val, perm, rows, cost, ghat,
                           datap);
        DTFM_HIP(hipGetLastError());
        return DTFM_OK;
    }
    switch (group_size(pr, rows)) {
    case 32: launch_eval<32>(pr, perm, rows, cost, ghat, datap, st); break;
    case 8: launch_eval<8>(pr, perm, rows, cost, ghat, datap, st); break;
    default: launch_eval<4>(pr, perm, rows, cost, ghat, datap, st); break;
    }
    DTFM_HIP(hipGetLastError());
    return DTFM_OK;
}

template <int NC>
static void launch_ls(const dtfm_problem *pr, int32_t *perm, size_t rows, int moves, double *cost, int64_t *applied,
                      hipStream_t st)
{
    size_t passes = (rows + NC - 1) / NC;
    const int wpb = waves_per_block(pr, passes);
    size_t blocks = (passes + wpb - 1) / wpb;
    if (blocks > (size_t)pr->f64_grid) blocks = pr->f64_grid;
    hipLaunchKernelGGL((k_ls_gain4_fast64<NC, false>), dim3((unsigned)blocks), dim3(wpb * 64), lds_total(NC, true, wpb), st,
                       pr->W_dp, pr->W_pp, pr->f64_rank, pr->f64_rank_val, perm, rows, moves, cost, applied,
                       dtfm_offspring_src{});
}

bool dtfm_fast64_ls_makes_offspring(const dtfm_problem *pr, size_t rows, int moves)
{
    return rows > 0 && moves >= 0 && full_rounds_rows(pr, rows) == rows && group_size(pr, rows) == 4;
}

int dtfm_fast64_offspring_ls_gain4_enqueue(const dtfm_problem *pr, const dtfm_offspring_src &src, int32_t *perm,
                                           size_t rows, int moves, double *cost, hipStream_t st)
{
    if (!dtfm_fast64_ls_makes_offspring(pr, rows, moves)) return DTFM_ERR_ARG;
    size_t passes = (rows + 3) / 4;
    const int wpb = waves_per_block(pr, passes);
    size_t blocks = (passes + wpb - 1) / wpb;
    if (blocks > (size_t)pr->f64_grid) blocks = pr->f64_grid;
    hipLaunchKernelGGL((k_ls_gain4_fast64<4, true>), dim3((unsigned)blocks), dim3(wpb * 64), lds_total(4, true, wpb), st,
                       pr->W_dp, pr->W_pp, pr->f64_rank, pr->f64_rank_val, perm, rows, moves, cost, (int64_t *)nullptr,
                       src);
    DTFM_HIP(hipGetLastError());
    return DTFM_OK;
}

int dtfm_fast64_ls_gain4_enqueue(const dtfm_problem *pr, int32_t *perm, size_t rows, int moves, double *cost,
                                 int64_t *applied, hipStream_t st)
{
    if (rows == 0) return DTFM_OK;
    const size_t head = full_rounds_rows(pr, rows);
    if (head < rows) {
        int rc = dtfm_fast64_ls_gain4_enqueue(pr, perm, head, moves, cost, applied, st);
        if (rc != DTFM_OK) return rc;
        return dtfm_fast64_ls_gain4_enqueue(pr, perm + head * NDEV, rows - head, moves, cost + head,
                                            applied ? applied + head * (size_t)moves : nullptr, st);
    }
    switch (group_size(pr, rows)) {
    case 32: launch_ls<32>(pr, perm, rows, moves, cost, applied, st); break;
    case 8: launch_ls<8>(pr, perm, rows, moves, cost, applied, st); break;
    default: launch_ls<4>(pr, perm, rows, moves, cost, applied, st); break;
    }
    DTFM_HIP(hipGetLastError());
    return DTFM_OK;
}
