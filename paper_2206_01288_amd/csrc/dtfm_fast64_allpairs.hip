// Sec. 3.4 local search over ALL position swaps for the 64-device shape (N = 64, D_dp = 8, D_pp = 8),
// with incremental move evaluation: one wavefront carries one candidate through all rounds and, per
// round, prices all 2016 swaps exactly (the same bits as evaluating each swapped allocation from
// scratch) without redoing the parts of Eqs. 2-4 that a swap leaves alone.
//
// A swap of slot i of stage j with slot i' of stage j' (j < j') changes
//   * DataP of stages j and j' (Eq. 2): their 2 x 8 row sums are redone in the new slot order;
//   * the 12 coarsened edges (j,k), (j',k), k outside {j,j'} (Eq. 3): in each of them ONE row of the
//     block is replaced. With F[j][k][i][c] = bottleneck optimum of the rows of C_j except slot i into
//     the columns of C_k except c (a 7-row subset programme, done once per round for every (j,k,i)),
//     the new edge is min_c max(F[j][k][i][c], w[new device][C_k[c]]): 15 operations;
//   * the edge (j,j'): a row and a column change; it is redone by the 8-row subset programme;
//   * Held-Karp (Eq. 4) is rerun on the patched coarsened graph, eight swaps per pass.
// A swap inside a stage changes only the order of that stage's DataP sums.
// The unchanged edges and the F tables are also where the round's own coarsened graph comes from
// (replacing a row by itself), so a round costs 448 seven-row programmes, 1792 eight-row programmes
// and 225 Held-Karp passes instead of 2016 full evaluations (56,448 eight-row programmes).
#include "dtfm_fast64_device.h"

namespace {

// ---- per-wavefront LDS slice ----
constexpr int N_MOVES = NDEV * (NDEV - 1) / 2;
constexpr int AP_OFF_CUR = 0;                          // u8 [64]: the candidate's current row, stage-major
constexpr int AP_OFF_EDGE = AP_OFF_CUR + 64;           // u16 [64 + 64 + 2*64*8]: edge ranks, one index space:
constexpr int AP_EDGE_GBM = 0;                         //   [u][v]      the round's own coarsened graph
constexpr int AP_EDGE_SCR = 64;                        //   [mv]        edge (j,j') after swap mv = 8 i + i'
constexpr int AP_EDGE_REP = 128;                       //   [side][mv][k] edge (j,k) (side 0) / (j',k) (side 1) after swap mv
constexpr int AP_EDGE_SCR_ODD = 128 + 1024;            //   [mv]        the same for odd batches, in the unused F[0][0] block
constexpr int AP_OFF_F = AP_OFF_EDGE + (128 + 1024) * 2;   // u16 [j][k][i][c]
constexpr int AP_OFF_DPM = AP_OFF_F + 8 * 8 * 8 * 8 * 2;   // double [64]: DataP after swap mv
constexpr int AP_OFF_DPB = AP_OFF_DPM + 64 * 8;            // double [8]: DataP of every stage of the current row
constexpr int AP_OFF_LIST = AP_OFF_DPB + 64;               // u8 [64]: the swaps of the batch that can still win
constexpr int AP_WAVE_BYTES = AP_OFF_LIST + 64;
constexpr int AP_LDS_TOTAL = LDS_TABLES + WAVES_PER_BLOCK * AP_WAVE_BYTES;
static_assert(AP_OFF_F % 16 == 0 && AP_OFF_DPM % 8 == 0 && AP_WAVE_BYTES % 16 == 0, "alignment");
static_assert(AP_LDS_TOTAL <= 160 * 1024, "LDS budget of a CU");

__device__ __forceinline__ uint2 split64(uint64_t v) { return make_uint2((uint32_t)v, (uint32_t)(v >> 32)); }
__device__ __forceinline__ uint64_t join64(uint2 v) { return ((uint64_t)v.y << 32) | v.x; }
// the 8 device bytes of a stage with byte i taken out (bytes above move down; the top byte is unused)
__device__ __forceinline__ uint2 drop_byte(uint2 v, int i)
{
    const uint64_t x = join64(v), low = (1ull << (8 * i)) - 1;
    return split64((x & low) | ((x >> 8) & ~low));
}
// ... with byte i replaced by device d
__device__ __forceinline__ uint2 put_byte(uint2 v, int i, uint32_t d)
{
    const uint64_t x = join64(v);
    return split64((x & ~(0xFFull << (8 * i))) | ((uint64_t)d << (8 * i)));
}

// new value of an edge whose block gets row `dev` in place of the row left out of F:
// min_c max(F[c], rank[dev][cols[c]])
__device__ __forceinline__ uint32_t replaced_row(const uint16_t *R, const uint16_t *F, uint32_t dev, uint2 cols)
{
    const uint4 f = *reinterpret_cast<const uint4 *>(F);
    const uint32_t fw[4] = {f.x, f.y, f.z, f.w};
    uint32_t best = 0xFFFFFFFFu;
#pragma unroll
    for (int c = 0; c < 8; c++) {
        const uint32_t fc = (fw[c >> 1] >> (16 * (c & 1))) & 0xFFFFu;
        const uint32_t w = R[dev * RSTRIDE + byte_of(cols, c)];
        best = min(best, max(fc, w));
    }
    return best;
}

// running minimum under (cost, key)
__device__ __forceinline__ void keep_best(double &bc, uint32_t &bk, double c, uint32_t k)
{
    if (c < bc || (c == bc && k < bk)) {
        bc = c;
        bk = k;
    }
}

__global__ void __launch_bounds__(WAVES_PER_BLOCK * 64)
k_ls_allpairs_fast64(const double *__restrict__ W_dp, const uint16_t *__restrict__ rank_tab,
                     const double *__restrict__ rank_val_g, int32_t *__restrict__ perm, size_t P, int moves,
                     double *__restrict__ cost, int64_t *__restrict__ applied, double *__restrict__ move_cost)
{
    extern __shared__ __align__(16) unsigned char smem[];
    stage_tables<false>(smem, rank_tab, rank_val_g, W_dp);
    __syncthreads();
    const uint16_t *R = reinterpret_cast<const uint16_t *>(smem);
    const double *rank_val = reinterpret_cast<const double *>(smem + LDS_RANK_BYTES);
    const double *Wdp = reinterpret_cast<const double *>(smem + LDS_RANK_BYTES + LDS_RVAL_BYTES);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned char *wl = smem + LDS_TABLES + wave * AP_WAVE_BYTES;
    unsigned char *cur = wl + AP_OFF_CUR;
    uint16_t *edge = reinterpret_cast<uint16_t *>(wl + AP_OFF_EDGE);
    uint16_t *F = reinterpret_cast<uint16_t *>(wl + AP_OFF_F);
    double *dpm = reinterpret_cast<double *>(wl + AP_OFF_DPM);
    double *dpb = reinterpret_cast<double *>(wl + AP_OFF_DPB);
    unsigned char *list = wl + AP_OFF_LIST;
    const int hm = lane >> 3, hv = lane & 7;   // Held-Karp role: swap slot within the pass, stage

    const int wpb = blockDim.x >> 6;   // wavefronts per workgroup: WAVES_PER_BLOCK, fewer when there are few rows
    for (size_t cand = (size_t)blockIdx.x * wpb + wave; cand < P; cand += (size_t)gridDim.x * wpb) {
        cur[lane] = (unsigned char)perm[cand * NDEV + lane];
        WAVE_LDS_SYNC();
        double cur_cost = 0.0;
#pragma nounroll
        for (int r = 0; r < moves; r++) {
            // ---- F tables: 448 seven-row programmes, two per lane: (j, k, i) and (j, k, i + 1) ----
#pragma nounroll
            for (int pass = 0; pass < 4; pass++) {
                int u = pass * 64 + lane;
                const bool valid = u < 224;
                if (!valid) u = 223;
                const int op = u >> 2, i0 = 2 * (u & 3);
                const int j = op / 7, kk = op - 7 * j, k = kk + (kk >= j ? 1 : 0);
                const uint2 cj = *reinterpret_cast<const uint2 *>(cur + 8 * j), ck = *reinterpret_cast<const uint2 *>(cur + 8 * k);
                const uint2 rowdev[2] = {drop_byte(cj, i0), drop_byte(cj, i0 + 1)};
                const uint2 coldev[2] = {ck, ck};
                uint32_t G[256];
                match_rows<7, false>(R, rowdev, coldev, G);
                if (valid) {
                    uint32_t lo[4], hi[4];
#pragma unroll
                    for (int m = 0; m < 4; m++) {
                        const uint32_t a = G[255 ^ (1 << (2 * m))], b = G[255 ^ (1 << (2 * m + 1))];
                        lo[m] = (a & 0xFFFFu) | (b << 16);
                        hi[m] = (a >> 16) | (b & 0xFFFF0000u);
                    }
                    uint16_t *f = F + ((j * 8 + k) * 8 + i0) * 8;
                    *reinterpret_cast<uint4 *>(f) = make_uint4(lo[0], lo[1], lo[2], lo[3]);
                    *reinterpret_cast<uint4 *>(f + 8) = make_uint4(hi[0], hi[1], hi[2], hi[3]);
                }
            }
            WAVE_LDS_SYNC();
            // ---- the row's own coarsened graph (slot 0 of C_u put back) and DataP of every stage ----
            {
                const int u = lane >> 3, v = lane & 7;
                const uint2 cu = *reinterpret_cast<const uint2 *>(cur + 8 * u), cv = *reinterpret_cast<const uint2 *>(cur + 8 * v);
                if (u != v) edge[AP_EDGE_GBM + lane] = (uint16_t)replaced_row(R, F + ((u * 8 + v) * 8) * 8, byte_of(cu, 0), cv);
                const double d = stage_datap(Wdp, cv);   // all 8 lanes groups compute all stages
                if (u == 0) dpb[v] = d;
            }
            WAVE_LDS_SYNC();
            double dp_base = dpb[0];
#pragma unroll
            for (int k = 1; k < 8; k++) dp_base = fmax(dp_base, dpb[k]);

            double bestc = INFINITY;
            uint32_t bestk = 0xFFFFFFFFu;   // key = 64 a + b of positions a < b: the order of the move indices
            // Held-Karp of the row itself (every group of 8 lanes computes the same)
            double pp_base;
            {
                double G[8];
                G[0] = 0.0;
#pragma unroll
                for (int d = 1; d < 8; d++) G[d] = rank_val[edge[AP_EDGE_GBM + hv * 8 + (hv ^ d)]];
                pp_base = hk_registers<false>(G, lane);
            }
            cur_cost = __dadd_rn(dp_base, pp_base);
            const bool prune = move_cost == nullptr;   // pricing every swap: nothing may be left out
            // 28 batches (j < j') of 64 swaps; Held-Karp takes eight swaps per pass
#pragma nounroll
            for (int batch = 0; batch < 28; batch++) {
                int j, jp;
                pair8_decode(batch, j, jp);
                const uint2 cj = *reinterpret_cast<const uint2 *>(cur + 8 * j), cjp = *reinterpret_cast<const uint2 *>(cur + 8 * jp);
                const int i = lane >> 3, ip = lane & 7;            // this lane's swap mv = lane
                const uint32_t x = byte_at(cj, i), y = byte_at(cjp, ip);
                // edges (j,k) and (j',k) with one row replaced
#pragma nounroll
                for (int k = 0; k < 8; k++) {
                    if (k == j || k == jp) continue;
                    const uint2 ck = *reinterpret_cast<const uint2 *>(cur + 8 * k);
                    edge[AP_EDGE_REP + lane * 8 + k] = (uint16_t)replaced_row(R, F + ((j * 8 + k) * 8 + i) * 8, y, ck);
                    edge[AP_EDGE_REP + (64 + lane) * 8 + k] = (uint16_t)replaced_row(R, F + ((jp * 8 + k) * 8 + ip) * 8, x, ck);
                }
                // edge (j,j'), for this batch and the next one at once (every other batch): lanes 0..31 take
                // this batch's swaps 2 l and 2 l + 1 (same i, i' and i' + 1), lanes 32..63 the next batch's
                if ((batch & 1) == 0) {
                    const int l = lane & 31, si = l >> 2, sp = 2 * (l & 3);
                    int sj = j, sjp = jp;
                    if (lane >= 32) pair8_decode(batch + 1 < 28 ? batch + 1 : batch, sj, sjp);
                    const uint2 scj = *reinterpret_cast<const uint2 *>(cur + 8 * sj), scjp = *reinterpret_cast<const uint2 *>(cur + 8 * sjp);
                    const uint32_t sx = byte_at(scj, si);
                    const uint2 rowdev[2] = {put_byte(scj, si, byte_at(scjp, sp)), put_byte(scj, si, byte_at(scjp, sp + 1))};
                    const uint2 coldev[2] = {put_byte(scjp, sp, sx), put_byte(scjp, sp + 1, sx)};
                    uint32_t G[256];
                    match_rows<8, false>(R, rowdev, coldev, G);
                    reinterpret_cast<uint32_t *>(edge + (lane < 32 ? AP_EDGE_SCR : AP_EDGE_SCR_ODD))[l] = G[255];
                }
                // DataP after the swap
                double dp_swap = fmax(stage_datap(Wdp, put_byte(cj, i, y)), stage_datap(Wdp, put_byte(cjp, ip, x)));
#pragma unroll
                for (int k = 0; k < 8; k++)
                    if (k != j && k != jp) dp_swap = fmax(dp_swap, dpb[k]);
                dpm[lane] = dp_swap;
                WAVE_LDS_SYNC();
                const int scr = (batch & 1) ? AP_EDGE_SCR_ODD : AP_EDGE_SCR;
                // rank of edge (v, u) of the coarsened graph after swap mv: the (j,j') edge, an edge of j or j' with a
                // row replaced, or an edge of the row's own graph
                auto edge_index = [&](int mv, int v, int u) -> int {
                    const bool vj = v == j, uj = u == j, vjp = v == jp, ujp = u == jp;
                    int e = AP_EDGE_GBM + v * 8 + u;
                    e = (vjp || ujp) ? AP_EDGE_REP + (64 + mv) * 8 + (vjp ? u : v) : e;
                    e = (vj || uj) ? AP_EDGE_REP + mv * 8 + (vj ? u : v) : e;
                    e = ((vj && ujp) || (vjp && uj)) ? scr + mv : e;
                    return e;
                };
                // ---- which swaps can still win: a lower bound on the cost after the swap against the cheapest so far ----
                // A path over the 8 stages gives each stage but its first an edge of its own (the one it is entered by),
                // each at least the stage's cheapest edge m_v, so Eq. 4 is at least sum_v m_v - max_v m_v; every rounded
                // path sum is within 7 roundings below its exact value and the bound is a sum of 7 non-negative terms,
                // within 7 roundings above its own, which the factor below more than covers. fl is monotone, so fl(DataP + bound) <= the swap's cost: a swap
                // whose bound is strictly above the cheapest cost so far (or the row's own) can neither be applied nor
                // tie with the winner, and is left out.
                int cnt = 64;
                if (prune) {
                    double thr = bestc;
#pragma unroll
                    for (int o = 32; o >= 1; o >>= 1) thr = fmin(thr, __shfl_xor(thr, o));
                    thr = fmin(thr, cur_cost);
                    double sum = 0.0, mx = 0.0;   // sum of the m_v but the largest, which stays in mx: no cancellation
#pragma unroll
                    for (int v = 0; v < 8; v++) {
                        uint32_t m = 0xFFFFu;
#pragma unroll
                        for (int u = 0; u < 8; u++)
                            if (u != v) m = min(m, (uint32_t)edge[edge_index(lane, v, u)]);
                        const double mw = rank_val[m];
                        if (v == 0) {
                            mx = mw;
                        } else {
                            sum = __dadd_rn(sum, fmin(mx, mw));
                            mx = fmax(mx, mw);
                        }
                    }
                    const double bound = __dadd_rn(dp_swap, __dmul_rn(sum, 1.0 - 1e-12));
                    const bool keep = !(bound > thr);
                    const uint64_t mask = __ballot(keep);
                    cnt = __popcll(mask);
                    const int rank = (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
                    if (keep) list[rank] = (unsigned char)lane;
                    WAVE_LDS_SYNC();
                }
#pragma nounroll
                for (int pass = 0; pass * 8 < cnt; pass++) {
                    const int slot = pass * 8 + hm;
                    const bool valid = slot < cnt;
                    const int mv = prune ? list[valid ? slot : cnt - 1] : slot;
                    double G[8];
                    G[0] = 0.0;
#pragma unroll
                    for (int d = 1; d < 8; d++) G[d] = rank_val[edge[edge_index(mv, hv, hv ^ d)]];
                    const double pp = hk_registers<false>(G, lane);
                    const double total = __dadd_rn(dpm[mv], pp);
                    const uint32_t a = 8 * j + (mv >> 3), b = 8 * jp + (mv & 7);
                    if (valid) keep_best(bestc, bestk, total, 64 * a + b);
                    if (move_cost != nullptr && hv == 0)
                        move_cost[cand * (size_t)N_MOVES + (a * NDEV - a * (a + 1) / 2 + (b - a - 1))] = total;
                }
                WAVE_LDS_SYNC();   // the next batch overwrites the slice
            }
            // ---- swaps inside a stage: only the order of that stage's sums changes ----
#pragma nounroll
            for (int pass = 0; pass < 4; pass++) {
                int t = pass * 64 + lane;
                const bool valid = t < 224;
                if (!valid) t = 223;
                const int s = t / 28, e = t - 28 * s;
                int i, k;
                pair8_decode(e, i, k);
                const uint2 cs = *reinterpret_cast<const uint2 *>(cur + 8 * s);
                const uint32_t di = byte_at(cs, i), dk = byte_at(cs, k);
                double d = stage_datap(Wdp, put_byte(put_byte(cs, i, dk), k, di));
#pragma unroll
                for (int q = 0; q < 8; q++)
                    if (q != s) d = fmax(d, dpb[q]);
                const uint32_t a = 8 * s + i, b = 8 * s + k;
                const double total = __dadd_rn(d, pp_base);
                if (valid) keep_best(bestc, bestk, total, 64 * a + b);
                if (move_cost != nullptr && valid)
                    move_cost[cand * (size_t)N_MOVES + (a * NDEV - a * (a + 1) / 2 + (b - a - 1))] = total;
            }
            // ---- cheapest swap of the round (lowest index on ties); applied iff strictly cheaper ----
#pragma unroll
            for (int o = 32; o >= 1; o >>= 1) {
                const double oc = __shfl_xor(bestc, o);
                const uint32_t ok = (uint32_t)__shfl_xor((int)bestk, o);
                keep_best(bestc, bestk, oc, ok);
            }
            if (move_cost != nullptr) break;   // pricing only: the row stays as it is
            const bool take = bestc < cur_cost;
            const int a = (int)(bestk >> 6), b = (int)(bestk & 63);
            if (applied != nullptr && lane == 0)
                applied[cand * (size_t)moves + r] = take ? (long long)a * NDEV - (long long)a * (a + 1) / 2 + (b - a - 1) : -1ll;
            WAVE_LDS_SYNC();
            if (take) {
                cur_cost = bestc;   // the same bits as pricing the new row from scratch
                const unsigned char da = cur[a], db = cur[b];
                WAVE_LDS_SYNC();
                if (lane == 0) {
                    cur[a] = db;
                    cur[b] = da;
                }
            }
            WAVE_LDS_SYNC();
        }
        if (move_cost == nullptr) {
            perm[cand * NDEV + lane] = cur[lane];
            if (lane == 0) cost[cand] = cur_cost;
        }
        WAVE_LDS_SYNC();
    }
}

}  // namespace

int dtfm_fast64_allpairs_prepare()
{
    DTFM_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_ls_allpairs_fast64),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, AP_LDS_TOTAL));
    return DTFM_OK;
}

// Wavefronts per workgroup: one workgroup fits a CU, so the workgroups get as few wavefronts (two at
// least) as give every row a wavefront of its own on the chip's CUs.
static int ap_waves_per_block(const dtfm_problem *pr, size_t rows)
{
    int w = 2;
    while (w < WAVES_PER_BLOCK && (rows + w - 1) / w > (size_t)pr->f64_grid) w <<= 1;
    return w;
}

// All `moves` >= 1 rounds of the ALL_PAIRS local search in one launch; perm in/out, cost out (the cost of
// the final rows), applied (rows * moves move indices or -1) may be null.
int dtfm_fast64_ls_allpairs_enqueue(const dtfm_problem *pr, int32_t *perm, size_t rows, int moves, double *cost,
                                    int64_t *applied, hipStream_t st)
{
    if (rows == 0 || moves <= 0) return DTFM_OK;
    const int wpb = ap_waves_per_block(pr, rows);
    size_t blocks = (rows + wpb - 1) / wpb;
    if (blocks > (size_t)pr->f64_grid) blocks = pr->f64_grid;
    hipLaunchKernelGGL(k_ls_allpairs_fast64, dim3((unsigned)blocks), dim3(wpb * 64), LDS_TABLES + wpb * AP_WAVE_BYTES, st, pr->W_dp,
                       pr->f64_rank, pr->f64_rank_val, perm, rows, moves, cost, applied, (double *)nullptr);
    DTFM_HIP(hipGetLastError());
    return DTFM_OK;
}

// The cost of every swap of every row: move_cost[p * 2016 + move index]; perm is only read.
int dtfm_fast64_move_costs_enqueue(const dtfm_problem *pr, const int32_t *perm, size_t rows, double *move_cost,
                                   hipStream_t st)
{
    if (rows == 0) return DTFM_OK;
    const int wpb = ap_waves_per_block(pr, rows);
    size_t blocks = (rows + wpb - 1) / wpb;
    if (blocks > (size_t)pr->f64_grid) blocks = pr->f64_grid;
    hipLaunchKernelGGL(k_ls_allpairs_fast64, dim3((unsigned)blocks), dim3(wpb * 64), LDS_TABLES + wpb * AP_WAVE_BYTES, st, pr->W_dp,
                       pr->f64_rank, pr->f64_rank_val, const_cast<int32_t *>(perm), rows, 1, (double *)nullptr,
                       (int64_t *)nullptr, move_cost);
    DTFM_HIP(hipGetLastError());
    return DTFM_OK;
}
