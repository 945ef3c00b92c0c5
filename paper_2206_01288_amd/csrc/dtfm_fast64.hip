// Fused population-evaluation kernel for the 64-device shape (N = 64, D_dp = 8, D_pp = 8): one
// wavefront evaluates one candidate end to end (Eqs. 1-4) with every intermediate in LDS.
//
//   DataP (Eq. 2)      lane = position; 8 gathers of W_dp (HBM/L2, 32 KiB table) summed in slot
//                      order (the device's own slot adds the zero diagonal), wave max.
//   Matching (Eq. 3)   the bottleneck value of a block depends only on the ORDER of its entries,
//                      so the kernel works on 16-bit ranks of W_pp (rank table in LDS, built once
//                      per problem) and maps the winning rank back to its fp64 value at the end:
//                      bit-identical to working on the doubles. Per stage pair a min-max dynamic
//                      programme over column subsets: g[S] = min_{c in S} max(g[S \ c],
//                      w[|S|-1][c]), g[all] = optimum. The 28 pairs are packed 7 to a 128-bit LDS
//                      word (4 groups, one lane per (group, S) item, packed 16-bit max/min).
//   Held-Karp (Eq. 4)  fp64 table [S][v] in LDS (reusing the matching tables' space), one lane per
//                      (S, v) item, layers of equal |S|.
// Which (group, S) or (S, v) item a lane handles in each step is fixed, so it comes from small
// constant tables built with the problem and held in registers across candidates.
#include "dtfm_internal.h"

#include <math.h>

#include <mutex>
#include <utility>
#include <vector>

namespace {

constexpr int NDEV = 64, NPAIR = 28, NGROUP = 4, PAIRS_PER_GROUP = 7;
constexpr int BINOM8[9] = {1, 8, 28, 56, 70, 56, 28, 8, 1};

// matching steps of layer k: each group's C(8,k) subsets padded to whole 16-lane passes
constexpr int match_steps(int k) { return (NGROUP * ((BINOM8[k] + 15) / 16) * 16 + 63) / 64; }   // k = 2..8
constexpr int hk_steps(int k) { return (BINOM8[k] * k + 63) / 64; }
constexpr int match_first(int k)
{
    int o = 0;
    for (int i = 2; i < k; i++) o += match_steps(i);
    return o;
}
constexpr int hk_first(int k)
{
    int o = 0;
    for (int i = 2; i < k; i++) o += hk_steps(i);
    return o;
}
constexpr int N_MSTEP = match_first(9);   // 19
constexpr int N_HSTEP = hk_first(9);      // 19

// LDS: shared rank table, then one slice per wavefront
constexpr int LDS_RANK_BYTES = NDEV * NDEV * 2;        // 8 KiB
constexpr int OFF_GT = 0;                              // u16 [4 groups][256 subsets][8]  16 KiB
constexpr int OFF_HK = 0;                              // fp64 [8 end nodes][256 subsets] (after matching)
constexpr int OFF_WST = 16384;                         // u16 [4 groups][64 entries][8]    4 KiB
constexpr int OFF_GHAT = OFF_WST + 4096;               // fp64 [8][8]
constexpr int OFF_PB = OFF_GHAT + 512;                 // u8 [64] perm, stage-major
constexpr int OFF_PBT = OFF_PB + 64;                   // u8 [64] perm, slot-major
constexpr int WAVE_LDS_BYTES = OFF_PBT + 64;           // 21120
constexpr int WAVES_PER_BLOCK = 7;
constexpr int LDS_TOTAL = LDS_RANK_BYTES + WAVES_PER_BLOCK * WAVE_LDS_BYTES;

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

struct step_consts {
    uint32_t m_nib[N_MSTEP], m_meta[N_MSTEP];
    uint32_t h_nib[N_HSTEP], h_a[N_HSTEP], h_b[N_HSTEP];
};

// One layer of the packed matching programme: every lane owns (group, S) items with |S| = K.
template <int K>
__device__ __forceinline__ void match_layer(unsigned char *wl, const step_consts &sc)
{
#pragma unroll
    for (int s = 0; s < match_steps(K); s++) {
        const uint32_t nib = sc.m_nib[match_first(K) + s], meta = sc.m_meta[match_first(K) + s];
        const uint32_t self = meta & 0xFFFFu;                 // byte offset of gt[group][S]
        const uint32_t wbase = ((meta >> 16) & 3u) * 1024u;   // byte offset of wst[group]
        uint4 acc = make_uint4(0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu);
#pragma unroll
        for (int t = 0; t < K; t++) {
            const uint32_t c = (nib >> (4 * t)) & 15u;
            const uint4 g = *reinterpret_cast<const uint4 *>(wl + OFF_GT + (self ^ (16u << c)));
            const uint4 w = *reinterpret_cast<const uint4 *>(wl + OFF_WST + wbase + (K - 1) * 128 + c * 16u);
            acc.x = pk_min(acc.x, pk_max(g.x, w.x));
            acc.y = pk_min(acc.y, pk_max(g.y, w.y));
            acc.z = pk_min(acc.z, pk_max(g.z, w.z));
            acc.w = pk_min(acc.w, pk_max(g.w, w.w));
        }
        if (meta >> 31) *reinterpret_cast<uint4 *>(wl + OFF_GT + self) = acc;
        __builtin_amdgcn_sched_barrier(0);   // keep one step's loads in flight, not the whole layer's
    }
    WAVE_LDS_SYNC();
}

// One layer of Held-Karp: every lane owns (S, v) items with |S| = K.
template <int K>
__device__ __forceinline__ void hk_layer(unsigned char *wl, const step_consts &sc)
{
#pragma unroll
    for (int s = 0; s < hk_steps(K); s++) {
        const uint32_t nib = sc.h_nib[hk_first(K) + s], a = sc.h_a[hk_first(K) + s], b = sc.h_b[hk_first(K) + s];
        const uint32_t rest8 = a & 0xFFFFu;       // byte offset of tab[0][S \ v]
        const uint32_t v8 = a >> 16;              // v * 8
        double best = INFINITY;
#pragma unroll
        for (int t = 0; t < K - 1; t++) {
            const uint32_t u = (nib >> (4 * t)) & 15u;
            const double x = *reinterpret_cast<const double *>(wl + OFF_HK + rest8 + u * 2048u);
            const double e = *reinterpret_cast<const double *>(wl + OFF_GHAT + u * 64u + v8);
            best = fmin(best, __dadd_rn(x, e));
        }
        if (b >> 31) *reinterpret_cast<double *>(wl + OFF_HK + (b & 0xFFFFu)) = best;
        __builtin_amdgcn_sched_barrier(0);
    }
    WAVE_LDS_SYNC();
}

__global__ void __launch_bounds__(WAVES_PER_BLOCK * 64)
k_eval_fast64(const double *__restrict__ W_dp, const uint16_t *__restrict__ rank_tab,
              const double *__restrict__ rank_val, const uint32_t *__restrict__ step_tab,
              const int32_t *__restrict__ perm, size_t P, double *__restrict__ cost,
              double *__restrict__ ghat_out, double *__restrict__ datap_out)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint16_t *R = reinterpret_cast<uint16_t *>(smem);
    unsigned char *wl = smem + LDS_RANK_BYTES + wave * WAVE_LDS_BYTES;

    // rank table -> LDS (8 KiB, 16 bytes per thread per pass)
    for (int i = threadIdx.x; i < LDS_RANK_BYTES / 16; i += blockDim.x)
        reinterpret_cast<uint4 *>(smem)[i] = reinterpret_cast<const uint4 *>(rank_tab)[i];
    // per-lane step constants -> registers
    step_consts sc;
#pragma unroll
    for (int i = 0; i < N_MSTEP; i++) {
        sc.m_nib[i] = step_tab[(0 * N_MSTEP + i) * 64 + lane];
        sc.m_meta[i] = step_tab[(1 * N_MSTEP + i) * 64 + lane];
    }
#pragma unroll
    for (int i = 0; i < N_HSTEP; i++) {
        sc.h_nib[i] = step_tab[(2 * N_MSTEP + 0 * N_HSTEP + i) * 64 + lane];
        sc.h_a[i] = step_tab[(2 * N_MSTEP + 1 * N_HSTEP + i) * 64 + lane];
        sc.h_b[i] = step_tab[(2 * N_MSTEP + 2 * N_HSTEP + i) * 64 + lane];
    }
    __syncthreads();

    const size_t nwaves = (size_t)gridDim.x * WAVES_PER_BLOCK;
    for (size_t cand = (size_t)blockIdx.x * WAVES_PER_BLOCK + wave; cand < P; cand += nwaves) {
        // The step constants are loop invariant; hide that from the optimiser, which would otherwise
        // hoist every address derived from them out of the loop and spill hundreds of registers.
#pragma unroll
        for (int i = 0; i < N_MSTEP; i++) {
            asm volatile("" : "+v"(sc.m_nib[i]));
            asm volatile("" : "+v"(sc.m_meta[i]));
        }
#pragma unroll
        for (int i = 0; i < N_HSTEP; i++) {
            asm volatile("" : "+v"(sc.h_nib[i]));
            asm volatile("" : "+v"(sc.h_a[i]));
            asm volatile("" : "+v"(sc.h_b[i]));
        }
        // ---- a1: candidate row, position = lane: stage = lane / 8, slot = lane % 8 ----
        const int d = perm[cand * NDEV + lane];
        wl[OFF_PB + lane] = (unsigned char)d;
        wl[OFF_PBT + (lane & 7) * 8 + (lane >> 3)] = (unsigned char)d;
        WAVE_LDS_SYNC();

        // ---- a2: DataP row sum of this lane's device over its stage, slot order ----
        const uint2 mates = *reinterpret_cast<const uint2 *>(wl + OFF_PB + (lane & ~7));
        const double *wrow = W_dp + d * NDEV;
        double wv[8];
#pragma unroll
        for (int k = 0; k < 8; k++) {
            const uint32_t m = ((k < 4 ? mates.x : mates.y) >> (8 * (k & 3))) & 0xFFu;
            wv[k] = wrow[m];   // own slot: the zero diagonal
        }

        // ---- a4 (1): gather the 28 blocks as ranks; lane = (row slot r, column slot c) ----
        {
            const uint2 rowdev = *reinterpret_cast<const uint2 *>(wl + OFF_PBT + (lane >> 3) * 8);  // slot r of stages 0..7
            const uint2 coldev = *reinterpret_cast<const uint2 *>(wl + OFF_PBT + (lane & 7) * 8);   // slot c of stages 0..7
            uint32_t rb[8], cb[8];
#pragma unroll
            for (int j = 0; j < 8; j++) {
                rb[j] = (((j < 4 ? rowdev.x : rowdev.y) >> (8 * (j & 3))) & 0xFFu) * NDEV;
                cb[j] = ((j < 4 ? coldev.x : coldev.y) >> (8 * (j & 3))) & 0xFFu;
            }
            uint32_t rk[NGROUP * 8];
            int t = 0;
#pragma unroll
            for (int j1 = 0; j1 < 8; j1++)
#pragma unroll
                for (int j2 = j1 + 1; j2 < 8; j2++) {
                    rk[(t / PAIRS_PER_GROUP) * 8 + (t % PAIRS_PER_GROUP)] = R[rb[j1] + cb[j2]];
                    t++;
                }
#pragma unroll
            for (int g = 0; g < NGROUP; g++) {
                rk[g * 8 + 7] = 0;
                uint4 v;
                v.x = rk[g * 8 + 0] | (rk[g * 8 + 1] << 16);
                v.y = rk[g * 8 + 2] | (rk[g * 8 + 3] << 16);
                v.z = rk[g * 8 + 4] | (rk[g * 8 + 5] << 16);
                v.w = rk[g * 8 + 6] | (rk[g * 8 + 7] << 16);
                *reinterpret_cast<uint4 *>(wl + OFF_WST + (g * 64 + lane) * 16) = v;
            }
        }
        WAVE_LDS_SYNC();

        // ---- a4 (2): min-max programme over column subsets, all 28 pairs at once ----
        if (lane < NGROUP * 8) {   // layer 1: g[{c}] = w[0][c]
            const int g = lane >> 3, c = lane & 7;
            *reinterpret_cast<uint4 *>(wl + OFF_GT + (g * 256 + (1 << c)) * 16) =
                *reinterpret_cast<const uint4 *>(wl + OFF_WST + (g * 64 + c) * 16);
        }
        WAVE_LDS_SYNC();
#ifndef EXP_SKIP_MATCH
        match_layer<2>(wl, sc);
        match_layer<3>(wl, sc);
        match_layer<4>(wl, sc);
        match_layer<5>(wl, sc);
        match_layer<6>(wl, sc);
        match_layer<7>(wl, sc);
        match_layer<8>(wl, sc);
#endif

        // ---- a4 (3): winning rank -> fp64 weight; lane = (u, v) entry of the coarsened graph ----
        double e = 0.0;
        {
            const int u = lane >> 3, v = lane & 7;
            const int a = u < v ? u : v, b = u < v ? v : u;
            const int t = a * 8 - a * (a + 1) / 2 + (b - a - 1);   // lexicographic pair number
            if (u != v) {
                const uint16_t r = *reinterpret_cast<const uint16_t *>(
                    wl + OFF_GT + ((t / PAIRS_PER_GROUP) * 256 + 255) * 16 + (t % PAIRS_PER_GROUP) * 2);
                e = rank_val[r];
            }
        }
        WAVE_LDS_SYNC();   // the Held-Karp table reuses the matching tables' space
        *reinterpret_cast<double *>(wl + OFF_GHAT + lane * 8) = e;
        if (ghat_out != nullptr) ghat_out[cand * 64 + lane] = e;

        // ---- a5: Held-Karp over the 8 stage nodes ----
        if (lane < 8) *reinterpret_cast<double *>(wl + OFF_HK + (lane * 256 + (1 << lane)) * 8) = 0.0;
        WAVE_LDS_SYNC();
#ifndef EXP_SKIP_HK
        hk_layer<2>(wl, sc);
        hk_layer<3>(wl, sc);
        hk_layer<4>(wl, sc);
        hk_layer<5>(wl, sc);
        hk_layer<6>(wl, sc);
        hk_layer<7>(wl, sc);
        hk_layer<8>(wl, sc);
#endif
        double pp = *reinterpret_cast<const double *>(wl + OFF_HK + ((lane & 7) * 256 + 255) * 8);
        pp = fmin(pp, __shfl_xor(pp, 1));
        pp = fmin(pp, __shfl_xor(pp, 2));
        pp = fmin(pp, __shfl_xor(pp, 4));

        // ---- a2/a3: finish DataP; a6: total ----
        double sum = 0.0;
#pragma unroll
        for (int k = 0; k < 8; k++) sum = __dadd_rn(sum, wv[k]);
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) sum = fmax(sum, __shfl_xor(sum, o));
        if (lane == 0) {
            if (cost != nullptr) cost[cand] = __dadd_rn(sum, pp);
            if (datap_out != nullptr) datap_out[cand] = sum;
        }
        WAVE_LDS_SYNC();   // next candidate overwrites the tables
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

// ---- which subset each lane handles, and in which order it visits the subset's columns ----------
// A 128-bit LDS read is served 16 lanes at a time; within such a pass two lanes that read different
// addresses with equal (address / 16) % 16 take an extra cycle each. Which subset S a lane owns and
// the order in which it removes S's columns are free, so they are chosen once (deterministic local
// search) to keep the predecessor reads gt[S \ c] of the 16 lanes of a pass on distinct slots.
struct match_item {
    uint8_t S, ord[8];
    bool valid;
};

int pass_cost(const match_item *it, int k)
{
    int total = 0;
    for (int t = 0; t <= k; t++) {   // t == k: the write of gt[S]
        int cnt[16] = {0};
        bool seen[256] = {false};
        int worst = 0;
        for (int i = 0; i < 16; i++) {
            if (!it[i].valid) continue;
            int a = t < k ? (it[i].S ^ (1 << it[i].ord[t])) : it[i].S;
            if (seen[a]) continue;   // same address: broadcast
            seen[a] = true;
            if (++cnt[a & 15] > worst) worst = cnt[a & 15];
        }
        total += worst;
    }
    return total;
}

std::vector<match_item> arrange_layer(int k)
{
    std::vector<match_item> arr;
    for (uint32_t S = 1; S < 256; S++)
        if (__builtin_popcount(S) == k) {
            match_item m = {};
            m.S = (uint8_t)S;
            m.valid = true;
            int t = 0;
            for (int c = 0; c < 8; c++)
                if (S & (1u << c)) m.ord[t++] = (uint8_t)c;
            arr.push_back(m);
        }
    while (arr.size() % 16) arr.push_back(match_item{});
    const int np = (int)arr.size() / 16;
    std::vector<int> cost(np);
    for (int p = 0; p < np; p++) cost[p] = pass_cost(&arr[p * 16], k);
    uint64_t rng = 0x9E3779B97F4A7C15ull + (uint64_t)k;
    auto next = [&rng](uint32_t n) {
        rng = rng * 6364136223846793005ull + 1442695040888963407ull;
        return (uint32_t)((rng >> 33) % n);
    };
    const int iters = 30000;
    for (int it = 0; it < iters; it++) {
        // accept equal-cost moves always, worse moves (by 1) early on with small probability
        const bool allow_worse = it < iters / 2 && next(16) == 0;
        int p = (int)next(np), i = (int)next(16);
        if (next(2) == 0 || np == 1) {
            match_item &m = arr[p * 16 + i];
            if (!m.valid || k < 2) continue;
            int a = (int)next(k), b = (int)next(k);
            if (a == b) continue;
            std::swap(m.ord[a], m.ord[b]);
            int c = pass_cost(&arr[p * 16], k);
            if (c <= cost[p] || (allow_worse && c == cost[p] + 1)) cost[p] = c;
            else std::swap(m.ord[a], m.ord[b]);
        } else {
            int q = (int)next(np), j = (int)next(16);
            if (q == p) continue;
            std::swap(arr[p * 16 + i], arr[q * 16 + j]);
            int cp = pass_cost(&arr[p * 16], k), cq = pass_cost(&arr[q * 16], k);
            int d = cp + cq - cost[p] - cost[q];
            if (d <= 0 || (allow_worse && d == 1)) {
                cost[p] = cp;
                cost[q] = cq;
            } else
                std::swap(arr[p * 16 + i], arr[q * 16 + j]);
        }
    }
    return arr;
}

}  // namespace

bool dtfm_fast64_applicable(const dtfm_problem *pr) { return pr->N == 64 && pr->D_dp == 8 && pr->D_pp == 8; }

// Builds the rank tables and the per-lane step tables of a 64-device problem.
int dtfm_fast64_prepare(dtfm_problem *pr)
{
    const int N = pr->N;
    DTFM_HIP(hipMalloc((void **)&pr->f64_rank, (size_t)N * N * sizeof(uint16_t)));
    DTFM_HIP(hipMalloc((void **)&pr->f64_rank_val, (size_t)N * N * sizeof(double)));
    DTFM_HIP(hipMemset(pr->f64_rank_val, 0, (size_t)N * N * sizeof(double)));
    hipLaunchKernelGGL(k_rank_weights, dim3((N * N + 255) / 256), dim3(256), 0, (hipStream_t) nullptr, pr->W_pp, N,
                       pr->f64_rank, pr->f64_rank_val);
    DTFM_HIP(hipGetLastError());

    std::vector<uint32_t> tab((size_t)(2 * N_MSTEP + 3 * N_HSTEP) * 64, 0u);
    uint32_t *m_nib = tab.data(), *m_meta = m_nib + N_MSTEP * 64;
    uint32_t *h_nib = m_meta + N_MSTEP * 64, *h_a = h_nib + N_HSTEP * 64, *h_b = h_a + N_HSTEP * 64;
    int ms = 0, hs = 0;
    static std::vector<match_item> arrangement[9];   // problem independent: built once per process
    static std::once_flag arranged;
    std::call_once(arranged, [] {
        for (int k = 2; k <= 8; k++) arrangement[k] = arrange_layer(k);
    });
    for (int k = 2; k <= 8; k++) {
        std::vector<uint32_t> layer;
        for (uint32_t S = 1; S < 256; S++)
            if (__builtin_popcount(S) == k) layer.push_back(S);
        // matching: passes of 16 lanes, each within one group; the same arrangement for every group
        const std::vector<match_item> &arr = arrangement[k];
        const int ppg = (int)arr.size() / 16;   // passes per group
        for (int s = 0; s < match_steps(k); s++, ms++)
            for (int lane = 0; lane < 64; lane++) {
                int pass = s * 4 + lane / 16;
                if (pass >= NGROUP * ppg) continue;
                uint32_t g = pass / ppg;
                const match_item &it = arr[(pass % ppg) * 16 + lane % 16];
                if (!it.valid) continue;
                uint32_t nib = 0;
                for (int t = 0; t < k; t++) nib |= (uint32_t)it.ord[t] << (4 * t);
                m_nib[ms * 64 + lane] = nib;
                m_meta[ms * 64 + lane] = ((g * 256 + it.S) * 16) | (g << 16) | 0x80000000u;
            }
        // Held-Karp: item i = (subset, end node v in it), subsets ascending, v ascending
        std::vector<std::pair<uint32_t, int>> items;
        for (uint32_t S : layer)
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
    size_t blocks = (rows + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK;
    if (blocks > (size_t)pr->f64_grid) blocks = pr->f64_grid;
    hipLaunchKernelGGL(k_eval_fast64, dim3((unsigned)blocks), dim3(WAVES_PER_BLOCK * 64), LDS_TOTAL, st, pr->W_dp,
                       pr->f64_rank, pr->f64_rank_val, pr->f64_steps, perm, rows, cost, ghat, datap);
    DTFM_HIP(hipGetLastError());
    return DTFM_OK;
}
