// Internal declarations shared by the translation units of libdtfm (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "dtfm.h"

#define DTFM_WAVE 64

// Largest D_pp whose Held-Karp table (2^D_pp x D_pp fp64) is kept in LDS by the general kernel:
// 2^10 * 10 * 8 B = 80 KiB of the CU's 160 KiB.
#define DTFM_HK_LDS_MAX_DPP 10
// Above that limit the table is processed in LDS blocks over the DTFM_HK_BLOCK_LOW lowest stages
// (2^10 rows x 18 fp64 = 144 KiB: one workgroup per CU); DTFM_HK_GLOBAL_GRID workgroups, each with
// its own exchange area in HBM for the entries that pass from block to block.
#define DTFM_HK_BLOCK_LOW 10
#define DTFM_HK_ROW_STRIDE 18   // doubles between rows of a block (16 slots + padding against bank conflicts)
#define DTFM_HK_GLOBAL_GRID 256

// Workgroup barrier that orders LDS accesses only: global memory operations in flight are not
// waited for.
#define DTFM_LDS_BARRIER()                                                  \
    do {                                                                    \
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");     \
        __builtin_amdgcn_s_barrier();                                       \
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");     \
    } while (0)

struct dtfm_layer_off {
    int off[DTFM_MAX_DPP + 2];  // off[k] = first index of the subsets of popcount k; off[n+1] = end
};

struct dtfm_problem {
    int N, D_dp, D_pp, npairs;
    int device;
    double c_dp, c_pp;
    double *W_dp;           // device, N*N
    double *W_pp;           // device, N*N
    uint32_t *hk_subsets;   // device, 2^D_pp - 1 subsets ordered by (popcount, value)
    uint32_t *W_rank;       // device, N*N: dense rank of W_pp[d][d'] among all entries (general shapes)
    uint16_t *W_code;       // device, N*N: 2 + (rank >> rank_shift), the codes of the matching kernel's first solve
    int rank_shift;         // smallest shift with which the codes stay below 0xffff
    double *rank_val;       // device: rank -> weight
    dtfm_layer_off hk_off;
    char *scratch;          // device arena, grown on demand
    size_t scratch_bytes;
    char *fixed_scratch;    // this device's copy of the library's fixed scratch area (allocation-free entry point)
    // fused kernel for the 64-device shape (N = 64, D_dp = 8, D_pp = 8)
    bool fast64;
    uint16_t *f64_rank;     // device, N*N: rank of W_pp[d][d'] among all off-diagonal weights
    double *f64_rank_val;   // device, N*N: rank -> weight
    int f64_grid;           // workgroups launched (one per CU)
};

// Bump allocator over the problem's scratch arena. With base == nullptr it only measures.
struct dtfm_arena {
    char *base;
    size_t off;
    template <typename T>
    T *take(size_t count)
    {
        size_t bytes = (count * sizeof(T) + 255) & ~(size_t)255;
        T *p = reinterpret_cast<T *>(base + off);
        off += bytes;
        return p;
    }
};

int dtfm_hip_fail(hipError_t e, const char *what);
#define DTFM_HIP(call)                                        \
    do {                                                      \
        hipError_t e__ = (call);                              \
        if (e__ != hipSuccess) return dtfm_hip_fail(e__, #call); \
    } while (0)

// ---- general-shape evaluation (dtfm_eval.hip) -------------------------------------------------
struct dtfm_eval_bufs {
    int32_t *pos;    // rows * N: position of every device in its row, or null (DataP by candidate)
    double *rowsum;  // rows * N: Eq. 2 row sum of the device at every position, or null
    double *datap;   // rows
    double *ghat;    // rows * D_pp * D_pp
    double *hk_tab;  // hk_grid exchange areas, or null when the table fits LDS
    size_t hk_grid;  // workgroups of the blocked Held-Karp kernel (each owns one exchange area)
    double *pp;      // rows: PipelineP-Cost (the Held-Karp value) of every row whose Held-Karp was run
    int32_t *list;   // rows: the rows whose Held-Karp is still to run (trial evaluations, see dtfm_trial_ref)
    int32_t *count;  // 1: length of list
};
// What a trial evaluation of the local search knows about the rows its trials were made from: with it, a trial
// whose coarsened graph equals its current row's, or is nowhere below it while DataP + the current PipelineP
// already reaches the current cost, is settled without Held-Karp (Eq. 4 depends on the graph only, and is
// monotone in every edge).
struct dtfm_trial_ref {
    const double *ghat_cur;   // rows * D_pp * D_pp: coarsened graphs of the current rows
    const double *pp_cur;     // rows: their PipelineP-Cost
    const double *cur;        // rows: their cost (Eq. 1)
    int trials_per_row;       // consecutive trial rows made from one current row (1, or 4 for BEST4)
};
// hk_grid_cap: upper limit on the number of exchange areas (0: DTFM_HK_GLOBAL_GRID); lean: without the per-position
// buffers of DataP by device (the evaluation then takes DataP by candidate)
dtfm_eval_bufs dtfm_eval_carve(const dtfm_problem *pr, dtfm_arena &ar, size_t rows, size_t hk_grid_cap = 0, bool lean = false);
// bytes of one exchange area of the blocked Held-Karp kernel (0 when the table fits LDS)
size_t dtfm_hk_exchange_bytes(const dtfm_problem *pr);
// enqueues a2..a6 for `rows` candidates; cost may be null (then only datap/ghat are produced)
int dtfm_eval_enqueue(const dtfm_problem *pr, const dtfm_eval_bufs &b, const int32_t *perm,
                      size_t rows, double *cost, hipStream_t st);
// the same when b.ghat already holds the coarsened graphs of rows that differ from `perm` only in stages
// inc_j < inc_jp (inc_j < 0: plain evaluation): only the edges of those two stages are matched again
int dtfm_eval_inc_enqueue(const dtfm_problem *pr, const dtfm_eval_bufs &b, const int32_t *perm, size_t rows,
                          double *cost, int inc_j, int inc_jp, hipStream_t st, const dtfm_trial_ref *ref = nullptr);
int dtfm_weights_enqueue(const double *lat_dev, const double *bw_dev, int N, double shard,
                         double c_pp, double *W_dp, double *W_pp, hipStream_t st);

// ---- assignment extraction (dtfm_assign.hip) ---------------------------------------------------
struct dtfm_assign_bufs {
    dtfm_eval_bufs ev;
    double *tab;      // Held-Karp tables kept for back-tracking, one per concurrently live workgroup
    int32_t *mates;   // rows * (D_pp - 1) * D_dp: matching of each adjacent pair of the order
};
dtfm_assign_bufs dtfm_assign_carve(const dtfm_problem *pr, dtfm_arena &ar, size_t rows);
int dtfm_assign_enqueue(const dtfm_problem *pr, const dtfm_assign_bufs &b, const int32_t *perm, size_t rows,
                        int32_t *stage_order, int32_t *sigma, hipStream_t st);

// ---- fused evaluation, 64-device shape (dtfm_fast64.hip) ---------------------------------------
bool dtfm_fast64_applicable(const dtfm_problem *pr);
int dtfm_fast64_prepare(dtfm_problem *pr);
void dtfm_fast64_release(dtfm_problem *pr);
// any of cost / ghat (rows*64) / datap (rows) may be null
int dtfm_fast64_enqueue(const dtfm_problem *pr, const int32_t *perm, size_t rows, double *cost, double *ghat,
                        double *datap, hipStream_t st);

// all `moves` rounds of the GAIN4 local search in one launch; perm in/out, cost out, applied may be null
int dtfm_fast64_ls_gain4_enqueue(const dtfm_problem *pr, int32_t *perm, size_t rows, int moves, double *cost,
                                 int64_t *applied, hipStream_t st);

// What the evolutionary search needs to make offspring k of generation g (Sec. 3.4: selection, crossover,
// mutation): the Philox key, the generation-start population (rows of N) and the operator counts.
struct dtfm_offspring_src {
    uint32_t k0, k1, g;
    const int32_t *pop;
    int P, m_x, m_m;
};
// True when the GAIN4 launch for `rows` offspring can make them itself (small populations, where a launch of
// its own for that step costs as much as a tenth of the generation).
bool dtfm_fast64_ls_makes_offspring(const dtfm_problem *pr, size_t rows, int moves);
// As dtfm_fast64_ls_gain4_enqueue, the rows made in the kernel from `src` instead of read: perm is only written.
int dtfm_fast64_offspring_ls_gain4_enqueue(const dtfm_problem *pr, const dtfm_offspring_src &src, int32_t *perm,
                                           size_t rows, int moves, double *cost, hipStream_t st);

// all `moves` >= 1 rounds of the ALL_PAIRS local search with incremental move evaluation in one launch
// (dtfm_fast64_allpairs.hip); perm in/out, cost out, applied may be null
int dtfm_fast64_allpairs_prepare();
int dtfm_fast64_ls_allpairs_enqueue(const dtfm_problem *pr, int32_t *perm, size_t rows, int moves, double *cost,
                                    int64_t *applied, hipStream_t st);

// cost of every swap of every row (rows * 2016 doubles); perm is only read
int dtfm_fast64_move_costs_enqueue(const dtfm_problem *pr, const int32_t *perm, size_t rows, double *move_cost,
                                   hipStream_t st);

// ---- search (dtfm_search.hip) -----------------------------------------------------------------
struct dtfm_ls_bufs {
    double *cur;        // P: current cost of each candidate
    int32_t *tmp_perm;  // rows * N: candidates with a move applied
    double *tmp_cost;   // rows
    int32_t *move_ab;   // 2 * P (GAIN4: proposed positions)
    size_t chunk;       // candidates per ALL_PAIRS chunk (every swap materialised)
    size_t group_chunk; // candidates per ALL_PAIRS chunk when the swaps go by stage pair, else 0
    double *all_cost;   // group_chunk * N (N - 1) / 2: the costs of a chunk's swaps by move index, or null
    size_t rows;        // rows evaluated per eval call
    double *ghat_cur;   // P * D_pp * D_pp: coarsened graphs of the current rows (GAIN4 / KL rounds)
    double *pp_cur;     // P: PipelineP-Cost of the current rows (GAIN4 / KL rounds)
    dtfm_eval_bufs ev;
};
// pricing: for dtfm_move_costs (every swap's exact cost, materialised)
dtfm_ls_bufs dtfm_ls_carve(const dtfm_problem *pr, dtfm_arena &ar, size_t P, int neighbourhood, bool pricing = false);
int dtfm_ls_enqueue(const dtfm_problem *pr, const dtfm_ls_bufs &b, int32_t *perm, size_t P, int moves,
                    int neighbourhood, double *cost, int64_t *applied, hipStream_t st);

// cost of every swap a < b of every row, out[p * N(N-1)/2 + move index]
int dtfm_move_costs_enqueue(const dtfm_problem *pr, const dtfm_ls_bufs &b, const int32_t *perm, size_t P, double *out,
                            hipStream_t st);

struct dtfm_ga_bufs {
    int32_t *off;       // lambda * N
    double *off_cost;   // lambda
    int32_t *next;      // P * N
    double *next_cost;  // P
    int32_t *rank;      // P + lambda: rank of each key under (cost, origin)
    dtfm_ls_bufs ls;
};
dtfm_ga_bufs dtfm_ga_carve(const dtfm_problem *pr, dtfm_arena &ar, const dtfm_ga_params &prm);
int dtfm_ga_enqueue(const dtfm_problem *pr, const dtfm_ga_bufs &b, uint64_t seed, int generations,
                    const dtfm_ga_params &prm, int32_t *population, double *cost, double *best_trace,
                    hipStream_t st);
int dtfm_philox_enqueue(uint64_t seed, uint32_t stream, uint32_t g, uint32_t k, uint32_t first_block,
                        int n_blocks, uint32_t *out, hipStream_t st);
int dtfm_validate_enqueue(const dtfm_problem *pr, const int32_t *perm, size_t P, int32_t *bad_rows,
                          hipStream_t st);
