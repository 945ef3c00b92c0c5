/*
 * dtfm: GPU (gfx950 / MI355X) evaluation of the scheduler cost model and search of
 * "Decentralized Training of Foundation Models in Heterogeneous Environments" (arXiv 2206.01288).
 *
 * C ABI. Every "device" pointer is HIP device memory on the current device, owned by the caller;
 * every "host" pointer is ordinary host memory. The three hot calls (eval_population,
 * local_search, evolve) only enqueue kernels on the caller's stream and return without
 * synchronising; results are valid once the stream has been synchronised. All functions return
 * a status code (DTFM_OK = 0); none aborts or throws. A problem handle owns device copies of the
 * weight matrices and a scratch area that grows on demand: when a hot call is given a larger
 * population than the handle has seen (or reserved with dtfm_reserve), that call first waits for
 * the whole device (hipDeviceSynchronize), frees the old area and allocates a larger one
 * (hipFree, hipMalloc), and only then enqueues. Call dtfm_reserve once, outside the hot loop, to
 * keep the hot calls free of that. Calls on one handle share its scratch area and must not
 * overlap in time (they race otherwise), whatever streams they are given.
 *
 * Candidate layout ("perm"): row-major P x N int32. Row p is a permutation of 0..N-1; position q
 * holds the device sigma_{i,j} (Sec. 2, assignment strategy) that runs pipeline stage
 * j = q / D_dp for micro-batch slot i = q % D_dp. The data-parallel group of stage j (Sec. 3.1)
 * is C_j = { perm[j*D_dp + i] : 0 <= i < D_dp }. The slot index has no influence on the cost
 * beyond the order in which the Eq. 2 sum is rounded.
 */
#ifndef DTFM_H
#define DTFM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dtfm_problem dtfm_problem;

enum {
    DTFM_OK = 0,
    DTFM_ERR_NULL = 1,          /* a required pointer is null */
    DTFM_ERR_SHAPE = 2,         /* N, D_dp, D_pp < 1, D_dp*D_pp != N, or above the supported limits */
    DTFM_ERR_VALUE = 3,         /* negative / non-finite latency or size, non-positive bandwidth */
    DTFM_ERR_ARG = 4,           /* bad P, rounds, neighbourhood, generations or GA parameter */
    DTFM_ERR_HIP = 5,           /* a HIP runtime call failed (no device, out of memory, ...) */
    DTFM_ERR_UNSUPPORTED = 6,   /* e.g. GAIN4 with D_dp < 2 or D_pp < 2 */
    DTFM_ERR_TOO_LARGE = 7      /* dtfm_eval_population_noalloc: P does not fit the fixed scratch area */
};

/* Supported limits: D_pp <= 16 (Held-Karp table 2^D_pp x D_pp), D_dp <= 64 (one wavefront lane
 * per device of a stage in the matching kernel), N <= 1024. */
#define DTFM_MAX_DPP 16
#define DTFM_MAX_DDP 64
#define DTFM_MAX_N 1024

enum { DTFM_ALL_PAIRS = 0, DTFM_GAIN4 = 1, DTFM_KL = 2, DTFM_BEST4 = 3 };

/* Sec. 2 (formalisation of the scheduling problem) and Eqs. 2-3: builds the problem instance.
 * latency, bandwidth: host, N*N row-major, entry [d*N + d'] = alpha_{d,d'} (seconds) and
 * beta_{d,d'} (bytes/second); the diagonal is ignored; asymmetric inputs are symmetrised by
 * averaging the two directions as in the definition of the communication graph G. c_dp, c_pp:
 * bytes per stage (gradients) and per micro-batch hop (activations). The two weight matrices
 *   W_dp[d][d'] = 2 (alpha + (c_dp / D_dp) / beta),   W_pp[d][d'] = 2 (alpha + c_pp / beta)
 * are computed on the device in fp64 and stay resident. The unit of the result is the unit of
 * alpha (seconds when bandwidth is bytes/second).
 * Errors: DTFM_ERR_NULL, DTFM_ERR_SHAPE, DTFM_ERR_VALUE, DTFM_ERR_HIP. On error *out is null. */
int dtfm_create_problem(const double *latency, const double *bandwidth, int N, double c_dp,
                        double c_pp, int D_dp, int D_pp, dtfm_problem **out);

/* Frees the handle and everything it owns (synchronises the device first). Null is allowed. */
void dtfm_destroy_problem(dtfm_problem *prob);

/* Copies the device-resident weight matrices to host buffers of N*N doubles each (either may be
 * null). Synchronous. For checking the weight kernel. */
int dtfm_get_weights(const dtfm_problem *prob, double *W_dp_host, double *W_pp_host);

/* Eq. 1: Comm-Cost of each of P candidates = DataP-Cost (Eq. 2 and the max over stages that
 * follows it) + PipelineP-Cost (Eq. 4: open-loop TSP, solved exactly by Held-Karp, over the
 * coarsened graph whose edges are the bottleneck perfect matchings of Eq. 3).
 * perm: device, P*N int32 (layout above), read only. cost: device, P doubles, written.
 * Rows are not checked for being permutations (see dtfm_validate_population); entries outside
 * 0..N-1 are undefined behaviour. P = 0 is a no-op. Errors: NULL, ARG (P < 0), HIP. */
int dtfm_eval_population(dtfm_problem *prob, const int32_t *perm, int P, double *cost,
                         void *hip_stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): dtfm_eval_population with the same arguments, results
 * and kernels, whose intermediate buffers (DataP per candidate, the coarsened graphs, and for
 * D_pp > 10 the Held-Karp exchange areas) lie in a fixed area of DTFM_FIXED_SCRATCH_BYTES that is
 * part of the library's device image (every GPU the library is used on holds one copy until the
 * process ends). The call allocates and frees nothing and does not synchronise. It needs
 * 8 (1 + D_pp^2) + 12 bytes per candidate (in pieces rounded up to 256 bytes), and for D_pp > 10 at least
 * one exchange area of 8 (D_pp - 10) 2^D_pp bytes behind that (3 MiB at D_pp = 16; as many areas
 * as fit are used, one per workgroup, so the Held-Karp step runs on fewer workgroups than in
 * dtfm_eval_population); a larger P returns DTFM_ERR_TOO_LARGE and enqueues nothing. The 64-device
 * shape (N = 64, D_dp = 8, D_pp = 8) needs no scratch and takes any P. All calls on one GPU share
 * the one area, which keeps the previous call's contents: calls that overlap in time on one GPU
 * race, also across problem handles and streams. The current device must be the one the
 * handle was created on (DTFM_ERR_ARG otherwise). Other errors as dtfm_eval_population. */
#define DTFM_FIXED_SCRATCH_BYTES (32u << 20)
int dtfm_eval_population_noalloc(dtfm_problem *prob, const int32_t *perm, int P, double *cost,
                                 void *hip_stream);

/* Grows the handle's scratch area, now, to what eval_population, coarsened_graph, get_assignment
 * and local_search with `neighbourhood` (move_costs counts as DTFM_ALL_PAIRS) on up to
 * max(P, lambda) rows and evolve with population P and lambda offspring need, so that those calls neither allocate nor synchronise
 * later. Synchronises the device when it has to grow the area. P or lambda may be 0.
 * Errors: NULL, ARG (negative sizes, unknown neighbourhood), HIP (out of memory). */
int dtfm_reserve(dtfm_problem *prob, int P, int lambda, int neighbourhood);

/* The intermediate quantities of the same evaluation, for checking: ghat (device, P*D_pp*D_pp
 * doubles, symmetric, zero diagonal) receives the coarsened graph of Sec. 3.3 (Eq. 3 per stage
 * pair), datap (device, P doubles) the DataP-Cost of Sec. 3.2. Either may be null. */
int dtfm_coarsened_graph(dtfm_problem *prob, const int32_t *perm, int P, double *ghat,
                         double *datap, void *hip_stream);

/* The assignment behind the cost of each candidate (Sec. 2, "Pipeline parallel": the pipelines
 * P_i = { sigma_{i,j} }; Sec. 3.3: devices matched between adjacent stage groups handle the same
 * micro-batch and the groups are ordered by the open-loop tour of Eq. 4). Neither optimum is unique
 * and the paper names no choice; the canonical ones taken here:
 *  - order: Held-Karp back-tracking. The tour ends in the lowest-numbered group attaining the
 *    minimum; the group before v in a tour over the set S is the lowest-numbered u in S \ v whose
 *    rounded value tab[S \ v][u] + Ghat[u][v] equals tab[S][v];
 *  - matching of adjacent groups (A, B) with Eq. 3 optimum T: the lexicographically smallest vector
 *    (slot of B matched to slot 0 of A, to slot 1 of A, ...) among the perfect matchings that use
 *    only device pairs with W_pp <= T;
 *  - pipeline i starts at slot i of the first group of the order and follows the matchings.
 * perm: device, P*N int32, read only. stage_order: device, P*D_pp int32, out: stage index at each
 * pipeline position, first to last. sigma: device, P*D_dp*D_pp int32, out: [p][i][k] = device of
 * pipeline i at position k (a member of stage stage_order[p][k]). Summing over k the largest
 * W_pp[sigma[i][k]][sigma[i][k+1]] over i, left to right, and adding DataP gives the bits of
 * dtfm_eval_population. Enqueues only. Errors: NULL, ARG (P < 0), HIP. */
int dtfm_get_assignment(dtfm_problem *prob, const int32_t *perm, int P, int32_t *stage_order,
                        int32_t *sigma, void *hip_stream);

/* Validity of Sec. 2 ("a valid assignment needs to be unique"): counts the rows of perm that are
 * not permutations of 0..N-1 into *bad_rows (device, one int32, overwritten). */
int dtfm_validate_population(dtfm_problem *prob, const int32_t *perm, int P, int32_t *bad_rows,
                             void *hip_stream);

/* Sec. 3.4 local search: `moves` rounds; in each round every candidate evaluates its
 * neighbourhood on the true cost (Eq. 1) and applies at most one swap of two positions, only if
 * the cost strictly decreases.
 *  DTFM_ALL_PAIRS: all N(N-1)/2 position pairs a < b in lexicographic order; the cheapest
 *    resulting allocation wins, the lowest move index on ties. A swap of two slots of the same
 *    stage leaves the partition C_1..C_Dpp (and so Eq. 1 as a function of the sets) unchanged and
 *    only reorders that stage's Eq. 2 sums; it is priced like any other move, so once no real move
 *    improves, such a swap can still be applied on a gain of one unit in the last place of the
 *    rounded sum (the oracle does the same; `applied` then names it and the cost drops by that).
 *  DTFM_GAIN4: the paper's neighbourhood ("Improving Local Search Strategy"): round r takes
 *    stage pair number r mod D_pp(D_pp-1)/2 in lexicographic order, the fastest link (smallest
 *    W_pp) inside each of the two stages, and among the four swaps of their end points the one
 *    of largest Gain (the paper's gain function with w = W_pp); that swap is the round's move.
 *  DTFM_BEST4: a second reading of the same passage (the paper does not say whether a swap is
 *    taken on its Gain or on the cost): the same stage pair per round and the same four candidate
 *    swaps as DTFM_GAIN4 (in the order (d1,d1'), (d1,d2'), (d2,d1'), (d2,d2')), all four priced by
 *    Eq. 1; the cheapest of them, the first on ties, is the round's move.
 *  DTFM_KL: the strategy the paper compares with ("Existing Local Search Strategy"), for
 *    ablations: same stage pair per round as DTFM_GAIN4; among all D_dp^2 swaps of a device of
 *    one stage with a device of the other, the one of largest Kernighan-Lin gain (the paper's
 *    gain_KL with w = W_pp; first in (slot, slot') order on ties) is the round's move.
 * perm: device, P*N, in/out. cost: device, P doubles, out: cost of the final rows.
 * applied: device, P*moves int64, may be null: the index (in the ALL_PAIRS numbering) of the
 * swap applied by candidate p in round r at [p*moves + r], or -1.
 * Errors: NULL, ARG (P < 0, moves < 0, unknown neighbourhood), UNSUPPORTED (GAIN4 or BEST4 with
 * D_dp < 2 or D_pp < 2, KL with D_pp < 2), HIP. */
int dtfm_local_search(dtfm_problem *prob, int32_t *perm, int P, int moves, int neighbourhood,
                      double *cost, int64_t *applied, void *hip_stream);

/* Move evaluation of the local search (Sec. 3.4, "find o* that leads to better cost"): the cost
 * (Eq. 1) of every allocation one swap away from each row. move_cost: device, P*N(N-1)/2 doubles,
 * out: at [p*N(N-1)/2 + m] the cost of row p with positions a < b exchanged, m the index of (a, b)
 * in lexicographic order, m = a*N - a(a+1)/2 + (b-a-1); the same bits as dtfm_eval_population on
 * the swapped row. perm: device, P*N, read only. Enqueues only. Errors: NULL, ARG (P < 0), HIP. */
int dtfm_move_costs(dtfm_problem *prob, const int32_t *perm, int P, double *move_cost, void *hip_stream);

/* Parameters of the evolutionary search. */
typedef struct {
    int32_t P;              /* population size, >= 1 */
    int32_t lambda;         /* offspring per generation, >= 1 */
    int32_t m_x;            /* crossover: device draws per offspring, >= 0 */
    int32_t m_m;            /* mutation: random position transpositions per offspring, >= 0 */
    int32_t ls_moves;       /* local-search rounds per offspring, >= 0 */
    int32_t neighbourhood;  /* DTFM_ALL_PAIRS, DTFM_GAIN4, DTFM_KL or DTFM_BEST4 */
    int32_t warm_start;     /* 1: `population` holds the initial population on entry */
} dtfm_ga_params;

/* Sec. 3.4 hybrid genetic algorithm, restated generation-wise: each generation draws, for each
 * of lambda offspring, two uniformly random parents from the generation-start population;
 * starts the child as parent 1 and m_x times picks a random device which, if parent 2 has it in
 * another stage, is swapped in the child with the device at a random slot of that stage; applies
 * m_m random transpositions; runs ls_moves local-search rounds; then keeps the P best of parents
 * and offspring ordered by (cost, origin index) with parents numbered first. All random numbers
 * are Philox4x32-10 words with key = seed and counter = (draw/4, candidate, generation, stream);
 * an integer in [0,n) is (word * n) >> 32. Unless warm_start, the initial population is P
 * Fisher-Yates shuffles of the identity.
 * population: device, P*N int32, out (in/out with warm_start); cost: device, P doubles, out,
 * ascending after at least one generation; best_trace: device, `generations` doubles, out:
 * lowest cost after each generation's replacement.
 * Errors: NULL, ARG, UNSUPPORTED (as for local_search), HIP. */
int dtfm_evolve(dtfm_problem *prob, uint64_t seed, int generations, const dtfm_ga_params *params,
                int32_t *population, double *cost, double *best_trace, void *hip_stream);

/* Fills out[0..n_blocks*4) (device, uint32) with the Philox4x32-10 blocks of counters
 * (first_block + b, k, g, stream) under key = seed: the generator of dtfm_evolve, exposed for
 * checking against published known-answer vectors. */
int dtfm_philox_blocks(uint64_t seed, uint32_t stream, uint32_t g, uint32_t k,
                       uint32_t first_block, int n_blocks, uint32_t *out, void *hip_stream);

/* Name of a status code; never null. */
const char *dtfm_status_string(int status);

/* Last HIP error text recorded by this library on the calling thread ("" if none). */
const char *dtfm_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* DTFM_H */
