// C ABI of libdtfm: argument checking, problem handle, scratch arena, dispatch to the kernels.
#include "dtfm_internal.h"

#include <math.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <new>
#include <vector>

static thread_local char g_hip_error[256] = "";

int dtfm_hip_fail(hipError_t e, const char *what)
{
    snprintf(g_hip_error, sizeof(g_hip_error), "%s: %s", what, hipGetErrorString(e));
    (void)hipGetLastError();  // clear the sticky-less error slot
    return DTFM_ERR_HIP;
}

extern "C" const char *dtfm_last_hip_error(void) { return g_hip_error; }

extern "C" const char *dtfm_status_string(int status)
{
    switch (status) {
    case DTFM_OK: return "ok";
    case DTFM_ERR_NULL: return "null pointer";
    case DTFM_ERR_SHAPE: return "bad shape (need N = D_dp * D_pp, all >= 1, D_pp <= 16, D_dp <= 64, N <= 1024)";
    case DTFM_ERR_VALUE: return "bad value (latency/size must be finite and >= 0, bandwidth finite and > 0)";
    case DTFM_ERR_ARG: return "bad argument";
    case DTFM_ERR_HIP: return "HIP runtime error";
    case DTFM_ERR_UNSUPPORTED: return "unsupported for this problem shape";
    case DTFM_ERR_TOO_LARGE: return "population too large for the fixed scratch area of the allocation-free entry point";
    default: return "unknown status";
    }
}

// Scratch area of the allocation-free entry point: part of the library's device image, so every GPU the
// library runs on holds its own copy from the first use of the library until the process ends. In host
// code the array's name is only a handle for hipGetSymbolAddress; kernels and copies get the address that
// call returns for the current device, looked up once per device.
static __device__ __align__(256) unsigned char scratch[DTFM_FIXED_SCRATCH_BYTES];
#define DTFM_MAX_DEVICES 64
static char *g_fixed_scratch[DTFM_MAX_DEVICES];
static std::mutex g_fixed_scratch_mutex;

// address of `scratch` on `device`, which must be the current device
static int fixed_scratch_of(int device, char **out)
{
    if (device < 0 || device >= DTFM_MAX_DEVICES) return DTFM_ERR_ARG;
    std::lock_guard<std::mutex> lock(g_fixed_scratch_mutex);
    if (g_fixed_scratch[device] == nullptr) {
        void *ptr = nullptr;
        DTFM_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        g_fixed_scratch[device] = static_cast<char *>(ptr);
    }
    *out = g_fixed_scratch[device];
    return DTFM_OK;
}

static int ensure_scratch(dtfm_problem *pr, size_t bytes)
{
    if (bytes <= pr->scratch_bytes) return DTFM_OK;
    // earlier work on any stream may still use the old arena
    DTFM_HIP(hipDeviceSynchronize());
    if (pr->scratch != nullptr) {
        DTFM_HIP(hipFree(pr->scratch));
        pr->scratch = nullptr;
        pr->scratch_bytes = 0;
    }
    size_t want = bytes + bytes / 8;  // head room so slightly larger calls do not reallocate
    hipError_t e = hipMalloc((void **)&pr->scratch, want);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        want = bytes;
        DTFM_HIP(hipMalloc((void **)&pr->scratch, want));
    }
    pr->scratch_bytes = want;
    return DTFM_OK;
}

extern "C" int dtfm_create_problem(const double *latency, const double *bandwidth, int N, double c_dp,
                                   double c_pp, int D_dp, int D_pp, dtfm_problem **out)
{
    if (out == nullptr) return DTFM_ERR_NULL;
    *out = nullptr;
    if (latency == nullptr || bandwidth == nullptr) return DTFM_ERR_NULL;
    if (N < 1 || D_dp < 1 || D_pp < 1 || (long long)D_dp * D_pp != N || D_pp > DTFM_MAX_DPP ||
        D_dp > DTFM_MAX_DDP || N > DTFM_MAX_N)
        return DTFM_ERR_SHAPE;
    if (!isfinite(c_dp) || !isfinite(c_pp) || c_dp < 0.0 || c_pp < 0.0) return DTFM_ERR_VALUE;
    for (int d = 0; d < N; d++)
        for (int e = 0; e < N; e++) {
            if (d == e) continue;
            double a = latency[(size_t)d * N + e], b = bandwidth[(size_t)d * N + e];
            if (!isfinite(a) || a < 0.0 || !isfinite(b) || !(b > 0.0)) return DTFM_ERR_VALUE;
        }

    dtfm_problem *pr = new (std::nothrow) dtfm_problem();
    if (pr == nullptr) return DTFM_ERR_HIP;
    memset(pr, 0, sizeof(*pr));
    pr->N = N;
    pr->D_dp = D_dp;
    pr->D_pp = D_pp;
    pr->npairs = D_pp * (D_pp - 1) / 2;
    pr->c_dp = c_dp;
    pr->c_pp = c_pp;

    // subsets of the D_pp stage nodes ordered by size, for the layered Held-Karp sweep
    std::vector<uint32_t> subs;
    subs.reserve(((size_t)1 << D_pp));
    for (int k = 0; k <= D_pp + 1; k++) pr->hk_off.off[k] = 0;
    for (int k = 1; k <= D_pp; k++) {
        pr->hk_off.off[k] = (int)subs.size();
        for (uint32_t S = 1; S < (1u << D_pp); S++)
            if (__builtin_popcount(S) == k) subs.push_back(S);
    }
    pr->hk_off.off[D_pp + 1] = (int)subs.size();

    double *lat_dev = nullptr, *bw_dev = nullptr;
    size_t mat = (size_t)N * N * sizeof(double);
    int rc = DTFM_OK;
    auto fail = [&](int code) {
        if (lat_dev) (void)hipFree(lat_dev);
        if (bw_dev) (void)hipFree(bw_dev);
        dtfm_destroy_problem(pr);
        return code;
    };
#define CREATE_HIP(call)                                                    \
    do {                                                                    \
        hipError_t e__ = (call);                                            \
        if (e__ != hipSuccess) return fail(dtfm_hip_fail(e__, #call));      \
    } while (0)
    CREATE_HIP(hipGetDevice(&pr->device));
    rc = fixed_scratch_of(pr->device, &pr->fixed_scratch);
    if (rc != DTFM_OK) return fail(rc);
    CREATE_HIP(hipMalloc((void **)&pr->W_dp, mat));
    CREATE_HIP(hipMalloc((void **)&pr->W_pp, mat));
    CREATE_HIP(hipMalloc((void **)&pr->hk_subsets, subs.size() * sizeof(uint32_t)));
    CREATE_HIP(hipMalloc((void **)&lat_dev, mat));
    CREATE_HIP(hipMalloc((void **)&bw_dev, mat));
    CREATE_HIP(hipMemcpy(pr->hk_subsets, subs.data(), subs.size() * sizeof(uint32_t), hipMemcpyHostToDevice));
    CREATE_HIP(hipMemcpy(lat_dev, latency, mat, hipMemcpyHostToDevice));
    CREATE_HIP(hipMemcpy(bw_dev, bandwidth, mat, hipMemcpyHostToDevice));
    // the shard of Sec. 3.2: each device of a stage manages c_dp / D_dp bytes
    double shard = c_dp / (double)D_dp;
    rc = dtfm_weights_enqueue(lat_dev, bw_dev, N, shard, c_pp, pr->W_dp, pr->W_pp, (hipStream_t) nullptr);
    if (rc != DTFM_OK) return fail(rc);
    CREATE_HIP(hipDeviceSynchronize());
    CREATE_HIP(hipFree(lat_dev));
    lat_dev = nullptr;
    CREATE_HIP(hipFree(bw_dev));
    bw_dev = nullptr;
    if (dtfm_fast64_applicable(pr)) {
        rc = dtfm_fast64_prepare(pr);
        if (rc != DTFM_OK) return fail(rc);
        pr->fast64 = true;
    } else {
        // dense ranks of the pipeline weights for the matching kernel: the device-computed W_pp
        // is read back, sorted and deduplicated once (cold path); at most N^2 <= 2^20 distinct values
        std::vector<double> w((size_t)N * N), vals;
        CREATE_HIP(hipMemcpy(w.data(), pr->W_pp, mat, hipMemcpyDeviceToHost));
        vals = w;
        std::sort(vals.begin(), vals.end());
        vals.erase(std::unique(vals.begin(), vals.end()), vals.end());
        // the matching kernel's first solve works on the table of 16-bit codes 2 + (rank >> shift) <= 0xfffe; the
        // table of ranks serves the entries inside the optimum's bucket when shift > 0
        pr->rank_shift = 0;
        while (((vals.size() - 1) >> pr->rank_shift) + 2 > 0xfffe) pr->rank_shift++;
        std::vector<uint32_t> rk(w.size());
        std::vector<uint16_t> code(w.size());
        for (size_t i = 0; i < w.size(); i++) {
            rk[i] = (uint32_t)(std::lower_bound(vals.begin(), vals.end(), w[i]) - vals.begin());
            code[i] = (uint16_t)(2u + (rk[i] >> pr->rank_shift));
        }
        CREATE_HIP(hipMalloc((void **)&pr->W_code, code.size() * sizeof(uint16_t)));
        CREATE_HIP(hipMemcpy(pr->W_code, code.data(), code.size() * sizeof(uint16_t), hipMemcpyHostToDevice));
        CREATE_HIP(hipMalloc((void **)&pr->W_rank, rk.size() * sizeof(uint32_t)));
        CREATE_HIP(hipMalloc((void **)&pr->rank_val, vals.size() * sizeof(double)));
        CREATE_HIP(hipMemcpy(pr->W_rank, rk.data(), rk.size() * sizeof(uint32_t), hipMemcpyHostToDevice));
        CREATE_HIP(hipMemcpy(pr->rank_val, vals.data(), vals.size() * sizeof(double), hipMemcpyHostToDevice));
    }
#undef CREATE_HIP
    *out = pr;
    return DTFM_OK;
}

extern "C" void dtfm_destroy_problem(dtfm_problem *pr)
{
    if (pr == nullptr) return;
    (void)hipDeviceSynchronize();
    if (pr->W_dp) (void)hipFree(pr->W_dp);
    if (pr->W_pp) (void)hipFree(pr->W_pp);
    if (pr->hk_subsets) (void)hipFree(pr->hk_subsets);
    if (pr->W_rank) (void)hipFree(pr->W_rank);
    if (pr->W_code) (void)hipFree(pr->W_code);
    if (pr->rank_val) (void)hipFree(pr->rank_val);
    if (pr->scratch) (void)hipFree(pr->scratch);
    dtfm_fast64_release(pr);
    delete pr;
}

extern "C" int dtfm_get_weights(const dtfm_problem *pr, double *W_dp_host, double *W_pp_host)
{
    if (pr == nullptr) return DTFM_ERR_NULL;
    size_t mat = (size_t)pr->N * pr->N * sizeof(double);
    DTFM_HIP(hipDeviceSynchronize());
    if (W_dp_host) DTFM_HIP(hipMemcpy(W_dp_host, pr->W_dp, mat, hipMemcpyDeviceToHost));
    if (W_pp_host) DTFM_HIP(hipMemcpy(W_pp_host, pr->W_pp, mat, hipMemcpyDeviceToHost));
    return DTFM_OK;
}

extern "C" int dtfm_eval_population(dtfm_problem *pr, const int32_t *perm, int P, double *cost,
                                    void *hip_stream)
{
    if (pr == nullptr) return DTFM_ERR_NULL;
    if (P < 0) return DTFM_ERR_ARG;
    if (P == 0) return DTFM_OK;
    if (perm == nullptr || cost == nullptr) return DTFM_ERR_NULL;
    hipStream_t st = (hipStream_t)hip_stream;
    dtfm_arena measure = {nullptr, 0};
    dtfm_eval_carve(pr, measure, (size_t)P);
    int rc = ensure_scratch(pr, measure.off);
    if (rc != DTFM_OK) return rc;
    dtfm_arena ar = {pr->scratch, 0};
    dtfm_eval_bufs b = dtfm_eval_carve(pr, ar, (size_t)P);
    return dtfm_eval_enqueue(pr, b, perm, (size_t)P, cost, st);
}

// Carves the evaluation buffers for P rows out of the fixed scratch area; with the blocked Held-Karp kernel
// as many exchange areas as still fit behind them (fewer workgroups than a call that may allocate).
static int carve_fixed(const dtfm_problem *pr, size_t P, dtfm_eval_bufs *b)
{
    dtfm_arena measure = {nullptr, 0};
    dtfm_eval_carve(pr, measure, P, 1, true);
    if (measure.off > DTFM_FIXED_SCRATCH_BYTES) return DTFM_ERR_TOO_LARGE;
    size_t cap = 0;
    const size_t area = (dtfm_hk_exchange_bytes(pr) + 255) & ~(size_t)255;
    if (area != 0) {
        cap = 1 + (DTFM_FIXED_SCRATCH_BYTES - measure.off) / area;
        if (cap > P) cap = P;
        // rounding of the carved pieces to 256 bytes: make sure the chosen number fits
        for (;; cap--) {
            dtfm_arena m2 = {nullptr, 0};
            dtfm_eval_carve(pr, m2, P, cap, true);
            if (m2.off <= DTFM_FIXED_SCRATCH_BYTES) break;
            if (cap == 1) return DTFM_ERR_TOO_LARGE;
        }
    }
    dtfm_arena ar = {pr->fixed_scratch, 0};
    *b = dtfm_eval_carve(pr, ar, P, cap, true);
    return DTFM_OK;
}

extern "C" int dtfm_eval_population_noalloc(dtfm_problem *pr, const int32_t *perm, int P, double *cost,
                                            void *hip_stream)
{
    if (pr == nullptr) return DTFM_ERR_NULL;
    if (P < 0) return DTFM_ERR_ARG;
    if (P == 0) return DTFM_OK;
    if (perm == nullptr || cost == nullptr) return DTFM_ERR_NULL;
    int device = -1;
    DTFM_HIP(hipGetDevice(&device));
    if (device != pr->device) return DTFM_ERR_ARG;   // the handle's matrices and scratch copy live on its device
    dtfm_eval_bufs b;
    int rc = carve_fixed(pr, (size_t)P, &b);
    if (rc != DTFM_OK) return rc;
    return dtfm_eval_enqueue(pr, b, perm, (size_t)P, cost, (hipStream_t)hip_stream);
}

extern "C" int dtfm_coarsened_graph(dtfm_problem *pr, const int32_t *perm, int P, double *ghat,
                                    double *datap, void *hip_stream)
{
    if (pr == nullptr) return DTFM_ERR_NULL;
    if (P < 0) return DTFM_ERR_ARG;
    if (P == 0) return DTFM_OK;
    if (perm == nullptr) return DTFM_ERR_NULL;
    hipStream_t st = (hipStream_t)hip_stream;
    dtfm_arena measure = {nullptr, 0};
    dtfm_eval_carve(pr, measure, (size_t)P);
    int rc = ensure_scratch(pr, measure.off);
    if (rc != DTFM_OK) return rc;
    dtfm_arena ar = {pr->scratch, 0};
    dtfm_eval_bufs b = dtfm_eval_carve(pr, ar, (size_t)P);
    rc = dtfm_eval_enqueue(pr, b, perm, (size_t)P, nullptr, st);
    if (rc != DTFM_OK) return rc;
    size_t n = pr->D_pp;
    if (ghat) DTFM_HIP(hipMemcpyAsync(ghat, b.ghat, (size_t)P * n * n * sizeof(double), hipMemcpyDeviceToDevice, st));
    if (datap) DTFM_HIP(hipMemcpyAsync(datap, b.datap, (size_t)P * sizeof(double), hipMemcpyDeviceToDevice, st));
    return DTFM_OK;
}

extern "C" int dtfm_get_assignment(dtfm_problem *pr, const int32_t *perm, int P, int32_t *stage_order,
                                   int32_t *sigma, void *hip_stream)
{
    if (pr == nullptr) return DTFM_ERR_NULL;
    if (P < 0) return DTFM_ERR_ARG;
    if (P == 0) return DTFM_OK;
    if (perm == nullptr || stage_order == nullptr || sigma == nullptr) return DTFM_ERR_NULL;
    hipStream_t st = (hipStream_t)hip_stream;
    dtfm_arena measure = {nullptr, 0};
    dtfm_assign_carve(pr, measure, (size_t)P);
    int rc = ensure_scratch(pr, measure.off);
    if (rc != DTFM_OK) return rc;
    dtfm_arena ar = {pr->scratch, 0};
    dtfm_assign_bufs b = dtfm_assign_carve(pr, ar, (size_t)P);
    return dtfm_assign_enqueue(pr, b, perm, (size_t)P, stage_order, sigma, st);
}

extern "C" int dtfm_validate_population(dtfm_problem *pr, const int32_t *perm, int P, int32_t *bad_rows,
                                        void *hip_stream)
{
    if (pr == nullptr || bad_rows == nullptr) return DTFM_ERR_NULL;
    if (P < 0) return DTFM_ERR_ARG;
    if (P > 0 && perm == nullptr) return DTFM_ERR_NULL;
    return dtfm_validate_enqueue(pr, perm, (size_t)P, bad_rows, (hipStream_t)hip_stream);
}

static int check_neighbourhood(const dtfm_problem *pr, int neighbourhood)
{
    if (neighbourhood != DTFM_ALL_PAIRS && neighbourhood != DTFM_GAIN4 && neighbourhood != DTFM_KL && neighbourhood != DTFM_BEST4)
        return DTFM_ERR_ARG;
    // the paper's neighbourhood needs a link inside a stage and a second stage to swap with
    if ((neighbourhood == DTFM_GAIN4 || neighbourhood == DTFM_BEST4) && (pr->D_dp < 2 || pr->D_pp < 2)) return DTFM_ERR_UNSUPPORTED;
    if (neighbourhood == DTFM_KL && pr->D_pp < 2) return DTFM_ERR_UNSUPPORTED;   // no second stage to swap with
    return DTFM_OK;
}

extern "C" int dtfm_local_search(dtfm_problem *pr, int32_t *perm, int P, int moves, int neighbourhood,
                                 double *cost, int64_t *applied, void *hip_stream)
{
    if (pr == nullptr) return DTFM_ERR_NULL;
    if (P < 0 || moves < 0) return DTFM_ERR_ARG;
    int rc = check_neighbourhood(pr, neighbourhood);
    if (rc != DTFM_OK) return rc;
    if (P == 0) return DTFM_OK;
    if (perm == nullptr || cost == nullptr) return DTFM_ERR_NULL;
    dtfm_arena measure = {nullptr, 0};
    dtfm_ls_carve(pr, measure, (size_t)P, neighbourhood);
    rc = ensure_scratch(pr, measure.off);
    if (rc != DTFM_OK) return rc;
    dtfm_arena ar = {pr->scratch, 0};
    dtfm_ls_bufs b = dtfm_ls_carve(pr, ar, (size_t)P, neighbourhood);
    return dtfm_ls_enqueue(pr, b, perm, (size_t)P, moves, neighbourhood, cost, applied, (hipStream_t)hip_stream);
}

extern "C" int dtfm_move_costs(dtfm_problem *pr, const int32_t *perm, int P, double *move_cost, void *hip_stream)
{
    if (pr == nullptr) return DTFM_ERR_NULL;
    if (P < 0) return DTFM_ERR_ARG;
    if (P == 0 || pr->N < 2) return DTFM_OK;
    if (perm == nullptr || move_cost == nullptr) return DTFM_ERR_NULL;
    dtfm_arena measure = {nullptr, 0};
    dtfm_ls_carve(pr, measure, (size_t)P, DTFM_ALL_PAIRS, true);
    int rc = ensure_scratch(pr, measure.off);
    if (rc != DTFM_OK) return rc;
    dtfm_arena ar = {pr->scratch, 0};
    dtfm_ls_bufs b = dtfm_ls_carve(pr, ar, (size_t)P, DTFM_ALL_PAIRS, true);
    return dtfm_move_costs_enqueue(pr, b, perm, (size_t)P, move_cost, (hipStream_t)hip_stream);
}

extern "C" int dtfm_evolve(dtfm_problem *pr, uint64_t seed, int generations, const dtfm_ga_params *prm,
                           int32_t *population, double *cost, double *best_trace, void *hip_stream)
{
    if (pr == nullptr || prm == nullptr || population == nullptr || cost == nullptr) return DTFM_ERR_NULL;
    if (generations < 0 || prm->P < 1 || prm->lambda < 1 || prm->m_x < 0 || prm->m_m < 0 || prm->ls_moves < 0)
        return DTFM_ERR_ARG;
    if (generations > 0 && best_trace == nullptr) return DTFM_ERR_NULL;
    int rc = check_neighbourhood(pr, prm->neighbourhood);
    if (rc == DTFM_ERR_UNSUPPORTED && prm->ls_moves == 0) rc = DTFM_OK;  // neighbourhood unused
    if (rc != DTFM_OK) return rc;
    dtfm_arena measure = {nullptr, 0};
    dtfm_ga_carve(pr, measure, *prm);
    rc = ensure_scratch(pr, measure.off);
    if (rc != DTFM_OK) return rc;
    dtfm_arena ar = {pr->scratch, 0};
    dtfm_ga_bufs b = dtfm_ga_carve(pr, ar, *prm);
    return dtfm_ga_enqueue(pr, b, seed, generations, *prm, population, cost, best_trace, (hipStream_t)hip_stream);
}

extern "C" int dtfm_reserve(dtfm_problem *pr, int P, int lambda, int neighbourhood)
{
    if (pr == nullptr) return DTFM_ERR_NULL;
    if (P < 0 || lambda < 0) return DTFM_ERR_ARG;
    if (neighbourhood != DTFM_ALL_PAIRS && neighbourhood != DTFM_GAIN4 && neighbourhood != DTFM_KL && neighbourhood != DTFM_BEST4)
        return DTFM_ERR_ARG;
    const size_t rows = (size_t)(P > lambda ? P : lambda);
    if (rows == 0) return DTFM_OK;
    size_t need = 0;
    auto grow = [&](const dtfm_arena &m) { need = m.off > need ? m.off : need; };
    dtfm_arena m = {nullptr, 0};
    dtfm_eval_carve(pr, m, rows);
    grow(m);
    m = {nullptr, 0};
    dtfm_ls_carve(pr, m, rows, neighbourhood);
    grow(m);
    if (neighbourhood == DTFM_ALL_PAIRS) {   // dtfm_move_costs materialises every swap of a chunk
        m = {nullptr, 0};
        dtfm_ls_carve(pr, m, rows, neighbourhood, true);
        grow(m);
    }
    m = {nullptr, 0};
    dtfm_assign_carve(pr, m, rows);
    grow(m);
    if (P > 0 && lambda > 0) {
        dtfm_ga_params prm = {P, lambda, 0, 0, 0, neighbourhood, 0};
        m = {nullptr, 0};
        dtfm_ga_carve(pr, m, prm);
        grow(m);
    }
    return ensure_scratch(pr, need);
}

extern "C" int dtfm_philox_blocks(uint64_t seed, uint32_t stream, uint32_t g, uint32_t k, uint32_t first_block,
                                  int n_blocks, uint32_t *out, void *hip_stream)
{
    if (n_blocks < 0) return DTFM_ERR_ARG;
    if (n_blocks > 0 && out == nullptr) return DTFM_ERR_NULL;
    return dtfm_philox_enqueue(seed, stream, g, k, first_block, n_blocks, out, (hipStream_t)hip_stream);
}
