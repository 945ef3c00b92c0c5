#!/usr/bin/env python3
"""Benchmark of the scheduler hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

Workload: configuration C2 of the build (N=64 devices, D_DP=8, D_PP=8, GPT-1.3B-shaped message
sizes, 8 regions x 8 devices synthetic geo-distributed network, population 4096).

A step is one pass of the whole hot path = one generation of the evolutionary search on the
device: parent selection, crossover, mutation, `ls_moves` local-search rounds on every offspring
(proposal, full cost evaluation of the proposed allocation, accept), evaluation, replacement and
trace. `value` counts every candidate allocation whose cost (Eq. 1: DataP + bottleneck matchings +
Held-Karp) was evaluated inside the timed region, per second. Inputs are resident in HBM before
the timed region starts.

Besides the contract line this prints, in the same JSON object:
  roofline      the population-evaluation work (kernel(s) behind dtfm_eval_population), timed
                with HIP events on the launch stream, against the chip's vector-ALU peak;
  cpu_baseline  the CPU oracle timed on a bounded sample of the same workload on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import workloads  # noqa: E402

# ---- algorithmic operation count of one candidate evaluation (N, D_dp, D_pp) -------------------
# DataP (Eq. 2): N (D_dp-1) fp64 adds and N + D_pp max.
# Matching (Eq. 3), chosen algorithm = min-max subset DP over the columns of each D_dp x D_dp
#   block on 16-bit ranks: a state with k columns takes k max and k-1 min, states with k >= 2:
#   sum_k C(D_dp,k) (2k-1) 16-bit ops per stage pair (1785 at D_dp = 8), packed two per 32-bit
#   lane-op. What ANY algorithm must do is look at the D_dp^2 entries of every block once
#   (reported as `matching_compulsory_ops`).
# Held-Karp (Eq. 4): D_pp (D_pp-1) 2^(D_pp-2) relaxations of one fp64 add and one fp64 min.
# Peak: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz = 39.32 T lane-ops/s for 32/64-bit vector ops
# (fp64 add/min/max issue at full rate), twice that for packed 16-bit ops.
VALU_LANE_OPS_PER_S = 256 * 4 * 16 * 2.4e9
# HBM bytes per candidate of the evaluation kernel, from the rocprofv3 FETCH_SIZE / WRITE_SIZE runs
# summarised in profiles/k_eval_fast64_C2_P1048576.md (297.9 MB + 34.9 MB per 1,048,576 candidates,
# each counter scaled by its reading for a 1 GiB device copy; 19 MB of the reads are the 72 KiB of
# tables every workgroup stages in LDS, 26 MB of the writes register spills). Algorithmic: 4N + 8 = 264 B.
MEASURED_HBM_BYTES_PER_CANDIDATE = 317.4
# Counter readings of the same launch from the same file (rocprofv3 --pmc): share of the vector-ALU
# issue slots and of the LDS cycles in use, vector instructions per candidate.
MEASURED_COUNTERS = {"valu_busy_frac": 0.826, "lds_busy_frac": 0.403, "lds_bank_conflict_frac_of_lds": 0.47,
                     "valu_instructions_per_candidate": 651, "hbm_GBps": 245.0, "hbm_frac_of_8TBps": 0.031,
                     "source": "profiles/k_eval_fast64_C2_P1048576.md"}


def algorithmic_ops(N, D_dp, D_pp):
    from math import comb
    pairs = D_pp * (D_pp - 1) // 2
    dp = N * (D_dp - 1) + N + D_pp
    match16 = pairs * sum(comb(D_dp, k) * (2 * k - 1) for k in range(2, D_dp + 1))
    hk = D_pp * (D_pp - 1) * 2 ** (D_pp - 2) * 2 if D_pp >= 2 else 0
    return {"datap_fp64": dp, "matching_u16": match16, "held_karp_fp64": hk,
            "matching_compulsory_ops": pairs * D_dp * D_dp}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--roofline-only", action="store_true",
                    help="only the population-evaluation launches plus one 1 GiB device copy (for rocprofv3 runs)")
    ap.add_argument("--general-shapes", action="store_true",
                    help="only population evaluations at configurations C4 and C5 (for rocprofv3 runs of the "
                         "general-shape kernels)")
    ap.add_argument("--ls-throughput", action="store_true",
                    help="only the GAIN4 local search, 8 rounds on 2^20 candidates (for rocprofv3 runs of the fused "
                         "local-search kernel at a chip-filling population)")
    ap.add_argument("--all-pairs", action="store_true",
                    help="only configuration 3: 20 rounds of the ALL_PAIRS local search on 4096 candidates (for "
                         "rocprofv3 runs of the incremental move-evaluation kernel)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (candidates are independent and would shard "
              "without exchange; no multi-GPU path is built); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2206_01288_amd as dtfm

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dtfm.load_library()  # fails loudly when the HIP library is not built

    if args.general_shapes:
        res = {}
        for name, Pg in (("C4", 1024), ("C5", 4096)):
            wg = workloads.config(name)
            pg = dtfm.create_problem(wg.latency, wg.bandwidth, wg.c_dp, wg.c_pp, wg.D_dp, wg.D_pp)
            perms = torch.from_numpy(workloads.random_population(Pg, wg.N, seed=1)).cuda()
            out = torch.empty(Pg, dtype=torch.float64, device="cuda")
            dtfm.eval_population(pg, perms, out)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(3):
                dtfm.eval_population(pg, perms, out)
            torch.cuda.synchronize()
            res[name] = {"population": Pg, "ms_per_eval_population": (time.perf_counter() - t0) / 3 * 1e3}
            dtfm.destroy_problem(pg)
        print(json.dumps({"general_shapes": res}))
        return

    if args.ls_throughput:
        # the GAIN4 local search at a chip-filling population: 8 rounds on 2^20 candidates (for rocprofv3 runs of
        # k_ls_gain4_fast64<32>)
        w2 = workloads.config("C2")
        p2 = dtfm.create_problem(w2.latency, w2.bandwidth, w2.c_dp, w2.c_pp, w2.D_dp, w2.D_pp)
        base = torch.from_numpy(workloads.random_population(1 << 16, w2.N, seed=3)).cuda().repeat(16, 1).contiguous()
        rounds = 8
        d = base.clone()
        for _ in range(5):
            dtfm.local_search(p2, d, rounds, dtfm.GAIN4)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(10):
            dtfm.local_search(p2, d, rounds, dtfm.GAIN4)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / 10 * 1e3
        print(json.dumps({"ls_throughput": {"candidates": int(base.shape[0]), "rounds": rounds, "ms": ms,
                                            "trial_evaluations_per_s": base.shape[0] * (rounds + 1) / (ms * 1e-3)}}))
        return

    if args.all_pairs:
        w3 = workloads.config("C3")
        p3 = dtfm.create_problem(w3.latency, w3.bandwidth, w3.c_dp, w3.c_pp, w3.D_dp, w3.D_pp)
        base = torch.from_numpy(workloads.random_population(4096, w3.N, seed=1)).cuda()
        rounds, M = 20, w3.N * (w3.N - 1) // 2
        dtfm.local_search(p3, base.clone(), rounds, dtfm.ALL_PAIRS)
        torch.cuda.synchronize()
        ms = []
        for _ in range(3):
            d = base.clone()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            dtfm.local_search(p3, d, rounds, dtfm.ALL_PAIRS)
            torch.cuda.synchronize()
            ms.append((time.perf_counter() - t0) * 1e3)
        print(json.dumps({"all_pairs": {"candidates": 4096, "rounds": rounds, "moves_per_round": M, "ms": min(ms),
                                        "move_evaluations_per_s": 4096 * rounds * M / (min(ms) * 1e-3)}}))
        return

    w = workloads.config("C2")
    P, N = w.P, w.N
    ls_moves, nb = 8, dtfm.GAIN4
    prob = dtfm.create_problem(w.latency, w.bandwidth, w.c_dp, w.c_pp, w.D_dp, w.D_pp)
    pop0 = torch.from_numpy(workloads.random_population(P, N, seed=1)).cuda()

    if args.roofline_only:
        # what the committed rocprofv3 summaries are taken from: the evaluation kernel at the roofline
        # launch size, and a plain copy of known size to calibrate the HBM byte counters
        perms = torch.from_numpy(workloads.random_population(1 << 16, N, seed=3)).cuda().repeat(16, 1).contiguous()
        out = torch.empty(perms.shape[0], dtype=torch.float64, device="cuda")
        for _ in range(130):     # as many as the timed run below makes (30 warm-up + 100 timed)
            dtfm.eval_population(prob, perms, out)
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda")     # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"roofline_only": True, "eval_launch_candidates": int(perms.shape[0]),
                          "copy_bytes_each_way": int(src.numel() * 4)}))
        return

    # ---- the timed steps: K generations of the evolutionary search ---------------------------
    pop = pop0.clone()
    # an idle part needs some tens of milliseconds of work to reach its clocks: spin it up (untimed,
    # on a copy) before the W warm-up steps, so that a small W does not time the ramp
    dtfm.evolve(prob, seed=3, generations=400, P=P, ls_moves=ls_moves, neighbourhood=nb, population=pop0.clone())
    if args.warmup > 0:
        pop, _, _ = dtfm.evolve(prob, seed=1, generations=args.warmup, P=P, ls_moves=ls_moves,
                                neighbourhood=nb, population=pop)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    pop, cost, trace = dtfm.evolve(prob, seed=2, generations=args.steps, P=P, ls_moves=ls_moves,
                                   neighbourhood=nb, population=pop)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    evals = P + args.steps * P * (1 + ls_moves)     # initial population + per offspring: LS rounds + 1
    elapsed = t1 - t0
    best = float(trace[-1].item()) if args.steps > 0 else float("nan")

    # ---- roofline of the population-evaluation work, HIP events on the launch stream ---------
    def time_eval(Pe, reps, warm):
        """Average duration of one dtfm_eval_population launch on Pe candidates: `warm` untimed
        launches (the clocks of an idle part take some tens of milliseconds to come up), then `reps`
        launches back to back between two HIP events recorded on the launch stream."""
        base = torch.from_numpy(workloads.random_population(min(Pe, 1 << 16), N, seed=3)).cuda()
        perms = base if Pe <= base.shape[0] else base.repeat(Pe // base.shape[0], 1).contiguous()
        out = torch.empty(Pe, dtype=torch.float64, device="cuda")
        for _ in range(warm):
            dtfm.eval_population(prob, perms, out)
        start, end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        start.record()
        for _ in range(reps):
            dtfm.eval_population(prob, perms, out)
        end.record()
        torch.cuda.synchronize()
        return start.elapsed_time(end) * 1e-3 / reps

    ops = algorithmic_ops(N, w.D_dp, w.D_pp)
    t_small = time_eval(P, 200, 50)
    P_big = 1 << 20
    t_big = time_eval(P_big, 100, 30)
    ops64 = ops["datap_fp64"] + ops["held_karp_fp64"]
    ops16 = ops["matching_u16"]
    total_ops = ops64 + ops16
    # blended peak: the time the ALUs need at full issue rate for this op mix
    t_min_per_cand = ops64 / VALU_LANE_OPS_PER_S + ops16 / (2 * VALU_LANE_OPS_PER_S)
    peak = total_ops / t_min_per_cand / 1e12
    achieved = total_ops * P_big / t_big / 1e12
    roofline = {"bound": "alu", "achieved": achieved, "peak": peak, "unit": "Tops/s",
                "frac": achieved / peak, "traffic": MEASURED_HBM_BYTES_PER_CANDIDATE * P_big,
                "traffic_unit": "bytes per launch (rocprofv3 counters, see profiles/)",
                "algorithmic_hbm_bytes_per_launch": (4 * N + 8) * P_big,
                "kernel": "k_eval_fast64 (dtfm_eval_population)", "launch_candidates": P_big,
                "launch_seconds": t_big, "launches_timed": 100, "ops_per_candidate": ops,
                "rocprof_counters": MEASURED_COUNTERS,
                "eval_population_cands_per_s": {"P=4096": P / t_small, "P=1048576": P_big / t_big}}

    # ---- CPU oracle on a bounded sample of the same workload ----------------------------------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        opr = oracle.Problem(w.latency, w.bandwidth, w.c_dp, w.c_pp, w.D_dp, w.D_pp)
        threads = max(1, min(16, os.cpu_count() or 1))
        sample = workloads.random_population(32 * P, N, seed=3)
        chunks = np.array_split(sample, threads * 4)
        c0 = time.perf_counter()
        with ThreadPoolExecutor(threads) as ex:
            res = list(ex.map(opr.eval_population, chunks))
        c1 = time.perf_counter()
        cpu = {"value": sample.shape[0] / (c1 - c0), "unit": "candidates/s", "cores": threads, "kind": "oracle",
               "sample": "%d random C2 candidates, full cost evaluation each (oracle eval_population), "
                         "%d threads over contiguous chunks" % (sample.shape[0], threads)}
        # the same on one core, and the oracle's evolutionary step (sequential C, one thread) on a
        # population of 512: evaluations per second inside it, and what that makes per generation of
        # the bench's size
        c0 = time.perf_counter()
        opr.eval_population(sample[:P])
        c1 = time.perf_counter()
        cpu["single_core_value"] = P / (c1 - c0)
        Pg = 512
        c0 = time.perf_counter()
        opr.evolve(2, 1, Pg, ls_moves=ls_moves, neighbourhood=oracle.GAIN4)
        c1 = time.perf_counter()
        ga_evals = Pg + Pg * (1 + ls_moves)
        cpu["ga_step"] = {"evaluations_per_s": ga_evals / (c1 - c0), "cores": 1,
                          "generations_per_s_at_population_%d" % P: ga_evals / (c1 - c0) / (P * (1 + ls_moves)),
                          "sample": "oracle evolve, 1 generation, population %d, %d GAIN4 rounds" % (Pg, ls_moves)}
        # the GPU result on the same rows must agree with what was just timed
        g = dtfm.eval_population(prob, torch.from_numpy(sample[:P]).cuda()).cpu().numpy()
        assert np.array_equal(g, np.concatenate(res)[:P]), "GPU and oracle disagree"

    line = {
        "metric": "candidate allocations evaluated/sec (N=64, D_DP=8, D_PP=8)",
        "value": evals / elapsed,
        "unit": "candidates/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": elapsed / max(args.steps, 1) * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f64",
        "data": "synthetic",
        "config": {"workload": "C2: N=64, D_DP=8, D_PP=8, GPT-1.3B-shaped sizes, 8x8-region synthetic network, "
                               "population 4096; step = one GA generation (select, crossover, mutation, "
                               "%d GAIN4 local-search rounds, evaluation, replacement)" % ls_moves,
                   "population": P, "offspring_per_generation": P, "ls_moves": ls_moves,
                   "evaluations_in_timed_region": evals},
        "generations_per_s": args.steps / elapsed,
        "best_cost_after_last_step_s": best,
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    # the timed GA step against the same peak, counting every evaluation as a full one (a trial
    # evaluation of the local search re-matches only 13 of the 28 stage pairs)
    equiv = total_ops * evals / elapsed / 1e12
    roofline["timed_step"] = {"kernel": "k_ls_gain4_fast64 (83 % of a generation)", "population": P,
                              "full_evaluation_equivalent_Tops_per_s": equiv, "frac_of_peak": equiv / peak,
                              "note": "4096 offspring give one wavefront of four candidates per SIMD: the "
                                      "step is bound by that wavefront's instruction stream, not by the "
                                      "chip's issue rate"}
    print(json.dumps(line))


if __name__ == "__main__":
    main()
