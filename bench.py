#!/usr/bin/env python3
"""Benchmark of the scheduler hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

Workload: configuration C2 of the build (N=64 devices, D_DP=8, D_PP=8, GPT-1.3B-shaped message
sizes, 8 regions x 8 devices synthetic geo-distributed network, population 4096). Inputs are
resident in HBM before any timed region starts.

A step is one dtfm_eval_population call on the whole population: the cost (Eq. 1: DataP +
bottleneck matchings + Held-Karp) of each of its 4096 candidate allocations. `value` = candidates
per second over the K timed steps: the first of the two metrics. The second, generations of the
evolutionary search per second (selection, crossover, mutation, 8 rounds of the four-candidate
local search per offspring, replacement, trace; population 4096), is timed in the same run and
reported as `generations_per_s`.

Besides the contract line this prints, in the same JSON object:
  roofline          the population-evaluation kernel at a chip-filling launch (2^20 candidates), timed
                    with HIP events on the launch stream, against the chip's vector-ALU peak: with the op
                    count of the algorithms chosen here and with the count no algorithm can avoid; the
                    same at the configured population; the GA generation with its own op count;
  roofline_general  the general-shape kernels at configurations C4 and C5 (D_PP = 16);
  cpu_baseline      the CPU oracle timed on a bounded sample of the same workload on the host cores.
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


def read_profile_figures(name):
    """The machine-readable figures of a committed rocprofv3 summary under profiles/ (the line that starts
    with `bench-figures:` holds a JSON object), with the file named as their source; None when the file or
    the line is missing. These are readings of the committed profile run, not of this run."""
    path = os.path.join(ROOT, "profiles", name)
    try:
        with open(path) as f:
            for ln in f:
                if ln.startswith("bench-figures:"):
                    d = json.loads(ln[len("bench-figures:"):])
                    d["source"] = "profiles/" + name + " (rocprofv3 run of `bench.py --roofline-only`, not of this run)"
                    return d
    except OSError:
        pass
    return None


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
    ap.add_argument("--ga-generations", type=int, default=100, help="generations of the evolutionary search timed for generations_per_s")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-general", action="store_true", help="skip the C4 / C5 general-shape timings")
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
        # launch size and at the configured population, and a plain copy of known size to calibrate the
        # HBM byte counters
        perms = torch.from_numpy(workloads.random_population(1 << 16, N, seed=3)).cuda().repeat(16, 1).contiguous()
        out = torch.empty(perms.shape[0], dtype=torch.float64, device="cuda")
        for _ in range(130):     # as many as the timed run below makes (30 warm-up + 100 timed)
            dtfm.eval_population(prob, perms, out)
        for _ in range(250):
            dtfm.eval_population(prob, pop0, out[:P])
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda")     # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"roofline_only": True, "eval_launch_candidates": int(perms.shape[0]),
                          "copy_bytes_each_way": int(src.numel() * 4)}))
        return

    dtfm.reserve(prob, 1 << 20, P, nb)     # no allocation or device synchronisation inside the timed calls

    # an idle part needs some tens of milliseconds of work to reach its clocks: spin it up (untimed,
    # on a copy) before the W warm-up steps, so that a small W does not time the ramp
    dtfm.evolve(prob, seed=3, generations=400, P=P, ls_moves=ls_moves, neighbourhood=nb, population=pop0.clone())

    # ---- metric (i), the timed steps: K launches of dtfm_eval_population on the configured population ----
    cost_out = torch.empty(P, dtype=torch.float64, device="cuda")
    for _ in range(args.warmup):
        dtfm.eval_population(prob, pop0, cost_out)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(args.steps):
        dtfm.eval_population(prob, pop0, cost_out)
    ev1.record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    t_small = ev0.elapsed_time(ev1) * 1e-3 / max(args.steps, 1)     # HIP events on the launch stream

    # ---- metric (ii): generations of the evolutionary search per second ------------------------------
    ga_gens = args.ga_generations
    pop, _, _ = dtfm.evolve(prob, seed=1, generations=20, P=P, ls_moves=ls_moves, neighbourhood=nb, population=pop0.clone())
    torch.cuda.synchronize()
    g0 = time.perf_counter()
    pop, cost, trace = dtfm.evolve(prob, seed=2, generations=ga_gens, P=P, ls_moves=ls_moves, neighbourhood=nb, population=pop)
    torch.cuda.synchronize()
    ga_elapsed = time.perf_counter() - g0
    best = float(trace[-1].item()) if ga_gens > 0 else float("nan")

    # ---- roofline of the population-evaluation kernel, HIP events on the launch stream ---------------
    def time_eval(problem, perms, reps, warm, fn=None):
        """Average duration of one launch of fn (default dtfm_eval_population) on `perms`: `warm` untimed
        launches, then `reps` back to back between two HIP events recorded on the launch stream."""
        out = torch.empty(perms.shape[0], dtype=torch.float64, device="cuda")
        call = (lambda: dtfm.eval_population(problem, perms, out)) if fn is None else fn
        for _ in range(warm):
            call()
        start, end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        start.record()
        for _ in range(reps):
            call()
        end.record()
        torch.cuda.synchronize()
        return start.elapsed_time(end) * 1e-3 / reps

    ops = algorithmic_ops(N, w.D_dp, w.D_pp)
    P_big = 1 << 20
    base = torch.from_numpy(workloads.random_population(1 << 16, N, seed=3)).cuda()
    t_big = time_eval(prob, base.repeat(P_big // base.shape[0], 1).contiguous(), 100, 30)
    ops64 = ops["datap_fp64"] + ops["held_karp_fp64"]
    ops16 = ops["matching_u16"]
    total_ops = ops64 + ops16
    # blended peak of the chosen algorithm's op mix: the time the ALUs need at full issue rate
    t_min_per_cand = ops64 / VALU_LANE_OPS_PER_S + ops16 / (2 * VALU_LANE_OPS_PER_S)
    peak = total_ops / t_min_per_cand / 1e12
    achieved = total_ops * P_big / t_big / 1e12
    # the count that does not depend on the matching algorithm: DataP + one look at every block entry + Held-Karp,
    # all at the 64-bit lane-op rate
    indep_ops = ops64 + ops["matching_compulsory_ops"]
    indep_peak = VALU_LANE_OPS_PER_S / 1e12
    prof = read_profile_figures("k_eval_fast64_C2_P1048576.md")
    roofline = {"bound": "alu", "achieved": achieved, "peak": peak, "unit": "Tops/s",
                "frac": achieved / peak,
                "traffic": prof.get("hbm_bytes_per_candidate", 0.0) * P_big if prof else None,
                "traffic_unit": "bytes per launch", "traffic_source": prof.get("source") if prof else None,
                "algorithmic_hbm_bytes_per_launch": (4 * N + 8) * P_big,
                "kernel": "k_eval_fast64<32> (dtfm_eval_population)", "launch_candidates": P_big,
                "launch_seconds": t_big, "launches_timed": 100, "ops_per_candidate": ops,
                "frac_is": "ops of the chosen algorithms (DataP, subset-DP matching on packed 16-bit ranks, Held-Karp) "
                           "against the blended peak of that mix",
                "algorithm_independent": {"ops_per_candidate": indep_ops, "achieved": indep_ops * P_big / t_big / 1e12,
                                          "peak": indep_peak, "unit": "Tops/s",
                                          "frac": indep_ops * P_big / t_big / 1e12 / indep_peak,
                                          "is": "DataP adds and maxima + one look at each of the D_dp^2 entries of every "
                                                "stage-pair block + Held-Karp add/min, against the 64-bit vector-op peak"},
                "at_configured_population": {"kernel": "k_eval_fast64_paired", "launch_candidates": P, "launch_seconds": t_small,
                                             "achieved": total_ops * P / t_small / 1e12, "frac": total_ops * P / t_small / 1e12 / peak,
                                             "algorithm_independent_frac": indep_ops * P / t_small / 1e12 / indep_peak},
                "rocprof_counters": prof,
                "eval_population_cands_per_s": {"P=%d" % P: P / t_small, "P=%d" % P_big: P_big / t_big}}
    # the GA generation against the same peak with the op count of what it does: per offspring one full evaluation
    # and ls_moves trial evaluations, each of which re-matches the 2 D_pp - 3 stage pairs of the round's two stages,
    # redoes their two DataP stages and runs Held-Karp in full
    trial_ops64 = 2 * (w.D_dp * (w.D_dp - 1) + w.D_dp) + w.D_pp + ops["held_karp_fp64"]
    trial_ops16 = (2 * w.D_pp - 3) * ops["matching_u16"] // (w.D_pp * (w.D_pp - 1) // 2)
    gen_t_min = P * ((ops64 + ls_moves * trial_ops64) / VALU_LANE_OPS_PER_S + (ops16 + ls_moves * trial_ops16) / (2 * VALU_LANE_OPS_PER_S))
    roofline["ga_generation"] = {"kernel": "k_ls_gain4_fast64<4, true> + k_rank_count + k_rank_place", "population": P,
                                 "ops_per_trial_evaluation": {"fp64": trial_ops64, "u16": trial_ops16},
                                 "seconds_per_generation": ga_elapsed / max(ga_gens, 1),
                                 "frac_of_alu_peak": gen_t_min / (ga_elapsed / max(ga_gens, 1)) if ga_gens > 0 else None}

    # ---- the general-shape kernels at C4 and C5: Held-Karp (D_pp = 16) and the rest, HIP events ------
    general = None
    if not args.no_general:
        general = {}
        for name, Pg in (("C4", 1024), ("C5", 4096)):
            wg = workloads.config(name)
            pg = dtfm.create_problem(wg.latency, wg.bandwidth, wg.c_dp, wg.c_pp, wg.D_dp, wg.D_pp)
            dtfm.reserve(pg, Pg, 0, nb)
            perms = torch.from_numpy(workloads.random_population(Pg, wg.N, seed=1)).cuda()
            t_eval = time_eval(pg, perms, 5, 2)
            gh = torch.empty((Pg, wg.D_pp, wg.D_pp), dtype=torch.float64, device="cuda")
            dpv = torch.empty(Pg, dtype=torch.float64, device="cuda")
            t_front = time_eval(pg, perms, 5, 2, fn=lambda: dtfm.coarsened_graph(pg, perms, out=(gh, dpv)))
            og = algorithmic_ops(wg.N, wg.D_dp, wg.D_pp)
            t_hk = max(t_eval - t_front, 1e-9)
            nh = wg.D_pp - 10
            xchg = 2 * (nh * 2 ** (nh - 1)) * 1024 * 8 if nh > 0 else 0     # exchange entries written and read back
            general[name] = {"population": Pg, "seconds_eval_population": t_eval,
                             "seconds_datap_and_matching": t_front, "seconds_held_karp": t_hk,
                             "candidates_per_s": Pg / t_eval,
                             "held_karp": {"relaxations_per_s": og["held_karp_fp64"] / 2 * Pg / t_hk,
                                           "achieved_Tops_per_s": og["held_karp_fp64"] * Pg / t_hk / 1e12,
                                           "peak_Tops_per_s": indep_peak,
                                           "frac_of_fp64_alu_peak": og["held_karp_fp64"] * Pg / t_hk / 1e12 / indep_peak,
                                           "exchange_bytes_per_s": xchg * Pg / t_hk,
                                           "exchange_frac_of_8TBps": xchg * Pg / t_hk / 8e12},
                             "datap_and_matching": {"block_entries_per_s": og["matching_compulsory_ops"] * Pg / t_front,
                                                    "datap_adds_per_s": wg.N * (wg.D_dp - 1) * Pg / t_front,
                                                    # every block entry is one lane of a gather from the table of codes;
                                                    # bare gathers of 64 random 2-byte columns of a table row run at 1.74
                                                    # lanes per cycle and CU (profiles/gather_rate_gfx950.md)
                                                    "gather_lanes_peak_per_s": 256 * 1.74 * 2.4e9,
                                                    "frac_of_gather_rate": og["matching_compulsory_ops"] * Pg / t_front
                                                                           / (256 * 1.74 * 2.4e9)},
                             "timing": "HIP events over 5 launches each of dtfm_eval_population and of dtfm_coarsened_graph "
                                       "(DataP + matching only); Held-Karp = the difference"}
            dtfm.destroy_problem(pg)

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
        "value": P * args.steps / elapsed,
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
                               "population 4096; step = one dtfm_eval_population call on the whole population "
                               "(Eq. 1 in full for each of its 4096 candidates)",
                   "population": P, "candidates_per_step": P},
        "value_at_population_1048576": P_big / t_big,
        "generations_per_s": ga_gens / ga_elapsed if ga_gens > 0 else None,
        "ga": {"generations_timed": ga_gens, "population": P, "offspring_per_generation": P, "ls_moves": ls_moves,
               "neighbourhood": "GAIN4", "ms_per_generation": ga_elapsed / max(ga_gens, 1) * 1e3,
               "evaluations_per_generation": {"full": P, "trial (2 D_pp - 3 of the stage pairs re-matched)": P * ls_moves},
               "best_cost_after_last_generation_s": best},
        "roofline": roofline,
        "roofline_general": general,
        "cpu_baseline": cpu,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
