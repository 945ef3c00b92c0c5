#!/usr/bin/env python3
"""Writes tests/golden/c5_evolve_seed7_P4096.txt: the first generations of the evolutionary search of
configuration 5 (N=1024, D_dp=64, D_pp=16, population 4096, Philox seed 7, 8 rounds of the
four-candidate local search per offspring) as the CPU ORACLE computes them.

    python tests/golden/make_c5_trace.py [--generations 2] [--threads 8]

With other arguments it writes the same kind of file for another configuration, e.g. the stored
tests/golden/c4_evolve_seed11_P1024_best4.txt (configuration 4 at its population, the four candidates of a
round judged by the cost):

    python tests/golden/make_c5_trace.py --config C4 --population 1024 --seed 11 --neighbourhood BEST4 \
        --generations 3 --out tests/golden/c4_evolve_seed11_P1024_best4.txt

Calls only oracle/ and the seeded input generator (workloads.py); nothing of the GPU library. The
oracle's evaluations are independent per candidate and run on `--threads` host threads
(oracle.Problem.evolve_by_generation, which tests/test_oracle_search.py shows equal to the oracle's
sequential evolve). One generation is 4096 x 9 cost evaluations of about 0.2 s each: about a quarter
of an hour on 8 cores.

File format (text): '#' comments; `key value` lines; doubles as 16 hex digits of their bit pattern.
  generation g (-1 = initial population): best cost, sha256 of the population (int32, row-major),
  sha256 of the costs (fp64); then the costs of the last generation in full, ascending.
"""
import argparse
import hashlib
import os
import struct
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
import workloads  # noqa: E402

OUT = os.path.join(HERE, "c5_evolve_seed7_P4096.txt")
SEED, P, LS_MOVES = 7, 4096, 8


def hexd(x):
    return "%016x" % struct.unpack("<Q", struct.pack("<d", float(x)))[0]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--generations", type=int, default=2)
    ap.add_argument("--threads", type=int, default=os.cpu_count() or 1)
    ap.add_argument("--out", default=OUT)
    ap.add_argument("--config", default="C5")
    ap.add_argument("--population", type=int, default=P)
    ap.add_argument("--seed", type=int, default=SEED)
    ap.add_argument("--neighbourhood", default="GAIN4", choices=["GAIN4", "KL", "BEST4"])
    args = ap.parse_args()
    return write_trace(args.config, args.seed, args.population, LS_MOVES, args.neighbourhood, args.generations,
                       args.threads, args.out)


def write_trace(config, SEED, P, LS_MOVES, neighbourhood, generations, threads, out):
    class args:   # the names used below
        pass
    args.generations, args.threads, args.out = generations, threads, out
    w = workloads.config(config)
    o = oracle.Problem(w.latency, w.bandwidth, w.c_dp, w.c_pp, w.D_dp, w.D_pp)
    lines = ["# written by tests/golden/make_c5_trace.py from the CPU oracle; do not edit",
             "# configuration %s: N=%d D_dp=%d D_pp=%d, workloads.config('%s'), defaults m_x=N/4, m_m=1" % (config[1:], w.N, w.D_dp, w.D_pp, config),
             "seed %d" % SEED, "population %d" % P, "ls_moves %d" % LS_MOVES, "neighbourhood %s" % neighbourhood,
             "generations %d" % args.generations]
    t0 = time.time()

    def report(g, pop, cost):
        pop = np.ascontiguousarray(pop, dtype="<i4")
        cost = np.ascontiguousarray(cost, dtype="<f8")
        lines.append("generation %d best %s population_sha256 %s cost_sha256 %s" % (
            g, hexd(cost.min()), hashlib.sha256(pop.tobytes()).hexdigest(), hashlib.sha256(cost.tobytes()).hexdigest()))
        print("generation %d done after %.0f s, best %.6f" % (g, time.time() - t0, cost.min()), flush=True)

    pop, cost, trace = o.evolve_by_generation(SEED, args.generations, P, ls_moves=LS_MOVES, neighbourhood=getattr(oracle, neighbourhood),
                                              threads=args.threads, on_generation=report)
    lines.append("best_trace " + " ".join(hexd(x) for x in trace))
    lines.append("final_costs")
    for i in range(0, P, 8):
        lines.append(" ".join(hexd(x) for x in cost[i:i + 8]))
    with open(args.out, "w") as f:
        f.write("\n".join(lines) + "\n")
    print("wrote", args.out)


if __name__ == "__main__":
    main()
