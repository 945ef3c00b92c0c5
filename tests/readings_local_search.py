"""Readings of the paper's local search (Sec. 3.4, "Improving Local Search Strategy") compared on the CPU.

    python -m tests.readings_local_search [--budget 200000] [--population 64] [--procs 6]

The paper says which four swaps a pair of stages offers (the end points of the fastest link inside each) and
how they are ranked (its Gain function); it does not say which stage pairs a local search visits, how many
swaps it tries, or whether a swap is applied on its gain or on the cost. This script runs the evolutionary
loop (the oracle's selection / crossover / mutation and replacement) with several readings of that local
search, all at the same budget of cost evaluations (Eq. 1), and prints the best cost reached (mean over
seeds 0, 1, 2, as in the paper's comparison of search strategies):

  none        no local search: every evaluation is a new offspring
  gain4       the build's reading: round r looks at stage pair r mod npairs, proposes the best of the four
              swaps by Gain, applies it iff the cost drops (1 evaluation per round, 8 rounds)
  gain4-sweep the same with one round per stage pair (npairs rounds): every pair visited once per offspring
  best4       round r looks at stage pair r mod npairs and evaluates all four swaps; the cheapest is applied
              iff the cost drops (4 evaluations per round, 2 rounds)
  global      every round ranks the four swaps of ALL stage pairs by Gain and tries them in that order until
              one lowers the cost (at most 4 evaluations per round, 2 rounds)
  kl          as gain4 with the Kernighan-Lin gain over all D_dp^2 swaps of the round's stage pair

TEST INFRASTRUCTURE (it drives the CPU oracle); nothing in the GPU library depends on it.
"""
import argparse
import itertools
from concurrent.futures import ProcessPoolExecutor

import numpy as np

import oracle
import workloads


def _swap(perm, a, b):
    q = perm.copy()
    q[a], q[b] = q[b], q[a]
    return q


class Run:
    def __init__(self, name, budget, generations=0):
        w = workloads.config(name)
        self.w = w
        self.pr = oracle.Problem(w.latency, w.bandwidth, w.c_dp, w.c_pp, w.D_dp, w.D_pp)
        self.pairs = list(itertools.combinations(range(w.D_pp), 2))
        self.evals = 0
        self.budget = budget
        self.generations = generations   # > 0: stop after that many generations instead of at the budget

    def cost(self, perm):
        self.evals += 1
        return self.pr.comm_cost(perm)

    def four(self, perm, pair_no):
        """The four swaps of stage pair `pair_no` with their gains: [(gain, a, b)] in the paper's order."""
        D = self.w.D_dp
        j, jp = self.pairs[pair_no]
        W = self.pr.W_pp
        Cj, Cjp = perm[j * D:(j + 1) * D], perm[jp * D:(jp + 1) * D]

        def fastest(C):
            best = None
            for i in range(D):
                for k in range(i + 1, D):
                    if best is None or W[C[i], C[k]] < best[0]:
                        best = (W[C[i], C[k]], i, k)
            return best[1], best[2]

        s, sp = fastest(Cj), fastest(Cjp)
        out = []
        for xi in (0, 1):
            for yi in (0, 1):
                x, mx, y, my = Cj[s[xi]], Cj[s[1 - xi]], Cjp[sp[yi]], Cjp[sp[1 - yi]]
                g = W[x, Cjp].sum() / D - W[x, mx] + W[y, Cj].sum() / D - W[y, my]
                out.append((g, j * D + s[xi], jp * D + sp[yi]))
        return out

    # ---- local searches: (perm, cost) -> (perm, cost) ----
    def ls_none(self, perm, c):
        return perm, c

    def ls_gain4(self, perm, c, rounds=8):
        for r in range(rounds):
            a, b, _ = self.pr.gain4_propose(perm, r)
            q = _swap(perm, a, b)
            cq = self.cost(q)
            if cq < c:
                perm, c = q, cq
        return perm, c

    def ls_gain4_sweep(self, perm, c):
        return self.ls_gain4(perm, c, rounds=len(self.pairs))

    def ls_kl(self, perm, c, rounds=8):
        for r in range(rounds):
            a, b, _ = self.pr.kl_propose(perm, r)
            q = _swap(perm, a, b)
            cq = self.cost(q)
            if cq < c:
                perm, c = q, cq
        return perm, c

    def ls_best4(self, perm, c, rounds=2):
        for r in range(rounds):
            best = None
            for _, a, b in self.four(perm, r % len(self.pairs)):
                q = _swap(perm, a, b)
                cq = self.cost(q)
                if best is None or cq < best[0]:
                    best = (cq, q)
            if best[0] < c:
                c, perm = best
        return perm, c

    def ls_global(self, perm, c, rounds=2, tries=4):
        for r in range(rounds):
            cands = []
            for t in range(len(self.pairs)):
                cands += self.four(perm, t)
            cands.sort(key=lambda e: -e[0])
            for _, a, b in cands[:tries]:
                q = _swap(perm, a, b)
                cq = self.cost(q)
                if cq < c:
                    perm, c = q, cq
                    break
        return perm, c

    def evolve(self, seed, P, ls):
        w = self.w
        pop = np.stack([oracle.init_candidate(seed, k, w.N) for k in range(P)])
        cost = np.array([self.cost(p) for p in pop])
        g = 0
        while (g < self.generations) if self.generations > 0 else (self.evals < self.budget):
            off, oc = [], []
            for k in range(P):
                child = oracle.make_offspring(seed, g, k, pop, w.D_dp, w.N // 4, 1)[0]
                child, c = ls(child, self.cost(child))
                off.append(child)
                oc.append(c)
                if self.generations <= 0 and self.evals >= self.budget:
                    break
            allp = np.concatenate([pop, np.stack(off)])
            allc = np.concatenate([cost, np.array(oc)])
            keep = np.lexsort((np.arange(len(allc)), allc))[:P]
            pop, cost = allp[keep], allc[keep]
            g += 1
        return cost[0], g


def one(args):
    name, variant, seed, budget, P, gens = args
    run = Run(name, budget, gens)
    best, gens = run.evolve(seed, P, getattr(run, "ls_" + variant.replace("-", "_")))
    return name, variant, seed, best, gens, run.evals


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--budget", type=int, default=200000)
    ap.add_argument("--population", type=int, default=64)
    ap.add_argument("--procs", type=int, default=6)
    ap.add_argument("--networks", default="C2b,C2")
    ap.add_argument("--generations", type=int, default=0, help="> 0: the same number of generations (offspring) for every "
                    "reading instead of the same number of evaluations")
    args = ap.parse_args()
    variants = ["none", "gain4", "gain4-sweep", "best4", "global", "kl"]
    jobs = [(n, v, s, args.budget, args.population, args.generations) for n in args.networks.split(",") for v in variants for s in (0, 1, 2)]
    with ProcessPoolExecutor(args.procs) as ex:
        res = list(ex.map(one, jobs))
    if args.generations > 0:
        print("%d generations each, population %d" % (args.generations, args.population))
    else:
        print("budget %d evaluations, population %d" % (args.budget, args.population))
    for n in args.networks.split(","):
        rand = Run(n, 0)
        rc = [rand.pr.comm_cost(p) for p in workloads.random_population(1024, rand.w.N, seed=9)]
        print("%s: random allocations mean %.3f, best of 1024 %.3f" % (n, np.mean(rc), np.min(rc)))
        for v in variants:
            rows = [r for r in res if r[0] == n and r[1] == v]
            print("  %-12s best cost mean %.3f  (seeds: %s; generations %s; evaluations %s)" % (
                v, np.mean([r[3] for r in rows]), " ".join("%.3f" % r[3] for r in rows), " ".join(str(r[4]) for r in rows),
                " ".join(str(r[5]) for r in rows)))


if __name__ == "__main__":
    main()
