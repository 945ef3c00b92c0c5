"""Python face of the CPU oracle (oracle/dtfm_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
cpu_baseline leg. The GPU library never imports this package and this package never imports the
GPU library. Everything here is argument marshalling around the plain-C functions; the
arithmetic lives in the C file, each function citing the passage of the paper it follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from ctypes import POINTER, c_double, c_int, c_long, c_uint32, c_uint64, c_void_p

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dtfm_oracle.c")
_LIB = os.path.join(_HERE, "libdtfm_oracle.so")

ALL_PAIRS = 0
GAIN4 = 1
KL = 2
BEST4 = 3


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no FMA contraction, so every written operation rounds once)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-ffp-contract=off",
                               "-fno-fast-math", "-Wall", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class GAParams(ctypes.Structure):
    _fields_ = [("P", c_int), ("lam", c_int), ("m_x", c_int), ("m_m", c_int),
                ("ls_moves", c_int), ("neighbourhood", c_int), ("warm_start", c_int)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        dp, ip, lp = POINTER(c_double), POINTER(c_int), POINTER(c_long)
        L.orc_weights.argtypes = [dp, dp, c_int, c_double, c_double, c_int, dp, dp]
        L.orc_datap_stage.argtypes = [dp, c_int, ip, c_int]
        L.orc_datap_stage.restype = c_double
        L.orc_datap.argtypes = [dp, c_int, ip, c_int, c_int]
        L.orc_datap.restype = c_double
        L.orc_threshold_feasible.argtypes = [dp, c_int, c_double]
        L.orc_threshold_feasible.restype = c_int
        L.orc_bottleneck_match.argtypes = [dp, c_int]
        L.orc_bottleneck_match.restype = c_double
        L.orc_bottleneck_match_brute.argtypes = [dp, c_int]
        L.orc_bottleneck_match_brute.restype = c_double
        L.orc_coarsen.argtypes = [dp, c_int, ip, c_int, c_int, c_int, dp]
        L.orc_open_tsp_held_karp.argtypes = [dp, c_int]
        L.orc_open_tsp_held_karp.restype = c_double
        L.orc_open_tsp_brute.argtypes = [dp, c_int]
        L.orc_open_tsp_brute.restype = c_double
        L.orc_comm_cost.argtypes = [dp, dp, c_int, c_int, c_int, ip, c_int]
        L.orc_comm_cost.restype = c_double
        L.orc_eval_population.argtypes = [dp, dp, c_int, c_int, c_int, ip, c_int, dp]
        L.orc_hk_path.argtypes = [dp, c_int, ip]
        L.orc_lexmin_matching.argtypes = [dp, c_int, c_double, ip]
        L.orc_lexmin_matching.restype = c_int
        L.orc_get_assignment.argtypes = [dp, c_int, c_int, c_int, ip, ip, ip]
        L.orc_four_candidates.argtypes = [dp, c_int, c_int, c_int, ip, c_int, ip, ip]
        L.orc_gain4_propose.argtypes = [dp, c_int, c_int, c_int, ip, c_int, ip, ip, dp]
        L.orc_kl_propose.argtypes = [dp, c_int, c_int, c_int, ip, c_int, ip, ip, dp]
        L.orc_local_search.argtypes = [dp, dp, c_int, c_int, c_int, ip, c_int, c_int, c_int, dp, lp]
        L.orc_philox4x32_10.argtypes = [POINTER(c_uint32), POINTER(c_uint32), POINTER(c_uint32)]
        L.orc_draw_randint.argtypes = [c_uint64, c_uint32, c_uint32, c_uint32, c_uint32, c_uint32]
        L.orc_draw_randint.restype = c_uint32
        L.orc_init_candidate.argtypes = [c_uint64, c_int, c_int, ip]
        L.orc_make_offspring.argtypes = [c_uint64, c_int, c_int, ip, c_int, c_int, c_int, c_int, c_int, ip, ip]
        L.orc_replace.argtypes = [c_int, c_int, c_int, ip, dp, ip, dp]
        L.orc_evolve.argtypes = [dp, dp, c_int, c_int, c_int, c_uint64, c_int, POINTER(GAParams), ip, dp, dp]
        _lib = L
    return _lib


def _d(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(POINTER(c_double))


def _i(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(POINTER(c_int))


class Problem:
    """Weights of one problem instance (Sec. 2 graph G folded into the Eq. 2 / Eq. 3 terms)."""

    def __init__(self, latency, bandwidth, c_dp, c_pp, D_dp, D_pp):
        latency = np.ascontiguousarray(latency, dtype=np.float64)
        N = latency.shape[0]
        assert D_dp * D_pp == N
        self.N, self.D_dp, self.D_pp = N, D_dp, D_pp
        self.c_dp, self.c_pp = float(c_dp), float(c_pp)
        self.W_dp = np.empty((N, N))
        self.W_pp = np.empty((N, N))
        _, pl = _d(latency)
        bwc, pb = _d(bandwidth)
        lib().orc_weights(pl, pb, N, self.c_dp, self.c_pp, D_dp,
                          self.W_dp.ctypes.data_as(POINTER(c_double)),
                          self.W_pp.ctypes.data_as(POINTER(c_double)))

    def _w(self):
        return (self.W_dp.ctypes.data_as(POINTER(c_double)), self.W_pp.ctypes.data_as(POINTER(c_double)))

    def datap(self, perm) -> float:
        perm, pp = _i(perm)
        return lib().orc_datap(self._w()[0], self.N, pp, self.D_dp, self.D_pp)

    def coarsen(self, perm, brute=False) -> np.ndarray:
        perm, pp = _i(perm)
        G = np.empty((self.D_pp, self.D_pp))
        lib().orc_coarsen(self._w()[1], self.N, pp, self.D_dp, self.D_pp, int(brute),
                          G.ctypes.data_as(POINTER(c_double)))
        return G

    def comm_cost(self, perm, brute=False) -> float:
        perm, pp = _i(perm)
        a, b = self._w()
        return lib().orc_comm_cost(a, b, self.N, self.D_dp, self.D_pp, pp, int(brute))

    def eval_population(self, perms) -> np.ndarray:
        perms, pp = _i(perms)
        P = perms.shape[0]
        cost = np.empty(P)
        a, b = self._w()
        lib().orc_eval_population(a, b, self.N, self.D_dp, self.D_pp, pp, P,
                                  cost.ctypes.data_as(POINTER(c_double)))
        return cost

    def get_assignment(self, perm):
        """(stage order [D_pp], pipelines sigma [D_dp, D_pp]) of one candidate, canonical choices."""
        perm, pp = _i(perm)
        order = np.empty(self.D_pp, dtype=np.int32)
        sigma = np.empty((self.D_dp, self.D_pp), dtype=np.int32)
        lib().orc_get_assignment(self._w()[1], self.N, self.D_dp, self.D_pp, pp,
                                 order.ctypes.data_as(POINTER(c_int)), sigma.ctypes.data_as(POINTER(c_int)))
        return order, sigma

    def gain4_propose(self, perm, r):
        perm, pp = _i(perm)
        a, b = c_int(), c_int()
        gains = np.empty(4)
        lib().orc_gain4_propose(self._w()[1], self.N, self.D_dp, self.D_pp, pp, r,
                                ctypes.byref(a), ctypes.byref(b), gains.ctypes.data_as(POINTER(c_double)))
        return a.value, b.value, gains

    def four_candidates(self, perm, r):
        """The four swaps [(a, b)] that round r's stage pair offers, in the paper's order."""
        perm, pp = _i(perm)
        a = np.empty(4, dtype=np.int32)
        b = np.empty(4, dtype=np.int32)
        lib().orc_four_candidates(self._w()[1], self.N, self.D_dp, self.D_pp, pp, r,
                                  a.ctypes.data_as(POINTER(c_int)), b.ctypes.data_as(POINTER(c_int)))
        return list(zip(a.tolist(), b.tolist()))

    def kl_propose(self, perm, r):
        """(position a, position b, gain_KL of all D_dp x D_dp swaps) for round r."""
        perm, pp = _i(perm)
        a, b = c_int(), c_int()
        gains = np.empty((self.D_dp, self.D_dp))
        lib().orc_kl_propose(self._w()[1], self.N, self.D_dp, self.D_pp, pp, r,
                             ctypes.byref(a), ctypes.byref(b), gains.ctypes.data_as(POINTER(c_double)))
        return a.value, b.value, gains

    def local_search(self, perms, rounds, neighbourhood):
        """Returns (perms_out, cost, applied[P x rounds])."""
        perms = np.array(perms, dtype=np.int32, order="C", copy=True)
        P = perms.shape[0]
        cost = np.empty(P)
        applied = np.empty((P, max(rounds, 0)), dtype=np.int64)
        a, b = self._w()
        lib().orc_local_search(a, b, self.N, self.D_dp, self.D_pp, perms.ctypes.data_as(POINTER(c_int)),
                               P, rounds, neighbourhood, cost.ctypes.data_as(POINTER(c_double)),
                               applied.ctypes.data_as(POINTER(c_long)))
        return perms, cost, applied

    def evolve(self, seed, generations, P, lam=None, m_x=None, m_m=1, ls_moves=8,
               neighbourhood=GAIN4, population=None):
        """Returns (population[P x N], cost[P], best_trace[generations])."""
        prm = GAParams(P, P if lam is None else lam, self.N // 4 if m_x is None else m_x, m_m,
                       ls_moves, neighbourhood, 0 if population is None else 1)
        pop = np.zeros((P, self.N), dtype=np.int32) if population is None else \
            np.array(population, dtype=np.int32, order="C", copy=True)
        cost = np.empty(P)
        trace = np.empty(generations)
        a, b = self._w()
        lib().orc_evolve(a, b, self.N, self.D_dp, self.D_pp, c_uint64(seed), generations,
                         ctypes.byref(prm), pop.ctypes.data_as(POINTER(c_int)),
                         cost.ctypes.data_as(POINTER(c_double)), trace.ctypes.data_as(POINTER(c_double)))
        return pop, cost, trace

    def evolve_by_generation(self, seed, generations, P, lam=None, m_x=None, m_m=1, ls_moves=8,
                             neighbourhood=GAIN4, threads=1, on_generation=None):
        """The run of `evolve` from a cold start, composed generation by generation from the oracle's own
        parts (init_candidate, eval_population, make_offspring, local_search, orc_replace) so that the
        evaluations, which are independent per candidate, can run on `threads` host threads and each
        generation can be reported: on_generation(g, population, cost) is called with g = -1 for the
        evaluated initial population and then after every replacement. Same results as evolve()."""
        from concurrent.futures import ThreadPoolExecutor
        lam = P if lam is None else lam
        m_x = self.N // 4 if m_x is None else m_x

        def split(rows):
            return [c for c in np.array_split(rows, max(1, min(len(rows), threads * 4))) if len(c)]

        with ThreadPoolExecutor(max(1, threads)) as ex:
            pop = np.stack([init_candidate(seed, k, self.N) for k in range(P)])
            cost = np.concatenate(list(ex.map(self.eval_population, split(pop))))
            if on_generation:
                on_generation(-1, pop, cost)
            trace = np.empty(generations)
            for g in range(generations):
                off = np.stack([make_offspring(seed, g, k, pop, self.D_dp, m_x, m_m)[0] for k in range(lam)])
                res = list(ex.map(lambda rows: self.local_search(rows, ls_moves, neighbourhood), split(off)))
                off = np.ascontiguousarray(np.concatenate([r[0] for r in res]), dtype=np.int32)
                off_cost = np.ascontiguousarray(np.concatenate([r[1] for r in res]))
                pop = np.ascontiguousarray(pop, dtype=np.int32)
                cost = np.ascontiguousarray(cost)
                lib().orc_replace(self.N, P, lam, pop.ctypes.data_as(POINTER(c_int)),
                                  cost.ctypes.data_as(POINTER(c_double)), off.ctypes.data_as(POINTER(c_int)),
                                  off_cost.ctypes.data_as(POINTER(c_double)))
                trace[g] = cost[0]
                if on_generation:
                    on_generation(g, pop, cost)
        return pop, cost, trace


def bottleneck_match(w, brute=False) -> float:
    w, pw = _d(w)
    n = w.shape[0]
    return lib().orc_bottleneck_match_brute(pw, n) if brute else lib().orc_bottleneck_match(pw, n)


def threshold_feasible(w, t) -> bool:
    w, pw = _d(w)
    return bool(lib().orc_threshold_feasible(pw, w.shape[0], float(t)))


def open_tsp(G, brute=False) -> float:
    G, pg = _d(G)
    n = G.shape[0]
    return lib().orc_open_tsp_brute(pg, n) if brute else lib().orc_open_tsp_held_karp(pg, n)


def hk_path(G) -> np.ndarray:
    G, pg = _d(G)
    order = np.empty(G.shape[0], dtype=np.int32)
    lib().orc_hk_path(pg, G.shape[0], order.ctypes.data_as(POINTER(c_int)))
    return order


def lexmin_matching(w, t):
    """Lexicographically smallest perfect matching within entries <= t, or None."""
    w, pw = _d(w)
    mate = np.empty(w.shape[0], dtype=np.int32)
    ok = lib().orc_lexmin_matching(pw, w.shape[0], float(t), mate.ctypes.data_as(POINTER(c_int)))
    return mate if ok else None


def datap_stage(W_dp, C) -> float:
    W_dp, pw = _d(W_dp)
    C, pc = _i(C)
    return lib().orc_datap_stage(pw, W_dp.shape[0], pc, len(C))


def philox4x32_10(ctr, key):
    c = (c_uint32 * 4)(*[int(x) for x in ctr])
    k = (c_uint32 * 2)(*[int(x) for x in key])
    o = (c_uint32 * 4)()
    lib().orc_philox4x32_10(c, k, o)
    return [int(x) for x in o]


def draw_randint(seed, stream, g, k, t, n) -> int:
    return int(lib().orc_draw_randint(c_uint64(seed), stream, g, k, t, n))


def init_candidate(seed, k, N) -> np.ndarray:
    out = np.empty(N, dtype=np.int32)
    lib().orc_init_candidate(c_uint64(seed), k, N, out.ctypes.data_as(POINTER(c_int)))
    return out


def make_offspring(seed, g, k, pop, D_dp, m_x, m_m):
    pop, pp = _i(pop)
    P, N = pop.shape
    child = np.empty(N, dtype=np.int32)
    par = np.empty(2, dtype=np.int32)
    lib().orc_make_offspring(c_uint64(seed), g, k, pp, P, N, D_dp, m_x, m_m,
                             child.ctypes.data_as(POINTER(c_int)), par.ctypes.data_as(POINTER(c_int)))
    return child, (int(par[0]), int(par[1]))
