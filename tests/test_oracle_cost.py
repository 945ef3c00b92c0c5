"""Pins for the cost-model part of the CPU oracle (Eqs. 1-4): closed forms, enumeration of the
definition on tiny instances, library cross-checks, invariances. No GPU."""
import itertools
import math

import numpy as np
import pytest
from scipy.sparse import csr_matrix
from scipy.sparse.csgraph import maximum_bipartite_matching

import oracle
import workloads
from tests import definition as dfn


def rel(a, b):
    return abs(a - b) / max(abs(a), abs(b), 1e-300)


# ---------------------------------------------------------------- weights (Sec. 2, Eqs. 2-3)
def test_weights_hand_computed():
    lat = np.array([[9.0, 0.010], [0.030, 9.0]])
    bw = np.array([[9.0, 1e9], [3e9, 9.0]])
    pr = oracle.Problem(lat, bw, c_dp=8e9, c_pp=1e9, D_dp=2, D_pp=1)
    # alpha = 0.02 s, beta = 2e9 B/s, shard = 4e9 B: 2*(0.02+2) and 2*(0.02+0.5)
    assert rel(pr.W_dp[0, 1], 4.04) < 1e-15 and rel(pr.W_pp[0, 1], 1.04) < 1e-15
    assert pr.W_dp[0, 1] == pr.W_dp[1, 0] and pr.W_pp[0, 1] == pr.W_pp[1, 0]
    assert pr.W_dp[0, 0] == 0.0 and pr.W_pp[1, 1] == 0.0


def test_weights_homogeneous_and_definition():
    lat, bw = workloads.network_homogeneous(8, bw_gbps=100.0, lat_ms=0.1)
    pr = oracle.Problem(lat, bw, 3.25e8, 8388608.0, 4, 2)
    off = ~np.eye(8, dtype=bool)
    assert np.all(pr.W_dp[off] == pr.W_dp[0, 1]) and np.all(pr.W_pp[off] == pr.W_pp[0, 1])
    assert rel(pr.W_dp[0, 1], 2 * (1e-4 + 3.25e8 / 4 / 12.5e9)) < 1e-14
    assert rel(pr.W_pp[0, 1], 2 * (1e-4 + 8388608.0 / 12.5e9)) < 1e-14
    lat, bw = workloads.network_iid(6, seed=3)
    lat = lat * np.random.default_rng(1).uniform(0.5, 1.5, size=lat.shape)  # make asymmetric
    pr = oracle.Problem(lat, bw, 7e7, 3e6, 3, 2)
    for d in range(6):
        for e in range(6):
            if d != e:
                assert pr.W_dp[d, e] == dfn.weights_entry(lat, bw, d, e, 7e7, 3)
                assert pr.W_pp[d, e] == dfn.weights_entry(lat, bw, d, e, 3e6, 1)
    assert np.array_equal(pr.W_dp, pr.W_dp.T) and np.array_equal(pr.W_pp, pr.W_pp.T)


def test_weights_asymmetric_two_site_average():
    lat, bw = workloads.network_two_site_asymmetric(2)
    pr = oracle.Problem(lat, bw, 4e8, 1e7, 2, 2)
    beta = (3.87 + 3.73) / 2 * 1e9 / 8
    assert rel(pr.W_pp[0, 2], 2 * (21.8e-3 + 1e7 / beta)) < 1e-14
    assert pr.W_pp[0, 2] == pr.W_pp[2, 0] == pr.W_pp[1, 3]
    assert rel(pr.W_dp[0, 1], 2 * (0.5e-3 + 2e8 / (10.40e9 / 8))) < 1e-14


# ---------------------------------------------------------------- DataP (Eq. 2)
def test_datap_pair_special_case_and_definition():
    w = workloads.config("C1")
    pr = oracle.Problem(w.latency, w.bandwidth, w.c_dp, w.c_pp, w.D_dp, w.D_pp)
    rng = np.random.default_rng(5)
    for _ in range(50):
        perm = rng.permutation(8).astype(np.int32)
        # D_dp = 2: each stage's cost is the weight of its single pair
        expect = max(pr.W_dp[perm[2 * j], perm[2 * j + 1]] for j in range(4))
        assert pr.datap(perm) == expect
    lat, bw = workloads.network_iid(12, seed=11)
    pr = oracle.Problem(lat, bw, 5e7, 2e6, 4, 3)
    for _ in range(50):
        perm = rng.permutation(12).astype(np.int32)
        assert pr.datap(perm) == dfn.datap_cost(pr.W_dp, dfn.groups_of(perm, 4))
        # independent of rounding order up to 1e-12: exact sums by fsum
        ex = max(max(math.fsum(pr.W_dp[d, e] for e in C if e != d) for d in C)
                 for C in dfn.groups_of(perm, 4))
        assert rel(pr.datap(perm), ex) < 1e-12


def test_datap_homogeneous_closed_form_and_degenerate():
    lat, bw = workloads.network_homogeneous(64)
    pr = oracle.Problem(lat, bw, 3.25e8, 8388608.0, 8, 8)
    perm = np.random.default_rng(0).permutation(64).astype(np.int32)
    closed = 2 * 7 * (1e-4 + 3.25e8 / (8 * 12.5e9))
    assert rel(pr.datap(perm), closed) < 1e-12
    lat, bw = workloads.network_iid(5, seed=2)
    pr = oracle.Problem(lat, bw, 1e6, 1e6, 1, 5)       # D_dp = 1: empty sum
    assert pr.datap(np.arange(5, dtype=np.int32)) == 0.0


# ---------------------------------------------------------------- bottleneck matching (Eq. 3)
def _py_brute_match(w):
    n = len(w)
    return min(max(w[i][pi[i]] for i in range(n)) for pi in itertools.permutations(range(n)))


@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 6])
def test_matching_against_enumeration(n):
    rng = np.random.default_rng(100 + n)
    for trial in range(40):
        w = rng.uniform(0.1, 5.0, size=(n, n))
        if trial % 3 == 0:
            w = np.round(w)          # many ties
        assert oracle.bottleneck_match(w) == _py_brute_match(w)
        assert oracle.bottleneck_match(w, brute=True) == _py_brute_match(w)


def test_matching_closed_forms_small():
    assert oracle.bottleneck_match(np.array([[3.5]])) == 3.5
    rng = np.random.default_rng(9)
    for _ in range(100):
        a, b, c, d = rng.uniform(0, 1, 4)
        assert oracle.bottleneck_match(np.array([[a, b], [c, d]])) == min(max(a, d), max(b, c))


@pytest.mark.parametrize("n", [7, 8])
def test_matching_fast_vs_c_enumeration(n):
    rng = np.random.default_rng(200 + n)
    for _ in range(10):
        w = rng.uniform(0.0, 1.0, size=(n, n))
        assert oracle.bottleneck_match(w) == oracle.bottleneck_match(w, brute=True)


@pytest.mark.parametrize("n", [8, 16, 64])
def test_matching_bounds_and_library_feasibility(n):
    rng = np.random.default_rng(300 + n)
    for trial in range(6):
        w = rng.uniform(0.0, 1.0, size=(n, n))
        if trial == 0:
            w = np.round(w * 8) / 8
        t = oracle.bottleneck_match(w)
        assert t in w                                                   # an entry of the block
        lower = max(w.min(axis=1).max(), w.min(axis=0).max())          # every row/col needs an edge
        upper = min(max(w[i, (i + s) % n] for i in range(n)) for s in range(n))  # some matchings
        assert lower <= t <= upper
        # independent library routine: a perfect matching exists at t, none strictly below t
        m = maximum_bipartite_matching(csr_matrix(w <= t), perm_type="column")
        assert np.all(m >= 0)
        m = maximum_bipartite_matching(csr_matrix(w < t), perm_type="column")
        assert np.any(m < 0)
        assert oracle.threshold_feasible(w, t) and not oracle.threshold_feasible(w, np.nextafter(t, -1))
        # monotone: raising one entry never lowers the optimum
        w2 = w.copy()
        w2[rng.integers(n), rng.integers(n)] += 1.0
        assert oracle.bottleneck_match(w2) >= t
        # transposing the block (swapping the two stages) keeps the value
        assert oracle.bottleneck_match(w.T.copy()) == t


# ---------------------------------------------------------------- open-loop TSP (Eq. 4)
def _sym(rng, n, lo=0.1, hi=3.0):
    g = rng.uniform(lo, hi, size=(n, n))
    g = np.triu(g, 1) + np.triu(g, 1).T
    return g


@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 6, 7])
def test_tsp_against_enumeration_bit_exact(n):
    rng = np.random.default_rng(400 + n)
    for _ in range(8):
        G = _sym(rng, n)
        ex = dfn.open_tsp(G.tolist())
        assert oracle.open_tsp(G) == ex
        assert oracle.open_tsp(G, brute=True) == ex


@pytest.mark.parametrize("n", [8, 9])
def test_tsp_held_karp_vs_c_enumeration(n):
    rng = np.random.default_rng(500 + n)
    G = _sym(rng, n)
    assert oracle.open_tsp(G) == oracle.open_tsp(G, brute=True)


def test_tsp_closed_forms():
    assert oracle.open_tsp(np.zeros((1, 1))) == 0.0
    assert oracle.open_tsp(np.array([[0, 2.5], [2.5, 0]])) == 2.5
    rng = np.random.default_rng(7)
    for _ in range(50):
        a, b, c = rng.uniform(0, 1, 3)   # edges 01, 02, 12: a 3-node path uses two of them
        G = np.array([[0, a, b], [a, 0, c], [b, c, 0]])
        assert oracle.open_tsp(G) == min(a + b, a + c, b + c)
    for n in (4, 8, 12, 16):
        G = np.full((n, n), 0.375)
        np.fill_diagonal(G, 0)
        assert oracle.open_tsp(G) == (n - 1) * 0.375      # dyadic weight: sums are exact
    for n in (5, 10, 16):
        x = rng.integers(0, 1 << 20, size=n).astype(float)  # points on a line, integer coords
        G = np.abs(x[:, None] - x[None, :])
        assert oracle.open_tsp(G) == x.max() - x.min()


def test_tsp_relabel_and_reversal_invariance():
    rng = np.random.default_rng(8)
    G = _sym(rng, 10)
    base = oracle.open_tsp(G)
    for _ in range(5):
        p = rng.permutation(10)
        assert oracle.open_tsp(G[np.ix_(p, p)].copy()) == base
    assert oracle.open_tsp(G[::-1, ::-1].copy()) == base


# ---------------------------------------------------------------- full cost (Eq. 1)
def _c1():
    w = workloads.config("C1")
    return w, oracle.Problem(w.latency, w.bandwidth, w.c_dp, w.c_pp, w.D_dp, w.D_pp)


def test_full_cost_every_partition_of_config1():
    w, pr = _c1()
    parts = list(dfn.all_partitions(range(8), 2))
    assert len(parts) == 105
    costs = {}
    for groups in parts:
        perm = np.array([d for C in groups for d in C], dtype=np.int32)
        ex = dfn.comm_cost(pr.W_dp.tolist(), pr.W_pp.tolist(), groups)
        assert pr.comm_cost(perm) == ex
        assert pr.comm_cost(perm, brute=True) == ex
        costs[frozenset(frozenset(C) for C in groups)] = ex
    gmin = min(costs.values())
    # ordered stages (2520) and all 8! permutations: cost depends on the partition only
    perms = np.array(list(itertools.permutations(range(8))), dtype=np.int32)
    assert perms.shape[0] == 40320
    c = pr.eval_population(perms)
    keys = [frozenset(frozenset(row[2 * j:2 * j + 2].tolist()) for j in range(4)) for row in perms]
    assert all(c[i] == costs[keys[i]] for i in range(0, 40320, 7))
    assert c.min() == gmin
    ordered = [i for i in range(40320) if all(perms[i, 2 * j] < perms[i, 2 * j + 1] for j in range(4))]
    assert len(ordered) == 2520 and c[ordered].min() == gmin


def test_full_cost_definition_other_shapes():
    rng = np.random.default_rng(21)
    for (D_dp, D_pp) in [(3, 3), (4, 2), (2, 5), (1, 6), (6, 1), (3, 4)]:
        N = D_dp * D_pp
        lat, bw = workloads.network_iid(N, seed=N)
        pr = oracle.Problem(lat, bw, 6e7, 5e6, D_dp, D_pp)
        for _ in range(6):
            perm = rng.permutation(N).astype(np.int32)
            ex = dfn.comm_cost(pr.W_dp.tolist(), pr.W_pp.tolist(), dfn.groups_of(perm, D_dp))
            assert pr.comm_cost(perm) == ex
            assert pr.comm_cost(perm, brute=True) == ex


def test_full_cost_homogeneous_closed_form_and_ties():
    w = workloads.config("C3h")
    pr = oracle.Problem(w.latency, w.bandwidth, w.c_dp, w.c_pp, w.D_dp, w.D_pp)
    perms = workloads.random_population(32, 64, seed=1)
    c = pr.eval_population(perms)
    alpha, beta = 0.1e-3, 100e9 / 8
    closed = 2 * 7 * (alpha + w.c_dp / (8 * beta)) + 7 * 2 * (alpha + w.c_pp / beta)
    assert np.all(c == c[0])                 # every allocation ties bit for bit
    assert rel(c[0], closed) < 1e-12


def test_full_cost_invariances():
    w = workloads.config("C2")
    pr = oracle.Problem(w.latency, w.bandwidth, w.c_dp, w.c_pp, w.D_dp, w.D_pp)
    rng = np.random.default_rng(3)
    for perm in workloads.random_population(6, 64, seed=2):
        base = pr.comm_cost(perm)
        stages = perm.reshape(8, 8)
        assert pr.comm_cost(stages[::-1].reshape(-1)) == base                   # reversed pipeline
        assert pr.comm_cost(stages[rng.permutation(8)].reshape(-1)) == base     # relabelled stages
        relab = np.stack([s[rng.permutation(8)] for s in stages]).reshape(-1)    # relabelled replicas
        assert rel(pr.comm_cost(relab), base) < 1e-12
        # the pipeline part is bit-invariant under replica relabelling (no rounding in Eq. 3)
        assert np.array_equal(pr.coarsen(relab), pr.coarsen(perm))


def test_paper_case5_table_network_ties():
    w = workloads.config("C2b")
    pr = oracle.Problem(w.latency, w.bandwidth, w.c_dp, w.c_pp, w.D_dp, w.D_pp)
    # one region per stage: every stage costs the intra-region value 2*7*(5ms + shard/2Gbps)
    perm = np.arange(64, dtype=np.int32)
    assert rel(pr.datap(perm), 14 * (5e-3 + w.c_dp / 8 / 0.25e9)) < 1e-12
    G = pr.coarsen(perm)
    # the stage-to-stage edge is then the region-to-region value, e.g. Oregon-Virginia 67 ms, 1.15 Gbps
    assert rel(G[0, 1], 2 * (67e-3 + w.c_pp / (1.15e9 / 8))) < 1e-12
    assert rel(G[5, 7], 2 * (12e-3 + w.c_pp / (1.09e9 / 8))) < 1e-12
    perms = workloads.random_population(16, 64, seed=4)
    for p in perms:
        assert pr.comm_cost(p) == dfn.datap_cost(pr.W_dp, dfn.groups_of(p, 8)) + oracle.open_tsp(pr.coarsen(p, brute=True), brute=True)
