"""Pins for the oracle's assignment extraction (stage order + pipelines behind a candidate's cost).

The paper fixes what an assignment is (Sec. 2: pipelines P_i = {sigma_{i,j}}; Sec. 3.3: matched
devices handle the same micro-batch, the stage groups are ordered by the open-loop tour) but not
which optimum to take. The tie-breaking rules are this build's; these tests pin that the oracle
implements exactly those rules, by enumeration on tiny cases, closed forms and re-derivation of the
cost from the output.
"""
import itertools

import numpy as np
import pytest

import oracle
import workloads


def _problem(w):
    return oracle.Problem(w.latency, w.bandwidth, w.c_dp, w.c_pp, w.D_dp, w.D_pp)


def _custom(N, D_dp, D_pp, seed):
    lat, bw = workloads.network_iid(N, seed=seed)
    return workloads.Workload("custom", N, D_dp, D_pp, 25e6, 4e6, lat, bw, 0)


# ---------------------------------------------------------------- lexicographically smallest matching
def _lexmin_brute(w, t):
    n = w.shape[0]
    for m in itertools.permutations(range(n)):          # permutations come in lexicographic order
        if all(w[r, m[r]] <= t for r in range(n)):
            return list(m)
    return None


@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 6])
def test_lexmin_matching_against_enumeration(n):
    rng = np.random.default_rng(n)
    for trial in range(40):
        w = rng.integers(0, 6, size=(n, n)).astype(np.float64)      # many ties
        for t in (oracle.bottleneck_match(w), float(rng.integers(0, 6))):
            got = oracle.lexmin_matching(w, t)
            want = _lexmin_brute(w, t)
            if want is None:
                assert got is None
            else:
                assert list(got) == want


def test_lexmin_matching_special_cases():
    # everything allowed: the identity; a permutation matrix of zeros: that permutation
    assert list(oracle.lexmin_matching(np.zeros((5, 5)), 0.0)) == [0, 1, 2, 3, 4]
    p = [3, 0, 4, 1, 2]
    w = np.ones((5, 5))
    for r, c in enumerate(p):
        w[r, c] = 0.0
    assert list(oracle.lexmin_matching(w, 0.0)) == p
    assert oracle.lexmin_matching(w, -1.0) is None
    # row 0 would like column 0, but then row 1 (which only has column 0) is stranded
    w = np.array([[0.0, 0.0], [0.0, 9.0]])
    assert list(oracle.lexmin_matching(w, 0.0)) == [1, 0]


# ---------------------------------------------------------------- canonical tour
def _table_by_enumeration(G):
    """best[(S, v)] = min over all orders of S ending in v of the left-to-right rounded sum."""
    n = G.shape[0]
    best = {}
    for k in range(1, n + 1):
        for S in itertools.combinations(range(n), k):
            for order in itertools.permutations(S):
                c = 0.0
                for a, b in zip(order, order[1:]):
                    c = c + G[a, b]
                key = (frozenset(S), order[-1])
                if key not in best or c < best[key]:
                    best[key] = c
    return best


def _canonical_path(G):
    n = G.shape[0]
    best = _table_by_enumeration(G)
    S = frozenset(range(n))
    v = min(range(n), key=lambda x: (best[(S, x)], x))
    rev = [v]
    while len(S) > 1:
        rest = S - {v}
        u = min(x for x in rest if best[(rest, x)] + G[x, v] == best[(S, v)])
        S, v = rest, u
        rev.append(v)
    return rev[::-1]


@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 6])
def test_hk_path_against_enumeration(n):
    rng = np.random.default_rng(100 + n)
    for trial in range(12):
        if trial % 2:
            A = rng.integers(1, 4, size=(n, n)).astype(np.float64)  # many equal tours
        else:
            A = rng.random((n, n))
        G = np.triu(A, 1) + np.triu(A, 1).T
        order = list(oracle.hk_path(G))
        assert order == _canonical_path(G)
        c = 0.0
        for a, b in zip(order, order[1:]):
            c = c + G[a, b]
        assert c == oracle.open_tsp(G)                  # same bits as the cost path's Held-Karp


def test_hk_path_end_node_is_lowest_among_all_optimal_tours():
    rng = np.random.default_rng(5)
    for trial in range(10):
        n = 6
        A = rng.integers(1, 3, size=(n, n)).astype(np.float64)
        G = np.triu(A, 1) + np.triu(A, 1).T
        opt = oracle.open_tsp(G, brute=True)
        ends = set()
        for order in itertools.permutations(range(n)):
            c = 0.0
            for a, b in zip(order, order[1:]):
                c = c + G[a, b]
            if c == opt:
                ends.add(order[-1])
        assert oracle.hk_path(G)[-1] == min(ends)


# ---------------------------------------------------------------- whole assignment
def _check_assignment(o, perm):
    N, D_dp, D_pp = o.N, o.D_dp, o.D_pp
    order, sigma = o.get_assignment(perm)
    assert sorted(order) == list(range(D_pp))
    stages = [set(perm[j * D_dp:(j + 1) * D_dp]) for j in range(D_pp)]
    for k in range(D_pp):                                   # position k holds stage order[k], each device once
        assert set(sigma[:, k]) == stages[order[k]]
    for i in range(D_dp):                                   # pipeline i starts at slot i of the first stage
        assert sigma[i, 0] == perm[order[0] * D_dp + i]
    G = o.coarsen(perm)
    pp = 0.0
    for k in range(D_pp - 1):
        hop = max(o.W_pp[sigma[i, k], sigma[i, k + 1]] for i in range(D_dp))
        assert hop == G[order[k], order[k + 1]]             # every chained matching attains Eq. 3's optimum
        pp = pp + hop
    assert o.datap(perm) + pp == o.comm_cost(perm)          # Eq. 1 re-derived from the output, same bits
    return order, sigma


@pytest.mark.parametrize("name", ["C1", "C2", "C2b"])
def test_assignment_reproduces_the_cost(name):
    w = workloads.config(name)
    o = _problem(w)
    for perm in workloads.random_population(12 if name != "C1" else 64, w.N, seed=3):
        _check_assignment(o, perm)


@pytest.mark.parametrize("D_dp,D_pp", [(1, 1), (1, 5), (5, 1), (2, 2), (3, 4), (4, 3), (6, 2)])
def test_assignment_small_shapes_against_enumeration(D_dp, D_pp):
    N = D_dp * D_pp
    o = _problem(_custom(N, D_dp, D_pp, seed=N))
    for perm in workloads.random_population(6, N, seed=1):
        order, sigma = _check_assignment(o, perm)
        G = o.coarsen(perm)
        assert list(order) == _canonical_path(G)
        slot = list(range(D_dp))
        for k in range(D_pp - 1):
            A, B = order[k], order[k + 1]
            blk = o.W_pp[np.ix_(perm[A * D_dp:(A + 1) * D_dp], perm[B * D_dp:(B + 1) * D_dp])]
            m = _lexmin_brute(blk, G[A, B])
            slot = [m[s] for s in slot]
            assert [perm[B * D_dp + s] for s in slot] == list(sigma[:, k + 1])


def test_assignment_homogeneous_closed_form():
    # all tours and all matchings tie: back-tracking picks 0 as the end, then 1, 2, ...: the order is
    # D_pp-1 .. 0; every matching is the identity, so pipeline i keeps slot i
    lat, bw = workloads.network_homogeneous(12)
    o = oracle.Problem(lat, bw, 1e6, 1e6, 3, 4)
    perm = workloads.random_population(1, 12, seed=2)[0]
    order, sigma = o.get_assignment(perm)
    assert list(order) == [3, 2, 1, 0]
    for i in range(3):
        assert list(sigma[i]) == [perm[j * 3 + i] for j in (3, 2, 1, 0)]


def test_assignment_config5_shape():
    w = workloads.config("C5")
    o = _problem(w)
    _check_assignment(o, workloads.random_population(1, w.N, seed=9)[0])
