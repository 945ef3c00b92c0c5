"""Pins for the search part of the CPU oracle (Sec. 3.4): local search neighbourhoods, Philox
draws, evolutionary loop. No GPU."""
import itertools
import os

import numpy as np
import pytest

import oracle
import workloads
from tests import definition as dfn

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _problem(name):
    w = workloads.config(name)
    return w, oracle.Problem(w.latency, w.bandwidth, w.c_dp, w.c_pp, w.D_dp, w.D_pp)


def _pair_index(N, a, b):
    return [(x, y) for x in range(N) for y in range(x + 1, N)].index((a, b))


# ---------------------------------------------------------------- ALL_PAIRS
def test_all_pairs_round_matches_independent_enumeration_config1():
    w, pr = _problem("C1")
    Wd, Wp = pr.W_dp.tolist(), pr.W_pp.tolist()
    moves = [(a, b) for a in range(8) for b in range(a + 1, 8)]
    assert len(moves) == 28
    perms = workloads.random_population(24, 8, seed=1)
    out, cost, applied = pr.local_search(perms, 1, oracle.ALL_PAIRS)
    for p in range(24):
        cur = dfn.comm_cost(Wd, Wp, dfn.groups_of(perms[p], 2))
        best, bi = None, -1
        for i, (a, b) in enumerate(moves):
            q = perms[p].copy()
            q[a], q[b] = q[b], q[a]
            c = dfn.comm_cost(Wd, Wp, dfn.groups_of(q, 2))
            if best is None or c < best:
                best, bi = c, i
        if best < cur:
            a, b = moves[bi]
            q = perms[p].copy()
            q[a], q[b] = q[b], q[a]
            assert applied[p, 0] == bi and np.array_equal(out[p], q) and cost[p] == best
        else:
            assert applied[p, 0] == -1 and np.array_equal(out[p], perms[p]) and cost[p] == cur


def test_all_pairs_monotone_fixed_point_and_global_optimum_config1():
    w, pr = _problem("C1")
    perms = workloads.random_population(64, 8, seed=1)
    c0 = pr.eval_population(perms)
    prev_perm, prev_cost = perms, c0
    gmin = pr.eval_population(np.array(list(itertools.permutations(range(8))), dtype=np.int32)).min()
    for rounds in range(1, 7):
        out, cost, applied = pr.local_search(perms, rounds, oracle.ALL_PAIRS)
        assert np.all(np.sort(out, axis=1) == np.arange(8))
        assert np.array_equal(cost, pr.eval_population(out))
        moved = applied[:, rounds - 1] >= 0
        assert np.all(cost[moved] < prev_cost[moved]) and np.all(cost[~moved] == prev_cost[~moved])
        assert np.all(cost >= gmin)
        # rounds are a prefix-consistent iteration: r rounds == r-1 rounds then one more
        nxt, c2, _ = pr.local_search(prev_perm, 1, oracle.ALL_PAIRS)
        assert np.array_equal(nxt, out) and np.array_equal(c2, cost)
        prev_perm, prev_cost = out, cost
    # once no move applies, nothing changes any more
    out2, cost2, applied2 = pr.local_search(prev_perm, 3, oracle.ALL_PAIRS)
    still = applied[:, -1] < 0
    assert np.all(applied2[still] == -1) and np.array_equal(out2[still], prev_perm[still])


def test_all_pairs_homogeneous_never_moves():
    lat, bw = workloads.network_homogeneous(12)
    pr = oracle.Problem(lat, bw, 3.25e8, 8388608.0, 3, 4)
    perms = workloads.random_population(5, 12, seed=3)
    out, cost, applied = pr.local_search(perms, 3, oracle.ALL_PAIRS)
    assert np.array_equal(out, perms) and np.all(applied == -1) and np.all(cost == cost[0])


def test_all_pairs_tie_takes_lowest_index():
    # two-site network without jitter: many moves tie exactly; the applied index must be the
    # first among the minimisers
    lat, bw = workloads.network_paper_table("paper_case4_network.txt", 3)
    pr = oracle.Problem(lat, bw, 1e8, 4e6, 3, 4)
    perms = workloads.random_population(10, 12, seed=8)
    out, cost, applied = pr.local_search(perms, 1, oracle.ALL_PAIRS)
    moves = [(a, b) for a in range(12) for b in range(a + 1, 12)]
    for p in range(10):
        cs = []
        for (a, b) in moves:
            q = perms[p].copy()
            q[a], q[b] = q[b], q[a]
            cs.append(pr.comm_cost(q))
        cur = pr.comm_cost(perms[p])
        if min(cs) < cur:
            assert applied[p, 0] == int(np.argmin(cs))     # numpy argmin: first minimiser
        else:
            assert applied[p, 0] == -1


# ---------------------------------------------------------------- GAIN4
def test_gain4_proposal_hand_computation():
    lat, bw = workloads.network_iid(12, seed=4)
    pr = oracle.Problem(lat, bw, 9e7, 6e6, 4, 3)
    W = pr.W_pp
    rng = np.random.default_rng(0)
    pairs = [(0, 1), (0, 2), (1, 2)]
    for r in range(7):
        perm = rng.permutation(12).astype(np.int32)
        j, jp = pairs[r % 3]
        Cj, Cjp = perm[4 * j:4 * j + 4], perm[4 * jp:4 * jp + 4]

        def fastest(C):
            best = None
            for i in range(4):
                for k in range(i + 1, 4):
                    if best is None or W[C[i], C[k]] < best[0]:
                        best = (W[C[i], C[k]], i, k)
            return best[1], best[2]
        s, sp = fastest(Cj), fastest(Cjp)
        gains = []
        for xi in range(2):
            for yi in range(2):
                x, mx = Cj[s[xi]], Cj[s[1 - xi]]
                y, my = Cjp[sp[yi]], Cjp[sp[1 - yi]]
                g = sum(W[x, d] for d in Cjp) / 4 - W[x, mx] + sum(W[y, d] for d in Cj) / 4 - W[y, my]
                gains.append(g)
        a, b, og = pr.gain4_propose(perm, r)
        assert np.allclose(og, gains, rtol=1e-13, atol=0)
        k = int(np.argmax(gains))
        assert (a, b) == (4 * j + s[k // 2], 4 * jp + sp[k % 2])


def test_gain4_local_search_invariants():
    w, pr = _problem("C2")
    perms = workloads.random_population(12, 64, seed=5)
    c0 = pr.eval_population(perms)
    out, cost, applied = pr.local_search(perms, 40, oracle.GAIN4)
    assert np.all(np.sort(out, axis=1) == np.arange(64))
    assert np.array_equal(cost, pr.eval_population(out))
    assert np.all(cost <= c0) and np.any(cost < c0)
    # replay the applied swaps: they reproduce the output, each strictly improving
    moves = [(a, b) for a in range(64) for b in range(a + 1, 64)]
    for p in range(12):
        q, c = perms[p].copy(), c0[p]
        for r in range(40):
            a, b, _ = pr.gain4_propose(q, r)
            if applied[p, r] >= 0:
                assert moves[applied[p, r]] == (a, b)
                q[a], q[b] = q[b], q[a]
                c2 = pr.comm_cost(q)
                assert c2 < c
                c = c2
            else:
                q2 = q.copy()
                q2[a], q2[b] = q2[b], q2[a]
                assert pr.comm_cost(q2) >= c
        assert np.array_equal(q, out[p]) and c == cost[p]


# ---------------------------------------------------------------- KL (the paper's comparison strategy)
def test_kl_gain_is_the_drop_in_cut_weight():
    # textbook meaning of the Kernighan-Lin gain: swapping x in A with y in B lowers the weight of the
    # cut between A and B by exactly gain(x, y). Checked against cuts summed independently.
    lat, bw = workloads.network_iid(15, seed=8)
    pr = oracle.Problem(lat, bw, 9e7, 6e6, 5, 3)
    W = pr.W_pp
    rng = np.random.default_rng(1)
    pairs = [(0, 1), (0, 2), (1, 2)]

    def cut(A, B):
        return sum(W[a, b] for a in A for b in B)
    for r in range(9):
        perm = rng.permutation(15).astype(np.int32)
        j, jp = pairs[r % 3]
        A, B = list(perm[5 * j:5 * j + 5]), list(perm[5 * jp:5 * jp + 5])
        a, b, gains = pr.kl_propose(perm, r)
        want = np.empty((5, 5))
        for sx in range(5):
            for sy in range(5):
                A2, B2 = A.copy(), B.copy()
                A2[sx], B2[sy] = B[sy], A[sx]
                want[sx, sy] = cut(A, B) - cut(A2, B2)
        assert np.allclose(gains, want, rtol=0, atol=1e-12 * cut(A, B))
        sx, sy = divmod(int(np.argmax(gains)), 5)          # first maximiser in (slot, slot') order
        assert (a, b) == (5 * j + sx, 5 * jp + sy)


def test_kl_gain_hand_values_on_a_tiny_case():
    # 4 devices, two stages of two; weights chosen by hand (W = 2 * latency when sizes are zero)
    lat = np.array([[0, 1, 4, 6], [1, 0, 3, 5], [4, 3, 0, 2], [6, 5, 2, 0]], dtype=np.float64) / 2
    pr = oracle.Problem(lat, np.ones((4, 4)), 0.0, 0.0, 2, 2)
    assert np.array_equal(pr.W_pp, 2 * lat)
    _, _, g = pr.kl_propose(np.arange(4, dtype=np.int32), 0)
    # x=0,y=2: (4+6) - 1 + (4+3) - 2 - 2*4 = 6;  x=0,y=3: 10 - 1 + 11 - 2 - 12 = 6
    # x=1,y=2: (3+5) - 1 + 7 - 2 - 6 = 6;         x=1,y=3: 8 - 1 + 11 - 2 - 10 = 6
    assert np.array_equal(g, np.full((2, 2), 6.0))
    lat[0, 2] = lat[2, 0] = 0.5                       # w[0][2] = 1
    pr = oracle.Problem(lat, np.ones((4, 4)), 0.0, 0.0, 2, 2)
    a, b, g = pr.kl_propose(np.arange(4, dtype=np.int32), 0)
    # x=0,y=2: (1+6) - 1 + (1+3) - 2 - 2 = 6; x=0,y=3: 7 - 1 + 11 - 2 - 12 = 3; x=1,y=2: 8 - 1 + 4 - 2 - 6 = 3
    assert np.array_equal(g, [[6.0, 3.0], [3.0, 6.0]]) and (a, b) == (0, 2)


def test_kl_local_search_invariants():
    w, pr = _problem("C2")
    perms = workloads.random_population(8, 64, seed=6)
    c0 = pr.eval_population(perms)
    out, cost, applied = pr.local_search(perms, 30, oracle.KL)
    assert np.all(np.sort(out, axis=1) == np.arange(64))
    assert np.array_equal(cost, pr.eval_population(out))
    assert np.all(cost <= c0)
    moves = [(a, b) for a in range(64) for b in range(a + 1, 64)]
    for p in range(8):
        q, c = perms[p].copy(), c0[p]
        for r in range(30):
            a, b, _ = pr.kl_propose(q, r)
            q2 = q.copy()
            q2[a], q2[b] = q2[b], q2[a]
            c2 = pr.comm_cost(q2)
            if applied[p, r] >= 0:
                assert moves[applied[p, r]] == (a, b) and c2 < c
                q, c = q2, c2
            else:
                assert c2 >= c
        assert np.array_equal(q, out[p]) and c == cost[p]


# ---------------------------------------------------------------- Philox
def test_philox_known_answers():
    n = 0
    with open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            v = [int(t, 16) for t in line.split()]
            assert oracle.philox4x32_10(v[0:4], v[4:6]) == v[6:10]
            n += 1
    assert n == 3


def test_randint_range_and_uniformity():
    xs = np.array([oracle.draw_randint(7, 2, 3, 5, t, 10) for t in range(4000)])
    assert xs.min() == 0 and xs.max() == 9
    counts = np.bincount(xs, minlength=10)
    assert counts.min() > 300 and counts.max() < 500
    # draws are a pure function of (seed, stream, generation, candidate, index)
    assert oracle.draw_randint(7, 2, 3, 5, 17, 1000) == oracle.draw_randint(7, 2, 3, 5, 17, 1000)
    assert len({oracle.draw_randint(7, s, 3, 5, 17, 1 << 30) for s in range(4)}) == 4


def test_init_candidates_are_uniformish_permutations():
    first = np.zeros(6, dtype=int)
    for k in range(3000):
        p = oracle.init_candidate(11, k, 6)
        assert sorted(p.tolist()) == list(range(6))
        first[p[0]] += 1
    assert first.min() > 400 and first.max() < 600


# ---------------------------------------------------------------- offspring + evolve
def test_offspring_is_balanced_mix_of_parents():
    pop = workloads.random_population(16, 24, seed=6)
    for k in range(20):
        child, (p1, p2) = oracle.make_offspring(3, 0, k, pop, 4, 6, 0)
        assert sorted(child.tolist()) == list(range(24))
        assert 0 <= p1 < 16 and 0 <= p2 < 16
        # without mutation every device sits in the stage it has in parent 1 or in parent 2,
        # or was displaced from a slot that a parent-2 device took over
        st = lambda perm: {int(d): q // 4 for q, d in enumerate(perm)}
        s1, s2, sc = st(pop[p1]), st(pop[p2]), st(child)
        moved_to_p2 = [d for d in range(24) if sc[d] != s1[d] and sc[d] == s2[d]]
        displaced = [d for d in range(24) if sc[d] != s1[d] and sc[d] != s2[d]]
        assert len(displaced) <= len(moved_to_p2) + 6
    # no crossover draws, no mutation: the child is parent 1
    child, (p1, _) = oracle.make_offspring(3, 0, 0, pop, 4, 0, 0)
    assert np.array_equal(child, pop[p1])
    # one mutation: exactly one transposition away (or identical when a == b)
    child2, _ = oracle.make_offspring(3, 0, 0, pop, 4, 0, 1)
    assert (child2 != child).sum() in (0, 2)


def test_evolve_invariants_config1():
    w, pr = _problem("C1")
    gmin = pr.eval_population(np.array(list(itertools.permutations(range(8))), dtype=np.int32)).min()
    pop, cost, trace = pr.evolve(seed=0, generations=12, P=16, ls_moves=2, neighbourhood=oracle.GAIN4)
    assert np.all(np.sort(pop, axis=1) == np.arange(8))
    assert np.array_equal(cost, pr.eval_population(pop))
    assert np.all(np.diff(cost) >= 0) and trace[-1] == cost[0]
    assert np.all(np.diff(trace) <= 0) and trace[-1] >= gmin
    pop2, cost2, trace2 = pr.evolve(seed=0, generations=12, P=16, ls_moves=2, neighbourhood=oracle.GAIN4)
    assert np.array_equal(pop, pop2) and np.array_equal(cost, cost2) and np.array_equal(trace, trace2)
    pop3, _, trace3 = pr.evolve(seed=1, generations=12, P=16, ls_moves=2, neighbourhood=oracle.GAIN4)
    assert not np.array_equal(pop, pop3)
    # with the exhaustive neighbourhood the tiny instance reaches the enumerated optimum
    _, cost4, trace4 = pr.evolve(seed=2, generations=6, P=16, ls_moves=3, neighbourhood=oracle.ALL_PAIRS)
    assert trace4[-1] == gmin


def test_evolve_generation_is_select_cross_mutate_search_replace():
    w, pr = _problem("C1")
    P, seed = 10, 5
    pop0, cost0, _ = pr.evolve(seed=seed, generations=0, P=P)
    assert np.array_equal(pop0, np.stack([oracle.init_candidate(seed, k, 8) for k in range(P)]))
    pop1, cost1, trace1 = pr.evolve(seed=seed, generations=1, P=P, m_x=2, m_m=1, ls_moves=3)
    off = np.stack([oracle.make_offspring(seed, 0, k, pop0, 2, 2, 1)[0] for k in range(P)])
    off, off_cost, _ = pr.local_search(off, 3, oracle.GAIN4)
    allp = np.concatenate([pop0, off])
    allc = np.concatenate([cost0, off_cost])
    order = np.lexsort((np.arange(2 * P), allc))[:P]       # by cost, then origin index
    assert np.array_equal(pop1, allp[order]) and np.array_equal(cost1, allc[order])
    assert trace1[0] == allc[order][0]
    # warm start continues the same trajectory: generation index is part of the counter, so a
    # one-generation run from pop0 equals generation 0 of the cold run
    pop1w, cost1w, _ = pr.evolve(seed=seed, generations=1, P=P, m_x=2, m_m=1, ls_moves=3, population=pop0)
    assert np.array_equal(pop1w, pop1) and np.array_equal(cost1w, cost1)


def test_evolve_steady_state_is_insert_and_drop_worst():
    # lambda = 1 is the paper's loop (Sec. 3.4): two random parents -> offspring -> local search ->
    # "add o*, remove the worst if o* is better". Re-composed here from the oracle's parts with the
    # replacement written as that sentence, generation by generation.
    w, pr = _problem("C1")
    P, seed, G = 7, 11, 25
    kw = dict(lam=1, m_x=2, m_m=1, ls_moves=2, neighbourhood=oracle.GAIN4)
    pop, cost, _ = pr.evolve(seed=seed, generations=0, P=P, **kw)
    inserted = 0
    for g in range(G):
        child = oracle.make_offspring(seed, g, 0, pop, 2, 2, 1)[0]
        child, ccost, _ = pr.local_search(child[None, :], 2, oracle.GAIN4)
        # incumbents in (cost, position) order; the worst is the last of them
        order = np.lexsort((np.arange(P), cost))
        pop, cost = pop[order], cost[order]
        if ccost[0] < cost[-1]:
            at = int(np.searchsorted(cost, ccost[0], side="right"))     # behind incumbents of equal cost
            pop = np.concatenate([pop[:at], child, pop[at:-1]])
            cost = np.concatenate([cost[:at], ccost, cost[at:-1]])
            inserted += 1
        want_pop, want_cost, trace = pr.evolve(seed=seed, generations=g + 1, P=P, **kw)
        assert np.array_equal(pop, want_pop) and np.array_equal(cost, want_cost)
        assert trace[-1] == cost[0]
    assert 0 < inserted < G      # both branches of the rule were exercised


def test_evolve_by_generation_equals_evolve():
    # the generation-wise, threaded composition used to write the stored configuration-5 trajectory gives
    # the bits of the oracle's sequential loop
    for name, P, lam, kw in (("C1", 10, None, {}), ("C2", 12, 5, dict(m_x=40, m_m=2, ls_moves=3)),
                             ("C1", 6, 1, dict(ls_moves=2)), ("C1", 4, 9, dict(neighbourhood=oracle.KL))):
        w, pr = _problem(name)
        want = pr.evolve(5, 4, P, lam=lam, **kw)
        seen = []
        got = pr.evolve_by_generation(5, 4, P, lam=lam, threads=3, on_generation=lambda g, p, c: seen.append((g, c.min())), **kw)
        assert all(np.array_equal(a, b) for a, b in zip(want, got))
        assert [g for g, _ in seen] == [-1, 0, 1, 2, 3] and [c for _, c in seen[1:]] == want[2].tolist()
