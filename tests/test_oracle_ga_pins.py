"""Pins for the evolutionary half of the CPU oracle (Sec. 3.4 "Hybrid Genetic Algorithm"): the draw
layout, the initial shuffle, selection / crossover / mutation, the round schedule and acceptance
rule of the local search inside the loop, and the replacement. The oracle is compared with
tests/definition_search.py (pure Python, written from the prose of the reading) on whole populations,
with a hand-worked case whose draws are printed below, and each comparison is shown to fail when a
plausible mistake is planted in the definition. No GPU."""
import os

import numpy as np
import pytest

import oracle
from tests import definition as dfn
from tests import definition_search as ds

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _network(N, seed):
    rng = np.random.default_rng(seed)
    lat = rng.uniform(1e-3, 0.1, (N, N))
    bw = 10.0 ** rng.uniform(8, 10, (N, N))
    lat, bw = (lat + lat.T) / 2, (bw + bw.T) / 2
    return lat, bw


# ---------------------------------------------------------------- the generator under the definition
def test_definition_philox_known_answers():
    n = 0
    with open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            v = [int(t, 16) for t in line.split()]
            assert ds.philox4x32_10(v[0:4], v[4:6]) == v[6:10]
            n += 1
    assert n == 3


def test_draw_layout_matches_oracle():
    # every word of the counter and of the key takes part, with values that tell them apart
    for seed in (0, 7, 0x123456789ABCDEF0, 2**64 - 1):
        for stream in range(4):
            for g in (0, 1, 99):
                for k in (0, 2, 4095):
                    for t in (0, 1, 3, 4, 5, 130):
                        for n in (2, 1000, 2**31):
                            want = ds.randint(ds.draw_word(seed, stream, g, k, t), n)
                            assert oracle.draw_randint(seed, stream, g, k, t, n) == want


@pytest.mark.parametrize("fault", ["counter_words_swapped", "stream_and_generation_swapped", "key_words_swapped"])
def test_draw_layout_comparison_catches_planted_mistakes(fault):
    bad = 0
    for seed in (7, 0x123456789ABCDEF0):
        for stream in range(4):
            for g in (0, 1, 99):
                for k in (0, 2, 4095):
                    for t in (0, 5):
                        got = oracle.draw_randint(seed, stream, g, k, t, 2**31)
                        bad += got != ds.randint(ds.draw_word(seed, stream, g, k, t, fault), 2**31)
    assert bad > 50


# ---------------------------------------------------------------- hand-worked case, N = 4, D_dp = 2
def test_hand_worked_shuffle_and_offspring_n4():
    seed = 2022
    # initial candidate 1: the three words of block (0, 1, 0, 0) that the shuffle uses
    words = [ds.draw_word(seed, ds.STREAM_INIT, 0, 1, t) for t in range(3)]
    assert words == [0xD126F35B, 0x22E1B473, 0xC943778F]
    # (word * n) >> 32 with n = 4, 3, 2: 0xd126f35b / 2^32 = 0.817 -> 3; 0x22e1b473 / 2^32 = 0.136 -> 0;
    # 0xc943778f / 2^32 = 0.786 -> 1
    assert [ds.randint(words[0], 4), ds.randint(words[1], 3), ds.randint(words[2], 2)] == [3, 0, 1]
    # identity 0 1 2 3; i=3 <-> 3: unchanged; i=2 <-> 0: 2 1 0 3; i=1 <-> 1: unchanged
    assert oracle.init_candidate(seed, 1, 4).tolist() == [2, 1, 0, 3]
    # candidate 2: draws 1, 1, 0: i=3 <-> 1: 0 3 2 1; i=2 <-> 1: 0 2 3 1; i=1 <-> 0: 2 0 3 1
    assert [oracle.draw_randint(seed, 0, 0, 2, t, n) for t, n in ((0, 4), (1, 3), (2, 2))] == [1, 1, 0]
    assert oracle.init_candidate(seed, 2, 4).tolist() == [2, 0, 3, 1]
    # candidate 0: draws 0, 2, 0: i=3 <-> 0: 3 1 2 0; i=2 <-> 2: unchanged; i=1 <-> 0: 1 3 2 0
    assert oracle.init_candidate(seed, 0, 4).tolist() == [1, 3, 2, 0]

    pop = np.array([[1, 3, 2, 0], [2, 1, 0, 3], [2, 0, 3, 1]], dtype=np.int32)
    # offspring 1 of generation 1, three crossover steps, one mutation:
    #   selection words 0x9cd8cc19, 0xeb974854 -> parents 1 and 2 (x3 >> 32)
    sel = [ds.draw_word(seed, ds.STREAM_SELECT, 1, 1, t) for t in range(2)]
    assert sel == [0x9CD8CC19, 0xEB974854] and [ds.randint(w, 3) for w in sel] == [1, 2]
    #   child = parent 1 = 2 1 | 0 3, parent 2 = 2 0 | 3 1 (stages of two)
    #   crossover draws (device, slot) = (2, 0), (0, 1), (1, 1)
    cx = [ds.draw_word(seed, ds.STREAM_CROSSOVER, 1, 1, t) for t in range(6)]
    assert [ds.randint(w, 4 if t % 2 == 0 else 2) for t, w in enumerate(cx)] == [2, 0, 0, 1, 1, 1]
    #   (2, 0): device 2 is in stage 0 in both: nothing
    #   (0, 1): device 0 is in stage 1 of the child, stage 0 of parent 2: it changes places with the
    #           device at slot 1 of stage 0 (device 1): 2 0 | 1 3
    #   (1, 1): device 1 is now in stage 1, as in parent 2: nothing
    #   mutation positions 3 and 1: 2 3 | 1 0
    mu = [ds.draw_word(seed, ds.STREAM_MUTATION, 1, 1, t) for t in range(2)]
    assert [ds.randint(w, 4) for w in mu] == [3, 1]
    child, parents = oracle.make_offspring(seed, 1, 1, pop, 2, 3, 1)
    assert parents == (1, 2) and child.tolist() == [2, 3, 1, 0]
    # without the mutation, and with only the first two crossover steps
    assert oracle.make_offspring(seed, 1, 1, pop, 2, 3, 0)[0].tolist() == [2, 0, 1, 3]
    assert oracle.make_offspring(seed, 1, 1, pop, 2, 1, 0)[0].tolist() == [2, 1, 0, 3]


# ---------------------------------------------------------------- whole populations against the definition
SHAPES = [(8, 2), (12, 3), (12, 2), (24, 4), (24, 6)]


def test_init_population_matches_definition():
    for N, _ in SHAPES:
        for seed in (0, 1, 2, 2**40 + 5):
            for k in list(range(40)) + [4095, 70000]:
                assert oracle.init_candidate(seed, k, N).tolist() == ds.init_candidate(seed, k, N)


@pytest.mark.parametrize("fault", ["shuffle_draw_index_is_i", "shuffle_range_excludes_i", "counter_words_swapped"])
def test_init_comparison_catches_planted_mistakes(fault):
    bad = sum(oracle.init_candidate(3, k, 12).tolist() != ds.init_candidate(3, k, 12, fault) for k in range(40))
    assert bad > 20


def _populations(N, P, seed):
    return [ds.init_candidate(seed + 100, k, N) for k in range(P)]


def test_offspring_match_definition():
    for N, D_dp in SHAPES:
        for P in (1, 2, 7, 16):
            pop = _populations(N, P, N + P)
            for seed in (0, 5):
                for m_x, m_m in ((0, 0), (1, 0), (N // 4, 1), (40, 3), (0, 5), (67, 2)):   # m_x above 32 too
                    for g in (0, 3):
                        for k in (0, 1, 9):
                            want, wpar = ds.make_offspring(seed, g, k, pop, D_dp, m_x, m_m)
                            got, gpar = oracle.make_offspring(seed, g, k, np.array(pop, dtype=np.int32), D_dp, m_x, m_m)
                            assert gpar == wpar and got.tolist() == want, (N, D_dp, P, seed, m_x, m_m, g, k)


@pytest.mark.parametrize("fault", ["parents_exchanged", "parent2_stage_read_from_child", "parent2_stage_by_position",
                                   "stream_and_generation_swapped"])
def test_offspring_comparison_catches_planted_mistakes(fault):
    pop = _populations(24, 16, 1)
    arr = np.array(pop, dtype=np.int32)
    bad = 0
    for k in range(40):
        want, _ = ds.make_offspring(5, 2, k, pop, 4, 6, 1, fault)
        bad += oracle.make_offspring(5, 2, k, arr, 4, 6, 1)[0].tolist() != want
    assert bad > 10


def test_gain4_proposal_and_round_schedule_match_definition():
    for N, D_dp in SHAPES:
        D_pp = N // D_dp
        lat, bw = _network(N, N)
        pr = oracle.Problem(lat, bw, 1e8, 4e6, D_dp, D_pp)
        W = pr.W_pp.tolist()
        for k in range(6):
            perm = ds.init_candidate(9, k, N)
            for r in range(2 * D_pp * (D_pp - 1) // 2 + 3):     # past one full cycle of stage pairs
                a, b, _ = pr.gain4_propose(perm, r)
                assert (a, b) == ds.gain4_proposal(W, perm, D_dp, D_pp, r)
                j, jp = ds.stage_pair_of_round(r, D_pp)
                assert a // D_dp == j and b // D_dp == jp


@pytest.mark.parametrize("nb,proposal", [(oracle.GAIN4, ds.gain4_proposal), (oracle.KL, ds.kl_proposal)])
def test_local_search_rounds_match_definition(nb, proposal):
    # the stage pair of each round, what is proposed, and acceptance on strict improvement of Eq. 1
    for N, D_dp in [(8, 2), (12, 3), (12, 2)]:
        D_pp = N // D_dp
        lat, bw = _network(N, 5 * N)
        pr = oracle.Problem(lat, bw, 2.5e8, 4e6, D_dp, D_pp)
        cost_fn = _cost_fn(pr, D_dp, True)
        pairs = [(a, b) for a in range(N) for b in range(a + 1, N)]
        rounds = D_pp * (D_pp - 1) + 3
        perms = np.array([ds.init_candidate(1, k, N) for k in range(5)], dtype=np.int32)
        out, cost, applied = pr.local_search(perms, rounds, nb)
        n_applied = 0
        for p in range(5):
            wperm, wcost, wapplied = ds.local_search(cost_fn, pr.W_pp.tolist(), perms[p].tolist(), D_dp, D_pp, rounds, proposal)
            assert out[p].tolist() == wperm and cost[p] == wcost
            assert [None if m < 0 else pairs[m] for m in applied[p]] == wapplied
            n_applied += sum(m is not None for m in wapplied)
        assert n_applied > 0


def test_best4_rounds_match_definition():
    # the four candidates of a round, their order, the choice by true cost with ties to the first, acceptance
    total = 0
    for N, D_dp in [(8, 2), (12, 3), (12, 2), (24, 4)]:
        D_pp = N // D_dp
        lat, bw = _network(N, 7 * N)
        pr = oracle.Problem(lat, bw, 2.5e8, 4e6, D_dp, D_pp)
        cost_fn = _cost_fn(pr, D_dp, N <= 12)
        W = pr.W_pp.tolist()
        pairs = [(a, b) for a in range(N) for b in range(a + 1, N)]
        rounds = D_pp * (D_pp - 1) // 2 + 2
        perms = np.array([ds.init_candidate(2, k, N) for k in range(4)], dtype=np.int32)
        for p in range(4):
            for r in range(rounds):
                assert pr.four_candidates(perms[p], r) == ds.four_candidates(W, perms[p].tolist(), D_dp, D_pp, r)
        out, cost, applied = pr.local_search(perms, rounds, oracle.BEST4)
        for p in range(4):
            wperm, wcost, wapplied = ds.local_search_best4(cost_fn, W, perms[p].tolist(), D_dp, D_pp, rounds)
            assert out[p].tolist() == wperm and cost[p] == wcost
            assert [None if m < 0 else pairs[m] for m in applied[p]] == wapplied
            total += sum(m is not None for m in wapplied)
    assert total > 0
    # the paper's own Case-5 tables: whole regions share their weights, so trials tie with each other
    import workloads
    w = workloads.config("C2b")
    pr = oracle.Problem(w.latency, w.bandwidth, w.c_dp, w.c_pp, w.D_dp, w.D_pp)
    cost_fn = _cost_fn(pr, w.D_dp, False)
    perms = workloads.random_population(6, 64, seed=4)
    out, cost, applied = pr.local_search(perms, 30, oracle.BEST4)
    for p in range(6):
        wperm, wcost, _ = ds.local_search_best4(cost_fn, pr.W_pp.tolist(), perms[p].tolist(), 8, 8, 30)
        assert out[p].tolist() == wperm and cost[p] == wcost
    # ties go to the first of the four: on a homogeneous network every trial ties with the current row: nothing moves
    lat, bw = np.full((8, 8), 1e-3), np.full((8, 8), 1e9)
    pr = oracle.Problem(lat, bw, 1e8, 4e6, 2, 4)
    perms = np.array([ds.init_candidate(3, k, 8) for k in range(3)], dtype=np.int32)
    out, cost, applied = pr.local_search(perms, 6, oracle.BEST4)
    assert np.array_equal(out, perms) and np.all(applied == -1)


def _cost_fn(pr, D_dp, brute):
    if brute:   # Eqs. 1-4 by enumeration of all stage orders and all matchings
        Wd, Wp = pr.W_dp.tolist(), pr.W_pp.tolist()
        return lambda perm: dfn.comm_cost(Wd, Wp, dfn.groups_of(perm, D_dp))
    return lambda perm: pr.comm_cost(np.array(perm, dtype=np.int32))


@pytest.mark.parametrize("N,D_dp,P,lam,gens,m_x,m_m,ls,brute", [
    (8, 2, 6, 6, 4, 2, 1, 3, True),
    (8, 2, 5, 9, 3, 5, 0, 7, True),        # lambda > P; more rounds than stage pairs
    (12, 3, 8, 3, 4, 3, 2, 2, True),       # lambda < P
    (12, 2, 4, 1, 12, 3, 1, 2, False),     # steady state
    (24, 4, 6, 6, 2, 40, 1, 4, False),     # m_x > 32
    (24, 6, 5, 7, 2, 6, 3, 0, False),      # no local search
])
def test_evolve_matches_definition(N, D_dp, P, lam, gens, m_x, m_m, ls, brute):
    D_pp = N // D_dp
    lat, bw = _network(N, 3 * N + D_dp)
    pr = oracle.Problem(lat, bw, 2.5e8, 4e6, D_dp, D_pp)
    cost_fn = _cost_fn(pr, D_dp, brute)
    for seed in (0, 11):
        wp, wc, wt = ds.evolve(cost_fn, pr.W_pp.tolist(), seed, gens, P, lam, N, D_dp, D_pp, m_x, m_m, ls)
        gp, gc, gt = pr.evolve(seed=seed, generations=gens, P=P, lam=lam, m_x=m_x, m_m=m_m, ls_moves=ls,
                               neighbourhood=oracle.GAIN4)
        assert gp.tolist() == wp
        assert gc.tolist() == wc and gt.tolist() == wt


def test_replacement_prefers_incumbents_and_lower_origin_on_ties():
    # homogeneous network: every allocation has the same cost bits, so only the origin index decides
    N, D_dp, D_pp, P = 8, 2, 4, 5
    lat = np.full((N, N), 1e-3)
    bw = np.full((N, N), 1e9)
    pr = oracle.Problem(lat, bw, 1e8, 4e6, D_dp, D_pp)
    pop0 = [ds.init_candidate(4, k, N) for k in range(P)]
    gp, gc, gt = pr.evolve(seed=4, generations=3, P=P, lam=7, m_x=2, m_m=1, ls_moves=2)
    assert gp.tolist() == pop0 and len(set(gc.tolist())) == 1
    # and the definition's replacement on a constructed pool with ties
    rows, costs = ds.replace([[0], [1], [2]], [2.0, 1.0, 2.0], [[3], [4]], [1.0, 2.0])
    assert rows == [[1], [3], [0]] and costs == [1.0, 1.0, 2.0]
