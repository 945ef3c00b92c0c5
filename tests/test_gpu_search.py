"""GPU parity: local search and evolutionary loop against the CPU oracle, bit for bit."""
import os

import numpy as np
import pytest
import torch

import oracle
import paper_2206_01288_amd as dtfm
import workloads
from tests.gpu_util import assert_costs_equal, both, custom, dev, host

pytestmark = pytest.mark.gpu
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _ls_parity(w, perms, moves, nb):
    o, g = both(w)
    ref_perm, ref_cost, ref_applied = o.local_search(perms, moves, nb)
    d = dev(perms)
    cost, applied = dtfm.local_search(g, d, moves, nb, want_applied=True)
    assert np.array_equal(host(d), ref_perm)
    assert np.array_equal(host(applied), ref_applied)
    assert_costs_equal(host(cost), ref_cost)
    return ref_applied


def test_all_pairs_config1():
    w = workloads.config("C1")
    applied = _ls_parity(w, workloads.random_population(64, 8, seed=1), 6, dtfm.ALL_PAIRS)
    assert (applied >= 0).any() and (applied < 0).any()


def test_all_pairs_config3_sample():
    w = workloads.config("C3")
    applied = _ls_parity(w, workloads.random_population(6, 64, seed=1), 3, dtfm.ALL_PAIRS)
    assert (applied >= 0).all()


def _swapped_rows(row):
    """every allocation one swap of positions a < b away from row, in move-index order"""
    N = row.shape[0]
    out = []
    for a in range(N):
        for b in range(a + 1, N):
            r = row.copy()
            r[a], r[b] = row[b], row[a]
            out.append(r)
    return np.array(out, dtype=np.int32)


@pytest.mark.parametrize("name,rows", [("C2", (0, 5, 11)), ("C2b", (1,)), ("C3h", (2,)), ("C1", (0, 1, 2, 3)), ("C4", (0,))])
def test_move_costs_every_swap_against_oracle(name, rows):
    # incremental move evaluation (64-device shape) and the generic path: the cost of EVERY swap of a row
    # equals the oracle's evaluation of the swapped row, bit for bit. C2b: the paper's table, heavy ties.
    w = workloads.config(name)
    o, g = both(w)
    perms = workloads.random_population(12, w.N, seed=21)
    if name == "C4":   # 32640 swaps of one row: the oracle prices a sample of them
        mc = host(dtfm.move_costs(g, dev(perms[:1])))
        sw = _swapped_rows(perms[0])
        sel = np.r_[0:60, 16000:16060, sw.shape[0] - 60:sw.shape[0]]
        assert_costs_equal(mc[0][sel], o.eval_population(sw[sel]))
        return
    mc = host(dtfm.move_costs(g, dev(perms)))
    assert mc.shape == (12, w.N * (w.N - 1) // 2)
    for p in rows:
        assert_costs_equal(mc[p], o.eval_population(_swapped_rows(perms[p])))
    # the argmin of a row's move costs is what one ALL_PAIRS round applies
    d = dev(perms)
    cur = host(dtfm.eval_population(g, d))
    cost, applied = dtfm.local_search(g, d, 1, dtfm.ALL_PAIRS, want_applied=True)
    best = np.argmin(mc, axis=1)
    exp = np.where(mc[np.arange(12), best] < cur, best, -1)
    assert np.array_equal(host(applied)[:, 0], exp)


def test_all_pairs_paper_table_ties_fused():
    # the paper's Case-5 tables (no jitter: many exactly equal weights) through the fused kernel
    w = workloads.config("C2b")
    _ls_parity(w, workloads.random_population(5, 64, seed=9), 3, dtfm.ALL_PAIRS)


def test_all_pairs_ragged_candidate_counts():
    # one wavefront per candidate, 8 per workgroup: counts around the workgroup size and the grid
    w = workloads.config("C2")
    o, g = both(w)
    for P in (1, 7, 9, 2049):
        perms = workloads.random_population(P, 64, seed=30 + P)
        d = dev(perms)
        cost, applied = dtfm.local_search(g, d, 2, dtfm.ALL_PAIRS, want_applied=True)
        sel = np.unique(np.r_[0, P // 2, P - 1])
        rp, rc, ra = o.local_search(perms[sel], 2, oracle.ALL_PAIRS)
        assert np.array_equal(host(d)[sel], rp) and np.array_equal(host(applied)[sel], ra)
        assert_costs_equal(host(cost)[sel], rc)
        assert dtfm.validate_population(g, d) == 0
        assert torch.equal(dtfm.eval_population(g, d), cost)


def test_all_pairs_homogeneous_never_moves():
    w = workloads.config("C3h")
    o, g = both(w)
    perms = workloads.random_population(96, 64, seed=1)
    d = dev(perms)
    cost, applied = dtfm.local_search(g, d, 2, dtfm.ALL_PAIRS, want_applied=True)
    assert np.array_equal(host(d), perms) and np.all(host(applied) == -1)
    c = host(cost)
    alpha, beta = 0.1e-3, 100e9 / 8
    closed = 2 * 7 * (alpha + w.c_dp / (8 * beta)) + 7 * 2 * (alpha + w.c_pp / beta)
    assert np.all(c == c[0]) and abs(c[0] - closed) <= 1e-12 * closed


def test_all_pairs_ties_take_lowest_index():
    lat, bw = workloads.network_paper_table("paper_case4_network.txt", 3)
    w = workloads.Workload("case4", 12, 3, 4, 1e8, 4e6, lat, bw, 0)
    _ls_parity(w, workloads.random_population(40, 12, seed=8), 4, dtfm.ALL_PAIRS)


@pytest.mark.parametrize("D_dp,D_pp,P,moves", [(2, 2, 9, 3), (3, 4, 33, 5), (1, 6, 5, 2), (6, 1, 5, 2), (1, 1, 3, 2),
                                                (4, 5, 19, 4), (1, 3, 7, 3), (7, 3, 6, 3), (17, 3, 3, 2), (5, 11, 4, 2)])
def test_all_pairs_odd_shapes(D_dp, D_pp, P, moves):
    # three stages and more: the swaps go by stage pair, from the current rows' coarsened graphs
    N = D_dp * D_pp
    _ls_parity(custom(N, D_dp, D_pp, seed=N), workloads.random_population(P, N, seed=4), moves, dtfm.ALL_PAIRS)


def test_gain4_config2():
    w = workloads.config("C2")
    applied = _ls_parity(w, workloads.random_population(64, 64, seed=5), 40, dtfm.GAIN4)
    assert (applied >= 0).any()


@pytest.mark.parametrize("P", [1, 2, 3, 5, 7])
def test_gain4_config2_ragged_small_populations(P):
    # fewer candidates than one wavefront pass holds, more rounds than there are stage pairs
    _ls_parity(workloads.config("C2"), workloads.random_population(P, 64, seed=20 + P), 31, dtfm.GAIN4)


@pytest.mark.parametrize("P", [5001, 8192, 9001, 16500, 65573, 114693])
def test_gain4_large_population_variants(P):
    # 5001, 8192: four candidates per wavefront pass, two wavefronts per SIMD; 9001, 16500: eight candidates per
    # wavefront pass (workgroups of four and of eight wavefronts);
    # 65573: thirty-two for the first 65536, a launch of its own for the rest; 114693: thirty-two, with a
    # ragged last group
    w = workloads.config("C2")
    o, g = both(w)
    perms = workloads.random_population(P, 64, seed=12)
    d = dev(perms)
    cost, applied = dtfm.local_search(g, d, 3, dtfm.GAIN4, want_applied=True)
    sel = np.r_[0:40, P // 2:P // 2 + 40, P - 40:P]
    rp, rc, ra = o.local_search(perms[sel], 3, oracle.GAIN4)
    assert np.array_equal(host(d)[sel], rp) and np.array_equal(host(applied)[sel], ra)
    assert_costs_equal(host(cost)[sel], rc)
    # every row: still a permutation, cost equals a fresh evaluation of the final row
    assert dtfm.validate_population(g, d) == 0
    assert torch.equal(dtfm.eval_population(g, d), cost)


def test_gain4_paper_table_ties():
    w = workloads.config("C2b")
    _ls_parity(w, workloads.random_population(32, 64, seed=6), 30, dtfm.GAIN4)


def test_gain4_config4_and_5_small():
    w = workloads.config("C4")
    _ls_parity(w, workloads.random_population(6, 256, seed=5), 4, dtfm.GAIN4)
    w = workloads.config("C5")
    _ls_parity(w, workloads.random_population(2, 1024, seed=5), 3, dtfm.GAIN4)


@pytest.mark.parametrize("D_dp,D_pp", [(2, 2), (3, 5), (2, 7), (9, 2)])
def test_gain4_odd_shapes(D_dp, D_pp):
    N = D_dp * D_pp
    _ls_parity(custom(N, D_dp, D_pp, seed=N), workloads.random_population(20, N, seed=4), 12, dtfm.GAIN4)


@pytest.mark.parametrize("name,P,rounds", [("C1", 40, 14), ("C2", 64, 30), ("C2b", 24, 30), ("C3h", 8, 5)])
def test_kl_neighbourhood_parity(name, P, rounds):
    w = workloads.config(name)
    _ls_parity(w, workloads.random_population(P, w.N, seed=8), rounds, dtfm.KL)


@pytest.mark.parametrize("D_dp,D_pp", [(1, 2), (2, 2), (3, 5), (2, 7), (9, 2), (64, 2), (16, 16)])
def test_kl_odd_shapes(D_dp, D_pp):
    N = D_dp * D_pp
    _ls_parity(custom(N, D_dp, D_pp, seed=N), workloads.random_population(5, N, seed=4), 4, dtfm.KL)


def test_kl_in_evolve():
    _evolve_parity(workloads.config("C2"), 2, 4, 24, ls_moves=5, neighbourhood=dtfm.KL)


def test_zero_moves_is_plain_evaluation():
    w = workloads.config("C2")
    o, g = both(w)
    perms = workloads.random_population(50, 64, seed=2)
    d = dev(perms)
    cost, _ = dtfm.local_search(g, d, 0, dtfm.ALL_PAIRS)
    assert np.array_equal(host(d), perms)
    assert_costs_equal(host(cost), o.eval_population(perms))


# ---------------------------------------------------------------- Philox + evolve
def test_philox_known_answers_on_device():
    with open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) as f:
        rows = [[int(t, 16) for t in l.split()] for l in f if l.strip() and not l.startswith("#")]
    for v in rows:
        # counter = (block, k, g, stream); key = (seed low, seed high)
        out = dtfm.philox_blocks(seed=v[4] | (v[5] << 32), stream_id=v[3], g=v[2], k=v[1], first_block=v[0],
                                 n_blocks=1)
        assert [int(x) & 0xFFFFFFFF for x in host(out)] == v[6:10]
    out = host(dtfm.philox_blocks(seed=7, stream_id=2, g=3, k=5, first_block=10, n_blocks=5))
    for b in range(5):
        assert [int(x) & 0xFFFFFFFF for x in out[4 * b:4 * b + 4]] == oracle.philox4x32_10([10 + b, 5, 3, 2], [7, 0])


def _evolve_parity(w, seed, gens, P, **kw):
    o, g = both(w)
    rp, rc, rt = o.evolve(seed, gens, P, **kw)
    pop, cost, trace = dtfm.evolve(g, seed, gens, P, **kw)
    assert np.array_equal(host(pop), rp)
    assert_costs_equal(host(cost), rc)
    assert np.array_equal(host(trace), rt)
    return rt


def test_evolve_config1():
    w = workloads.config("C1")
    _evolve_parity(w, 0, 12, 16, ls_moves=2, neighbourhood=dtfm.GAIN4)
    _evolve_parity(w, 2, 6, 16, ls_moves=3, neighbourhood=dtfm.ALL_PAIRS)
    _evolve_parity(w, 3, 0, 7)
    _evolve_parity(w, 4, 5, 9, lam=4, m_x=3, m_m=2, ls_moves=0)


def test_evolve_steady_state_lambda_one():
    # the paper's loop: one offspring per generation, inserted iff better than the worst
    _evolve_parity(workloads.config("C1"), 11, 40, 7, lam=1, m_x=2, m_m=1, ls_moves=2, neighbourhood=dtfm.GAIN4)
    _evolve_parity(workloads.config("C2"), 3, 30, 12, lam=1, ls_moves=4, neighbourhood=dtfm.GAIN4)
    _evolve_parity(workloads.config("C2"), 4, 5, 6, lam=1, ls_moves=1, neighbourhood=dtfm.ALL_PAIRS)
    _evolve_parity(workloads.config("C2"), 5, 10, 20, lam=3, ls_moves=2, neighbourhood=dtfm.GAIN4)


def test_evolve_config2_shape():
    w = workloads.config("C2")
    trace = _evolve_parity(w, 1, 6, 48, ls_moves=8, neighbourhood=dtfm.GAIN4)
    assert np.all(np.diff(trace) <= 0)


def test_evolve_replacement_across_key_chunks():
    # populations and offspring counts that are not multiples of the rank kernel's 64-key chunks and 256-element blocks, with the
    # parents/offspring boundary inside a chunk; odd and even generation counts (the population alternates
    # between two buffers); the homogeneous network makes every cost tie, so only origin indices decide
    w = workloads.config("C1")
    _evolve_parity(w, 21, 3, 300, lam=77, ls_moves=1, neighbourhood=dtfm.GAIN4)
    _evolve_parity(w, 22, 4, 257, lam=600, m_x=2, ls_moves=0)
    _evolve_parity(workloads.config("C3h"), 23, 2, 130, lam=140, ls_moves=1, neighbourhood=dtfm.GAIN4)


def test_evolve_many_crossover_and_mutation_draws():
    # more draws per offspring than the offspring kernel generates at a time (128), odd counts
    _evolve_parity(workloads.config("C2"), 31, 2, 10, m_x=131, m_m=129, ls_moves=0)
    _evolve_parity(workloads.config("C1"), 32, 3, 6, m_x=257, m_m=1, ls_moves=1, neighbourhood=dtfm.GAIN4)


def test_evolve_config5_shape_small_population():
    w = workloads.config("C5")
    _evolve_parity(w, 7, 2, 5, ls_moves=2, neighbourhood=dtfm.GAIN4)


def test_evolve_warm_start_and_determinism():
    w = workloads.config("C2")
    o, g = both(w)
    pop0 = workloads.random_population(24, 64, seed=3)
    rp, rc, rt = o.evolve(5, 3, 24, ls_moves=4, population=pop0)
    pop, cost, trace = dtfm.evolve(g, 5, 3, 24, ls_moves=4, population=dev(pop0))
    assert np.array_equal(host(pop), rp) and np.array_equal(host(trace), rt)
    pop2, cost2, trace2 = dtfm.evolve(g, 5, 3, 24, ls_moves=4, population=dev(pop0))
    assert torch.equal(pop, pop2) and torch.equal(cost, cost2) and torch.equal(trace, trace2)


# ---------------------------------------------------------------- the configurations at full size
def test_config3_full_size_twenty_rounds():
    # 4096 candidates x 20 rounds x 2016 moves on the GPU; what the oracle can do in seconds is compared
    # on sampled candidates (candidates do not interact), the rest by properties that hold at any size
    w = workloads.config("C3")
    o, g = both(w)
    perms = workloads.random_population(4096, 64, seed=1)
    d = dev(perms)
    c0 = host(dtfm.eval_population(g, d))
    cost, applied = dtfm.local_search(g, d, 20, dtfm.ALL_PAIRS, want_applied=True)
    out, cost, applied = host(d), host(cost), host(applied)
    assert np.array_equal(np.sort(out, axis=1), np.tile(np.arange(64, dtype=np.int32), (4096, 1)))
    assert np.array_equal(cost, host(dtfm.eval_population(g, dev(out))))
    assert np.all(cost <= c0) and np.all(cost[(applied >= 0).any(axis=1)] < c0[(applied >= 0).any(axis=1)])
    moves = np.array([(a, b) for a in range(64) for b in range(a + 1, 64)])
    replay = perms.copy()
    rows = np.arange(4096)
    for r in range(20):
        m = applied[:, r]
        on = m >= 0
        a, b = moves[m[on], 0], moves[m[on], 1]
        replay[rows[on], a], replay[rows[on], b] = replay[rows[on], b].copy(), replay[rows[on], a].copy()
    assert np.array_equal(replay, out)
    for p in (17, 3001):
        rp, rc, ra = o.local_search(perms[p:p + 1], 20, oracle.ALL_PAIRS)
        assert np.array_equal(out[p], rp[0]) and np.array_equal(applied[p], ra[0])
        assert_costs_equal(cost[p:p + 1], rc)


def test_config2_bench_step_two_generations():
    # the step bench.py times (population 4096, 4096 offspring, 8 GAIN4 rounds), two generations, against the
    # oracle in full: populations, costs and trace bit for bit
    _evolve_parity(workloads.config("C2"), 2, 2, 4096, ls_moves=8, neighbourhood=dtfm.GAIN4)


def test_config5_full_size_generations():
    # the search of configuration 5 at its population (fewer generations than its 100): properties on
    # everything, oracle costs on sampled survivors
    w = workloads.config("C5")
    o, g = both(w)
    pop, cost, trace = dtfm.evolve(g, 7, 4, 4096, ls_moves=8, neighbourhood=dtfm.GAIN4)
    pop, cost, trace = host(pop), host(cost), host(trace)
    assert np.array_equal(np.sort(pop, axis=1), np.tile(np.arange(1024, dtype=np.int32), (4096, 1)))
    assert np.all(np.diff(cost) >= 0) and np.all(np.diff(trace) <= 0) and trace[-1] == cost[0]
    idx = [0, 1500, 4095]
    assert_costs_equal(cost[idx], o.eval_population(pop[idx]))
    rand = o.eval_population(workloads.random_population(3, 1024, seed=1))
    assert cost[0] < rand.min()


@pytest.mark.parametrize("name,P,rounds", [("C1", 40, 14), ("C2", 64, 30), ("C2b", 24, 30), ("C3h", 8, 5), ("C4", 6, 4),
                                           ("C5", 2, 3)])
def test_best4_local_search(name, P, rounds):
    # the four candidates of the paper's neighbourhood judged by the cost: rows, costs and applied moves against the oracle
    w = workloads.config(name)
    applied = _ls_parity(w, workloads.random_population(P, w.N, seed=8), rounds, dtfm.BEST4)
    if name in ("C1", "C2", "C2b", "C4"):
        assert (applied >= 0).any()
    if name == "C3h":
        assert (applied == -1).all()


@pytest.mark.parametrize("D_dp,D_pp", [(2, 2), (3, 5), (2, 7), (9, 2), (4, 11), (17, 3)])
def test_best4_odd_shapes(D_dp, D_pp):
    N = D_dp * D_pp
    _ls_parity(custom(N, D_dp, D_pp, seed=N), workloads.random_population(7, N, seed=4), 9, dtfm.BEST4)


def test_evolve_with_best4():
    _evolve_parity(workloads.config("C2"), 2, 3, 24, ls_moves=3, neighbourhood=dtfm.BEST4)
    _evolve_parity(workloads.config("C1"), 5, 4, 9, lam=4, ls_moves=4, neighbourhood=dtfm.BEST4)
    _evolve_parity(custom(48, 4, 12, seed=3), 1, 2, 6, ls_moves=2, neighbourhood=dtfm.BEST4)


def _read_golden(name="c5_evolve_seed7_P4096.txt"):
    """tests/golden/c5_evolve_seed7_P4096.txt, written by tests/golden/make_c5_trace.py from the CPU oracle."""
    import os
    import struct
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", name)
    unhex = lambda t: struct.unpack("<d", struct.pack("<Q", int(t, 16)))[0]
    meta, gens, costs, in_costs = {}, {}, [], False
    with open(path) as f:
        for ln in f:
            t = ln.split()
            if not t or t[0].startswith("#"):
                continue
            if in_costs:
                costs += [unhex(x) for x in t]
            elif t[0] == "generation":
                gens[int(t[1])] = {"best": unhex(t[3]), "pop": t[5], "cost": t[7]}
            elif t[0] == "best_trace":
                meta["trace"] = np.array([unhex(x) for x in t[1:]])
            elif t[0] == "final_costs":
                in_costs = True
            else:
                meta[t[0]] = t[1]
    return meta, gens, np.array(costs)


def test_config5_trajectory_against_stored_oracle_run():
    # configuration 5 at its population (4096, Philox seed 7, 8 rounds of the four-candidate local search): the first
    # generations against the run of the CPU oracle stored under tests/golden (initial population, every generation's
    # population and costs by their SHA-256, the best-cost trace and the final costs bit for bit)
    import hashlib
    meta, gens, final_costs = _read_golden()
    G, P = int(meta["generations"]), int(meta["population"])
    assert (int(meta["seed"]), P, int(meta["ls_moves"]), meta["neighbourhood"]) == (7, 4096, 8, "GAIN4") and G >= 2
    w = workloads.config("C5")
    _, g = both(w)
    sha = lambda a: hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()
    for gen in range(0, G + 1):
        pop, cost, trace = dtfm.evolve(g, 7, gen, P, ls_moves=8, neighbourhood=dtfm.GAIN4)
        pop, cost, trace = host(pop), host(cost), host(trace)
        want = gens[gen - 1]
        assert pop.dtype == np.int32 and cost.dtype == np.float64
        assert sha(pop) == want["pop"], "population after generation %d" % (gen - 1)
        assert sha(cost) == want["cost"], "costs after generation %d" % (gen - 1)
        assert cost.min() == want["best"]
    assert np.array_equal(trace, meta["trace"]) and np.array_equal(cost, final_costs)


def test_config4_best4_trajectory_against_stored_oracle_run():
    # configuration 4 at its population (1024, Philox seed 11, 8 rounds in which the round's four candidates are
    # judged by the cost): every generation of the stored CPU-oracle run, populations and costs by SHA-256, the
    # best-cost trace and the final costs bit for bit
    import hashlib
    meta, gens, final_costs = _read_golden("c4_evolve_seed11_P1024_best4.txt")
    G, P = int(meta["generations"]), int(meta["population"])
    assert (int(meta["seed"]), P, int(meta["ls_moves"]), meta["neighbourhood"]) == (11, 1024, 8, "BEST4") and G >= 2
    w = workloads.config("C4")
    _, g = both(w)
    sha = lambda a: hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()
    for gen in (0, 1, G):
        pop, cost, trace = dtfm.evolve(g, 11, gen, P, ls_moves=8, neighbourhood=dtfm.BEST4)
        pop, cost, trace = host(pop), host(cost), host(trace)
        want = gens[gen - 1]
        assert sha(pop) == want["pop"], "population after generation %d" % (gen - 1)
        assert sha(cost) == want["cost"], "costs after generation %d" % (gen - 1)
        assert cost.min() == want["best"]
    assert np.array_equal(trace, meta["trace"]) and np.array_equal(cost, final_costs)


def test_search_calls_are_ordered_on_a_side_stream():
    # local_search, evolve and move_costs enqueue on the caller's current stream: work queued behind them
    # on that stream sees their results, and the results equal those of the default stream
    w = workloads.config("C2")
    o, g = both(w)
    perms = workloads.random_population(200, 64, seed=41)
    ref = dev(perms)
    ref_cost, _ = dtfm.local_search(g, ref, 5, dtfm.GAIN4)
    ref_pop, ref_pc, ref_tr = dtfm.evolve(g, 9, 3, 64, ls_moves=2)
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        d = dev(perms)
        cost, _ = dtfm.local_search(g, d, 5, dtfm.GAIN4)
        again = dtfm.eval_population(g, d)          # queued behind the search on the same stream
        pop, pc, tr = dtfm.evolve(g, 9, 3, 64, ls_moves=2)
        mc = dtfm.move_costs(g, d[:3].contiguous())
    s.synchronize()
    assert torch.equal(d, ref) and torch.equal(cost, ref_cost) and torch.equal(again, cost)
    assert torch.equal(pop, ref_pop) and torch.equal(pc, ref_pc) and torch.equal(tr, ref_tr)
    assert torch.equal(mc, dtfm.move_costs(g, ref[:3].contiguous()))


@pytest.mark.parametrize("seed", range(16))
def test_random_shapes_every_call(seed):
    # a seeded sweep over shapes the other tests do not name: every call of the library against the oracle on the
    # same small inputs (evaluation, the three neighbourhoods, move costs, the evolutionary loop)
    rng = np.random.default_rng(1000 + seed)
    D_dp = int(rng.choice([1, 2, 3, 4, 5, 6, 7, 8, 9, 11, 13, 16, 17, 24, 33]))
    D_pp = int(rng.integers(1, 13)) if D_dp <= 16 else int(rng.integers(1, 5))
    N = D_dp * D_pp
    P = int(rng.integers(1, 30))
    w = custom(N, D_dp, D_pp, seed=2000 + seed)
    o, g = both(w)
    perms = workloads.random_population(P, N, seed=seed)
    assert_costs_equal(host(dtfm.eval_population(g, dev(perms))), o.eval_population(perms))
    if D_dp >= 2 and D_pp >= 2:
        _ls_parity(w, perms, 4, dtfm.GAIN4)
        _ls_parity(w, perms, 3, dtfm.KL)
        _ls_parity(w, perms, 3, dtfm.BEST4)
    if 2 <= N <= 40:
        _ls_parity(w, perms, 2, dtfm.ALL_PAIRS)
        M = N * (N - 1) // 2
        mc = host(dtfm.move_costs(g, dev(perms[:2]))).reshape(-1, M)
        for p in range(mc.shape[0]):
            m = 0
            for a in range(N):
                for b in range(a + 1, N):
                    if (a * 7 + b + seed) % 5 == 0:      # a fifth of the moves
                        q = perms[p].copy()
                        q[a], q[b] = q[b], q[a]
                        assert mc[p, m] == o.eval_population(q[None])[0]
                    m += 1
    if N >= 2:
        nb = dtfm.GAIN4 if (D_dp >= 2 and D_pp >= 2) else dtfm.ALL_PAIRS
        _evolve_parity(w, seed, 2, max(2, P // 3), lam=int(rng.integers(1, 9)), ls_moves=1 if N <= 40 or nb == dtfm.GAIN4 else 0,
                       neighbourhood=nb)
