"""Randomized parity sweep: shapes, networks, populations and search settings drawn from a seeded generator, every
entry point against the oracle, bit for bit. The fixed cases of the other files pick the shapes by hand; this one
walks through combinations nobody picked (each seed: a handful of cases, a second or less each)."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

import paper_2206_01288_amd as dtfm
import workloads
from tests.gpu_util import both, dev, host, oracle_eval_threaded

pytestmark = pytest.mark.gpu

D_DP_CHOICES = [1, 2, 3, 4, 5, 7, 8, 9, 12, 15, 16, 17, 20, 24, 31, 32, 33, 40, 48, 63, 64]


def _network(rng, N, kind, seed):
    if kind == 1:   # rounded latencies, one bandwidth: ties everywhere
        lat, bw = workloads.network_iid(N, seed=seed)
        return np.round(lat * 50) / 50 + 0.01, np.full_like(bw, 1e9)
    if kind == 2:   # four device classes: a handful of distinct link weights
        cls = rng.integers(0, 4, size=N)
        base_lat = np.array([[0.1, 5, 20, 60], [5, 0.2, 30, 70], [20, 30, 0.1, 40], [60, 70, 40, 0.3]]) * 1e-3
        base_bw = np.array([[100, 5, 2, 1], [5, 50, 1.5, 0.8], [2, 1.5, 80, 1.2], [1, 0.8, 1.2, 60]]) * 1e9 / 8
        return base_lat[cls][:, cls].copy(), base_bw[cls][:, cls].copy()
    if kind == 3:   # wide ranges
        return workloads.network_iid(N, seed=seed, lat_ms=(0.05, 300.0), log10_bw_gbps=(-2.0, 2.0))
    return workloads.network_iid(N, seed=seed)


def _search_equal(o, g, perms, rounds, nb, threads=1):
    d = dev(perms.copy())
    cost, applied = dtfm.local_search(g, d, rounds, nb, want_applied=True)
    chunks = [c for c in np.array_split(perms, threads) if len(c)]
    with ThreadPoolExecutor(threads) as ex:
        res = list(ex.map(lambda rows: o.local_search(rows, rounds, nb), chunks))
    assert np.array_equal(host(d), np.concatenate([r[0] for r in res]))
    assert np.array_equal(host(cost), np.concatenate([r[1] for r in res]))
    assert np.array_equal(host(applied), np.concatenate([r[2] for r in res]))


@pytest.mark.parametrize("sweep_seed", [11, 12, 13, 14])
def test_random_shapes_every_entry_point(sweep_seed):
    rng = np.random.default_rng(sweep_seed)
    done = 0
    while done < 10:
        D_pp, D_dp = int(rng.integers(1, 17)), int(rng.choice(D_DP_CHOICES))
        N = D_dp * D_pp
        if N > 1024 or N < 2:
            continue
        done += 1
        kind, seed = int(rng.integers(0, 4)), int(rng.integers(1, 10**6))
        lat, bw = _network(rng, N, kind, seed)
        w = workloads.Workload("sweep", N, D_dp, D_pp, float(10 ** rng.uniform(6, 9)), float(10 ** rng.uniform(5, 8)),
                               lat, bw, 0)
        heavy = D_pp > 10   # Held-Karp on 2^D_pp subsets: keep the oracle's share small
        P = int(rng.choice([1, 3, 9, 20] if heavy else [1, 3, 17, 64, 130]))
        if N >= 512:
            P = min(P, 6)
        o, g = both(w)
        perms = workloads.random_population(P, N, seed=seed + 1)
        what = "D_dp=%d D_pp=%d network %d seed %d P=%d" % (D_dp, D_pp, kind, seed, P)
        assert np.array_equal(host(dtfm.eval_population(g, dev(perms))), oracle_eval_threaded(o, perms)), what
        ghat, datap = dtfm.coarsened_graph(g, dev(perms))
        for p in range(min(P, 4)):
            assert np.array_equal(host(ghat)[p], o.coarsen(perms[p])), what
            assert host(datap)[p] == o.datap(perms[p]), what
        rounds = int(rng.integers(1, 5))
        if D_pp >= 2:
            for nb in ([dtfm.GAIN4, dtfm.KL, dtfm.BEST4] if D_dp >= 2 else [dtfm.KL]):
                if heavy and N >= 256 and nb != dtfm.GAIN4:
                    continue
                _search_equal(o, g, perms, rounds, nb)
        if N <= 48 and D_pp <= 10:
            _search_equal(o, g, perms[:min(P, 3)], 2, dtfm.ALL_PAIRS)
        if (not heavy or N <= 64) and D_pp >= 2 and D_dp >= 2:
            Pg = int(rng.choice([2, 5, 16]))
            lam = int(rng.choice([1, Pg, Pg + 3]))
            pop, cost, trace = dtfm.evolve(g, seed, 2, Pg, lam=lam, ls_moves=rounds, neighbourhood=dtfm.GAIN4)
            pop_o, cost_o, trace_o = o.evolve(seed, 2, Pg, lam=lam, ls_moves=rounds, neighbourhood=dtfm.GAIN4)
            assert np.array_equal(host(pop), pop_o) and np.array_equal(host(cost), cost_o), what
            assert np.array_equal(host(trace), trace_o), what
        order, sigma = dtfm.get_assignment(g, dev(perms[:min(P, 3)]))
        for p in range(min(P, 3)):
            order_o, sigma_o = o.get_assignment(perms[p])
            assert np.array_equal(host(order)[p], order_o) and np.array_equal(host(sigma)[p], sigma_o), what
        dtfm.destroy_problem(g)


@pytest.mark.parametrize("sweep_seed", [21, 22])
def test_random_networks_on_the_64_device_shape(sweep_seed):
    rng = np.random.default_rng(sweep_seed)
    for _ in range(6):
        seed, kind = int(rng.integers(1, 10**6)), int(rng.integers(0, 3))
        lat, bw = workloads.network_iid(64, seed=seed)
        if kind == 1:
            lat, bw = np.round(lat * 40) / 40 + 0.01, np.full_like(bw, 1e9)
        if kind == 2:
            lat, bw = workloads.network_regions(8, 8, seed=seed)
        w = workloads.Workload("sweep64", 64, 8, 8, float(10 ** rng.uniform(6, 9)), float(10 ** rng.uniform(5, 8)), lat, bw, 0)
        o, g = both(w)
        P = int(rng.choice([1, 5, 255, 4096, 4099, 8193, 30000, 66000]))   # every group size and a ragged tail
        perms = workloads.random_population(P, 64, seed=seed + 1)
        what = "network %d seed %d P=%d" % (kind, seed, P)
        assert np.array_equal(host(dtfm.eval_population(g, dev(perms))), oracle_eval_threaded(o, perms)), what
        rounds = int(rng.integers(1, 12))
        for nb in (dtfm.GAIN4, dtfm.KL, dtfm.BEST4):
            _search_equal(o, g, perms[:min(P, 600)], rounds, nb, threads=16)
        _search_equal(o, g, perms[:min(P, 4)], 2, dtfm.ALL_PAIRS)
        Pg = int(rng.choice([3, 64, 300]))
        lam, gens = int(rng.choice([1, Pg, Pg // 2 + 1])), int(rng.integers(1, 4))
        m_m, nb = int(rng.choice([1, 2, 5])), int(rng.choice([dtfm.GAIN4, dtfm.KL, dtfm.BEST4]))
        pop, cost, trace = dtfm.evolve(g, seed, gens, Pg, lam=lam, m_m=m_m, ls_moves=rounds, neighbourhood=nb)
        pop_o, cost_o, trace_o = o.evolve_by_generation(seed, gens, Pg, lam=lam, m_m=m_m, ls_moves=rounds, neighbourhood=nb,
                                                        threads=16)
        assert np.array_equal(host(pop), pop_o) and np.array_equal(host(cost), cost_o), what
        assert np.array_equal(host(trace), trace_o), what
        dtfm.destroy_problem(g)
