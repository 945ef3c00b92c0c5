"""GPU parity: libdtfm (through the C ABI) against the CPU oracle, cost model part (Eqs. 1-4)."""
import itertools

import numpy as np
import pytest
import torch

import oracle
import paper_2206_01288_amd as dtfm
import workloads
from tests.gpu_util import assert_costs_equal, both, custom, dev, host, oracle_eval_threaded

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["C1", "C2", "C2b", "C3h", "C4", "C5"])
def test_weights_bit_exact(name):
    w = workloads.config(name)
    o, g = both(w)
    W_dp, W_pp = dtfm.get_weights(g)
    assert np.array_equal(W_dp, o.W_dp) and np.array_equal(W_pp, o.W_pp)


def test_weights_asymmetric_input():
    lat, bw = workloads.network_two_site_asymmetric(4)
    w = workloads.Workload("asym", 8, 4, 2, 4e8, 1e7, lat, bw, 0)
    o, g = both(w)
    W_dp, W_pp = dtfm.get_weights(g)
    assert np.array_equal(W_dp, o.W_dp) and np.array_equal(W_pp, o.W_pp)


def test_config1_population_and_every_allocation():
    w = workloads.config("C1")
    o, g = both(w)
    perms = workloads.random_population(64, 8, seed=1)
    assert_costs_equal(host(dtfm.eval_population(g, dev(perms))), o.eval_population(perms))
    allp = np.array(list(itertools.permutations(range(8))), dtype=np.int32)
    c = host(dtfm.eval_population(g, dev(allp)))
    ref = o.eval_population(allp)
    assert_costs_equal(c, ref)
    assert int(np.argmin(c)) == int(np.argmin(ref))     # argmin, lowest index on ties


@pytest.mark.parametrize("name,P", [("C2", 4096), ("C2b", 1024), ("C3h", 256)])
def test_config2_full_population(name, P):
    w = workloads.config(name)
    o, g = both(w)
    perms = workloads.random_population(P, 64, seed=1)
    dperm = dev(perms)
    c = host(dtfm.eval_population(g, dperm))
    assert_costs_equal(c, o.eval_population(perms))
    assert int(np.argmin(c)) == int(np.argmin(o.eval_population(perms)))
    ghat, datap = dtfm.coarsened_graph(g, dperm[:64].contiguous())
    ghat, datap = host(ghat), host(datap)
    for p in range(64):
        assert np.array_equal(ghat[p], o.coarsen(perms[p]))
        assert datap[p] == o.datap(perms[p])
    if name == "C3h":
        assert np.all(c == c[0])


def test_config2_population_eight_candidates_per_wavefront():
    # populations between 8193 and 65535 take the eight-candidates-per-wavefront variant of the fused kernel
    w = workloads.config("C2")
    o, g = both(w)
    perms = workloads.random_population(20003, 64, seed=11)
    dperm = dev(perms)
    c = host(dtfm.eval_population(g, dperm))
    assert_costs_equal(c, o.eval_population(perms))
    ghat, datap = dtfm.coarsened_graph(g, dperm)
    ghat, datap = host(ghat), host(datap)
    for p in (0, 1, 2, 3, 9999, 20000, 20001, 20002):
        assert np.array_equal(ghat[p], o.coarsen(perms[p])) and datap[p] == o.datap(perms[p])


@pytest.mark.parametrize("P", [65573, 114693])
def test_config2_population_thirty_two_candidates_per_wavefront(P):
    # 65536 candidates and more: 32 per wavefront pass (7 full matching passes, 4 Held-Karp passes).
    # 65573: one full round of 65536 and a launch of its own for the other 37;
    # 114693 = 3585 groups of 32 in one launch, with a ragged last group of 5
    w = workloads.config("C2")
    o, g = both(w)
    perms = workloads.random_population(P, 64, seed=13)
    dperm = dev(perms)
    c = host(dtfm.eval_population(g, dperm))
    sel = np.r_[0:1100, 30000:31100, P - 1100:P]
    assert_costs_equal(c[sel], o.eval_population(perms[sel]))
    # every row: the same bits as the four-per-wavefront variant gives on chunks of 4096
    for lo in range(0, P, 4096):
        assert np.array_equal(c[lo:lo + 4096], host(dtfm.eval_population(g, dperm[lo:lo + 4096].contiguous())))
    ghat, datap = dtfm.coarsened_graph(g, dperm)
    ghat, datap = host(ghat), host(datap)
    for p in (0, 31, 32, 33, 40000, P - 6, P - 5, P - 1):
        assert np.array_equal(ghat[p], o.coarsen(perms[p])) and datap[p] == o.datap(perms[p])


@pytest.mark.parametrize("P", [2047, 2049, 4095, 4096, 4097, 8191, 8192, 8193, 16383, 16385, 65535, 65536])
def test_population_sizes_where_the_group_size_changes(P):
    # 4 candidates per wavefront pass up to 8192, 8 up to 65535, 32 from 65536; workgroups of 2, 4 or 8
    # wavefronts (as few as give every pass a wavefront of its own): around each switch the costs
    # are those of the oracle (sampled) and, row by row, those of small separately evaluated chunks
    w = workloads.config("C2")
    o, g = both(w)
    perms = workloads.random_population(P, 64, seed=40)
    dperm = dev(perms)
    c = host(dtfm.eval_population(g, dperm))
    sel = np.r_[0:64, P // 2:P // 2 + 64, P - 64:P]
    assert_costs_equal(c[sel], o.eval_population(perms[sel]))
    for lo in range(0, P, 1500):
        assert np.array_equal(c[lo:lo + 1500], host(dtfm.eval_population(g, dperm[lo:lo + 1500].contiguous())))


def test_config2_roofline_launch_size_sampled():
    # the launch bench.py's roofline is taken on: 2^20 candidates (the 65,536 distinct rows repeated 16 times, as
    # there); oracle costs on sampled rows, and every repeat of a row must give the same bits
    w = workloads.config("C2")
    o, g = both(w)
    base = workloads.random_population(1 << 16, 64, seed=3)
    dperm = dev(base).repeat(16, 1).contiguous()
    c = host(dtfm.eval_population(g, dperm)).reshape(16, 1 << 16)
    assert np.all(c == c[0])
    idx = np.random.default_rng(5).choice(1 << 16, size=768, replace=False)
    assert_costs_equal(c[7, idx], o.eval_population(base[idx]))


def test_config4_full_population_every_row():
    # the configured launch (1024 candidates, D_pp = 16: blocked Held-Karp, 16 x 16 matchings): every row against the oracle
    w = workloads.config("C4")
    o, g = both(w)
    perms = workloads.random_population(1024, 256, seed=1)
    c = host(dtfm.eval_population(g, dev(perms)))
    ref = oracle_eval_threaded(o, perms)
    assert_costs_equal(c, ref)
    assert int(np.argmin(c)) == int(np.argmin(ref))
    # reversal of the pipeline keeps the bits
    rev = perms.reshape(1024, 16, 16)[:, ::-1, :].reshape(1024, 256).copy()
    assert np.array_equal(host(dtfm.eval_population(g, dev(rev))), c)


def test_config5_population_every_row_of_256():
    # 256 candidates of configuration 5 (64 x 64 matchings, sliced DataP, blocked Held-Karp): every row against the oracle
    w = workloads.config("C5")
    o, g = both(w)
    perms = workloads.random_population(256, 1024, seed=1)
    dperm = dev(perms)
    c = host(dtfm.eval_population(g, dperm))
    ref = oracle_eval_threaded(o, perms)
    assert_costs_equal(c, ref)
    assert int(np.argmin(c)) == int(np.argmin(ref))
    ghat, datap = dtfm.coarsened_graph(g, dperm[:2].contiguous())
    assert np.array_equal(host(ghat)[1], o.coarsen(perms[1]))
    rev = perms.reshape(256, 16, 64)[:, ::-1, :].reshape(256, 1024).copy()
    assert np.array_equal(host(dtfm.eval_population(g, dev(rev))), c)


def test_config5_full_population_launch_sampled():
    # the configured launch of configuration 5 (4096 candidates): the rows of the 256-candidate launch above, placed
    # across the large one, give the same bits; 32 more rows against the oracle
    w = workloads.config("C5")
    o, g = both(w)
    small = workloads.random_population(256, 1024, seed=1)
    perms = workloads.random_population(4096, 1024, seed=2)
    where = np.arange(256) * 16 + 7
    perms[where] = small
    c = host(dtfm.eval_population(g, dev(perms)))
    assert np.array_equal(c[where], host(dtfm.eval_population(g, dev(small))))
    idx = np.random.default_rng(5).choice(4096, size=32, replace=False)
    assert_costs_equal(c[idx], oracle_eval_threaded(o, perms[idx]))


@pytest.mark.parametrize("D_dp,D_pp", [(1, 1), (1, 5), (5, 1), (2, 2), (3, 4), (7, 3), (4, 9), (3, 10),
                                        (2, 11), (5, 12), (3, 13), (2, 14), (2, 15), (17, 2), (20, 3), (33, 2),
                                        (40, 2), (64, 3), (16, 8), (8, 16)])
def test_odd_and_degenerate_shapes(D_dp, D_pp):
    N = D_dp * D_pp
    w = custom(N, D_dp, D_pp, seed=N + 1)
    o, g = both(w)
    for P in (1, 67) + ((300,) if D_pp == 13 else ()):   # 300: more candidates than workgroups
        perms = workloads.random_population(P, N, seed=P)
        assert_costs_equal(host(dtfm.eval_population(g, dev(perms))), o.eval_population(perms))


@pytest.mark.parametrize("D_dp,D_pp,P", [(24, 16, 24), (40, 13, 24), (48, 16, 16), (64, 12, 12)])
def test_matching_on_bucketed_ranks(D_dp, D_pp, P):
    # more than 65,532 distinct pipeline weights: the matching kernel first solves on ranks shifted into 16 bits and,
    # where a block holds several ranks of the optimum's bucket, solves again inside the bucket. Every stage pair of
    # every candidate against the oracle's coarsened graph; a few whole costs too.
    N = D_dp * D_pp
    w = custom(N, D_dp, D_pp, seed=N + 3)
    assert N * (N - 1) // 2 > 65532
    o, g = both(w)
    perms = workloads.random_population(P, N, seed=D_dp)
    ghat, datap = dtfm.coarsened_graph(g, dev(perms))
    ghat = host(ghat)
    for p in range(P):
        assert np.array_equal(ghat[p], o.coarsen(perms[p])), (D_dp, D_pp, p)
    assert_costs_equal(host(dtfm.eval_population(g, dev(perms[:3]))), o.eval_population(perms[:3]))


@pytest.mark.parametrize("D_dp,D_pp", [(48, 16), (64, 16), (44, 13)])
def test_datap_by_device_and_by_candidate_agree_with_the_oracle(D_dp, D_pp):
    # W_dp beyond an XCD's L2: launches of 64 rows and more take DataP by device (rows of W_dp in LDS, positions
    # from the inverse of each row), smaller ones and rows that are not 16-byte aligned take it by candidate slices
    N = D_dp * D_pp
    w = custom(N, D_dp, D_pp, seed=N + 9)
    o, g = both(w)
    perms = workloads.random_population(150, N, seed=D_pp)
    ref = np.array([o.datap(perms[p]) for p in range(150)])
    for P in (150, 64, 63, 5):
        _, datap = dtfm.coarsened_graph(g, dev(perms[:P]))
        assert np.array_equal(host(datap), ref[:P]), (D_dp, D_pp, P)
    # the same rows behind a 4-byte offset: not 16-byte aligned
    buf = torch.empty(150 * N + 1, dtype=torch.int32, device="cuda")
    buf[1:] = dev(perms).reshape(-1)
    _, datap = dtfm.coarsened_graph(g, buf[1:].view(150, N))
    assert np.array_equal(host(datap), ref)


def test_rows_that_are_not_permutations_do_no_harm():
    # entries inside 0..N-1 but repeated: the cost of such a row means nothing, the call must complete and the
    # other rows keep their values
    w = workloads.config("C5")
    o, g = both(w)
    perms = workloads.random_population(96, 1024, seed=11)
    good = host(dtfm.eval_population(g, dev(perms)))
    bad = perms.copy()
    bad[7, :] = 3
    bad[40, 100:200] = bad[40, 0:100]
    c = host(dtfm.eval_population(g, dev(bad)))
    keep = np.ones(96, dtype=bool)
    keep[[7, 40]] = False
    assert np.array_equal(c[keep], good[keep])


def test_ragged_population_sizes_and_empty():
    w = workloads.config("C2")
    o, g = both(w)
    for P in (1, 3, 63, 65, 255, 257):
        perms = workloads.random_population(P, 64, seed=P)
        assert_costs_equal(host(dtfm.eval_population(g, dev(perms))), o.eval_population(perms))
    empty = torch.empty((0, 64), dtype=torch.int32, device="cuda")
    assert dtfm.eval_population(g, empty).numel() == 0


def test_ties_heavy_matching_blocks():
    # rounded weights: many equal entries in every matching block and many equal path sums
    lat, bw = workloads.network_iid(48, seed=5)
    lat = np.round(lat * 200) / 200 + 0.005
    bw = np.full_like(bw, 1e9)
    w = workloads.Workload("ties", 48, 6, 8, 0.0, 0.0, lat, bw, 0)
    o, g = both(w)
    perms = workloads.random_population(300, 48, seed=2)
    assert_costs_equal(host(dtfm.eval_population(g, dev(perms))), o.eval_population(perms))


@pytest.mark.parametrize("D_dp,D_pp", [(6, 4), (20, 3), (64, 12)])
def test_homogeneous_network_on_general_shapes(D_dp, D_pp):
    # one link class: every matching block holds a single weight (one rank besides the diagonal's), every path the
    # same sum; the closed form is (D_dp - 1) w_dp + (D_pp - 1) w_pp summed left to right
    N = D_dp * D_pp
    lat = np.full((N, N), 1e-3)
    bw = np.full((N, N), 1e9)
    w = workloads.Workload("flat", N, D_dp, D_pp, 6e7, 5e6, lat, bw, 0)
    o, g = both(w)
    perms = workloads.random_population(70, N, seed=N)
    c = host(dtfm.eval_population(g, dev(perms)))
    assert_costs_equal(c, o.eval_population(perms))
    assert np.all(c == c[0])


def test_deterministic_and_stream_ordered():
    w = workloads.config("C2")
    o, g = both(w)
    perms = dev(workloads.random_population(1000, 64, seed=9))
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        a = dtfm.eval_population(g, perms)
        b = dtfm.eval_population(g, perms)
    s.synchronize()
    assert torch.equal(a, b)


def test_validate_population():
    w = workloads.config("C2")
    o, g = both(w)
    perms = workloads.random_population(100, 64, seed=3)
    assert dtfm.validate_population(g, dev(perms)) == 0
    perms[7, 3] = perms[7, 4]
    perms[50, 0] = 64
    perms[99, 63] = -1
    assert dtfm.validate_population(g, dev(perms)) == 3


def test_error_paths_on_device():
    w = workloads.config("C1")
    o, g = both(w)
    L = dtfm.load_library()
    perms = dev(workloads.random_population(4, 8, seed=0))
    cost = torch.empty(4, dtype=torch.float64, device="cuda")
    assert L.dtfm_eval_population(g.handle, perms.data_ptr(), -1, cost.data_ptr(), None) == 4
    assert L.dtfm_eval_population(g.handle, None, 4, cost.data_ptr(), None) == 1
    assert L.dtfm_local_search(g.handle, perms.data_ptr(), 4, 1, 7, cost.data_ptr(), None, None) == 4
    w1 = custom(5, 1, 5, seed=1)
    o1, g1 = both(w1)
    p1 = dev(workloads.random_population(4, 5, seed=0))
    assert L.dtfm_local_search(g1.handle, p1.data_ptr(), 4, 1, dtfm.GAIN4, cost.data_ptr(), None, None) == 6


def test_reserve_keeps_hot_calls_from_growing_the_arena():
    w = workloads.config("C4")
    _, g = both(w)
    dtfm.reserve(g, 64, 64, dtfm.GAIN4)
    perms = dev(workloads.random_population(64, w.N, seed=3))
    a = host(dtfm.eval_population(g, perms))
    pop, cost, trace = dtfm.evolve(g, 1, 1, 64, ls_moves=1)
    b = host(dtfm.eval_population(g, perms))
    assert np.array_equal(a, b)
    with pytest.raises(dtfm.DtfmError):
        dtfm.reserve(g, -1)
    dtfm.destroy_problem(g)
