"""Helpers for the GPU parity tests: the same seeded workload handed to the oracle and to libdtfm."""
import numpy as np
import torch

import oracle
import paper_2206_01288_amd as dtfm
import workloads


def both(w):
    """(oracle problem, GPU problem) for a workloads.Workload."""
    o = oracle.Problem(w.latency, w.bandwidth, w.c_dp, w.c_pp, w.D_dp, w.D_pp)
    g = dtfm.create_problem(w.latency, w.bandwidth, w.c_dp, w.c_pp, w.D_dp, w.D_pp)
    return o, g


def custom(N, D_dp, D_pp, seed, c_dp=6e7, c_pp=5e6):
    lat, bw = workloads.network_iid(N, seed=seed)
    return workloads.Workload("custom", N, D_dp, D_pp, c_dp, c_pp, lat, bw, 0)


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def oracle_eval_threaded(o, perms, threads=16):
    """The oracle's eval_population over host threads (candidates are independent; ctypes releases the GIL)."""
    from concurrent.futures import ThreadPoolExecutor
    chunks = [c for c in np.array_split(perms, threads * 2) if len(c)]
    with ThreadPoolExecutor(threads) as ex:
        return np.concatenate(list(ex.map(o.eval_population, chunks)))


def assert_costs_equal(gpu, ref):
    """spec bar: 1e-9 relative; the build's own bar: identical bits."""
    gpu, ref = np.asarray(gpu), np.asarray(ref)
    assert gpu.shape == ref.shape
    assert np.all(np.abs(gpu - ref) <= 1e-9 * np.abs(ref)), "relative error above 1e-9"
    assert np.array_equal(gpu, ref), "costs differ in the last bits: max rel %.3e" % (
        np.max(np.abs(gpu - ref) / np.maximum(np.abs(ref), 1e-300)))
