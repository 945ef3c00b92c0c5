"""GPU test of the allocation-free entry point dtfm_eval_population_noalloc (through the C ABI): its
costs against those of dtfm_eval_population, bit for bit, on two calls in a row of which the second
has the smaller input (the fixed scratch area keeps the first call's contents), for the shapes that
take the different kernels; and its size limit."""
import numpy as np
import pytest
import torch

import paper_2206_01288_amd as dtfm
import workloads
from tests.gpu_util import assert_costs_equal, custom, dev, host

pytestmark = pytest.mark.gpu


def _problem(w):
    return dtfm.create_problem(w.latency, w.bandwidth, w.c_dp, w.c_pp, w.D_dp, w.D_pp)


@pytest.mark.parametrize("name,shape,P1,P2", [
    ("C1", None, 300, 37),                    # general kernels, Held-Karp table in LDS
    ("custom", (36, 3, 12), 200, 9),          # blocked Held-Karp: exchange areas in the fixed scratch
    ("C4", None, 160, 23),                    # D_pp = 16: few exchange areas, several candidates per workgroup
    ("C5", None, 24, 5),                      # sliced DataP (zeroed scratch), 64 x 64 matchings
    ("C2", None, 5000, 100),                  # 64-device shape: no scratch at all
])
def test_noalloc_equals_eval_population_twice(name, shape, P1, P2):
    w = workloads.config(name) if shape is None else custom(*shape, seed=77)
    g = _problem(w)
    for P, seed in ((P1, 11), (P2, 12)):
        perms = dev(workloads.random_population(P, w.N, seed=seed))
        want = host(dtfm.eval_population(g, perms))
        out = torch.full((P,), -1.0, dtype=torch.float64, device="cuda")
        before = torch.cuda.memory_allocated()
        dtfm.eval_population_noalloc(g, perms, out)
        assert torch.cuda.memory_allocated() == before
        assert_costs_equal(host(out), want)
    dtfm.destroy_problem(g)


def test_noalloc_rejects_what_does_not_fit():
    w = workloads.config("C4")               # needs 8 (1 + 256) bytes per candidate and one 3 MiB exchange area
    g = _problem(w)
    limit = (dtfm.FIXED_SCRATCH_BYTES - (3 << 20)) // (8 * 257)
    P = limit + 64
    perms = torch.zeros((P, w.N), dtype=torch.int32, device="cuda")
    out = torch.full((P,), -1.0, dtype=torch.float64, device="cuda")
    with pytest.raises(dtfm.DtfmError) as e:
        dtfm.eval_population_noalloc(g, perms, out)
    assert e.value.status == 7
    torch.cuda.synchronize()
    assert bool((out == -1.0).all())          # nothing was enqueued
    # P = 0 is a no-op
    dtfm.eval_population_noalloc(g, perms[:0], out[:0])
    dtfm.destroy_problem(g)
