"""Host-side checks that need no GPU: the C-ABI library loads, exports every symbol the header
declares, and rejects bad arguments with the documented status codes before touching a device."""
import os
import re

import numpy as np
import pytest

import paper_2206_01288_amd as dtfm

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "dtfm.h")).read()
    declared = set(re.findall(r"\b(dtfm_[a-z0-9_]+)\s*\(", header))
    assert declared == set(dtfm.DECLARED_SYMBOLS)
    L = dtfm.load_library()
    for name in declared:
        assert hasattr(L, name), name


def test_status_strings():
    L = dtfm.load_library()
    seen = set()
    for s in range(0, 9):
        text = L.dtfm_status_string(s)
        assert text is not None and len(text) > 0
        seen.add(text)
    assert len(seen) == 9 and L.dtfm_status_string(0) == b"ok"


@pytest.mark.parametrize("kw,status", [
    (dict(N=4, D_dp=2, D_pp=3), 2),            # D_dp * D_pp != N
    (dict(N=4, D_dp=0, D_pp=4), 2),
    (dict(N=34, D_dp=2, D_pp=17), 2),          # D_pp above the Held-Karp limit
    (dict(N=4, D_dp=2, D_pp=2, c_dp=-1.0), 3),
    (dict(N=4, D_dp=2, D_pp=2, c_pp=float("nan")), 3),
    (dict(N=4, D_dp=2, D_pp=2, bad_bw=0.0), 3),
    (dict(N=4, D_dp=2, D_pp=2, bad_lat=-1e-3), 3),
    (dict(N=4, D_dp=2, D_pp=2, bad_lat=float("inf")), 3),
])
def test_create_problem_rejects_bad_input(kw, status):
    N = kw["N"]
    lat = np.full((N, N), 1e-3)
    bw = np.full((N, N), 1e9)
    if "bad_bw" in kw:
        bw[1, 2] = kw["bad_bw"]
    if "bad_lat" in kw:
        lat[2, 1] = kw["bad_lat"]
    # the diagonal is ignored, whatever it holds
    np.fill_diagonal(lat, float("nan"))
    np.fill_diagonal(bw, -1.0)
    with pytest.raises(dtfm.DtfmError) as e:
        dtfm.create_problem(lat, bw, kw.get("c_dp", 1e6), kw.get("c_pp", 1e6), kw["D_dp"], kw["D_pp"])
    assert e.value.status == status


def test_null_arguments():
    L = dtfm.load_library()
    assert L.dtfm_eval_population(None, None, 1, None, None) == 1
    assert L.dtfm_local_search(None, None, 1, 1, 0, None, None, None) == 1
    assert L.dtfm_evolve(None, 0, 1, None, None, None, None, None) == 1
    assert L.dtfm_move_costs(None, None, 1, None, None) == 1
    assert L.dtfm_philox_blocks(0, 0, 0, 0, 0, -1, None, None) == 4
    assert L.dtfm_philox_blocks(0, 0, 0, 0, 0, 3, None, None) == 1
    L.dtfm_destroy_problem(None)


def test_bench_refuses_more_than_one_gpu():
    # every figure of this build is a one-GPU figure: bench.py --gpus N with N > 1 exits with a message
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
