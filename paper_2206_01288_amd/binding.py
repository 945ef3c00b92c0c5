"""ctypes binding of libdtfm.so: argument marshalling only; every step runs in the HIP kernels."""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, c_char_p, c_double, c_int, c_int32, c_uint32, c_uint64, c_void_p

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libdtfm.so")

ALL_PAIRS = 0
GAIN4 = 1
KL = 2
BEST4 = 3
FIXED_SCRATCH_BYTES = 32 << 20     # DTFM_FIXED_SCRATCH_BYTES of include/dtfm.h

# every entry point include/dtfm.h declares
DECLARED_SYMBOLS = [
    "dtfm_create_problem", "dtfm_destroy_problem", "dtfm_get_weights", "dtfm_eval_population",
    "dtfm_coarsened_graph", "dtfm_get_assignment", "dtfm_validate_population", "dtfm_local_search",
    "dtfm_move_costs", "dtfm_evolve", "dtfm_eval_population_noalloc", "dtfm_reserve",
    "dtfm_philox_blocks", "dtfm_status_string", "dtfm_last_hip_error",
]


class DtfmError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__("dtfm status %d: %s" % (status, text))
        self.status = status


class GAParams(ctypes.Structure):
    _fields_ = [("P", c_int32), ("lam", c_int32), ("m_x", c_int32), ("m_m", c_int32),
                ("ls_moves", c_int32), ("neighbourhood", c_int32), ("warm_start", c_int32)]


_lib = None


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads libdtfm.so. Raises if it has not been built (python -m paper_2206_01288_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError("libdtfm.so is not built: run `python -m paper_2206_01288_amd.build` "
                          "(there is no CPU fallback)")
    L = ctypes.CDLL(_LIB_PATH)
    dp = POINTER(c_double)
    L.dtfm_create_problem.argtypes = [dp, dp, c_int, c_double, c_double, c_int, c_int, POINTER(c_void_p)]
    L.dtfm_create_problem.restype = c_int
    L.dtfm_destroy_problem.argtypes = [c_void_p]
    L.dtfm_destroy_problem.restype = None
    L.dtfm_get_weights.argtypes = [c_void_p, dp, dp]
    L.dtfm_eval_population.argtypes = [c_void_p, c_void_p, c_int, c_void_p, c_void_p]
    L.dtfm_eval_population_noalloc.argtypes = [c_void_p, c_void_p, c_int, c_void_p, c_void_p]
    L.dtfm_reserve.argtypes = [c_void_p, c_int, c_int, c_int]
    L.dtfm_coarsened_graph.argtypes = [c_void_p, c_void_p, c_int, c_void_p, c_void_p, c_void_p]
    L.dtfm_get_assignment.argtypes = [c_void_p, c_void_p, c_int, c_void_p, c_void_p, c_void_p]
    L.dtfm_validate_population.argtypes = [c_void_p, c_void_p, c_int, c_void_p, c_void_p]
    L.dtfm_local_search.argtypes = [c_void_p, c_void_p, c_int, c_int, c_int, c_void_p, c_void_p, c_void_p]
    L.dtfm_move_costs.argtypes = [c_void_p, c_void_p, c_int, c_void_p, c_void_p]
    L.dtfm_evolve.argtypes = [c_void_p, c_uint64, c_int, POINTER(GAParams), c_void_p, c_void_p, c_void_p, c_void_p]
    L.dtfm_philox_blocks.argtypes = [c_uint64, c_uint32, c_uint32, c_uint32, c_uint32, c_int, c_void_p, c_void_p]
    L.dtfm_status_string.argtypes = [c_int]
    L.dtfm_status_string.restype = c_char_p
    L.dtfm_last_hip_error.argtypes = []
    L.dtfm_last_hip_error.restype = c_char_p
    _lib = L
    return L


def _check(status: int):
    if status != 0:
        L = load_library()
        text = L.dtfm_status_string(status).decode()
        if status == 5:
            text += " (" + L.dtfm_last_hip_error().decode() + ")"
        raise DtfmError(status, text)


def _stream(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return c_void_p(s.cuda_stream)


def _dev_ptr(t, dtype, numel=None, name="tensor"):
    import torch
    if t is None:
        return c_void_p(0)
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("%s must be a device tensor" % name)
    if t.dtype != dtype or not t.is_contiguous():
        raise TypeError("%s must be contiguous %s" % (name, dtype))
    if numel is not None and t.numel() != numel:
        raise ValueError("%s must have %d elements, has %d" % (name, numel, t.numel()))
    return c_void_p(t.data_ptr())


class Problem:
    """Owner of one dtfm_problem handle."""

    def __init__(self, handle: int, N: int, D_dp: int, D_pp: int):
        self.handle = c_void_p(handle)
        self.N, self.D_dp, self.D_pp = N, D_dp, D_pp

    def close(self):
        if self.handle is not None and self.handle.value:
            load_library().dtfm_destroy_problem(self.handle)
        self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def create_problem(latency, bandwidth, c_dp, c_pp, D_dp, D_pp) -> Problem:
    """latency [s], bandwidth [bytes/s]: host arrays N x N. See dtfm_create_problem."""
    L = load_library()
    lat = np.ascontiguousarray(latency, dtype=np.float64)
    bw = np.ascontiguousarray(bandwidth, dtype=np.float64)
    if lat.ndim != 2 or lat.shape[0] != lat.shape[1] or bw.shape != lat.shape:
        raise ValueError("latency and bandwidth must be N x N")
    N = lat.shape[0]
    out = c_void_p(0)
    _check(L.dtfm_create_problem(lat.ctypes.data_as(POINTER(c_double)), bw.ctypes.data_as(POINTER(c_double)),
                                 N, float(c_dp), float(c_pp), int(D_dp), int(D_pp), ctypes.byref(out)))
    return Problem(out.value, N, int(D_dp), int(D_pp))


def destroy_problem(prob: Problem):
    prob.close()


def get_weights(prob: Problem):
    L = load_library()
    W_dp = np.empty((prob.N, prob.N))
    W_pp = np.empty((prob.N, prob.N))
    _check(L.dtfm_get_weights(prob.handle, W_dp.ctypes.data_as(POINTER(c_double)),
                              W_pp.ctypes.data_as(POINTER(c_double))))
    return W_dp, W_pp


def eval_population(prob: Problem, perm, cost=None, stream=None):
    """perm: device int32 [P, N]; returns (and fills) cost: device float64 [P]."""
    import torch
    L = load_library()
    P = perm.shape[0] if perm.dim() == 2 else 0
    if cost is None:
        cost = torch.empty(P, dtype=torch.float64, device=perm.device)
    _check(L.dtfm_eval_population(prob.handle, _dev_ptr(perm, torch.int32, P * prob.N, "perm"), P,
                                  _dev_ptr(cost, torch.float64, P, "cost"), _stream(stream)))
    return cost


def eval_population_noalloc(prob: Problem, perm, cost, stream=None):
    """dtfm_eval_population_noalloc: as eval_population, with the caller's `cost` tensor (nothing is allocated)."""
    import torch
    L = load_library()
    P = perm.shape[0] if perm.dim() == 2 else 0
    _check(L.dtfm_eval_population_noalloc(prob.handle, _dev_ptr(perm, torch.int32, P * prob.N, "perm"), P,
                                          _dev_ptr(cost, torch.float64, P, "cost"), _stream(stream)))
    return cost


def reserve(prob: Problem, P: int, lam: int = 0, neighbourhood: int = GAIN4):
    """dtfm_reserve: grows the handle's scratch area once, ahead of the hot calls."""
    _check(load_library().dtfm_reserve(prob.handle, int(P), int(lam), int(neighbourhood)))


def coarsened_graph(prob: Problem, perm, stream=None, out=None):
    """Returns (ghat [P, D_pp, D_pp], datap [P]) device tensors (`out`: the pair to fill instead of new ones)."""
    import torch
    L = load_library()
    P = perm.shape[0]
    if out is not None:
        ghat, datap = out
    else:
        ghat = torch.empty((P, prob.D_pp, prob.D_pp), dtype=torch.float64, device=perm.device)
        datap = torch.empty(P, dtype=torch.float64, device=perm.device)
    _check(L.dtfm_coarsened_graph(prob.handle, _dev_ptr(perm, torch.int32, P * prob.N, "perm"), P,
                                  _dev_ptr(ghat, torch.float64, P * prob.D_pp * prob.D_pp, "ghat"),
                                  _dev_ptr(datap, torch.float64, P, "datap"), _stream(stream)))
    return ghat, datap


def get_assignment(prob: Problem, perm, stream=None):
    """Returns (stage_order [P, D_pp], sigma [P, D_dp, D_pp]) int32 device tensors."""
    import torch
    L = load_library()
    P = perm.shape[0]
    order = torch.empty((P, prob.D_pp), dtype=torch.int32, device=perm.device)
    sigma = torch.empty((P, prob.D_dp, prob.D_pp), dtype=torch.int32, device=perm.device)
    _check(L.dtfm_get_assignment(prob.handle, _dev_ptr(perm, torch.int32, P * prob.N, "perm"), P,
                                 _dev_ptr(order, torch.int32), _dev_ptr(sigma, torch.int32), _stream(stream)))
    return order, sigma


def validate_population(prob: Problem, perm, stream=None) -> int:
    import torch
    L = load_library()
    P = perm.shape[0]
    bad = torch.empty(1, dtype=torch.int32, device=perm.device)
    _check(L.dtfm_validate_population(prob.handle, _dev_ptr(perm, torch.int32, P * prob.N, "perm"), P,
                                      _dev_ptr(bad, torch.int32), _stream(stream)))
    return int(bad.item())


def local_search(prob: Problem, perm, moves: int, neighbourhood: int = ALL_PAIRS, cost=None,
                 applied=None, want_applied: bool = False, stream=None):
    """perm: device int32 [P, N], modified in place. Returns (cost [P], applied [P, moves] or None)."""
    import torch
    L = load_library()
    P = perm.shape[0]
    if cost is None:
        cost = torch.empty(P, dtype=torch.float64, device=perm.device)
    if applied is None and want_applied:
        applied = torch.empty((P, moves), dtype=torch.int64, device=perm.device)
    _check(L.dtfm_local_search(prob.handle, _dev_ptr(perm, torch.int32, P * prob.N, "perm"), P, int(moves),
                               int(neighbourhood), _dev_ptr(cost, torch.float64, P, "cost"),
                               _dev_ptr(applied, torch.int64, P * moves, "applied") if applied is not None
                               else c_void_p(0), _stream(stream)))
    return cost, applied


def move_costs(prob: Problem, perm, out=None, stream=None):
    """perm: device int32 [P, N] (read only). Returns the cost of every swap, device float64 [P, N(N-1)/2]."""
    import torch
    L = load_library()
    P, M = perm.shape[0], prob.N * (prob.N - 1) // 2
    if out is None:
        out = torch.empty((P, M), dtype=torch.float64, device=perm.device)
    _check(L.dtfm_move_costs(prob.handle, _dev_ptr(perm, torch.int32, P * prob.N, "perm"), P,
                             _dev_ptr(out, torch.float64, P * M, "move_cost"), _stream(stream)))
    return out


def evolve(prob: Problem, seed: int, generations: int, P: int, lam=None, m_x=None, m_m: int = 1,
           ls_moves: int = 8, neighbourhood: int = GAIN4, population=None, stream=None, device="cuda"):
    """Returns (population [P, N] int32, cost [P], best_trace [generations]) device tensors."""
    import torch
    L = load_library()
    prm = GAParams(int(P), int(P if lam is None else lam), int(prob.N // 4 if m_x is None else m_x), int(m_m),
                   int(ls_moves), int(neighbourhood), 0 if population is None else 1)
    if population is None:
        population = torch.empty((P, prob.N), dtype=torch.int32, device=device)
    cost = torch.empty(P, dtype=torch.float64, device=population.device)
    trace = torch.empty(max(generations, 0), dtype=torch.float64, device=population.device)
    _check(L.dtfm_evolve(prob.handle, c_uint64(seed), int(generations), ctypes.byref(prm),
                         _dev_ptr(population, torch.int32, P * prob.N, "population"),
                         _dev_ptr(cost, torch.float64, P, "cost"),
                         _dev_ptr(trace, torch.float64) if generations > 0 else c_void_p(0), _stream(stream)))
    return population, cost, trace


def philox_blocks(seed: int, stream_id: int, g: int, k: int, first_block: int, n_blocks: int, device="cuda",
                  stream=None):
    import torch
    L = load_library()
    out = torch.empty(4 * n_blocks, dtype=torch.int32, device=device)
    _check(L.dtfm_philox_blocks(c_uint64(seed), stream_id, g, k, first_block, n_blocks,
                                _dev_ptr(out, torch.int32), _stream(stream)))
    return out
