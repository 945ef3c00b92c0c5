"""MI355X (gfx950) evaluation of the allocation cost model and search of arXiv 2206.01288.

Thin ctypes binding over libdtfm.so (hand-written HIP kernels behind a C ABI, see include/dtfm.h).
PyTorch is used only to own device memory and to name the HIP stream. There is no CPU fallback:
loading fails loudly when the library has not been built.
"""
from .binding import (ALL_PAIRS, GAIN4, KL, BEST4, FIXED_SCRATCH_BYTES, DtfmError, GAParams, Problem, create_problem, destroy_problem,
                      eval_population, eval_population_noalloc, reserve, coarsened_graph, get_assignment, validate_population, local_search, move_costs, evolve,
                      philox_blocks, get_weights, library_path, load_library, DECLARED_SYMBOLS)

__all__ = ["ALL_PAIRS", "GAIN4", "KL", "BEST4", "FIXED_SCRATCH_BYTES", "DtfmError", "GAParams", "Problem", "create_problem", "destroy_problem",
           "eval_population", "eval_population_noalloc", "reserve", "coarsened_graph", "get_assignment", "validate_population", "local_search", "move_costs",
           "evolve",
           "philox_blocks", "get_weights", "library_path", "load_library", "DECLARED_SYMBOLS"]
