"""Sparbit Allgather hot path for MI355X (gfx950): schedule builder, HIP copy
kernels and their C-ABI, with a thin ctypes binding.

Importing the package is cheap and touches neither torch nor the GPU; the
binding (and with it the shared library) is loaded on first attribute access.
"""
import importlib

_BINDING_NAMES = {
    "SPARBIT", "RING", "RECURSIVE_DOUBLING", "BRUCK", "DIRECT",
    "MODE_AUTO", "MODE_PER_STEP", "MODE_PERSISTENT", "MODE_DATAFLOW", "MODE_TREE",
    "SparbitError", "Plan", "lib", "lib_path",
    "sparbit_allgather", "sparbit_allgather_static", "sparbit_last_launch_info", "sparbit_allgather_algo",
    "sparbit_allgather_steps",
    "sparbit_allgather_mode", "sparbit_allgatherv", "sparbit_finalize", "sparbit_strerror",
    "sparbit_tune", "sparbit_barrier_timeouts", "ALGOS",
}


def __getattr__(name):
    if name in _BINDING_NAMES:
        return getattr(importlib.import_module(".binding", __name__), name)
    raise AttributeError(f"module {__name__!r} has no attribute {name!r}")
