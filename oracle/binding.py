"""ctypes access to the C oracle (test infrastructure, not product code).

Argument marshalling only: all arithmetic of the schedules lives in
sparbit_oracle.c.  The shared object is compiled with gcc on first use.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sparbit_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

SPARBIT, RING, RECURSIVE_DOUBLING, BRUCK, NAIVE = 0, 1, 2, 3, 4
ALGOS = {
    "sparbit": SPARBIT,
    "ring": RING,
    "recursive_doubling": RECURSIVE_DOUBLING,
    "bruck": BRUCK,
    "naive": NAIVE,
}


class OracleError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"oracle error {code}: {msg}")
        self.code = code


def build(force: bool = False) -> str:
    """Compile sparbit_oracle.c into liboracle.so with gcc (plain C11, -O2)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(
            ["gcc", "-std=c11", "-O2", "-Wall", "-Wextra", "-fPIC", "-shared", _SRC, "-o", tmp]
        )
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.oracle_num_steps.argtypes = [ctypes.c_int, ctypes.c_int]
        lib.oracle_num_steps.restype = ctypes.c_int
        lib.oracle_naive_allgather.argtypes = [
            ctypes.c_int, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]
        lib.oracle_naive_allgather.restype = ctypes.c_int
        lib.oracle_allgather.argtypes = [
            ctypes.c_int, ctypes.c_int, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t,
            ctypes.POINTER(ctypes.c_size_t)]
        lib.oracle_allgather.restype = ctypes.c_int
        lib.oracle_allgatherv.argtypes = [
            ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_size_t, ctypes.POINTER(ctypes.c_size_t)]
        lib.oracle_allgatherv.restype = ctypes.c_int
        lib.oracle_strerror.argtypes = [ctypes.c_int]
        lib.oracle_strerror.restype = ctypes.c_char_p
        _lib = lib
    return _lib


def _check(rc: int):
    if rc != 0:
        raise OracleError(rc, _load().oracle_strerror(rc).decode())


def num_steps(algo: int, p: int) -> int:
    return _load().oracle_num_steps(algo, p)


def _as_bytes(a: np.ndarray, nbytes: int, name: str) -> np.ndarray:
    if not (isinstance(a, np.ndarray) and a.flags.c_contiguous and a.nbytes == nbytes):
        raise ValueError(f"{name}: need a C-contiguous numpy array of {nbytes} bytes")
    return a


def naive_allgather(p: int, block_bytes: int, send: np.ndarray, recv: np.ndarray) -> None:
    _as_bytes(send, p * block_bytes, "send")
    _as_bytes(recv, p * p * block_bytes, "recv")
    _check(_load().oracle_naive_allgather(p, block_bytes, send.ctypes.data, recv.ctypes.data))


@dataclass
class OracleRun:
    """What one simulated call reports besides the receive buffers."""
    steps_run: int
    step_info: np.ndarray      # [num_steps, 3] int32: d, ignore flag, blocks sent by rank 0
    sent_per_rank: np.ndarray  # [p] int64
    trace: Optional[np.ndarray]  # [messages, 5] int32: step, src, dst, src_slot, dst_slot


def allgather(algo: int, p: int, block_bytes: int, send: Optional[np.ndarray], recv: np.ndarray,
              max_steps: int = -1, want_trace: bool = False) -> OracleRun:
    """Simulate `algo` on host memory.  `recv` (p*p*block_bytes) is updated in
    place; slots that the executed steps do not write keep the caller's bytes."""
    lib = _load()
    if p < 1 or block_bytes < 1:
        _check(lib.oracle_allgather(algo, p, max(block_bytes, 0), None, None, 0,
                                    None, None, None, 0, None))
    if send is not None:
        _as_bytes(send, p * block_bytes, "send")
    _as_bytes(recv, p * p * block_bytes, "recv")
    if not recv.flags.writeable:
        raise ValueError("recv must be writeable")
    total = max(lib.oracle_num_steps(algo, p), 0)
    step_info = np.zeros((total, 3), dtype=np.int32)
    sent = np.zeros(p, dtype=np.int64)
    trace = None
    cap = 0
    if want_trace:
        cap = p * p  # a slot is written at most once, so at most p*p deliveries
        trace = np.zeros((cap, 5), dtype=np.int32)
    n = ctypes.c_size_t(0)
    rc = lib.oracle_allgather(
        algo, p, block_bytes,
        None if send is None else send.ctypes.data, recv.ctypes.data, max_steps,
        step_info.ctypes.data if total else None, sent.ctypes.data,
        None if trace is None else trace.ctypes.data, cap, ctypes.byref(n))
    _check(rc)
    ran = total if max_steps < 0 else min(max_steps, total)
    return OracleRun(ran, step_info[:ran].copy(), sent,
                     None if trace is None else trace[: n.value].copy())


def allgatherv(algo: int, p: int, counts, displs, row_bytes: int, send: Optional[np.ndarray],
               recv: np.ndarray, max_steps: int = -1, want_trace: bool = False) -> OracleRun:
    """MPI_Allgatherv simulation: rank k contributes counts[k] bytes that land at
    byte displs[k] of every receive buffer; `recv` holds p buffers row_bytes apart,
    `send` is laid out like one receive buffer (or None for in place)."""
    lib = _load()
    c = np.ascontiguousarray(counts, dtype=np.uint64)
    d = np.ascontiguousarray(displs, dtype=np.uint64)
    if c.shape != (p,) or d.shape != (p,):
        raise ValueError("counts and displs need p entries")
    if send is not None:
        _as_bytes(send, row_bytes, "send")
    _as_bytes(recv, p * row_bytes, "recv")
    total = max(lib.oracle_num_steps(algo, p), 0)
    step_info = np.zeros((total, 3), dtype=np.int32)
    sent = np.zeros(p, dtype=np.int64)
    trace, cap = None, 0
    if want_trace:
        cap = p * p
        trace = np.zeros((cap, 5), dtype=np.int32)
    n = ctypes.c_size_t(0)
    rc = lib.oracle_allgatherv(
        algo, p, c.ctypes.data, d.ctypes.data, row_bytes,
        None if send is None else send.ctypes.data, recv.ctypes.data, max_steps,
        step_info.ctypes.data if total else None, sent.ctypes.data,
        None if trace is None else trace.ctypes.data, cap, ctypes.byref(n))
    _check(rc)
    ran = total if max_steps < 0 else min(max_steps, total)
    return OracleRun(ran, step_info[:ran].copy(), sent,
                     None if trace is None else trace[: n.value].copy())
