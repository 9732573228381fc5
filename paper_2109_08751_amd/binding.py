"""Thin ctypes binding over libsparbit.so: argument marshalling only.

Every function has the name and the argument order of its C entry point in
include/sparbit.h.  Buffers may be given as torch tensors (their data_ptr() is
passed; they must be contiguous CUDA/HIP tensors) or as raw integer device
addresses; `stream` may be a torch.cuda.Stream, an integer hipStream_t or None
(= torch's current stream when torch is loaded with a GPU, else the null
stream).  There is no fallback: if the shared library is absent and cannot be
built, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

from . import build as _build

SPARBIT, RING, RECURSIVE_DOUBLING, BRUCK, DIRECT = 0, 1, 2, 3, 4
MODE_AUTO, MODE_PER_STEP, MODE_PERSISTENT, MODE_DATAFLOW, MODE_TREE = 0, 1, 2, 3, 4
ALGOS = {"sparbit": SPARBIT, "ring": RING, "recursive_doubling": RECURSIVE_DOUBLING,
         "bruck": BRUCK, "direct": DIRECT}


class SparbitError(RuntimeError):
    def __init__(self, code: int, where: str):
        msg = lib.sparbit_strerror(code).decode()
        if code == -4:
            msg += f" (hipError_t {lib.sparbit_last_hip_error()})"
        super().__init__(f"{where}: {msg} [{code}]")
        self.code = code


class _Step(ctypes.Structure):
    _fields_ = [("distance", ctypes.c_int), ("nblocks", ctypes.c_int), ("ignore", ctypes.c_int),
                ("dst", ctypes.POINTER(ctypes.c_int32)), ("src", ctypes.POINTER(ctypes.c_int32)),
                ("send_slot", ctypes.POINTER(ctypes.c_int32)),
                ("recv_slot", ctypes.POINTER(ctypes.c_int32))]


def lib_path() -> str:
    return _build.LIB_PATH


def _load() -> ctypes.CDLL:
    # A process must hold ONE HIP runtime.  torch ships its own copy under the
    # same soname; loading torch first makes the dynamic linker hand that copy
    # to libsparbit.so too, so streams and device pointers mean the same thing
    # on both sides.  Without torch the system runtime is used.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    if _build.is_stale():  # absent, or older than a source: never run a binary that is behind the sources
        try:
            _build.build_library()
        except RuntimeError:
            if not os.path.exists(_build.LIB_PATH):
                raise  # no library and no way to build one: no silent fallback
            import warnings
            warnings.warn("libsparbit.so is older than its sources and could not be rebuilt")
    L = ctypes.CDLL(_build.LIB_PATH)
    vp, sz, ci = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
    L.sparbit_allgather.argtypes = [vp, vp, ci, sz, vp]
    L.sparbit_allgather_static.argtypes = [vp, vp, ci, sz, vp]
    L.sparbit_last_launch_info.argtypes = [ctypes.c_char_p, sz, ctypes.POINTER(ci)]
    L.sparbit_allgather_algo.argtypes = [vp, vp, ci, sz, ci, vp]
    L.sparbit_allgather_mode.argtypes = [vp, vp, ci, sz, ci, ci, vp]
    L.sparbit_allgather_steps.argtypes = [vp, vp, ci, sz, ci, ci, ci, vp]
    L.sparbit_allgatherv.argtypes = [vp, vp, ci, vp, vp, sz, ci, vp]
    L.sparbit_plan_create.argtypes = [ci, ci, ctypes.POINTER(vp)]
    L.sparbit_plan_num_steps.argtypes = [vp]
    L.sparbit_plan_step.argtypes = [vp, ci, ctypes.POINTER(_Step)]
    L.sparbit_plan_destroy.argtypes = [vp]
    L.sparbit_plan_destroy.restype = None
    L.sparbit_finalize.argtypes = []
    L.sparbit_finalize.restype = None
    L.sparbit_strerror.argtypes = [ci]
    L.sparbit_strerror.restype = ctypes.c_char_p
    L.sparbit_last_hip_error.argtypes = []
    L.sparbit_tune.argtypes = [ctypes.c_char_p, ctypes.c_longlong]
    L.sparbit_barrier_timeouts.argtypes = [vp, ctypes.POINTER(ctypes.c_uint64)]
    for name in ("sparbit_allgather", "sparbit_allgather_static", "sparbit_last_launch_info", "sparbit_allgather_algo", "sparbit_allgather_mode",
                 "sparbit_allgather_steps", "sparbit_allgatherv", "sparbit_plan_create", "sparbit_plan_num_steps",
                 "sparbit_plan_step", "sparbit_last_hip_error", "sparbit_tune",
                 "sparbit_barrier_timeouts"):
        getattr(L, name).restype = ci
    return L


lib = _load()


def _ptr(buf) -> Optional[int]:
    if buf is None:
        return None
    if isinstance(buf, int):
        return buf
    if hasattr(buf, "data_ptr"):
        if not buf.is_cuda:
            raise TypeError("buffers must live in device memory")
        if not buf.is_contiguous():
            raise TypeError("buffers must be contiguous")
        return buf.data_ptr()
    raise TypeError(f"cannot take a device address from {type(buf).__name__}")


def _stream(stream) -> Optional[int]:
    if stream is None:
        import sys
        torch = sys.modules.get("torch")
        if torch is not None and torch.cuda.is_available():
            return torch.cuda.current_stream().cuda_stream or None
        return None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _check(rc: int, where: str) -> None:
    if rc != 0:
        raise SparbitError(rc, where)


def sparbit_allgather(sendbufs, recvbufs, p: int, block_bytes: int, stream=None) -> None:
    _check(lib.sparbit_allgather(_ptr(sendbufs), _ptr(recvbufs), p, block_bytes, _stream(stream)),
           "sparbit_allgather")


def sparbit_allgather_static(sendbufs, recvbufs, p: int, block_bytes: int, stream=None) -> None:
    _check(lib.sparbit_allgather_static(_ptr(sendbufs), _ptr(recvbufs), p, block_bytes, _stream(stream)),
           "sparbit_allgather_static")


def sparbit_last_launch_info() -> tuple:
    """(kernel name, launches) of this thread's last call."""
    name = ctypes.create_string_buffer(256)
    n = ci_zero()
    _check(lib.sparbit_last_launch_info(name, 256, ctypes.byref(n)), "sparbit_last_launch_info")
    return name.value.decode(), n.value


def ci_zero():
    return ctypes.c_int(0)


def sparbit_allgather_algo(sendbufs, recvbufs, p: int, block_bytes: int, algo: int, stream=None) -> None:
    _check(lib.sparbit_allgather_algo(_ptr(sendbufs), _ptr(recvbufs), p, block_bytes, algo,
                                      _stream(stream)), "sparbit_allgather_algo")


def sparbit_allgather_mode(sendbufs, recvbufs, p: int, block_bytes: int, algo: int, mode: int,
                           stream=None) -> None:
    _check(lib.sparbit_allgather_mode(_ptr(sendbufs), _ptr(recvbufs), p, block_bytes, algo, mode,
                                      _stream(stream)), "sparbit_allgather_mode")


def sparbit_allgather_steps(sendbufs, recvbufs, p: int, block_bytes: int, algo: int,
                            first_step: int, last_step: int, stream=None) -> None:
    _check(lib.sparbit_allgather_steps(_ptr(sendbufs), _ptr(recvbufs), p, block_bytes, algo,
                                       first_step, last_step, _stream(stream)),
           "sparbit_allgather_steps")


def sparbit_allgatherv(sendbufs, recvbufs, p: int, counts, displs, row_bytes: int, algo: int = SPARBIT,
                       stream=None) -> None:
    c = np.ascontiguousarray(counts, dtype=np.uint64)
    d = np.ascontiguousarray(displs, dtype=np.uint64)
    if c.shape != (p,) or d.shape != (p,):
        raise ValueError("counts and displs need p entries")
    _check(lib.sparbit_allgatherv(_ptr(sendbufs), _ptr(recvbufs), p, c.ctypes.data, d.ctypes.data, row_bytes,
                                  algo, _stream(stream)), "sparbit_allgatherv")


def sparbit_finalize() -> None:
    lib.sparbit_finalize()


def sparbit_strerror(code: int) -> str:
    return lib.sparbit_strerror(code).decode()


def sparbit_tune(key: str, value: int) -> None:
    _check(lib.sparbit_tune(key.encode(), value), f"sparbit_tune({key!r})")


def sparbit_barrier_timeouts(stream=None) -> int:
    n = ctypes.c_uint64(0)
    _check(lib.sparbit_barrier_timeouts(_stream(stream), ctypes.byref(n)), "sparbit_barrier_timeouts")
    return n.value


class Plan:
    """sparbit_plan_create / _num_steps / _step / _destroy; tables come back as
    numpy copies of the library's arrays."""

    def __init__(self, p: int, algo: int = SPARBIT):
        self._h = ctypes.c_void_p()
        _check(lib.sparbit_plan_create(p, algo, ctypes.byref(self._h)), "sparbit_plan_create")
        self.p, self.algo = p, algo

    @property
    def num_steps(self) -> int:
        return lib.sparbit_plan_num_steps(self._h)

    def step(self, s: int) -> dict:
        st = _Step()
        _check(lib.sparbit_plan_step(self._h, s, ctypes.byref(st)), "sparbit_plan_step")
        p, n = self.p, st.nblocks

        def arr(ptr, count, shape):
            if count == 0:
                return np.zeros(shape, dtype=np.int32)
            return np.ctypeslib.as_array(ptr, shape=(count,)).copy().reshape(shape)

        return {"distance": st.distance, "nblocks": n, "ignore": st.ignore,
                "dst": arr(st.dst, p, (p,)), "src": arr(st.src, p, (p,)),
                "send_slot": arr(st.send_slot, p * n, (p, n)),
                "recv_slot": arr(st.recv_slot, p * n, (p, n))}

    def close(self) -> None:
        if self._h:
            lib.sparbit_plan_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
