"""Raw HIP events through ctypes, on the HIP runtime torch has already loaded.

Used by the benchmark to time the similarity kernel on the stream it is launched on
(krul_pair_similarity_timed records two such events around that kernel)."""
from __future__ import annotations

import ctypes

import torch  # noqa: F401  (loads the HIP runtime)

_hip = None


def _runtime() -> ctypes.CDLL:
    global _hip
    if _hip is None:
        path = None
        with open("/proc/self/maps") as f:
            for line in f:
                if "libamdhip64" in line:
                    path = line.split()[-1]
                    break
        if path is None:
            raise RuntimeError("HIP runtime is not loaded in this process")
        _hip = ctypes.CDLL(path)
        _hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        _hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        _hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        _hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        _hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
    return _hip


def _check(rc: int, what: str):
    if rc != 0:
        raise RuntimeError(f"{what} failed with hipError {rc}")


def create() -> int:
    ev = ctypes.c_void_p()
    _check(_runtime().hipEventCreate(ctypes.byref(ev)), "hipEventCreate")
    return ev.value


def destroy(ev: int):
    _check(_runtime().hipEventDestroy(ctypes.c_void_p(ev)), "hipEventDestroy")


def record(ev: int, stream: int):
    _check(_runtime().hipEventRecord(ctypes.c_void_p(ev), ctypes.c_void_p(stream)), "hipEventRecord")


def elapsed_ms(begin: int, end: int) -> float:
    _check(_runtime().hipEventSynchronize(ctypes.c_void_p(end)), "hipEventSynchronize")
    ms = ctypes.c_float()
    _check(_runtime().hipEventElapsedTime(ctypes.byref(ms), ctypes.c_void_p(begin), ctypes.c_void_p(end)),
           "hipEventElapsedTime")
    return float(ms.value)
