"""Minimal ctypes access to the HIP runtime that is already loaded in the process (the one PyTorch ships),
used for event timing on the stream the library launches on."""
from __future__ import annotations

import ctypes as C

import torch  # noqa: F401  (loads the HIP runtime)


def _loaded_runtime_path() -> str:
    with open("/proc/self/maps") as f:
        paths = sorted({line.split()[-1] for line in f if "libamdhip64" in line})
    if not paths:
        raise RuntimeError("no HIP runtime is loaded in this process")
    return paths[0]


_hip = None


def hip() -> C.CDLL:
    global _hip
    if _hip is None:
        _hip = C.CDLL(_loaded_runtime_path())
        _hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        _hip.hipEventRecord.argtypes = [C.c_void_p, C.c_void_p]
        _hip.hipEventSynchronize.argtypes = [C.c_void_p]
        _hip.hipEventDestroy.argtypes = [C.c_void_p]
    return _hip


def _ok(code: int, what: str):
    if code != 0:
        raise RuntimeError(f"{what} failed with HIP error {code}")


class Events:
    """A host array of n timing events, usable as the argument of hire_set_stage_events."""

    def __init__(self, n: int):
        self.n = n
        self.array = (C.c_void_p * n)()
        for i in range(n):
            ev = C.c_void_p()
            _ok(hip().hipEventCreate(C.byref(ev)), "hipEventCreate")
            self.array[i] = ev

    def record(self, i: int, stream_handle: int):
        _ok(hip().hipEventRecord(self.array[i], C.c_void_p(stream_handle)), "hipEventRecord")

    def synchronize(self, i: int):
        _ok(hip().hipEventSynchronize(self.array[i]), "hipEventSynchronize")

    def elapsed_ms(self, i: int, j: int) -> float:
        ms = C.c_float(0.0)
        _ok(hip().hipEventElapsedTime(C.byref(ms), self.array[i], self.array[j]), "hipEventElapsedTime")
        return float(ms.value)

    def __del__(self):
        try:
            for i in range(self.n):
                hip().hipEventDestroy(self.array[i])
        except Exception:
            pass
