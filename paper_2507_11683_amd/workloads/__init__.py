"""Seeded synthetic workloads: the five benchmark configurations and their input series.

This module only describes and generates INPUTS (shapes of the paper's Table 1 datasets,
traffic-shaped values).  It holds none of the method's arithmetic and is the one module
that both the CPU oracle's tests and the HIP path's callers may use.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "traffic_gen.c")
_LIB = os.path.join(_HERE, "libtraffic_gen.so")
_lib = None


@dataclass(frozen=True)
class Workload:
    """One benchmark configuration.  T entries, N nodes, F features; P input / Q target steps;
    B batch size; the epoch is the shuffle of (seed, epoch) split over `world`, rank `rank`."""
    name: str
    T: int
    N: int
    F: int
    P: int
    Q: int
    B: int
    storage: str          # "f32" or "bf16": how the resident series is stored
    seed: int
    epochs: tuple
    world: int
    rank: int
    data_seed: int
    gen_flags: int        # bit 0: per-node amplitude/phase, bit 1: weekly modulation

    @property
    def n_windows(self) -> int:
        return self.T - self.P - self.Q + 1

    @property
    def row_elems(self) -> int:
        return self.N * self.F

    @property
    def series_bytes_f32(self) -> int:
        return self.T * self.N * self.F * 4

    def bytes_per_snapshot(self, out_bytes: int = 4) -> int:
        """Algorithmic bytes per snapshot: every element of the (P+Q)-step span is read once in
        the storage type and written once in the output type (fp32 unless stated)."""
        s_in = 4 if self.storage == "f32" else 2
        return (self.P + self.Q) * self.N * self.F * (s_in + out_bytes)


WORKLOADS = {
    w.name: w
    for w in [
        Workload("tiny", 2000, 207, 2, 12, 12, 64, "f32", 0, (0,), 1, 0, 1001, 0),
        Workload("medium", 34272, 207, 2, 12, 12, 64, "f32", 0, (0,), 1, 0, 1002, 1),
        Workload("medium_wide", 52116, 325, 2, 12, 12, 64, "f32", 0, (0,), 1, 0, 1003, 3),
        Workload("statewide", 105120, 11160, 2, 12, 12, 32, "f32", 0, (0,), 1, 0, 1004, 1),
        Workload("statewide_bf16_rank3of16", 105120, 11160, 2, 12, 12, 32, "bf16", 7, (0, 1, 2),
                 16, 3, 1004, 1),
    ]
}


def build(force: bool = False) -> str:
    """Compile the generator with gcc + OpenMP.  Returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c11", _SRC,
                               "-o", tmp, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.traffic_series_fill.restype = ctypes.c_int
        lib.traffic_series_fill.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64,
                                            ctypes.c_uint64, ctypes.c_int, ctypes.c_int64,
                                            ctypes.c_int64]
        _lib = lib
    return _lib


def traffic_series(T: int, N: int, data_seed: int, gen_flags: int, out: np.ndarray | None = None,
                   t_begin: int = 0, t_end: int | None = None) -> np.ndarray:
    """[T, N, 2] fp32: channel 0 speed, channel 1 time of day.  `out` may be any writable
    C-contiguous float32 buffer of that shape (for example the numpy view of a pinned tensor)."""
    if out is None:
        out = np.empty((T, N, 2), dtype=np.float32)
    if out.shape != (T, N, 2) or out.dtype != np.float32 or not out.flags.c_contiguous:
        raise ValueError("out must be a C-contiguous float32 [T, N, 2] array")
    rc = _load().traffic_series_fill(out.ctypes.data, T, N, data_seed, gen_flags, t_begin,
                                     T if t_end is None else t_end)
    if rc != 0:
        raise RuntimeError(f"traffic_series_fill failed (rc={rc})")
    return out


def make_series(w: Workload, out: np.ndarray | None = None) -> np.ndarray:
    if w.F != 2:
        raise ValueError("the traffic generator produces F=2 series")
    return traffic_series(w.T, w.N, w.data_seed, w.gen_flags, out=out)
