"""CPU oracle for index-batched snapshot construction: ctypes wrapper over pgti_oracle.c.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this module; it is used
by the tests, by the smoke check and by the CPU-baseline leg of the benchmark.  It imports
nothing from the HIP package either.  Every function here only marshals numpy arrays into
the C functions, each of which cites the passage of the paper it follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pgti_oracle.c")
_LIB = os.path.join(_HERE, "libpgti_oracle.so")
# No FMA contraction, no fast-math: every fp32 operation is a single IEEE-754 RNE operation.
_CFLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC", "-std=c11"]

_lock = threading.Lock()
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (about a second).  Returns the path of the library."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", *_CFLAGS, _SRC, "-o", tmp, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is not None:
            return _lib
        lib = ctypes.CDLL(build())
        i64, u64, i32p = ctypes.c_int64, ctypes.c_uint64, ctypes.POINTER(ctypes.c_int32)
        vp, fp = ctypes.c_void_p, ctypes.POINTER(ctypes.c_float)
        lib.oracle_window_count.restype = i64
        lib.oracle_window_count.argtypes = [i64, i64, i64]
        lib.oracle_eq1_materialized_elements.restype = i64
        lib.oracle_eq1_materialized_elements.argtypes = [i64] * 4
        lib.oracle_eq2_index_batching_elements.restype = i64
        lib.oracle_eq2_index_batching_elements.argtypes = [i64] * 4
        lib.oracle_mix64.restype = u64
        lib.oracle_mix64.argtypes = [u64]
        lib.oracle_splitmix64_next.restype = u64
        lib.oracle_splitmix64_next.argtypes = [ctypes.POINTER(u64)]
        lib.oracle_key.restype = u64
        lib.oracle_key.argtypes = [u64, u64, u64]
        lib.oracle_keys.restype = ctypes.c_int
        lib.oracle_keys.argtypes = [u64, u64, i64, vp]
        lib.oracle_sort_pairs.restype = ctypes.c_int
        lib.oracle_sort_pairs.argtypes = [vp, i64, vp]
        lib.oracle_epoch_perm.restype = ctypes.c_int
        lib.oracle_epoch_perm.argtypes = [u64, u64, i64, vp]
        lib.oracle_epoch_indices_ex.restype = ctypes.c_int
        lib.oracle_epoch_indices_ex.argtypes = [ctypes.c_int, i64, i64, i64, i64, u64, u64, i64, i64, vp,
                                                ctypes.POINTER(i64)]
        lib.oracle_rank_share.restype = ctypes.c_int
        lib.oracle_rank_share.argtypes = [i64, i64, i64, ctypes.POINTER(i64), ctypes.POINTER(i64)]
        lib.oracle_bf16_from_f32.restype = ctypes.c_uint16
        lib.oracle_bf16_from_f32.argtypes = [ctypes.c_float]
        lib.oracle_f32_from_bf16.restype = ctypes.c_float
        lib.oracle_f32_from_bf16.argtypes = [ctypes.c_uint16]
        lib.oracle_store_bf16.restype = None
        lib.oracle_store_bf16.argtypes = [vp, i64, vp]
        lib.oracle_standardize.restype = ctypes.c_float
        lib.oracle_standardize.argtypes = [ctypes.c_float] * 3
        lib.oracle_build_batch.restype = ctypes.c_int
        lib.oracle_build_batch.argtypes = [vp, ctypes.c_int, i64, i64, i64, i64, i64, vp, vp, vp,
                                           i64, vp, vp]
        lib.oracle_build_batch_bf16_out.restype = ctypes.c_int
        lib.oracle_build_batch_bf16_out.argtypes = [vp, ctypes.c_int, i64, i64, i64, i64, i64, vp, vp, vp,
                                                    i64, vp, vp]
        lib.oracle_alg1_preprocess.restype = ctypes.c_int
        lib.oracle_alg1_preprocess.argtypes = [vp, i64, i64, i64, i64, i64, vp, vp, vp, vp]
        lib.oracle_alg1_train_stats.restype = ctypes.c_int
        lib.oracle_alg1_train_stats.argtypes = [vp, i64, i64, i64, i64, i64,
                                                ctypes.POINTER(ctypes.c_double),
                                                ctypes.POINTER(ctypes.c_double)]
        lib.oracle_alg1_train_stats_fraction.restype = ctypes.c_int
        lib.oracle_alg1_train_stats_fraction.argtypes = [vp, i64, i64, i64, i64, i64, ctypes.c_double,
                                                         ctypes.POINTER(ctypes.c_double),
                                                         ctypes.POINTER(ctypes.c_double)]
        lib.oracle_add_time_of_day.restype = ctypes.c_int
        lib.oracle_add_time_of_day.argtypes = [vp, i64, i64, i64, i64, vp]
        lib.oracle_series_stats.restype = ctypes.c_int
        lib.oracle_series_stats.argtypes = [vp, i64, i64, i64, vp, vp]
        _lib = lib
        return lib


F32, BF16 = 0, 1


def _ptr(a: np.ndarray) -> int:
    return a.ctypes.data


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise ValueError(f"oracle: {what} rejected its arguments (rc={rc})")


def _c(a, dtype) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def window_count(T: int, P: int, Q: int) -> int:
    return int(_load().oracle_window_count(T, P, Q))


def eq1_materialized_elements(entries: int, horizon: int, nodes: int, features: int) -> int:
    return int(_load().oracle_eq1_materialized_elements(entries, horizon, nodes, features))


def eq2_index_batching_elements(entries: int, horizon: int, nodes: int, features: int) -> int:
    return int(_load().oracle_eq2_index_batching_elements(entries, horizon, nodes, features))


def mix64(z: int) -> int:
    return int(_load().oracle_mix64(z & 0xFFFFFFFFFFFFFFFF))


def splitmix64_stream(state: int, count: int) -> list[int]:
    st = ctypes.c_uint64(state)
    lib = _load()
    return [int(lib.oracle_splitmix64_next(ctypes.byref(st))) for _ in range(count)]


def key(seed: int, epoch: int, i: int) -> int:
    return int(_load().oracle_key(seed, epoch, i))


def keys(seed: int, epoch: int, n: int) -> np.ndarray:
    """key(seed, epoch, i) for i = 0 .. n-1."""
    out = np.empty(max(n, 0), dtype=np.uint64)
    _check(_load().oracle_keys(seed, epoch, n, _ptr(out)), "keys")
    return out


def sort_pairs(keys: np.ndarray) -> np.ndarray:
    keys = _c(keys, np.uint64)
    out = np.empty(keys.shape[0], dtype=np.int32)
    _check(_load().oracle_sort_pairs(_ptr(keys), keys.shape[0], _ptr(out)), "sort_pairs")
    return out


def epoch_perm(seed: int, epoch: int, n: int) -> np.ndarray:
    out = np.empty(max(n, 0), dtype=np.int32)
    _check(_load().oracle_epoch_perm(seed, epoch, n, _ptr(out)), "epoch_perm")
    return out


def rank_share(n: int, rank: int, world: int) -> tuple[int, int]:
    lo, hi = ctypes.c_int64(), ctypes.c_int64()
    _check(_load().oracle_rank_share(n, rank, world, ctypes.byref(lo), ctypes.byref(hi)),
           "rank_share")
    return int(lo.value), int(hi.value)


def epoch_indices(seed: int, epoch: int, rank: int, world: int, n: int) -> np.ndarray:
    """One rank's share of the epoch: perm[lo:hi)."""
    lo, hi = rank_share(n, rank, world)
    return epoch_perm(seed, epoch, n)[lo:hi].copy()


ORDER_SHUFFLE, ORDER_SEQUENTIAL, ORDER_BATCH_SHUFFLE = 0, 1, 2


def epoch_indices_ex(order: int, n_windows: int, first_start: int, n_starts: int, B: int, seed: int,
                     epoch: int, rank: int = 0, world: int = 1) -> np.ndarray:
    """One rank's share for any order (global shuffle / sequential / batch-level shuffle) over the
    range of starts [first_start, first_start + n_starts)."""
    out = np.empty(max(n_starts, 1), dtype=np.int32)
    n = ctypes.c_int64()
    _check(_load().oracle_epoch_indices_ex(order, n_windows, first_start, n_starts, B, seed, epoch, rank,
                                           world, _ptr(out), ctypes.byref(n)), "epoch_indices_ex")
    return out[:n.value].copy()


def bf16_from_f32(v: float) -> int:
    return int(_load().oracle_bf16_from_f32(v))


def store_bf16(a: np.ndarray) -> np.ndarray:
    """fp32 array -> uint16 array of bf16 bit patterns (round to nearest, ties to even)."""
    a = _c(a, np.float32)
    out = np.empty(a.shape, dtype=np.uint16)
    _load().oracle_store_bf16(_ptr(a), a.size, _ptr(out))
    return out


def widen_bf16(b: np.ndarray) -> np.ndarray:
    lib = _load()
    flat = _c(b, np.uint16).ravel()
    return np.array([lib.oracle_f32_from_bf16(int(v)) for v in flat],
                    dtype=np.float32).reshape(np.shape(b))


def standardize(v: float, mu: float, sigma: float) -> float:
    return float(_load().oracle_standardize(v, mu, sigma))


def build_batch(series: np.ndarray, storage: int, P: int, Q: int, mean, std,
                starts, out=None) -> tuple[np.ndarray, np.ndarray]:
    """x[count,P,N,F], y[count,Q,N,F] for the given starts.  `series` is [T,N,F], float32 for
    storage F32 or uint16 bf16 bit patterns for storage BF16.  `out` = (x, y) float32 C-contiguous
    arrays with at least that many elements receives the result in place of fresh arrays (callers
    that check many batches reuse their buffers); the returned views have the shapes above."""
    want = np.float32 if storage == F32 else np.uint16
    if series.dtype != want or not series.flags.c_contiguous or series.ndim != 3:
        raise ValueError("series must be a C-contiguous [T,N,F] array of the storage dtype")
    T, N, F = series.shape
    mean, std = _c(mean, np.float32), _c(std, np.float32)
    starts = _c(starts, np.int32)
    if mean.shape != (F,) or std.shape != (F,):
        raise ValueError("mean/std must have F entries")
    count = starts.shape[0]
    if out is None:
        x = np.empty((count, P, N, F), dtype=np.float32)
        y = np.empty((count, Q, N, F), dtype=np.float32)
    else:
        bx, by = out
        for b, steps in ((bx, P), (by, Q)):
            if b.dtype != np.float32 or not b.flags.c_contiguous or b.size < count * steps * N * F:
                raise ValueError("out buffers must be C-contiguous float32 with room for the batch")
        x = bx.reshape(-1)[:count * P * N * F].reshape(count, P, N, F)
        y = by.reshape(-1)[:count * Q * N * F].reshape(count, Q, N, F)
    _check(_load().oracle_build_batch(_ptr(series), storage, T, N, F, P, Q, _ptr(mean), _ptr(std),
                                      _ptr(starts), count, _ptr(x), _ptr(y)), "build_batch")
    return x, y


def build_batch_bf16_out(series: np.ndarray, storage: int, P: int, Q: int, mean, std,
                         starts, out=None) -> tuple[np.ndarray, np.ndarray]:
    """Like build_batch, outputs as uint16 bf16 bit patterns (`out` buffers are uint16 then)."""
    want = np.float32 if storage == F32 else np.uint16
    if series.dtype != want or not series.flags.c_contiguous or series.ndim != 3:
        raise ValueError("series must be a C-contiguous [T,N,F] array of the storage dtype")
    T, N, F = series.shape
    mean, std = _c(mean, np.float32), _c(std, np.float32)
    starts = _c(starts, np.int32)
    count = starts.shape[0]
    if out is None:
        x = np.empty((count, P, N, F), dtype=np.uint16)
        y = np.empty((count, Q, N, F), dtype=np.uint16)
    else:
        bx, by = out
        for b, steps in ((bx, P), (by, Q)):
            if b.dtype != np.uint16 or not b.flags.c_contiguous or b.size < count * steps * N * F:
                raise ValueError("out buffers must be C-contiguous uint16 with room for the batch")
        x = bx.reshape(-1)[:count * P * N * F].reshape(count, P, N, F)
        y = by.reshape(-1)[:count * Q * N * F].reshape(count, Q, N, F)
    _check(_load().oracle_build_batch_bf16_out(_ptr(series), storage, T, N, F, P, Q, _ptr(mean), _ptr(std),
                                               _ptr(starts), count, _ptr(x), _ptr(y)), "build_batch_bf16_out")
    return x, y


def alg1_preprocess(data: np.ndarray, P: int, Q: int, mean, std) -> tuple[np.ndarray, np.ndarray]:
    data = _c(data, np.float32)
    T, N, F = data.shape
    n = window_count(T, P, Q)
    mean, std = _c(mean, np.float32), _c(std, np.float32)
    x = np.empty((n, P, N, F), dtype=np.float32)
    y = np.empty((n, Q, N, F), dtype=np.float32)
    _check(_load().oracle_alg1_preprocess(_ptr(data), T, N, F, P, Q, _ptr(mean), _ptr(std),
                                          _ptr(x), _ptr(y)), "alg1_preprocess")
    return x, y


def alg1_train_stats(data: np.ndarray, P: int, Q: int) -> tuple[float, float]:
    data = _c(data, np.float32)
    T, N, F = data.shape
    m, s = ctypes.c_double(), ctypes.c_double()
    _check(_load().oracle_alg1_train_stats(_ptr(data), T, N, F, P, Q, ctypes.byref(m),
                                           ctypes.byref(s)), "alg1_train_stats")
    return float(m.value), float(s.value)


def alg1_train_stats_fraction(data: np.ndarray, P: int, Q: int, fraction: float) -> tuple[float, float]:
    data = _c(data, np.float32)
    T, N, F = data.shape
    m, s = ctypes.c_double(), ctypes.c_double()
    _check(_load().oracle_alg1_train_stats_fraction(_ptr(data), T, N, F, P, Q, fraction, ctypes.byref(m),
                                                    ctypes.byref(s)), "alg1_train_stats_fraction")
    return float(m.value), float(s.value)


def add_time_of_day(data: np.ndarray, period: int) -> np.ndarray:
    """[T,N,F] -> [T,N,F+1] with the time-of-day channel (t mod period)/period appended."""
    data = _c(data, np.float32)
    T, N, F = data.shape
    out = np.empty((T, N, F + 1), dtype=np.float32)
    _check(_load().oracle_add_time_of_day(_ptr(data), T, N, F, period, _ptr(out)), "add_time_of_day")
    return out


def series_stats(data: np.ndarray) -> tuple[np.ndarray, np.ndarray]:
    data = _c(data, np.float32)
    T, N, F = data.shape
    mean = np.empty(F, dtype=np.float32)
    std = np.empty(F, dtype=np.float32)
    _check(_load().oracle_series_stats(_ptr(data), T, N, F, _ptr(mean), _ptr(std)), "series_stats")
    return mean, std
