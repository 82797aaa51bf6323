"""Python binding of the C-ABI index-batching library (include/pgti.h).

Argument marshalling only: every step of the path (resident store, epoch index generation,
batch build) runs in the HIP kernels behind the C calls.  PyTorch is used for device memory
(`tensor.data_ptr()`) and streams (`torch.cuda.current_stream().cuda_stream`), nothing else.
There is no CPU fallback: if libpgti.so is missing or cannot be loaded this module raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np
import torch  # imported before the library so that both share one HIP runtime in the process

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libpgti.so")

PGTI_F32, PGTI_BF16 = 0, 1
PGTI_OK, PGTI_ERR_ARG, PGTI_ERR_STATE, PGTI_ERR_RANGE = 0, -1, -2, -3
PGTI_ERR_STATS, PGTI_ERR_OOM, PGTI_ERR_HIP = -4, -5, -6
_STATUS_NAMES = {-1: "PGTI_ERR_ARG", -2: "PGTI_ERR_STATE", -3: "PGTI_ERR_RANGE",
                 -4: "PGTI_ERR_STATS", -5: "PGTI_ERR_OOM", -6: "PGTI_ERR_HIP"}

# name -> (restype, argtypes): every symbol include/pgti.h declares
_vp, _i64, _i32, _u64, _u32 = (ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_uint64,
                               ctypes.c_uint32)
SIGNATURES = {
    "pgti_create": (ctypes.c_int, [ctypes.POINTER(_vp), ctypes.c_int]),
    "pgti_destroy": (None, [_vp]),
    "pgti_set_sort_test_hooks": (ctypes.c_int, [_vp, _u32, _u32]),
    "pgti_load_series": (ctypes.c_int, [_vp, _vp, _i64, _i32, _i32, _i32, _i32, _i32, ctypes.c_int, _vp, _vp]),
    "pgti_load_series_device": (ctypes.c_int, [_vp, _vp, _i64, _i32, _i32, _i32, _i32, _i32, ctypes.c_int, _vp, _vp]),
    "pgti_get_stats": (ctypes.c_int, [_vp, _vp, _vp]),
    "pgti_epoch_indices": (ctypes.c_int, [_vp, _u64, _u64, _u32, _u32, ctypes.POINTER(_i64)]),
    "pgti_epoch_indices_static": (_i64, [ctypes.c_int, _i64, _u64, _u64, _u32, _u32, _vp, _i64, _vp]),
    "pgti_get_indices": (_i64, [_vp, _vp, _i64]),
    "pgti_num_batches": (_i64, [_vp]),
    "pgti_build_batch": (ctypes.c_int, [_vp, _i64, _vp, _vp, _vp]),
    "pgti_build_batches": (_i64, [_vp, _i64, _i32, _vp, _vp, _vp]),
    "pgti_build_batches_bf16": (_i64, [_vp, _i64, _i32, _vp, _vp, _vp]),
    "pgti_last_error": (ctypes.c_char_p, []),
}

PGTI_ORDER_SHUFFLE, PGTI_ORDER_SEQUENTIAL, PGTI_ORDER_BATCH_SHUFFLE = 0, 1, 2


class EpochSpec(ctypes.Structure):
    """Mirror of pgti_epoch_spec."""
    _fields_ = [("order", _i32), ("reserved", _i32), ("first_start", _i64), ("n_starts", _i64),
                ("seed", _u64), ("epoch", _u64), ("rank", _u32), ("world", _u32)]


PGTI_STATS_GIVEN, PGTI_STATS_FEATURE_GLOBAL, PGTI_STATS_ALG1_TRAIN = 0, 1, 2


class LoadSpec(ctypes.Structure):
    """Mirror of pgti_load_spec."""
    _fields_ = [("T", _i64), ("N", _i32), ("F_in", _i32), ("P", _i32), ("Q", _i32), ("B", _i32),
                ("storage", _i32), ("source_on_device", _i32), ("stats_rule", _i32),
                ("time_of_day_period", _i32), ("reserved", _i32), ("train_fraction", ctypes.c_double),
                ("mean", _vp), ("std", _vp)]


SIGNATURES["pgti_load_series_ex"] = (ctypes.c_int, [_vp, _vp, ctypes.POINTER(LoadSpec)])
SIGNATURES["pgti_epoch_indices_ex"] = (ctypes.c_int, [_vp, ctypes.POINTER(EpochSpec), ctypes.POINTER(_i64)])

_lib = None


class PgtiError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{_STATUS_NAMES.get(status, status)}: {message}")
        self.status = status


def load_library() -> ctypes.CDLL:
    """Loads libpgti.so (built in-tree by paper_2507_11683_amd/build.py).  Fails loudly."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2507_11683_amd.build` "
                              "(or __graft_entry__.build()) first; there is no fallback path")
        lib = ctypes.CDLL(LIB_PATH)
        for name, (restype, argtypes) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = restype
            fn.argtypes = argtypes
        _lib = lib
    return _lib


def _check(rc: int) -> int:
    if rc < 0:
        raise PgtiError(int(rc), load_library().pgti_last_error().decode())
    return int(rc)


def _stats_ptrs(mean, std, F: int):
    if mean is None and std is None:
        return None, None, None
    if mean is None or std is None:
        raise PgtiError(PGTI_ERR_ARG, "pass both mean and std, or neither")
    m = np.ascontiguousarray(mean, dtype=np.float32)
    s = np.ascontiguousarray(std, dtype=np.float32)
    if m.shape != (F,) or s.shape != (F,):
        raise PgtiError(PGTI_ERR_ARG, f"mean/std must have F={F} entries")
    return m.ctypes.data, s.ctypes.data, (m, s)


def _stream_handle(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream
    return int(stream)


class Context:
    """One resident series on one GPU; methods carry the names of the C calls."""

    def __init__(self, device: int = 0):
        self._h = _vp()
        self._lib = load_library()
        _check(self._lib.pgti_create(ctypes.byref(self._h), device))
        self.device = device
        self.shape = None

    # -- pgti_destroy -------------------------------------------------------------------------
    def destroy(self) -> None:
        if self._h:
            self._lib.pgti_destroy(self._h)
            self._h = _vp()

    close = destroy

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.destroy()

    # -- pgti_set_sort_test_hooks ------------------------------------------------------------------
    def set_sort_test_hooks(self, bucket_cap: int = 0, key_bits: int = 0) -> None:
        _check(self._lib.pgti_set_sort_test_hooks(self._h, bucket_cap, key_bits))

    # -- pgti_load_series / pgti_load_series_device ----------------------------------------------
    def load_series(self, series, P: int, Q: int, B: int, storage: int = PGTI_F32, mean=None,
                    std=None) -> None:
        """series: fp32 [T, N, F], a numpy array / CPU tensor (pinned or not) or a CUDA tensor."""
        if isinstance(series, torch.Tensor):
            if series.dtype != torch.float32 or not series.is_contiguous() or series.dim() != 3:
                raise PgtiError(PGTI_ERR_ARG, "series must be a contiguous float32 [T, N, F] tensor")
            T, N, F = series.shape
            ptr, on_device = series.data_ptr(), series.is_cuda
        else:
            if series.dtype != np.float32 or not series.flags.c_contiguous or series.ndim != 3:
                raise PgtiError(PGTI_ERR_ARG, "series must be a C-contiguous float32 [T, N, F] array")
            T, N, F = series.shape
            ptr, on_device = series.ctypes.data, False
        mp, sp, _keep = _stats_ptrs(mean, std, F)
        fn = self._lib.pgti_load_series_device if on_device else self._lib.pgti_load_series
        _check(fn(self._h, ptr, T, N, F, P, Q, B, storage, mp, sp))
        self.shape = (T, N, F, P, Q, B)

    # -- pgti_load_series_ex ----------------------------------------------------------------------
    def load_series_ex(self, series, P: int, Q: int, B: int, storage: int = PGTI_F32,
                       stats_rule: int = PGTI_STATS_FEATURE_GLOBAL, time_of_day_period: int = 0,
                       train_fraction: float = 0.70, mean=None, std=None) -> None:
        """Load with on-device preprocessing: optional time-of-day feature and computed statistics."""
        if isinstance(series, torch.Tensor):
            if series.dtype != torch.float32 or not series.is_contiguous() or series.dim() != 3:
                raise PgtiError(PGTI_ERR_ARG, "series must be a contiguous float32 [T, N, F] tensor")
            T, N, F_in = series.shape
            ptr, on_device = series.data_ptr(), series.is_cuda
        else:
            if series.dtype != np.float32 or not series.flags.c_contiguous or series.ndim != 3:
                raise PgtiError(PGTI_ERR_ARG, "series must be a C-contiguous float32 [T, N, F] array")
            T, N, F_in = series.shape
            ptr, on_device = series.ctypes.data, False
        F = F_in + (1 if time_of_day_period > 0 else 0)
        mp, sp, _keep = _stats_ptrs(mean, std, F)
        spec = LoadSpec(T, N, F_in, P, Q, B, storage, int(on_device), stats_rule, time_of_day_period, 0,
                        train_fraction, mp, sp)
        _check(self._lib.pgti_load_series_ex(self._h, ptr, ctypes.byref(spec)))
        self.shape = (T, N, F, P, Q, B)

    # -- pgti_get_stats ---------------------------------------------------------------------------
    def get_stats(self):
        F = self.shape[2]
        m, s = np.empty(F, np.float32), np.empty(F, np.float32)
        _check(self._lib.pgti_get_stats(self._h, m.ctypes.data, s.ctypes.data))
        return m, s

    # -- pgti_epoch_indices -----------------------------------------------------------------------
    def epoch_indices(self, seed: int, epoch: int, rank: int = 0, world: int = 1) -> int:
        n = _i64(0)
        _check(self._lib.pgti_epoch_indices(self._h, seed, epoch, rank, world, ctypes.byref(n)))
        return int(n.value)

    # -- pgti_epoch_indices_ex --------------------------------------------------------------------
    def epoch_indices_ex(self, order: int, seed: int = 0, epoch: int = 0, rank: int = 0, world: int = 1,
                         first_start: int = 0, n_starts: int = -1) -> int:
        spec = EpochSpec(order, 0, first_start, n_starts, seed, epoch, rank, world)
        n = _i64(0)
        _check(self._lib.pgti_epoch_indices_ex(self._h, ctypes.byref(spec), ctypes.byref(n)))
        return int(n.value)

    # -- pgti_get_indices -------------------------------------------------------------------------
    def get_indices(self) -> np.ndarray:
        cap = self.shape[0]
        out = np.empty(cap, dtype=np.int32)
        n = self._lib.pgti_get_indices(self._h, out.ctypes.data, cap)
        _check(n)
        return out[:n].copy()

    # -- pgti_num_batches -------------------------------------------------------------------------
    def num_batches(self) -> int:
        return _check(self._lib.pgti_num_batches(self._h))

    # -- pgti_build_batch -------------------------------------------------------------------------
    def build_batch(self, batch_no: int, out_x: torch.Tensor, out_y: torch.Tensor, stream=None) -> int:
        """Enqueues the batch on `stream` (default: torch's current stream); returns B'."""
        T, N, F, P, Q, B = self.shape
        for t, steps, name in ((out_x, P, "out_x"), (out_y, Q, "out_y")):
            if not (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()):
                raise PgtiError(PGTI_ERR_ARG, f"{name} must be a contiguous float32 CUDA tensor")
            if t.numel() < B * steps * N * F:
                raise PgtiError(PGTI_ERR_ARG, f"{name} holds fewer than B*{steps}*N*F elements")
        return _check(self._lib.pgti_build_batch(self._h, batch_no, out_x.data_ptr(), out_y.data_ptr(),
                                                 _stream_handle(stream)))

    # -- pgti_build_batches -----------------------------------------------------------------------
    def build_batches(self, first_batch: int, k: int, out_x: torch.Tensor, out_y: torch.Tensor,
                      stream=None) -> int:
        """k consecutive batches in one launch into out_x[k,B,P,N,F], out_y[k,B,Q,N,F]; returns the
        number of valid samples."""
        T, N, F, P, Q, B = self.shape
        for t, steps, name in ((out_x, P, "out_x"), (out_y, Q, "out_y")):
            if not (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()):
                raise PgtiError(PGTI_ERR_ARG, f"{name} must be a contiguous float32 CUDA tensor")
            if t.numel() < max(k, 0) * B * steps * N * F:
                raise PgtiError(PGTI_ERR_ARG, f"{name} holds fewer than k*B*{steps}*N*F elements")
        return _check(self._lib.pgti_build_batches(self._h, first_batch, k, out_x.data_ptr(),
                                                   out_y.data_ptr(), _stream_handle(stream)))

    # -- pgti_build_batches_bf16 ------------------------------------------------------------------
    def build_batches_bf16(self, first_batch: int, k: int, out_x: torch.Tensor, out_y: torch.Tensor,
                           stream=None) -> int:
        """Like build_batches with bfloat16 outputs out_x[k,B,P,N,F], out_y[k,B,Q,N,F]."""
        T, N, F, P, Q, B = self.shape
        for t, steps, name in ((out_x, P, "out_x"), (out_y, Q, "out_y")):
            if not (t.is_cuda and t.dtype == torch.bfloat16 and t.is_contiguous()):
                raise PgtiError(PGTI_ERR_ARG, f"{name} must be a contiguous bfloat16 CUDA tensor")
            if t.numel() < max(k, 0) * B * steps * N * F:
                raise PgtiError(PGTI_ERR_ARG, f"{name} holds fewer than k*B*{steps}*N*F elements")
        return _check(self._lib.pgti_build_batches_bf16(self._h, first_batch, k, out_x.data_ptr(),
                                                        out_y.data_ptr(), _stream_handle(stream)))

    def build_batches_bf16_raw(self, first_batch: int, k: int, x_ptr: int, y_ptr: int, stream_handle: int) -> int:
        return self._lib.pgti_build_batches_bf16(self._h, first_batch, k, x_ptr, y_ptr, stream_handle)

    def build_batches_raw(self, first_batch: int, k: int, x_ptr: int, y_ptr: int, stream_handle: int) -> int:
        return self._lib.pgti_build_batches(self._h, first_batch, k, x_ptr, y_ptr, stream_handle)

    def build_batch_raw(self, batch_no: int, x_ptr: int, y_ptr: int, stream_handle: int) -> int:
        """Same call with raw device addresses (no per-call tensor checks): for timed loops."""
        return self._lib.pgti_build_batch(self._h, batch_no, x_ptr, y_ptr, stream_handle)


PGTI_STATIC_MAX_WINDOWS = 1 << 20


def epoch_indices_static(n_windows: int, seed: int, epoch: int, rank: int, world: int,
                         share_out: torch.Tensor, stream=None, device: int = 0) -> int:
    """pgti_epoch_indices_static: the share of (seed, epoch, rank, world) over n_windows starts into the
    caller's int32 CUDA tensor, with no allocation anywhere in the call.  Returns the share length."""
    if not (share_out.is_cuda and share_out.dtype == torch.int32 and share_out.is_contiguous()):
        raise PgtiError(PGTI_ERR_ARG, "share_out must be a contiguous int32 CUDA tensor")
    return _check(load_library().pgti_epoch_indices_static(device, n_windows, seed, epoch, rank, world,
                                                           share_out.data_ptr(), share_out.numel(),
                                                           _stream_handle(stream)))


def last_error() -> str:
    return load_library().pgti_last_error().decode()
