"""ctypes binding of libadacons.so -- argument marshalling only.

Every step of the aggregation runs in the library's HIP kernels; this module turns
torch tensors into (device pointer, size) pairs and status codes into exceptions.
The functions carry the names of the C entry points in ``include/adacons.h``.
There is no CPU fallback: without the built library, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np
import torch

from . import build as _build

ADACONS_N_MAX = 128
ADACONS_GRAM_N_MAX = 64
ADACONS_F32, ADACONS_BF16 = 0, 1
ADACONS_OK, ADACONS_EINVAL, ADACONS_EUNSUPPORTED, ADACONS_EALIGN, ADACONS_EHIP, ADACONS_ENOMEM = 0, 1, 2, 3, 4, 5
ADACONS_FLAG_MOMENTUM, ADACONS_FLAG_NORMALIZE, ADACONS_FLAG_DEFAULT = 1, 2, 3
ADACONS_FLAG_INDEX_EMA, ADACONS_FLAG_LAMBDA_EQ13 = 4, 8
ADACONS_NUM_ZERO_NORM, ADACONS_NUM_NONFINITE, ADACONS_NUM_UNIFORM_FALLBACK = 1, 2, 4
ADACONS_TUNE_GRAM_BLOCKS_PER_CU = 0
ADACONS_TUNE_WSUM_BLOCKS_PER_CU = 1
ADACONS_TUNE_CACHED_HEAD_MB = 2
ADACONS_TUNE_GRAM_PRODUCTS = 3
ADACONS_TUNE_STATS_ONLY = 4
ADACONS_TUNE_WSUM_PARK_KB = 5
ADACONS_TUNE_SHORT_PATH = 6
ADACONS_TUNE_WSUM_ROW_SLICES = 7

EXPORTS = [
    "adacons_init_state", "adacons_destroy_state", "adacons_reset_state", "adacons_aggregate",
    "adacons_coeffs", "adacons_gram", "adacons_read_gram", "adacons_weighted_sum",
    "adacons_state_export", "adacons_state_import", "adacons_tune", "adacons_profile_begin",
    "adacons_profile_end", "adacons_status_string", "adacons_last_error",
    "adacons_aggregate_apply", "adacons_worker_stats", "adacons_update_from_stats", "adacons_worker_scale",
    "adacons_init_layers", "adacons_destroy_layers", "adacons_aggregate_layers", "adacons_layer_coeffs",
    "adacons_aggregate_noalloc",
]


class AdaConsError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = _lib.adacons_last_error().decode() if _lib is not None else ""
        name = _lib.adacons_status_string(status).decode() if _lib is not None else str(status)
        super().__init__(f"{where}: {name} ({msg})")


def _load() -> ctypes.CDLL:
    path = _build.LIB_PATH
    if not os.path.exists(path):
        _build.build_library()          # nothing built yet: build once, loudly
    lib = ctypes.CDLL(path)
    vp, i32, i64, dbl, u32 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_double, ctypes.c_uint
    dp = ctypes.POINTER(ctypes.c_double)
    sig = {
        "adacons_init_state": [ctypes.POINTER(vp), i32, i64, dbl, u32, vp],
        "adacons_destroy_state": [vp],
        "adacons_reset_state": [vp, vp],
        "adacons_aggregate": [vp, i32, i64, i32, vp, vp, vp],
        "adacons_aggregate_apply": [vp, i32, i64, i32, vp, vp, ctypes.c_float, vp],
        "adacons_aggregate_noalloc": [vp, i32, i64, i32, dbl, u32, vp, vp, vp, vp, vp],
        "adacons_worker_stats": [vp, vp, i64, i32, vp, vp, vp],
        "adacons_update_from_stats": [vp, dp, dp, vp],
        "adacons_worker_scale": [vp, i64, i32, vp, i32, vp],
        "adacons_coeffs": [vp, dp, dp, dp, ctypes.POINTER(ctypes.c_uint32), vp],
        "adacons_gram": [vp, i32, i64, i32, vp, vp],
        "adacons_read_gram": [vp, dp, vp],
        "adacons_weighted_sum": [vp, i32, i64, i32, dp, vp, vp, vp],
        "adacons_state_export": [vp, dp, ctypes.POINTER(i64), vp],
        "adacons_state_import": [vp, dp, i64, vp],
        "adacons_tune": [vp, i32, i32],
        "adacons_profile_begin": [vp, i32],
        "adacons_profile_end": [vp, dp, dp, dp, ctypes.POINTER(i32), vp],
        "adacons_init_layers": [ctypes.POINTER(vp), i32, i32, ctypes.POINTER(i64), i32, dbl, u32, vp],
        "adacons_destroy_layers": [vp],
        "adacons_aggregate_layers": [vp, i32, i64, i32, vp, vp, vp],
        "adacons_layer_coeffs": [vp, dp, dp, dp, ctypes.POINTER(ctypes.c_uint32), vp],
    }
    for name, args in sig.items():
        fn = getattr(lib, name)
        fn.argtypes = args
        fn.restype = ctypes.c_int
    lib.adacons_status_string.argtypes = [ctypes.c_int]
    lib.adacons_status_string.restype = ctypes.c_char_p
    lib.adacons_last_error.argtypes = []
    lib.adacons_last_error.restype = ctypes.c_char_p
    return lib


_lib = None
_lib = _load()


def library_path() -> str:
    return _build.LIB_PATH


def _check(rc: int, where: str) -> None:
    if rc != ADACONS_OK:
        raise AdaConsError(rc, where)


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, torch.cuda.Stream):
        return ctypes.c_void_p(stream.cuda_stream)
    return ctypes.c_void_p(int(stream))


def _matrix(G: torch.Tensor):
    """(pointer, N, d, dtype code) of a contiguous N x d device tensor."""
    if G.dim() != 2 or not G.is_contiguous():
        raise ValueError("G must be a contiguous N x d tensor")
    if not G.is_cuda:
        raise ValueError("G must live in device memory (there is no CPU path)")
    if G.dtype == torch.float32:
        dt = ADACONS_F32
    elif G.dtype == torch.bfloat16:
        dt = ADACONS_BF16
    else:
        raise TypeError(f"unsupported dtype {G.dtype}")
    return ctypes.c_void_p(G.data_ptr()), int(G.shape[0]), int(G.shape[1]), dt


def _dptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


# ---- the C entry points, same names -------------------------------------------------------
def adacons_init_state(N: int, d_max: int, beta: float = 0.99, flags: int = ADACONS_FLAG_DEFAULT,
                       stream=None) -> ctypes.c_void_p:
    st = ctypes.c_void_p()
    _check(_lib.adacons_init_state(ctypes.byref(st), N, d_max, beta, flags, _stream(stream)), "adacons_init_state")
    return st


def adacons_destroy_state(st) -> None:
    _check(_lib.adacons_destroy_state(st), "adacons_destroy_state")


def adacons_reset_state(st, stream=None) -> None:
    _check(_lib.adacons_reset_state(st, _stream(stream)), "adacons_reset_state")


def adacons_aggregate(G: torch.Tensor, st, out: torch.Tensor, stream=None) -> None:
    g, N, d, dt = _matrix(G)
    if out.dtype != torch.float32 or not out.is_cuda or not out.is_contiguous() or out.numel() != d:
        raise ValueError("out must be a contiguous float32 device tensor of d elements")
    _check(_lib.adacons_aggregate(g, N, d, dt, st, ctypes.c_void_p(out.data_ptr()), _stream(stream)),
           "adacons_aggregate")


def adacons_aggregate_apply(G: torch.Tensor, st, w: torch.Tensor, lr: float, stream=None) -> None:
    g, N, d, dt = _matrix(G)
    if w.dtype != torch.float32 or not w.is_cuda or not w.is_contiguous() or w.numel() != d:
        raise ValueError("w must be a contiguous float32 device tensor of d elements")
    _check(_lib.adacons_aggregate_apply(g, N, d, dt, st, ctypes.c_void_p(w.data_ptr()), float(lr), _stream(stream)),
           "adacons_aggregate_apply")


def adacons_aggregate_noalloc(G: torch.Tensor, m: torch.Tensor, out: torch.Tensor, beta: float = 0.99,
                              flags: int = ADACONS_FLAG_DEFAULT, coeffs: torch.Tensor | None = None,
                              numeric_flags: torch.Tensor | None = None, stream=None) -> None:
    """m: N float64 on the device (the carried state, updated in place); coeffs: 3 N float64 on the
    device or None; numeric_flags: one int32 on the device or None."""
    g, N, d, dt = _matrix(G)
    if out.dtype != torch.float32 or not out.is_cuda or not out.is_contiguous() or out.numel() != d:
        raise ValueError("out must be a contiguous float32 device tensor of d elements")
    if m.dtype != torch.float64 or not m.is_cuda or not m.is_contiguous() or m.numel() != N:
        raise ValueError("m must be a contiguous float64 device tensor of N elements")
    if coeffs is not None and (coeffs.dtype != torch.float64 or not coeffs.is_cuda or not coeffs.is_contiguous()
                               or coeffs.numel() != 3 * N):
        raise ValueError("coeffs must be a contiguous float64 device tensor of 3 N elements")
    if numeric_flags is not None and (numeric_flags.dtype != torch.int32 or not numeric_flags.is_cuda
                                      or numeric_flags.numel() != 1):
        raise ValueError("numeric_flags must be a device tensor of one int32")
    _check(_lib.adacons_aggregate_noalloc(g, N, d, dt, float(beta), int(flags), ctypes.c_void_p(m.data_ptr()),
                                          ctypes.c_void_p(coeffs.data_ptr()) if coeffs is not None else None,
                                          ctypes.c_void_p(numeric_flags.data_ptr()) if numeric_flags is not None else None,
                                          ctypes.c_void_p(out.data_ptr()), _stream(stream)),
           "adacons_aggregate_noalloc")


def _vector(v: torch.Tensor):
    if v.dim() != 1 or not v.is_contiguous() or not v.is_cuda:
        raise ValueError("expected a contiguous 1-D device tensor")
    if v.dtype == torch.float32:
        return ctypes.c_void_p(v.data_ptr()), int(v.numel()), ADACONS_F32
    if v.dtype == torch.bfloat16:
        return ctypes.c_void_p(v.data_ptr()), int(v.numel()), ADACONS_BF16
    raise TypeError(f"unsupported dtype {v.dtype}")


def adacons_worker_stats(g: torch.Tensor, gsum: torch.Tensor, st, stats: torch.Tensor, stream=None) -> None:
    pg, d, dt = _vector(g)
    ps, d2, dt2 = _vector(gsum)
    if d != d2 or dt != dt2:
        raise ValueError("g and gsum must have the same length and dtype")
    if stats.dtype != torch.float64 or not stats.is_cuda or stats.numel() != 3 or not stats.is_contiguous():
        raise ValueError("stats must be a device tensor of 3 float64")
    _check(_lib.adacons_worker_stats(pg, ps, d, dt, st, ctypes.c_void_p(stats.data_ptr()), _stream(stream)),
           "adacons_worker_stats")


def adacons_update_from_stats(st, sq, dot, stream=None) -> None:
    sq = np.ascontiguousarray(sq, dtype=np.float64)
    dot = np.ascontiguousarray(dot, dtype=np.float64)
    if sq.shape != dot.shape or sq.ndim != 1:
        raise ValueError("sq and dot must be vectors of N entries")
    _check(_lib.adacons_update_from_stats(st, _dptr(sq), _dptr(dot), _stream(stream)), "adacons_update_from_stats")


def adacons_worker_scale(g: torch.Tensor, st, worker: int, stream=None) -> None:
    pg, d, dt = _vector(g)
    _check(_lib.adacons_worker_scale(pg, d, dt, st, int(worker), _stream(stream)), "adacons_worker_scale")


def adacons_coeffs(st, N: int, stream=None) -> dict:
    gamma, raw, smooth = np.empty(N), np.empty(N), np.empty(N)
    nf = ctypes.c_uint32(0)
    _check(_lib.adacons_coeffs(st, _dptr(gamma), _dptr(raw), _dptr(smooth), ctypes.byref(nf), _stream(stream)),
           "adacons_coeffs")
    return {"gamma": gamma, "raw": raw, "smoothed": smooth, "numeric_flags": int(nf.value)}


def adacons_gram(G: torch.Tensor, st, stream=None) -> None:
    g, N, d, dt = _matrix(G)
    _check(_lib.adacons_gram(g, N, d, dt, st, _stream(stream)), "adacons_gram")


def adacons_read_gram(st, N: int, stream=None) -> np.ndarray:
    K = np.empty((N, N))
    _check(_lib.adacons_read_gram(st, _dptr(K), _stream(stream)), "adacons_read_gram")
    return K


def adacons_weighted_sum(G: torch.Tensor, gamma, st, out: torch.Tensor, stream=None) -> None:
    g, N, d, dt = _matrix(G)
    gam = np.ascontiguousarray(gamma, dtype=np.float64)
    if gam.shape != (N,):
        raise ValueError("gamma must have N entries")
    if out.dtype != torch.float32 or not out.is_cuda or not out.is_contiguous() or out.numel() != d:
        raise ValueError("out must be a contiguous float32 device tensor of d elements")
    _check(_lib.adacons_weighted_sum(g, N, d, dt, _dptr(gam), st, ctypes.c_void_p(out.data_ptr()), _stream(stream)),
           "adacons_weighted_sum")


def adacons_state_export(st, N: int, stream=None):
    m = np.empty(N)
    step = ctypes.c_int64(0)
    _check(_lib.adacons_state_export(st, _dptr(m), ctypes.byref(step), _stream(stream)), "adacons_state_export")
    return m, int(step.value)


def adacons_state_import(st, m, step: int, stream=None) -> None:
    m = np.ascontiguousarray(m, dtype=np.float64)
    _check(_lib.adacons_state_import(st, _dptr(m), step, _stream(stream)), "adacons_state_import")


def adacons_tune(st, key: int, value: int) -> None:
    _check(_lib.adacons_tune(st, key, value), "adacons_tune")


def adacons_profile_begin(st, max_calls: int) -> None:
    _check(_lib.adacons_profile_begin(st, max_calls), "adacons_profile_begin")


def adacons_profile_end(st, stream=None) -> dict:
    g, c, w, n = ctypes.c_double(0), ctypes.c_double(0), ctypes.c_double(0), ctypes.c_int(0)
    _check(_lib.adacons_profile_end(st, ctypes.byref(g), ctypes.byref(c), ctypes.byref(w), ctypes.byref(n),
                                    _stream(stream)), "adacons_profile_end")
    return {"gram_ms": g.value, "coeff_ms": c.value, "wsum_ms": w.value, "calls": n.value}


def adacons_init_layers(N: int, offsets, dtype: int, beta: float = 0.99, flags: int = ADACONS_FLAG_DEFAULT,
                        stream=None) -> ctypes.c_void_p:
    off = np.ascontiguousarray(offsets, dtype=np.int64)
    ls = ctypes.c_void_p()
    _check(_lib.adacons_init_layers(ctypes.byref(ls), N, off.shape[0] - 1,
                                    off.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), dtype, beta, flags,
                                    _stream(stream)), "adacons_init_layers")
    return ls


def adacons_destroy_layers(ls) -> None:
    _check(_lib.adacons_destroy_layers(ls), "adacons_destroy_layers")


def adacons_aggregate_layers(G: torch.Tensor, ls, out: torch.Tensor, stream=None) -> None:
    g, N, d, dt = _matrix(G)
    if out.dtype != torch.float32 or not out.is_cuda or not out.is_contiguous() or out.numel() != d:
        raise ValueError("out must be a contiguous float32 device tensor of d elements")
    _check(_lib.adacons_aggregate_layers(g, N, d, dt, ls, ctypes.c_void_p(out.data_ptr()), _stream(stream)),
           "adacons_aggregate_layers")


def adacons_layer_coeffs(ls, N: int, L: int, stream=None) -> dict:
    gamma, raw, smooth = np.empty((L, N)), np.empty((L, N)), np.empty((L, N))
    nf = np.zeros(L, dtype=np.uint32)
    _check(_lib.adacons_layer_coeffs(ls, _dptr(gamma), _dptr(raw), _dptr(smooth),
                                     nf.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)), _stream(stream)),
           "adacons_layer_coeffs")
    return {"gamma": gamma, "raw": raw, "smoothed": smooth, "numeric_flags": nf}


# ---- small convenience wrappers that own a state ------------------------------------------
class AdaConsLayers:
    """Layer-wise aggregation: one coefficient stream per contiguous column segment."""

    def __init__(self, N: int, offsets, dtype: torch.dtype = torch.float32, beta: float = 0.99,
                 flags: int = ADACONS_FLAG_DEFAULT, stream=None):
        self.N = int(N)
        self.offsets = np.ascontiguousarray(offsets, dtype=np.int64)
        self.L = int(self.offsets.shape[0] - 1)
        dt = ADACONS_BF16 if dtype == torch.bfloat16 else ADACONS_F32
        self._ls = adacons_init_layers(self.N, self.offsets, dt, beta, flags, stream)

    def close(self) -> None:
        if getattr(self, "_ls", None):
            adacons_destroy_layers(self._ls)
            self._ls = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def aggregate(self, G: torch.Tensor, out: torch.Tensor | None = None, stream=None) -> torch.Tensor:
        if out is None:
            out = torch.empty(G.shape[1], dtype=torch.float32, device=G.device)
        adacons_aggregate_layers(G, self._ls, out, stream)
        return out

    def coeffs(self, stream=None) -> dict:
        return adacons_layer_coeffs(self._ls, self.N, self.L, stream)



class AdaCons:
    """One coefficient stream (Eq. 11 state) for N workers; thin owner of an adacons_state."""

    def __init__(self, N: int, d_max: int, beta: float = 0.99, flags: int = ADACONS_FLAG_DEFAULT, stream=None):
        self.N, self.d_max = int(N), int(d_max)
        self._st = adacons_init_state(self.N, self.d_max, beta, flags, stream)

    def close(self) -> None:
        if getattr(self, "_st", None):
            adacons_destroy_state(self._st)
            self._st = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def aggregate(self, G: torch.Tensor, out: torch.Tensor | None = None, stream=None) -> torch.Tensor:
        if out is None:
            out = torch.empty(G.shape[1], dtype=torch.float32, device=G.device)
        adacons_aggregate(G, self._st, out, stream)
        return out

    def aggregate_apply(self, G: torch.Tensor, w: torch.Tensor, lr: float, stream=None) -> torch.Tensor:
        adacons_aggregate_apply(G, self._st, w, lr, stream)
        return w

    def coeffs(self, stream=None) -> dict:
        return adacons_coeffs(self._st, self.N, stream)

    def worker_stats(self, g: torch.Tensor, gsum: torch.Tensor, stream=None) -> torch.Tensor:
        stats = torch.empty(3, dtype=torch.float64, device=g.device)
        adacons_worker_stats(g, gsum, self._st, stats, stream)
        return stats

    def update_from_stats(self, sq, dot, stream=None) -> None:
        if len(sq) != self.N or len(dot) != self.N:
            raise ValueError("one pair per worker")
        adacons_update_from_stats(self._st, sq, dot, stream)

    def worker_scale(self, g: torch.Tensor, worker: int, stream=None) -> torch.Tensor:
        adacons_worker_scale(g, self._st, worker, stream)
        return g

    def gram(self, G: torch.Tensor, stream=None) -> np.ndarray:
        adacons_gram(G, self._st, stream)
        return adacons_read_gram(self._st, self.N, stream)

    def weighted_sum(self, G: torch.Tensor, gamma, out: torch.Tensor | None = None, stream=None) -> torch.Tensor:
        if out is None:
            out = torch.empty(G.shape[1], dtype=torch.float32, device=G.device)
        adacons_weighted_sum(G, gamma, self._st, out, stream)
        return out

    def reset(self, stream=None) -> None:
        adacons_reset_state(self._st, stream)

    def export_state(self, stream=None):
        return adacons_state_export(self._st, self.N, stream)

    def import_state(self, m, step: int, stream=None) -> None:
        adacons_state_import(self._st, m, step, stream)

    def tune(self, key: int, value: int) -> None:
        adacons_tune(self._st, key, value)

    def profile_begin(self, max_calls: int) -> None:
        adacons_profile_begin(self._st, max_calls)

    def profile_end(self, stream=None) -> dict:
        return adacons_profile_end(self._st, stream)
