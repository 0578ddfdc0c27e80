"""ctypes binding of include/a3gnn_cpu.h: the multi-threaded host sampler (argument marshalling
only).  Chosen explicitly by the caller; the GPU path never uses it."""
import ctypes as C
from typing import Optional, Sequence

import numpy as np

from .binding import A3Error, HostBlocks, lib

A3CPU_MAX_HOPS = 8


class _CpuBlocks(C.Structure):
    _fields_ = [
        ("num_hops", C.c_int32),
        ("n_dst", C.c_int64 * A3CPU_MAX_HOPS),
        ("n_src", C.c_int64 * A3CPU_MAX_HOPS),
        ("n_edges", C.c_int64 * A3CPU_MAX_HOPS),
        ("blk_indptr", C.c_void_p * A3CPU_MAX_HOPS),
        ("blk_indices", C.c_void_p * A3CPU_MAX_HOPS),
        ("blk_eids", C.c_void_p * A3CPU_MAX_HOPS),
        ("input_nodes", C.c_void_p),
    ]


_typed = False


def _lib():
    global _typed
    L = lib()
    if not _typed:
        L.a3cpu_create.argtypes = [C.POINTER(C.c_void_p), C.c_int]
        L.a3cpu_create.restype = C.c_int
        L.a3cpu_destroy.argtypes = [C.c_void_p]
        L.a3cpu_destroy.restype = C.c_int
        L.a3cpu_workers.argtypes = [C.c_void_p]
        L.a3cpu_workers.restype = C.c_int
        L.a3cpu_last_error.argtypes = [C.c_void_p]
        L.a3cpu_last_error.restype = C.c_char_p
        L.a3cpu_sample_blocks.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int64,
                                          C.c_void_p, C.c_int64, C.POINTER(C.c_int32), C.c_int32,
                                          C.c_void_p, C.c_uint32, C.c_uint64, C.POINTER(_CpuBlocks)]
        L.a3cpu_sample_blocks.restype = C.c_int
        L.a3cpu_check_vector_forms.argtypes = [C.POINTER(C.c_int)]
        L.a3cpu_check_vector_forms.restype = C.c_int
        L.a3cpu_set_vector_form.argtypes = [C.c_int]
        L.a3cpu_set_vector_form.restype = C.c_int
        L.a3cpu_set_first_bar_percent.argtypes = [C.c_int]
        L.a3cpu_set_first_bar_percent.restype = C.c_int
        _typed = True
    return L


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else C.c_void_p(a.ctypes.data)


def _copy(p, n, dtype):
    if n == 0 or not p:
        return np.zeros(0, dtype=dtype)
    return np.ctypeslib.as_array(C.cast(p, C.POINTER(np.ctypeslib.as_ctypes_type(dtype))), shape=(n,)).copy()


def check_vector_forms():
    """(cases in which a vector form of the draws differs from the scalar form, vector forms run)"""
    n = C.c_int(0)
    return _lib().a3cpu_check_vector_forms(C.byref(n)), n.value


def set_vector_form(form: int) -> bool:
    """0 = widest available, 1 = scalar, 2 = AVX2, 3 = AVX-512; False if this CPU lacks the form"""
    return _lib().a3cpu_set_vector_form(form) == 0


def set_first_bar_percent(percent: int) -> bool:
    """expected number of draws that clear the one-class scan's fixed bar, in percent of 2 m + 12"""
    return _lib().a3cpu_set_first_bar_percent(percent) == 0


class CpuSampler:
    """An a3cpu_sampler with n_workers threads (0 = one per hardware thread)."""

    def __init__(self, n_workers: int = 0):
        self._h = C.c_void_p()
        rc = _lib().a3cpu_create(C.byref(self._h), n_workers)
        if rc != 0:
            raise A3Error(rc, (_lib().a3cpu_last_error(None) or b"").decode())
        self.n_workers = _lib().a3cpu_workers(self._h)

    def close(self):
        if self._h:
            _lib().a3cpu_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def sample_blocks(self, indptr: np.ndarray, indices: np.ndarray, seeds: np.ndarray,
                      fanouts: Sequence[int], cache_map: Optional[np.ndarray] = None,
                      bias_q16: int = 65536, rng_seed: int = 0) -> HostBlocks:
        assert indptr.dtype == np.int64 and indptr.flags.c_contiguous
        assert indices.dtype in (np.int32, np.int64) and indices.flags.c_contiguous
        seeds = np.ascontiguousarray(seeds, dtype=indices.dtype)
        assert cache_map is None or (cache_map.dtype == np.int32 and cache_map.flags.c_contiguous)
        fan = (C.c_int32 * len(fanouts))(*fanouts)
        cb = _CpuBlocks()
        rc = _lib().a3cpu_sample_blocks(self._h, _ptr(indptr), _ptr(indices), indices.dtype.itemsize,
                                        indptr.shape[0] - 1, _ptr(seeds), seeds.shape[0], fan,
                                        len(fanouts), _ptr(cache_map), bias_q16, rng_seed, C.byref(cb))
        if rc != 0:
            raise A3Error(rc, (_lib().a3cpu_last_error(self._h) or b"").decode())
        H = cb.num_hops
        return HostBlocks(H, list(cb.n_dst[:H]), list(cb.n_src[:H]), list(cb.n_edges[:H]),
                          [_copy(cb.blk_indptr[h], cb.n_dst[h] + 1, np.int32) for h in range(H)],
                          [_copy(cb.blk_indices[h], cb.n_edges[h], np.int32) for h in range(H)],
                          [_copy(cb.blk_eids[h], cb.n_edges[h], np.int64) for h in range(H)],
                          _copy(cb.input_nodes, cb.n_src[H - 1], indices.dtype))
