"""ctypes marshalling for the CPU oracle (test infrastructure; no arithmetic here)."""
import ctypes as C
import os
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

from . import build as _build

MAX_HOPS = 8
_lib = None


class _Blocks(C.Structure):
    _fields_ = [
        ("num_hops", C.c_int32),
        ("n_dst", C.c_int64 * MAX_HOPS),
        ("n_src", C.c_int64 * MAX_HOPS),
        ("n_edges", C.c_int64 * MAX_HOPS),
        ("blk_indptr", C.POINTER(C.c_int32) * MAX_HOPS),
        ("blk_indices", C.POINTER(C.c_int32) * MAX_HOPS),
        ("blk_eids", C.POINTER(C.c_int64) * MAX_HOPS),
        ("input_nodes", C.POINTER(C.c_int64)),
        ("seconds_sample", C.c_double),
        ("seconds_relabel", C.c_double),
    ]


def lib():
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path):
            path = _build.build()
        L = C.CDLL(path)
        L.oracle_philox4x32_10.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        L.oracle_philox4x32_10.restype = None
        L.oracle_draw.argtypes = [C.c_uint64, C.c_uint32, C.c_uint64, C.c_uint64]
        L.oracle_draw.restype = C.c_uint32
        L.oracle_fixlog2_q32.argtypes = [C.c_uint64]
        L.oracle_fixlog2_q32.restype = C.c_uint64
        L.oracle_key.argtypes = [C.c_uint32, C.c_uint32]
        L.oracle_key.restype = C.c_uint64
        L.oracle_select.argtypes = [C.c_uint64, C.c_uint32, C.c_uint64, C.c_int64, C.c_int64,
                                    C.c_void_p, C.c_void_p]
        L.oracle_select.restype = C.c_int64
        L.oracle_sample_blocks.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_void_p,
                                           C.c_int64, C.c_void_p, C.c_int32, C.c_void_p, C.c_uint32,
                                           C.c_uint64, C.POINTER(_Blocks)]
        L.oracle_sample_blocks.restype = C.c_int
        L.oracle_free_blocks.argtypes = [C.POINTER(_Blocks)]
        L.oracle_free_blocks.restype = None
        L.oracle_block_mean.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_void_p,
                                        C.c_int32, C.c_int64, C.c_void_p]
        L.oracle_block_mean.restype = C.c_int
        L.oracle_count_accesses.argtypes = [C.c_void_p, C.c_int32, C.c_int64, C.c_int64, C.c_void_p]
        L.oracle_count_accesses.restype = C.c_int
        L.oracle_rank_cache.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p]
        L.oracle_rank_cache.restype = C.c_int
        L.oracle_cache_fifo_update.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_int64,
                                               C.c_void_p, C.c_int64, C.c_void_p, C.c_int32, C.c_int64,
                                               C.c_void_p]
        L.oracle_cache_fifo_update.restype = C.c_int64
        L.oracle_gather_features.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                             C.c_int32, C.c_int64, C.c_int64, C.c_void_p]
        L.oracle_gather_features.restype = C.c_int
        _lib = L
    return _lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def philox4x32_10(ctr, key_):
    c = np.asarray(ctr, dtype=np.uint32)
    k = np.asarray(key_, dtype=np.uint32)
    o = np.zeros(4, dtype=np.uint32)
    lib().oracle_philox4x32_10(_ptr(c), _ptr(k), _ptr(o))
    return [int(v) for v in o]


def draw(rng_seed: int, hop: int, node: int, slot: int) -> int:
    return int(lib().oracle_draw(rng_seed, hop, node, slot))


def fixlog2_q32(U: int) -> int:
    return int(lib().oracle_fixlog2_q32(U))


def key(x: int, w_q16: int) -> int:
    return int(lib().oracle_key(x, w_q16))


def select(rng_seed: int, hop: int, node: int, deg: int, fanout: int, weights_q16=None):
    w = None if weights_q16 is None else np.ascontiguousarray(weights_q16, dtype=np.uint32)
    if w is not None:
        assert w.shape == (deg,)
    chosen = np.zeros(max(min(deg, fanout), 1), dtype=np.int64)
    m = lib().oracle_select(rng_seed, hop, node, deg, fanout, _ptr(w), _ptr(chosen))
    return [int(s) for s in chosen[:m]]


@dataclass
class OracleBlocks:
    num_hops: int
    n_dst: List[int]
    n_src: List[int]
    n_edges: List[int]
    blk_indptr: List[np.ndarray] = field(default_factory=list)
    blk_indices: List[np.ndarray] = field(default_factory=list)
    blk_eids: List[np.ndarray] = field(default_factory=list)
    input_nodes: np.ndarray = None
    seconds_sample: float = 0.0
    seconds_relabel: float = 0.0


def _take(p, n, dtype):
    if n == 0:
        return np.zeros(0, dtype=dtype)
    return np.ctypeslib.as_array(p, shape=(n,)).astype(dtype, copy=True)


def sample_blocks(indptr, indices, seeds, fanouts, cache_map=None, bias_q16=65536, rng_seed=0):
    indptr = np.ascontiguousarray(indptr, dtype=np.int64)
    indices = np.ascontiguousarray(indices)
    assert indices.dtype in (np.int32, np.int64)
    seeds = np.ascontiguousarray(seeds, dtype=indices.dtype)
    fan = np.ascontiguousarray(fanouts, dtype=np.int32)
    cm = None if cache_map is None else np.ascontiguousarray(cache_map, dtype=np.int32)
    num_nodes = indptr.shape[0] - 1
    if cm is not None:
        assert cm.shape == (num_nodes,)
    b = _Blocks()
    rc = lib().oracle_sample_blocks(_ptr(indptr), _ptr(indices), indices.dtype.itemsize, num_nodes,
                                    _ptr(seeds), seeds.shape[0], _ptr(fan), fan.shape[0], _ptr(cm),
                                    bias_q16, rng_seed, C.byref(b))
    if rc != 0:
        lib().oracle_free_blocks(C.byref(b))
        raise ValueError("oracle_sample_blocks: bad argument")
    H = b.num_hops
    res = OracleBlocks(H, list(b.n_dst[:H]), list(b.n_src[:H]), list(b.n_edges[:H]))
    for h in range(H):
        res.blk_indptr.append(_take(b.blk_indptr[h], b.n_dst[h] + 1, np.int32))
        res.blk_indices.append(_take(b.blk_indices[h], b.n_edges[h], np.int32))
        res.blk_eids.append(_take(b.blk_eids[h], b.n_edges[h], np.int64))
    res.input_nodes = _take(b.input_nodes, b.n_src[H - 1], np.int64)
    res.seconds_sample = b.seconds_sample
    res.seconds_relabel = b.seconds_relabel
    lib().oracle_free_blocks(C.byref(b))
    return res


def gather_features(feat_dev, feat_host, cache_map, ids):
    ids = np.ascontiguousarray(ids)
    assert ids.dtype in (np.int32, np.int64)
    ref = feat_dev if feat_dev is not None else feat_host
    dim = ref.shape[1]
    row_bytes = dim * ref.dtype.itemsize
    fd = None if feat_dev is None else np.ascontiguousarray(feat_dev)
    fh = None if feat_host is None else np.ascontiguousarray(feat_host)
    cm = None if cache_map is None else np.ascontiguousarray(cache_map, dtype=np.int32)
    out = np.zeros((ids.shape[0], dim), dtype=ref.dtype)
    rc = lib().oracle_gather_features(_ptr(fd), _ptr(fh), _ptr(cm), _ptr(ids), ids.dtype.itemsize,
                                      ids.shape[0], row_bytes, _ptr(out))
    if rc != 0:
        raise ValueError("oracle_gather_features: bad argument")
    return out


def block_mean(blk_indptr, blk_indices, x):
    """mean of the source rows of every destination of one block, in double: [n_dst, dim]"""
    ip = np.ascontiguousarray(blk_indptr, dtype=np.int32)
    ix = np.ascontiguousarray(blk_indices, dtype=np.int32)
    x = np.ascontiguousarray(x)
    assert x.ndim == 2 and x.dtype in (np.float32, np.float16)
    n_dst = ip.shape[0] - 1
    out = np.zeros((n_dst, x.shape[1]), dtype=np.float64)
    rc = lib().oracle_block_mean(_ptr(ip), _ptr(ix), n_dst, x.shape[0], _ptr(x),
                                 0 if x.dtype == np.float32 else 1, x.shape[1], _ptr(out))
    if rc != 0:
        raise ValueError("oracle_block_mean: bad argument")
    return out


def count_accesses(ids, counts):
    """counts[id] += 1 for every id, in place (counts: uint32 [num_nodes])"""
    ids = np.ascontiguousarray(ids)
    assert ids.dtype in (np.int32, np.int64)
    assert counts.dtype == np.uint32 and counts.flags.c_contiguous
    rc = lib().oracle_count_accesses(_ptr(ids), ids.dtype.itemsize, ids.shape[0], counts.shape[0],
                                     _ptr(counts))
    if rc != 0:
        raise ValueError("oracle_count_accesses: bad argument")


def rank_cache(counts, n_cached):
    """(cache_map, order) of the static fill by access count"""
    counts = np.ascontiguousarray(counts, dtype=np.uint32)
    n = counts.shape[0]
    cache_map = np.zeros(n, dtype=np.int32)
    order = np.zeros(n, dtype=np.int32)
    rc = lib().oracle_rank_cache(_ptr(counts), n, n_cached, _ptr(cache_map), _ptr(order))
    if rc != 0:
        raise ValueError("oracle_rank_cache: bad argument")
    return cache_map, order


def cache_fifo_update(cache_map, slot_owner, head, feat_dev, ids, rows):
    """one mini-batch through the FIFO cache, in place; head is an int32 array of one element.
    Returns the number of misses."""
    ids = np.ascontiguousarray(ids)
    rows = np.ascontiguousarray(rows)
    assert cache_map.dtype == np.int32 and slot_owner.dtype == np.int32 and head.dtype == np.int32
    assert feat_dev.flags.c_contiguous and feat_dev.ndim == 2
    row_bytes = feat_dev.shape[1] * feat_dev.dtype.itemsize
    assert rows.size == 0 or rows.shape[1] * rows.dtype.itemsize == row_bytes
    m = lib().oracle_cache_fifo_update(_ptr(cache_map), cache_map.shape[0], _ptr(slot_owner),
                                       _ptr(head), slot_owner.shape[0], _ptr(feat_dev), row_bytes,
                                       _ptr(ids), ids.dtype.itemsize, ids.shape[0], _ptr(rows))
    if m < 0:
        raise ValueError("oracle_cache_fifo_update: bad argument")
    return int(m)
