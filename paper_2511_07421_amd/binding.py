"""ctypes binding of include/a3gnn.h: argument marshalling only.

The entry points keep their C names (lib().a3_create, ...); Context wraps them for torch
tensors.  There is no fallback: if the HIP library is missing, loading raises.
"""
import ctypes as C
import os
from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import torch

A3_MAX_HOPS = 8
A3_MAX_FANOUT = 1024
A3_OK, A3_ERR_INVALID_ARG, A3_ERR_CAPACITY, A3_ERR_HIP, A3_ERR_INPUT = 0, -1, -2, -3, -4
A3_VALIDATE, A3_NO_EIDS, A3_HOST_ONLY, A3_FORCE_RADIX, A3_PROFILE, A3_TEST_MAP_RANGE, A3_TEST_FEW_DRAWS, A3_TEST_SMALL_GRID = 1, 2, 4, 8, 16, 32, 64, 128
A3_PROFILE_RETRIEVE = 256
A3_STATIC_MAP = 512
A3_PROFILE_DEPTH = 256
A3_FIFO_STATIC_MAX_IDS = 1 << 22
A3_PIPE_SEQUENTIAL, A3_PIPE_MODE1, A3_PIPE_MODE2 = 0, 1, 2
A3_PIPE_MAX_WORKERS = 8
A3_F32, A3_F16 = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_lib = None


def library_path() -> str:
    return os.path.join(_HERE, "liba3gnn.so")


class _CBlocks(C.Structure):
    _fields_ = [
        ("num_hops", C.c_int32),
        ("n_dst", C.c_int64 * A3_MAX_HOPS),
        ("n_src", C.c_int64 * A3_MAX_HOPS),
        ("n_edges", C.c_int64 * A3_MAX_HOPS),
        ("blk_indptr", C.c_void_p * A3_MAX_HOPS),
        ("blk_indices", C.c_void_p * A3_MAX_HOPS),
        ("blk_eids", C.c_void_p * A3_MAX_HOPS),
        ("input_nodes", C.c_void_p),
    ]


def lib():
    """The loaded C-ABI library.  Built by `python -m paper_2511_07421_amd.build` (hipcc)."""
    global _lib
    if _lib is None:
        path = library_path()
        if not os.path.exists(path):
            from . import build as _build
            _build.build()
        L = C.CDLL(path)
        L.a3_create.argtypes = [C.POINTER(C.c_void_p), C.c_int, C.c_void_p, C.c_int64, C.c_int32,
                                C.POINTER(C.c_int32), C.c_uint32]
        L.a3_create.restype = C.c_int
        L.a3_destroy.argtypes = [C.c_void_p]
        L.a3_destroy.restype = C.c_int
        L.a3_set_stream.argtypes = [C.c_void_p, C.c_void_p]
        L.a3_set_stream.restype = C.c_int
        L.a3_validate_graph.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_int64]
        L.a3_validate_graph.restype = C.c_int
        L.a3_validate_cache_map.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64]
        L.a3_validate_cache_map.restype = C.c_int
        L.a3_set_gather_host_workgroups.argtypes = [C.c_void_p, C.c_int32]
        L.a3_set_gather_host_workgroups.restype = C.c_int
        L.a3_reserve.argtypes = [C.c_void_p, C.c_int64]
        L.a3_reserve.restype = C.c_int
        L.a3_device_map_changed.argtypes = [C.c_void_p]
        L.a3_device_map_changed.restype = C.c_int
        L.a3_pipeline_reserve.argtypes = [C.c_void_p, C.c_int64]
        L.a3_pipeline_reserve.restype = C.c_int
        L.a3_last_error.argtypes = [C.c_void_p]
        L.a3_last_error.restype = C.c_char_p
        L.a3_sample_blocks.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int64,
                                       C.c_void_p, C.c_int64, C.POINTER(C.c_int32), C.c_int32,
                                       C.c_void_p, C.c_uint32, C.c_uint64, C.POINTER(_CBlocks)]
        L.a3_sample_blocks.restype = C.c_int
        L.a3_gather_features.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                         C.c_int32, C.c_int64, C.c_int64, C.c_void_p]
        L.a3_gather_features.restype = C.c_int
        L.a3_sample_blocks_begin.argtypes = L.a3_sample_blocks.argtypes[:-1]
        L.a3_sample_blocks_begin.restype = C.c_int
        L.a3_sample_blocks_end.argtypes = [C.c_void_p, C.POINTER(_CBlocks)]
        L.a3_sample_blocks_end.restype = C.c_int
        L.a3_sample_gather_begin.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int64,
                                             C.c_void_p, C.c_int64, C.POINTER(C.c_int32), C.c_int32,
                                             C.c_void_p, C.c_uint32, C.c_uint64, C.c_void_p, C.c_int64,
                                             C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_int64, C.c_int64]
        L.a3_sample_gather_begin.restype = C.c_int
        L.a3_sample_stats.argtypes = [C.c_void_p, C.POINTER(C.c_int64)]
        L.a3_sample_stats.restype = C.c_int
        L.a3_gather_input_features.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                               C.c_int64, C.c_void_p, C.c_int64]
        L.a3_gather_input_features.restype = C.c_int
        L.a3_gather_features_strided.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64,
                                                 C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_int64,
                                                 C.c_void_p, C.c_int64]
        L.a3_gather_features_strided.restype = C.c_int
        L.a3_gather_input_features_strided.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p,
                                                       C.c_int64, C.c_void_p, C.c_int64, C.c_void_p,
                                                       C.c_int64, C.c_int64]
        L.a3_gather_input_features_strided.restype = C.c_int
        L.a3_profile_read.argtypes = [C.c_void_p, C.c_int, C.POINTER(C.c_float), C.c_int,
                                      C.POINTER(C.c_int)]
        L.a3_profile_read.restype = C.c_int
        L.a3_block_mean.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_void_p,
                                    C.c_int32, C.c_int64, C.c_void_p]
        L.a3_block_mean.restype = C.c_int
        L.a3_block_mean_of_hop.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_int64,
                                           C.c_void_p, C.c_int64]
        L.a3_block_mean_of_hop.restype = C.c_int
        L.a3_cache_count_accesses.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_int64,
                                              C.c_void_p]
        L.a3_cache_count_accesses.restype = C.c_int
        L.a3_cache_rank.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p]
        L.a3_cache_rank.restype = C.c_int
        L.a3_cache_fifo_update.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p,
                                           C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_int32,
                                           C.c_int64, C.c_void_p]
        L.a3_cache_fifo_update.restype = C.c_int
        L.a3_cache_fifo_update_static.argtypes = L.a3_cache_fifo_update.argtypes
        L.a3_cache_fifo_update_static.restype = C.c_int
        L.a3_block_mean_strided.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64,
                                            C.c_void_p, C.c_int64, C.c_int32, C.c_int64, C.c_void_p, C.c_int64]
        L.a3_block_mean_strided.restype = C.c_int
        L.a3_block_mean_of_hop_strided.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_int64, C.c_int32,
                                                   C.c_int64, C.c_void_p, C.c_int64, C.c_int64]
        L.a3_block_mean_of_hop_strided.restype = C.c_int
        L.a3_pipeline_create.argtypes = [C.POINTER(C.c_void_p), C.c_int, C.c_int, C.c_int, C.c_int64,
                                         C.c_int32, C.POINTER(C.c_int32), C.c_uint32]
        L.a3_pipeline_create.restype = C.c_int
        L.a3_pipeline_destroy.argtypes = [C.c_void_p]
        L.a3_pipeline_destroy.restype = C.c_int
        L.a3_pipeline_last_error.argtypes = [C.c_void_p]
        L.a3_pipeline_last_error.restype = C.c_char_p
        L.a3_pipeline_workers.argtypes = [C.c_void_p]
        L.a3_pipeline_workers.restype = C.c_int
        L.a3_pipeline_workspace_bytes.argtypes = [C.c_void_p]
        L.a3_pipeline_workspace_bytes.restype = C.c_int64
        L.a3_pipeline_stream.argtypes = [C.c_void_p, C.c_int]
        L.a3_pipeline_stream.restype = C.c_void_p
        L.a3_pipeline_submit.argtypes = L.a3_sample_blocks_begin.argtypes + [
            C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_int64, C.c_int64]
        L.a3_pipeline_submit.restype = C.c_int
        L.a3_pipeline_wait.argtypes = [C.c_void_p, C.POINTER(_CBlocks)]
        L.a3_pipeline_wait.restype = C.c_int
        _lib = L
    return _lib


class A3Error(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"a3gnn error {code}: {message}")
        self.code = code


class _DevView:
    """Exposes ctx-owned device memory to torch without a copy."""

    def __init__(self, ptr: int, n: int, typestr: str):
        self.__cuda_array_interface__ = {"shape": (n,), "typestr": typestr, "data": (ptr, False),
                                         "version": 2, "strides": None}


def _view(ptr, n: int, dtype: torch.dtype, device) -> torch.Tensor:
    if n == 0 or not ptr:
        return torch.empty(0, dtype=dtype, device=device)
    typestr = {torch.int32: "<i4", torch.int64: "<i8"}[dtype]
    return torch.as_tensor(_DevView(int(ptr), int(n), typestr), device=device)


class Blocks:
    """Result of Context.sample_blocks.  Counts are plain ints; the arrays are zero-copy tensor
    views of context-owned device memory, created on first access and valid until the next
    sample_blocks on the context."""

    def __init__(self, cb: "_CBlocks", idx_dtype: torch.dtype, device):
        H = cb.num_hops
        self.num_hops = H
        self.n_dst = list(cb.n_dst[:H])
        self.n_src = list(cb.n_src[:H])
        self.n_edges = list(cb.n_edges[:H])
        self._ptr_indptr = list(cb.blk_indptr[:H])
        self._ptr_indices = list(cb.blk_indices[:H])
        self._ptr_eids = list(cb.blk_eids[:H])
        self._ptr_input = cb.input_nodes
        self._idx_dtype = idx_dtype
        self._device = device
        self._cache = {}

    def _get(self, name, make):
        if name not in self._cache:
            self._cache[name] = make()
        return self._cache[name]

    @property
    def blk_indptr(self) -> List[torch.Tensor]:
        return self._get("indptr", lambda: [_view(p, n + 1, torch.int32, self._device)
                                            for p, n in zip(self._ptr_indptr, self.n_dst)])

    @property
    def blk_indices(self) -> List[torch.Tensor]:
        return self._get("indices", lambda: [_view(p, n, torch.int32, self._device)
                                             for p, n in zip(self._ptr_indices, self.n_edges)])

    @property
    def blk_eids(self) -> List[Optional[torch.Tensor]]:
        return self._get("eids", lambda: [None if not p else _view(p, n, torch.int64, self._device)
                                          for p, n in zip(self._ptr_eids, self.n_edges)])

    @property
    def input_nodes(self) -> torch.Tensor:
        return self._get("input", lambda: _view(self._ptr_input, self.n_src[-1], self._idx_dtype,
                                                self._device))

    def to_host(self) -> "HostBlocks":
        """Independent host copies (numpy arrays), for comparisons."""
        return HostBlocks(self.num_hops, list(self.n_dst), list(self.n_src), list(self.n_edges),
                          [t.cpu().numpy() for t in self.blk_indptr],
                          [t.cpu().numpy() for t in self.blk_indices],
                          [None if t is None else t.cpu().numpy() for t in self.blk_eids],
                          self.input_nodes.cpu().numpy())


@dataclass
class HostBlocks:
    num_hops: int
    n_dst: List[int]
    n_src: List[int]
    n_edges: List[int]
    blk_indptr: list = field(default_factory=list)
    blk_indices: list = field(default_factory=list)
    blk_eids: list = field(default_factory=list)
    input_nodes: object = None


def _dptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _row_stride(t: Optional[torch.Tensor]) -> int:
    """Bytes from one row of a 2-D tensor to the next.  Rows must be dense (unit stride inside a
    row) but may be padded: a column slice of a wider buffer, t = buf[:, :dim], is accepted.
    For an OUTPUT tensor the columns of buf beyond dim are padding, not data: where every stride
    in use is a multiple of 16 bytes, a row is copied up to the next multiple of 16 bytes, so up
    to 14 bytes of buf after each out row receive padding bytes of the source row."""
    if t is None:
        return 0
    assert t.dim() == 2 and (t.shape[1] == 1 or t.stride(1) == 1), "rows must be dense"
    assert t.shape[0] <= 1 or t.stride(0) >= t.shape[1], "rows overlap"
    return (t.stride(0) if t.shape[0] > 1 else t.shape[1]) * t.element_size()


class Context:
    """An a3_ctx bound to a device and to torch's current stream on it."""

    def __init__(self, max_seeds: int, max_fanouts: Sequence[int], device: int = 0, flags: int = 0,
                 stream: Optional[int] = None):
        self._h = C.c_void_p()
        self.flags = flags
        self.device = torch.device("cuda", device) if not (flags & A3_HOST_ONLY) else torch.device("cpu")
        if stream is None and not (flags & A3_HOST_ONLY):
            stream = torch.cuda.current_stream(self.device).cuda_stream
        fan = (C.c_int32 * len(max_fanouts))(*max_fanouts)
        rc = lib().a3_create(C.byref(self._h), device, C.c_void_p(stream or 0), max_seeds,
                             len(max_fanouts), fan, flags)
        if rc != A3_OK:
            raise A3Error(rc, (lib().a3_last_error(None) or b"").decode())

    def close(self):
        if self._h:
            lib().a3_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc: int):
        if rc != A3_OK:
            raise A3Error(rc, (lib().a3_last_error(self._h) or b"").decode())

    def set_stream(self, stream: int):
        self._check(lib().a3_set_stream(self._h, C.c_void_p(stream)))

    def set_gather_host_workgroups(self, n: int):
        self._check(lib().a3_set_gather_host_workgroups(self._h, n))

    def reserve(self, num_nodes: int):
        """allocate now what depends on the graph's size, so that no later sampling call does"""
        self._check(lib().a3_reserve(self._h, num_nodes))

    def device_map_changed(self):
        """A3_STATIC_MAP contexts: the map was rewritten, or another one lives at its address now"""
        self._check(lib().a3_device_map_changed(self._h))

    def validate_graph(self, indptr: torch.Tensor, indices: torch.Tensor):
        """raises A3Error (A3_ERR_INPUT) unless (indptr, indices) is a CSR with sorted, repeat-free rows"""
        assert indptr.dtype == torch.int64 and indptr.is_contiguous() and indptr.numel() >= 1
        assert indices.dtype in (torch.int32, torch.int64) and indices.is_contiguous()
        self._check(lib().a3_validate_graph(self._h, _dptr(indptr), _dptr(indices), indices.element_size(),
                                            indptr.numel() - 1, indices.numel()))

    def validate_cache_map(self, cache_map: torch.Tensor, n_dev_rows: int, n_host_rows: int):
        """raises A3Error (A3_ERR_INPUT) unless every node names a row of its store and none is shared"""
        assert cache_map.dtype == torch.int32 and cache_map.is_contiguous()
        self._check(lib().a3_validate_cache_map(self._h, _dptr(cache_map), cache_map.numel(), n_dev_rows,
                                                n_host_rows))

    def profile_read(self, kind: int) -> List[float]:
        """device milliseconds of the calls of this kind (0 sample, 1 gather) since the last read"""
        buf = (C.c_float * A3_PROFILE_DEPTH)()
        n = C.c_int(0)
        self._check(lib().a3_profile_read(self._h, kind, buf, A3_PROFILE_DEPTH, C.byref(n)))
        return [float(buf[i]) for i in range(n.value)]

    def sample_blocks(self, indptr: torch.Tensor, indices: torch.Tensor, seeds: torch.Tensor,
                      fanouts: Sequence[int], cache_map: Optional[torch.Tensor] = None,
                      bias_q16: int = 65536, rng_seed: int = 0) -> Blocks:
        assert indptr.dtype == torch.int64 and indptr.is_contiguous()
        assert indices.dtype in (torch.int32, torch.int64) and indices.is_contiguous()
        assert seeds.dtype == indices.dtype and seeds.is_contiguous()
        assert cache_map is None or (cache_map.dtype == torch.int32 and cache_map.is_contiguous())
        num_nodes = indptr.shape[0] - 1
        fan = (C.c_int32 * len(fanouts))(*fanouts)
        cb = _CBlocks()
        rc = lib().a3_sample_blocks(self._h, _dptr(indptr), _dptr(indices), indices.element_size(),
                                    num_nodes, _dptr(seeds), seeds.shape[0], fan, len(fanouts),
                                    _dptr(cache_map), bias_q16, rng_seed, C.byref(cb))
        self._check(rc)
        return Blocks(cb, indices.dtype, indices.device)

    def sample_blocks_begin(self, indptr: torch.Tensor, indices: torch.Tensor, seeds: torch.Tensor,
                            fanouts: Sequence[int], cache_map: Optional[torch.Tensor] = None,
                            bias_q16: int = 65536, rng_seed: int = 0) -> None:
        assert indptr.dtype == torch.int64 and indptr.is_contiguous()
        assert indices.dtype in (torch.int32, torch.int64) and indices.is_contiguous()
        assert seeds.dtype == indices.dtype and seeds.is_contiguous()
        assert cache_map is None or (cache_map.dtype == torch.int32 and cache_map.is_contiguous())
        fan = (C.c_int32 * len(fanouts))(*fanouts)
        rc = lib().a3_sample_blocks_begin(self._h, _dptr(indptr), _dptr(indices),
                                          indices.element_size(), indptr.shape[0] - 1, _dptr(seeds),
                                          seeds.shape[0], fan, len(fanouts), _dptr(cache_map),
                                          bias_q16, rng_seed)
        self._check(rc)
        self._begun = (indices.dtype, indices.device)

    def sample_gather_begin(self, indptr: torch.Tensor, indices: torch.Tensor, seeds: torch.Tensor,
                            fanouts: Sequence[int], cache_map: Optional[torch.Tensor], bias_q16: int,
                            rng_seed: int, feat_dev: Optional[torch.Tensor],
                            feat_host: Optional[torch.Tensor], out: torch.Tensor) -> None:
        """sample_blocks_begin and gather_input_features as one queued unit: the rows of the nodes a
        hop has numbered travel on a second stream while the next hop is sampled.  Ended with
        sample_blocks_end; out[:n] is whole for work queued on the context's stream afterwards."""
        assert indptr.dtype == torch.int64 and indptr.is_contiguous()
        assert indices.dtype in (torch.int32, torch.int64) and indices.is_contiguous()
        assert seeds.dtype == indices.dtype and seeds.is_contiguous()
        assert cache_map is None or (cache_map.dtype == torch.int32 and cache_map.is_contiguous())
        ref = feat_dev if feat_dev is not None else feat_host
        assert ref is not None and ref.dim() == 2
        assert feat_host is None or feat_host.is_pinned(), "feat_host must be pinned host memory"
        assert out.dim() == 2 and out.shape[1] == ref.shape[1] and out.dtype == ref.dtype
        fan = (C.c_int32 * len(fanouts))(*fanouts)
        rc = lib().a3_sample_gather_begin(self._h, _dptr(indptr), _dptr(indices), indices.element_size(),
                                          indptr.shape[0] - 1, _dptr(seeds), seeds.shape[0], fan,
                                          len(fanouts), _dptr(cache_map), bias_q16, rng_seed,
                                          _dptr(feat_dev), _row_stride(feat_dev), _dptr(feat_host),
                                          _row_stride(feat_host), ref.shape[1] * ref.element_size(),
                                          _dptr(out), _row_stride(out), out.shape[0])
        self._check(rc)
        self._begun = (indices.dtype, indices.device)

    def sample_blocks_end(self) -> Blocks:
        cb = _CBlocks()
        self._check(lib().a3_sample_blocks_end(self._h, C.byref(cb)))
        return Blocks(cb, *self._begun)

    def sample_stats(self) -> dict:
        """which paths the last ended sampling call took (see a3_sample_stats)"""
        buf = (C.c_int64 * 5)()
        self._check(lib().a3_sample_stats(self._h, buf))
        return {"weight_classes": int(buf[0]), "deferred_wide_nodes": int(buf[1]),
                "deferred_hubs": int(buf[2]), "exhaustive_nodes": int(buf[3]),
                "launch_plan": int(buf[4])}

    def gather_input_features(self, feat_dev: Optional[torch.Tensor],
                              feat_host: Optional[torch.Tensor], cache_map: Optional[torch.Tensor],
                              out: torch.Tensor) -> torch.Tensor:
        """rows of the last sampled input nodes -> out[:n]; may be queued before sample_blocks_end.
        If out is a column slice of a wider buffer, the bytes between its rows are padding and
        may be overwritten (see _row_stride)."""
        ref = feat_dev if feat_dev is not None else feat_host
        assert ref is not None and ref.dim() == 2
        assert feat_host is None or feat_host.is_pinned(), "feat_host must be pinned host memory"
        assert out.dim() == 2 and out.shape[1] == ref.shape[1] and out.dtype == ref.dtype
        row_bytes = ref.shape[1] * ref.element_size()
        rc = lib().a3_gather_input_features_strided(self._h, _dptr(feat_dev), _row_stride(feat_dev),
                                                    _dptr(feat_host), _row_stride(feat_host),
                                                    _dptr(cache_map), row_bytes, _dptr(out),
                                                    _row_stride(out), out.shape[0])
        self._check(rc)
        return out

    def gather_features(self, feat_dev: Optional[torch.Tensor], feat_host: Optional[torch.Tensor],
                        cache_map: Optional[torch.Tensor], ids: torch.Tensor,
                        out: Optional[torch.Tensor] = None) -> torch.Tensor:
        """out[i] = the row of ids[i] from the device cache or the host store, as cache_map says.
        If out is a column slice of a wider buffer, the bytes between its rows are padding and
        may be overwritten (see _row_stride)."""
        ref = feat_dev if feat_dev is not None else feat_host
        assert ref is not None and ref.dim() == 2
        for t in (feat_dev, feat_host):
            assert t is None or (t.dtype == ref.dtype and t.shape[1] == ref.shape[1])
        assert feat_host is None or feat_host.is_pinned(), "feat_host must be pinned host memory"
        assert ids.dtype in (torch.int32, torch.int64) and ids.is_contiguous()
        row_bytes = ref.shape[1] * ref.element_size()
        if out is None:
            out = torch.empty((ids.shape[0], ref.shape[1]), dtype=ref.dtype, device=ids.device)
        assert out.shape == (ids.shape[0], ref.shape[1]) and out.dtype == ref.dtype
        rc = lib().a3_gather_features_strided(self._h, _dptr(feat_dev), _row_stride(feat_dev),
                                              _dptr(feat_host), _row_stride(feat_host), _dptr(cache_map),
                                              _dptr(ids), ids.element_size(), ids.shape[0], row_bytes,
                                              _dptr(out), _row_stride(out))
        self._check(rc)
        return out

    @staticmethod
    def _dtype_code(t: torch.Tensor) -> int:
        assert t.dtype in (torch.float32, torch.float16), "features must be float32 or float16"
        return A3_F32 if t.dtype == torch.float32 else A3_F16

    def block_mean(self, blk_indptr: torch.Tensor, blk_indices: torch.Tensor, x: torch.Tensor,
                   out: Optional[torch.Tensor] = None) -> torch.Tensor:
        """mean of the source rows x[blk_indices[e]] of every destination of one block; the bytes
        between the rows of a padded out are padding and may be overwritten (see _row_stride)"""
        assert blk_indptr.dtype == torch.int32 and blk_indptr.is_contiguous()
        assert blk_indices.dtype == torch.int32 and blk_indices.is_contiguous()
        n_dst = blk_indptr.shape[0] - 1
        if out is None:
            out = torch.empty((n_dst, x.shape[1]), dtype=x.dtype, device=x.device)
        assert out.shape == (n_dst, x.shape[1]) and out.dtype == x.dtype
        rc = lib().a3_block_mean_strided(self._h, _dptr(blk_indptr), _dptr(blk_indices), n_dst,
                                         x.shape[0], _dptr(x), _row_stride(x), self._dtype_code(x),
                                         x.shape[1], _dptr(out), _row_stride(out))
        self._check(rc)
        return out

    def block_mean_of_hop(self, hop: int, x: torch.Tensor, out: torch.Tensor) -> torch.Tensor:
        """the same for block `hop` of the last sampled mini-batch, counts taken on the device;
        may be queued before sample_blocks_end; writes out[:n_dst[hop]] (and, in a padded out, may
        overwrite the padding between rows)"""
        assert out.dim() == 2 and out.shape[1] == x.shape[1] and out.dtype == x.dtype
        rc = lib().a3_block_mean_of_hop_strided(self._h, hop, _dptr(x), _row_stride(x),
                                                self._dtype_code(x), x.shape[1], _dptr(out),
                                                _row_stride(out), out.shape[0])
        self._check(rc)
        return out

    def cache_count_accesses(self, counts: torch.Tensor, ids: Optional[torch.Tensor] = None) -> None:
        """counts[id] += 1 for every id; ids = None: the input nodes of the last sampled mini-batch
        (count taken on the device, may be queued before sample_blocks_end)"""
        assert counts.dtype == torch.int32 and counts.is_contiguous(), "counts: int32 tensor (read as uint32)"
        assert ids is None or (ids.dtype in (torch.int32, torch.int64) and ids.is_contiguous())
        if ids is not None and ids.shape[0] == 0:
            return  # an empty tensor has no address; a null `ids` would mean "the last input nodes"
        rc = lib().a3_cache_count_accesses(self._h, _dptr(ids), 0 if ids is None else ids.element_size(),
                                           0 if ids is None else ids.shape[0], counts.shape[0],
                                           _dptr(counts))
        self._check(rc)

    def cache_rank(self, counts: torch.Tensor, n_cached: int):
        """(cache_map, order) of the static fill ranked by (count descending, id ascending)"""
        assert counts.dtype == torch.int32 and counts.is_contiguous()
        n = counts.shape[0]
        cache_map = torch.empty(n, dtype=torch.int32, device=counts.device)
        order = torch.empty(n, dtype=torch.int32, device=counts.device)
        self._check(lib().a3_cache_rank(self._h, _dptr(counts), n, n_cached, _dptr(cache_map),
                                        _dptr(order)))
        return cache_map, order

    def cache_fifo_update(self, cache_map: torch.Tensor, slot_owner: torch.Tensor,
                          fifo_state: torch.Tensor, feat_dev: torch.Tensor, rows: torch.Tensor,
                          ids: Optional[torch.Tensor] = None, static_scratch: bool = False) -> None:
        """one mini-batch through the FIFO cache, in place; ids = None: the input nodes of the last
        sampled mini-batch, rows then being what gather_input_features wrote.  static_scratch:
        a3_cache_fifo_update_static, the form that allocates nothing (at most
        A3_FIFO_STATIC_MAX_IDS ids)"""
        for t in (cache_map, slot_owner, fifo_state):
            assert t.dtype == torch.int32 and t.is_contiguous()
        assert fifo_state.shape[0] >= 4
        assert feat_dev.dim() == 2 and feat_dev.is_contiguous() and rows.is_contiguous()
        assert rows.dim() == 2 and rows.shape[1] == feat_dev.shape[1] and rows.dtype == feat_dev.dtype
        assert ids is None or (ids.dtype in (torch.int32, torch.int64) and ids.is_contiguous()
                               and ids.shape[0] <= rows.shape[0])
        row_bytes = feat_dev.shape[1] * feat_dev.element_size()
        if ids is not None and ids.shape[0] == 0:
            return  # an empty tensor has no address; a null `ids` would mean "the last input nodes"
        call = lib().a3_cache_fifo_update_static if static_scratch else lib().a3_cache_fifo_update
        rc = call(self._h, _dptr(cache_map), cache_map.shape[0], _dptr(slot_owner),
                  _dptr(fifo_state), slot_owner.shape[0], _dptr(feat_dev),
                  row_bytes, _dptr(ids), 0 if ids is None else ids.element_size(),
                  0 if ids is None else ids.shape[0], _dptr(rows))
        self._check(rc)


class Pipeline:
    """An a3_pipeline: n_workers mini-batches in flight on streams of their own, scheduled as the
    paper's sequential / parallel mode 1 / parallel mode 2 templates.  submit() queues sampling and
    feature retrieve of one mini-batch, wait() returns the oldest one's Blocks once both are done."""

    def __init__(self, mode: int, n_workers: int, max_seeds: int, max_fanouts: Sequence[int],
                 device: int = 0, flags: int = 0):
        self._h = C.c_void_p()
        self.device = torch.device("cuda", device) if not (flags & A3_HOST_ONLY) else torch.device("cpu")
        fan = (C.c_int32 * len(max_fanouts))(*max_fanouts)
        rc = lib().a3_pipeline_create(C.byref(self._h), device, mode, n_workers, max_seeds,
                                      len(max_fanouts), fan, flags)
        if rc != A3_OK:
            raise A3Error(rc, (lib().a3_pipeline_last_error(None) or b"").decode())
        self.mode = mode
        self.n_workers = lib().a3_pipeline_workers(self._h)
        self._begun = []

    def close(self):
        if self._h:
            lib().a3_pipeline_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc: int):
        if rc != A3_OK:
            raise A3Error(rc, (lib().a3_pipeline_last_error(self._h) or b"").decode())

    def reserve(self, num_nodes: int):
        """Context.reserve on every worker: no mini-batch of the pipeline allocates afterwards"""
        self._check(lib().a3_pipeline_reserve(self._h, num_nodes))

    @property
    def workspace_bytes(self) -> int:
        return int(lib().a3_pipeline_workspace_bytes(self._h))

    def stream(self, w: int) -> int:
        return int(lib().a3_pipeline_stream(self._h, w) or 0)

    def submit(self, indptr: torch.Tensor, indices: torch.Tensor, seeds: torch.Tensor,
               fanouts: Sequence[int], cache_map: Optional[torch.Tensor], bias_q16: int,
               rng_seed: int, feat_dev: Optional[torch.Tensor], feat_host: Optional[torch.Tensor],
               out: Optional[torch.Tensor]) -> None:
        """The tensors must be complete on the device (the pipeline's streams do not wait for
        torch's); out = None queues sampling only."""
        assert indptr.dtype == torch.int64 and indptr.is_contiguous()
        assert indices.dtype in (torch.int32, torch.int64) and indices.is_contiguous()
        assert seeds.dtype == indices.dtype and seeds.is_contiguous()
        assert cache_map is None or (cache_map.dtype == torch.int32 and cache_map.is_contiguous())
        row_bytes, out_rows = 0, 0
        if out is not None:
            ref = feat_dev if feat_dev is not None else feat_host
            assert ref is not None and ref.dim() == 2
            assert feat_host is None or feat_host.is_pinned(), "feat_host must be pinned host memory"
            assert out.dim() == 2 and out.shape[1] == ref.shape[1] and out.dtype == ref.dtype
            row_bytes, out_rows = ref.shape[1] * ref.element_size(), out.shape[0]
        fan = (C.c_int32 * len(fanouts))(*fanouts)
        rc = lib().a3_pipeline_submit(self._h, _dptr(indptr), _dptr(indices), indices.element_size(),
                                      indptr.shape[0] - 1, _dptr(seeds), seeds.shape[0], fan,
                                      len(fanouts), _dptr(cache_map), bias_q16, rng_seed,
                                      _dptr(feat_dev), _row_stride(feat_dev), _dptr(feat_host),
                                      _row_stride(feat_host), row_bytes, _dptr(out), _row_stride(out),
                                      out_rows)
        self._check(rc)
        self._begun.append((indices.dtype, indices.device))

    def wait(self) -> Blocks:
        cb = _CBlocks()
        rc = lib().a3_pipeline_wait(self._h, C.byref(cb))
        if self._begun and rc != A3_ERR_INVALID_ARG:
            begun = self._begun.pop(0)
        self._check(rc)
        return Blocks(cb, *begun)
