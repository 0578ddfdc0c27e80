"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every declared
symbol, and rejects bad arguments before touching a device."""
import ctypes as C
import os
import re

import pytest

import paper_2511_07421_amd as a3

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(a3.library_path()):
        from paper_2511_07421_amd import build
        build.build()
    return a3.lib()


def test_every_declared_symbol_is_exported(L):
    names = set()
    for fn in os.listdir(os.path.join(ROOT, "include")):
        if fn.endswith(".h"):
            text = open(os.path.join(ROOT, "include", fn)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names |= set(re.findall(r"\b(a3(?:cpu)?_[a-z_]+)\s*\(", text))
    assert {"a3_create", "a3_destroy", "a3_set_stream", "a3_last_error", "a3_sample_blocks",
            "a3_gather_features", "a3_pipeline_submit", "a3_block_mean", "a3_cache_fifo_update",
            "a3cpu_sample_blocks"} <= names
    for n in names:
        assert hasattr(L, n), n


def _create(L, max_seeds, fanouts, flags):
    h = C.c_void_p()
    fan = (C.c_int32 * len(fanouts))(*fanouts)
    rc = L.a3_create(C.byref(h), 0, None, max_seeds, len(fanouts), fan, flags)
    return rc, h


def test_create_argument_errors(L):
    assert _create(L, -1, [2], a3.A3_HOST_ONLY)[0] == a3.A3_ERR_INVALID_ARG
    assert _create(L, 4, [0], a3.A3_HOST_ONLY)[0] == a3.A3_ERR_INVALID_ARG
    assert _create(L, 4, [a3.A3_MAX_FANOUT + 1], a3.A3_HOST_ONLY)[0] == a3.A3_ERR_INVALID_ARG
    assert _create(L, 4, [2] * 9, a3.A3_HOST_ONLY)[0] == a3.A3_ERR_INVALID_ARG
    assert b"max_hops" in L.a3_last_error(None)
    # 2^20 seeds x 1024 x 1024 local ids do not fit int32
    assert _create(L, 1 << 20, [1024, 1024], a3.A3_HOST_ONLY)[0] == a3.A3_ERR_CAPACITY
    assert L.a3_create(None, 0, None, 4, 1, (C.c_int32 * 1)(2), a3.A3_HOST_ONLY) == a3.A3_ERR_INVALID_ARG
    rc, h = _create(L, 4, [2, 2], a3.A3_HOST_ONLY)
    assert rc == a3.A3_OK and h.value
    assert L.a3_destroy(h) == a3.A3_OK
    assert L.a3_destroy(None) == a3.A3_OK


def test_sample_and_gather_argument_errors(L):
    rc, h = _create(L, 8, [3, 2], a3.A3_HOST_ONLY)
    assert rc == a3.A3_OK
    blocks = a3.binding._CBlocks()
    dummy = C.create_string_buffer(64)
    p = C.cast(dummy, C.c_void_p)
    fan = (C.c_int32 * 2)(3, 2)

    def sample(indptr=p, indices=p, ib=4, n=10, seeds=p, ns=4, f=fan, nh=2, cm=None, bias=65536,
               out=C.byref(blocks)):
        return L.a3_sample_blocks(h, indptr, indices, ib, n, seeds, ns, f, nh, cm, bias, 0, out)

    assert sample(indptr=None) == a3.A3_ERR_INVALID_ARG
    assert sample(ib=2) == a3.A3_ERR_INVALID_ARG
    assert sample(seeds=None) == a3.A3_ERR_INVALID_ARG
    assert sample(ns=-1) == a3.A3_ERR_INVALID_ARG
    assert sample(nh=0) == a3.A3_ERR_INVALID_ARG
    assert sample(f=(C.c_int32 * 2)(3, 0)) == a3.A3_ERR_INVALID_ARG
    assert sample(bias=65535) == a3.A3_ERR_INVALID_ARG
    assert b"bias" in L.a3_last_error(h)
    assert sample(out=None) == a3.A3_ERR_INVALID_ARG
    assert sample(ns=9) == a3.A3_ERR_CAPACITY
    assert sample(f=(C.c_int32 * 2)(4, 2)) == a3.A3_ERR_CAPACITY
    assert sample(f=(C.c_int32 * 3)(3, 2, 2), nh=3) == a3.A3_ERR_CAPACITY
    # valid arguments, but the context has no device: fails loudly instead of computing elsewhere
    assert sample() == a3.A3_ERR_HIP
    assert b"without a device" in L.a3_last_error(h)

    def gather(fd=p, fh=None, cm=None, ids=p, ib=4, n=2, rb=8, out=p):
        return L.a3_gather_features(h, fd, fh, cm, ids, ib, n, rb, out)

    assert gather(ib=3) == a3.A3_ERR_INVALID_ARG
    assert gather(n=-1) == a3.A3_ERR_INVALID_ARG
    assert gather(rb=0) == a3.A3_ERR_INVALID_ARG
    assert gather(rb=7) == a3.A3_ERR_INVALID_ARG
    assert gather(ids=None) == a3.A3_ERR_INVALID_ARG
    assert gather(out=None) == a3.A3_ERR_INVALID_ARG
    assert gather(fd=None, fh=None) == a3.A3_ERR_INVALID_ARG
    assert gather(fd=None, fh=p, cm=None) == a3.A3_ERR_INVALID_ARG
    assert gather() == a3.A3_ERR_HIP
    assert L.a3_sample_blocks(None, p, p, 4, 10, p, 4, fan, 2, None, 65536, 0, C.byref(blocks)) == a3.A3_ERR_INVALID_ARG

    # sampling and retrieve as one unit: the checks of both, before anything is queued
    def unit(indptr=p, ns=4, bias=65536, fd=p, fh=None, cm=None, rb=8, out=p, rows=100, ds=0, os_=0):
        return L.a3_sample_gather_begin(h, indptr, p, 4, 10, p, ns, fan, 2, cm, bias, 0, fd, ds, fh, 0, rb, out, os_, rows)

    assert L.a3_sample_gather_begin(None, p, p, 4, 10, p, 4, fan, 2, None, 65536, 0, p, 0, None, 0, 8, p, 0, 100) == a3.A3_ERR_INVALID_ARG
    assert unit(indptr=None) == a3.A3_ERR_INVALID_ARG
    assert unit(bias=1) == a3.A3_ERR_INVALID_ARG
    assert unit(ns=9) == a3.A3_ERR_CAPACITY
    assert unit(rb=7) == a3.A3_ERR_INVALID_ARG
    assert unit(out=None) == a3.A3_ERR_INVALID_ARG
    assert unit(rows=-1) == a3.A3_ERR_INVALID_ARG
    assert unit(fd=None, fh=None) == a3.A3_ERR_INVALID_ARG
    assert unit(fd=None, fh=p, cm=None) == a3.A3_ERR_INVALID_ARG
    assert unit(ds=6) == a3.A3_ERR_INVALID_ARG           # a stride below the row
    assert unit() == a3.A3_ERR_HIP
    assert L.a3_destroy(h) == a3.A3_OK


def test_python_wrapper_raises_with_message():
    ctx = a3.Context(8, [3, 2], flags=a3.A3_HOST_ONLY)
    import torch
    indptr = torch.zeros(5, dtype=torch.int64)
    idx = torch.zeros(4, dtype=torch.int32)
    with pytest.raises(a3.A3Error) as ei:
        ctx.sample_blocks(indptr, idx, idx[:2], [3, 2])
    assert ei.value.code == a3.A3_ERR_HIP
    with pytest.raises(a3.A3Error) as ei:
        ctx.sample_blocks(indptr, idx, idx[:2], [9, 2])
    assert ei.value.code == a3.A3_ERR_CAPACITY
    ctx.close()


def test_pipeline_argument_errors(L):
    fan = (C.c_int32 * 2)(3, 2)
    h = C.c_void_p()
    assert L.a3_pipeline_create(None, 0, 1, 2, 8, 2, fan, a3.A3_HOST_ONLY) == a3.A3_ERR_INVALID_ARG
    assert L.a3_pipeline_create(C.byref(h), 0, 3, 2, 8, 2, fan, a3.A3_HOST_ONLY) == a3.A3_ERR_INVALID_ARG
    assert b"mode" in L.a3_pipeline_last_error(None)
    assert L.a3_pipeline_create(C.byref(h), 0, 1, 0, 8, 2, fan, a3.A3_HOST_ONLY) == a3.A3_ERR_INVALID_ARG
    assert L.a3_pipeline_create(C.byref(h), 0, 1, a3.A3_PIPE_MAX_WORKERS + 1, 8, 2, fan,
                                a3.A3_HOST_ONLY) == a3.A3_ERR_INVALID_ARG
    # the workers' own limits are checked as in a3_create
    assert L.a3_pipeline_create(C.byref(h), 0, 1, 2, -1, 2, fan, a3.A3_HOST_ONLY) == a3.A3_ERR_INVALID_ARG
    assert L.a3_pipeline_create(C.byref(h), 0, a3.A3_PIPE_SEQUENTIAL, 4, 8, 2, fan,
                                a3.A3_HOST_ONLY) == a3.A3_OK
    assert L.a3_pipeline_workers(h) == 1  # the sequential template has one worker
    assert L.a3_pipeline_destroy(h) == a3.A3_OK
    assert L.a3_pipeline_create(C.byref(h), 0, a3.A3_PIPE_MODE2, 3, 8, 2, fan, a3.A3_HOST_ONLY) == a3.A3_OK
    assert L.a3_pipeline_workers(h) == 3
    assert L.a3_pipeline_stream(h, 7) is None
    blocks = a3.binding._CBlocks()
    assert L.a3_pipeline_wait(h, C.byref(blocks)) == a3.A3_ERR_INVALID_ARG  # nothing in flight
    dummy = C.create_string_buffer(64)
    p = C.cast(dummy, C.c_void_p)

    def submit(indptr=p, ns=4, bias=65536, row_bytes=0, out=None, out_rows=0, feat=None, stride=0):
        return L.a3_pipeline_submit(h, indptr, p, 4, 10, p, ns, fan, 2, None, bias, 0, feat, stride, None,
                                    0, row_bytes, out, 0, out_rows)

    assert submit(indptr=None) == a3.A3_ERR_INVALID_ARG
    assert submit(bias=1) == a3.A3_ERR_INVALID_ARG
    assert submit(ns=9) == a3.A3_ERR_CAPACITY
    assert submit(row_bytes=-2) == a3.A3_ERR_INVALID_ARG
    assert submit(row_bytes=3, out=p, out_rows=1, feat=p) == a3.A3_ERR_INVALID_ARG  # odd row
    assert submit(row_bytes=8, out=None, out_rows=4, feat=p) == a3.A3_ERR_INVALID_ARG
    assert submit(row_bytes=8, out=p, out_rows=4, feat=None) == a3.A3_ERR_INVALID_ARG  # no store
    assert submit(row_bytes=8, out=p, out_rows=4, feat=p, stride=6) == a3.A3_ERR_INVALID_ARG  # stride < row
    assert submit() == a3.A3_ERR_HIP  # valid arguments, but no device behind the pipeline
    assert b"without a device" in L.a3_pipeline_last_error(h)
    assert L.a3_pipeline_wait(h, C.byref(blocks)) == a3.A3_ERR_INVALID_ARG  # still nothing in flight
    assert L.a3_pipeline_destroy(h) == a3.A3_OK
    assert L.a3_pipeline_destroy(None) == a3.A3_OK


def test_block_mean_argument_errors(L):
    rc, h = _create(L, 8, [3, 2], a3.A3_HOST_ONLY)
    assert rc == a3.A3_OK
    dummy = C.create_string_buffer(64)
    p = C.cast(dummy, C.c_void_p)

    def mean(ip=p, ix=p, n_dst=2, n_src=3, x=p, dt=a3.A3_F32, dim=4, out=p):
        return L.a3_block_mean(h, ip, ix, n_dst, n_src, x, dt, dim, out)

    assert L.a3_block_mean(None, p, p, 2, 3, p, 0, 4, p) == a3.A3_ERR_INVALID_ARG
    assert mean(n_dst=-1) == a3.A3_ERR_INVALID_ARG
    assert mean(n_src=1 << 31) == a3.A3_ERR_INVALID_ARG
    assert mean(dt=2) == a3.A3_ERR_INVALID_ARG
    assert b"x_dtype" in L.a3_last_error(h)
    assert mean(dim=0) == a3.A3_ERR_INVALID_ARG
    assert mean(ip=None) == a3.A3_ERR_INVALID_ARG
    assert mean(x=None) == a3.A3_ERR_INVALID_ARG
    assert mean(out=None) == a3.A3_ERR_INVALID_ARG
    assert mean() == a3.A3_ERR_HIP  # valid arguments, no device
    assert L.a3_block_mean_of_hop(h, 0, None, 0, 4, p, 2) == a3.A3_ERR_INVALID_ARG
    assert L.a3_block_mean_of_hop(h, 0, p, 0, 4, None, 2) == a3.A3_ERR_INVALID_ARG
    assert L.a3_block_mean_of_hop(h, 0, p, 0, 4, p, 2) == a3.A3_ERR_HIP
    assert L.a3_destroy(h) == a3.A3_OK


def test_cache_policy_argument_errors(L):
    rc, h = _create(L, 8, [3, 2], a3.A3_HOST_ONLY)
    assert rc == a3.A3_OK
    dummy = C.create_string_buffer(64)
    p = C.cast(dummy, C.c_void_p)
    assert L.a3_cache_count_accesses(None, p, 4, 3, 10, p) == a3.A3_ERR_INVALID_ARG
    assert L.a3_cache_count_accesses(h, p, 4, 3, -1, p) == a3.A3_ERR_INVALID_ARG
    assert L.a3_cache_count_accesses(h, p, 4, 3, 10, None) == a3.A3_ERR_INVALID_ARG
    assert L.a3_cache_count_accesses(h, p, 2, 3, 10, p) == a3.A3_ERR_INVALID_ARG
    assert L.a3_cache_count_accesses(h, p, 4, -3, 10, p) == a3.A3_ERR_INVALID_ARG
    assert L.a3_cache_count_accesses(h, p, 4, 3, 10, p) == a3.A3_ERR_HIP
    assert L.a3_cache_rank(h, p, 10, 11, p, None) == a3.A3_ERR_INVALID_ARG
    assert L.a3_cache_rank(h, p, -1, 0, p, None) == a3.A3_ERR_INVALID_ARG
    assert L.a3_cache_rank(h, None, 10, 2, p, None) == a3.A3_ERR_INVALID_ARG
    assert L.a3_cache_rank(h, p, 10, 2, p, None) == a3.A3_ERR_HIP

    # the allocating form and the one on static scratch check their arguments alike
    for call in (L.a3_cache_fifo_update, L.a3_cache_fifo_update_static):
        def fifo(cm=p, n=10, owner=p, st=p, slots=4, feat=p, rb=8, ids=p, ib=4, n_ids=2, rows=p):
            return call(h, cm, n, owner, st, slots, feat, rb, ids, ib, n_ids, rows)

        assert fifo(cm=None) == a3.A3_ERR_INVALID_ARG
        assert fifo(slots=0) == a3.A3_ERR_INVALID_ARG
        assert fifo(rb=7) == a3.A3_ERR_INVALID_ARG
        assert fifo(rows=None) == a3.A3_ERR_INVALID_ARG
        assert fifo(ib=3) == a3.A3_ERR_INVALID_ARG
        assert fifo() == a3.A3_ERR_HIP
    assert L.a3_destroy(h) == a3.A3_OK


def test_strided_argument_errors(L):
    rc, h = _create(L, 8, [3, 2], a3.A3_HOST_ONLY)
    assert rc == a3.A3_OK
    dummy = C.create_string_buffer(64)
    p = C.cast(dummy, C.c_void_p)

    def gather(ds=0, hs=0, os_=0, rb=8):
        return L.a3_gather_features_strided(h, p, ds, p, hs, None, p, 4, 2, rb, p, os_)

    assert gather(ds=6) == a3.A3_ERR_INVALID_ARG          # stride below the row
    assert b"stride" in L.a3_last_error(h)
    assert gather(hs=9) == a3.A3_ERR_INVALID_ARG          # odd stride
    assert gather(os_=-16) == a3.A3_ERR_INVALID_ARG
    assert gather(ds=128, hs=0, os_=16) == a3.A3_ERR_HIP  # valid, but no device
    assert L.a3_gather_input_features_strided(h, p, 4, None, 0, None, 8, p, 0, 2) == a3.A3_ERR_INVALID_ARG
    assert L.a3_block_mean_strided(h, p, p, 2, 3, p, 12, a3.A3_F32, 4, p, 0) == a3.A3_ERR_INVALID_ARG
    assert L.a3_block_mean_strided(h, p, p, 2, 3, p, 32, a3.A3_F32, 4, p, 64) == a3.A3_ERR_HIP
    assert L.a3_block_mean_of_hop_strided(h, 0, p, 0, a3.A3_F16, 4, p, 6, 2) == a3.A3_ERR_INVALID_ARG
    assert L.a3_destroy(h) == a3.A3_OK


def test_validate_argument_errors(L):
    L.a3_validate_graph.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_int64]
    L.a3_validate_cache_map.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64]
    rc, h = _create(L, 8, [3, 2], a3.A3_HOST_ONLY)
    assert rc == a3.A3_OK
    dummy = C.create_string_buffer(64)
    p = C.cast(dummy, C.c_void_p)
    assert L.a3_validate_graph(h, None, p, 4, 3, 5) == a3.A3_ERR_INVALID_ARG
    assert L.a3_validate_graph(h, p, None, 4, 3, 5) == a3.A3_ERR_INVALID_ARG
    assert L.a3_validate_graph(h, p, p, 2, 3, 5) == a3.A3_ERR_INVALID_ARG
    assert L.a3_validate_graph(h, p, p, 4, -1, 5) == a3.A3_ERR_INVALID_ARG
    assert L.a3_validate_graph(h, p, p, 4, 1 << 31, 5) == a3.A3_ERR_INVALID_ARG   # needs 8-byte ids
    assert L.a3_validate_graph(h, p, p, 8, 3, 5) == a3.A3_ERR_HIP                 # valid, but no device
    assert L.a3_validate_cache_map(h, None, 3, 1, 2) == a3.A3_ERR_INVALID_ARG
    assert L.a3_validate_cache_map(h, p, 3, -1, 2) == a3.A3_ERR_INVALID_ARG
    assert L.a3_validate_cache_map(h, p, 3, (1 << 31) + 1, 2) == a3.A3_ERR_INVALID_ARG
    assert L.a3_validate_cache_map(h, p, 3, 1, 2) == a3.A3_ERR_HIP
    assert L.a3_set_gather_host_workgroups(h, 16) == a3.A3_OK
    assert L.a3_set_gather_host_workgroups(h, -1) == a3.A3_ERR_INVALID_ARG
    assert L.a3_reserve(None, 10) == a3.A3_ERR_INVALID_ARG
    assert L.a3_reserve(h, -1) == a3.A3_ERR_INVALID_ARG
    assert L.a3_reserve(h, 10) == a3.A3_ERR_HIP                                   # valid, but no device
    assert L.a3_pipeline_reserve(None, 10) == a3.A3_ERR_INVALID_ARG
    assert L.a3_device_map_changed(None) == a3.A3_ERR_INVALID_ARG
    assert L.a3_device_map_changed(h) == a3.A3_OK
    assert L.a3_destroy(h) == a3.A3_OK
