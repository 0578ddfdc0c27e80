"""The FIFO cache update that allocates nothing (a3_cache_fifo_update_static, for callers that
cannot call hipMalloc) against the allocating entry point it is a variant of: both are called
through the C ABI on copies of the same state, two calls in a row, the second with a smaller
input, and every output (device map, slot owners, ring state, cached rows) must be equal.
Collected last: a failure here must not hide the tests before it."""
import ctypes as C

import numpy as np
import pytest
import torch

import paper_2511_07421_amd as a3

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _ptr(t):
    return C.c_void_p(t.data_ptr())


def _fresh_state(N, n_slots, dim, dtype):
    cm = (-torch.arange(N, dtype=torch.int32) - 1).to(DEV)
    owner = torch.full((n_slots,), -1, dtype=torch.int32, device=DEV)
    state = torch.zeros(4, dtype=torch.int32, device=DEV)
    cache = torch.zeros((n_slots, dim), dtype=dtype, device=DEV)
    return cm, owner, state, cache


@pytest.mark.parametrize("idx_dtype,dtype,dim", [(np.int32, torch.float32, 25), (np.int64, torch.float16, 64)])
def test_static_scratch_update_equals_allocating_update(idx_dtype, dtype, dim):
    L = a3.lib()
    N, n_slots = 60_000, 4_000
    rng = np.random.default_rng(17)
    table = torch.from_numpy(rng.standard_normal((N, dim)).astype(np.float32)).to(dtype)
    fan = (C.c_int32 * 1)(2)
    stream = torch.cuda.current_stream(torch.device(DEV)).cuda_stream
    ctxs = []
    for _ in range(2):
        h = C.c_void_p()
        assert L.a3_create(C.byref(h), 0, C.c_void_p(stream), 8, 1, fan, 0) == a3.A3_OK
        ctxs.append(h)
    ref, new = _fresh_state(N, n_slots, dim, dtype), _fresh_state(N, n_slots, dim, dtype)
    row_bytes = dim * table.element_size()
    # 5 000 ids span five tiles of 1 024 and a ragged tail and overflow the 4 000 slots; the second
    # call is smaller (one full tile and a tail), so stale scratch of the first would show
    for n_ids in (5_000, 1_500):
        print(f"[case] fifo static n_ids={n_ids} idx={idx_dtype.__name__} dim={dim}", flush=True)
        ids = rng.choice(N, size=n_ids, replace=False).astype(idx_dtype)
        d_ids = torch.from_numpy(ids).to(DEV)
        d_rows = table[torch.from_numpy(ids.astype(np.int64))].to(DEV).contiguous()
        for call, h, (cm, owner, state, cache) in ((L.a3_cache_fifo_update, ctxs[0], ref),
                                                   (L.a3_cache_fifo_update_static, ctxs[1], new)):
            rc = call(h, _ptr(cm), N, _ptr(owner), _ptr(state), n_slots, _ptr(cache), row_bytes,
                      _ptr(d_ids), d_ids.element_size(), n_ids, _ptr(d_rows))
            assert rc == a3.A3_OK, L.a3_last_error(h)
        torch.cuda.synchronize()
        for got, want in zip(new, ref):
            assert torch.equal(got, want)
        assert int(ref[2][1].item()) > 0          # there were misses, the update did something
    # beyond the static scratch: refused with a clear error, nothing queued
    big = torch.zeros(a3.A3_FIFO_STATIC_MAX_IDS + 1, dtype=torch.int32, device=DEV)
    rows1 = torch.zeros((1, dim), dtype=dtype, device=DEV)
    cm, owner, state, cache = new
    rc = L.a3_cache_fifo_update_static(ctxs[1], _ptr(cm), N, _ptr(owner), _ptr(state), n_slots, _ptr(cache),
                                       row_bytes, _ptr(big), 4, big.shape[0], _ptr(rows1))
    assert rc == a3.A3_ERR_CAPACITY
    assert b"A3_FIFO_STATIC_MAX_IDS" in L.a3_last_error(ctxs[1])
    for h in ctxs:
        L.a3_destroy(h)


def test_static_scratch_update_on_the_last_sampled_input_nodes():
    """ids == NULL: the input nodes of the context's last mini-batch, count on the device"""
    from workloads import get_config, make_graph, make_features, seed_batch
    w = get_config("mini_copurchase")
    g = make_graph(w.num_nodes, w.mean_degree, w.d_min, w.d_max, w.a, w.symmetric, w.graph_seed, w.idx_dtype)
    full = make_features(w.num_nodes, 12, torch.float32)
    N, n_slots, dim = w.num_nodes, 2_000, 12
    d_ip, d_ix = g.indptr.to(DEV), g.indices.to(DEV)
    host_store = full.clone().pin_memory()
    results = []
    for static in (False, True):
        ctx = a3.Context(w.batch, w.fanouts)
        cm, owner, state, cache = _fresh_state(N, n_slots, dim, torch.float32)
        rows = torch.zeros((N, dim), dtype=torch.float32, device=DEV)
        for b, batch in enumerate((w.batch, w.batch // 4)):      # the second mini-batch is smaller
            seeds = torch.from_numpy(seed_batch(N, batch, 3, b, dtype=np.int32)).to(DEV)
            ctx.sample_blocks_begin(d_ip, d_ix, seeds, w.fanouts, cm, 4 * 65536, b)
            ctx.gather_input_features(cache, host_store, cm, rows)
            ctx.cache_fifo_update(cm, owner, state, cache, rows, static_scratch=static)
            ctx.sample_blocks_end()
        torch.cuda.synchronize()
        results.append((cm, owner, state, cache))
        ctx.close()
    for got, want in zip(results[1], results[0]):
        assert torch.equal(got, want)
