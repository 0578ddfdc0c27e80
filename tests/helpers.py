"""Shared checks on sampled blocks (used on oracle output and on GPU output alike).
They use only the CSR graph and the definitions; no oracle call, no GPU call."""
import numpy as np


def check_block_invariants(indptr, indices, seeds, fanouts, blocks):
    """blocks: object with num_hops, n_dst, n_src, n_edges, blk_indptr, blk_indices, blk_eids,
    input_nodes (numpy arrays on host)."""
    indptr = np.asarray(indptr)
    indices = np.asarray(indices)
    S = np.asarray(blocks.input_nodes).astype(np.int64)
    H = blocks.num_hops
    assert H == len(fanouts)
    assert S.shape[0] == blocks.n_src[H - 1]
    assert np.array_equal(S[:len(seeds)], np.asarray(seeds).astype(np.int64))
    assert np.unique(S).shape[0] == S.shape[0], "local -> global map must be injective"
    assert blocks.n_dst[0] == len(seeds)
    for h in range(H):
        n_dst, n_src, n_e = blocks.n_dst[h], blocks.n_src[h], blocks.n_edges[h]
        if h > 0:
            assert n_dst == blocks.n_src[h - 1]
        assert n_dst <= n_src <= n_dst + n_e
        bp = np.asarray(blocks.blk_indptr[h]).astype(np.int64)
        bi = np.asarray(blocks.blk_indices[h]).astype(np.int64)
        be = np.asarray(blocks.blk_eids[h]).astype(np.int64)
        assert bp.shape[0] == n_dst + 1 and bp[0] == 0 and bp[-1] == n_e
        assert bi.shape[0] == n_e and be.shape[0] == n_e
        dst_global = S[:n_dst]
        deg = indptr[dst_global + 1] - indptr[dst_global]
        assert np.array_equal(np.diff(bp), np.minimum(deg, fanouts[h])), "min(fanout, degree) samples per node"
        if n_e == 0:
            assert n_src == n_dst
            continue
        assert bi.min() >= 0 and bi.max() < n_src
        dst_of_edge = np.repeat(np.arange(n_dst), np.diff(bp))
        # every sampled edge is a CSR edge of its destination, and its source is what the CSR holds
        row0 = indptr[dst_global][dst_of_edge]
        row1 = indptr[dst_global + 1][dst_of_edge]
        assert np.all((be >= row0) & (be < row1))
        assert np.array_equal(indices[be].astype(np.int64), S[bi])
        # slots strictly increasing inside a destination: no slot twice, CSR order
        same = dst_of_edge[1:] == dst_of_edge[:-1]
        assert np.all(be[1:][same] > be[:-1][same])
        # new sources are numbered in order of first use, right after the destinations;
        # first appearance comes from a library routine (np.unique with return_index)
        g = indices[be].astype(np.int64)
        is_old = np.isin(g, dst_global)
        new_g = g[~is_old]
        uniq, first = np.unique(new_g, return_index=True)
        expect_new = new_g[np.sort(first)]
        assert np.array_equal(S[n_dst:n_src], expect_new)
        # every source of this hop is used by some edge or is a destination
        used = np.zeros(n_src, dtype=bool)
        used[bi] = True
        assert np.all(used[n_dst:])


def blocks_equal(a, b):
    """exact equality of two block sets (host numpy)"""
    assert a.num_hops == b.num_hops
    assert list(a.n_dst) == list(b.n_dst)
    assert list(a.n_src) == list(b.n_src)
    assert list(a.n_edges) == list(b.n_edges)
    for h in range(a.num_hops):
        assert np.array_equal(np.asarray(a.blk_indptr[h]), np.asarray(b.blk_indptr[h])), f"indptr hop {h}"
        assert np.array_equal(np.asarray(a.blk_eids[h]), np.asarray(b.blk_eids[h])), f"eids hop {h}"
        assert np.array_equal(np.asarray(a.blk_indices[h]), np.asarray(b.blk_indices[h])), f"indices hop {h}"
    assert np.array_equal(np.asarray(a.input_nodes).astype(np.int64),
                          np.asarray(b.input_nodes).astype(np.int64))
