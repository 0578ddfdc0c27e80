"""Pins for the oracle's neighbour aggregation (mean over the sampled sources of each destination):
a dense normalised-adjacency product by a library matmul, closed forms, and the invariants of a
mean, chosen so that a wrong divisor, a transposed operand, an off-by-one row range or a
mis-decoded half fails one of them."""
import numpy as np
import pytest

import oracle


def _random_block(rng, n_dst, n_src, max_deg):
    deg = rng.integers(0, max_deg + 1, size=n_dst)
    indptr = np.zeros(n_dst + 1, dtype=np.int32)
    indptr[1:] = np.cumsum(deg)
    indices = rng.integers(0, n_src, size=int(indptr[-1])).astype(np.int32)
    return indptr, indices


def test_equals_dense_normalised_adjacency_product():
    rng = np.random.default_rng(1)
    n_dst, n_src, dim = 37, 90, 19
    indptr, indices = _random_block(rng, n_dst, n_src, 9)
    x = rng.standard_normal((n_src, dim)).astype(np.float32)
    A = np.zeros((n_dst, n_src))
    for i in range(n_dst):
        for e in range(indptr[i], indptr[i + 1]):
            A[i, indices[e]] += 1.0          # a source sampled twice counts twice
        if indptr[i + 1] > indptr[i]:
            A[i] /= indptr[i + 1] - indptr[i]
    want = A @ x.astype(np.float64)
    got = oracle.block_mean(indptr, indices, x)
    assert got.shape == (n_dst, dim)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-13)


def test_closed_forms():
    # worked by hand: rows 0..3 of x are [1,2], [3,4], [5,6], [7,8]
    x = np.array([[1, 2], [3, 4], [5, 6], [7, 8]], dtype=np.float32)
    indptr = np.array([0, 2, 2, 3, 6], dtype=np.int32)
    indices = np.array([0, 3, 2, 1, 1, 2], dtype=np.int32)
    got = oracle.block_mean(indptr, indices, x)
    want = np.array([[4.0, 5.0],             # (row0 + row3) / 2
                     [0.0, 0.0],             # no sampled edge: zeros
                     [5.0, 6.0],             # one edge: the row itself
                     [11.0 / 3, 14.0 / 3]])  # (row1 + row1 + row2) / 3
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-15)


def test_mean_invariants():
    rng = np.random.default_rng(2)
    n_dst, n_src, dim = 50, 64, 8
    indptr, indices = _random_block(rng, n_dst, n_src, 12)
    x = rng.standard_normal((n_src, dim)).astype(np.float32)
    base = oracle.block_mean(indptr, indices, x)
    deg = np.diff(indptr)
    # constant features: the mean is that constant wherever there is an edge
    const = oracle.block_mean(indptr, indices, np.full((n_src, dim), 2.5, dtype=np.float32))
    assert np.all(const[deg > 0] == 2.5) and np.all(const[deg == 0] == 0.0)
    # the order of a destination's edges does not matter
    perm = indices.copy()
    for i in range(n_dst):
        perm[indptr[i]:indptr[i + 1]] = perm[indptr[i]:indptr[i + 1]][::-1]
    np.testing.assert_allclose(oracle.block_mean(indptr, perm, x), base, rtol=0, atol=1e-14)
    # linear in the features (2x is exact in binary)
    np.testing.assert_array_equal(oracle.block_mean(indptr, indices, 2 * x), 2 * base)
    # every value lies between the smallest and largest source value of its row
    for i in np.flatnonzero(deg > 0)[:10]:
        rows = x[indices[indptr[i]:indptr[i + 1]]].astype(np.float64)
        assert np.all(base[i] >= rows.min(0) - 1e-12) and np.all(base[i] <= rows.max(0) + 1e-12)


def test_half_input_is_decoded_as_ieee_binary16():
    rng = np.random.default_rng(3)
    n_dst, n_src, dim = 20, 40, 6
    indptr, indices = _random_block(rng, n_dst, n_src, 7)
    xh = rng.standard_normal((n_src, dim)).astype(np.float16)
    xh[0, 0] = np.float16(6.0e-8)      # subnormal
    xh[1, 1] = np.float16(-65504.0)    # largest magnitude
    xh[2, 2] = np.float16(-0.0)
    indices[:3] = [0, 1, 2]
    got = oracle.block_mean(indptr, indices, xh)
    want = oracle.block_mean(indptr, indices, xh.astype(np.float32))  # numpy's own half decoding
    np.testing.assert_array_equal(got, want)


def test_bad_index_is_refused():
    x = np.zeros((3, 2), dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.block_mean(np.array([0, 1], dtype=np.int32), np.array([3], dtype=np.int32), x)
    with pytest.raises(ValueError):
        oracle.block_mean(np.array([0, 1], dtype=np.int32), np.array([-1], dtype=np.int32), x)
