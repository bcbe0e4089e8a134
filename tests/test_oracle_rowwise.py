"""Pins of the row-wise operator oracle (Intra-DP Sec. IV-A, Eq. 1): matrix product of row
bands with a replicated parameter matrix."""
import numpy as np
import pytest

import workloads
from oracle import planner


def _rand(shape, seed):
    return np.random.Generator(np.random.PCG64(seed)).standard_normal(shape, dtype=np.float32)


def test_brute_force_tiny(oracle):
    x, w, b = _rand((5, 4), 1), _rand((3, 4), 2), _rand((3,), 3)
    r = _rand((5, 3), 4)
    want = np.empty((5, 3), np.float32)
    for i in range(5):
        for c in range(3):
            acc = 0.0
            for j in range(4):
                acc += float(x[i, j]) * float(w[c, j])
            want[i, c] = np.float32(max(acc + float(b[c]) + float(r[i, c]), 0.0))
    got = oracle.rowwise(x, w, b, r, "relu", "f32")
    np.testing.assert_array_equal(got, want)


def test_against_fp64_matmul(oracle):
    x, w = _rand((37, 129), 5), _rand((61, 129), 6)
    b = _rand((61,), 7)
    got = oracle.rowwise(x, w, b, None, "none", "f32")
    want = x.astype(np.float64) @ w.astype(np.float64).T + b.astype(np.float64)
    # double accumulation in another order, one rounding to fp32
    np.testing.assert_allclose(got, want, rtol=0, atol=2.0 ** -23 * np.abs(want).max())
    assert np.abs(got - want.astype(np.float32)).max() <= 2.0 ** -22 * np.abs(want).max()


def test_identity_and_column_selection(oracle):
    x = _rand((9, 6), 8)
    np.testing.assert_array_equal(oracle.rowwise(x, np.eye(6, dtype=np.float32), None, None, "none", "f32"), x)
    # a one-hot input row picks one column of W^T, i.e. element j of every row of W
    w = _rand((4, 6), 9)
    for j in range(6):
        e = np.zeros((1, 6), np.float32)
        e[0, j] = 1.0
        np.testing.assert_array_equal(oracle.rowwise(e, w, None, None, "none", "f32")[0], w[:, j])
    # W is n x k with one row per output column: a transposed operand would fail here
    w2 = np.zeros((2, 6), np.float32)
    w2[1, 5] = 1.0
    np.testing.assert_array_equal(oracle.rowwise(x, w2, None, None, "none", "f32")[:, 1], x[:, 5])


def test_equals_one_by_one_convolution(oracle):
    """Eq. 1 is the 1x1 convolution on a tensor whose pixels are the matrix rows."""
    m, k, n = 23, 16, 10
    x, w, b = _rand((m, k), 10), _rand((n, k), 11), _rand((n,), 12)
    got = oracle.rowwise(x, w, b, None, "relu6", "f32")
    chain = workloads.Chain("pw", (1, k, m, 1), "f32", 1)
    chain.add(workloads.CONV, k, n, 1, 1, 0, 1, "relu6")
    t = workloads.Tensors(np.ascontiguousarray(x.T.reshape(1, k, m, 1)), [w.reshape(n, k, 1, 1)], [b])
    conv = oracle.run_chain(chain, t)                      # 1 x n x m x 1
    np.testing.assert_array_equal(got, conv[0, :, :, 0].T)


def test_rows_are_independent_and_bands_equal_whole(oracle):
    chain = workloads.RowChain("c", 29, 12, "f32", 4)
    chain.add(20, "relu").add(12, "none", residual_from=-1).add(7, "relu6")
    t = workloads.make_row_tensors(chain, zero_bias=False, seed=3)
    whole = oracle.run_row_chain(chain, t)
    assert not np.isnan(whole).any()
    bands = [(r.lo, r.hi) if hasattr(r, "lo") else tuple(r) for r in planner.split_rows(chain.m, 4)]
    assert bands == [(0, 8), (8, 15), (15, 22), (22, 29)]          # numpy.array_split sizes 8,7,7,7
    np.testing.assert_array_equal(oracle.run_row_chain(chain, t, bands), whole)
    np.testing.assert_array_equal(oracle.run_row_chain(chain, t, bands[::-1]), whole)
    # changing one input row changes that output row only
    t2 = workloads.Tensors(t.x.copy(), t.weights, t.biases)
    t2.x[11] += 1.0
    other = oracle.run_row_chain(chain, t2)
    keep = np.arange(chain.m) != 11
    np.testing.assert_array_equal(other[keep], whole[keep])
    assert not np.array_equal(other[11], whole[11])


def test_small_integers_exact_and_bf16_single_rounding(oracle):
    rng = np.random.Generator(np.random.PCG64(4))
    x = rng.integers(-3, 4, (13, 40)).astype(np.float32)
    w = rng.integers(-2, 3, (9, 40)).astype(np.float32)
    want = (x.astype(np.int64) @ w.astype(np.int64).T).astype(np.float32)
    np.testing.assert_array_equal(oracle.rowwise(x, w, None, None, "none", "f32"), want)
    np.testing.assert_array_equal(oracle.rowwise(x, w, None, None, "none", "bf16"),
                                  workloads.to_bf16_values(want))
    # 1 + 2^-8 + 2^-16 rounds to 1 + 2^-7 only if the sum is rounded once
    x1 = np.array([[1.0, 2.0 ** -8, 2.0 ** -16]], np.float32)
    w1 = np.ones((1, 3), np.float32)
    assert oracle.rowwise(x1, w1, None, None, "none", "bf16")[0, 0] == np.float32(1 + 2.0 ** -7)
