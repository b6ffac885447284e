"""Pins for the low-rank part of the CPU oracle (no GPU)."""
import numpy as np
import pytest

import oracle

RNG = np.random.default_rng(23)

# (T, n_in, n_out, r)
SHAPES = [(5, 12, 18, 5), (3, 8, 4, 7), (4, 20, 12, 1), (1, 9, 9, 9), (6, 7, 31, 3)]


def rand_lr(T, n_in, n_out, r):
    return RNG.standard_normal((T, n_in)), RNG.standard_normal((r, n_in)), RNG.standard_normal((n_out, r))


@pytest.mark.parametrize("shape", SHAPES)
def test_equals_dense_product_of_the_factors(shape):
    """W = V U (Section 2.1, Low-Rank) in the paper's in x out orientation; the stored factors are its
    V and U transposed."""
    X, V, U = rand_lr(*shape)
    W_paper = V.T @ U.T                                   # (i x r)(r x o)
    Y = oracle.lowrank_forward(X, V, U, nthreads=2)
    np.testing.assert_allclose(Y, X @ W_paper, rtol=1e-12, atol=1e-12)
    Wm = oracle.materialize_lowrank(V, U)
    np.testing.assert_allclose(Wm, W_paper.T, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(oracle.dense_forward(X, Wm), Y, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("shape", SHAPES)
def test_rank_and_operation_count(shape):
    T, n_in, n_out, r = shape
    X, V, U = rand_lr(*shape)
    W = oracle.materialize_lowrank(V, U)
    sv = np.linalg.svd(W, compute_uv=False)
    assert np.sum(sv > 1e-10 * sv[0]) == min(r, n_in, n_out)
    _, macs = oracle.lowrank_forward(X, V, U, nthreads=3, return_macs=True)
    assert macs == T * r * (n_in + n_out)                 # n r (i + o), Section 2.1
    assert V.size + U.size == r * (n_in + n_out)


@pytest.mark.parametrize("shape", SHAPES)
def test_monarch_with_one_block_and_blast_with_unit_coupling(shape):
    """A Monarch layer with a single block and a BLAST layer with a single block and s = 1 are both
    the plain low-rank layer (Section 2.1: both structures generalise low-rank)."""
    T, n_in, n_out, r = shape
    X, V, U = rand_lr(*shape)
    Y = oracle.lowrank_forward(X, V, U)
    np.testing.assert_allclose(oracle.monarch_forward(X, V[None], U[None]), Y, rtol=1e-12, atol=1e-12)
    Yb = oracle.blast_forward(X, U[None], np.ones((1, 1, r)), V.T[None].copy())
    np.testing.assert_allclose(Yb, Y, rtol=1e-12, atol=1e-12)


def test_transposed_operand_or_swapped_factor_would_fail():
    """Asymmetric closed form: V picks input features, U places them. X = e_a, V row c = e_a,
    U column c = e_o gives Y = e_o exactly."""
    n_in, n_out, r = 6, 9, 4
    V = np.zeros((r, n_in)); U = np.zeros((n_out, r))
    picks = [(0, 5, 2), (1, 0, 8), (2, 3, 3), (3, 2, 0)]  # (rank index, input feature, output feature)
    for c, a, o in picks:
        V[c, a] = 1.0 + c
        U[o, c] = 10.0 * (1 + c)
    X = np.eye(n_in)
    Y = oracle.lowrank_forward(X, V, U)
    want = np.zeros((n_in, n_out))
    for c, a, o in picks:
        want[a, o] = (1.0 + c) * 10.0 * (1 + c)
    np.testing.assert_array_equal(Y, want)


def test_linearity_zero_and_row_independence():
    X, V, U = rand_lr(7, 10, 14, 4)
    X2 = RNG.standard_normal(X.shape)
    f = lambda x: oracle.lowrank_forward(x, V, U)
    np.testing.assert_allclose(f(2.0 * X - 3.0 * X2), 2.0 * f(X) - 3.0 * f(X2), rtol=1e-11, atol=1e-11)
    assert not f(np.zeros_like(X)).any()
    perm = RNG.permutation(7)
    np.testing.assert_array_equal(f(X[perm]), f(X)[perm])
    assert oracle.lowrank_forward(np.zeros((0, 10)), V, U).shape == (0, 14)
