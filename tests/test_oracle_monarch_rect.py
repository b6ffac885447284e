"""Pins for the Monarch oracle with different block counts on the input and output side (no GPU)."""
import numpy as np
import pytest

import oracle

RNG = np.random.default_rng(31)

# (T, n_in, n_out, b1, b2, r'): b1 != b2, p != q, r' != b
SHAPES = [
    (5, 12, 20, 3, 4, 2),
    (3, 8, 9, 4, 3, 1),
    (4, 10, 6, 1, 3, 2),     # one input block
    (2, 15, 7, 5, 1, 3),     # one output block
    (6, 16, 16, 2, 8, 5),
    (3, 12, 12, 4, 4, 2),    # square case
]


def rand_rect(T, n_in, n_out, b1, b2, rp):
    X = RNG.standard_normal((T, n_in))
    R = RNG.standard_normal((b1, rp * b2, n_in // b1))
    L = RNG.standard_normal((b2, n_out // b2, b1 * rp))
    return X, R, L


def dense_from_block_definition(R, L, b1, b2):
    """Paper-oriented W (in x out): block (l, k) = V_{l,k} U_{l,k} (Section 2.1, Monarch), the slices
    being read off the stored tensors by the two storage orders of Section 4 (optimisation 1)."""
    p, q = R.shape[2], L.shape[1]
    rp = R.shape[1] // b2
    R4 = R.reshape(b1, rp, b2, p)      # [l, rho, k, a]
    L4 = L.reshape(b2, q, b1, rp)      # [k, j, l, rho]
    W = np.zeros((b1 * p, b2 * q))
    for l in range(b1):
        for k in range(b2):
            W[l * p:(l + 1) * p, k * q:(k + 1) * q] = R4[l, :, k, :].T @ L4[k, :, l, :].T
    return W


@pytest.mark.parametrize("shape", SHAPES)
def test_equals_block_definition_in_both_output_orders(shape):
    T, n_in, n_out, b1, b2, rp = shape
    X, R, L = rand_rect(*shape)
    W = dense_from_block_definition(R, L, b1, b2)
    q = n_out // b2
    Yb = oracle.monarch_rect_forward(X, R, L, b1, b2, oracle.OUT_BLOCKED, nthreads=2)
    np.testing.assert_allclose(Yb, X @ W, rtol=1e-12, atol=1e-12)
    Yi = oracle.monarch_rect_forward(X, R, L, b1, b2, oracle.OUT_INTERLEAVED, nthreads=3)
    # interleaved: feature (k, j) at j*b2 + k
    np.testing.assert_allclose(Yi.reshape(T, q, b2), Yb.reshape(T, b2, q).transpose(0, 2, 1), rtol=0, atol=0)


@pytest.mark.parametrize("shape", SHAPES)
def test_parameter_and_operation_counts(shape):
    T, n_in, n_out, b1, b2, rp = shape
    X, R, L = rand_rect(*shape)
    p, q = n_in // b1, n_out // b2
    assert R.size + L.size == b1 * b2 * rp * (p + q)                  # Section 2.1, Monarch parameter count
    _, macs = oracle.monarch_rect_forward(X, R, L, b1, b2, return_macs=True)
    assert macs == T * b1 * b2 * rp * (p + q)


def test_square_case_equals_the_square_oracle():
    T, n, b, rp = 5, 24, 4, 3
    X, R, L = rand_rect(T, n, 36, b, b, rp)
    for order in (oracle.OUT_INTERLEAVED, oracle.OUT_BLOCKED):
        np.testing.assert_array_equal(oracle.monarch_rect_forward(X, R, L, b, b, order),
                                      oracle.monarch_forward(X, R, L, order))


def test_block_rank_and_block_locality():
    T, n_in, n_out, b1, b2, rp = 4, 18, 20, 3, 5, 2
    X, R, L = rand_rect(T, n_in, n_out, b1, b2, rp)
    Wt = oracle.monarch_rect_forward(np.eye(n_in), R, L, b1, b2, oracle.OUT_BLOCKED)   # rows of W (in x out)
    p, q = n_in // b1, n_out // b2
    for l in range(b1):
        for k in range(b2):
            sv = np.linalg.svd(Wt[l * p:(l + 1) * p, k * q:(k + 1) * q], compute_uv=False)
            assert np.sum(sv > 1e-10 * sv[0]) == min(rp, p, q)
    # one input block alone
    X2 = np.zeros_like(X); X2[:, p:2 * p] = X[:, p:2 * p]
    np.testing.assert_allclose(oracle.monarch_rect_forward(X2, R, L, b1, b2, oracle.OUT_BLOCKED), X2[:, p:2 * p] @ Wt[p:2 * p], rtol=1e-12, atol=1e-12)


def test_invalid_shapes():
    X, R, L = rand_rect(2, 12, 20, 3, 4, 2)
    with pytest.raises((ValueError, AssertionError)):
        oracle.monarch_rect_forward(X[:, :11], R, L, 3, 4)
