"""Pins for the Monarch part of the CPU oracle (no GPU).

Each test checks the oracle against something the paper or the mathematics
fixes, computed here by a different route (numpy einsum over the paper's
per-block definition, plain library GEMMs for special cases, invariants).
"""
import numpy as np
import pytest

import oracle

RNG = np.random.default_rng(7)

# (T, n_in, n_out, nblocks, r): rectangular, r' != b, p != q != r, so that a
# swapped index or a transposed operand cannot cancel out.
SHAPES = [
    (5, 12, 18, 3, 6),    # p=4 q=6 r'=2
    (3, 8, 8, 2, 8),      # r' = 4
    (4, 20, 12, 4, 4),    # r' = 1
    (2, 6, 15, 3, 9),     # r' = 3
    (7, 16, 16, 4, 16),   # square, r = n/b
]


def rand_monarch(T, n_in, n_out, b, r):
    X = RNG.standard_normal((T, n_in))
    R = RNG.standard_normal((b, r, n_in // b))
    L = RNG.standard_normal((b, n_out // b, r))
    return X, R, L


def blocks_from_definition(R, L):
    """W_{l,k} = V_{l,k} U_{l,k} (Section 2.1, Monarch), with V_{l,k}, U_{l,k} read off the
    stored tensors by the storage orders of Section 4 (optimisation 1): the middle
    dimension of the first factor is ordered (r', b2) with b2 fastest, the innermost
    dimension of the second factor is ordered (b1, r') with r' fastest."""
    b, r, p = R.shape
    q = L.shape[1]
    rp = r // b
    R4 = R.reshape(b, rp, b, p)        # [l, rho, k, a]
    L4 = L.reshape(b, q, b, rp)        # [k, j, l, rho]
    W = np.zeros((b, b, p, q))         # [l, k] -> p x q block, paper orientation (in x out)
    for l in range(b):
        for k in range(b):
            V_lk = R4[l, :, k, :].T    # p x r'
            U_lk = L4[k, :, l, :].T    # r' x q
            W[l, k] = V_lk @ U_lk
    return W


def forward_from_blocks(X, Wb, interleaved):
    """Y_k = sum_l X_l W_{l,k} (Section 2.1, Monarch)."""
    b, _, p, q = Wb.shape
    T = X.shape[0]
    Yk = np.zeros((b, T, q))
    for k in range(b):
        for l in range(b):
            Yk[k] += X[:, l * p:(l + 1) * p] @ Wb[l, k]
    if interleaved:                     # (b2, n, q) -> (n, q, b2)
        return Yk.transpose(1, 2, 0).reshape(T, q * b)
    return Yk.transpose(1, 0, 2).reshape(T, b * q)   # (n, b2, q)


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("order", [oracle.OUT_INTERLEAVED, oracle.OUT_BLOCKED])
def test_struct_equals_block_definition(shape, order):
    X, R, L = rand_monarch(*shape)
    Y = oracle.monarch_forward(X, R, L, order, nthreads=2)
    Yref = forward_from_blocks(X, blocks_from_definition(R, L), order == oracle.OUT_INTERLEAVED)
    np.testing.assert_allclose(Y, Yref, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("order", [oracle.OUT_INTERLEAVED, oracle.OUT_BLOCKED])
def test_materialised_weight(shape, order):
    T, n_in, n_out, b, r = shape
    X, R, L = rand_monarch(*shape)
    W = oracle.materialize_monarch(R, L, order)
    Wb = blocks_from_definition(R, L)
    p, q = n_in // b, n_out // b
    for l in range(b):
        for k in range(b):
            rows = [(j * b + k) if order == oracle.OUT_INTERLEAVED else (k * q + j) for j in range(q)]
            np.testing.assert_allclose(W[rows][:, l * p:(l + 1) * p], Wb[l, k].T, rtol=1e-12, atol=1e-12)
    # brute-force X W^T, both through the oracle's dense routine and through numpy
    Y = oracle.monarch_forward(X, R, L, order)
    np.testing.assert_allclose(oracle.dense_forward(X, W), Y, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(X @ W.T, Y, rtol=1e-12, atol=1e-12)


def test_einsum_of_layout_statement():
    T, n_in, n_out, b, r = 4, 12, 18, 3, 6
    X, R, L = rand_monarch(T, n_in, n_out, b, r)
    rp, p, q = r // b, n_in // b, n_out // b
    Yk = np.einsum("tla,lrka,kjlr->tkj", X.reshape(T, b, p), R.reshape(b, rp, b, p), L.reshape(b, q, b, rp))
    np.testing.assert_allclose(oracle.monarch_forward(X, R, L, oracle.OUT_BLOCKED), Yk.reshape(T, -1), rtol=1e-12)
    np.testing.assert_allclose(oracle.monarch_forward(X, R, L, oracle.OUT_INTERLEAVED),
                               Yk.transpose(0, 2, 1).reshape(T, -1), rtol=1e-12)


def test_one_block_is_two_gemms():
    # nblocks = 1: both permutations are the identity and the layer is low-rank, Y = (X R^T) L^T
    X, R, L = rand_monarch(6, 10, 14, 1, 5)
    Yref = (X @ R[0].T) @ L[0].T
    for order in (oracle.OUT_INTERLEAVED, oracle.OUT_BLOCKED):
        np.testing.assert_allclose(oracle.monarch_forward(X, R, L, order), Yref, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("b,r", [(2, 4), (3, 6), (4, 4), (4, 8), (8, 8), (4, 1024), (16, 64)])
def test_middle_permutation(b, r):
    perm = oracle.monarch_middle_perm(b, r)
    N = b * r
    assert sorted(perm.tolist()) == list(range(N))               # bijection
    # stride permutation: reshape the middle vector as (r, b) and transpose
    np.testing.assert_array_equal(perm, np.arange(N).reshape(r, b).T.reshape(-1))
    is_involution = np.array_equal(perm[perm], np.arange(N))
    assert is_involution == (r == b or b == 1 or r == 1)          # involution exactly for the square case N = b^2
    # with the first factor's rows re-laid out (r' fastest, then b2: optimisation 1) only the
    # block transpose b1 <-> b2 of contiguous r'-runs is left, and that is an involution for every b
    rp = r // b
    relayout = np.arange(N).reshape(b, rp, b).transpose(0, 2, 1).reshape(-1)   # new[l][k*r'+rho] <- old[l][rho*b+k]
    block_T = np.arange(N).reshape(b, b, rp).transpose(1, 0, 2).reshape(-1)    # new[k][l][rho] <- old[l][k][rho]
    np.testing.assert_array_equal(relayout[block_T], perm)
    np.testing.assert_array_equal(block_T[block_T], np.arange(N))


def test_square_monarch_permutation_involution_through_forward():
    # square Monarch (N = b^2 middle width, r = b): with identity factors the layer is P applied twice... i.e. X itself
    b = 4
    n = b * b
    R = np.stack([np.eye(b) for _ in range(b)])       # r = p = b
    L = np.stack([np.eye(b) for _ in range(b)])       # q = r = b
    X = RNG.standard_normal((3, n))
    Y = oracle.monarch_forward(X, R, L, oracle.OUT_INTERLEAVED)
    np.testing.assert_array_equal(Y, X)                # P (P^T x) = x
    Yb = oracle.monarch_forward(X, R, L, oracle.OUT_BLOCKED)
    perm = oracle.monarch_middle_perm(b, b)
    np.testing.assert_array_equal(Yb, X[:, perm])      # only the middle permutation is left
    np.testing.assert_array_equal(Yb[:, perm], X)      # and it is an involution


def test_linearity_and_rows():
    T, n_in, n_out, b, r = 6, 12, 18, 3, 6
    X1, R, L = rand_monarch(T, n_in, n_out, b, r)
    X2 = RNG.standard_normal((T, n_in))
    f = lambda X: oracle.monarch_forward(X, R, L)
    np.testing.assert_allclose(f(2.5 * X1 - 0.75 * X2), 2.5 * f(X1) - 0.75 * f(X2), rtol=1e-11, atol=1e-12)
    assert not f(np.zeros((T, n_in))).any()
    order = RNG.permutation(T)
    np.testing.assert_array_equal(f(X1[order]), f(X1)[order])     # tokens are independent
    np.testing.assert_array_equal(oracle.monarch_forward(X1, R, L, nthreads=1),
                                  oracle.monarch_forward(X1, R, L, nthreads=3))


def test_identity_input_returns_weight_and_block_rank():
    n_in, n_out, b, r = 12, 18, 3, 6
    _, R, L = rand_monarch(1, n_in, n_out, b, r)
    Y = oracle.monarch_forward(np.eye(n_in), R, L, oracle.OUT_BLOCKED)
    W = oracle.materialize_monarch(R, L, oracle.OUT_BLOCKED)
    np.testing.assert_allclose(Y, W.T, rtol=1e-12, atol=1e-13)
    p, q, rp = n_in // b, n_out // b, r // b
    for l in range(b):
        for k in range(b):
            blk = W[k * q:(k + 1) * q, l * p:(l + 1) * p]
            assert np.linalg.matrix_rank(blk, tol=1e-9) == rp     # every block has rank r'
    assert np.linalg.matrix_rank(W, tol=1e-9) > rp * b // 2       # while W itself is not low-rank by construction


def test_block_locality():
    T, n_in, n_out, b, r = 3, 12, 18, 3, 6
    X, R, L = rand_monarch(T, n_in, n_out, b, r)
    p = n_in // b
    base = oracle.monarch_forward(X, R, L, oracle.OUT_BLOCKED)
    # zeroing the first factor's block l must be the same as zeroing input block l
    for l in range(b):
        X0 = X.copy(); X0[:, l * p:(l + 1) * p] = 0
        R0 = R.copy(); R0[l] = 0
        np.testing.assert_allclose(oracle.monarch_forward(X0, R, L, oracle.OUT_BLOCKED),
                                   oracle.monarch_forward(X, R0, L, oracle.OUT_BLOCKED), rtol=1e-12, atol=1e-13)
    # zeroing the second factor's block k zeroes exactly output block k
    q = n_out // b
    for k in range(b):
        L0 = L.copy(); L0[k] = 0
        Y = oracle.monarch_forward(X, R, L0, oracle.OUT_BLOCKED)
        assert not Y[:, k * q:(k + 1) * q].any()
        mask = np.ones(n_out, bool); mask[k * q:(k + 1) * q] = False
        np.testing.assert_array_equal(Y[:, mask], base[:, mask])


@pytest.mark.parametrize("shape", SHAPES)
def test_mac_and_parameter_counts(shape):
    T, n_in, n_out, b, r = shape
    X, R, L = rand_monarch(*shape)
    _, macs = oracle.monarch_forward(X, R, L, return_macs=True, nthreads=2)
    assert macs == T * r * (n_in + n_out)          # n r (i + o), Section 2.1 / Table 2
    rp, p, q = r // b, n_in // b, n_out // b
    assert R.size + L.size == b * b * rp * (p + q) == r * (n_in + n_out)


def test_config0_against_dense_weight():
    """Monarch 256x256, 4 blocks of 64x64, fp32-stored inputs, T = 8: structured result equals
    X W^T for the materialised dense 256x256 W."""
    import blr_inputs as bi
    cfg = bi.CONFIGS["C0"]
    lay = bi.make_layer(cfg)
    X = bi.activations(8, 256, "f32", scale=cfg["x_scale"])
    assert lay.R.shape == (4, 64, 64) and lay.L.shape == (4, 64, 64)
    Y = oracle.monarch_forward(X.f64, lay.R.f64, lay.L.f64)
    Wb = blocks_from_definition(lay.R.f64, lay.L.f64)
    W = np.zeros((256, 256))
    for l in range(4):
        for k in range(4):
            W[k::4, l * 64:(l + 1) * 64] = Wb[l, k].T     # interleaved rows j*4 + k
    np.testing.assert_allclose(Y, X.f64 @ W.T, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(oracle.materialize_monarch(lay.R.f64, lay.L.f64), W, rtol=1e-12, atol=1e-15)


def test_invalid_arguments():
    X, R, L = rand_monarch(2, 12, 18, 3, 6)
    with pytest.raises(ValueError):
        oracle.monarch_forward(X, R, L, out_order=5)
    with pytest.raises(ValueError):
        oracle.monarch_middle_perm(3, 7)
