"""Pins for the BLAST part of the CPU oracle, and the Monarch<->BLAST cross-check (no GPU)."""
import numpy as np
import pytest

import oracle

RNG = np.random.default_rng(11)

# (T, n_in, n_out, b, r): q = n_in/b != p = n_out/b, r not a multiple of b
SHAPES = [
    (5, 12, 18, 3, 5),
    (3, 8, 4, 2, 7),
    (4, 20, 12, 4, 3),
    (2, 16, 16, 16, 6),   # 1x1 blocks
    (6, 10, 15, 5, 1),    # rank one
]


def rand_blast(T, n_in, n_out, b, r):
    X = RNG.standard_normal((T, n_in))
    U = RNG.standard_normal((b, n_out // b, r))
    S = RNG.standard_normal((b, b, r))
    V = RNG.standard_normal((b, n_in // b, r))
    return X, U, S, V


def dense_from_definition(U, S, V):
    """Block (input j, output i) of the paper-oriented weight (in x out) is V_j diag(s_ij) U_i^T
    (Section 2.1, BLAST: W_{l,k} = V_l S_{l,k} U_k with the stored U_k transposed)."""
    b, p, r = U.shape
    q = V.shape[1]
    W = np.zeros((b * q, b * p))
    for j in range(b):
        for i in range(b):
            W[j * q:(j + 1) * q, i * p:(i + 1) * p] = V[j] @ np.diag(S[i, j]) @ U[i].T
    return W


@pytest.mark.parametrize("shape", SHAPES)
def test_struct_equals_block_definition(shape):
    X, U, S, V = rand_blast(*shape)
    Y = oracle.blast_forward(X, U, S, V, nthreads=2)
    W = dense_from_definition(U, S, V)
    np.testing.assert_allclose(Y, X @ W, rtol=1e-12, atol=1e-12)
    Wm = oracle.materialize_blast(U, S, V)
    np.testing.assert_allclose(Wm, W.T, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(oracle.dense_forward(X, Wm), Y, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("shape", SHAPES)
def test_paper_formula_per_output_block(shape):
    """Y_k = (sum_l (X_l V_l) S_{l,k}) U_k (Section 2.1, BLAST)."""
    T, n_in, n_out, b, r = shape
    X, U, S, V = rand_blast(*shape)
    q, p = n_in // b, n_out // b
    Y = np.zeros((T, n_out))
    for i in range(b):
        acc = np.zeros((T, r))
        for j in range(b):
            acc += (X[:, j * q:(j + 1) * q] @ V[j]) @ np.diag(S[i, j])
        Y[:, i * p:(i + 1) * p] = acc @ U[i].T
    np.testing.assert_allclose(oracle.blast_forward(X, U, S, V), Y, rtol=1e-12, atol=1e-12)


def test_single_block_is_u_diag_s_vt():
    X, U, S, V = rand_blast(6, 9, 7, 1, 4)
    W = U[0] @ np.diag(S[0, 0]) @ V[0].T            # n_out x n_in
    np.testing.assert_allclose(oracle.blast_forward(X, U, S, V), X @ W.T, rtol=1e-12, atol=1e-13)


def test_all_ones_coupling_is_low_rank():
    # S = 1 recovers a plain low-rank layer (Section 2.1, BLAST): Y = (X Vstack) Ustack^T
    T, n_in, n_out, b, r = 5, 12, 18, 3, 5
    X, U, _, V = rand_blast(T, n_in, n_out, b, r)
    S = np.ones((b, b, r))
    Vs = V.reshape(n_in, r)
    Us = U.reshape(n_out, r)
    np.testing.assert_allclose(oracle.blast_forward(X, U, S, V), (X @ Vs) @ Us.T, rtol=1e-12, atol=1e-12)
    assert np.linalg.matrix_rank(oracle.materialize_blast(U, S, V), tol=1e-9) == r


@pytest.mark.parametrize("n_in,n_out,b,rp", [(12, 18, 3, 2), (8, 8, 2, 4), (20, 12, 4, 1), (16, 16, 4, 4)])
def test_monarch_is_a_blast_layer(n_in, n_out, b, rp):
    """Monarch is recovered from BLAST by a 0/1 coupling (Section 2.1, BLAST). With BLAST rank
    r_B = b r', index (m, rho): V_j[:, (m,rho)] = V_{j,(j+m) mod b}[:, rho],
    U_i[:, (m,rho)] = U_{(i-m) mod b, i}[rho, :], S[i][j][(m,rho)] = [m == (i-j) mod b].
    The two oracles are written independently; they must agree."""
    r = b * rp
    T = 5
    X = RNG.standard_normal((T, n_in))
    R = RNG.standard_normal((b, r, n_in // b))
    L = RNG.standard_normal((b, n_out // b, r))
    p, q = n_in // b, n_out // b
    Vb = np.zeros((b, p, r)); Ub = np.zeros((b, q, r)); Sb = np.zeros((b, b, r))
    for m in range(b):
        for rho in range(rp):
            e = m * rp + rho
            for j in range(b):
                Vb[j, :, e] = R[j, rho * b + (j + m) % b, :]
            for i in range(b):
                Ub[i, :, e] = L[i, :, ((i - m) % b) * rp + rho]
                for j in range(b):
                    Sb[i, j, e] = 1.0 if m == (i - j) % b else 0.0
    Ym = oracle.monarch_forward(X, R, L, oracle.OUT_BLOCKED)
    Yb = oracle.blast_forward(X, Ub, Sb, Vb)
    np.testing.assert_allclose(Yb, Ym, rtol=1e-12, atol=1e-12)


def test_linearity_and_rows():
    T, n_in, n_out, b, r = 6, 12, 18, 3, 5
    X1, U, S, V = rand_blast(T, n_in, n_out, b, r)
    X2 = RNG.standard_normal((T, n_in))
    f = lambda X: oracle.blast_forward(X, U, S, V)
    np.testing.assert_allclose(f(1.5 * X1 + 4.0 * X2), 1.5 * f(X1) + 4.0 * f(X2), rtol=1e-11, atol=1e-12)
    assert not f(np.zeros((T, n_in))).any()
    order = RNG.permutation(T)
    np.testing.assert_array_equal(f(X1[order]), f(X1)[order])
    np.testing.assert_array_equal(oracle.blast_forward(X1, U, S, V, nthreads=1),
                                  oracle.blast_forward(X1, U, S, V, nthreads=4))


def test_identity_input_block_ranks_and_shared_spaces():
    n_in, n_out, b, r = 12, 20, 2, 3
    _, U, S, V = rand_blast(1, n_in, n_out, b, r)
    W = oracle.materialize_blast(U, S, V)
    np.testing.assert_allclose(oracle.blast_forward(np.eye(n_in), U, S, V), W.T, rtol=1e-12, atol=1e-13)
    q, p = n_in // b, n_out // b
    for i in range(b):
        for j in range(b):
            assert np.linalg.matrix_rank(W[i * p:(i + 1) * p, j * q:(j + 1) * q], tol=1e-9) == r
        # all blocks of output block-row i share the column space of U_i ...
        assert np.linalg.matrix_rank(np.hstack([W[i * p:(i + 1) * p, j * q:(j + 1) * q] for j in range(b)]), tol=1e-9) == r
    for j in range(b):
        # ... and all blocks of input block-column j share the row space of V_j^T
        assert np.linalg.matrix_rank(np.vstack([W[i * p:(i + 1) * p, j * q:(j + 1) * q] for i in range(b)]), tol=1e-9) == r


def test_block_locality():
    T, n_in, n_out, b, r = 3, 12, 18, 3, 5
    X, U, S, V = rand_blast(T, n_in, n_out, b, r)
    q, p = n_in // b, n_out // b
    base = oracle.blast_forward(X, U, S, V)
    for j in range(b):
        X0 = X.copy(); X0[:, j * q:(j + 1) * q] = 0
        V0 = V.copy(); V0[j] = 0
        S0 = S.copy(); S0[:, j, :] = 0
        ref = oracle.blast_forward(X0, U, S, V)
        np.testing.assert_allclose(oracle.blast_forward(X, U, S, V0), ref, rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(oracle.blast_forward(X, U, S0, V), ref, rtol=1e-12, atol=1e-13)
    for i in range(b):
        S0 = S.copy(); S0[i] = 0
        Y = oracle.blast_forward(X, U, S0, V)
        assert not Y[:, i * p:(i + 1) * p].any()
        mask = np.ones(n_out, bool); mask[i * p:(i + 1) * p] = False
        np.testing.assert_array_equal(Y[:, mask], base[:, mask])


@pytest.mark.parametrize("shape", SHAPES)
def test_mac_and_parameter_counts(shape):
    T, n_in, n_out, b, r = shape
    X, U, S, V = rand_blast(*shape)
    _, macs = oracle.blast_forward(X, U, S, V, return_macs=True, nthreads=2)
    assert macs == T * r * (n_in + n_out + b * b)      # n r (i + o + b^2), Section 2.1 / Table 2
    assert U.size + S.size + V.size == r * (n_in + n_out + b * b)


def test_config1_shapes_and_sampled_rows():
    """The ViT-B-width BLAST configuration: factor shapes as stated, and rows generated as a
    sample carry the same values as the corresponding rows of the full activation tensor."""
    import blr_inputs as bi
    cfg = bi.CONFIGS["C1"]
    lay = bi.make_layer(cfg)
    assert lay.U.shape == (16, 48, 96) and lay.V.shape == (16, 48, 96) and lay.S.shape == (16, 16, 96)
    rows = np.array([0, 5, 6303])
    Xs = bi.activations(6304, 768, "bf16", rows=rows)
    Xf = bi.activations(64, 768, "bf16")
    np.testing.assert_array_equal(Xs.bits[:2], Xf.bits[[0, 5]])
    Y = oracle.blast_forward(Xs.f64, lay.U.f64, lay.S.f64, lay.V.f64)
    W = dense_from_definition(lay.U.f64, lay.S.f64, lay.V.f64)
    np.testing.assert_allclose(Y, Xs.f64 @ W, rtol=1e-10, atol=1e-12)
