"""TEST INFRASTRUCTURE (oracle): BLAST forward with a quantised intermediate, plain numpy in fp64.

The paper names the quantisation of intermediate activations as future work (Conclusion, "Limitation and
Future Work") and fixes no format. The reading built here: the first intermediate Z = X_j V_j
(Section 2.1 "BLAST", the product in front of the coupling) is stored as 8-bit floats in the OCP 8-bit
floating point format E4M3 (1 sign, 4 exponent bits with bias 7, 3 mantissa bits, no infinities, largest
finite value 448, subnormals down to 2^-9), rounded to nearest with ties to even and saturating at +-448;
everything else is as in the unquantised operator. Only tests, bench.py's CPU leg and smoke() may import this.

Pins (tests/test_oracle_quant.py): the value grid of the format (126 positive values, the spec's extreme
values), idempotence, monotonicity, hand-worked ties, and PyTorch's float8_e4m3fn cast on random inputs.
"""
from __future__ import annotations

import numpy as np

E4M3_MAX = 448.0          # 1.75 * 2^8
E4M3_MIN_NORMAL = 2.0 ** -6
E4M3_MIN_SUBNORMAL = 2.0 ** -9


def e4m3_round(x: np.ndarray) -> np.ndarray:
    """Nearest E4M3 value of every element (ties to even mantissa), saturating at +-448; fp64 in, fp64 out."""
    x = np.asarray(x, dtype=np.float64)
    a = np.minimum(np.abs(x), E4M3_MAX)
    # spacing of the format around a: 2^(e-3) with e = floor(log2 a), at least the subnormal spacing 2^-9
    e = np.floor(np.log2(np.maximum(a, E4M3_MIN_NORMAL)))
    e = np.clip(e, -6, 8)
    quantum = 2.0 ** (e - 3)
    q = np.rint(a / quantum) * quantum          # np.rint rounds halves to even; a / quantum is exact (power of two)
    return np.copysign(np.minimum(q, E4M3_MAX), x)


def blast_forward_qz(X, U, S, V):
    """Y for BLAST factors U[b][p][r], S[b][b][r] (output block, input block), V[b][q][r] with the first
    intermediate rounded to E4M3:
        Z[t][j][rho] = e4m3( sum_c X[t][j q + c] V[j][c][rho] )
        A[t][i][rho] = sum_j S[i][j][rho] Z[t][j][rho]
        Y[t][i p + a] = sum_rho A[t][i][rho] U[i][a][rho]
    Returns (Y, Z) so that a test can look at the quantised intermediate as well."""
    X, U, S, V = (np.asarray(t, dtype=np.float64) for t in (X, U, S, V))
    T, n_in = X.shape
    b, p, r = U.shape
    q = V.shape[1]
    assert V.shape == (b, q, r) and S.shape == (b, b, r) and b * q == n_in
    Z = np.empty((T, b, r))
    for j in range(b):
        Z[:, j, :] = e4m3_round(X[:, j * q:(j + 1) * q] @ V[j])
    A = np.einsum("ijr,tjr->tir", S, Z)
    Y = np.einsum("tir,iar->tia", A, U).reshape(T, b * p)
    return Y, Z
