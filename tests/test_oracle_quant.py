"""Pins of the quantised-intermediate oracle (oracle/quant.py): the E4M3 rounding against what the OCP 8-bit
floating point format fixes (value grid, extreme values, round to nearest even, saturation), against
PyTorch's own float8_e4m3fn cast, and the quantised BLAST forward against the plain oracle."""
import numpy as np
import pytest

import blr_inputs as bi
import oracle
from oracle import quant


def e4m3_grid():
    """Every non-negative finite value of the format, from its definition: exponent field E = 0 holds the
    subnormals m * 2^-9, E = 1..15 the normals (1 + m/8) * 2^(E-7); E = 15, m = 7 is the NaN code."""
    vals = [m * 2.0 ** -9 for m in range(8)]
    vals += [(1 + m / 8) * 2.0 ** (E - 7) for E in range(1, 16) for m in range(8) if not (E == 15 and m == 7)]
    return np.array(sorted(set(vals)))


def test_grid_of_the_format():
    g = e4m3_grid()
    assert len(g) == 127 and g[0] == 0.0 and g[1] == 2.0 ** -9 and g[-1] == 448.0
    # every grid value is a fixed point, with either sign
    assert np.array_equal(quant.e4m3_round(g), g)
    assert np.array_equal(quant.e4m3_round(-g), -g)
    # a dense sweep lands on the grid and nowhere else
    x = np.concatenate([np.linspace(0, 500, 200001), np.geomspace(1e-5, 500, 100001)])
    r = quant.e4m3_round(x)
    assert set(np.unique(r)) == set(g)
    # nearest: no grid value is closer than the chosen one
    d = np.abs(np.minimum(x, 448.0)[:, None] - g[None, :]).min(axis=1)
    assert np.allclose(np.abs(np.minimum(x, 448.0) - r), d, rtol=0, atol=1e-15)
    assert np.all(np.diff(r[:200001]) >= 0)                       # monotone


def test_ties_saturation_and_signs():
    f = quant.e4m3_round
    # spacing 2 in [16, 32): 17 lies between 16 (mantissa 0) and 18 (mantissa 1) -> even -> 16; 19 -> 20
    assert f(np.array([17.0, 19.0, 21.0, 23.0])).tolist() == [16.0, 20.0, 20.0, 24.0]
    # spacing 1/8 in [1, 2)
    assert f(np.array([1.0625, 1.1875, 1.06, 1.07])).tolist() == [1.0, 1.25, 1.0, 1.125]
    # subnormals: spacing 2^-9; half of the smallest subnormal ties to zero (even), just above rounds up
    s = 2.0 ** -9
    assert f(np.array([0.5 * s, 0.51 * s, 1.5 * s, 2.5 * s])).tolist() == [0.0, s, 2 * s, 2 * s]
    # boundary between subnormals and normals: 7.5 * 2^-9 ties to 8 * 2^-9 = 2^-6 (even)
    assert f(np.array([7.5 * s])).tolist() == [2.0 ** -6]
    # saturation, no infinities; 464 = halfway to the code that does not exist still gives 448
    assert f(np.array([448.0, 449.0, 464.0, 1e6, np.inf, -1e6])).tolist() == [448.0, 448.0, 448.0, 448.0, 448.0, -448.0]
    assert f(np.array([-17.0, -1.1875, 0.0, -0.0])).tolist() == [-16.0, -1.25, 0.0, 0.0]
    assert np.array_equal(f(f(np.linspace(-460, 460, 9999))), f(np.linspace(-460, 460, 9999)))   # idempotent


def test_against_the_library_cast():
    torch = pytest.importorskip("torch")
    if not hasattr(torch, "float8_e4m3fn"):
        pytest.skip("this PyTorch has no float8_e4m3fn")
    rng = np.random.default_rng(3)
    x = np.concatenate([rng.normal(0, 1, 20000), rng.normal(0, 40, 20000), rng.uniform(-0.03, 0.03, 20000)]).astype(np.float32)
    x = x[np.abs(x) <= 448.0]                                     # the library cast does not saturate
    lib = torch.from_numpy(x).to(torch.float8_e4m3fn).to(torch.float32).numpy().astype(np.float64)
    assert np.array_equal(quant.e4m3_round(x.astype(np.float64)), lib)


def test_quantised_forward_reduces_to_the_plain_oracle():
    """With factors and inputs for which every Z is exactly an E4M3 value the quantised forward IS the plain
    forward; in general it differs from it by no more than the rounding of Z allows."""
    rng = np.random.default_rng(5)
    b, q, p, r, T = 4, 8, 6, 16, 9
    # small integers: Z = sum of q products of values in {-1, 0, 1} is an integer of magnitude <= 8, an E4M3 value
    X = rng.integers(-1, 2, (T, b * q)).astype(np.float64)
    V = rng.integers(-1, 2, (b, q, r)).astype(np.float64)
    S = rng.normal(size=(b, b, r))
    U = rng.normal(size=(b, p, r))
    Yq, Z = quant.blast_forward_qz(X, U, S, V)
    assert np.array_equal(quant.e4m3_round(Z), Z) and np.abs(Z).max() <= 8
    assert np.allclose(Yq, oracle.blast_forward(X, U, S, V), rtol=1e-12, atol=1e-12)
    # general values: |Z - e4m3(Z)| <= 2^-4 |Z| for normal Z, so |Y - Yq| <= 2^-4 sum |S| |Z| |U|
    lay = bi.blast_layer(128, 96, 4, 32, "bf16", seed=7)
    Xh = bi.activations(11, 128, "bf16", seed=8).f64
    Yq, Z = quant.blast_forward_qz(Xh, lay.U.f64, lay.S.f64, lay.V.f64)
    Y = oracle.blast_forward(Xh, lay.U.f64, lay.S.f64, lay.V.f64)
    bound = np.einsum("tir,iar->tia", np.einsum("ijr,tjr->tir", np.abs(lay.S.f64), np.abs(Z) * 2.0 ** -4 + 2.0 ** -10),
                      np.abs(lay.U.f64)).reshape(Y.shape)
    assert np.all(np.abs(Y - Yq) <= bound + 1e-12)
    assert np.abs(Y - Yq).max() > 0                              # the rounding is really there
