"""Pins of the chain oracle (CPU only): the glue functions against closed forms and library
routines, the chain against a re-evaluation with materialised dense weights."""
import math
import numpy as np
import scipy.special

import blr_inputs as bi
from oracle import binding as oracle
from oracle import chain as oc


def test_rmsnorm_closed_forms():
    rng = np.random.default_rng(1)
    x = rng.normal(size=(5, 64))
    y = oc.rmsnorm(x, eps=0.0)
    # unit mean square per row; direction preserved; scale invariance
    np.testing.assert_allclose(np.mean(y * y, axis=1), 1.0, rtol=1e-12)
    np.testing.assert_allclose(y * np.sqrt(np.mean(x * x, axis=1, keepdims=True)), x, rtol=1e-12)
    np.testing.assert_allclose(oc.rmsnorm(7.5 * x, eps=0.0), y, rtol=1e-12)
    # a constant row of value c maps to sign(c); eps only matters near zero
    np.testing.assert_allclose(oc.rmsnorm(np.full((1, 8), -3.0), eps=0.0), -1.0, rtol=1e-15)
    np.testing.assert_allclose(oc.rmsnorm(np.zeros((1, 8))), 0.0)
    # eps enters under the root: a row with mean square s gives 1/sqrt(s + eps)
    row = np.array([[2.0, 0.0, 0.0, 0.0]])                      # mean square 1
    np.testing.assert_allclose(oc.rmsnorm(row, eps=3.0)[0, 0], 2.0 / math.sqrt(1.0 + 3.0), rtol=1e-15)


def test_silu_against_library_sigmoid_and_closed_forms():
    x = np.linspace(-20, 20, 401)
    np.testing.assert_allclose(oc.silu(x), x * scipy.special.expit(x), rtol=1e-12, atol=1e-300)
    assert oc.silu(0.0) == 0.0
    np.testing.assert_allclose(oc.silu(1.0), 1.0 / (1.0 + math.exp(-1.0)), rtol=1e-15)
    # silu(x) - silu(-x) = x
    np.testing.assert_allclose(oc.silu(x) - oc.silu(-x), x, rtol=1e-12, atol=1e-12)
    # large |x|: identity on the right, zero on the left
    np.testing.assert_allclose(oc.silu(40.0), 40.0, rtol=1e-15)
    assert abs(oc.silu(-40.0)) < 1e-15


def _dense_linear(x, W):
    return x @ W.T


def _small_chain(op):
    prm = dict(nblocks=4, r_square=16, r_mlp=16) if op == "monarch" else dict(b=4, r_square=8, r_mlp=16)
    layers = bi.chain_layers(op, n_layers=2, hidden=32, mlp=64, params=prm, dtype="f32")
    x0 = bi.activations(6, 32, "f32")
    return layers, x0


def test_chain_equals_dense_reevaluation():
    """The chain through the structured oracle operators equals the same wiring, written out again
    here, through the materialised dense weights (a different evaluation of every linear)."""
    for op in ("monarch", "blast"):
        layers, x0 = _small_chain(op)
        if op == "monarch":
            lin = lambda x, f: oracle.monarch_forward(x, f.R.f64, f.L.f64)
            mat = lambda f: oracle.materialize_monarch(f.R.f64, f.L.f64)
        else:
            lin = lambda x, f: oracle.blast_forward(x, f.U.f64, f.S.f64, f.V.f64)
            mat = lambda f: oracle.materialize_blast(f.U.f64, f.S.f64, f.V.f64)
        trace = []
        h = oc.chain_forward(x0.f64, layers, lin, trace=trace)
        assert len(trace) == 2 and h.shape == (6, 32)
        g = x0.f64.copy()
        for layer in layers:
            W = {k: mat(v) for k, v in layer.items()}
            n1 = g / np.sqrt((g * g).mean(axis=1, keepdims=True) + oc.EPS)
            a = (n1 @ W["q"].T + n1 @ W["k"].T + n1 @ W["v"].T) / math.sqrt(3.0)
            g = g + a @ W["o"].T
            n2 = g / np.sqrt((g * g).mean(axis=1, keepdims=True) + oc.EPS)
            gate = n2 @ W["gate"].T
            g = g + ((gate * scipy.special.expit(gate)) * (n2 @ W["up"].T)) @ W["down"].T
        np.testing.assert_allclose(h, g, rtol=1e-10, atol=1e-12)
        # residual structure: the trace's h of layer 0 feeds layer 1
        np.testing.assert_allclose(trace[1]["n1"], oc.rmsnorm(trace[0]["h"]), rtol=1e-14)


def test_chain_rows_are_independent_and_layers_use_distinct_streams():
    layers, x0 = _small_chain("blast")
    lin = lambda x, f: oracle.blast_forward(x, f.U.f64, f.S.f64, f.V.f64)
    h = oc.chain_forward(x0.f64, layers, lin)
    h_sub = oc.chain_forward(x0.f64[[4, 1]], layers, lin)
    np.testing.assert_allclose(h_sub, h[[4, 1]], rtol=1e-13)
    # no two linears share factor values
    firsts = [float(layers[l][n].U.f64.ravel()[0]) for l in range(2) for n in bi.CHAIN_LINEARS]
    assert len(set(firsts)) == len(firsts)


def test_chain_shapes_of_the_benchmark_configuration():
    c = bi.CHAIN
    assert (c["hidden"], c["mlp"], c["n_layers"], c["T"]) == (2048, 8192, 16, 2048)
    assert bi.chain_linear_shape("gate", 2048, 8192) == (2048, 8192)
    assert bi.chain_linear_shape("down", 2048, 8192) == (8192, 2048)
    assert bi.chain_linear_shape("o", 2048, 8192) == (2048, 2048)
