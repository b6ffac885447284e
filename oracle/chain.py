"""CPU oracle of the decoder-layer linear chain (seven BLR linears per layer, no attention).

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT (see blr_oracle.cpp). Plain numpy in fp64; the linears
are the fp64 oracle operators. The paper replaces the Q/O projections and the MLP of Llama decoder
layers with BLR linears (Section 5, "Llama") but defines no attention-free chain, so the wiring below
is this build's reading of the benchmark configuration, chosen so that activations keep unit scale
through 112 chained linears:

    n1 = rmsnorm(h);  a = (W_q n1 + W_k n1 + W_v n1) / sqrt(3);  h = h + W_o a
    n2 = rmsnorm(h);  h = h + W_down( silu(W_gate n2) * W_up n2 )

rmsnorm has no weight: x / sqrt(mean(x^2) + eps) over the feature axis; silu(x) = x / (1 + exp(-x)).
No intermediate is rounded. Parity pins: tests/test_oracle_chain.py (closed forms of the glue
functions; the chain against a dense re-evaluation with materialised weights).
"""
import numpy as np

EPS = 1e-6


def rmsnorm(h, eps=EPS):
    h = np.asarray(h, dtype=np.float64)
    return h / np.sqrt(np.mean(h * h, axis=-1, keepdims=True) + eps)


def silu(x):
    x = np.asarray(x, dtype=np.float64)
    return x / (1.0 + np.exp(-x))


def layer_forward(h, layer, linear, eps=EPS, trace=None):
    """One decoder layer. `layer` maps q,k,v,o,gate,up,down to whatever `linear(x, factors)` accepts."""
    n1 = rmsnorm(h, eps)
    q, k, v = linear(n1, layer["q"]), linear(n1, layer["k"]), linear(n1, layer["v"])
    a = (q + k + v) / np.sqrt(3.0)
    o = linear(a, layer["o"])
    h = h + o
    n2 = rmsnorm(h, eps)
    g, u = linear(n2, layer["gate"]), linear(n2, layer["up"])
    m = silu(g) * u
    d = linear(m, layer["down"])
    h = h + d
    if trace is not None:
        trace.append(dict(n1=n1, q=q, k=k, v=v, a=a, o=o, n2=n2, g=g, u=u, m=m, d=d, h=h))
    return h


def chain_forward(x0, layers, linear, eps=EPS, trace=None):
    h = np.asarray(x0, dtype=np.float64)
    for layer in layers:
        h = layer_forward(h, layer, linear, eps, trace)
    return h
