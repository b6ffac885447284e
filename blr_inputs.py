"""Seeded synthetic inputs for the BLR linear forward path.

This module is the only code shared by the CPU oracle's tests and the GPU
library's tests/benchmark. It holds no arithmetic of the method itself: it
draws i.i.d. Gaussian tensors from a counter-based generator, scales them,
rounds them to the storage type (bf16 round-to-nearest-even, or fp32) and
hands back both the stored bit pattern (what is uploaded to the GPU) and the
exact fp64 value of that bit pattern (what the oracle consumes). The GPU never
generates numbers, so both sides see identical inputs.

Generator: element k of tensor `tid` under base seed `seed` uses the two
64-bit words splitmix64(key + 2k), splitmix64(key + 2k + 1), with
key = splitmix64(seed ^ (tid * 0xD1342543DE82EF95)), mapped to uniforms and to
one standard normal by the Box-Muller transform, all in fp64.

The layer recipes follow the benchmark configurations: Gaussian factors scaled
by 1/sqrt(fan-in of the block) (Monarch) or 1/sqrt(r) (BLAST), X ~ N(0,1),
shapes taken from the paper's Table 3 layer list (Llama-7B, Llama-3.2-1B,
ViT-B/GPT2-S widths). They stand in for the trained, compressed models the
paper measures, which are not available offline; kernel run time does not
depend on values.
"""
from __future__ import annotations

import math
import os
from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 20861
_M64 = (1 << 64) - 1
_CHUNK = 1 << 22


def _splitmix64_scalar(x: int) -> int:
    z = (x + 0x9E3779B97F4A7C15) & _M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    return z ^ (z >> 31)


def _splitmix64(x: np.ndarray) -> np.ndarray:
    with np.errstate(over="ignore"):
        z = x + np.uint64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        return z ^ (z >> np.uint64(31))


def standard_normal(seed: int, tid: int, index: np.ndarray) -> np.ndarray:
    """N(0,1) draws (fp64) for the flat element indices `index` of tensor `tid`."""
    key = np.uint64(_splitmix64_scalar((seed ^ (tid * 0xD1342543DE82EF95)) & _M64))
    idx = index.astype(np.uint64, copy=False)
    with np.errstate(over="ignore"):
        h1 = _splitmix64(key + idx * np.uint64(2))
        h2 = _splitmix64(key + idx * np.uint64(2) + np.uint64(1))
    u1 = ((h1 >> np.uint64(11)).astype(np.float64) + 1.0) * (1.0 / 9007199254740992.0)
    u2 = (h2 >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)
    return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * math.pi * u2)


def round_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp64 -> bf16 bit pattern (uint16), round to nearest even via fp32."""
    bits = x.astype(np.float32).view(np.uint32)
    rounded = bits + np.uint32(0x7FFF) + ((bits >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


@dataclass
class HostTensor:
    """A stored tensor: `bits` is what goes to the GPU (uint16 for bf16, float32
    for fp32); `f64` is the exact value of those bits."""
    dtype: str
    bits: np.ndarray
    f64: np.ndarray

    @property
    def shape(self):
        return self.bits.shape


def store(values: np.ndarray, dtype: str) -> HostTensor:
    """Round an fp64 array to the storage type."""
    if dtype == "bf16":
        bits = round_to_bf16_bits(values)
        return HostTensor(dtype, bits, bf16_bits_to_f64(bits).reshape(values.shape))
    if dtype == "f32":
        f = values.astype(np.float32)
        return HostTensor(dtype, f, f.astype(np.float64))
    raise ValueError(dtype)


def gaussian(seed: int, tid: int, shape, scale: float, dtype: str, rows=None) -> HostTensor:
    """Tensor of N(0,1)*scale entries. `rows` (optional, 1-D int array) selects
    rows of the leading dimension of the full tensor, so that samples of a large
    tensor carry exactly the values the full tensor would."""
    shape = tuple(int(s) for s in shape)
    inner = int(np.prod(shape[1:])) if len(shape) > 1 else 1
    lead = np.arange(shape[0], dtype=np.int64) if rows is None else np.asarray(rows, dtype=np.int64)
    out_shape = (len(lead),) + shape[1:]
    n = len(lead) * inner
    bits = np.empty(n, dtype=np.uint16 if dtype == "bf16" else np.float32)
    vals = np.empty(n, dtype=np.float64)
    col = np.arange(inner, dtype=np.int64)
    rows_per_chunk = max(1, _CHUNK // max(inner, 1))
    for r0 in range(0, len(lead), rows_per_chunk):
        r1 = min(len(lead), r0 + rows_per_chunk)
        idx = (lead[r0:r1, None] * inner + col[None, :]).reshape(-1)
        ht = store(standard_normal(seed, tid, idx) * scale, dtype)
        bits[r0 * inner:r1 * inner] = ht.bits
        vals[r0 * inner:r1 * inner] = ht.f64
    return HostTensor(dtype, bits.reshape(out_shape), vals.reshape(out_shape))


# tensor ids of the per-tensor random streams
TID_X, TID_R, TID_L, TID_U, TID_S, TID_V, TID_W, TID_LRV, TID_LRU = 1, 2, 3, 4, 5, 6, 7, 8, 9


@dataclass
class MonarchLayer:
    n_in: int
    n_out: int
    nblocks: int
    r: int
    dtype: str
    R: HostTensor = field(repr=False, default=None)
    L: HostTensor = field(repr=False, default=None)


@dataclass
class BlastLayer:
    n_in: int
    n_out: int
    b: int
    r: int
    dtype: str
    U: HostTensor = field(repr=False, default=None)
    S: HostTensor = field(repr=False, default=None)
    V: HostTensor = field(repr=False, default=None)


@dataclass
class LowRankLayer:
    n_in: int
    n_out: int
    r: int
    dtype: str
    V: HostTensor = field(repr=False, default=None)
    U: HostTensor = field(repr=False, default=None)


def lowrank_layer(n_in, n_out, r, dtype, seed=BASE_SEED, layer_id=0):
    """V[r][n_in] ~ N(0,1)/sqrt(n_in), U[n_out][r] ~ N(0,1)/sqrt(r)."""
    off = 16 * layer_id
    return LowRankLayer(n_in, n_out, r, dtype,
                        V=gaussian(seed, TID_LRV + off, (r, n_in), 1.0 / math.sqrt(n_in), dtype),
                        U=gaussian(seed, TID_LRU + off, (n_out, r), 1.0 / math.sqrt(r), dtype))


def monarch_layer(n_in, n_out, nblocks, r, dtype, seed=BASE_SEED, scale_R=None, scale_L=None, layer_id=0):
    """R[nblocks][r][n_in/nblocks] ~ N(0,1)/sqrt(n_in/nblocks), L[nblocks][n_out/nblocks][r] ~ N(0,1)/sqrt(r)."""
    p, q = n_in // nblocks, n_out // nblocks
    sR = 1.0 / math.sqrt(p) if scale_R is None else scale_R
    sL = 1.0 / math.sqrt(r) if scale_L is None else scale_L
    off = 16 * layer_id
    return MonarchLayer(n_in, n_out, nblocks, r, dtype,
                        R=gaussian(seed, TID_R + off, (nblocks, r, p), sR, dtype),
                        L=gaussian(seed, TID_L + off, (nblocks, q, r), sL, dtype))


def blast_layer(n_in, n_out, b, r, dtype, seed=BASE_SEED, layer_id=0):
    """U[b][n_out/b][r], S[b][b][r], V[b][n_in/b][r], all ~ N(0,1)/sqrt(r)."""
    q, p = n_in // b, n_out // b
    s = 1.0 / math.sqrt(r)
    off = 16 * layer_id
    return BlastLayer(n_in, n_out, b, r, dtype,
                      U=gaussian(seed, TID_U + off, (b, p, r), s, dtype),
                      S=gaussian(seed, TID_S + off, (b, b, r), s, dtype),
                      V=gaussian(seed, TID_V + off, (b, q, r), s, dtype))


def activations(T, n_in, dtype, seed=BASE_SEED, scale=1.0, rows=None) -> HostTensor:
    return gaussian(seed, TID_X, (T, n_in), scale, dtype, rows=rows)


def dense_weight(n_in, n_out, dtype, seed=BASE_SEED) -> HostTensor:
    return gaussian(seed, TID_W, (n_out, n_in), 1.0 / math.sqrt(n_in), dtype)


# The benchmark configurations. T sweeps are given where the configuration names one.
T_SWEEP = (1, 16, 128, 512, 2048, 8192)
CONFIGS = {
    # Monarch 256x256, 4 blocks of 64x64, fp32, T=8; all entries N(0,1)/sqrt(64)
    "C0": dict(op="monarch", n_in=256, n_out=256, nblocks=4, r=64, dtype="f32", T=(8,), x_scale=1.0 / 8.0),
    # BLAST at ViT-B / GPT2-S width, 197 tokens x batch 32
    "C1": dict(op="blast", n_in=768, n_out=768, b=16, r=96, dtype="bf16", T=(6304,), x_scale=1.0),
    # Monarch, Llama-7B attention projection and MLP up
    "C2a": dict(op="monarch", n_in=4096, n_out=4096, nblocks=4, r=1024, dtype="bf16", T=T_SWEEP, x_scale=1.0),
    "C2b": dict(op="monarch", n_in=4096, n_out=11008, nblocks=4, r=1024, dtype="bf16", T=T_SWEEP, x_scale=1.0),
    # BLAST, Llama-7B attention projection and MLP down
    "C3a": dict(op="blast", n_in=4096, n_out=4096, b=16, r=640, dtype="bf16", T=T_SWEEP, x_scale=1.0),
    "C3b": dict(op="blast", n_in=11008, n_out=4096, b=16, r=1024, dtype="bf16", T=T_SWEEP, x_scale=1.0),
    # plain low-rank at the attention-projection shape: the rank of the roofline example (Section 3,
    # Table 2) and the small rank at which full fusion pays on the paper's hardware (Appendix, Full Fusion)
    "LRa": dict(op="lowrank", n_in=4096, n_out=4096, r=1024, dtype="bf16", T=T_SWEEP, x_scale=1.0),
    "LRb": dict(op="lowrank", n_in=4096, n_out=4096, r=128, dtype="bf16", T=T_SWEEP, x_scale=1.0),
}


# Layer shapes of the paper's Table 3 (Appendix, Layer Details): (model, layer, n_in, n_out, tokens,
# {method: (r, b)}); for Monarch r is the paper's r (per-block rank r' = r / b), which is also the
# width of one middle block at the library boundary. The token count n is "determined by the model
# and application" in the paper and not printed: 1024 (the roofline example's n) for the language
# models, 197 for ViT-B, 256 for DiT-XL/2 are this build's stand-ins.
TABLE3 = (
    ("Llama-7B", "qkvo_proj", 4096, 4096, 1024, {"lowrank": (1024, 1), "monarch": (1024, 16), "blast": (1024, 16)}),
    ("Llama-7B", "gate_up_proj", 4096, 11008, 1024, {"lowrank": (1488, 1), "monarch": (1536, 16), "blast": (1488, 16)}),
    ("Llama-7B", "down_proj", 11008, 4096, 1024, {"lowrank": (1488, 1), "monarch": (1536, 16), "blast": (1488, 16)}),
    ("Llama-3.2-1B", "qo_proj", 2048, 2048, 1024, {"lowrank": (256, 1), "monarch": (256, 16), "blast": (256, 16)}),
    ("Llama-3.2-1B", "gate_proj", 2048, 8192, 1024, {"lowrank": (512, 1), "monarch": (512, 16), "blast": (512, 16)}),
    ("Llama-3.2-1B", "up_proj", 2048, 8192, 1024, {"lowrank": (768, 1), "monarch": (768, 16), "blast": (768, 16)}),
    ("Llama-3.2-1B", "down_proj", 8192, 2048, 1024, {"lowrank": (768, 1), "monarch": (768, 16), "blast": (768, 16)}),
    ("GPT2-S", "c_attn", 768, 2304, 1024, {"lowrank": (192, 1), "monarch": (192, 4), "blast": (192, 6)}),
    ("GPT2-S", "c_fc", 768, 3072, 1024, {"lowrank": (192, 1), "monarch": (192, 4), "blast": (192, 6)}),
    ("GPT2-S", "c_proj", 3072, 768, 1024, {"lowrank": (192, 1), "monarch": (192, 4), "blast": (192, 6)}),
    ("ViT-B", "attn_qkv", 768, 2304, 197, {"lowrank": (128, 1), "monarch": (128, 4), "blast": (128, 3)}),
    ("ViT-B", "fc1", 768, 3072, 197, {"lowrank": (128, 1), "monarch": (128, 4), "blast": (128, 3)}),
    ("ViT-B", "fc2", 3072, 768, 197, {"lowrank": (128, 1), "monarch": (128, 4), "blast": (128, 3)}),
    ("DiT-XL/2", "qkv_proj", 1152, 3456, 256, {"lowrank": (384, 1), "blast": (384, 9)}),
    ("DiT-XL/2", "fc1", 1152, 4608, 256, {"lowrank": (256, 1), "blast": (256, 9)}),
    ("DiT-XL/2", "adaLN_proj", 1152, 6912, 256, {"lowrank": (256, 1), "blast": (256, 9)}),
)


def table3_cfg(row, method: str) -> dict:
    """Configuration dictionary (as in CONFIGS) of one Table 3 row and method."""
    _, _, n_in, n_out, n, methods = row
    r, b = methods[method]
    cfg = dict(op=method, n_in=n_in, n_out=n_out, r=r, dtype="bf16", T=(n,), x_scale=1.0)
    if method == "monarch":
        cfg["nblocks"] = b
    elif method == "blast":
        cfg["b"] = b
    return cfg


def make_layer(cfg: dict, seed=BASE_SEED, layer_id=0):
    if cfg["op"] == "lowrank":
        return lowrank_layer(cfg["n_in"], cfg["n_out"], cfg["r"], cfg["dtype"], seed, layer_id=layer_id)
    if cfg["op"] == "monarch":
        return monarch_layer(cfg["n_in"], cfg["n_out"], cfg["nblocks"], cfg["r"], cfg["dtype"], seed, layer_id=layer_id)
    return blast_layer(cfg["n_in"], cfg["n_out"], cfg["b"], cfg["r"], cfg["dtype"], seed, layer_id=layer_id)


# Decoder-layer linear chain at Llama-1B width: seven BLR linears per layer (q, k, v, o square;
# gate, up hidden -> mlp; down mlp -> hidden), no attention.
CHAIN = dict(hidden=2048, mlp=8192, n_layers=16, T=2048, dtype="bf16",
             monarch=dict(nblocks=4, r_square=512, r_mlp=512),
             blast=dict(b=16, r_square=256, r_mlp=512))
CHAIN_LINEARS = ("q", "k", "v", "o", "gate", "up", "down")


def chain_linear_shape(name: str, hidden: int, mlp: int):
    """(n_in, n_out) of one of the seven linears of a layer."""
    if name in ("gate", "up"):
        return hidden, mlp
    if name == "down":
        return mlp, hidden
    return hidden, hidden


def chain_layers(op: str, n_layers=None, hidden=None, mlp=None, seed=BASE_SEED, params=None, dtype=None):
    """Factors of every linear of the chain: a list (one entry per layer) of dicts name -> layer.
    Every linear draws from its own random streams (layer_id = 1 + 7 * layer + position)."""
    c = CHAIN
    n_layers = c["n_layers"] if n_layers is None else n_layers
    hidden = c["hidden"] if hidden is None else hidden
    mlp = c["mlp"] if mlp is None else mlp
    dtype = c["dtype"] if dtype is None else dtype
    prm = dict(c[op]) if params is None else dict(params)
    def make(item):
        l, pos, name = item
        n_in, n_out = chain_linear_shape(name, hidden, mlp)
        r = prm["r_square"] if n_in == n_out else prm["r_mlp"]
        lid = 1 + 7 * l + pos
        if op == "monarch":
            return monarch_layer(n_in, n_out, prm["nblocks"], r, dtype, seed, layer_id=lid)
        return blast_layer(n_in, n_out, prm["b"], r, dtype, seed, layer_id=lid)

    items = [(l, pos, name) for l in range(n_layers) for pos, name in enumerate(CHAIN_LINEARS)]
    # every tensor is a pure function of (seed, stream id, element index): generation order is free,
    # and numpy releases the interpreter lock inside its array kernels
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as ex:
        made = list(ex.map(make, items))
    out = [dict() for _ in range(n_layers)]
    for (l, _, name), lay in zip(items, made):
        out[l][name] = lay
    return out
