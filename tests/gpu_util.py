"""Helpers of the GPU parity tests: upload seeded host tensors, call the library through its
Python binding (which calls the C ABI), bring results back as fp64, compare with the oracle."""
import numpy as np
import torch

import blr_inputs as bi
from paper_2512_20861_amd import binding as B

TOL = {"bf16": 2e-2, "f32": 1e-5}     # max|delta| / max|Y_ref|


def to_dev(ht: bi.HostTensor) -> torch.Tensor:
    if ht.dtype == "bf16":
        return torch.from_numpy(ht.bits.view(np.int16).copy()).view(torch.bfloat16).cuda()
    return torch.from_numpy(ht.bits.copy()).cuda()


def to_f64(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        bits = t.view(torch.int16).cpu().numpy().view(np.uint16)
        return bi.bf16_bits_to_f64(bits).reshape(tuple(t.shape))
    return t.cpu().numpy().astype(np.float64)


def empty_out(T, n_out, dtype: str) -> torch.Tensor:
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    # poison the output so that elements the kernel fails to write are caught
    return torch.full((T, n_out), float("nan"), dtype=td, device="cuda")


def rel_err(Y: np.ndarray, Yref: np.ndarray) -> float:
    assert Y.shape == Yref.shape
    assert np.isfinite(Y).all(), "output holds NaN/Inf (unwritten or overflowed elements)"
    return float(np.abs(Y - Yref).max() / max(np.abs(Yref).max(), 1e-300))


def run_monarch(X, lay, flags=0):
    Xd, Rd, Ld = to_dev(X), to_dev(lay.R), to_dev(lay.L)
    Y = empty_out(X.shape[0], lay.n_out, lay.dtype)
    B.monarch_forward(Xd, Rd, Ld, Y, lay.nblocks, lay.r, flags)
    torch.cuda.synchronize()
    return Y


def run_lowrank(X, lay, flags=0):
    Y = empty_out(X.shape[0], lay.n_out, lay.dtype)
    B.lowrank_forward(to_dev(X), to_dev(lay.V), to_dev(lay.U), Y, flags)
    torch.cuda.synchronize()
    return Y


def run_blast_group(X, lays, flags=0):
    """The layers of `lays` (one shape, same input) as one grouped call; returns Y[T][len(lays)*n_out]."""
    l0 = lays[0]
    Xd = to_dev(X)
    Ud = torch.stack([to_dev(l.U) for l in lays], dim=0).contiguous()
    Sd = torch.cat([to_dev(l.S) for l in lays], dim=2).contiguous()
    Vd = torch.cat([to_dev(l.V) for l in lays], dim=2).contiguous()
    packed = B.blast_pack(Ud, Sd, Vd, l0.n_in, l0.n_out, l0.b, len(lays) * l0.r)
    Y = empty_out(X.shape[0], len(lays) * l0.n_out, l0.dtype)
    B.blast_group_forward(Xd, Ud, packed, Y, l0.b, l0.r, len(lays), flags)
    torch.cuda.synchronize()
    return Y


def run_blast(X, lay, flags=0, packed=False):
    Xd, Ud, Sd, Vd = to_dev(X), to_dev(lay.U), to_dev(lay.S), to_dev(lay.V)
    Y = empty_out(X.shape[0], lay.n_out, lay.dtype)
    if packed:
        packed = B.blast_pack(Ud, Sd, Vd, lay.n_in, lay.n_out, lay.b, lay.r)
        B.blast_forward(Xd, Ud, None, packed, Y, lay.b, lay.r, flags | B.BLAST_PACKED)
    else:
        B.blast_forward(Xd, Ud, Sd, Vd, Y, lay.b, lay.r, flags)
    torch.cuda.synchronize()
    return Y
