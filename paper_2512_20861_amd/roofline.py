"""Closed-form FLOP / byte model of the (B)LR linear layers and the MI355X roofline.

`table2` restates the paper's Table 2 (FLOP and memory traffic per method in 16-bit storage,
including the intermediate round trips of the unfused execution). `algorithmic` is what an
ideal implementation must move: X once, every factor once, Y once - no intermediates.
"""
from __future__ import annotations

HBM_PEAK = 8.0e12          # bytes/s, MI355X HBM3E
MFMA_BF16_PEAK = 2.5e15    # FLOP/s, MI355X dense bf16 MFMA
BREAKPOINT = MFMA_BF16_PEAK / HBM_PEAK


def params(op: str, n_in: int, n_out: int, r: int = 0, b: int = 1) -> int:
    if op == "dense":
        return n_in * n_out
    if op in ("lowrank", "monarch"):
        return r * (n_in + n_out)
    if op == "blast":
        return r * (n_in + n_out + b * b)
    raise ValueError(op)


def flops(op: str, T: int, n_in: int, n_out: int, r: int = 0, b: int = 1) -> int:
    """2 x multiply-adds of the factor-by-factor evaluation (Section 2.1; Table 2, FLOP column)."""
    return 2 * T * params(op, n_in, n_out, r, b)


def table2(op: str, n: int, i: int, o: int, r: int = 0, b: int = 1):
    """(FLOP, bytes) of Table 2 for 16-bit storage: the byte count includes the intermediate
    tensors written and read back by the unfused execution (2nr low-rank, 4bnr Monarch, 8bnr BLAST)."""
    if op == "dense":
        return 2 * n * i * o, 2 * (n * i + i * o + n * o)
    if op == "lowrank":
        return 2 * n * r * (i + o), 2 * (n * i + i * r + r * o + n * o + 2 * n * r)
    if op == "monarch":
        return 2 * n * r * (i + o), 2 * (n * i + i * r + r * o + n * o + 4 * b * n * r)
    if op == "blast":
        return 2 * n * r * (i + o + b * b), 2 * (n * i + i * r + r * o + r * b * b + n * o + 8 * b * n * r)
    raise ValueError(op)


def intensity(op, n, i, o, r=0, b=1) -> float:
    f, m = table2(op, n, i, o, r, b)
    return f / m


def algorithmic_bytes(op: str, T: int, n_in: int, n_out: int, r: int = 0, b: int = 1, elem: int = 2) -> int:
    return elem * (T * n_in + params(op, n_in, n_out, r, b) + T * n_out)


def floors(op: str, T: int, n_in: int, n_out: int, r: int = 0, b: int = 1, elem: int = 2):
    """(memory floor, MFMA floor) in seconds on MI355X for the ideal implementation."""
    return (algorithmic_bytes(op, T, n_in, n_out, r, b, elem) / HBM_PEAK,
            flops(op, T, n_in, n_out, r, b) / MFMA_BF16_PEAK)


def bound(op, T, n_in, n_out, r=0, b=1, elem=2) -> str:
    mem, mfma = floors(op, T, n_in, n_out, r, b, elem)
    return "hbm" if mem >= mfma else "mfma"
