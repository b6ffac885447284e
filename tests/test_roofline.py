"""The closed-form traffic model against the paper's Table 2 example and parameter counts (no GPU)."""
import os

from paper_2512_20861_amd import roofline as rf

GOLD = os.path.join(os.path.dirname(__file__), "golden", "table2_example.txt")


def _gold():
    out = {}
    for line in open(GOLD):
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            out[k] = float(v)
    return out


def test_table2_example():
    g = _gold()
    n, i, o, r, b = (int(g[k]) for k in ("n", "i", "o", "r", "b"))
    a = {op: rf.intensity(op, n, i, o, r, b) for op in ("dense", "lowrank", "monarch", "blast")}
    for op in a:
        assert abs(a[op] - g["alpha_" + op]) < 0.01, (op, a[op])
    # ordering stated in the text: dense and low-rank compute-bound, Monarch and BLAST memory-bound on the A40
    assert a["dense"] > a["lowrank"] > g["a40_breakpoint"] > a["monarch"] > a["blast"]


def test_flop_and_parameter_formulas():
    # Section 2.1: Monarch with b1 = b2 = b, r = r'b has r(i+o) parameters; BLAST r(i+o+b^2)
    assert rf.params("monarch", 4096, 4096, 1024, 4) == 1024 * 8192
    assert rf.params("blast", 4096, 4096, 640, 16) == 640 * (8192 + 256)
    assert rf.flops("blast", 10, 768, 768, 96, 16) == 2 * 10 * 96 * (1536 + 256)
    assert rf.flops("dense", 3, 5, 7) == 2 * 3 * 5 * 7
    # the intermediates are what separates Table 2 from the ideal traffic
    n, i, o, r, b = 1024, 4096, 4096, 1024, 16
    assert rf.table2("monarch", n, i, o, r, b)[1] - rf.algorithmic_bytes("monarch", n, i, o, r, b) == 2 * 4 * b * n * r
    assert rf.table2("blast", n, i, o, r, b)[1] - rf.algorithmic_bytes("blast", n, i, o, r, b) == 2 * 8 * b * n * r


def test_bound_flips_with_tokens():
    # Monarch 4096x4096, 4 blocks, r = 1024 on MI355X: weight streaming at small T, MFMA at large T
    assert rf.bound("monarch", 1, 4096, 4096, 1024, 4) == "hbm"
    assert rf.bound("monarch", 128, 4096, 4096, 1024, 4) == "hbm"
    assert rf.bound("monarch", 8192, 4096, 4096, 1024, 4) == "mfma"
    mem, mfma = rf.floors("monarch", 8192, 4096, 4096, 1024, 4)
    assert abs(mem * 1e6 - 18.9) < 0.1 and abs(mfma * 1e6 - 55.0) < 0.1
