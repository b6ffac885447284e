"""The pins must notice a plausible mistake anywhere in the oracle: each case below plants one (a
transposed operand, a wrong storage order, a swapped index, a dropped term, a wrong sign) in a COPY of
the oracle's source, builds it, and runs the oracle's own pin tests against that build in a child
process; at least one pin has to fail. The unaltered copy has to pass the same way. Nothing here
touches the GPU library."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(ROOT, "oracle", "blr_oracle.cpp")

MONARCH, RECT, BLAST, LOWRANK = ("test_oracle_monarch.py", "test_oracle_monarch_rect.py",
                                 "test_oracle_blast.py", "test_oracle_lowrank.py")

# (name, pin files that must notice, text in the source, replacement); every alteration keeps all indices in range
MISTAKES = [
    ("dense: weight read transposed", [MONARCH, BLAST, LOWRANK],
     "acc += X[t * n_in + a] * W[(int64_t)o * n_in + a];", "acc += X[t * n_in + a] * W[(int64_t)a * n_out + o];"),
    ("monarch: first factor's rows taken block-major instead of rank-major", [MONARCH],
     "= Z[(size_t)l * r + rho * b + k];", "= Z[(size_t)l * r + k * rp + rho];"),
    ("monarch: middle vector written rank-major instead of block-major", [MONARCH],
     "Zp[(size_t)k * r + l * rp + rho] =", "Zp[(size_t)k * r + rho * b + l] ="),
    ("monarch: output block and position swapped", [MONARCH],
     "y[o] = Yb[(size_t)k * q + j];", "y[o] = Yb[(size_t)(k * q + j) % b * q + (k * q + j) / b];"),
    ("monarch: first term of the second product dropped", [MONARCH],
     "for (int m = 0; m < r; ++m) acc += Zp[(size_t)k * r + m] * row[m];", "for (int m = 1; m < r; ++m) acc += Zp[(size_t)k * r + m] * row[m];"),
    ("monarch: materialised weight reads the second factor in the other order", [MONARCH],
     "L[((int64_t)k * q + j) * r + l * rp + rho];", "L[((int64_t)k * q + j) * r + rho * b + l];"),
    ("general monarch: first factor's rows taken block-major", [RECT],
     "= Z[(size_t)l * w1 + rho * b2 + k];", "= Z[(size_t)l * w1 + k * rp + rho];"),
    ("general monarch: middle vector written rank-major", [RECT],
     "Zp[(size_t)k * w2 + l * rp + rho] =", "Zp[(size_t)k * w2 + rho * b1 + l] ="),
    ("blast: coupling read transposed (s_ji for s_ij)", [BLAST],
     "const double* s = S + ((int64_t)i * b + j) * r;", "const double* s = S + ((int64_t)j * b + i) * r;"),
    ("blast: coupling subtracted", [BLAST],
     "a[rho] += s[rho] * z[rho];", "a[rho] -= s[rho] * z[rho];"),
    ("blast: right factor read as [block][rank][column]", [BLAST],
     "z[rho] += xv * vrow[rho];", "z[rho] += xv * V[((int64_t)j * r + rho) * q + c];"),
    ("blast: left factor read as [block][rank][row]", [BLAST],
     "for (int rho = 0; rho < r; ++rho) acc += av[rho] * urow[rho];", "for (int rho = 0; rho < r; ++rho) acc += av[rho] * U[((int64_t)i * r + rho) * p + a];"),
    ("blast: first input block left out of the coupling", [BLAST],
     "for (int j = 0; j < b; ++j) {\n                    const double* s = S", "for (int j = 1; j < b; ++j) {\n                    const double* s = S"),
    ("blast: materialised weight couples with s_ji", [BLAST],
     "S[((int64_t)i * b + j) * r + rho] *", "S[((int64_t)j * b + i) * r + rho] *"),
    ("low-rank: right factor read transposed", [LOWRANK],
     "for (int a = 0; a < n_in; ++a) acc += x[a] * vrow[a];", "for (int a = 0; a < n_in; ++a) acc += x[a] * V[(int64_t)a * r + c];"),
    ("low-rank: first rank index dropped from the second product", [LOWRANK],
     "for (int c = 0; c < r; ++c) acc += Z[c] * urow[c];", "for (int c = 1; c < r; ++c) acc += Z[c] * urow[c];"),
    ("low-rank: materialised weight reads the left factor transposed", [LOWRANK],
     "acc += U[(int64_t)o * r + c] * V[(int64_t)c * n_in + a];", "acc += U[(int64_t)c * n_out + o] * V[(int64_t)c * n_in + a];"),
]


def _build(text, path):
    src = path + ".cpp"
    with open(src, "w") as f:
        f.write(text)
    subprocess.check_call(["g++", "-O1", "-std=c++17", "-shared", "-fPIC", "-pthread", src, "-o", path])


def _pins_pass(lib, files):
    env = dict(os.environ, BLR_ORACLE_LIB=lib)
    res = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] +
                         [os.path.join(HERE, f) for f in files], cwd=ROOT, env=env, capture_output=True, text=True)
    assert res.returncode in (0, 1), res.stdout[-2000:] + res.stderr[-2000:]   # 1 = tests failed; anything else is a broken run
    return res.returncode == 0


def test_every_planted_mistake_fails_a_pin(tmp_path):
    source = open(SRC).read()
    for name, _, old, new in MISTAKES:
        assert source.count(old) == 1, f"{name}: the text to alter must occur exactly once"

    def run(case):
        k, (name, files, old, new) = case
        lib = str(tmp_path / f"altered_{k}.so")
        _build(source.replace(old, new), lib)
        return name, _pins_pass(lib, files)

    with ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(run, enumerate(MISTAKES)))
    unnoticed = [name for name, passed in results if passed]
    assert not unnoticed, f"no pin noticed: {unnoticed}"


def test_the_unaltered_copy_passes_the_same_way(tmp_path):
    lib = str(tmp_path / "unaltered.so")
    _build(open(SRC).read(), lib)
    assert _pins_pass(lib, [MONARCH, RECT, BLAST, LOWRANK])
