"""Seeded random shapes through every dispatch regime (few tokens, every tile size, partial tiles in
all three GEMM dimensions, partial last k-step, batched/scattered outputs), each against the oracle."""
import numpy as np
import pytest

import blr_inputs as bi
import oracle

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2512_20861_amd import binding
    binding.lib()


def _gu():
    import gpu_util
    return gpu_util


def _dense_shapes():
    rng = np.random.default_rng(20861)
    out = []
    for _ in range(28):
        M = int(rng.choice([1, 3, 16, 17, 31, 32, 33, 64, 65, 127, 129, 200, 300, 513, 700]))
        N = int(rng.integers(1, 140)) * 8
        K = int(rng.integers(1, 140)) * 8
        out.append((M, K, N))
    out += [(1100, 264, 2056), (260, 1048, 264), (33, 8, 8), (2, 4096, 16)]
    return out


@pytest.mark.parametrize("T,n_in,n_out", _dense_shapes())
def test_dense_random_shape(T, n_in, n_out):
    gu = _gu()
    W = bi.dense_weight(n_in, n_out, "bf16", seed=T * 131 + n_in)
    X = bi.activations(T, n_in, "bf16", seed=n_out)
    Y = gu.empty_out(T, n_out, "bf16")
    gu.B.dense_reference_forward(gu.to_dev(X), gu.to_dev(W), Y)
    torch.cuda.synchronize()
    err = gu.rel_err(gu.to_f64(Y), oracle.dense_forward(X.f64, W.f64))
    assert err <= gu.TOL["bf16"], (T, n_in, n_out, err)


def _dense_large_shapes():
    """Enough tiles for the large-tile rules: several rounds of workgroups, a last round split off along rows or columns,
    ragged token and column counts, contraction lengths with a partial last step of 64."""
    rng = np.random.default_rng(4096)
    out = []
    for _ in range(12):
        M = int(rng.integers(1500, 9000))
        N = int(rng.integers(128, 750)) * 8
        K = int(rng.integers(17, 88)) * 8
        out.append((M, K, N))
    return out


@pytest.mark.parametrize("T,n_in,n_out", _dense_large_shapes())
def test_dense_random_large_shape(T, n_in, n_out):
    gu = _gu()
    W = bi.dense_weight(n_in, n_out, "bf16", seed=T * 7 + n_out)
    X = bi.activations(T, n_in, "bf16", seed=n_in)
    Y = gu.empty_out(T, n_out, "bf16")
    gu.B.dense_reference_forward(gu.to_dev(X), gu.to_dev(W), Y)
    torch.cuda.synchronize()
    out = gu.to_f64(Y)
    assert np.isfinite(out).all()
    err = gu.rel_err(out, oracle.dense_forward(X.f64, W.f64))
    assert err <= gu.TOL["bf16"], (T, n_in, n_out, err)


def _monarch_shapes():
    rng = np.random.default_rng(7)
    out = []
    for _ in range(16):
        b = int(rng.choice([1, 2, 3, 4, 8]))
        p, q, rp = (int(rng.integers(1, 40)) * 8 for _ in range(3))
        T = int(rng.choice([1, 5, 16, 30, 33, 100, 257, 600]))
        out.append((T, b * p, b * q, b, b * rp))
    return out


@pytest.mark.parametrize("T,n_in,n_out,nb,r", _monarch_shapes())
@pytest.mark.parametrize("order", ["interleaved", "blocked"])
def test_monarch_random_shape(T, n_in, n_out, nb, r, order):
    gu = _gu()
    lay = bi.monarch_layer(n_in, n_out, nb, r, "bf16", seed=T + n_in)
    X = bi.activations(T, n_in, "bf16", seed=r)
    blocked = order == "blocked"
    Y = gu.to_f64(gu.run_monarch(X, lay, gu.B.MONARCH_OUT_BLOCKED if blocked else 0))
    Yref = oracle.monarch_forward(X.f64, lay.R.f64, lay.L.f64, oracle.OUT_BLOCKED if blocked else oracle.OUT_INTERLEAVED)
    err = gu.rel_err(Y, Yref)
    assert err <= gu.TOL["bf16"], (T, n_in, n_out, nb, r, order, err)


def _blast_shapes():
    rng = np.random.default_rng(11)
    out = []
    for _ in range(16):
        b = int(rng.choice([1, 2, 4, 5, 8, 16]))
        q, p = (int(rng.integers(1, 24)) * 8 for _ in range(2))
        r = int(rng.integers(1, 60)) * 8
        T = int(rng.choice([1, 7, 16, 33, 100, 129, 300, 1100]))
        out.append((T, b * q, b * p, b, r))
    return out


@pytest.mark.parametrize("T,n_in,n_out,b,r", _blast_shapes())
@pytest.mark.parametrize("mode", ["packed", "fused12", "three"])
def test_blast_random_shape(T, n_in, n_out, b, r, mode):
    gu = _gu()
    lay = bi.blast_layer(n_in, n_out, b, r, "bf16", seed=T + r)
    X = bi.activations(T, n_in, "bf16", seed=n_in)
    flags = {"fused12": gu.B.BLAST_FUSED_STAGE12, "three": gu.B.BLAST_THREE_KERNELS}.get(mode, 0)
    Y = gu.to_f64(gu.run_blast(X, lay, flags, packed=True))
    err = gu.rel_err(Y, oracle.blast_forward(X.f64, lay.U.f64, lay.S.f64, lay.V.f64))
    assert err <= gu.TOL["bf16"], (T, n_in, n_out, b, r, mode, err)


def _lowrank_shapes():
    # narrow ranks with long contraction indices and few tiles hit the split contraction; the rest the plain tiles
    rng = np.random.default_rng(29)
    out = []
    for _ in range(16):
        T = int(rng.choice([1, 7, 33, 64, 100, 130, 300, 520, 900]))
        n_in = int(rng.integers(8, 400)) * 8
        n_out = int(rng.integers(1, 200)) * 8
        r = int(rng.choice([8, 16, 40, 64, 96, 128, 200, 256, 384]))
        out.append((T, n_in, n_out, r))
    out += [(512, 4096, 512, 128), (96, 8192, 64, 64), (40, 1000, 1000, 24)]
    return out


@pytest.mark.parametrize("T,n_in,n_out,r", _lowrank_shapes())
def test_lowrank_random_shape(T, n_in, n_out, r):
    gu = _gu()
    lay = bi.lowrank_layer(n_in, n_out, r, "bf16", seed=T + n_out)
    X = bi.activations(T, n_in, "bf16", seed=r + 1)
    Y = gu.to_f64(gu.run_lowrank(X, lay))
    err = gu.rel_err(Y, oracle.lowrank_forward(X.f64, lay.V.f64, lay.U.f64))
    assert err <= gu.TOL["bf16"], (T, n_in, n_out, r, err)


def _monarch_rect_shapes():
    rng = np.random.default_rng(37)
    out = []
    for _ in range(16):
        b1, b2 = int(rng.choice([1, 2, 3, 4, 8, 16])), int(rng.choice([1, 2, 3, 4, 6, 9, 16]))
        p, q = int(rng.integers(1, 30)) * 8, int(rng.integers(1, 30)) * 8
        rp = int(rng.choice([8, 16, 24, 32, 64]))
        T = int(rng.choice([1, 5, 16, 33, 100, 257, 600]))
        out.append((T, b1 * p, b2 * q, b1, b2, rp))
    return out


@pytest.mark.parametrize("T,n_in,n_out,b1,b2,rp", _monarch_rect_shapes())
@pytest.mark.parametrize("order", ["interleaved", "blocked"])
def test_monarch_rect_random_shape(T, n_in, n_out, b1, b2, rp, order):
    gu = _gu()
    p, q = n_in // b1, n_out // b2
    R = bi.gaussian(T + n_in, 41, (b1, rp * b2, p), 1.0 / np.sqrt(p), "bf16")
    L = bi.gaussian(T + n_in, 42, (b2, q, b1 * rp), 1.0 / np.sqrt(b1 * rp), "bf16")
    X = bi.activations(T, n_in, "bf16", seed=rp)
    blocked = order == "blocked"
    Y = gu.empty_out(T, n_out, "bf16")
    gu.B.monarch_rect_forward(gu.to_dev(X), gu.to_dev(R), gu.to_dev(L), Y, b1, b2, rp, gu.B.MONARCH_OUT_BLOCKED if blocked else 0)
    torch.cuda.synchronize()
    Yref = oracle.monarch_rect_forward(X.f64, R.f64, L.f64, b1, b2, oracle.OUT_BLOCKED if blocked else oracle.OUT_INTERLEAVED)
    err = gu.rel_err(gu.to_f64(Y), Yref)
    assert err <= gu.TOL["bf16"], (T, n_in, n_out, b1, b2, rp, order, err)


def _group_shapes():
    rng = np.random.default_rng(2512)
    out = []
    for _ in range(12):
        b = int(rng.choice([2, 4, 8, 16]))
        q, p = (int(rng.integers(1, 24)) * 8 for _ in range(2))
        r = int(rng.integers(1, 40)) * 8
        members = int(rng.integers(2, 5))
        T = int(rng.choice([1, 17, 64, 129, 300, 700, 1500]))
        mode = str(rng.choice(["default", "fused12", "three"]))
        if mode == "fused12" and (b * q) % 64:
            mode = "default"                      # the fused kernel walks the input in chunks of 64 columns
        out.append((T, b * q, b * p, b, r, members, mode))
    return out


@pytest.mark.parametrize("T,n_in,n_out,b,r,members,mode", _group_shapes())
def test_blast_group_random_shape(T, n_in, n_out, b, r, members, mode):
    """Grouped BLAST layers (one call for layers that share their input): every member against the
    oracle's layer on its own factors."""
    gu = _gu()
    B = gu.B
    if B.blast_group_workspace_bytes(T, n_in, n_out, b, r, members) == 0:
        pytest.skip("no grouped execution for this shape (single-kernel size, or no matrix-core kernels)")
    lays = [bi.blast_layer(n_in, n_out, b, r, "bf16", seed=T + n_in, layer_id=m) for m in range(members)]
    X = bi.activations(T, n_in, "bf16", seed=n_out)
    flags = {"fused12": B.BLAST_FUSED_STAGE12, "three": B.BLAST_THREE_KERNELS}.get(mode, 0)
    Y = gu.to_f64(gu.run_blast_group(X, lays, flags))
    for m, lay in enumerate(lays):
        err = gu.rel_err(Y[:, m * n_out:(m + 1) * n_out], oracle.blast_forward(X.f64, lay.U.f64, lay.S.f64, lay.V.f64))
        assert err <= gu.TOL["bf16"], (T, n_in, n_out, b, r, members, mode, m, err)


def _large_interleaved_shapes():
    rng = np.random.default_rng(20861 + 3)
    out = []
    for _ in range(8):
        b = int(rng.choice([8, 16, 32]))
        q = int(rng.integers(8, 130)) * 8
        p = int(rng.integers(1, 8)) * 8
        rp = int(rng.choice([8, 16, 24]))
        T = (4 << 20) // (b * q) + int(rng.integers(1, 200))       # just past 4 M output elements
        out.append((T, b * p, b * q, b, b * rp))
    return out


@pytest.mark.parametrize("T,n_in,n_out,nb,r", _large_interleaved_shapes())
def test_monarch_large_interleaved_output_random_shape(T, n_in, n_out, nb, r):
    """Interleaved outputs large enough to be written in the blocked order and permuted by a second
    pass (8 blocks and more): whole tensor against the oracle."""
    gu = _gu()
    lay = bi.monarch_layer(n_in, n_out, nb, r, "bf16", seed=T)
    X = bi.activations(T, n_in, "bf16", seed=n_out)
    Y = gu.to_f64(gu.run_monarch(X, lay, gu.B.MONARCH_TWO_KERNELS))
    err = gu.rel_err(Y, oracle.monarch_forward(X.f64, lay.R.f64, lay.L.f64, oracle.OUT_INTERLEAVED))
    assert err <= gu.TOL["bf16"], (T, n_in, n_out, nb, r, err)
