"""GPU parity on the layer shapes of the paper's Table 3 (Appendix, Layer Details): every model,
layer and method, at the token count the benchmark uses for that model, in the launch
configuration bench.py times. The oracle recomputes a sample of token rows (rows are independent)."""
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


CASES = [(row, m) for row in bi.TABLE3 for m in row[5]]


@pytest.mark.parametrize("row,method", CASES, ids=[f"{r[0]}-{r[1]}-{m}" for r, m in CASES])
def test_table3_shape(row, method):
    import gpu_util as gu
    cfg = bi.table3_cfg(row, method)
    T = cfg["T"][0]
    lay = bi.make_layer(cfg)
    X = bi.activations(T, cfg["n_in"], "bf16")
    rng = np.random.default_rng(T + cfg["r"])
    rows = np.array(sorted({0, T - 1, 63, 64, 127, 128, T // 2} | set(rng.integers(0, T, size=16).tolist())), dtype=np.int64)
    if method == "monarch":
        Y = gu.run_monarch(X, lay)
        Yref = oracle.monarch_forward(X.f64[rows], lay.R.f64, lay.L.f64)
    elif method == "blast":
        Y = gu.run_blast(X, lay, packed=gu.B.blast_packed_bytes(cfg["n_in"], cfg["n_out"], cfg["b"], cfg["r"]) > 0)
        Yref = oracle.blast_forward(X.f64[rows], lay.U.f64, lay.S.f64, lay.V.f64)
    else:
        Y = gu.run_lowrank(X, lay)
        Yref = oracle.lowrank_forward(X.f64[rows], lay.V.f64, lay.U.f64)
    assert torch.isfinite(Y.float()).all()
    err = gu.rel_err(gu.to_f64(Y[torch.from_numpy(rows).cuda()]), Yref)
    print(f"{row[0]} {row[1]} {method} (r, b) = {row[5][method]} T={T}: {len(rows)} sampled rows, rel err {err:.3e}")
    assert err <= gu.TOL["bf16"]
