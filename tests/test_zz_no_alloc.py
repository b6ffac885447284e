"""The entry point that allocates nothing (blr_monarch_forward_static: the intermediate lives in a static
device array inside the library) against blr_monarch_forward with a caller-provided workspace, through
the C ABI: same kernels, so the results must agree bit for bit; two calls in a row, the second with a
smaller input, so that stale contents of the shared array would show."""
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


def _run_both(T, n_in, n_out, nb, r, flags, seed):
    import gpu_util as gu
    B = gu.B
    L = B.lib()
    lay = bi.monarch_layer(n_in, n_out, nb, r, "bf16", seed=seed)
    X = bi.activations(T, n_in, "bf16", seed=seed + 1)
    Xd, Rd, Ld = gu.to_dev(X), gu.to_dev(lay.R), gu.to_dev(lay.L)
    need = L.blr_monarch_workspace_bytes(T, n_in, n_out, nb, r, B.BF16)
    assert 0 < need <= L.blr_static_scratch_bytes()
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    Yw, Ys = gu.empty_out(T, n_out, "bf16"), gu.empty_out(T, n_out, "bf16")
    stream = torch.cuda.current_stream().cuda_stream
    print(f"static-scratch Monarch: T={T} {n_in}->{n_out} nblocks={nb} r={r} flags={flags:#x}", flush=True)
    st = L.blr_monarch_forward(Xd.data_ptr(), Rd.data_ptr(), Ld.data_ptr(), Yw.data_ptr(), T, n_in, n_out, nb, r, B.BF16, flags,
                               ws.data_ptr(), ws.numel(), stream)
    assert st == B.OK
    st = L.blr_monarch_forward_static(Xd.data_ptr(), Rd.data_ptr(), Ld.data_ptr(), Ys.data_ptr(), T, n_in, n_out, nb, r, B.BF16, flags, stream)
    assert st == B.OK
    torch.cuda.synchronize()
    assert torch.equal(Yw.view(torch.int16), Ys.view(torch.int16)), "static-scratch call differs from the workspace call"
    rows = np.unique(np.concatenate([[0, T - 1, T // 2], np.random.default_rng(seed).integers(0, T, 12)]))
    oflag = oracle.OUT_BLOCKED if flags & B.MONARCH_OUT_BLOCKED else oracle.OUT_INTERLEAVED
    Yref = oracle.monarch_forward(X.f64[rows], lay.R.f64, lay.L.f64, oflag)
    err = gu.rel_err(gu.to_f64(Ys[torch.from_numpy(rows).cuda()]), Yref)
    assert err <= gu.TOL["bf16"], err


def test_static_scratch_matches_workspace_call_twice_in_a_row():
    import gpu_util as gu
    B = gu.B
    # two GEMM kernels with Z' in the array (a few row tiles and a ragged tail), then a smaller input
    _run_both(1000, 1024, 1536, 4, 512, B.MONARCH_TWO_KERNELS, seed=31)
    _run_both(200, 512, 768, 4, 256, B.MONARCH_TWO_KERNELS | B.MONARCH_OUT_BLOCKED, seed=33)
    # a shape whose interleaved output also goes through the blocked-order copy in the array
    _run_both(1024, 2048, 2048, 16, 256, B.MONARCH_TWO_KERNELS, seed=35)


def test_static_scratch_rejects_sizes_beyond_the_array():
    import gpu_util as gu
    B = gu.B
    L = B.lib()
    T, n, nb, r = 16384, 4096, 4, 1024                       # Z' alone is 128 MiB
    assert L.blr_monarch_workspace_bytes(T, n, n, nb, r, B.BF16) > L.blr_static_scratch_bytes()
    x = torch.zeros(16, dtype=torch.bfloat16, device="cuda")
    p = x.data_ptr()                                          # never dereferenced: the size check comes first
    assert L.blr_monarch_forward_static(p, p, p, p, T, n, n, nb, r, B.BF16, 0, None) == B.ERR_WORKSPACE
    assert L.blr_monarch_forward_static(p, p, p, p, 4, 64, 64, 3, 16, B.BF16, 0, None) == B.ERR_INVALID_ARG
