"""GPU parity: the HIP library (through its C ABI) against the fp64 CPU oracle, element by
element on identical seeded inputs. Tolerance: max|delta| / max|Y_ref| <= 2e-2 for bf16 storage
(bf16 x bf16 -> fp32 MFMA, bf16 intermediates and output), <= 1e-5 for the fp32 path."""
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
    binding.lib()      # fails loudly if the HIP library is not built


def _gu():
    import gpu_util
    return gpu_util


# ---------------------------------------------------------------- Monarch
MONARCH_CASES = [
    # T, n_in, n_out, nblocks, r, dtype
    (8, 256, 256, 4, 64, "f32"),         # the fp32 check configuration
    (8, 256, 256, 4, 64, "bf16"),
    (300, 512, 768, 4, 256, "bf16"),     # several 128-row tiles and a ragged token tail; p != q != r
    (77, 512, 1376, 4, 128, "bf16"),     # q = 344: a ragged column tail
    (130, 384, 384, 2, 96, "bf16"),      # K = 192 and 96: not multiples of 64
    (37, 36, 60, 3, 9, "bf16"),          # rows not 16-byte aligned: portable kernels
    (37, 36, 60, 3, 9, "f32"),
    (1, 512, 512, 4, 128, "bf16"),
    (65, 1024, 1024, 16, 256, "bf16"),   # 16 blocks as in the paper's Llama settings, r' = 16
    (300, 2048, 2048, 16, 256, "bf16"),  # wide layer, one round of workgroups: the single kernel with one workgroup per compute unit
    (50, 1536, 1536, 8, 256, "bf16"),    # ... up to 64 tokens with any number of blocks
    (600, 512, 8192, 16, 256, "bf16"),   # 4.9 M outputs: interleaved order via the blocked order and the permutation pass
    (1100, 1024, 4096, 8, 256, "bf16"),  # ... with 8 blocks
    (2101, 512, 2048, 16, 256, "bf16"),  # ... short rows: three tokens per workgroup of the pass, the last group ragged
    (270, 512, 16640, 8, 128, "bf16"),   # ... q = 2080 > 2032: two segments per row, the second short
    (1100, 1024, 4096, 4, 256, "bf16"),  # 4 blocks: scattered stores at any size
    (1030, 512, 2048, 64, 512, "bf16"),  # 64 blocks of 32 outputs: the pass with its shortest rows per block
]


@pytest.mark.parametrize("T,n_in,n_out,nb,r,dtype", MONARCH_CASES)
@pytest.mark.parametrize("order", ["interleaved", "blocked"])
@pytest.mark.parametrize("generic", [False, True])
def test_monarch_parity(T, n_in, n_out, nb, r, dtype, order, generic):
    gu = _gu()
    lay = bi.monarch_layer(n_in, n_out, nb, r, dtype)
    X = bi.activations(T, n_in, dtype)
    flags = (gu.B.MONARCH_OUT_BLOCKED if order == "blocked" else 0) | (gu.B.FORCE_GENERIC if generic else 0)
    Y = gu.to_f64(gu.run_monarch(X, lay, flags))
    Yref = oracle.monarch_forward(X.f64, lay.R.f64, lay.L.f64,
                                  oracle.OUT_BLOCKED if order == "blocked" else oracle.OUT_INTERLEAVED)
    err = gu.rel_err(Y, Yref)
    print(f"monarch {T}x{n_in}->{n_out} b={nb} r={r} {dtype} {order} generic={generic}: rel err {err:.3e}")
    assert err <= gu.TOL[dtype]


# ---------------------------------------------------------------- BLAST
BLAST_CASES = [
    # T, n_in, n_out, b, r, dtype
    (333, 768, 768, 16, 96, "bf16"),     # ViT-B-width configuration at a ragged token count
    (130, 1024, 512, 8, 72, "bf16"),     # q = 128, p = 64, r not a multiple of 16
    (70, 512, 2048, 16, 256, "bf16"),
    (50, 36, 30, 3, 10, "bf16"),         # misaligned: portable kernels
    (50, 36, 30, 3, 10, "f32"),
    (9, 256, 256, 4, 64, "f32"),
    (1, 768, 768, 16, 96, "bf16"),
    (200, 1152, 1152, 9, 128, "bf16"),   # b = 9 (DiT-XL/2 rows of the paper's layer table)
    (300, 2752, 1024, 16, 328, "bf16"),  # q = 172: partial last k-chunk; r = 328: partial last rank tile
    (150, 2560, 2560, 5, 200, "bf16"),   # odd number of blocks
    (1100, 512, 256, 16, 1000, "bf16"),  # fused stage 1+2 on 128-token tiles (more than 128 of them), ragged in T and r
    (1000, 512, 256, 16, 1024, "bf16"),  # ... and on 64-token tiles: 256 workgroups, the last token tile ragged
]


@pytest.mark.parametrize("T,n_in,n_out,b,r,dtype", BLAST_CASES)
@pytest.mark.parametrize("mode", ["canonical", "packed", "generic", "fused12", "three"])
def test_blast_parity(T, n_in, n_out, b, r, dtype, mode):
    gu = _gu()
    if mode in ("packed", "fused12", "three") and (dtype != "bf16" or (n_in // b) % 8 or r % 8):
        pytest.skip("packed factors exist only for the bf16 MFMA path")
    lay = bi.blast_layer(n_in, n_out, b, r, dtype)
    X = bi.activations(T, n_in, dtype)
    flags = {"generic": gu.B.FORCE_GENERIC, "fused12": gu.B.BLAST_FUSED_STAGE12, "three": gu.B.BLAST_THREE_KERNELS}.get(mode, 0)
    Y = gu.to_f64(gu.run_blast(X, lay, flags, packed=(mode in ("packed", "fused12", "three"))))
    Yref = oracle.blast_forward(X.f64, lay.U.f64, lay.S.f64, lay.V.f64)
    err = gu.rel_err(Y, Yref)
    print(f"blast {T}x{n_in}->{n_out} b={b} r={r} {dtype} {mode}: rel err {err:.3e}")
    assert err <= gu.TOL[dtype]


BLAST_GROUP_CASES = [
    # T, n_in, n_out, b, r, members
    (333, 1024, 512, 16, 72, 3),      # concatenated rank 216: partial last rank tile; ragged T
    (130, 2816, 1024, 16, 168, 2),    # q = 176: input chunks that straddle blocks
    (1100, 512, 256, 16, 504, 2),     # more than 128 of the 128-token fused tiles
    (70, 512, 2048, 8, 256, 4),       # b = 8, four members
    (1, 2048, 2048, 16, 256, 3),      # one token
]


@pytest.mark.parametrize("T,n_in,n_out,b,r,members", BLAST_GROUP_CASES)
@pytest.mark.parametrize("mode", ["default", "fused12", "three"])
def test_blast_group_parity(T, n_in, n_out, b, r, members, mode):
    """Layers that share their input, run as one grouped call: every member's columns equal the
    oracle's layer on that member's own factors."""
    gu = _gu()
    lays = [bi.blast_layer(n_in, n_out, b, r, "bf16", layer_id=m) for m in range(members)]
    X = bi.activations(T, n_in, "bf16")
    flags = {"fused12": gu.B.BLAST_FUSED_STAGE12, "three": gu.B.BLAST_THREE_KERNELS}.get(mode, 0)
    Y = gu.to_f64(gu.run_blast_group(X, lays, flags))
    assert Y.shape == (T, members * n_out)
    for m, lay in enumerate(lays):
        Yref = oracle.blast_forward(X.f64, lay.U.f64, lay.S.f64, lay.V.f64)
        err = gu.rel_err(Y[:, m * n_out:(m + 1) * n_out], Yref)
        print(f"blast group {T}x{n_in}->{members}x{n_out} b={b} r={r} {mode} member {m}: rel err {err:.3e}")
        assert err <= gu.TOL["bf16"]


def test_blast_group_equals_members_bit_for_bit():
    """Grouping changes launches, not arithmetic: each member's columns are the bits of its own call
    when both take the same execution of stages 1 and 2."""
    gu = _gu()
    T, n_in, n_out, b, r = 400, 2048, 1024, 16, 256
    lays = [bi.blast_layer(n_in, n_out, b, r, "bf16", layer_id=m) for m in range(3)]
    X = bi.activations(T, n_in, "bf16")
    for flag in (gu.B.BLAST_FUSED_STAGE12, gu.B.BLAST_THREE_KERNELS):
        Yg = gu.run_blast_group(X, lays, flag)
        for m, lay in enumerate(lays):
            Ym = gu.run_blast(X, lay, flag, packed=True)
            assert torch.equal(Yg[:, m * n_out:(m + 1) * n_out], Ym), (flag, m)


def _to_blocked(X64, b):
    """Feature j*b + k -> position k*(n/b) + j (the BLOCKED output order of a Monarch layer with b blocks)."""
    T, n = X64.shape
    return X64.reshape(T, n // b, b).transpose(0, 2, 1).reshape(T, n)


@pytest.mark.parametrize("T,n_in,n_out,nb,r,dtype", [
    (8, 256, 256, 4, 64, "f32"), (8, 256, 256, 4, 64, "bf16"), (333, 512, 768, 4, 256, "bf16"),
    (100, 1024, 512, 2, 128, "bf16"), (1, 2048, 2048, 4, 512, "bf16"), (700, 8192, 2048, 4, 512, "bf16"),
    (50, 144, 72, 3, 12, "bf16")])
@pytest.mark.parametrize("generic", [False, True])
def test_monarch_blocked_input(T, n_in, n_out, nb, r, dtype, generic):
    """A layer fed an activation in the BLOCKED order of an upstream layer, with its first factor
    re-ordered once by the library, equals the oracle's layer on the canonical activation."""
    gu = _gu()
    B = gu.B
    lay = bi.monarch_layer(n_in, n_out, nb, r, dtype)
    X = bi.activations(T, n_in, dtype)
    # the same values in blocked order, in the storage type
    Xd = gu.to_dev(X)
    Xb = Xd.reshape(T, n_in // nb, nb).transpose(1, 2).reshape(T, n_in).contiguous()
    Rp = B.monarch_permute_first_factor(gu.to_dev(lay.R), n_in, nb, r)
    # the re-ordering is a pure permutation of each row of R
    Rh = gu.to_f64(Rp).reshape(nb * r, n_in // nb)
    ref_rows = lay.R.f64.reshape(nb * r, n_in // nb // nb, nb).transpose(0, 2, 1).reshape(nb * r, n_in // nb)
    assert np.array_equal(Rh, ref_rows)
    Y = gu.empty_out(T, n_out, dtype)
    B.monarch_forward(Xb, Rp, gu.to_dev(lay.L), Y, nb, r, B.MONARCH_IN_BLOCKED | (B.FORCE_GENERIC if generic else 0))
    torch.cuda.synchronize()
    Yref = oracle.monarch_forward(X.f64, lay.R.f64, lay.L.f64)
    err = gu.rel_err(gu.to_f64(Y), Yref)
    print(f"monarch blocked input {T}x{n_in}->{n_out} b={nb} r={r} {dtype} generic={generic}: rel err {err:.3e}")
    assert err <= gu.TOL[dtype]
    assert np.array_equal(_to_blocked(X.f64, nb), gu.to_f64(Xb))


def test_monarch_blocked_pair_equals_canonical_pair():
    """Producer with BLOCKED output feeding a consumer with BLOCKED input (an elementwise step in
    between) reproduces the canonical two-layer result: the permutation is never materialised."""
    gu = _gu()
    B = gu.B
    T, n0, n1, n2, nb = 200, 512, 2048, 512, 4
    A = bi.monarch_layer(n0, n1, nb, 128, "bf16", layer_id=3)
    C = bi.monarch_layer(n1, n2, nb, 128, "bf16", layer_id=4)
    X = bi.activations(T, n0, "bf16")
    H = gu.empty_out(T, n1, "bf16")
    B.monarch_forward(gu.to_dev(X), gu.to_dev(A.R), gu.to_dev(A.L), H, nb, 128, B.MONARCH_OUT_BLOCKED)
    B.silu_mul(H, H, H)                                    # any elementwise map commutes with the permutation
    Rp = B.monarch_permute_first_factor(gu.to_dev(C.R), n1, nb, 128)
    Y = gu.empty_out(T, n2, "bf16")
    B.monarch_forward(H, Rp, gu.to_dev(C.L), Y, nb, 128, B.MONARCH_IN_BLOCKED)
    torch.cuda.synchronize()
    from oracle import chain as oc
    h = oracle.monarch_forward(X.f64, A.R.f64, A.L.f64)
    yref = oracle.monarch_forward(oc.silu(h) * h, C.R.f64, C.L.f64)
    err = gu.rel_err(gu.to_f64(Y), yref)
    print(f"monarch blocked pair: rel err {err:.3e}")
    assert err <= gu.TOL["bf16"]


# ---------------------------------------------------------------- dense
@pytest.mark.parametrize("T,n_in,n_out,dtype", [(200, 320, 200, "bf16"), (200, 320, 200, "f32"),
                                                (129, 1024, 130, "bf16"), (5, 100, 7, "bf16"), (1, 64, 64, "f32")])
@pytest.mark.parametrize("generic", [False, True])
def test_dense_parity(T, n_in, n_out, dtype, generic):
    gu = _gu()
    W = bi.dense_weight(n_in, n_out, dtype)
    X = bi.activations(T, n_in, dtype)
    Y = gu.empty_out(T, n_out, dtype)
    gu.B.dense_reference_forward(gu.to_dev(X), gu.to_dev(W), Y, gu.B.FORCE_GENERIC if generic else 0)
    torch.cuda.synchronize()
    err = gu.rel_err(gu.to_f64(Y), oracle.dense_forward(X.f64, W.f64))
    print(f"dense {T}x{n_in}->{n_out} {dtype} generic={generic}: rel err {err:.3e}")
    assert err <= gu.TOL[dtype]


# enough 256 x 256 tiles for the large-tile kernel, whose steps are 64 contraction indices deep: an even and an odd
# number of steps, a last step with 8 valid indices, ragged token and output counts (a last row of tiles with one row)
# (the last case: 8 x 43 tiles are one round and a third; the column tiles that fill the round and the remaining
# 2816 columns go out as two products)
@pytest.mark.parametrize("T,n_in,n_out", [(2561, 328, 4100), (2600, 456, 4096), (2560, 448, 4096), (2817, 192, 3848), (2048, 256, 11008)])
def test_dense_large_tile_short_and_partial_steps(T, n_in, n_out):
    gu = _gu()
    W = bi.dense_weight(n_in, n_out, "bf16")
    X = bi.activations(T, n_in, "bf16")
    Y = gu.empty_out(T, n_out, "bf16")
    gu.B.dense_reference_forward(gu.to_dev(X), gu.to_dev(W), Y, 0)
    torch.cuda.synchronize()
    out = gu.to_f64(Y)
    assert np.isfinite(out).all()
    err = gu.rel_err(out, oracle.dense_forward(X.f64, W.f64))
    print(f"dense {T}x{n_in}->{n_out} large tile: rel err {err:.3e}")
    assert err <= gu.TOL["bf16"]


# more workgroups than one round on each of the four small tiles (128x128, 128x64, 64x128, 64x64 by the dispatch
# rules), which take 64-deep steps on two stages: whole steps and a partial last step, odd and even step counts
@pytest.mark.parametrize("T,n_out", [(6304, 768), (2800, 768), (64, 40960), (1400, 768)])
@pytest.mark.parametrize("n_in", [320, 328, 448])
def test_dense_multi_round_small_tiles(T, n_in, n_out):
    gu = _gu()
    W = bi.dense_weight(n_in, n_out, "bf16")
    X = bi.activations(T, n_in, "bf16")
    Y = gu.empty_out(T, n_out, "bf16")
    gu.B.dense_reference_forward(gu.to_dev(X), gu.to_dev(W), Y, 0)
    torch.cuda.synchronize()
    out = gu.to_f64(Y)
    assert np.isfinite(out).all()
    err = gu.rel_err(out, oracle.dense_forward(X.f64, W.f64))
    print(f"dense {T}x{n_in}->{n_out} small tiles, several rounds: rel err {err:.3e}")
    assert err <= gu.TOL["bf16"]


# ---------------------------------------------------------------- Monarch, different block counts on the two sides
# (T, n_in, n_out, b_in, b_out, r_block, dtype): MFMA-aligned and ragged shapes, few and many tokens
MONARCH_RECT_CASES = [
    (8, 256, 192, 4, 2, 16, "f32"),
    (70, 512, 768, 2, 4, 32, "bf16"),
    (1, 1024, 512, 8, 2, 16, "bf16"),
    (300, 768, 2304, 4, 12, 16, "bf16"),
    (515, 1024, 1024, 16, 4, 8, "bf16"),
    (130, 60, 84, 3, 4, 5, "bf16"),
    (33, 60, 84, 5, 2, 3, "f32"),
    (200, 1152, 3456, 9, 3, 24, "bf16"),
    (3000, 1024, 2048, 4, 4, 72, "bf16"),   # several rounds of the deep-step tiles: gathered weight rows with a ragged column count (288), a partial last step (K = 288)
]


@pytest.mark.parametrize("T,n_in,n_out,b1,b2,rp,dtype", MONARCH_RECT_CASES)
@pytest.mark.parametrize("order", ["interleaved", "blocked"])
@pytest.mark.parametrize("generic", [False, True])
def test_monarch_rect_parity(T, n_in, n_out, b1, b2, rp, dtype, order, generic):
    gu = _gu()
    B = gu.B
    p, q = n_in // b1, n_out // b2
    R = bi.gaussian(bi.BASE_SEED, 41, (b1, rp * b2, p), 1.0 / np.sqrt(p), dtype)
    L = bi.gaussian(bi.BASE_SEED, 42, (b2, q, b1 * rp), 1.0 / np.sqrt(b1 * rp), dtype)
    X = bi.activations(T, n_in, dtype)
    Y = gu.empty_out(T, n_out, dtype)
    flags = (B.MONARCH_OUT_BLOCKED if order == "blocked" else 0) | (B.FORCE_GENERIC if generic else 0)
    B.monarch_rect_forward(gu.to_dev(X), gu.to_dev(R), gu.to_dev(L), Y, b1, b2, rp, flags)
    torch.cuda.synchronize()
    Yref = oracle.monarch_rect_forward(X.f64, R.f64, L.f64, b1, b2, oracle.OUT_BLOCKED if order == "blocked" else oracle.OUT_INTERLEAVED)
    err = gu.rel_err(gu.to_f64(Y), Yref)
    print(f"monarch rect T={T} {n_in}->{n_out} b=({b1},{b2}) r'={rp} {dtype} {order} generic={generic}: rel err {err:.3e}")
    assert err <= gu.TOL[dtype]


# ---------------------------------------------------------------- low-rank
# ranks below, at and above a tile; token counts in every GEMM regime (few-token stream, small and
# large tiles); ragged sizes; a row length that is not 16-byte aligned (portable kernels)
LOWRANK_CASES = [
    (8, 256, 256, 64, "f32"),
    (70, 256, 192, 32, "bf16"),
    (1, 512, 384, 128, "bf16"),
    (17, 1024, 520, 96, "bf16"),
    (300, 768, 3072, 128, "bf16"),
    (515, 1000, 776, 200, "bf16"),
    (1100, 2048, 2048, 256, "bf16"),
    (130, 100, 36, 10, "bf16"),
    (33, 100, 36, 10, "f32"),
]


@pytest.mark.parametrize("T,n_in,n_out,r,dtype", LOWRANK_CASES)
@pytest.mark.parametrize("generic", [False, True])
def test_lowrank_parity(T, n_in, n_out, r, dtype, generic):
    gu = _gu()
    lay = bi.lowrank_layer(n_in, n_out, r, dtype)
    X = bi.activations(T, n_in, dtype)
    Y = gu.run_lowrank(X, lay, gu.B.FORCE_GENERIC if generic else 0)
    err = gu.rel_err(gu.to_f64(Y), oracle.lowrank_forward(X.f64, lay.V.f64, lay.U.f64))
    print(f"lowrank T={T} {n_in}->{n_out} r={r} {dtype} generic={generic}: rel err {err:.3e}")
    assert err <= gu.TOL[dtype]


def test_lowrank_stage_flags_and_bit_identity():
    gu = _gu()
    B = gu.B
    lay = bi.lowrank_layer(1024, 768, 128, "bf16")
    X = bi.activations(600, 1024, "bf16")
    Xd, Vd, Ud = gu.to_dev(X), gu.to_dev(lay.V), gu.to_dev(lay.U)
    ws = torch.empty(B.lowrank_workspace_bytes(600, 1024, 768, 128, B.BF16), dtype=torch.uint8, device="cuda")
    Y0 = gu.empty_out(600, 768, "bf16")
    B.lowrank_forward(Xd, Vd, Ud, Y0, 0, ws)
    Y1 = gu.empty_out(600, 768, "bf16")
    B.lowrank_forward(Xd, Vd, Ud, Y1, B.ONLY_FIRST_STAGE, ws)
    torch.cuda.synchronize()
    assert torch.isnan(Y1).all()                        # the first stage alone does not touch Y
    Z = gu.to_f64(ws[:600 * 128 * 2].view(torch.bfloat16).view(600, 128))   # Z comes first in the workspace
    assert gu.rel_err(Z, X.f64 @ lay.V.f64.T) <= gu.TOL["bf16"]
    B.lowrank_forward(Xd, Vd, Ud, Y1, B.ONLY_LAST_STAGE, ws)
    torch.cuda.synchronize()
    assert torch.equal(Y0, Y1)
    for _ in range(3):
        Y2 = gu.empty_out(600, 768, "bf16")
        B.lowrank_forward(Xd, Vd, Ud, Y2, 0, ws)
        torch.cuda.synchronize()
        assert torch.equal(Y0, Y2)


# ---------------------------------------------------------------- edge cases and properties
def test_zero_tokens_and_status_codes():
    gu = _gu()
    B = gu.B
    lay = bi.monarch_layer(64, 64, 4, 16, "bf16")
    Rd, Ld = gu.to_dev(lay.R), gu.to_dev(lay.L)
    X0 = torch.empty((0, 64), dtype=torch.bfloat16, device="cuda")
    Y0 = torch.empty((0, 64), dtype=torch.bfloat16, device="cuda")
    B.monarch_forward(X0, Rd, Ld, Y0, 4, 16)                      # T = 0: ok, nothing launched
    X = gu.to_dev(bi.activations(4, 64, "bf16"))
    Y = gu.empty_out(4, 64, "bf16")
    small = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(B.BlrError) as e:
        B.monarch_forward(X, Rd, Ld, Y, 4, 16, workspace=small)
    assert e.value.status == B.ERR_WORKSPACE
    with pytest.raises(ValueError):
        B.monarch_forward(X, Rd, Ld, Y, 3, 16)                    # 3 does not divide 64: refused by the binding ...
    ws = torch.empty(1 << 16, dtype=torch.uint8, device="cuda")
    st = B.lib().blr_monarch_forward(X.data_ptr(), Rd.data_ptr(), Ld.data_ptr(), Y.data_ptr(), 4, 64, 64, 3, 16, B.BF16, 0,
                                     ws.data_ptr(), ws.numel(), None)
    assert st == B.ERR_INVALID_ARG                                # ... and by the library itself
    torch.cuda.synchronize()
    assert torch.isnan(Y.float()).all()                           # failed calls launched nothing


def test_run_to_run_bit_identical():
    gu = _gu()
    lay = bi.monarch_layer(512, 768, 4, 256, "bf16")
    X = bi.activations(300, 512, "bf16")
    a = gu.run_monarch(X, lay).view(torch.int16).cpu()
    b = gu.run_monarch(X, lay).view(torch.int16).cpu()
    assert torch.equal(a, b)
    bl = bi.blast_layer(768, 768, 16, 96, "bf16")
    Xb = bi.activations(333, 768, "bf16")
    a = gu.run_blast(Xb, bl).view(torch.int16).cpu()
    b = gu.run_blast(Xb, bl, packed=True).view(torch.int16).cpu()
    assert torch.equal(a, b)                                      # per-call re-layout == offline re-layout


def test_linearity_on_gpu():
    gu = _gu()
    lay = bi.blast_layer(256, 256, 4, 64, "f32")
    X1 = bi.activations(33, 256, "f32")
    X2 = bi.gaussian(99, bi.TID_X, (33, 256), 1.0, "f32")
    X3 = bi.store(2.0 * X1.f64 - 0.5 * X2.f64, "f32")
    f = lambda X: gu.to_f64(gu.run_blast(X, lay))
    np.testing.assert_allclose(f(X3), 2.0 * f(X1) - 0.5 * f(X2), rtol=0, atol=2e-5 * np.abs(f(X1)).max())


# Single-kernel Monarch / low-rank (intermediate on chip): forced by flag, against the oracle and
# against the two-kernel execution of the same call. Shapes cover several column tiles per wavefront,
# one and several output ranges per block, a ragged last token tile, wavefronts with and without tiles
# in either phase, b1 != b2, and outputs that do / do not allow 16-byte stores.
FUSED_MONARCH_CASES = [
    # T, n_in, n_out, b1, b2, r'
    (197, 768, 2304, 4, 4, 32),
    (1024, 768, 2304, 4, 4, 48),
    (70, 768, 3072, 4, 4, 48),
    (33, 256, 200, 2, 5, 16),
    (100, 1024, 1152, 4, 4, 32),
    (64, 2048, 512, 8, 2, 16),
    (300, 256, 72, 1, 3, 64),
    (31, 1024, 768, 4, 4, 48),
    (500, 768, 768, 4, 4, 16),
    (130, 512, 1040, 4, 13, 48),
]


@pytest.mark.parametrize("T,n_in,n_out,b1,b2,rp", FUSED_MONARCH_CASES)
@pytest.mark.parametrize("order", ["interleaved", "blocked"])
def test_monarch_single_kernel_parity(T, n_in, n_out, b1, b2, rp, order):
    gu = _gu()
    B = gu.B
    p, q = n_in // b1, n_out // b2
    R = bi.gaussian(T + n_in, 51, (b1, rp * b2, p), 1.0 / np.sqrt(p), "bf16")
    L = bi.gaussian(T + n_in, 52, (b2, q, b1 * rp), 1.0 / np.sqrt(b1 * rp), "bf16")
    X = bi.activations(T, n_in, "bf16", seed=rp + b2)
    blocked = order == "blocked"
    fl = B.MONARCH_OUT_BLOCKED if blocked else 0
    Xd, Rd, Ld = gu.to_dev(X), gu.to_dev(R), gu.to_dev(L)
    Y1, Y2 = gu.empty_out(T, n_out, "bf16"), gu.empty_out(T, n_out, "bf16")
    B.monarch_rect_forward(Xd, Rd, Ld, Y1, b1, b2, rp, fl | B.MONARCH_FUSED)
    B.monarch_rect_forward(Xd, Rd, Ld, Y2, b1, b2, rp, fl | B.MONARCH_TWO_KERNELS)
    torch.cuda.synchronize()
    Yref = oracle.monarch_rect_forward(X.f64, R.f64, L.f64, b1, b2, oracle.OUT_BLOCKED if blocked else oracle.OUT_INTERLEAVED)
    assert gu.rel_err(gu.to_f64(Y1), Yref) <= gu.TOL["bf16"]
    assert gu.rel_err(gu.to_f64(Y2), Yref) <= gu.TOL["bf16"]
    assert gu.rel_err(gu.to_f64(Y1), gu.to_f64(Y2)) <= gu.TOL["bf16"]
    if b1 == b2:                                            # the square entry point takes the same path
        Y3 = gu.empty_out(T, n_out, "bf16")
        B.monarch_forward(Xd, Rd, Ld, Y3, b1, rp * b1, fl | B.MONARCH_FUSED)
        torch.cuda.synchronize()
        assert torch.equal(Y3, Y1)


@pytest.mark.parametrize("T,n_in,n_out,r", [(197, 256, 2304, 128), (1024, 224, 3072, 192), (40, 160, 1152, 64), (333, 256, 768, 256), (65, 96, 40, 32)])
def test_lowrank_single_kernel_parity(T, n_in, n_out, r):
    gu = _gu()
    B = gu.B
    lay = bi.lowrank_layer(n_in, n_out, r, "bf16", seed=T + r)
    X = bi.activations(T, n_in, "bf16", seed=n_out)
    Yref = oracle.lowrank_forward(X.f64, lay.V.f64, lay.U.f64)
    Y1 = gu.to_f64(gu.run_lowrank(X, lay, B.MONARCH_FUSED))
    Y2 = gu.to_f64(gu.run_lowrank(X, lay, B.MONARCH_TWO_KERNELS))
    assert gu.rel_err(Y1, Yref) <= gu.TOL["bf16"]
    assert gu.rel_err(Y2, Yref) <= gu.TOL["bf16"]


def test_single_kernel_is_unsupported_where_its_shape_rules_fail():
    gu = _gu()
    B = gu.B
    lay = bi.monarch_layer(256, 256, 4, 32, "bf16", seed=3)       # r' = 8
    X = bi.activations(8, 256, "bf16", seed=4)
    with pytest.raises(RuntimeError):
        gu.run_monarch(X, lay, B.MONARCH_FUSED)


@pytest.mark.parametrize("T", [4096, 4100])
def test_monarch_default_dispatch_around_the_token_limit_of_the_single_kernel(T):
    """768 -> 2304, 4 blocks, r = 192 (the GPT2-S attention projection of the paper's layer table): the
    default call (single kernel up to 4096 tokens, two GEMMs above) against the oracle on sampled rows."""
    gu = _gu()
    B = gu.B
    lay = bi.monarch_layer(768, 2304, 4, 192, "bf16", seed=77)
    X = bi.activations(T, 768, "bf16", seed=78)
    Y = gu.to_f64(gu.run_monarch(X, lay))
    rows = np.unique(np.concatenate([np.arange(0, 40), np.arange(T - 40, T), np.random.default_rng(5).integers(0, T, 200)]))
    Yref = oracle.monarch_forward(X.f64[rows], lay.R.f64, lay.L.f64)
    assert gu.rel_err(Y[rows], Yref) <= gu.TOL["bf16"]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_monarch_group_first_factor_and_grouped_call(dtype):
    """Three Monarch layers of one shape on the same input as one layer with 3 * nblocks output blocks:
    the library's re-layout of the stacked first factors against the index formula, and each member's
    column slice of the grouped call against the oracle's result for that member alone."""
    gu = _gu()
    B = gu.B
    n_in, n_out, nb, r, T, members = 256, 384, 4, 64, 77, 3
    lays = [bi.monarch_layer(n_in, n_out, nb, r, dtype, seed=50 + m) for m in range(members)]
    X = bi.activations(T, n_in, dtype, seed=60)
    Rs = torch.stack([gu.to_dev(l.R) for l in lays], dim=0).contiguous()
    Rg = B.monarch_group_first_factor(Rs, n_in, nb, r)
    torch.cuda.synchronize()
    rp, p = r // nb, n_in // nb
    host = np.stack([l.R.f64.reshape(nb, rp, nb, p) for l in lays], axis=0)            # [m][l][rho][k][a]
    want = host.transpose(1, 2, 0, 3, 4).reshape(nb, rp * members * nb, p)             # [l][rho][m][k][a]
    assert np.array_equal(gu.to_f64(Rg), want)
    Lg = torch.cat([gu.to_dev(l.L) for l in lays], dim=0).contiguous()
    Y = gu.empty_out(T, members * n_out, dtype)
    B.monarch_rect_forward(gu.to_dev(X), Rg, Lg, Y, nb, members * nb, rp, B.MONARCH_OUT_BLOCKED)
    torch.cuda.synchronize()
    Yh = gu.to_f64(Y)
    for m, l in enumerate(lays):
        ref = oracle.monarch_forward(X.f64, l.R.f64, l.L.f64, oracle.OUT_BLOCKED)
        assert gu.rel_err(Yh[:, m * n_out:(m + 1) * n_out], ref) <= gu.TOL[dtype]


# (the last shape: enough tokens for the 256 x 256 tile with the 8-bit epilogue, and a second, short chunk of tokens)
@pytest.mark.parametrize("shape", [(700, 1024, 512, 16, 256), (333, 2048, 1024, 16, 512), (2100, 768, 3072, 6, 192), (64, 1024, 1024, 8, 128),
                                   (6200, 4096, 512, 16, 256)])
def test_blast_quantised_intermediate(shape):
    """BLAST with Z stored as E4M3 between the stage-1 product and the coupling (the paper's future work on
    quantised intermediate activations) against the oracle that rounds Z the same way, at the stated bf16
    bound; the distance to the UNQUANTISED oracle is printed (the price of the 8-bit intermediate)."""
    gu = _gu()
    B = gu.B
    from oracle import quant
    T, n_in, n_out, b, r = shape
    lay = bi.blast_layer(n_in, n_out, b, r, "bf16", seed=21)
    X = bi.activations(T, n_in, "bf16", seed=22)
    Y = gu.to_f64(gu.run_blast(X, lay, B.BLAST_Z_FP8, packed=True))
    Yq, Z = quant.blast_forward_qz(X.f64, lay.U.f64, lay.S.f64, lay.V.f64)
    Yx = oracle.blast_forward(X.f64, lay.U.f64, lay.S.f64, lay.V.f64)
    err_q, err_x = gu.rel_err(Y, Yq), gu.rel_err(Y, Yx)
    print(f"BLAST {n_in}->{n_out} b={b} r={r} T={T}, Z in E4M3: rel err {err_q:.3e} against the quantised oracle, "
          f"{err_x:.3e} against the exact one (oracle's own quantisation distance {gu.rel_err(Yq, Yx):.3e}); max |Z| {np.abs(Z).max():.2f}")
    assert err_q <= gu.TOL["bf16"]
    # without the flag the same call is the unquantised three-kernel execution
    Y3 = gu.to_f64(gu.run_blast(X, lay, B.BLAST_THREE_KERNELS, packed=True))
    assert gu.rel_err(Y3, Yx) <= gu.TOL["bf16"]


@pytest.mark.parametrize("shape", [
    (197, 768, 2304, 3, 128),      # ViT-B attn_qkv of the paper's layer-wise table: 8 output ranges per block
    (1024, 768, 3072, 6, 192),     # GPT2-S c_fc: one range per block, wavefronts with 2, 2, ..., 0 rank tiles
    (256, 1152, 4608, 9, 256),     # DiT fc1: 9 blocks, q = 128
    (45, 96, 120, 3, 32),          # one token tile with a ragged tail, a range that is not a multiple of 8 outputs (p = 40)
    (1, 64, 80, 2, 32),            # a single token; p = 40: three 16-wide output tiles per block, the last one ragged
    (333, 512, 1000, 2, 256),      # q = 256 and r = 256: the longest contraction indices it takes; p = 500
    (2100, 768, 768, 4, 64),       # more workgroups than compute units: 4 wavefronts per workgroup
])
def test_blast_single_kernel_for_few_wide_blocks(shape):
    """The whole-layer kernel for few, wide blocks (coupling accumulated in registers), forced by its flag, with
    packed and with canonical factors, against the oracle; and the library's own choice for the same call."""
    gu = _gu()
    B = gu.B
    T, n_in, n_out, b, r = shape
    lay = bi.blast_layer(n_in, n_out, b, r, "bf16", seed=31)
    X = bi.activations(T, n_in, "bf16", seed=32)
    Yref = oracle.blast_forward(X.f64, lay.U.f64, lay.S.f64, lay.V.f64)
    Yp = gu.to_f64(gu.run_blast(X, lay, B.BLAST_ONE_KERNEL, packed=True))
    Yc = gu.to_f64(gu.run_blast(X, lay, B.BLAST_ONE_KERNEL, packed=False))
    Yd = gu.to_f64(gu.run_blast(X, lay, 0, packed=True))
    errs = [gu.rel_err(Y, Yref) for Y in (Yp, Yc, Yd)]
    print(f"BLAST {n_in}->{n_out} b={b} r={r} T={T}: one kernel rel err {errs[0]:.3e} (packed) {errs[1]:.3e} (canonical), default {errs[2]:.3e}")
    assert max(errs) <= gu.TOL["bf16"]
    assert np.array_equal(Yp, Yc)


def test_blast_single_kernel_status_codes():
    gu = _gu()
    B = gu.B
    L = B.lib()
    x = torch.zeros(64, dtype=torch.bfloat16, device="cuda")
    p = x.data_ptr()
    one = B.BLAST_PACKED | B.BLAST_ONE_KERNEL
    # input blocks longer than 256, a rank beyond 256 or not a multiple of 32, fp32: no such kernel
    assert L.blr_blast_forward(p, p, None, p, p, 100, 3072, 768, 3, 128, B.BF16, one, p, 1 << 30, None) == B.ERR_UNSUPPORTED
    assert L.blr_blast_forward(p, p, None, p, p, 100, 1152, 3456, 9, 384, B.BF16, one, p, 1 << 30, None) == B.ERR_UNSUPPORTED
    assert L.blr_blast_forward(p, p, None, p, p, 100, 768, 2304, 3, 112, B.BF16, one, p, 1 << 30, None) == B.ERR_UNSUPPORTED
    assert L.blr_blast_forward(p, p, p, p, p, 100, 768, 2304, 3, 128, B.F32, B.BLAST_ONE_KERNEL, p, 1 << 30, None) == B.ERR_UNSUPPORTED
    # layers the kernel for many narrow blocks serves keep that kernel's packed layout
    assert L.blr_blast_forward(p, p, None, p, p, 100, 768, 768, 16, 96, B.BF16, one, p, 1 << 30, None) == B.ERR_UNSUPPORTED
    # one execution at a time, and no stages to select in a single kernel
    for other in (B.BLAST_FUSED_STAGE12, B.BLAST_THREE_KERNELS, B.BLAST_Z_FP8, B.ONLY_FIRST_STAGE, B.ONLY_LAST_STAGE):
        assert L.blr_blast_forward(p, p, None, p, p, 100, 768, 2304, 3, 128, B.BF16, one | other, p, 1 << 30, None) == B.ERR_INVALID_ARG
    # with packed factors the forced single kernel needs no workspace at all
    assert L.blr_blast_workspace_bytes(197, 768, 2304, 3, 128, B.BF16, one) == 0


def test_blast_quantised_intermediate_status_codes():
    gu = _gu()
    B = gu.B
    L = B.lib()
    x = torch.zeros(64, dtype=torch.bfloat16, device="cuda")
    p = x.data_ptr()
    # the single-kernel layer, r not a multiple of 16, fp32, and the fused execution cannot take the flag
    assert L.blr_blast_workspace_bytes(100, 768, 768, 16, 96, B.BF16, B.BLAST_PACKED | B.BLAST_Z_FP8) == 0
    assert L.blr_blast_forward(p, p, None, p, p, 100, 768, 768, 16, 96, B.BF16, B.BLAST_PACKED | B.BLAST_Z_FP8, p, 1 << 30, None) == B.ERR_UNSUPPORTED
    assert L.blr_blast_forward(p, p, None, p, p, 100, 1024, 1024, 16, 264, B.BF16, B.BLAST_PACKED | B.BLAST_Z_FP8, p, 1 << 30, None) == B.ERR_UNSUPPORTED
    assert L.blr_blast_forward(p, p, p, p, p, 100, 1024, 1024, 16, 256, B.F32, B.BLAST_Z_FP8, p, 1 << 30, None) == B.ERR_UNSUPPORTED
    assert L.blr_blast_forward(p, p, None, p, p, 100, 1024, 1024, 16, 256, B.BF16, B.BLAST_PACKED | B.BLAST_Z_FP8 | B.BLAST_FUSED_STAGE12, p, 1 << 30, None) == B.ERR_INVALID_ARG
    # Z takes half the bytes of A in the workspace
    full = L.blr_blast_workspace_bytes(1000, 1024, 1024, 16, 256, B.BF16, B.BLAST_PACKED | B.BLAST_THREE_KERNELS)
    half = L.blr_blast_workspace_bytes(1000, 1024, 1024, 16, 256, B.BF16, B.BLAST_PACKED | B.BLAST_Z_FP8)
    assert full == 2 * 1000 * 16 * 256 * 2 and half == 1000 * 16 * 256 * 2 + 1000 * 16 * 256
