"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, sizes workspaces as documented, and rejects bad arguments before touching a device."""
import ctypes
import os
import re

import pytest

from paper_2512_20861_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "blr.h")

if not os.path.exists(B.LIB_PATH):
    from paper_2512_20861_amd import build as _build
    _build.build_library()

FAKE = 0x10000          # a non-null, 16-byte aligned address that is never dereferenced on these paths


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(blr_[a-z_0-9]+)\s*\(", text)))


def test_header_symbols_are_exported():
    names = declared_symbols()
    assert set(B.EXPORTS) == set(names)
    lib = B.lib()
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings():
    assert B.status_string(B.OK) == "ok"
    for s in (B.ERR_INVALID_ARG, B.ERR_UNSUPPORTED, B.ERR_WORKSPACE, B.ERR_LAUNCH):
        assert B.status_string(s) not in ("ok", "unknown status")
    assert B.status_string(77) == "unknown status"


def test_workspace_sizes():
    # Monarch: Z'[T][nblocks][r] in the storage type, rounded up to 256 bytes
    assert B.monarch_workspace_bytes(8, 256, 256, 4, 64, B.F32) == 8 * 4 * 64 * 4
    assert B.monarch_workspace_bytes(512, 4096, 4096, 4, 1024, B.BF16) == 512 * 4096 * 2
    # outputs of 4 M elements and more: plus the blocked-order copy of one chunk of tokens (64 MiB at most)
    # with 8 blocks or more and outputs of 4 M elements or more: plus the blocked-order copy of one chunk of tokens (64 MiB at most)
    assert B.monarch_workspace_bytes(8192, 4096, 4096, 16, 1024, B.BF16) == 8192 * 16 * 1024 * 2 + 8192 * 4096 * 2
    assert B.monarch_workspace_bytes(32768, 2048, 8192, 16, 512, B.BF16) == 32768 * 16 * 512 * 2 + 4096 * 8192 * 2
    assert B.monarch_workspace_bytes(8192, 4096, 4096, 16, 1024, B.F32) == 8192 * 16 * 1024 * 4     # bf16 only
    assert B.monarch_workspace_bytes(8192, 4096, 4096, 4, 1024, B.BF16) == 8192 * 4096 * 2           # not for 4 blocks
    assert B.monarch_workspace_bytes(8192, 4104, 4104, 12, 1032, B.BF16) == 8192 * 12 * 1032 * 2     # not for 12 blocks
    assert B.monarch_workspace_bytes(8, 250, 256, 4, 64, B.F32) == 0          # invalid shape -> 0
    # BLAST: the whole-layer kernel needs no intermediate; packed factors add nothing
    assert B.blast_workspace_bytes(6304, 768, 768, 16, 96, B.BF16, B.BLAST_PACKED) == 0
    unpacked = B.blast_workspace_bytes(6304, 768, 768, 16, 96, B.BF16, 0)
    assert unpacked == B.blast_packed_bytes(768, 768, 16, 96)
    # Sp (one 16x16 tile per rank index) + V and U in fragment order (1 KiB per block x tile x k-step)
    assert B.blast_packed_bytes(768, 768, 16, 96) == 96 * 512 + 16 * 3 * 3 * 1024 + 16 * 3 * 3 * 1024
    # larger ranks: Sp + the row-major transpose of V + a canonical copy of S (few-token coupling)
    assert B.blast_packed_bytes(4096, 4096, 16, 640) == 640 * 512 + 4096 * 640 * 2 + 16 * 16 * 640 * 2
    # large ranks: Z and A of one chunk of tokens (three-kernel path), or A alone (fused stage 1 + coupling)
    assert B.blast_workspace_bytes(512, 4096, 4096, 16, 640, B.BF16, B.BLAST_PACKED) == 2 * 512 * 16 * 640 * 2
    assert B.blast_workspace_bytes(512, 4096, 4096, 16, 640, B.BF16, B.BLAST_PACKED | B.BLAST_FUSED_STAGE12) == 512 * 16 * 640 * 2
    # enough 128-token x 64-rank tiles (16 x 10 >= 128): the fused kernel is the default, A for all tokens
    assert B.blast_workspace_bytes(2048, 4096, 4096, 16, 640, B.BF16, B.BLAST_PACKED) == 2048 * 16 * 640 * 2
    assert B.blast_workspace_bytes(2048, 4096, 4096, 16, 640, B.BF16, B.BLAST_PACKED | B.BLAST_THREE_KERNELS) == 2 * 2048 * 16 * 640 * 2
    # many tokens: the chunk (a multiple of 256 tokens whose Z and A are 48 MiB each at most) bounds the workspace
    chunk = (48 << 20) // (16 * 640 * 2) // 256 * 256
    assert B.blast_workspace_bytes(100000, 4096, 4096, 16, 640, B.BF16, B.BLAST_PACKED | B.BLAST_THREE_KERNELS) == 2 * chunk * 16 * 640 * 2
    # portable path keeps Z and A
    assert B.blast_workspace_bytes(50, 36, 30, 3, 10, B.F32, 0) == 2 * ((50 * 3 * 10 * 4 + 255) // 256 * 256)
    assert B.blast_packed_bytes(768, 768, 32, 96) == 0 and B.blast_packed_bytes(768, 768, 16, 96, B.F32) == 0


def _monarch(T=4, n_in=64, n_out=64, nb=4, r=16, dt=B.BF16, flags=0, X=FAKE, R=FAKE, L=FAKE, Y=FAKE, ws=FAKE, wsb=1 << 20):
    return B.lib().blr_monarch_forward(X, R, L, Y, T, n_in, n_out, nb, r, dt, flags, ws, wsb, None)


def _blast(T=4, n_in=64, n_out=64, b=4, r=16, dt=B.BF16, flags=0, X=FAKE, U=FAKE, S=FAKE, V=FAKE, Y=FAKE, ws=FAKE, wsb=1 << 20):
    return B.lib().blr_blast_forward(X, U, S, V, Y, T, n_in, n_out, b, r, dt, flags, ws, wsb, None)


def test_monarch_argument_checks():
    assert _monarch(T=0) == B.OK                                   # empty batch: nothing launched
    assert _monarch(T=0, X=None, Y=None) == B.OK
    assert _monarch(T=-1) == B.ERR_INVALID_ARG
    assert _monarch(R=None) == B.ERR_INVALID_ARG
    assert _monarch(X=None) == B.ERR_INVALID_ARG
    assert _monarch(n_in=66) == B.ERR_INVALID_ARG                  # nblocks does not divide n_in
    assert _monarch(n_out=62) == B.ERR_INVALID_ARG
    assert _monarch(r=18) == B.ERR_INVALID_ARG                     # nblocks does not divide r
    assert _monarch(nb=0) == B.ERR_INVALID_ARG
    assert _monarch(dt=7) == B.ERR_INVALID_ARG
    assert _monarch(flags=0x8000) == B.ERR_INVALID_ARG
    assert _monarch(flags=B.ONLY_FIRST_STAGE | B.ONLY_LAST_STAGE) == B.ERR_INVALID_ARG
    assert _blast(flags=B.BLAST_FUSED_STAGE12 | B.BLAST_THREE_KERNELS) == B.ERR_INVALID_ARG
    assert _monarch(flags=B.BLAST_THREE_KERNELS) == B.ERR_INVALID_ARG
    # single-kernel execution: exclusive with the two-kernel flag, the stage flags, the portable kernels, a blocked input
    for other in (B.MONARCH_TWO_KERNELS, B.ONLY_FIRST_STAGE, B.ONLY_LAST_STAGE, B.FORCE_GENERIC, B.MONARCH_IN_BLOCKED):
        assert _monarch(n_in=512, n_out=512, nb=4, r=64, flags=B.MONARCH_FUSED | other) == B.ERR_INVALID_ARG
    # ... and unsupported where its shape rules do not hold: 16 | r/nblocks, 32 | n_in/nblocks, bf16
    assert _monarch(n_in=512, n_out=512, nb=4, r=32, flags=B.MONARCH_FUSED) == B.ERR_UNSUPPORTED
    assert _monarch(n_in=64, n_out=64, nb=4, r=64, flags=B.MONARCH_FUSED) == B.ERR_UNSUPPORTED
    assert _monarch(n_in=512, n_out=512, nb=4, r=64, dt=B.F32, flags=B.MONARCH_FUSED) == B.ERR_UNSUPPORTED
    assert _monarch(n_in=512, n_out=512, nb=4, r=64, flags=B.MONARCH_FUSED, ws=None) == B.ERR_WORKSPACE   # same workspace contract
    # blocked input needs nblocks^2 | n_in
    assert _monarch(n_in=60, n_out=60, nb=6, r=12, flags=B.MONARCH_IN_BLOCKED) == B.ERR_INVALID_ARG
    L = B.lib()
    assert L.blr_monarch_permute_first_factor(FAKE, FAKE, 64, 4, 16, B.BF16, None) == B.ERR_INVALID_ARG      # in place
    assert L.blr_monarch_permute_first_factor(FAKE, FAKE + 0x1000, 60, 6, 12, B.BF16, None) == B.ERR_INVALID_ARG
    assert L.blr_monarch_permute_first_factor(None, FAKE, 64, 4, 16, B.BF16, None) == B.ERR_INVALID_ARG
    assert _monarch(X=FAKE + 2) == B.ERR_INVALID_ARG               # misaligned pointer
    assert _monarch(ws=None) == B.ERR_WORKSPACE
    assert _monarch(wsb=16) == B.ERR_WORKSPACE


def test_blast_single_kernel_flag_checks():
    """The forced single kernel for few, wide blocks: decided on the host before anything is enqueued."""
    one = B.BLAST_ONE_KERNEL
    ok = dict(n_in=768, n_out=2304, b=3, r=128)
    for other in (B.BLAST_FUSED_STAGE12, B.BLAST_THREE_KERNELS, B.BLAST_Z_FP8, B.FORCE_GENERIC, B.ONLY_FIRST_STAGE, B.ONLY_LAST_STAGE):
        assert _blast(flags=one | other, **ok) == B.ERR_INVALID_ARG
    assert _blast(flags=one, n_in=3072, n_out=768, b=3, r=128) == B.ERR_UNSUPPORTED      # input blocks longer than 256
    assert _blast(flags=one, n_in=768, n_out=2304, b=3, r=112) == B.ERR_UNSUPPORTED      # 32 does not divide r
    assert _blast(flags=one, n_in=1152, n_out=3456, b=9, r=384) == B.ERR_UNSUPPORTED     # r beyond 256
    assert _blast(flags=one, dt=B.F32, **ok) == B.ERR_UNSUPPORTED
    assert _blast(flags=one, n_in=768, n_out=768, b=16, r=96) == B.ERR_UNSUPPORTED       # served by the kernel for many narrow blocks
    assert _blast(flags=one, T=0, **ok) == B.OK                                          # empty batch: nothing launched
    # with packed factors it needs no workspace; with canonical ones only room for the packed copies
    assert B.blast_workspace_bytes(197, 768, 2304, 3, 128, B.BF16, B.BLAST_PACKED | one) == 0
    assert B.blast_workspace_bytes(197, 768, 2304, 3, 128, B.BF16, one) == B.blast_packed_bytes(768, 2304, 3, 128, B.BF16)


def test_monarch_rect_argument_checks():
    L = B.lib()
    def call(T=4, n_in=60, n_out=64, b1=3, b2=4, rp=2, dt=B.BF16, flags=0, X=FAKE, R=FAKE, Lf=FAKE, Y=FAKE, ws=FAKE, wsb=1 << 20):
        return L.blr_monarch_rect_forward(X, R, Lf, Y, T, n_in, n_out, b1, b2, rp, dt, flags, ws, wsb, None)
    assert B.monarch_rect_workspace_bytes(10, 60, 64, 3, 4, 2, B.BF16) == (10 * 3 * 4 * 2 * 2 + 255) // 256 * 256
    assert B.monarch_rect_workspace_bytes(10, 61, 64, 3, 4, 2, B.BF16) == 0
    # the square case needs exactly what blr_monarch_forward needs
    assert B.monarch_rect_workspace_bytes(512, 4096, 4096, 4, 4, 256, B.BF16) == B.monarch_workspace_bytes(512, 4096, 4096, 4, 1024, B.BF16)
    assert call(T=0) == B.OK
    assert call(T=0, X=None, Y=None) == B.OK
    assert call(n_in=61) == B.ERR_INVALID_ARG                      # b_in does not divide n_in
    assert call(n_out=62) == B.ERR_INVALID_ARG                     # b_out does not divide n_out
    assert call(rp=0) == B.ERR_INVALID_ARG
    assert call(b1=0) == B.ERR_INVALID_ARG
    assert call(R=None) == B.ERR_INVALID_ARG
    assert call(Y=None) == B.ERR_INVALID_ARG
    assert call(flags=B.MONARCH_IN_BLOCKED) == B.ERR_INVALID_ARG   # blocked input is defined for equal block counts only
    assert call(flags=B.BLAST_PACKED) == B.ERR_INVALID_ARG
    assert call(Lf=FAKE + 8) == B.ERR_INVALID_ARG
    assert call(ws=None) == B.ERR_WORKSPACE
    assert call(wsb=100) == B.ERR_WORKSPACE


def test_blast_argument_checks():
    assert _blast(T=0) == B.OK
    assert _blast(T=-3) == B.ERR_INVALID_ARG
    assert _blast(S=None) == B.ERR_INVALID_ARG
    # with packed factors S may be null: the call gets as far as the workspace check
    assert _blast(S=None, flags=B.BLAST_PACKED, T=64, n_in=4096, n_out=4096, b=16, r=640, wsb=1024) == B.ERR_WORKSPACE
    assert _blast(Y=None) == B.ERR_INVALID_ARG
    assert _blast(n_in=66) == B.ERR_INVALID_ARG
    assert _blast(n_out=30) == B.ERR_INVALID_ARG
    assert _blast(b=0) == B.ERR_INVALID_ARG
    assert _blast(r=0) == B.ERR_INVALID_ARG
    assert _blast(flags=0x1) == B.ERR_INVALID_ARG                  # a Monarch flag
    assert _blast(dt=B.F32, flags=B.BLAST_PACKED) == B.ERR_INVALID_ARG
    assert _blast(flags=B.BLAST_PACKED | B.FORCE_GENERIC) == B.ERR_INVALID_ARG
    assert _blast(T=64, n_in=4096, n_out=4096, b=16, r=640, wsb=1024) == B.ERR_WORKSPACE
    assert _blast(T=64, n_in=4096, n_out=4096, b=16, r=640, ws=None, wsb=0) == B.ERR_WORKSPACE


def _lowrank(T=4, n_in=64, n_out=48, r=16, dt=B.BF16, flags=0, X=FAKE, V=FAKE, U=FAKE, Y=FAKE, ws=FAKE, wsb=1 << 20):
    return B.lib().blr_lowrank_forward(X, V, U, Y, T, n_in, n_out, r, dt, flags, ws, wsb, None)


def test_lowrank_argument_checks():
    assert B.lowrank_workspace_bytes(8192, 4096, 4096, 128, B.BF16) == 8192 * 128 * 2     # Z[T][r]
    assert B.lowrank_workspace_bytes(3, 10, 10, 5, B.F32) == 256                          # rounded up to 256 bytes
    assert B.lowrank_workspace_bytes(3, 10, 0, 5, B.F32) == 0
    assert _lowrank(T=0) == B.OK
    assert _lowrank(T=0, X=None, Y=None) == B.OK
    assert _lowrank(T=-1) == B.ERR_INVALID_ARG
    assert _lowrank(V=None) == B.ERR_INVALID_ARG
    assert _lowrank(U=None) == B.ERR_INVALID_ARG
    assert _lowrank(Y=None) == B.ERR_INVALID_ARG
    assert _lowrank(r=0) == B.ERR_INVALID_ARG
    assert _lowrank(n_in=-4) == B.ERR_INVALID_ARG
    assert _lowrank(dt=5) == B.ERR_INVALID_ARG
    assert _lowrank(flags=B.MONARCH_OUT_BLOCKED) == B.ERR_INVALID_ARG
    assert _lowrank(flags=B.ONLY_FIRST_STAGE | B.ONLY_LAST_STAGE) == B.ERR_INVALID_ARG
    assert _lowrank(U=FAKE + 4) == B.ERR_INVALID_ARG
    assert _lowrank(ws=None) == B.ERR_WORKSPACE
    assert _lowrank(wsb=64) == B.ERR_WORKSPACE


def test_dense_and_pack_argument_checks():
    lib = B.lib()
    assert lib.blr_dense_reference_forward(FAKE, FAKE, FAKE, 0, 8, 8, B.BF16, 0, None) == B.OK
    assert lib.blr_dense_reference_forward(FAKE, None, FAKE, 4, 8, 8, B.BF16, 0, None) == B.ERR_INVALID_ARG
    assert lib.blr_dense_reference_forward(FAKE, FAKE, FAKE, 4, 0, 8, B.BF16, 0, None) == B.ERR_INVALID_ARG
    assert lib.blr_dense_reference_forward(FAKE, FAKE, FAKE, 4, 8, 8, B.BF16, 0x2, None) == B.ERR_INVALID_ARG
    assert lib.blr_blast_pack(FAKE, FAKE, FAKE, FAKE, 64, 64, 4, 16, B.F32, None) == B.ERR_INVALID_ARG
    assert lib.blr_blast_pack(FAKE, FAKE, FAKE, FAKE, 64, 64, 32, 16, B.BF16, None) == B.ERR_INVALID_ARG
    assert lib.blr_blast_pack(None, FAKE, FAKE, FAKE, 64, 64, 4, 16, B.BF16, None) == B.ERR_INVALID_ARG
    assert lib.blr_blast_pack(FAKE, FAKE, FAKE, FAKE, 36, 30, 3, 10, B.BF16, None) == B.ERR_UNSUPPORTED


def test_blast_group_argument_checks():
    lib = B.lib()
    def grp(X=FAKE, U=FAKE, P=FAKE, Y=FAKE, T=256, n_in=2048, n_out=2048, b=16, r=256, members=3, dt=B.BF16, flags=0, ws=FAKE, wsb=1 << 40):
        return lib.blr_blast_group_forward(X, U, P, Y, T, n_in, n_out, b, r, members, dt, flags, ws, wsb, None)
    need = lib.blr_blast_group_workspace_bytes(256, 2048, 2048, 16, 256, 3, B.BF16, 0)
    # the group's workspace is that of one layer with the concatenated rank
    assert need == lib.blr_blast_workspace_bytes(256, 2048, 2048, 16, 768, B.BF16, B.BLAST_PACKED) > 0
    assert grp(T=0, X=None, Y=None) == B.OK
    assert grp(U=None) == B.ERR_INVALID_ARG
    assert grp(P=None) == B.ERR_INVALID_ARG
    assert grp(X=None) == B.ERR_INVALID_ARG
    assert grp(members=0) == B.ERR_INVALID_ARG
    assert grp(r=0) == B.ERR_INVALID_ARG
    assert grp(n_in=2050) == B.ERR_INVALID_ARG                       # b does not divide n_in
    assert grp(flags=B.BLAST_PACKED) == B.ERR_INVALID_ARG            # implied, not a flag of this entry point
    assert grp(flags=B.FORCE_GENERIC) == B.ERR_INVALID_ARG
    assert grp(flags=B.BLAST_FUSED_STAGE12 | B.BLAST_THREE_KERNELS) == B.ERR_INVALID_ARG
    assert grp(X=FAKE + 2) == B.ERR_INVALID_ARG                      # not 16-byte aligned
    assert grp(wsb=need - 1) == B.ERR_WORKSPACE
    assert grp(ws=None) == B.ERR_WORKSPACE
    # no matrix-core kernels for the concatenated layer, or a layer of the single-kernel size: members run one by one
    for kw in (dict(dt=B.F32), dict(r=12), dict(n_in=36, n_out=30, b=3, r=8), dict(n_in=768, n_out=768, b=16, r=32, members=2)):
        args = dict(T=256, n_in=2048, n_out=2048, b=16, r=256, members=3, dt=B.BF16); args.update(kw)
        assert lib.blr_blast_group_workspace_bytes(args["T"], args["n_in"], args["n_out"], args["b"], args["r"], args["members"], args["dt"], 0) == 0, kw
        assert grp(**kw) == B.ERR_UNSUPPORTED, kw


def test_glue_argument_checks():
    L = B.lib()
    A, C, D = FAKE, FAKE + 0x1000, FAKE + 0x2000
    # no tokens: nothing to do, pointers not looked at
    assert L.blr_rmsnorm(None, None, 0, 8, 1e-6, B.BF16, None) == B.OK
    assert L.blr_residual_add_rmsnorm(None, None, None, 0, 8, 1e-6, B.BF16, None) == B.OK
    assert L.blr_sum3_scaled(None, None, None, None, 0, 8, 1.0, B.BF16, None) == B.OK
    assert L.blr_silu_mul(None, None, None, 0, 8, B.F32, None) == B.OK
    # bad shapes, dtype, eps
    assert L.blr_rmsnorm(A, C, -1, 8, 1e-6, B.BF16, None) == B.ERR_INVALID_ARG
    assert L.blr_rmsnorm(A, C, 4, 0, 1e-6, B.BF16, None) == B.ERR_INVALID_ARG
    assert L.blr_rmsnorm(A, C, 4, 8, -1.0, B.BF16, None) == B.ERR_INVALID_ARG
    assert L.blr_rmsnorm(A, C, 4, 8, 1e-6, 5, None) == B.ERR_INVALID_ARG
    # null pointers and forbidden aliasing
    assert L.blr_rmsnorm(A, None, 4, 8, 1e-6, B.BF16, None) == B.ERR_INVALID_ARG
    assert L.blr_rmsnorm(A, A, 4, 8, 1e-6, B.BF16, None) == B.ERR_INVALID_ARG
    assert L.blr_residual_add_rmsnorm(A, A, C, 4, 8, 1e-6, B.BF16, None) == B.ERR_INVALID_ARG
    assert L.blr_residual_add_rmsnorm(A, C, A, 4, 8, 1e-6, B.BF16, None) == B.ERR_INVALID_ARG
    assert L.blr_residual_add_rmsnorm(A, C, C, 4, 8, 1e-6, B.BF16, None) == B.ERR_INVALID_ARG
    assert L.blr_residual_add_rmsnorm(A, None, D, 4, 8, 1e-6, B.BF16, None) == B.ERR_INVALID_ARG
    assert L.blr_sum3_scaled(A, C, None, D, 4, 8, 1.0, B.BF16, None) == B.ERR_INVALID_ARG
    assert L.blr_silu_mul(A, None, D, 4, 8, B.BF16, None) == B.ERR_INVALID_ARG


def test_missing_library_fails_loudly(tmp_path, monkeypatch):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(ImportError):
        B.lib()


def test_python_wrappers_marshal_every_entry_point(monkeypatch):
    """Every wrapper of the binding builds a call the C prototype accepts (argument count and types),
    checked on the CPU with host tensors standing in for device tensors: the launching functions
    through their marshallers (nothing is called), the one-time re-layouts through a recorder that
    stands in for their entry points (size queries run for real)."""
    torch = pytest.importorskip("torch")
    real = B.lib()
    calls = []

    def fits(name, args):
        fn = getattr(real, name)
        assert len(args) == len(fn.argtypes), (name, len(args), len(fn.argtypes))
        for t, a in zip(fn.argtypes, args):
            t(a) if not isinstance(a, t) else a          # raises if the value does not fit the C type
        calls.append(name)

    RELAYOUTS = ("blr_blast_pack", "blr_monarch_permute_first_factor", "blr_monarch_group_first_factor")

    class Recorder:
        def __getattr__(self, name):
            if name not in RELAYOUTS:
                return getattr(real, name)
            def rec(*args):
                fits(name, args)
                return B.OK
            return rec

    monkeypatch.setattr(B, "_lib", Recorder())
    monkeypatch.setattr(B, "_is_gpu", lambda t: isinstance(t, torch.Tensor))
    monkeypatch.setattr(B, "_ptr", lambda t: None if t is None else t.data_ptr())
    monkeypatch.setattr(B, "_ptr_rows", lambda t: t.data_ptr())
    monkeypatch.setattr(B, "_stream", lambda s: None)
    bf = lambda *shape: torch.zeros(shape, dtype=torch.bfloat16)
    ws = torch.zeros(1 << 22, dtype=torch.uint8)
    T, n, b, r = 8, 64, 4, 16

    def marshal(fn, *args):
        name, cargs, result, keep = fn.marshal(*args)
        fits(name, cargs)
        assert result is not None and all(k is None or isinstance(k, torch.Tensor) for k in keep)

    marshal(B.monarch_forward, bf(T, n), bf(b, r, n // b), bf(b, n // b, r), bf(T, n), b, r, 0, ws)
    marshal(B.monarch_forward_static, bf(T, n), bf(b, r, n // b), bf(b, n // b, r), bf(T, n), b, r, 0)
    marshal(B.monarch_rect_forward, bf(T, n), bf(2, 4 * b, n // 2), bf(b, n // b, 2 * 4), bf(T, n), 2, b, 4, 0, ws)
    B.monarch_permute_first_factor(bf(b, r, n // b), n, b, r)
    assert tuple(B.monarch_group_first_factor(bf(3, b, r, n // b), n, b, r).shape) == (b, 3 * r, n // b)
    marshal(B.lowrank_forward, bf(T, n), bf(r, n), bf(48, r), bf(T, 48), 0, ws)
    marshal(B.blast_forward, bf(T, n), bf(b, n // b, r), bf(b, b, r), bf(b, n // b, r), bf(T, n), b, r, 0, ws)
    packed = B.blast_pack(bf(16, 48, 96), bf(16, 16, 96), bf(16, 48, 96), 768, 768, 16, 96)
    marshal(B.blast_forward, bf(T, 768), bf(16, 48, 96), None, packed, bf(T, 768), 16, 96, B.BLAST_PACKED, ws)
    gpacked = torch.zeros(B.blast_packed_bytes(2048, 2048, 16, 3 * 256), dtype=torch.uint8)
    marshal(B.blast_group_forward, bf(T, 2048), bf(3, 16, 128, 256), gpacked, bf(T, 3 * 2048), 16, 256, 3, 0,
            torch.zeros(B.blast_group_workspace_bytes(T, 2048, 2048, 16, 256, 3) + 16, dtype=torch.uint8))
    marshal(B.dense_reference_forward, bf(T, n), bf(n, n), bf(T, n))
    marshal(B.rmsnorm, bf(T, n), bf(T, n))
    marshal(B.residual_add_rmsnorm, bf(T, n), bf(T, n), bf(T, n))
    marshal(B.residual_add_rmsnorm, bf(T, n), bf(T, n), None)
    marshal(B.sum3_scaled, bf(T, n), bf(T, n), bf(T, n), bf(T, n), 0.5)
    marshal(B.silu_mul, bf(T, n), bf(T, n), bf(T, n))
    wide = bf(T, 3 * n)                                    # column slices of a wider tensor take the strided entry points
    marshal(B.sum3_scaled, wide[:, :n], wide[:, n:2 * n], wide[:, 2 * n:], bf(T, n), 0.5)
    marshal(B.silu_mul, wide[:, :n], wide[:, n:2 * n], bf(T, n))
    launching = {n_ for n_ in B.EXPORTS if not n_.endswith("_bytes") and n_ != "blr_status_string"}
    assert set(calls) == launching


def test_python_wrappers_reject_mismatched_tensors(monkeypatch):
    """A factor, output or workspace that does not fit the sizes of the call is refused by the binding
    before any pointer reaches the library (on the device it would be an out-of-bounds access)."""
    torch = pytest.importorskip("torch")
    monkeypatch.setattr(B, "_is_gpu", lambda t: isinstance(t, torch.Tensor))
    monkeypatch.setattr(B, "_ptr", lambda t: None if t is None else t.data_ptr())
    monkeypatch.setattr(B, "_stream", lambda s: None)
    bf = lambda *shape: torch.zeros(shape, dtype=torch.bfloat16)
    ws = torch.zeros(1 << 20, dtype=torch.uint8)
    T, n, b, r = 8, 64, 4, 16
    good = (bf(T, n), bf(b, r, n // b), bf(b, n // b, r), bf(T, n), b, r, 0, ws)
    B.monarch_forward.marshal(*good)
    for i, bad in ((1, bf(b, r + 4, n // b)), (2, bf(b, n // b, 2 * r)), (3, bf(T + 1, n)), (1, torch.zeros((b, r, n // b))),
                   (7, torch.zeros(1 << 20, dtype=torch.float32))):
        args = list(good)
        args[i] = bad
        with pytest.raises(ValueError):
            B.monarch_forward.marshal(*args)
    with pytest.raises(ValueError):
        B.monarch_forward.marshal(bf(T, n), bf(3, r, n // b), bf(3, n // b, r), bf(T, n), 3, r, 0, ws)     # 3 does not divide 64
    with pytest.raises(ValueError):
        B.blast_forward.marshal(bf(T, n), bf(b, n // b, r), bf(b, b, r), bf(b, n // b, r + 8), bf(T, n), b, r, 0, ws)
    with pytest.raises(ValueError):
        B.blast_forward.marshal(bf(T, n), bf(b, n // b, r), None, torch.zeros(8, dtype=torch.uint8), bf(T, n), b, r, B.BLAST_PACKED, ws)
    with pytest.raises(ValueError):
        B.lowrank_forward.marshal(bf(T, n), bf(r, n + 8), bf(48, r), bf(T, 48), 0, ws)
    with pytest.raises(ValueError):
        B.dense_reference_forward.marshal(bf(T, n), bf(n, n + 8), bf(T, n))
