"""Thin Python binding of the C-ABI library (include/blr.h): argument marshalling only.

Every function has the name of the C entry point without the `blr_` prefix, takes torch tensors
that live on the GPU (PyTorch is used for device memory and streams, nothing else), and passes
their device pointers, the sizes read off their shapes, and the current HIP stream to the library.
Nothing is computed here. If the shared library has not been built the import of the library
fails loudly; there is no fallback.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libblr.so")

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_LAUNCH = 0, 1, 2, 3, 4
F32, BF16 = 0, 1
MONARCH_OUT_INTERLEAVED, MONARCH_OUT_BLOCKED, BLAST_PACKED, FORCE_GENERIC = 0, 1, 2, 0x100
MONARCH_IN_BLOCKED = 4
ONLY_FIRST_STAGE, ONLY_LAST_STAGE = 0x200, 0x400
BLAST_FUSED_STAGE12 = 0x800
BLAST_THREE_KERNELS = 0x1000
MONARCH_FUSED, MONARCH_TWO_KERNELS = 0x2000, 0x4000

EXPORTS = ("blr_status_string", "blr_monarch_workspace_bytes", "blr_monarch_forward",
           "blr_blast_workspace_bytes", "blr_blast_forward", "blr_blast_packed_bytes",
           "blr_blast_pack", "blr_dense_reference_forward",
           "blr_rmsnorm", "blr_residual_add_rmsnorm", "blr_sum3_scaled", "blr_silu_mul",
           "blr_monarch_permute_first_factor", "blr_lowrank_workspace_bytes", "blr_lowrank_forward",
           "blr_monarch_rect_workspace_bytes", "blr_monarch_rect_forward", "blr_sum3_scaled_ld", "blr_silu_mul_ld",
           "blr_blast_group_workspace_bytes", "blr_blast_group_forward")
# entry points that enqueue work and return a status: the ones prepared() can record
_LAUNCHERS = ("blr_monarch_forward", "blr_blast_forward", "blr_dense_reference_forward", "blr_lowrank_forward", "blr_monarch_rect_forward",
              "blr_rmsnorm", "blr_residual_add_rmsnorm", "blr_sum3_scaled", "blr_silu_mul", "blr_sum3_scaled_ld", "blr_silu_mul_ld",
              "blr_blast_group_forward")

_lib = None
_last_workspace = None     # the workspace the latest forward call ran with (kept alive for prepared())


class BlrError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


def lib() -> ctypes.CDLL:
    """Load libblr.so (built by paper_2512_20861_amd.build / __graft_entry__.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2512_20861_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, ci, cu, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_uint, ctypes.c_size_t
        L.blr_status_string.restype = ctypes.c_char_p
        L.blr_status_string.argtypes = [ci]
        L.blr_monarch_workspace_bytes.restype = sz
        L.blr_monarch_workspace_bytes.argtypes = [i64, ci, ci, ci, ci, ci]
        L.blr_monarch_forward.restype = ci
        L.blr_monarch_forward.argtypes = [vp, vp, vp, vp, i64, ci, ci, ci, ci, ci, cu, vp, sz, vp]
        L.blr_monarch_rect_workspace_bytes.restype = sz
        L.blr_monarch_rect_workspace_bytes.argtypes = [i64, ci, ci, ci, ci, ci, ci]
        L.blr_monarch_rect_forward.restype = ci
        L.blr_monarch_rect_forward.argtypes = [vp, vp, vp, vp, i64, ci, ci, ci, ci, ci, ci, cu, vp, sz, vp]
        L.blr_lowrank_workspace_bytes.restype = sz
        L.blr_lowrank_workspace_bytes.argtypes = [i64, ci, ci, ci, ci]
        L.blr_lowrank_forward.restype = ci
        L.blr_lowrank_forward.argtypes = [vp, vp, vp, vp, i64, ci, ci, ci, ci, cu, vp, sz, vp]
        L.blr_blast_workspace_bytes.restype = sz
        L.blr_blast_workspace_bytes.argtypes = [i64, ci, ci, ci, ci, ci, cu]
        L.blr_blast_forward.restype = ci
        L.blr_blast_forward.argtypes = [vp, vp, vp, vp, vp, i64, ci, ci, ci, ci, ci, cu, vp, sz, vp]
        L.blr_blast_group_workspace_bytes.restype = sz
        L.blr_blast_group_workspace_bytes.argtypes = [i64, ci, ci, ci, ci, ci, ci, cu]
        L.blr_blast_group_forward.restype = ci
        L.blr_blast_group_forward.argtypes = [vp, vp, vp, vp, i64, ci, ci, ci, ci, ci, ci, cu, vp, sz, vp]
        L.blr_blast_packed_bytes.restype = sz
        L.blr_blast_packed_bytes.argtypes = [ci, ci, ci, ci, ci]
        L.blr_blast_pack.restype = ci
        L.blr_blast_pack.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, ci, vp]
        L.blr_dense_reference_forward.restype = ci
        L.blr_dense_reference_forward.argtypes = [vp, vp, vp, i64, ci, ci, ci, cu, vp]
        L.blr_monarch_permute_first_factor.restype = ci
        L.blr_monarch_permute_first_factor.argtypes = [vp, vp, ci, ci, ci, ci, vp]
        cf = ctypes.c_float
        L.blr_rmsnorm.restype = ci
        L.blr_rmsnorm.argtypes = [vp, vp, i64, ci, cf, ci, vp]
        L.blr_residual_add_rmsnorm.restype = ci
        L.blr_residual_add_rmsnorm.argtypes = [vp, vp, vp, i64, ci, cf, ci, vp]
        L.blr_sum3_scaled.restype = ci
        L.blr_sum3_scaled.argtypes = [vp, vp, vp, vp, i64, ci, cf, ci, vp]
        L.blr_silu_mul.restype = ci
        L.blr_silu_mul.argtypes = [vp, vp, vp, i64, ci, ci, vp]
        L.blr_sum3_scaled_ld.restype = ci
        L.blr_sum3_scaled_ld.argtypes = [vp, vp, vp, vp, i64, ci, i64, cf, ci, vp]
        L.blr_silu_mul_ld.restype = ci
        L.blr_silu_mul_ld.argtypes = [vp, vp, vp, i64, ci, i64, ci, vp]
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().blr_status_string(status).decode()


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float32:
        return F32
    raise TypeError(f"unsupported storage type {t.dtype}")


def _ptr(t):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensors must be contiguous GPU tensors")
    return t.data_ptr()


def _ptr_rows(t):
    """Pointer of a GPU tensor [T][d] whose rows may be further apart than d (a column slice)."""
    if not t.is_cuda or t.dim() != 2 or t.stride(1) != 1:
        raise ValueError("expected a 2-D GPU tensor with contiguous rows")
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _check(status: int, where: str):
    if status != OK:
        raise BlrError(status, where)


def monarch_workspace_bytes(T, n_in, n_out, nblocks, r, dt) -> int:
    return lib().blr_monarch_workspace_bytes(T, n_in, n_out, nblocks, r, dt)


def monarch_forward(X, R, L, Y, nblocks, r, flags=0, workspace=None, stream=None):
    """Y[T][n_out] <- Monarch(X[T][n_in]; R[nblocks][r][n_in/nblocks], L[nblocks][n_out/nblocks][r])."""
    T, n_in = X.shape
    n_out = Y.shape[1]
    dt = _dt(X)
    if workspace is None:
        workspace = torch.empty(max(monarch_workspace_bytes(T, n_in, n_out, nblocks, r, dt), 16),
                                dtype=torch.uint8, device=X.device)
    global _last_workspace
    _last_workspace = workspace
    _check(lib().blr_monarch_forward(_ptr(X), _ptr(R), _ptr(L), _ptr(Y), T, n_in, n_out, nblocks, r, dt, flags,
                                     _ptr(workspace), workspace.numel(), _stream(stream)), "blr_monarch_forward")
    return Y


def monarch_rect_workspace_bytes(T, n_in, n_out, b_in, b_out, r_block, dt) -> int:
    return lib().blr_monarch_rect_workspace_bytes(T, n_in, n_out, b_in, b_out, r_block, dt)


def monarch_rect_forward(X, R, L, Y, b_in, b_out, r_block, flags=0, workspace=None, stream=None):
    """Monarch with b_in input and b_out output blocks: R[b_in][r_block*b_out][n_in/b_in], L[b_out][n_out/b_out][b_in*r_block]."""
    T, n_in = X.shape
    n_out = Y.shape[1]
    dt = _dt(X)
    if workspace is None:
        workspace = torch.empty(max(monarch_rect_workspace_bytes(T, n_in, n_out, b_in, b_out, r_block, dt), 16),
                                dtype=torch.uint8, device=X.device)
    global _last_workspace
    _last_workspace = workspace
    _check(lib().blr_monarch_rect_forward(_ptr(X), _ptr(R), _ptr(L), _ptr(Y), T, n_in, n_out, b_in, b_out, r_block, dt, flags,
                                          _ptr(workspace), workspace.numel(), _stream(stream)), "blr_monarch_rect_forward")
    return Y


def monarch_permute_first_factor(R, n_in, nblocks, r, stream=None):
    """First factor re-ordered for MONARCH_IN_BLOCKED (one-time weight preparation); returns the new tensor."""
    Rp = torch.empty_like(R)
    _check(lib().blr_monarch_permute_first_factor(_ptr(R), _ptr(Rp), n_in, nblocks, r, _dt(R), _stream(stream)),
           "blr_monarch_permute_first_factor")
    return Rp


def lowrank_workspace_bytes(T, n_in, n_out, r, dt) -> int:
    return lib().blr_lowrank_workspace_bytes(T, n_in, n_out, r, dt)


def lowrank_forward(X, V, U, Y, flags=0, workspace=None, stream=None):
    """Y[T][n_out] <- (X[T][n_in] V[r][n_in]^T) U[n_out][r]^T."""
    T, n_in = X.shape
    n_out, r = U.shape
    dt = _dt(X)
    if workspace is None:
        workspace = torch.empty(max(lowrank_workspace_bytes(T, n_in, n_out, r, dt), 16), dtype=torch.uint8, device=X.device)
    global _last_workspace
    _last_workspace = workspace
    _check(lib().blr_lowrank_forward(_ptr(X), _ptr(V), _ptr(U), _ptr(Y), T, n_in, n_out, r, dt, flags,
                                     _ptr(workspace), workspace.numel(), _stream(stream)), "blr_lowrank_forward")
    return Y


def blast_workspace_bytes(T, n_in, n_out, b, r, dt, flags=0) -> int:
    return lib().blr_blast_workspace_bytes(T, n_in, n_out, b, r, dt, flags)


def blast_forward(X, U, S, V, Y, b, r, flags=0, workspace=None, stream=None):
    """Y[T][n_out] <- BLAST(X[T][n_in]; U[b][n_out/b][r], S[b][b][r], V[b][n_in/b][r]);
    with BLAST_PACKED in flags, V is the buffer returned by blast_pack and S is None."""
    T, n_in = X.shape
    n_out = Y.shape[1]
    dt = _dt(X)
    if workspace is None:
        workspace = torch.empty(max(blast_workspace_bytes(T, n_in, n_out, b, r, dt, flags), 16),
                                dtype=torch.uint8, device=X.device)
    global _last_workspace
    _last_workspace = workspace
    _check(lib().blr_blast_forward(_ptr(X), _ptr(U), _ptr(S), _ptr(V), _ptr(Y), T, n_in, n_out, b, r, dt, flags,
                                   _ptr(workspace), workspace.numel(), _stream(stream)), "blr_blast_forward")
    return Y


def blast_group_workspace_bytes(T, n_in, n_out, b, r, members, dt=BF16, flags=0) -> int:
    return lib().blr_blast_group_workspace_bytes(T, n_in, n_out, b, r, members, dt, flags)


def blast_group_forward(X, U, packed, Y, b, r, members, flags=0, workspace=None, stream=None):
    """Y[T][members*n_out] <- `members` BLAST layers of one shape on the same X[T][n_in];
    U[members][b][n_out/b][r] stacked, `packed` = blast_pack of the members' S and V concatenated
    along the rank index (rank members*r)."""
    T, n_in = X.shape
    n_out = Y.shape[1] // members
    dt = _dt(X)
    if workspace is None:
        workspace = torch.empty(max(blast_group_workspace_bytes(T, n_in, n_out, b, r, members, dt, flags), 16),
                                dtype=torch.uint8, device=X.device)
    global _last_workspace
    _last_workspace = workspace
    _check(lib().blr_blast_group_forward(_ptr(X), _ptr(U), _ptr(packed), _ptr(Y), T, n_in, n_out, b, r, members, dt, flags,
                                         _ptr(workspace), workspace.numel(), _stream(stream)), "blr_blast_group_forward")
    return Y


def blast_packed_bytes(n_in, n_out, b, r, dt=BF16) -> int:
    return lib().blr_blast_packed_bytes(n_in, n_out, b, r, dt)


def blast_pack(U, S, V, n_in, n_out, b, r, stream=None):
    """One-time re-layout of the BLAST factors; returns the opaque packed buffer to pass as `V`
    (with `S=None`) to blast_forward together with the BLAST_PACKED flag."""
    dt = _dt(V)
    packed = torch.empty(max(blast_packed_bytes(n_in, n_out, b, r, dt), 16), dtype=torch.uint8, device=V.device)
    _check(lib().blr_blast_pack(_ptr(U), _ptr(S), _ptr(V), _ptr(packed), n_in, n_out, b, r, dt, _stream(stream)),
           "blr_blast_pack")
    return packed


def prepared(fn, *args, **kw):
    """Marshal the arguments of `fn` (one of the launching functions of this module) ONCE and return
    a zero-argument callable that re-issues exactly that C call. For tight launch loops: the
    per-call cost is one foreign-function call, no tensor or stream look-ups. The tensors must stay
    alive (pass an explicit workspace, or keep the returned callable's `.keepalive`) and the stream
    is the one current at preparation time."""
    captured = []

    real = lib()

    class _Recorder:
        def __getattr__(self, name):
            if name not in _LAUNCHERS:
                return getattr(real, name)      # size queries run for real
            def rec(*cargs):
                captured.append((name, cargs))
                return OK
            return rec

    global _lib
    _lib = _Recorder()
    try:
        fn(*args, **kw)
    finally:
        _lib = real
    (name, cargs), = captured
    cfn = getattr(real, name)
    conv = tuple(t(a) if not isinstance(a, t) else a for t, a in zip(cfn.argtypes, cargs))

    def call():
        st = cfn(*conv)
        if st != OK:
            raise BlrError(st, name)
    call.keepalive = (args, kw, _last_workspace)
    return call


def dense_reference_forward(X, W, Y, flags=0, stream=None):
    """Y[T][n_out] <- X[T][n_in] W[n_out][n_in]^T."""
    T, n_in = X.shape
    n_out = Y.shape[1]
    _check(lib().blr_dense_reference_forward(_ptr(X), _ptr(W), _ptr(Y), T, n_in, n_out, _dt(X), flags,
                                             _stream(stream)), "blr_dense_reference_forward")
    return Y


def rmsnorm(H, N, eps=1e-6, stream=None):
    """N[t] <- H[t] / sqrt(mean(H[t]^2) + eps)."""
    T, d = H.shape
    _check(lib().blr_rmsnorm(_ptr(H), _ptr(N), T, d, eps, _dt(H), _stream(stream)), "blr_rmsnorm")
    return N


def residual_add_rmsnorm(H, Y, N=None, eps=1e-6, stream=None):
    """H <- H + Y in place; if N is given, N <- rmsnorm(H) of the updated H."""
    T, d = H.shape
    _check(lib().blr_residual_add_rmsnorm(_ptr(H), _ptr(Y), _ptr(N), T, d, eps, _dt(H), _stream(stream)),
           "blr_residual_add_rmsnorm")
    return H


def sum3_scaled(Q, K, V, A, scale, stream=None):
    """A <- (Q + K + V) * scale. Q, K, V may be column slices of one wider tensor (equal row strides)."""
    T, d = Q.shape
    if Q.stride(0) != d:
        assert Q.stride(0) == K.stride(0) == V.stride(0) and Q.stride(1) == 1 and A.is_contiguous()
        _check(lib().blr_sum3_scaled_ld(_ptr_rows(Q), _ptr_rows(K), _ptr_rows(V), _ptr(A), T, d, Q.stride(0), scale, _dt(Q), _stream(stream)),
               "blr_sum3_scaled_ld")
        return A
    _check(lib().blr_sum3_scaled(_ptr(Q), _ptr(K), _ptr(V), _ptr(A), T, d, scale, _dt(Q), _stream(stream)), "blr_sum3_scaled")
    return A


def silu_mul(G, U, M, stream=None):
    """M <- silu(G) * U. G, U may be column slices of one wider tensor (equal row strides)."""
    T, d = G.shape
    if G.stride(0) != d:
        assert G.stride(0) == U.stride(0) and G.stride(1) == 1 and M.is_contiguous()
        _check(lib().blr_silu_mul_ld(_ptr_rows(G), _ptr_rows(U), _ptr(M), T, d, G.stride(0), _dt(G), _stream(stream)), "blr_silu_mul_ld")
        return M
    _check(lib().blr_silu_mul(_ptr(G), _ptr(U), _ptr(M), T, d, _dt(G), _stream(stream)), "blr_silu_mul")
    return M
