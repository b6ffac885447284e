"""Thin Python binding of the C-ABI library (include/blr.h): argument marshalling only.

Every function has the name of the C entry point without the `blr_` prefix, takes torch tensors
that live on the GPU (PyTorch is used for device memory and streams, nothing else), and passes
their device pointers, the sizes read off their shapes, and the current HIP stream to the library.
Nothing is computed here. If the shared library has not been built the import of the library
fails loudly; there is no fallback.

Every launching function is made of a pure marshaller (tensors -> name of the C entry point, its
argument tuple, the value to return, the objects to keep alive), which also checks shapes, storage
types and devices against each other before any pointer reaches the library: a factor of the wrong
size would otherwise become an out-of-bounds read on the device. `prepared()` calls the same
marshaller once and re-issues the C call from the stored tuple.
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
BLAST_Z_FP8 = 0x8000
BLAST_ONE_KERNEL = 0x10000

EXPORTS = ("blr_status_string", "blr_monarch_workspace_bytes", "blr_monarch_forward",
           "blr_blast_workspace_bytes", "blr_blast_forward", "blr_blast_packed_bytes",
           "blr_blast_pack", "blr_dense_reference_forward",
           "blr_rmsnorm", "blr_residual_add_rmsnorm", "blr_sum3_scaled", "blr_silu_mul",
           "blr_monarch_permute_first_factor", "blr_lowrank_workspace_bytes", "blr_lowrank_forward",
           "blr_monarch_rect_workspace_bytes", "blr_monarch_rect_forward", "blr_sum3_scaled_ld", "blr_silu_mul_ld",
           "blr_blast_group_workspace_bytes", "blr_blast_group_forward",
           "blr_monarch_group_first_factor", "blr_static_scratch_bytes", "blr_monarch_forward_static")

_lib = None


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
        L.blr_static_scratch_bytes.restype = sz
        L.blr_static_scratch_bytes.argtypes = []
        L.blr_monarch_forward_static.restype = ci
        L.blr_monarch_forward_static.argtypes = [vp, vp, vp, vp, i64, ci, ci, ci, ci, ci, cu, vp]
        L.blr_monarch_group_first_factor.restype = ci
        L.blr_monarch_group_first_factor.argtypes = [vp, vp, ci, ci, ci, ci, ci, vp]
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


def _is_gpu(t) -> bool:
    return isinstance(t, torch.Tensor) and t.is_cuda


def _expect(t, what, shape=None, numel=None, like=None):
    """`t` is a GPU tensor of `like`'s storage type and device with the given shape (or element count)."""
    if not _is_gpu(t):
        raise ValueError(f"{what}: expected a GPU tensor")
    if like is not None and (t.dtype != like.dtype or t.device != like.device):
        raise ValueError(f"{what}: {t.dtype} on {t.device}, expected {like.dtype} on {like.device}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{what}: shape {tuple(t.shape)}, expected {tuple(shape)}")
    if numel is not None and t.numel() != numel:
        raise ValueError(f"{what}: {t.numel()} elements, expected {numel}")


def _div(n, d, what):
    if d <= 0 or n % d:
        raise ValueError(f"{what}: {n} is not a multiple of {d}")
    return n // d


def _workspace(ws, need, like):
    if ws is None:
        ws = torch.empty(max(need, 16), dtype=torch.uint8, device=like.device)
    if not _is_gpu(ws) or ws.dtype != torch.uint8 or ws.device != like.device or not ws.is_contiguous():
        raise ValueError("workspace: expected a contiguous uint8 GPU tensor on the inputs' device")
    return ws


def _launcher(marshal):
    """Public launching function from its marshaller `marshal(*args) -> (c_name, c_args, result, keepalive)`."""
    def call(*args, **kw):
        name, cargs, result, _ = marshal(*args, **kw)
        _check(getattr(lib(), name)(*cargs), name)
        return result
    call.marshal = marshal
    call.__name__, call.__doc__ = marshal.__name__.lstrip("_"), marshal.__doc__
    return call


def prepared(fn, *args, **kw):
    """Marshal the arguments of `fn` (one of the launching functions of this module) ONCE and return
    a zero-argument callable that re-issues exactly that C call. For tight launch loops and graph
    capture: the per-call cost is one foreign-function call, no tensor or stream look-ups. The
    callable keeps the tensors (and a workspace it had to create) alive; the stream is the one
    current at preparation time."""
    name, cargs, _, keep = fn.marshal(*args, **kw)
    cfn = getattr(lib(), name)
    conv = tuple(t(a) if not isinstance(a, t) else a for t, a in zip(cfn.argtypes, cargs))

    def call():
        st = cfn(*conv)
        if st != OK:
            raise BlrError(st, name)
    call.keepalive = keep
    return call


def monarch_workspace_bytes(T, n_in, n_out, nblocks, r, dt) -> int:
    return lib().blr_monarch_workspace_bytes(T, n_in, n_out, nblocks, r, dt)


def _monarch_checks(X, R, L, Y, b_in, b_out, r_block):
    T, n_in = X.shape
    n_out = Y.shape[1]
    _expect(Y, "Y", (T, n_out), like=X)
    _expect(R, "R", (b_in, r_block * b_out, _div(n_in, b_in, "n_in / blocks")), like=X)
    _expect(L, "L", (b_out, _div(n_out, b_out, "n_out / blocks"), b_in * r_block), like=X)
    return T, n_in, n_out


@_launcher
def monarch_forward(X, R, L, Y, nblocks, r, flags=0, workspace=None, stream=None):
    """Y[T][n_out] <- Monarch(X[T][n_in]; R[nblocks][r][n_in/nblocks], L[nblocks][n_out/nblocks][r])."""
    T, n_in, n_out = _monarch_checks(X, R, L, Y, nblocks, nblocks, _div(r, nblocks, "r / nblocks"))
    dt = _dt(X)
    ws = _workspace(workspace, monarch_workspace_bytes(T, n_in, n_out, nblocks, r, dt), X)
    return ("blr_monarch_forward", (_ptr(X), _ptr(R), _ptr(L), _ptr(Y), T, n_in, n_out, nblocks, r, dt, flags,
                                    _ptr(ws), ws.numel(), _stream(stream)), Y, (X, R, L, Y, ws))


def static_scratch_bytes() -> int:
    return lib().blr_static_scratch_bytes()


@_launcher
def monarch_forward_static(X, R, L, Y, nblocks, r, flags=0, stream=None):
    """monarch_forward without a workspace: the intermediate lives in the library's static device array."""
    T, n_in, n_out = _monarch_checks(X, R, L, Y, nblocks, nblocks, _div(r, nblocks, "r / nblocks"))
    return ("blr_monarch_forward_static", (_ptr(X), _ptr(R), _ptr(L), _ptr(Y), T, n_in, n_out, nblocks, r, _dt(X), flags,
                                           _stream(stream)), Y, (X, R, L, Y))


def monarch_rect_workspace_bytes(T, n_in, n_out, b_in, b_out, r_block, dt) -> int:
    return lib().blr_monarch_rect_workspace_bytes(T, n_in, n_out, b_in, b_out, r_block, dt)


@_launcher
def monarch_rect_forward(X, R, L, Y, b_in, b_out, r_block, flags=0, workspace=None, stream=None):
    """Monarch with b_in input and b_out output blocks: R[b_in][r_block*b_out][n_in/b_in], L[b_out][n_out/b_out][b_in*r_block]."""
    T, n_in, n_out = _monarch_checks(X, R, L, Y, b_in, b_out, r_block)
    dt = _dt(X)
    ws = _workspace(workspace, monarch_rect_workspace_bytes(T, n_in, n_out, b_in, b_out, r_block, dt), X)
    return ("blr_monarch_rect_forward", (_ptr(X), _ptr(R), _ptr(L), _ptr(Y), T, n_in, n_out, b_in, b_out, r_block, dt, flags,
                                         _ptr(ws), ws.numel(), _stream(stream)), Y, (X, R, L, Y, ws))


def monarch_permute_first_factor(R, n_in, nblocks, r, stream=None):
    """First factor re-ordered for MONARCH_IN_BLOCKED (one-time weight preparation); returns the new tensor."""
    _expect(R, "R", (nblocks, r, _div(n_in, nblocks, "n_in / nblocks")))
    Rp = torch.empty_like(R)
    _check(lib().blr_monarch_permute_first_factor(_ptr(R), _ptr(Rp), n_in, nblocks, r, _dt(R), _stream(stream)),
           "blr_monarch_permute_first_factor")
    return Rp


def monarch_group_first_factor(R_stack, n_in, nblocks, r, stream=None):
    """First factors of several Monarch layers of one shape, stacked [members][nblocks][r][n_in/nblocks],
    as the first factor [nblocks][members*r][n_in/nblocks] of one layer with members*nblocks output
    blocks (one-time weight preparation); returns the new tensor."""
    members = R_stack.shape[0]
    p = _div(n_in, nblocks, "n_in / nblocks")
    _expect(R_stack, "R_stack", (members, nblocks, r, p))
    Rg = torch.empty((nblocks, members * r, p), dtype=R_stack.dtype, device=R_stack.device)
    _check(lib().blr_monarch_group_first_factor(_ptr(R_stack), _ptr(Rg), n_in, nblocks, r, members, _dt(R_stack), _stream(stream)),
           "blr_monarch_group_first_factor")
    return Rg


def lowrank_workspace_bytes(T, n_in, n_out, r, dt) -> int:
    return lib().blr_lowrank_workspace_bytes(T, n_in, n_out, r, dt)


@_launcher
def lowrank_forward(X, V, U, Y, flags=0, workspace=None, stream=None):
    """Y[T][n_out] <- (X[T][n_in] V[r][n_in]^T) U[n_out][r]^T."""
    T, n_in = X.shape
    n_out, r = U.shape
    _expect(Y, "Y", (T, n_out), like=X)
    _expect(V, "V", (r, n_in), like=X)
    _expect(U, "U", (n_out, r), like=X)
    dt = _dt(X)
    ws = _workspace(workspace, lowrank_workspace_bytes(T, n_in, n_out, r, dt), X)
    return ("blr_lowrank_forward", (_ptr(X), _ptr(V), _ptr(U), _ptr(Y), T, n_in, n_out, r, dt, flags,
                                    _ptr(ws), ws.numel(), _stream(stream)), Y, (X, V, U, Y, ws))


def blast_workspace_bytes(T, n_in, n_out, b, r, dt, flags=0) -> int:
    return lib().blr_blast_workspace_bytes(T, n_in, n_out, b, r, dt, flags)


@_launcher
def blast_forward(X, U, S, V, Y, b, r, flags=0, workspace=None, stream=None):
    """Y[T][n_out] <- BLAST(X[T][n_in]; U[b][n_out/b][r], S[b][b][r], V[b][n_in/b][r]);
    with BLAST_PACKED in flags, V is the buffer returned by blast_pack and S is None."""
    T, n_in = X.shape
    n_out = Y.shape[1]
    dt = _dt(X)
    _expect(Y, "Y", (T, n_out), like=X)
    _expect(U, "U", (b, _div(n_out, b, "n_out / b"), r), like=X)
    if flags & BLAST_PACKED:
        if V.dtype != torch.uint8 or V.numel() < max(blast_packed_bytes(n_in, n_out, b, r, dt), 16) or not _is_gpu(V) or V.device != X.device:
            raise ValueError("V: with BLAST_PACKED, expected the uint8 buffer blast_pack returned for these sizes")
    else:
        _expect(S, "S", (b, b, r), like=X)
        _expect(V, "V", (b, _div(n_in, b, "n_in / b"), r), like=X)
    ws = _workspace(workspace, blast_workspace_bytes(T, n_in, n_out, b, r, dt, flags), X)
    return ("blr_blast_forward", (_ptr(X), _ptr(U), _ptr(S), _ptr(V), _ptr(Y), T, n_in, n_out, b, r, dt, flags,
                                  _ptr(ws), ws.numel(), _stream(stream)), Y, (X, U, S, V, Y, ws))


def blast_group_workspace_bytes(T, n_in, n_out, b, r, members, dt=BF16, flags=0) -> int:
    return lib().blr_blast_group_workspace_bytes(T, n_in, n_out, b, r, members, dt, flags)


@_launcher
def blast_group_forward(X, U, packed, Y, b, r, members, flags=0, workspace=None, stream=None):
    """Y[T][members*n_out] <- `members` BLAST layers of one shape on the same X[T][n_in];
    U[members][b][n_out/b][r] stacked, `packed` = blast_pack of the members' S and V concatenated
    along the rank index (rank members*r)."""
    T, n_in = X.shape
    n_out = _div(Y.shape[1], members, "columns of Y / members")
    dt = _dt(X)
    _expect(Y, "Y", (T, members * n_out), like=X)
    _expect(U, "U", (members, b, _div(n_out, b, "n_out / b"), r), like=X)
    if packed.dtype != torch.uint8 or packed.numel() < max(blast_packed_bytes(n_in, n_out, b, members * r, dt), 16) or packed.device != X.device:
        raise ValueError("packed: expected the uint8 buffer blast_pack returned for rank members*r")
    ws = _workspace(workspace, blast_group_workspace_bytes(T, n_in, n_out, b, r, members, dt, flags), X)
    return ("blr_blast_group_forward", (_ptr(X), _ptr(U), _ptr(packed), _ptr(Y), T, n_in, n_out, b, r, members, dt, flags,
                                        _ptr(ws), ws.numel(), _stream(stream)), Y, (X, U, packed, Y, ws))


def blast_packed_bytes(n_in, n_out, b, r, dt=BF16) -> int:
    return lib().blr_blast_packed_bytes(n_in, n_out, b, r, dt)


def blast_pack(U, S, V, n_in, n_out, b, r, stream=None):
    """One-time re-layout of the BLAST factors; returns the opaque packed buffer to pass as `V`
    (with `S=None`) to blast_forward together with the BLAST_PACKED flag."""
    dt = _dt(V)
    _expect(V, "V", (b, _div(n_in, b, "n_in / b"), r))
    _expect(S, "S", (b, b, r), like=V)
    _expect(U, "U", numel=n_out * r, like=V)          # [b][n_out/b][r], or several members of a group stacked
    packed = torch.empty(max(blast_packed_bytes(n_in, n_out, b, r, dt), 16), dtype=torch.uint8, device=V.device)
    _check(lib().blr_blast_pack(_ptr(U), _ptr(S), _ptr(V), _ptr(packed), n_in, n_out, b, r, dt, _stream(stream)),
           "blr_blast_pack")
    return packed


@_launcher
def dense_reference_forward(X, W, Y, flags=0, stream=None):
    """Y[T][n_out] <- X[T][n_in] W[n_out][n_in]^T."""
    T, n_in = X.shape
    n_out = Y.shape[1]
    _expect(Y, "Y", (T, n_out), like=X)
    _expect(W, "W", (n_out, n_in), like=X)
    return ("blr_dense_reference_forward", (_ptr(X), _ptr(W), _ptr(Y), T, n_in, n_out, _dt(X), flags, _stream(stream)), Y, (X, W, Y))


@_launcher
def rmsnorm(H, N, eps=1e-6, stream=None):
    """N[t] <- H[t] / sqrt(mean(H[t]^2) + eps)."""
    T, d = H.shape
    _expect(N, "N", (T, d), like=H)
    return ("blr_rmsnorm", (_ptr(H), _ptr(N), T, d, eps, _dt(H), _stream(stream)), N, (H, N))


@_launcher
def residual_add_rmsnorm(H, Y, N=None, eps=1e-6, stream=None):
    """H <- H + Y in place; if N is given, N <- rmsnorm(H) of the updated H."""
    T, d = H.shape
    _expect(Y, "Y", (T, d), like=H)
    if N is not None:
        _expect(N, "N", (T, d), like=H)
    return ("blr_residual_add_rmsnorm", (_ptr(H), _ptr(Y), _ptr(N), T, d, eps, _dt(H), _stream(stream)), H, (H, Y, N))


@_launcher
def sum3_scaled(Q, K, V, A, scale, stream=None):
    """A <- (Q + K + V) * scale. Q, K, V may be column slices of one wider tensor (equal row strides)."""
    T, d = Q.shape
    for t, what in ((K, "K"), (V, "V"), (A, "A")):
        _expect(t, what, (T, d), like=Q)
    if Q.stride(0) != d:
        if not (Q.stride(0) == K.stride(0) == V.stride(0) and Q.stride(1) == 1 and A.is_contiguous()):
            raise ValueError("column slices must share one row stride and the output must be contiguous")
        return ("blr_sum3_scaled_ld", (_ptr_rows(Q), _ptr_rows(K), _ptr_rows(V), _ptr(A), T, d, Q.stride(0), scale, _dt(Q),
                                       _stream(stream)), A, (Q, K, V, A))
    return ("blr_sum3_scaled", (_ptr(Q), _ptr(K), _ptr(V), _ptr(A), T, d, scale, _dt(Q), _stream(stream)), A, (Q, K, V, A))


@_launcher
def silu_mul(G, U, M, stream=None):
    """M <- silu(G) * U. G, U may be column slices of one wider tensor (equal row strides)."""
    T, d = G.shape
    _expect(U, "U", (T, d), like=G)
    _expect(M, "M", (T, d), like=G)
    if G.stride(0) != d:
        if not (G.stride(0) == U.stride(0) and G.stride(1) == 1 and M.is_contiguous()):
            raise ValueError("column slices must share one row stride and the output must be contiguous")
        return ("blr_silu_mul_ld", (_ptr_rows(G), _ptr_rows(U), _ptr(M), T, d, G.stride(0), _dt(G), _stream(stream)), M, (G, U, M))
    return ("blr_silu_mul", (_ptr(G), _ptr(U), _ptr(M), T, d, _dt(G), _stream(stream)), M, (G, U, M))
