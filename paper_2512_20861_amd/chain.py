"""Decoder-layer linear chain on the GPU: seven BLR linears per layer with the glue kernels between
them, every step one call into the C-ABI library (this module only owns buffers and the call list).

Wiring per layer (h is the residual stream, all tensors [T][hidden] or [T][mlp] in bf16 or fp32):

    n = rmsnorm(h);  a = (W_q n + W_k n + W_v n) / sqrt(3);  h += W_o a
    n = rmsnorm(h);  h += W_down( silu(W_gate n) * W_up n )

The residual addition and the following normalisation are one kernel. In an all-Monarch chain the
linears whose output only meets elementwise steps before the next linear (q, k, v -> o; gate, up ->
down) write the BLOCKED output order and their consumer reads it with a first factor re-ordered
once at set-up (the paper's optimisation 3), so no interleaving permutation is ever executed there.
There the linears that share an input (q, k, v; gate, up) also run as ONE call each: n Monarch layers of
equal shape are one general Monarch layer with n * nblocks output blocks once the rows of their
first factors are interleaved (done once at set-up by blr_monarch_group_first_factor), which turns 2 n launch-bound GEMMs into two
larger ones; their outputs lie side by side in one tensor and the glue reads them as column slices.
In an all-BLAST chain the same linears run as one grouped BLAST call each (stages 1 and 2 on the
members' concatenated rank indices, one stage-3 product per member).
"""
from __future__ import annotations

import math

import numpy as np
import torch

from . import binding as B

LINEARS = ("q", "k", "v", "o", "gate", "up", "down")


def upload(ht) -> torch.Tensor:
    """Host tensor of the seeded generator (bits + dtype) -> device tensor of the same bits."""
    if ht.dtype == "bf16":
        return torch.from_numpy(ht.bits.view(np.int16).copy()).view(torch.bfloat16).cuda()
    return torch.from_numpy(ht.bits.copy()).cuda()


class _Linear:
    """Device-resident factors of one BLR linear and the argument tuple of its forward call."""

    def __init__(self, host, out_blocked=False, in_blocked=False):
        self.n_in, self.n_out, self.r = host.n_in, host.n_out, host.r
        self.dt = B.BF16 if host.dtype == "bf16" else B.F32
        self.mflags = 0
        if hasattr(host, "R"):
            self.op, self.nb = "monarch", host.nblocks
            self.R, self.L = upload(host.R), upload(host.L)
            if out_blocked:
                self.mflags |= B.MONARCH_OUT_BLOCKED
            if in_blocked:
                self.R = B.monarch_permute_first_factor(self.R, self.n_in, self.nb, self.r)
                self.mflags |= B.MONARCH_IN_BLOCKED
        else:
            self.op, self.b = "blast", host.b
            self.U, self.S, self.V = upload(host.U), upload(host.S), upload(host.V)
            self.S0, self.V0 = self.S, self.V              # canonical forms for a group's own pack; dropped by DeviceChain
            self.flags = 0
            if B.blast_packed_bytes(self.n_in, self.n_out, self.b, self.r, self.dt) > 0:
                self.packed = B.blast_pack(self.U, self.S, self.V, self.n_in, self.n_out, self.b, self.r)
                self.flags = B.BLAST_PACKED
                self.S = self.V = None                      # only the packed form is read from now on

    def workspace_bytes(self, T):
        if self.op == "monarch":
            return B.monarch_workspace_bytes(T, self.n_in, self.n_out, self.nb, self.r, self.dt)
        return B.blast_workspace_bytes(T, self.n_in, self.n_out, self.b, self.r, self.dt, self.flags)

    def call_args(self, X, Y, ws):
        if self.op == "monarch":
            return (B.monarch_forward, X, self.R, self.L, Y, self.nb, self.r, self.mflags, ws)
        if self.flags & B.BLAST_PACKED:
            return (B.blast_forward, X, self.U, None, self.packed, Y, self.b, self.r, self.flags, ws)
        return (B.blast_forward, X, self.U, self.S, self.V, Y, self.b, self.r, self.flags, ws)


class _MonarchGroup:
    """n Monarch linears of equal shape that read the same input, as one general Monarch layer:
    R_g[l][rho * (n b) + layer * b + k] = R_layer[l][rho * b + k],  L_g[layer * b + k] = L_layer[k].
    Output [T][n * n_out], layer by layer, each in the blocked order."""

    def __init__(self, members):
        m0 = members[0]
        assert all(m.op == "monarch" and (m.n_in, m.n_out, m.r, m.nb, m.dt) == (m0.n_in, m0.n_out, m0.r, m0.nb, m0.dt) for m in members)
        self.n, self.n_in, self.n_out, self.nb, self.dt = len(members), m0.n_in, m0.n_out, m0.nb, m0.dt
        self.rp = m0.r // m0.nb
        # the members' first factors one after the other -> the grouped layer's first factor (library call);
        # the second factors one after the other ARE the grouped layer's second factor
        self.R = B.monarch_group_first_factor(torch.stack([m.R for m in members], dim=0).contiguous(), m0.n_in, m0.nb, m0.r)
        self.L = torch.cat([m.L for m in members], dim=0).contiguous()
        self.flags = B.MONARCH_OUT_BLOCKED

    def workspace_bytes(self, T):
        return B.monarch_rect_workspace_bytes(T, self.n_in, self.n * self.n_out, self.nb, self.n * self.nb, self.rp, self.dt)

    def call_args(self, X, Y, ws):
        return (B.monarch_rect_forward, X, self.R, self.L, Y, self.nb, self.n * self.nb, self.rp, self.flags, ws)


class _BlastGroup:
    """n BLAST linears of equal shape that read the same input, as one call: stages 1 and 2 act on
    every rank index by itself, so the members' S and V concatenate along the rank index (packed once
    here); U stays per member. Output [T][n * n_out], member by member."""

    def __init__(self, members):
        m0 = members[0]
        assert all(m.op == "blast" and (m.n_in, m.n_out, m.r, m.b, m.dt) == (m0.n_in, m0.n_out, m0.r, m0.b, m0.dt) for m in members)
        self.n, self.n_in, self.n_out, self.b, self.r, self.dt = len(members), m0.n_in, m0.n_out, m0.b, m0.r, m0.dt
        self.U = torch.stack([m.U for m in members], dim=0).contiguous()
        S = torch.cat([m.S0 for m in members], dim=2).contiguous()
        V = torch.cat([m.V0 for m in members], dim=2).contiguous()
        self.packed = B.blast_pack(self.U, S, V, self.n_in, self.n_out, self.b, self.n * self.r)

    @staticmethod
    def possible(members, T):
        m0 = members[0]
        return all(m.op == "blast" for m in members) and \
            B.blast_group_workspace_bytes(T, m0.n_in, m0.n_out, m0.b, m0.r, len(members), m0.dt) > 0

    def workspace_bytes(self, T):
        return B.blast_group_workspace_bytes(T, self.n_in, self.n_out, self.b, self.r, self.n, self.dt)

    def call_args(self, X, Y, ws):
        return (B.blast_group_forward, X, self.U, self.packed, Y, self.b, self.r, self.n, 0, ws)


class DeviceChain:
    OUT_BLOCKED = ("q", "k", "v", "gate", "up")          # only elementwise steps between these and their consumer
    IN_BLOCKED = ("o", "down")

    def __init__(self, host_layers, T, eps=1e-6, blocked_chaining=True, grouped=True):
        first = host_layers[0]
        self.T, self.eps = T, eps
        self.hidden, self.mlp = first["q"].n_in, first["gate"].n_out
        nb = getattr(first["q"], "nblocks", 0)
        self.blocked = bool(blocked_chaining and nb and self.hidden % (nb * nb) == 0 and self.mlp % (nb * nb) == 0)
        self.layers = [{name: _Linear(layer[name], self.blocked and name in self.OUT_BLOCKED,
                                      self.blocked and name in self.IN_BLOCKED) for name in LINEARS}
                       for layer in host_layers]
        td = torch.bfloat16 if first["q"].dtype == "bf16" else torch.float32
        new = lambda d: torch.empty((T, d), dtype=td, device="cuda")
        self.h, self.n = new(self.hidden), new(self.hidden)
        self.a, self.o, self.dn = (new(self.hidden) for _ in range(3))
        # grouped calls (all-Monarch chain with blocked chaining; all-BLAST chain whose groups have
        # matrix-core kernels): q, k, v and gate, up are column slices
        L0 = self.layers[0]
        blast_groups = all(_BlastGroup.possible(g, T) for g in ([L0[n] for n in "qkv"], [L0["gate"], L0["up"]]))
        self.grouped = bool(grouped and (self.blocked or blast_groups))
        if self.grouped:
            self.qkv, self.gu, self.m = new(3 * self.hidden), new(2 * self.mlp), new(self.mlp)
            self.q, self.k, self.v = (self.qkv[:, i * self.hidden:(i + 1) * self.hidden] for i in range(3))
            self.g, self.u = self.gu[:, :self.mlp], self.gu[:, self.mlp:]
            Group = _MonarchGroup if self.blocked else _BlastGroup
            self.groups = [{"qkv": Group([L[n] for n in "qkv"]), "gu": Group([L["gate"], L["up"]])} for L in self.layers]
        else:
            self.q, self.k, self.v = (new(self.hidden) for _ in range(3))
            self.g, self.u = new(self.mlp), new(self.mlp)
            self.m = self.g                              # the SiLU gate is applied in place
            self.groups = []
        for L in self.layers:
            for lin in L.values():
                if lin.op == "blast":
                    lin.S0 = lin.V0 = None                   # the groups hold their own packed copies
        need = max([lin.workspace_bytes(T) for layer in self.layers for lin in layer.values()] +
                   [grp.workspace_bytes(T) for layer in self.groups for grp in layer.values()])
        self.ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")

    def call_list(self):
        """[(label, (fn, *args)), ...] in execution order; h must hold the input when the first one runs."""
        c = [("rmsnorm", (B.rmsnorm, self.h, self.n, self.eps))]
        last = len(self.layers) - 1
        for li, L in enumerate(self.layers):
            if self.grouped:
                c.append((f"{li}.qkv", self.groups[li]["qkv"].call_args(self.n, self.qkv, self.ws)))
            else:
                c.append((f"{li}.q", L["q"].call_args(self.n, self.q, self.ws)))
                c.append((f"{li}.k", L["k"].call_args(self.n, self.k, self.ws)))
                c.append((f"{li}.v", L["v"].call_args(self.n, self.v, self.ws)))
            c.append((f"{li}.a", (B.sum3_scaled, self.q, self.k, self.v, self.a, 1.0 / math.sqrt(3.0))))
            c.append((f"{li}.o", L["o"].call_args(self.a, self.o, self.ws)))
            c.append((f"{li}.h1", (B.residual_add_rmsnorm, self.h, self.o, self.n, self.eps)))
            if self.grouped:
                c.append((f"{li}.gu", self.groups[li]["gu"].call_args(self.n, self.gu, self.ws)))
            else:
                c.append((f"{li}.gate", L["gate"].call_args(self.n, self.g, self.ws)))
                c.append((f"{li}.up", L["up"].call_args(self.n, self.u, self.ws)))
            c.append((f"{li}.m", (B.silu_mul, self.g, self.u, self.m)))
            c.append((f"{li}.down", L["down"].call_args(self.m, self.dn, self.ws)))
            c.append((f"{li}.h2", (B.residual_add_rmsnorm, self.h, self.dn, None if li == last else self.n, self.eps)))
        return c

    def prepared(self):
        """Zero-argument callables (arguments marshalled once) on the stream that is current now."""
        return [B.prepared(*args) for _, args in self.call_list()]

    def forward(self, x0, record=False, rows=None):
        """Run the chain on x0 [T][hidden] (device tensor); returns h. With record=True also returns, per
        call label, a copy of the tensor that call wrote and of the tensor it read (a grouped call is
        recorded under the labels of its member linears, each with its own slice of the output);
        `rows` (an index tensor) restricts the copies to those token rows."""
        self.h.copy_(x0)
        taps = {}
        keep = (lambda t: t.clone()) if rows is None else (lambda t: t[rows].clone())
        for label, args in self.call_list():
            if record:
                src = keep(args[1])
            args[0](*args[1:])
            if record:
                if args[0] in (B.monarch_rect_forward, B.blast_group_forward):
                    li, grp = label.split(".")
                    for name, part in zip(("q", "k", "v") if grp == "qkv" else ("gate", "up"),
                                          (self.q, self.k, self.v) if grp == "qkv" else (self.g, self.u)):
                        taps[f"{li}.{name}"] = (src, keep(part))
                    continue
                out = {B.rmsnorm: lambda a: a[2], B.sum3_scaled: lambda a: a[4], B.silu_mul: lambda a: a[3],
                       B.residual_add_rmsnorm: lambda a: a[1], B.monarch_forward: lambda a: a[4],
                       B.blast_forward: lambda a: a[5]}[args[0]](args)
                taps[label] = (src, keep(out))
        return (self.h, taps) if record else self.h
