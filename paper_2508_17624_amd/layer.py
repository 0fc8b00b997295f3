"""Sequencing of the library calls for adapter-aware MoE layers (paper Sec. 2.1 + Sec. 4).

No arithmetic happens here: this module only owns device buffers (PyTorch tensors), loads a
pool from per-class weight stacks, and issues the C-ABI calls in order on the current stream:

    moe_gate_logits -> moe_route_reroute_permute -> moe_grouped_ffn (routed, on the pool's
    virtual weight tensors) -> moe_grouped_ffn (shared experts) -> moe_unpermute (+ residual)
"""
from __future__ import annotations

import torch

from . import binding as B


def load_layer(pool: B.ExpertPool, layer: int, base, adapters, tuned):
    """base = (w13 [M,2I,H], w2 [M,H,I]); adapters[i] = (w13 [e_i,2I,H], w2 [e_i,H,I]) for adapter
    i+1 with ascending tuned expert ids tuned[i].  Tensors may live on the host or the device."""
    pool.map(layer, 0, list(range(pool.M)), base[0], base[1])
    for i, (w13, w2) in enumerate(adapters):
        pool.map(layer, i + 1, [int(e) for e in tuned[i]], w13 if len(tuned[i]) else None, w2 if len(tuned[i]) else None)


class LayerBuffers:
    """Every intermediate of one layer pass, allocated once; layers of a stack share one set."""

    def __init__(self, T_max: int, M: int, k: int, H: int, I: int, P: int, S: int, dtype: torch.dtype, device):
        self.T_max, self.M, self.k, self.H, self.I, self.P, self.S, self.dtype = T_max, M, k, H, I, P, S, dtype
        i32 = dict(dtype=torch.int32, device=device)
        self.logits = torch.empty((T_max, M), dtype=torch.float32, device=device)
        self.ids = torch.empty((T_max, k), **i32)
        self.w = torch.empty((T_max, k), dtype=torch.float32, device=device)
        self.slot = torch.empty((T_max, k), **i32)
        self.counts = torch.empty(P, **i32)
        self.offsets = torch.empty(P + 1, **i32)
        self.por = torch.empty(T_max * k, **i32)
        self.rop = torch.empty(T_max * k, **i32)
        self.y = torch.empty((T_max * k, H), dtype=dtype, device=device)
        self.out = torch.empty((T_max, H), dtype=dtype, device=device)
        lib = B.lib()
        self.dt = B.EW_BF16 if dtype == torch.bfloat16 else B.EW_F32
        self.ws_perm = B._workspace(lib.moe_reroute_permute_workspace_bytes(T_max, k, P), device)
        self.ws_ffn = B._workspace(lib.moe_grouped_ffn_workspace_bytes(T_max, k, H, I, P, self.dt), device)
        if S:
            self.side = torch.cuda.Stream(device=device) if torch.device(device).type == "cuda" else None
            self.ev_in, self.ev_out = torch.cuda.Event(), torch.cuda.Event()
            self.y_sh = torch.empty((S * T_max, H), dtype=dtype, device=device)
            self.ws_sh = B._workspace(lib.moe_grouped_ffn_workspace_bytes(S * T_max, 1, H, I, S, self.dt), device)
            self.sh_counts = torch.empty(S, **i32)
            self.sh_offsets = torch.empty(S + 1, **i32)
            self.sh_por = torch.empty(S * T_max, **i32)
            self._sh_T = -1

    def shared_index(self, T: int):
        """Row map of the shared experts (structure only): slab s holds tokens 0..T-1 in order."""
        if self._sh_T != T:
            S = self.S
            self.sh_counts.fill_(T)
            self.sh_offsets.copy_(torch.arange(S + 1, dtype=torch.int32) * T)
            self.sh_por[:S * T].copy_(torch.arange(S * T, dtype=torch.int32) % T)
            self._sh_T = T


class MoELayer:
    """One MoE layer bound to a pool layer."""

    def __init__(self, pool: B.ExpertPool, layer: int, Wg: torch.Tensor, shared_w13, shared_w2, k: int, I: int,
                 T_max: int, dtype: torch.dtype, bias: torch.Tensor | None = None, renormalize: bool = False,
                 buffers: LayerBuffers | None = None):
        self.pool, self.layer, self.k, self.I, self.dtype = pool, layer, k, I, dtype
        self.M, self.N, self.P = pool.M, pool.N, pool.P
        self.Wg, self.bias, self.renormalize = Wg, bias, renormalize
        self.w13_base, self.w2_base, self.emap, _ = pool.view(layer)
        self.H = Wg.shape[1]
        self.S = 0 if shared_w13 is None else shared_w13.shape[0]
        self.shared_w13, self.shared_w2 = shared_w13, shared_w2
        self.T_max = T_max
        self.buf = buffers if buffers is not None else LayerBuffers(T_max, self.M, k, self.H, I, self.P, self.S, dtype, Wg.device)
        b = self.buf
        assert (b.T_max, b.M, b.k, b.H, b.I, b.P, b.S, b.dtype) == (T_max, self.M, k, self.H, I, self.P, self.S, dtype)
        self.dt = b.dt
        # The shared experts depend only on the layer input: they run on a stream of their own
        # (default priority) beside the router and the routed experts and are joined before the
        # combine.  At decode sizes their few workgroups would otherwise leave most CUs idle.
        self.side = b.side if self.S else None

    # intermediates of the last forward (views of the shared buffers)
    logits = property(lambda self: self.buf.logits)
    ids = property(lambda self: self.buf.ids)
    w = property(lambda self: self.buf.w)
    slot = property(lambda self: self.buf.slot)
    counts = property(lambda self: self.buf.counts)
    offsets = property(lambda self: self.buf.offsets)
    por = property(lambda self: self.buf.por)
    rop = property(lambda self: self.buf.rop)
    y = property(lambda self: self.buf.y)
    out = property(lambda self: self.buf.out)
    ws_ffn = property(lambda self: self.buf.ws_ffn)

    def route(self, x: torch.Tensor, aid: torch.Tensor, logits: torch.Tensor | None = None):
        """Router scores (unless given) and the fused top-k + rerouting + permutation; fills the buffers."""
        lib, st, b = B.lib(), B._stream(), self.buf
        T, H, k, P = x.shape[0], self.H, self.k, self.P
        if logits is None:
            logits = b.logits
            B._check(lib.moe_gate_logits(x.data_ptr(), self.dt, self.Wg.data_ptr(), T, H, self.M,
                                         aid.data_ptr() if self.bias is not None else None,
                                         self.bias.data_ptr() if self.bias is not None else None,
                                         logits.data_ptr(), st))
        B._check(lib.moe_route_reroute_permute(logits.data_ptr(), aid.data_ptr(), self.emap, T, self.M, k, self.N, P,
                                               int(self.renormalize), b.ids.data_ptr(), b.w.data_ptr(),
                                               b.slot.data_ptr(), b.counts.data_ptr(), b.offsets.data_ptr(),
                                               b.por.data_ptr(), b.rop.data_ptr(), B._ptr(b.ws_perm),
                                               b.ws_perm.numel() if b.ws_perm is not None else 0, st))

    def forward(self, x: torch.Tensor, aid: torch.Tensor, logits: torch.Tensor | None = None,
                residual: torch.Tensor | None = None, out: torch.Tensor | None = None) -> torch.Tensor:
        lib, st, b = B.lib(), B._stream(), self.buf
        T, H, k, P, I = x.shape[0], self.H, self.k, self.P, self.I
        assert T <= self.T_max and x.dtype == self.dtype and x.is_contiguous()
        sh_ptr = None
        if self.S:
            b.shared_index(T)
            main = torch.cuda.current_stream()
            b.ev_in.record(main)                      # x (and the row map) are ready on the main stream
            self.side.wait_event(b.ev_in)
            B._check(lib.moe_grouped_ffn(x.data_ptr(), self.dt, self.S * T, 1, H, I, self.S, b.sh_counts.data_ptr(),
                                         b.sh_offsets.data_ptr(), b.sh_por.data_ptr(), self.shared_w13.data_ptr(),
                                         self.shared_w2.data_ptr(), b.y_sh.data_ptr(), b.ws_sh.data_ptr(),
                                         b.ws_sh.numel(), self.side.cuda_stream))
            b.ev_out.record(self.side)
            sh_ptr = b.y_sh.data_ptr()
        self.route(x, aid, logits)
        B._check(lib.moe_grouped_ffn(x.data_ptr(), self.dt, T, k, H, I, P, b.counts.data_ptr(),
                                     b.offsets.data_ptr(), b.por.data_ptr(), self.w13_base, self.w2_base,
                                     b.y.data_ptr(), b.ws_ffn.data_ptr(), b.ws_ffn.numel(), st))
        if self.S:
            torch.cuda.current_stream().wait_event(b.ev_out)
        dst = b.out if out is None else out
        B._check(lib.moe_unpermute(b.y.data_ptr(), b.rop.data_ptr(), b.w.data_ptr(), sh_ptr, self.S,
                                   residual.data_ptr() if residual is not None else None, T, k, H, self.dt,
                                   dst.data_ptr(), st))
        return dst[:T]


class MoEStack:
    """L MoE layers over one pool, chained as a pre-norm residual stream
    h_{l+1} = h_l + MoE_l(rmsnorm(h_l)) (no attention: only the MoE-layer path is exercised; the
    normalisation keeps random-initialised layers at a bounded scale).  The layers share one set
    of work buffers."""

    def __init__(self, pool: B.ExpertPool, gates, shared, k: int, I: int, T_max: int, dtype: torch.dtype, eps: float = 1e-6):
        """gates[l]: Wg [M,H]; shared[l]: (w13 [S,2I,H], w2 [S,H,I]) or (None, None)."""
        H, dev = gates[0].shape[1], gates[0].device
        S = 0 if shared[0][0] is None else shared[0][0].shape[0]
        self.buf = LayerBuffers(T_max, pool.M, k, H, I, pool.P, S, dtype, dev)
        self.layers = [MoELayer(pool, l, gates[l], shared[l][0], shared[l][1], k, I, T_max, dtype, buffers=self.buf)
                       for l in range(len(gates))]
        self.h = [torch.empty((T_max, H), dtype=dtype, device=dev) for _ in range(2)]
        self.normed = torch.empty((T_max, H), dtype=dtype, device=dev)
        self.eps = eps

    def forward(self, x: torch.Tensor, aid: torch.Tensor, first: int = 0, last: int | None = None) -> torch.Tensor:
        """Runs layers [first, last) on x; returns the hidden state after the last of them.
        self.normed holds the last layer's normalised input afterwards."""
        last = len(self.layers) if last is None else last
        T, h = x.shape[0], x
        lib, st = B.lib(), B._stream()
        for l in range(first, last):
            dst = self.h[l & 1]
            if dst.data_ptr() == h.data_ptr():
                dst = self.h[(l + 1) & 1]
            B._check(lib.moe_rmsnorm(h.data_ptr(), self.buf.dt, T, h.shape[1], self.eps, self.normed.data_ptr(), st))
            self.layers[l].forward(self.normed[:T], aid, residual=h, out=dst)
            h = dst[:T]
        return h
