"""Sequencing of the library calls for adapter-aware MoE layers (paper Sec. 2.1 + Sec. 4).

No arithmetic happens here: this module only owns device buffers (PyTorch tensors), loads a
pool from per-class weight stacks, and issues the C-ABI calls in order on the current stream:

    moe_gate_logits -> moe_route_reroute_permute_plan (also writes the FFN's work plan) ->
    moe_grouped_ffn_planned (routed experts on the pool's virtual weight tensors and the shared
    experts, one launch) -> moe_unpermute (+ residual; in a stack also the next layer's norm)

fp32 layers (test-only kernels) call moe_route_reroute_permute and moe_grouped_ffn instead, the
shared experts' call on a second stream.
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
        self.out = torch.empty((T_max, H), dtype=dtype, device=device)
        lib = B.lib()
        self.dt = B.EW_BF16 if dtype == torch.bfloat16 else B.EW_F32
        self.ws_perm = B._workspace(lib.moe_reroute_permute_workspace_bytes(T_max, k, P), device)
        # one launch for routed and shared experts where the library supports it (bf16)
        self.planned = dtype == torch.bfloat16 and H % 128 == 0 and I % 128 == 0
        self.fused_shared = bool(S) and self.planned
        Sf = S if self.fused_shared else 0
        self.y = torch.empty((T_max * (k + Sf), H), dtype=dtype, device=device)
        self.ws_ffn = B._workspace(lib.moe_grouped_ffn_workspace_bytes(T_max, k + Sf, H, I, P + Sf, self.dt), device)
        if S and not self.fused_shared:
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
        self.T_max = self._T = T_max
        self.buf = buffers if buffers is not None else LayerBuffers(T_max, self.M, k, self.H, I, self.P, self.S, dtype, Wg.device)
        b = self.buf
        assert (b.T_max, b.M, b.k, b.H, b.I, b.P, b.S, b.dtype) == (T_max, self.M, k, self.H, I, self.P, self.S, dtype)
        self.dt = b.dt
        # Two-call layers only: the shared experts depend only on the layer input, so their call runs on a stream of its
        # own (default priority) beside the router and the routed experts and is joined before the combine.
        self.side = b.side if self.S and not b.fused_shared else None

    # intermediates of the last forward (views of the shared buffers)
    logits = property(lambda self: self.buf.logits)
    ids = property(lambda self: self.buf.ids)
    w = property(lambda self: self.buf.w)
    slot = property(lambda self: self.buf.slot)
    counts = property(lambda self: self.buf.counts)
    offsets = property(lambda self: self.buf.offsets)
    por = property(lambda self: self.buf.por)
    rop = property(lambda self: self.buf.rop)
    y = property(lambda self: self.buf.y[:self._T * self.k])                 # routed rows of the last forward
    y_shared = property(lambda self: self.buf.y[self._T * self.k:self._T * (self.k + self.S)] if self.buf.fused_shared
                        else self.buf.y_sh[:self.S * self._T])              # [S*T, H] shared-expert outputs of the last forward
    out = property(lambda self: self.buf.out)
    ws_ffn = property(lambda self: self.buf.ws_ffn)

    def route(self, x: torch.Tensor, aid: torch.Tensor, logits: torch.Tensor | None = None, plan: bool = False):
        """Router scores (unless given) and the fused top-k + rerouting + permutation; fills the buffers.
        plan: also have the grouped FFN's work plan written into its workspace (bf16 layers)."""
        lib, st, b = B.lib(), B._stream(), self.buf
        T, H, k, P = x.shape[0], self.H, self.k, self.P
        if logits is None:
            logits = b.logits
            B._check(lib.moe_gate_logits(x.data_ptr(), self.dt, self.Wg.data_ptr(), T, H, self.M,
                                         aid.data_ptr() if self.bias is not None else None,
                                         self.bias.data_ptr() if self.bias is not None else None,
                                         logits.data_ptr(), st))
        args = (logits.data_ptr(), aid.data_ptr(), self.emap, T, self.M, k, self.N, P, int(self.renormalize), b.ids.data_ptr(),
                b.w.data_ptr(), b.slot.data_ptr(), b.counts.data_ptr(), b.offsets.data_ptr(), b.por.data_ptr(), b.rop.data_ptr(),
                B._ptr(b.ws_perm), b.ws_perm.numel() if b.ws_perm is not None else 0)
        if plan:
            B._check(lib.moe_route_reroute_permute_plan(*args, H, self.I, self.S if b.fused_shared else 0, self.dt,
                                                        b.ws_ffn.data_ptr(), b.ws_ffn.numel(), st))
        else:
            B._check(lib.moe_route_reroute_permute(*args, st))

    def forward(self, x: torch.Tensor, aid: torch.Tensor, logits: torch.Tensor | None = None,
                residual: torch.Tensor | None = None, out: torch.Tensor | None = None,
                normed_out: torch.Tensor | None = None, eps: float = 0.0) -> torch.Tensor:
        """normed_out: if given, also receives the RMS-normalised result (the next layer's input in a stack)."""
        lib, st, b = B.lib(), B._stream(), self.buf
        T, H, k, P, I = x.shape[0], self.H, self.k, self.P, self.I
        assert T <= self.T_max and x.dtype == self.dtype and x.is_contiguous()
        self._T = T
        sh_ptr = None
        two_calls = self.S and not b.fused_shared
        if two_calls:
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
        planned = b.planned                       # bf16 layers: the permutation call writes the FFN's work plan
        self.route(x, aid, logits, plan=planned)
        if planned:
            fused = self.S and b.fused_shared
            B._check(lib.moe_grouped_ffn_planned(x.data_ptr(), self.dt, T, k, H, I, P, self.S if fused else 0,
                                                 b.counts.data_ptr(), b.offsets.data_ptr(), b.por.data_ptr(), self.w13_base,
                                                 self.w2_base, self.shared_w13.data_ptr() if fused else None,
                                                 self.shared_w2.data_ptr() if fused else None, b.y.data_ptr(),
                                                 b.ws_ffn.data_ptr(), b.ws_ffn.numel(), st))
            if fused:
                sh_ptr = b.y.data_ptr() + T * k * H * b.y.element_size()
        else:
            B._check(lib.moe_grouped_ffn(x.data_ptr(), self.dt, T, k, H, I, P, b.counts.data_ptr(),
                                         b.offsets.data_ptr(), b.por.data_ptr(), self.w13_base, self.w2_base,
                                         b.y.data_ptr(), b.ws_ffn.data_ptr(), b.ws_ffn.numel(), st))
        if two_calls:
            torch.cuda.current_stream().wait_event(b.ev_out)
        dst = b.out if out is None else out
        res_ptr = residual.data_ptr() if residual is not None else None
        if normed_out is not None:
            B._check(lib.moe_unpermute_rmsnorm(b.y.data_ptr(), b.rop.data_ptr(), b.w.data_ptr(), sh_ptr, self.S, res_ptr, T, k, H,
                                               self.dt, dst.data_ptr(), eps, normed_out.data_ptr(), st))
        else:
            B._check(lib.moe_unpermute(b.y.data_ptr(), b.rop.data_ptr(), b.w.data_ptr(), sh_ptr, self.S, res_ptr, T, k, H,
                                       self.dt, dst.data_ptr(), st))
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
        self._normed = [torch.empty((T_max, H), dtype=dtype, device=dev) for _ in range(2)]
        self.normed = self._normed[0]
        self.eps = eps

    def forward(self, x: torch.Tensor, aid: torch.Tensor, first: int = 0, last: int | None = None) -> torch.Tensor:
        """Runs layers [first, last) on x; returns the hidden state after the last of them.
        self.normed holds the last layer's normalised input afterwards.  Only the first layer's input is normalised by
        a call of its own: every layer's combine also writes the normalised input of the next one."""
        last = len(self.layers) if last is None else last
        T, h = x.shape[0], x
        lib, st = B.lib(), B._stream()
        cur = self._normed[0]
        B._check(lib.moe_rmsnorm(h.data_ptr(), self.buf.dt, T, h.shape[1], self.eps, cur.data_ptr(), st))
        for l in range(first, last):
            dst = self.h[l & 1]
            if dst.data_ptr() == h.data_ptr():
                dst = self.h[(l + 1) & 1]
            nxt = self._normed[1] if cur is self._normed[0] else self._normed[0]
            self.layers[l].forward(cur[:T], aid, residual=h, out=dst, normed_out=nxt if l + 1 < last else None, eps=self.eps)
            self.normed = cur
            h = dst[:T]
            cur = nxt
        return h
