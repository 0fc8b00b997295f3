"""Sequencing of the library calls for one adapter-aware MoE layer (paper Sec. 2.1 + Sec. 4).

No arithmetic happens here: this module only owns device buffers (PyTorch tensors), loads a
pool from per-class weight stacks, and issues the C-ABI calls in order on the current stream:

    moe_gate_logits -> moe_route_reroute_permute -> moe_grouped_ffn (routed, on the pool's
    virtual weight tensors) -> moe_grouped_ffn (shared experts) -> moe_unpermute
"""
from __future__ import annotations

import torch

from . import binding as B


def _el_size(dtype: torch.dtype) -> int:
    return 2 if dtype == torch.bfloat16 else 4


def load_layer(pool: B.ExpertPool, layer: int, base, adapters, tuned):
    """base = (w13 [M,2I,H], w2 [M,H,I]); adapters[i] = (w13 [e_i,2I,H], w2 [e_i,H,I]) for adapter
    i+1 with ascending tuned expert ids tuned[i].  Tensors may live on the host or the device."""
    pool.map(layer, 0, list(range(pool.M)), base[0], base[1])
    for i, (w13, w2) in enumerate(adapters):
        pool.map(layer, i + 1, [int(e) for e in tuned[i]], w13 if len(tuned[i]) else None, w2 if len(tuned[i]) else None)


class MoELayer:
    """One MoE layer bound to a pool layer.  All buffers are allocated once, at construction."""

    def __init__(self, pool: B.ExpertPool, layer: int, Wg: torch.Tensor, shared_w13, shared_w2, k: int, I: int,
                 T_max: int, dtype: torch.dtype, bias: torch.Tensor | None = None, renormalize: bool = False):
        dev = Wg.device
        self.pool, self.layer, self.k, self.I, self.dtype = pool, layer, k, I, dtype
        self.M, self.N, self.P = pool.M, pool.N, pool.P
        self.Wg, self.bias, self.renormalize = Wg, bias, renormalize
        self.w13_base, self.w2_base, self.emap, _ = pool.view(layer)
        self.H = Wg.shape[1]
        self.S = 0 if shared_w13 is None else shared_w13.shape[0]
        self.shared_w13, self.shared_w2 = shared_w13, shared_w2
        self.T_max = T_max
        H, P, S = self.H, self.P, self.S
        i32 = dict(dtype=torch.int32, device=dev)
        self.logits = torch.empty((T_max, self.M), dtype=torch.float32, device=dev)
        self.ids = torch.empty((T_max, k), **i32)
        self.w = torch.empty((T_max, k), dtype=torch.float32, device=dev)
        self.slot = torch.empty((T_max, k), **i32)
        self.counts = torch.empty(P, **i32)
        self.offsets = torch.empty(P + 1, **i32)
        self.por = torch.empty(T_max * k, **i32)
        self.rop = torch.empty(T_max * k, **i32)
        self.y = torch.empty((T_max * k, H), dtype=dtype, device=dev)
        self.out = torch.empty((T_max, H), dtype=dtype, device=dev)
        lib = B.lib()
        dt = B.EW_BF16 if dtype == torch.bfloat16 else B.EW_F32
        self.dt = dt
        self.ws_perm = B._workspace(lib.moe_reroute_permute_workspace_bytes(T_max, k, P), dev)
        self.ws_ffn = B._workspace(lib.moe_grouped_ffn_workspace_bytes(T_max, k, H, I, P, dt), dev)
        if S:
            self.y_sh = torch.empty((S * T_max, H), dtype=dtype, device=dev)
            self.ws_sh = B._workspace(lib.moe_grouped_ffn_workspace_bytes(S * T_max, 1, H, I, S, dt), dev)
            self._sh_T = -1
            self.sh_counts = torch.empty(S, **i32)
            self.sh_offsets = torch.empty(S + 1, **i32)
            self.sh_por = torch.empty(S * T_max, **i32)

    def _shared_index(self, T: int):
        """Row map of the shared experts (structure only): slab s holds tokens 0..T-1 in order."""
        if self._sh_T != T:
            S = self.S
            self.sh_counts.fill_(T)
            self.sh_offsets.copy_(torch.arange(S + 1, dtype=torch.int32) * T)
            self.sh_por[:S * T].copy_(torch.arange(S * T, dtype=torch.int32) % T)
            self._sh_T = T

    def forward(self, x: torch.Tensor, aid: torch.Tensor, logits: torch.Tensor | None = None) -> torch.Tensor:
        lib, st = B.lib(), B._stream()
        T, H, k, P, I = x.shape[0], self.H, self.k, self.P, self.I
        assert T <= self.T_max and x.dtype == self.dtype and x.is_contiguous()
        if logits is None:
            logits = self.logits
            B._check(lib.moe_gate_logits(x.data_ptr(), self.dt, self.Wg.data_ptr(), T, H, self.M,
                                         aid.data_ptr() if self.bias is not None else None,
                                         self.bias.data_ptr() if self.bias is not None else None,
                                         logits.data_ptr(), st))
        B._check(lib.moe_route_reroute_permute(logits.data_ptr(), aid.data_ptr(), self.emap, T, self.M, k, self.N, P,
                                               int(self.renormalize), self.ids.data_ptr(), self.w.data_ptr(),
                                               self.slot.data_ptr(), self.counts.data_ptr(), self.offsets.data_ptr(),
                                               self.por.data_ptr(), self.rop.data_ptr(), B._ptr(self.ws_perm),
                                               self.ws_perm.numel() if self.ws_perm is not None else 0, st))
        B._check(lib.moe_grouped_ffn(x.data_ptr(), self.dt, T, k, H, I, P, self.counts.data_ptr(),
                                     self.offsets.data_ptr(), self.por.data_ptr(), self.w13_base, self.w2_base,
                                     self.y.data_ptr(), self.ws_ffn.data_ptr(), self.ws_ffn.numel(), st))
        sh_ptr = None
        if self.S:
            self._shared_index(T)
            B._check(lib.moe_grouped_ffn(x.data_ptr(), self.dt, self.S * T, 1, H, I, self.S, self.sh_counts.data_ptr(),
                                         self.sh_offsets.data_ptr(), self.sh_por.data_ptr(), self.shared_w13.data_ptr(),
                                         self.shared_w2.data_ptr(), self.y_sh.data_ptr(), self.ws_sh.data_ptr(),
                                         self.ws_sh.numel(), st))
            sh_ptr = self.y_sh.data_ptr()
        B._check(lib.moe_unpermute(self.y.data_ptr(), self.rop.data_ptr(), self.w.data_ptr(), sh_ptr, self.S, T, k, H,
                                   self.dt, self.out.data_ptr(), st))
        return self.out[:T]
