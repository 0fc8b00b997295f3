"""ExpertWeave MoE-layer hot path for AMD MI355X: thin Python binding over libexpertweave.so.

The library (csrc/, C ABI in include/expertweave.h) does all the work; see `binding` for the
marshalling layer and `build` for the hipcc build.
"""
from . import binding  # noqa: F401
from .binding import (  # noqa: F401
    ExpertPool, EWError, EW_F32, EW_BF16, EW_POOL_VMM, EW_POOL_PADDED, EW_POOL_FAKE, EW_POOL_EAGER_UNMAP,
    moe_route_topk, moe_reroute_permute, moe_route_reroute_permute, moe_grouped_ffn, moe_unpermute,
    moe_gate_logits, moe_rmsnorm, moe_reroute_singleop, moe_grouped_ffn_with_shared, moe_unpermute_rmsnorm,
    moe_reroute_permute_static, lib,
)
