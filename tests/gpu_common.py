"""Shared plumbing of the GPU parity tests: synthetic inputs -> torch tensors, error metrics."""
import numpy as np
import torch

import workloads as wl


def to_torch(a: np.ndarray, device="cuda") -> torch.Tensor:
    """numpy array from the workload generators -> tensor; uint16 means bf16 bit patterns."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).to(device)
    return torch.from_numpy(a).to(device)


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu", torch.float64).numpy()


def rel_l2(got: np.ndarray, ref: np.ndarray) -> float:
    d = np.linalg.norm((got - ref).ravel())
    n = np.linalg.norm(ref.ravel())
    return float(d / n) if n > 0 else float(d)


def max_abs(got: np.ndarray, ref: np.ndarray) -> float:
    return float(np.max(np.abs(got - ref))) if got.size else 0.0


# tolerances stated by the benchmark spec for bf16 FFN outputs vs the fp64 oracle
FFN_REL_L2 = 1e-2
FFN_MAX_ABS = 2e-2


def layer_inputs(cfg, layer=0, T=None):
    """Everything one layer needs, as numpy (generator output)."""
    tuned = wl.tuned_sets(cfg, layer)
    aid = wl.adapter_ids(cfg, T)
    x = wl.tokens(cfg, T)
    Wg = wl.gate_weight(cfg, layer)
    base = wl.stacked_expert_weights(cfg, layer, 0, cfg.M)
    adapters = [wl.stacked_expert_weights(cfg, layer, a + 1, len(tuned[a])) for a in range(cfg.N)]
    shared = wl.shared_weights(cfg, layer) if cfg.S else None
    bias = wl.logit_bias_table(cfg, tuned) if cfg.gate_bias else None
    return dict(tuned=tuned, aid=aid, x=x, Wg=Wg, base=base, adapters=adapters, shared=shared, bias=bias)
