"""Seeded draws for the workload configurations.

Every piece of data is drawn from its own numpy PCG64 stream keyed by
(config seed, stream tag, layer, class, index), so a single expert's weights or
a single layer's tuned sets can be regenerated alone, in any order, on any
machine.  bf16 data is carried as uint16 bit patterns (numpy has no bf16):
the oracle widens them exactly to float, the HIP path views them as bf16.

Nothing here is arithmetic of the method: no routing, no remap table, no FFN.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
import os

import numpy as np

from .configs import MoEConfig

# stream tags
_TUNED, _AID, _TOKENS, _GATE, _EXPERT, _SHARED, _IDS = range(7)


def _rng(cfg: MoEConfig, tag: int, *key: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([cfg.seed, tag, *key])))


# ----------------------------------------------------------------------------- dtype packing
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _pack(cfg: MoEConfig, a: np.ndarray) -> np.ndarray:
    return f32_to_bf16_bits(a) if cfg.dtype == "bf16" else a.astype(np.float32, copy=False)


# ----------------------------------------------------------------------------- structure
def tuned_sets(cfg: MoEConfig, layer: int = 0) -> list[np.ndarray]:
    """For each adapter 1..N: ascending int32 ids of the base experts it fine-tunes in `layer`.

    The count is uniform in [tuned_lo, tuned_hi]; the ids are a uniform draw without replacement
    (per-layer variation of the count mirrors paper Sec. 3.1 / Table 1).
    """
    out = []
    for a in range(1, cfg.N + 1):
        g = _rng(cfg, _TUNED, layer, a)
        e = int(g.integers(cfg.tuned_lo, cfg.tuned_hi + 1))
        out.append(np.sort(g.choice(cfg.M, size=e, replace=False)).astype(np.int32))
    return out


def class_probabilities(cfg: MoEConfig) -> np.ndarray:
    c = np.arange(cfg.N + 1, dtype=np.float64)
    p = np.ones_like(c) if cfg.aid_dist == "uniform" else (c + 1.0) ** (-cfg.zipf_s)
    return p / p.sum()


def adapter_ids(cfg: MoEConfig, T: int | None = None) -> np.ndarray:
    """Per-token adapter id, int32 [T]; 0 = base model, 1..N = adapters."""
    T = cfg.T if T is None else T
    g = _rng(cfg, _AID)
    return g.choice(cfg.N + 1, size=T, p=class_probabilities(cfg)).astype(np.int32)


def adapter_ids_powerlaw(cfg: MoEConfig, T: int, n_adapters: int, alpha: float) -> np.ndarray:
    """Per-token adapter id in 1..n_adapters (no base-model requests), int32 [T], with skewed popularity
    as in the paper's end-to-end workloads (Sec. 5.1): a share variable x in (0, 1] is drawn from the
    power distribution with shape alpha (density alpha * x^(alpha-1); alpha = 1 is uniform, smaller
    alpha puts most requests on the first few adapters) and the request goes to adapter 1 + floor(n x)."""
    assert 1 <= n_adapters <= cfg.N and alpha > 0
    g = _rng(cfg, _AID, 7, n_adapters, int(round(alpha * 1000)))
    x = g.power(alpha, size=T)
    return (1 + np.minimum((x * n_adapters).astype(np.int64), n_adapters - 1)).astype(np.int32)


def tokens(cfg: MoEConfig, T: int | None = None) -> np.ndarray:
    """Hidden states [T, H] ~ N(0,1): float32, or bf16 bit patterns for bf16 configs."""
    T = cfg.T if T is None else T
    g = _rng(cfg, _TOKENS)
    return _pack(cfg, g.standard_normal((T, cfg.H), dtype=np.float32))


def gate_weight(cfg: MoEConfig, layer: int = 0) -> np.ndarray:
    """Router weight [M, H], float32 ~ N(0, weight_std)."""
    g = _rng(cfg, _GATE, layer)
    return (g.standard_normal((cfg.M, cfg.H), dtype=np.float32) * np.float32(cfg.weight_std))


def _one_expert(cfg: MoEConfig, tag: int, layer: int, cls: int, idx: int, I: int):
    g = _rng(cfg, tag, layer, cls, idx)
    s = np.float32(cfg.weight_std)
    w13 = g.standard_normal((2 * I, cfg.H), dtype=np.float32) * s   # gate rows [0,I), up rows [I,2I)
    w2 = g.standard_normal((cfg.H, I), dtype=np.float32) * s
    return _pack(cfg, w13), _pack(cfg, w2)


def expert_weights(cfg: MoEConfig, layer: int, cls: int, idx: int):
    """One routed expert's (w13 [2I,H], w2 [H,I]).

    cls = 0: base expert `idx` (0..M-1).  cls = a >= 1: the idx-th tuned expert (rank in the
    ascending tuned list) of adapter a.
    """
    return _one_expert(cfg, _EXPERT, layer, cls, idx, cfg.I)


def stacked_expert_weights(cfg: MoEConfig, layer: int, cls: int, n: int, threads: int | None = None):
    """n experts of one class stacked: (w13 [n,2I,H], w2 [n,H,I]); drawn in parallel threads."""
    el = np.uint16 if cfg.dtype == "bf16" else np.float32
    w13 = np.empty((n, 2 * cfg.I, cfg.H), dtype=el)
    w2 = np.empty((n, cfg.H, cfg.I), dtype=el)

    def job(i):
        w13[i], w2[i] = expert_weights(cfg, layer, cls, i)

    threads = threads or min(16, len(os.sched_getaffinity(0)))
    if n:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(job, range(n)))
    return w13, w2


def shared_weights(cfg: MoEConfig, layer: int = 0):
    """Shared experts: (w13 [S,2I,H], w2 [S,H,I]); never remapped, never tuned."""
    el = np.uint16 if cfg.dtype == "bf16" else np.float32
    w13 = np.empty((cfg.S, 2 * cfg.I, cfg.H), dtype=el)
    w2 = np.empty((cfg.S, cfg.H, cfg.I), dtype=el)
    for s in range(cfg.S):
        w13[s], w2[s] = _one_expert(cfg, _SHARED, layer, 0, s, cfg.I)
    return w13, w2


def logit_bias_table(cfg: MoEConfig, tuned: list[np.ndarray]) -> np.ndarray:
    """float32 [N+1, M]: gate_bias at (a, e) where adapter a tunes expert e, else 0.

    A property of the synthetic traffic (tokens of a domain prefer the experts their adapter
    tuned), not of the method: the router itself is shared by all classes (paper Sec. 2.2).
    """
    b = np.zeros((cfg.N + 1, cfg.M), dtype=np.float32)
    for a, J in enumerate(tuned, start=1):
        b[a, J] = np.float32(cfg.gate_bias)
    return b


def distinct_topk_ids(cfg: MoEConfig, T: int | None = None) -> np.ndarray:
    """int32 [T, k]: k distinct expert ids per token, uniform over [0, M) (integer microbench)."""
    T = cfg.T if T is None else T
    g = _rng(cfg, _IDS)
    # the first k entries of a uniformly random ordering of 0..M-1, via random sort keys
    keys = g.random((T, cfg.M), dtype=np.float32)
    return np.argpartition(keys, cfg.k, axis=1)[:, :cfg.k].astype(np.int32)
