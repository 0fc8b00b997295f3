"""numpy oracle of one ExpertWeave MoE layer (test infrastructure; see package docstring).

Stages, in the paper's order (Sec. 2.1 and Sec. 4.1/4.3):
  router scores -> top-k -> batched rerouting through the ESFT expert map ->
  dispatch (replicate, permute, group by slot) -> expert FFN per group over the
  virtual weight tensor -> weighted combine and un-permute (+ shared experts).

All floating point is fp64; bf16 inputs (uint16 bit patterns) are widened exactly.
Adapter ids follow the library's convention: 0 = base model, a = 1..N = adapter a,
which is the paper's adapter index i = a-1 (the paper marks base tokens with -1).
"""
from __future__ import annotations

import numpy as np


# ----------------------------------------------------------------------------- helpers
def as_f64(a) -> np.ndarray:
    """Widen float32/float64 arrays, or bf16 bit patterns (uint16), exactly to float64."""
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


# ----------------------------------------------------------------------------- router (Sec. 2.1)
def gate_logits(x, Wg, aid=None, bias=None) -> np.ndarray:
    """Router scores g(x) = x . Wg^T (+ a per-class additive bias of the synthetic traffic),
    computed in fp64 and rounded once to float32: the type both sides take top-k in."""
    z = as_f64(x) @ as_f64(Wg).T
    if bias is not None:
        z = z + as_f64(bias)[np.asarray(aid)]
    return z.astype(np.float32)


def softmax(logits) -> np.ndarray:
    z = as_f64(logits)
    z = z - z.max(axis=-1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=-1, keepdims=True)


def route_topk(logits, k: int, renormalize: bool = False):
    """Top-k experts per token (Sec. 2.1): the k largest float32 logits in descending order,
    equal logits ordered by lower expert index.  Combine weight = softmax probability over all
    experts of each chosen one; optionally divided by their sum."""
    logits = np.asarray(logits, dtype=np.float32)
    ids = np.argsort(-logits, axis=-1, kind="stable")[:, :k].astype(np.int32)
    p = softmax(logits)
    w = np.take_along_axis(p, ids.astype(np.int64), axis=-1)
    if renormalize:
        w = w / w.sum(axis=-1, keepdims=True)
    return ids, w


# ----------------------------------------------------------------------------- expert map (Sec. 4.1)
def build_expert_map(M: int, N: int, E_max: int, tuned) -> np.ndarray:
    """ESFT expert map with a leading identity row for base-model tokens: int32 [N+1, M].

    Row a (adapter a, the paper's i = a-1):  Pi[i, j] = j if adapter i does not tune expert j,
    else Delta_i + delta_ij with Delta_i = M + i*E_max and delta_ij the rank of j among the
    adapter's tuned experts taken in ascending order (0 <= delta < e_i).
    `tuned[i]` lists adapter i's tuned experts; missing/empty = tunes nothing."""
    Pi = np.tile(np.arange(M, dtype=np.int32), (N + 1, 1))
    for i in range(N):
        J = np.sort(np.asarray(tuned[i], dtype=np.int64)) if i < len(tuned) else np.zeros(0, np.int64)
        if len(J) > E_max:
            raise ValueError("adapter tunes more experts than E_max")
        if len(np.unique(J)) != len(J) or (len(J) and (J[0] < 0 or J[-1] >= M)):
            raise ValueError("tuned experts must be distinct ids in [0, M)")
        delta_base = M + i * E_max
        for d, j in enumerate(J):
            Pi[i + 1, j] = delta_base + d
    return Pi


def reroute(ids, aid, expert_map) -> np.ndarray:
    """Batched rerouting (Sec. 4.1, 4.3): TopK'(x) = { Pi[A(x), j] : j in TopK(x) }, per token."""
    ids = np.asarray(ids)
    aid = np.asarray(aid)
    return np.asarray(expert_map)[aid[:, None], ids].astype(np.int32)


# ----------------------------------------------------------------------------- dispatch (Sec. 2.1)
def permute(slot, P: int):
    """Group the T*k (token, choice) pairs by slot: tokens of one slot form one contiguous chunk.

    Pair index p = t*k + j.  Within a chunk pairs keep ascending p (stable), which makes the
    permutation unique.  Returns counts [P], exclusive offsets [P+1], pair_of_row (sorted row ->
    pair) and row_of_pair (its inverse), all int32."""
    flat = np.asarray(slot).reshape(-1).astype(np.int64)
    counts = np.bincount(flat, minlength=P).astype(np.int32)
    if len(counts) != P:
        raise ValueError("slot id outside [0, P)")
    offsets = np.zeros(P + 1, dtype=np.int32)
    offsets[1:] = np.cumsum(counts)
    pair_of_row = np.argsort(flat, kind="stable").astype(np.int32)
    row_of_pair = np.empty_like(pair_of_row)
    row_of_pair[pair_of_row] = np.arange(len(flat), dtype=np.int32)
    return counts, offsets, pair_of_row, row_of_pair


# ----------------------------------------------------------------------------- virtual weight tensor
class VirtualWeights:
    """The unified expert pool of one layer seen as the paper's virtual weight tensor
    [M + N*E_max, H_out, H_in] (Sec. 4.1): slots [0, M) are the base experts, slots
    [Delta_i, Delta_i + e_i) adapter i's tuned experts in ascending order of the expert they
    replace; the padding up to Delta_i + E_max has no backing and must never be read.

    base = (w13 [M, 2I, H], w2 [M, H, I]); adapters[i] = (w13 [e_i, 2I, H], w2 [e_i, H, I]).
    w13 holds the gate projection in rows [0, I) and the up projection in rows [I, 2I)."""

    def __init__(self, M: int, E_max: int, base, adapters):
        self.M, self.E_max, self.base, self.adapters = M, E_max, base, list(adapters)

    def slot(self, s: int):
        if s < self.M:
            return as_f64(self.base[0][s]), as_f64(self.base[1][s])
        i, d = divmod(s - self.M, self.E_max)
        if i >= len(self.adapters) or d >= len(self.adapters[i][0]):
            raise IndexError(f"slot {s} is unmapped padding of the virtual weight tensor")
        return as_f64(self.adapters[i][0][d]), as_f64(self.adapters[i][1][d])


# ----------------------------------------------------------------------------- expert FFN
def silu(z):
    return z / (1.0 + np.exp(-z))


def expert_ffn(x, w13, w2) -> np.ndarray:
    """SwiGLU expert on rows x [n, H]:  (silu(x.Wg^T) * (x.Wu^T)) . W2^T, with Wg = w13[:I], Wu = w13[I:]."""
    x, w13, w2 = as_f64(x), as_f64(w13), as_f64(w2)
    I = w13.shape[0] // 2
    g = x @ w13[:I].T
    u = x @ w13[I:].T
    return (silu(g) * u) @ w2.T


def grouped_ffn(x, k: int, counts, offsets, pair_of_row, weights: VirtualWeights) -> np.ndarray:
    """Grouped expert computation over the permuted tokens (Sec. 2.1): sorted row r of slot s is
    token pair_of_row[r] // k run through slot s's expert.  Returns y_sorted [T*k, H], fp64."""
    x = as_f64(x)
    y = np.zeros((len(pair_of_row), x.shape[1]), dtype=np.float64)
    for s in np.nonzero(np.asarray(counts))[0]:
        lo, hi = int(offsets[s]), int(offsets[s + 1])
        w13, w2 = weights.slot(int(s))
        y[lo:hi] = expert_ffn(x[np.asarray(pair_of_row[lo:hi]) // k], w13, w2)
    return y


def shared_ffn(x, sh_w13, sh_w2) -> np.ndarray:
    """Shared experts: every token through each of the S shared SwiGLU experts, summed, weight 1."""
    x = as_f64(x)
    out = np.zeros_like(x)
    for s in range(len(sh_w13)):
        out += expert_ffn(x, sh_w13[s], sh_w2[s])
    return out


def unpermute(y_sorted, row_of_pair, w, shared_out=None) -> np.ndarray:
    """Combine (Sec. 2.1): out[t] = shared[t] + sum_j w[t, j] * y_sorted[row_of_pair[t*k + j]]."""
    w = as_f64(w)
    T, k = w.shape
    y = as_f64(y_sorted)[np.asarray(row_of_pair).reshape(T, k)]        # [T, k, H]
    out = np.einsum("tk,tkh->th", w, y)
    if shared_out is not None:
        out = out + as_f64(shared_out)
    return out


# ----------------------------------------------------------------------------- whole layer
def moe_layer(x, logits, aid, k: int, M: int, N: int, E_max: int, tuned, base, adapters,
              shared=None, renormalize: bool = False) -> dict:
    """One adapter-aware MoE layer forward; returns every intermediate."""
    P = M + N * E_max
    ids, w = route_topk(logits, k, renormalize)
    expert_map = build_expert_map(M, N, E_max, tuned)
    slot = reroute(ids, aid, expert_map)
    counts, offsets, pair_of_row, row_of_pair = permute(slot, P)
    vw = VirtualWeights(M, E_max, base, adapters)
    y_sorted = grouped_ffn(x, k, counts, offsets, pair_of_row, vw)
    sh = shared_ffn(x, *shared) if shared is not None and len(shared[0]) else None
    out = unpermute(y_sorted, row_of_pair, w, sh)
    return dict(ids=ids, w=w, expert_map=expert_map, slot=slot, counts=counts, offsets=offsets,
                pair_of_row=pair_of_row, row_of_pair=row_of_pair, y_sorted=y_sorted,
                shared_out=sh, out=out)


def merged_model_layer(x, logits, aid, k: int, M: int, tuned, base, adapters, shared=None,
                       renormalize: bool = False) -> np.ndarray:
    """Independent cross-check (the paper's accuracy claim, Sec. 5 Table 3: shared serving equals
    each adapter's merged model).  For each class build the merged expert list (base experts with
    the adapter's tuned ones swapped in) and run its tokens through a plain MoE layer, token by
    token: no expert map, no slots, no permutation."""
    x = as_f64(x)
    ids, w = route_topk(logits, k, renormalize)
    out = np.zeros_like(x)
    for a in np.unique(aid):
        merged = [(base[0][e], base[1][e]) for e in range(M)]
        if a > 0:
            J = np.sort(np.asarray(tuned[a - 1]))
            for d, e in enumerate(J):
                merged[int(e)] = (adapters[a - 1][0][d], adapters[a - 1][1][d])
        for t in np.nonzero(np.asarray(aid) == a)[0]:
            acc = np.zeros(x.shape[1])
            for j in range(k):
                w13, w2 = merged[int(ids[t, j])]
                acc += w[t, j] * expert_ffn(x[t:t + 1], w13, w2)[0]
            out[t] = acc
    if shared is not None and len(shared[0]):
        out += shared_ffn(x, *shared)
    return out


# ----------------------------------------------------------------------------- stacking aid
def rmsnorm(x, eps: float = 1e-6) -> np.ndarray:
    """Unit-gain RMS normalisation x / sqrt(mean(x^2) + eps), fp64.  Not part of the paper's method
    (Sec. 4.1 leaves the layers around the experts unchanged): it only keeps a chain of
    random-initialised MoE layers, h' = h + MoE(norm(h)), at a bounded scale."""
    x = as_f64(x)
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)
