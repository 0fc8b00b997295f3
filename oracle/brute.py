"""Brute-force twin of oracle.moe for tiny inputs (test infrastructure).

Pure-Python loops over tokens, experts and features; Python floats (fp64); no sorting
routines, no vectorised library calls.  It exists to pin oracle.moe: the two are written
differently on purpose (selection by repeated scan instead of argsort, bucket lists instead
of a stable sort, explicit dot products instead of matmul, and the rerouting rule applied
from the tuned lists directly instead of through a precomputed table).
"""
from __future__ import annotations

import math


def topk_row(row, k):
    """k rounds of: scan left to right, keep the first strictly-largest not yet taken."""
    taken, ids = set(), []
    for _ in range(k):
        best = None
        for e, v in enumerate(row):
            if e in taken:
                continue
            if best is None or v > row[best]:
                best = e
        taken.add(best)
        ids.append(best)
    return ids


def softmax_row(row):
    m = max(row)
    ex = [math.exp(float(v) - float(m)) for v in row]
    s = math.fsum(ex)
    return [v / s for v in ex]


def route_topk(logits, k, renormalize=False):
    ids, w = [], []
    for row in logits:
        row = [float(v) for v in row]
        sel = topk_row(row, k)
        p = softmax_row(row)
        ww = [p[e] for e in sel]
        if renormalize:
            s = math.fsum(ww)
            ww = [v / s for v in ww]
        ids.append(sel)
        w.append(ww)
    return ids, w


def reroute_pair(a, j, M, E_max, tuned):
    """Slot of base expert j for a token of class a (0 = base), straight from the rule of
    Sec. 4.1: untouched unless adapter a tunes j, else Delta + rank of j in its tuned list."""
    if a == 0:
        return j
    J = sorted(int(e) for e in tuned[a - 1])
    if j not in J:
        return j
    return M + (a - 1) * E_max + J.index(j)


def permute(slots, P):
    """slots: list of T lists of k slot ids.  Buckets filled in pair order."""
    buckets = [[] for _ in range(P)]
    p = 0
    for row in slots:
        for s in row:
            buckets[s].append(p)
            p += 1
    counts = [len(b) for b in buckets]
    offsets = [0]
    for c in counts:
        offsets.append(offsets[-1] + c)
    pair_of_row = [q for b in buckets for q in b]
    row_of_pair = [0] * p
    for r, q in enumerate(pair_of_row):
        row_of_pair[q] = r
    return counts, offsets, pair_of_row, row_of_pair


def dot(a, b):
    return math.fsum(float(p) * float(q) for p, q in zip(a, b))


def expert_ffn_row(x, w13, w2):
    """x: H floats; w13: 2I rows of H (gate rows then up rows); w2: H rows of I."""
    I = len(w13) // 2
    act = []
    for i in range(I):
        g = dot(x, w13[i])
        u = dot(x, w13[I + i])
        act.append(g / (1.0 + math.exp(-g)) * u)
    return [dot(act, w2[h]) for h in range(len(w2))]


def moe_layer(x, logits, aid, k, M, N, E_max, tuned, base, adapters, shared=None, renormalize=False):
    """Token by token: pick experts, swap in the adapter's version of each picked expert if it
    tunes it, run, weight, add.  `base`/`adapters`/`shared` are nested lists (or arrays) of
    per-expert (w13, w2) stacked as in oracle.moe.  Returns (ids, w, slots, out)."""
    ids, w = route_topk(logits, k, renormalize)
    T, H = len(x), len(x[0])
    slots, out = [], []
    for t in range(T):
        a = int(aid[t])
        row = [reroute_pair(a, j, M, E_max, tuned) for j in ids[t]]
        slots.append(row)
        acc = [0.0] * H
        for jj, j in enumerate(ids[t]):
            if a > 0 and j in [int(e) for e in tuned[a - 1]]:
                d = sorted(int(e) for e in tuned[a - 1]).index(j)
                w13, w2 = adapters[a - 1][0][d], adapters[a - 1][1][d]
            else:
                w13, w2 = base[0][j], base[1][j]
            y = expert_ffn_row(x[t], w13, w2)
            for h in range(H):
                acc[h] += w[t][jj] * y[h]
        if shared is not None:
            for s in range(len(shared[0])):
                y = expert_ffn_row(x[t], shared[0][s], shared[1][s])
                for h in range(H):
                    acc[h] += y[h]
        out.append(acc)
    return ids, w, slots, out
