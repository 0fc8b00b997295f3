"""Pins of the CPU oracle against things other than itself: the brute-force twin, closed forms,
invariants, library special cases, and the figures/tables the paper quotes in its text.
All CPU; none of these touches the HIP path."""
import math

import numpy as np
import pytest
import scipy.special
import torch

import workloads as wl
from oracle import brute, moe


def tiny_problem(seed_index=0, H=16, M=8, I=12, S=1, k=2, T=24, N=3, E_max=3, lo=0, hi=3, dtype="f32"):
    cfg = wl.get_config(0).with_(index=100 + seed_index, H=H, M=M, I=I, S=S, k=k, T=T, N=N,
                                 E_max=E_max, tuned_lo=lo, tuned_hi=hi, dtype=dtype, weight_std=0.3)
    tuned = wl.tuned_sets(cfg)
    aid = wl.adapter_ids(cfg)
    x = wl.tokens(cfg)
    Wg = wl.gate_weight(cfg)
    base = wl.stacked_expert_weights(cfg, 0, 0, M, threads=1)
    adapters = [wl.stacked_expert_weights(cfg, 0, a + 1, len(tuned[a]), threads=1) for a in range(N)]
    shared = wl.shared_weights(cfg)
    logits = moe.gate_logits(x, Wg)
    return cfg, tuned, aid, x, logits, base, adapters, shared


# ----------------------------------------------------------------------------- top-k and weights
def test_topk_matches_brute_force_with_ties():
    rng = np.random.default_rng(1)
    # few distinct values -> many ties, plus signed zeros
    logits = rng.integers(-2, 3, size=(50, 10)).astype(np.float32)
    logits[logits == 0] = np.where(rng.random((logits == 0).sum()) < 0.5, 0.0, -0.0)
    for k in (1, 3, 10):
        ids, w = moe.route_topk(logits, k)
        bids, bw = brute.route_topk(logits.tolist(), k)
        assert ids.tolist() == bids
        np.testing.assert_allclose(w, np.array(bw), rtol=1e-13)


def test_topk_closed_forms():
    E, k = 64, 6
    inc = np.arange(E, dtype=np.float32)[None, :]
    assert moe.route_topk(inc, k)[0].tolist() == [[63, 62, 61, 60, 59, 58]]
    eq = np.zeros((1, E), dtype=np.float32)
    ids, w = moe.route_topk(eq, k)
    assert ids.tolist() == [[0, 1, 2, 3, 4, 5]]
    np.testing.assert_allclose(w, 1.0 / E, rtol=1e-15)            # uniform softmax
    # two-way tie for the last place: the lower index wins
    z = np.zeros((1, 8), dtype=np.float32); z[0, [5, 2]] = 3.0; z[0, [6, 1]] = 1.0
    assert moe.route_topk(z, 3)[0].tolist() == [[2, 5, 1]]


def test_softmax_weights_against_library_and_invariants():
    rng = np.random.default_rng(2)
    logits = (rng.standard_normal((40, 64)) * 3).astype(np.float32)
    p = moe.softmax(logits)
    np.testing.assert_allclose(p, scipy.special.softmax(logits.astype(np.float64), axis=-1), rtol=1e-12)
    np.testing.assert_allclose(p.sum(-1), 1.0, rtol=1e-14)
    ids, w = moe.route_topk(logits, 6)
    np.testing.assert_allclose(w, np.take_along_axis(p, ids.astype(np.int64), -1))
    assert np.all(np.diff(w, axis=-1) <= 0)                         # descending score order
    _, wr = moe.route_topk(logits, 6, renormalize=True)
    np.testing.assert_allclose(wr.sum(-1), 1.0, rtol=1e-14)
    np.testing.assert_allclose(wr * w.sum(-1, keepdims=True), w, rtol=1e-14)
    # large logits do not overflow (max subtraction)
    big = np.array([[1e4, 1e4 - 1.0, -1e4]], dtype=np.float32)
    np.testing.assert_allclose(moe.softmax(big)[0, :2], [1 / (1 + math.exp(-1)), 1 / (1 + math.e)], rtol=1e-12)


# ----------------------------------------------------------------------------- expert map / reroute
def test_expert_map_fig4_ranges(golden_fig4):
    g = golden_fig4
    M, N, E_max = g["M"], g["N"], g["E_max"]
    rng = np.random.default_rng(3)
    tuned = [np.sort(rng.choice(M, g["e_0"], replace=False)), np.sort(rng.choice(M, g["e_1"], replace=False))]
    Pi = moe.build_expert_map(M, N, E_max, tuned)
    assert Pi.shape == (N + 1, M)
    assert Pi[0].tolist() == list(range(M))                         # base marker row: identity
    for i, (delta, e) in enumerate([(g["Delta_0"], g["e_0"]), (g["Delta_1"], g["e_1"])]):
        row = Pi[i + 1]
        moved = np.nonzero(row != np.arange(M))[0]
        assert moved.tolist() == tuned[i].tolist()                  # exactly the tuned experts move
        assert row[moved].tolist() == list(range(delta, delta + e)) # Delta_i + rank, 0 <= delta < e_i
        assert delta == M + i * E_max
    # a K = 6 token batch: slots stay in [0,M) U [Delta_i, Delta_i+e_i)
    ids = wl.distinct_topk_ids(wl.get_config(3).with_(T=500, k=g["K"]))
    aid = rng.integers(0, N + 1, 500).astype(np.int32)
    slot = moe.reroute(ids, aid, Pi)
    for t in range(500):
        a = aid[t]
        for j, s in zip(ids[t], slot[t]):
            assert s == brute.reroute_pair(int(a), int(j), M, E_max, tuned)
        assert len(set(slot[t].tolist())) == g["K"]                # injective per token
    assert np.array_equal(slot[aid == 0], ids[aid == 0])            # base-only tokens unchanged


def test_expert_map_rejects_bad_adapters():
    with pytest.raises(ValueError):
        moe.build_expert_map(8, 1, 2, [[1, 2, 3]])                  # more than E_max
    with pytest.raises(ValueError):
        moe.build_expert_map(8, 1, 2, [[1, 1]])                     # duplicates
    with pytest.raises(ValueError):
        moe.build_expert_map(8, 1, 2, [[8]])                        # out of range
    assert np.array_equal(moe.build_expert_map(8, 2, 2, [[], []]), np.tile(np.arange(8), (3, 1)))


# ----------------------------------------------------------------------------- permutation
@pytest.mark.parametrize("T,k,P", [(1, 1, 1), (7, 2, 5), (300, 6, 384), (64, 6, 128)])
def test_permute_invariants_and_brute_force(T, k, P):
    rng = np.random.default_rng(T * 31 + k)
    slot = rng.integers(0, P, size=(T, k)).astype(np.int32)
    counts, offsets, por, rop = moe.permute(slot, P)
    n = T * k
    assert counts.sum() == n and offsets[0] == 0 and offsets[-1] == n
    assert np.array_equal(np.diff(offsets), counts)
    assert sorted(por.tolist()) == list(range(n))                   # bijection
    assert np.array_equal(rop[por], np.arange(n)) and np.array_equal(por[rop], np.arange(n))
    flat = slot.reshape(-1)
    assert np.all(np.diff(flat[por]) >= 0)                          # grouped by slot
    for s in range(P):
        chunk = por[offsets[s]:offsets[s + 1]]
        assert np.all(flat[chunk] == s) and np.all(np.diff(chunk) > 0)   # stable inside a chunk
    bc, bo, bp, br = brute.permute(slot.tolist(), P)
    assert (counts.tolist(), offsets.tolist(), por.tolist(), rop.tolist()) == (bc, bo, bp, br)


def test_permute_empty_and_out_of_range():
    counts, offsets, por, rop = moe.permute(np.zeros((0, 6), np.int32), 12)
    assert counts.tolist() == [0] * 12 and offsets.tolist() == [0] * 13 and len(por) == 0 == len(rop)
    with pytest.raises(ValueError):
        moe.permute(np.array([[12]]), 12)


# ----------------------------------------------------------------------------- expert FFN
def test_expert_ffn_is_a_swiglu_mlp_library_check():
    rng = np.random.default_rng(5)
    H, I, n = 24, 10, 7
    x = rng.standard_normal((n, H)); w13 = rng.standard_normal((2 * I, H)); w2 = rng.standard_normal((H, I))
    y = moe.expert_ffn(x, w13, w2)
    F = torch.nn.functional
    tx, t13, t2 = (torch.from_numpy(a) for a in (x, w13, w2))
    ref = F.linear(F.silu(F.linear(tx, t13[:I])) * F.linear(tx, t13[I:]), t2).numpy()
    np.testing.assert_allclose(y, ref, rtol=1e-12, atol=1e-12)
    # a transposed or swapped operand must not survive: gate and up are not interchangeable
    swapped = np.concatenate([w13[I:], w13[:I]])
    assert not np.allclose(moe.expert_ffn(x, swapped, w2), ref)
    # brute force, one row
    np.testing.assert_allclose(y[0], brute.expert_ffn_row(x[0].tolist(), w13.tolist(), w2.tolist()), rtol=1e-11)
    assert np.all(moe.expert_ffn(x, w13, np.zeros_like(w2)) == 0)
    # silu closed forms
    assert moe.silu(0.0) == 0.0 and math.isclose(moe.silu(1.0), 1 / (1 + math.exp(-1)))
    assert math.isclose(moe.silu(-1.0), -1 / (1 + math.e))


def test_bf16_bits_widen_exactly():
    vals = np.array([1.0, -2.5, 0.02, 3.140625, 1e-3], dtype=np.float32)
    bits = wl.f32_to_bf16_bits(vals)
    back = torch.from_numpy(vals).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(moe.as_f64(bits), back)
    np.testing.assert_array_equal(wl.bf16_bits_to_f32(bits).astype(np.float64), back)


# ----------------------------------------------------------------------------- whole layer
@pytest.mark.parametrize("seed_index,renorm", [(0, False), (1, True)])
def test_layer_matches_brute_force(seed_index, renorm):
    cfg, tuned, aid, x, logits, base, adapters, shared = tiny_problem(seed_index)
    r = moe.moe_layer(x, logits, aid, cfg.k, cfg.M, cfg.N, cfg.E_max, tuned, base, adapters, shared, renorm)
    bids, bw, bslots, bout = brute.moe_layer(x.tolist(), logits.tolist(), aid.tolist(), cfg.k, cfg.M, cfg.N,
                                             cfg.E_max, tuned, base, adapters, shared, renorm)
    assert r["ids"].tolist() == bids and r["slot"].tolist() == bslots
    np.testing.assert_allclose(r["w"], np.array(bw), rtol=1e-12)
    np.testing.assert_allclose(r["out"], np.array(bout), rtol=1e-9, atol=1e-12)
    # y_sorted rows are the per-pair expert outputs in sorted order
    for row in (0, len(r["pair_of_row"]) // 2, len(r["pair_of_row"]) - 1):
        p = int(r["pair_of_row"][row]); t, j = divmod(p, cfg.k)
        s = int(r["slot"][t, j])
        w13, w2 = moe.VirtualWeights(cfg.M, cfg.E_max, base, adapters).slot(s)
        np.testing.assert_allclose(r["y_sorted"][row], brute.expert_ffn_row(x[t].tolist(), w13.tolist(), w2.tolist()),
                                   rtol=1e-9, atol=1e-12)


def test_merge_equivalence_and_base_invariants():
    cfg, tuned, aid, x, logits, base, adapters, shared = tiny_problem(2, T=40, lo=1, hi=3)
    args = (cfg.k, cfg.M, cfg.N, cfg.E_max, tuned, base, adapters, shared)
    r = moe.moe_layer(x, logits, aid, *args)
    merged = moe.merged_model_layer(x, logits, aid, cfg.k, cfg.M, tuned, base, adapters, shared)
    np.testing.assert_allclose(r["out"], merged, rtol=1e-10, atol=1e-13)
    # adapters matter: base-only serving of the same batch differs on tokens whose picks were tuned
    r0 = moe.moe_layer(x, logits, np.zeros_like(aid), *args)
    assert np.array_equal(r0["slot"], r0["ids"]) and r0["slot"].max() < cfg.M
    changed = np.any(r["slot"] != r["ids"], axis=1)
    assert changed.any()
    assert np.allclose(r["out"][~changed], r0["out"][~changed], rtol=1e-12)
    assert not np.allclose(r["out"][changed], r0["out"][changed])
    # an all-base batch equals a plain MoE layer with no adapters at all
    plain = moe.moe_layer(x, logits, np.zeros_like(aid), cfg.k, cfg.M, 0, cfg.E_max, [], base, [], shared)
    np.testing.assert_array_equal(plain["out"], r0["out"])


def test_adapter_with_zero_tuned_experts_equals_base():
    cfg, tuned, aid, x, logits, base, adapters, shared = tiny_problem(3)
    tuned0 = [np.zeros(0, np.int32) for _ in tuned]
    empty = [(a[0][:0], a[1][:0]) for a in adapters]
    r = moe.moe_layer(x, logits, aid, cfg.k, cfg.M, cfg.N, cfg.E_max, tuned0, base, empty, shared)
    r0 = moe.moe_layer(x, logits, np.zeros_like(aid), cfg.k, cfg.M, cfg.N, cfg.E_max, tuned0, base, empty, shared)
    assert np.array_equal(r["slot"], r["ids"])
    np.testing.assert_array_equal(r["out"], r0["out"])
    assert np.array_equal(r["counts"][cfg.M:], np.zeros(cfg.N * cfg.E_max, np.int32))


def test_single_expert_layer_reduces_to_one_mlp_and_output_is_linear_in_w():
    cfg, tuned, aid, x, logits, base, adapters, shared = tiny_problem(4, M=1, k=1, N=0, E_max=1, lo=0, hi=0)
    r = moe.moe_layer(x, logits, aid * 0, 1, 1, 0, 1, [], base, [], None)
    assert np.all(r["w"] == 1.0)
    np.testing.assert_allclose(r["out"], moe.expert_ffn(x, base[0][0], base[1][0]), rtol=1e-14)
    cfg, tuned, aid, x, logits, base, adapters, shared = tiny_problem(5)
    r = moe.moe_layer(x, logits, aid, cfg.k, cfg.M, cfg.N, cfg.E_max, tuned, base, adapters, None)
    np.testing.assert_allclose(moe.unpermute(r["y_sorted"], r["row_of_pair"], 2.0 * r["w"]), 2.0 * r["out"], rtol=1e-14)
    sh = moe.shared_ffn(x, *shared)
    np.testing.assert_allclose(moe.unpermute(r["y_sorted"], r["row_of_pair"], 0.0 * r["w"], sh), sh)


def test_unmapped_padding_slot_is_never_readable():
    cfg, tuned, aid, x, logits, base, adapters, shared = tiny_problem(6, lo=1, hi=2)
    vw = moe.VirtualWeights(cfg.M, cfg.E_max, base, adapters)
    with pytest.raises(IndexError):
        vw.slot(cfg.M + 0 * cfg.E_max + len(tuned[0]))              # first padding slot of adapter 1


# ----------------------------------------------------------------------------- planted mistakes
def test_pins_detect_planted_mistakes(monkeypatch):
    """The brute-force pin must fail when a plausible bug is planted in oracle.moe."""
    cfg, tuned, aid, x, logits, base, adapters, shared = tiny_problem(7, lo=1, hi=3)
    _, _, _, bout = brute.moe_layer(x.tolist(), logits.tolist(), aid.tolist(), cfg.k, cfg.M, cfg.N, cfg.E_max,
                                    tuned, base, adapters, shared)
    bout = np.array(bout)

    def run():
        return moe.moe_layer(x, logits, aid, cfg.k, cfg.M, cfg.N, cfg.E_max, tuned, base, adapters, shared)["out"]

    assert np.allclose(run(), bout, rtol=1e-9)
    with monkeypatch.context() as m:                                # wrong sign in the activation
        m.setattr(moe, "silu", lambda z: z / (1.0 + np.exp(z)))
        assert not np.allclose(run(), bout, rtol=1e-3)
    with monkeypatch.context() as m:                                # Delta_i off by one adapter
        real = moe.build_expert_map
        m.setattr(moe, "build_expert_map", lambda M, N, E, t: real(M, N, E, list(t[1:]) + [t[0]]))
        assert not np.allclose(run(), bout, rtol=1e-3)
    with monkeypatch.context() as m:                                # un-permute through the wrong index
        real_p = moe.permute
        m.setattr(moe, "permute", lambda s, P: (lambda c, o, a, b: (c, o, a, a))(*real_p(s, P)))
        assert not np.allclose(run(), bout, rtol=1e-3)
    with monkeypatch.context() as m:                                # dropped shared experts
        m.setattr(moe, "shared_ffn", lambda x_, a, b: np.zeros_like(moe.as_f64(x_)))
        assert not np.allclose(run(), bout, rtol=1e-3)


def test_rmsnorm_closed_forms():
    """The stacking aid: unit RMS afterwards, invariant to positive scaling, closed form on a constant row."""
    rng = np.random.default_rng(5)
    x = rng.standard_normal((7, 64)) * rng.uniform(0.1, 30.0, size=(7, 1))
    n = moe.rmsnorm(x, eps=0.0)
    np.testing.assert_allclose(np.sqrt((n * n).mean(axis=1)), 1.0, rtol=1e-12)
    np.testing.assert_allclose(moe.rmsnorm(3.5 * x, eps=0.0), n, rtol=1e-12)
    np.testing.assert_allclose(moe.rmsnorm(np.full((1, 16), -2.0), eps=0.0), -1.0, rtol=1e-12)
    np.testing.assert_allclose(moe.rmsnorm(np.full((1, 16), 2.0), eps=12.0), 0.5, rtol=1e-12)   # 2 / sqrt(4 + 12)
    e = np.zeros((1, 9)); e[0, 3] = 5.0
    np.testing.assert_allclose(moe.rmsnorm(e, eps=0.0)[0, 3], 3.0, rtol=1e-12)                  # 5 / sqrt(25 / 9)


# ----------------------------------------------------------------------------- router scores
def test_gate_logits_brute_force_one_hot_and_bias_rows():
    """Router scores g(x) = x . Wg^T (Sec. 2.1) with the per-class bias of the synthetic traffic: explicit dot
    products on a non-square shape (a transposed operand cannot survive), a one-hot token (the score row is a
    column of Wg), and a bias table whose rows all differ (a wrong class row cannot survive)."""
    rng = np.random.default_rng(17)
    T, H, E, N = 9, 5, 7, 3
    x = rng.standard_normal((T, H)).astype(np.float32)
    Wg = rng.standard_normal((E, H)).astype(np.float32)
    aid = np.array([0, 1, 2, 3, 3, 2, 1, 0, 2], dtype=np.int32)
    bias = (10.0 * np.arange(N + 1, dtype=np.float32)[:, None] + np.arange(E, dtype=np.float32)[None, :])   # row a = 10a + e
    z = moe.gate_logits(x, Wg)
    assert z.shape == (T, E) and z.dtype == np.float32
    for t in range(T):
        for e in range(E):
            want = brute.dot(x[t].tolist(), Wg[e].tolist())
            assert z[t, e] == np.float32(want)                       # fp64 sum rounded once to float32
    zb = moe.gate_logits(x, Wg, aid, bias)
    for t in range(T):
        for e in range(E):
            want = brute.dot(x[t].tolist(), Wg[e].tolist()) + 10.0 * int(aid[t]) + e
            assert zb[t, e] == np.float32(want)
    # base-model tokens (row 0 of this table is 0..E-1, not zero: the row is looked up, not skipped)
    np.testing.assert_allclose(zb[aid == 0], z[aid == 0].astype(np.float64) + np.arange(E), rtol=1e-6)
    # one-hot tokens: the scores are the matching column of Wg, scaled
    onehot = np.zeros((H, H), dtype=np.float32)
    onehot[np.arange(H), np.arange(H)] = 2.0
    np.testing.assert_array_equal(moe.gate_logits(onehot, Wg), (2.0 * Wg.T.astype(np.float64)).astype(np.float32))
    # bf16 bit patterns widen exactly before the product
    xb = wl.f32_to_bf16_bits(x)
    np.testing.assert_array_equal(moe.gate_logits(xb, Wg), moe.gate_logits(wl.bf16_bits_to_f32(xb), Wg))
    # planted mistakes: bias row of the wrong class, transposed gate
    wrong = moe.gate_logits(x, Wg, (aid + 1) % (N + 1), bias)
    assert not np.allclose(wrong, zb)
    with pytest.raises(ValueError):
        moe.gate_logits(x, Wg.T.copy())
