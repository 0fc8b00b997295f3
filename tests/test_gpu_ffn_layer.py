"""GPU parity: grouped SwiGLU FFN, un-permute, gate logits and the whole layer, against the fp64
oracle.  bf16 tolerance (stated by the benchmark spec): relative L2 <= 1e-2 and max-abs <= 2e-2."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import moe
from gpu_common import FFN_MAX_ABS, FFN_REL_L2, layer_inputs, max_abs, rel_l2, to_f64, to_torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ew():
    import paper_2508_17624_amd as m
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    m.lib()
    return m


def _dense_pool(cfg, inp, poison=True):
    """The virtual weight tensors as plain device tensors [P, ...]; slots that hold no expert are
    filled with NaN so that any read of them shows up in the output."""
    dt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    fill = float("nan") if poison else 0.0
    w13 = torch.full((cfg.P, 2 * cfg.I, cfg.H), fill, dtype=dt, device="cuda")
    w2 = torch.full((cfg.P, cfg.H, cfg.I), fill, dtype=dt, device="cuda")
    w13[:cfg.M] = to_torch(inp["base"][0]); w2[:cfg.M] = to_torch(inp["base"][1])
    for a, (a13, a2) in enumerate(inp["adapters"]):
        s0 = cfg.M + a * cfg.E_max
        if len(a13):
            w13[s0:s0 + len(a13)] = to_torch(a13); w2[s0:s0 + len(a2)] = to_torch(a2)
    return w13, w2


def _oracle_layer(cfg, inp, logits, aid=None):
    return moe.moe_layer(inp["x"], logits, inp["aid"] if aid is None else aid, cfg.k, cfg.M, cfg.N, cfg.E_max,
                         inp["tuned"], inp["base"], inp["adapters"], inp["shared"])


SMALL_BF16 = wl.get_config(1).with_(index=51, H=256, I=128, T=96, M=8, N=3, E_max=4, k=3, S=2, tuned_lo=0, tuned_hi=4,
                                    weight_std=0.04)   # keeps outputs O(0.5), like the full-size layer


@pytest.fixture
def ffn_path(ew, request):
    """Forces one of the bf16 kernels (1 = register streaming, 2 = tiled GEMM, 3 = LDS-direct streaming), then restores automatic."""
    ew.binding.tune_ffn(path=request.param)
    yield request.param
    ew.binding.tune_ffn()


@pytest.mark.parametrize("ffn_path", [1, 2, 3], indirect=True, ids=["stream", "gemm", "ws"])
@pytest.mark.parametrize("cfg", [SMALL_BF16, SMALL_BF16.with_(index=52, T=5, k=2), SMALL_BF16.with_(index=53, T=700, H=384, I=256)],
                         ids=["t96", "t5", "t700"])
def test_grouped_ffn_bf16_small(ew, cfg, ffn_path):
    """Several slots, empty slots, slots with more rows than one tile (t700), NaN padding; both kernels."""
    inp = layer_inputs(cfg)
    logits = moe.gate_logits(inp["x"], inp["Wg"])
    ref = _oracle_layer(cfg, inp, logits)
    w13, w2 = _dense_pool(cfg, inp)
    x = to_torch(inp["x"])
    dev = lambda a: torch.from_numpy(a).cuda()
    y = ew.moe_grouped_ffn(x, cfg.k, cfg.I, cfg.P, dev(ref["counts"]), dev(ref["offsets"]), dev(ref["pair_of_row"]), w13, w2)
    got = to_f64(y)
    assert np.isfinite(got).all(), "a slot without an expert was read"
    assert rel_l2(got, ref["y_sorted"]) <= FFN_REL_L2 and max_abs(got, ref["y_sorted"]) <= FFN_MAX_ABS
    # per-row check so one bad row cannot hide in the norm
    rows = np.linalg.norm(got - ref["y_sorted"], axis=1) / (np.linalg.norm(ref["y_sorted"], axis=1) + 1e-6)
    assert rows.max() <= 3e-2
    # un-permute with shared experts
    sh13, sh2 = to_torch(inp["shared"][0]), to_torch(inp["shared"][1])
    T, S = cfg.T, cfg.S
    shc = torch.full((S,), T, dtype=torch.int32, device="cuda")
    sho = (torch.arange(S + 1, dtype=torch.int32) * T).cuda()
    shp = (torch.arange(S * T, dtype=torch.int32) % T).cuda()
    ysh = ew.moe_grouped_ffn(x, 1, cfg.I, S, shc, sho, shp, sh13, sh2, num_rows=S * T)
    ref_sh = np.stack([moe.expert_ffn(inp["x"], inp["shared"][0][s], inp["shared"][1][s]) for s in range(S)])
    assert rel_l2(to_f64(ysh).reshape(S, T, -1), ref_sh) <= FFN_REL_L2
    out = ew.moe_unpermute(y, dev(ref["row_of_pair"]), dev(ref["w"].astype(np.float32)), ysh)
    assert rel_l2(to_f64(out), ref["out"]) <= FFN_REL_L2 and max_abs(to_f64(out), ref["out"]) <= FFN_MAX_ABS


@pytest.mark.parametrize("nf", [0, 8, 4, 1], ids=["auto", "nf8", "nf4", "nf1"])
def test_grouped_ffn_work_plan_edges(ew, nf):
    """The device-built work plan at its limits: 2048 slots, hundreds of them active (more than 64 entries per
    list), counts on every chunking boundary (1, 31..33, 255..257, 511..513, 700 rows), slots of more than eight
    chunks, which the plan cuts into several entries (2049, 2100, 4100 rows), first and last slot in use, every
    kernel shape.  Rows come straight from x (k = 1, shuffled row map)."""
    rng = np.random.default_rng(77)
    P, H, I = 2048, 128, 128
    counts = np.zeros(P, np.int32)
    special = [1, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257, 511, 512, 513, 700, 2049, 2100, 4100]
    slots = rng.choice(np.arange(1, P - 1), size=len(special) + 560, replace=False)
    counts[slots[:len(special)]] = special
    counts[slots[len(special):]] = rng.integers(1, 24, size=560)
    counts[0], counts[P - 1] = 5, 40
    offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    rows = int(offsets[-1])
    por = rng.permutation(rows).astype(np.int32)
    x = torch.from_numpy(rng.standard_normal((rows, H), dtype=np.float32)).cuda().bfloat16()
    w13 = (torch.from_numpy(rng.standard_normal((P, 2 * I, H), dtype=np.float32)) * 0.08).cuda().bfloat16()
    w2 = (torch.from_numpy(rng.standard_normal((P, H, I), dtype=np.float32)) * 0.08).cuda().bfloat16()
    dev = lambda a: torch.from_numpy(a).cuda()
    ew.binding.tune_ffn(path=3 if nf else 0, ws_frags=nf)
    try:
        y = ew.moe_grouped_ffn(x, 1, I, P, dev(counts), dev(offsets), dev(por), w13, w2, num_rows=rows)
        torch.cuda.synchronize()
    finally:
        ew.binding.tune_ffn()
    got, xs = to_f64(y), to_f64(x)
    check = list(slots[:len(special)]) + [0, P - 1] + list(rng.choice(slots[len(special):], 40, replace=False))
    for s in check:
        r0, r1 = offsets[s], offsets[s + 1]
        ref = moe.expert_ffn(xs[por[r0:r1]], to_f64(w13[s]), to_f64(w2[s]))
        assert rel_l2(got[r0:r1], ref) <= FFN_REL_L2 and max_abs(got[r0:r1], ref) <= FFN_MAX_ABS, f"slot {s} ({counts[s]} rows)"
    assert np.isfinite(got).all()


@pytest.mark.gpu
@pytest.mark.parametrize("T,k,P,S,nf", [(37, 2, 24, 3, 2), (300, 4, 40, 2, 4), (300, 4, 40, 2, 8), (64, 6, 96, 1, 2), (1100, 2, 6, 2, 8),
                                        (300, 4, 40, 2, 0)],
                         ids=["ragged37", "t300-nf4", "t300-nf8", "decode64", "few-slots", "t300-auto"])
def test_grouped_ffn_with_shared(ew, T, k, P, S, nf):
    """Routed + shared experts in one launch: every row against the oracle's expert FFN, and -- when all calls are made
    with one kernel shape (nf > 0; the shapes walk the contraction in different orders) -- bit for bit against two plain
    moe_grouped_ffn calls (the same kernels on the same rows)."""
    rng = np.random.default_rng(100 + T)
    H, I = 256, 128
    ids = np.stack([rng.choice(P, k, replace=False) for _ in range(T)]).astype(np.int32)
    ids[:, 0] = np.where(rng.random(T) < 0.5, 3, ids[:, 0])               # one crowded slot; a repeat inside a token is fine here
    flat = ids.reshape(-1)
    por = np.argsort(flat, kind="stable").astype(np.int32)
    counts = np.bincount(flat, minlength=P).astype(np.int32)
    offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    dev = lambda a: torch.from_numpy(a).cuda()
    bf = lambda *shape, scale=1.0: (torch.from_numpy(rng.standard_normal(shape, dtype=np.float32)) * scale).cuda().bfloat16()
    x, w13, w2, s13, s2 = bf(T, H), bf(P, 2 * I, H, scale=0.05), bf(P, H, I, scale=0.05), bf(S, 2 * I, H, scale=0.05), bf(S, H, I, scale=0.05)
    ew.binding.tune_ffn(path=3 if nf else 0, ws_frags=nf)
    try:
        y = ew.binding.moe_grouped_ffn_with_shared(x, k, I, P, dev(counts), dev(offsets), dev(por), w13, w2, s13, s2)
        y_routed = ew.moe_grouped_ffn(x, k, I, P, dev(counts), dev(offsets), dev(por), w13, w2)
        sh_counts = np.full(S, T, np.int32)
        sh_offsets = (np.arange(S + 1) * T).astype(np.int32)
        sh_por = (np.arange(S * T) % T).astype(np.int32)
        y_shared = ew.moe_grouped_ffn(x, 1, I, S, dev(sh_counts), dev(sh_offsets), dev(sh_por), s13, s2, num_rows=S * T)
        torch.cuda.synchronize()
    finally:
        ew.binding.tune_ffn()
    assert y.shape == (T * (k + S), H)
    if nf:
        assert torch.equal(y[:T * k], y_routed) and torch.equal(y[T * k:], y_shared)
    got, xs = to_f64(y), to_f64(x)
    for s in range(P):
        r0, r1 = offsets[s], offsets[s + 1]
        if r1 > r0:
            ref = moe.expert_ffn(xs[por[r0:r1] // k], to_f64(w13[s]), to_f64(w2[s]))
            assert rel_l2(got[r0:r1], ref) <= FFN_REL_L2 and max_abs(got[r0:r1], ref) <= FFN_MAX_ABS, f"slot {s}"
    for s in range(S):
        ref = moe.expert_ffn(xs, to_f64(s13[s]), to_f64(s2[s]))
        blk = got[T * k + s * T:T * k + (s + 1) * T]
        assert rel_l2(blk, ref) <= FFN_REL_L2 and max_abs(blk, ref) <= FFN_MAX_ABS, f"shared expert {s}"
    # limits: fp32 and S = 0 are refused
    with pytest.raises(ew.EWError):
        ew.binding.moe_grouped_ffn_with_shared(x.float(), k, I, P, dev(counts), dev(offsets), dev(por), w13.float(), w2.float(),
                                               s13.float(), s2.float())
    with pytest.raises(ew.EWError):
        ew.binding.moe_grouped_ffn_with_shared(x, k, I, P, dev(counts), dev(offsets), dev(por), w13, w2, s13[:0], s2[:0])


@pytest.mark.parametrize("T,k,E,N,S", [(64, 6, 64, 4, 2), (300, 4, 32, 2, 1), (40, 2, 192, 15, 0), (3000, 2, 16, 3, 2)],
                         ids=["decode64", "one-block-300", "plan-launch-P1632", "multi-block-3000"])
def test_permutation_call_can_write_the_ffn_plan(ew, T, k, E, N, S):
    """moe_route_reroute_permute_plan + moe_grouped_ffn_planned against the plain pair of calls: same permutation, same
    FFN output bit for bit (the plan is the same plan, whoever writes it)."""
    B = ew.binding
    rng = np.random.default_rng(T + E)
    H, I, E_max = 256, 128, 8 if E < 100 else 96
    P = E + N * E_max
    dev = lambda a: torch.from_numpy(a).cuda()
    logits = dev(rng.standard_normal((T, E), dtype=np.float32))
    aid_np = rng.integers(0, N + 1, T).astype(np.int32)
    tuned = [np.sort(rng.choice(E, E_max, replace=False)) for _ in range(N)]
    emap = dev(moe.build_expert_map(E, N, E_max, tuned).astype(np.int32))
    aid = dev(aid_np)
    bf = lambda *shape: (torch.from_numpy(rng.standard_normal(shape, dtype=np.float32)) * 0.05).cuda().bfloat16()
    x, w13, w2 = bf(T, H) * 20, bf(P, 2 * I, H), bf(P, H, I)
    s13, s2 = (bf(S, 2 * I, H), bf(S, H, I)) if S else (None, None)
    lib, st, i32 = B.lib(), B._stream(), dict(dtype=torch.int32, device="cuda")
    dt = B.EW_BF16

    def run(planned):
        ids, w = torch.empty((T, k), **i32), torch.empty((T, k), dtype=torch.float32, device="cuda")
        slot, counts, offsets = torch.empty((T, k), **i32), torch.empty(P, **i32), torch.empty(P + 1, **i32)
        por, rop = torch.empty(T * k, **i32), torch.empty(T * k, **i32)
        ws = B._workspace(lib.moe_reroute_permute_workspace_bytes(T, k, P), "cuda")
        ws_ffn = B._workspace(lib.moe_grouped_ffn_workspace_bytes(T, k + S, H, I, P + S, dt), "cuda")
        ws_ffn.fill_(0x5A)                                                  # whatever a previous call left there
        y = torch.empty((T * (k + S), H), dtype=torch.bfloat16, device="cuda")
        args = (logits.data_ptr(), aid.data_ptr(), emap.data_ptr(), T, E, k, N, P, 0, ids.data_ptr(), w.data_ptr(), slot.data_ptr(),
                counts.data_ptr(), offsets.data_ptr(), por.data_ptr(), rop.data_ptr(), B._ptr(ws), ws.numel() if ws is not None else 0)
        ffn = (x.data_ptr(), dt, T, k, H, I, P, S, counts.data_ptr(), offsets.data_ptr(), por.data_ptr(), w13.data_ptr(),
               w2.data_ptr(), B._ptr(s13), B._ptr(s2), y.data_ptr(), ws_ffn.data_ptr(), ws_ffn.numel(), st)
        if planned:
            B._check(lib.moe_route_reroute_permute_plan(*args, H, I, S, dt, ws_ffn.data_ptr(), ws_ffn.numel(), st))
            B._check(lib.moe_grouped_ffn_planned(*ffn))
        else:
            B._check(lib.moe_route_reroute_permute(*args, st))
            if S:
                B._check(lib.moe_grouped_ffn_with_shared(*ffn))
            else:
                B._check(lib.moe_grouped_ffn(*(ffn[:7] + ffn[8:13] + ffn[15:])))
        torch.cuda.synchronize()
        return ids, w, slot, counts, offsets, por, rop, y

    plain, planned = run(False), run(True)
    for name, a, b in zip(("ids", "w", "slot", "counts", "offsets", "pair_of_row", "row_of_pair", "y"), plain, planned):
        assert torch.equal(a, b), name
    # and the plain pair is the oracle's permutation
    ids_ref, _ = moe.route_topk(logits.cpu().numpy(), k)
    slot_ref = moe.reroute(ids_ref, aid_np, emap.cpu().numpy())
    counts_ref, offsets_ref, por_ref, rop_ref = moe.permute(slot_ref, P)
    np.testing.assert_array_equal(planned[5].cpu().numpy(), por_ref)
    np.testing.assert_array_equal(planned[3].cpu().numpy(), counts_ref)
    # fp32 has no plan
    with pytest.raises(ew.EWError):
        ws_ffn = B._workspace(lib.moe_grouped_ffn_workspace_bytes(T, k + S, H, I, P + S, B.EW_F32), "cuda")
        i = lambda *sh: torch.empty(sh, **i32)
        B._check(lib.moe_route_reroute_permute_plan(logits.data_ptr(), aid.data_ptr(), emap.data_ptr(), T, E, k, N, P, 0,
                                                    i(T, k).data_ptr(), torch.empty((T, k), device="cuda").data_ptr(),
                                                    i(T, k).data_ptr(), i(P).data_ptr(), i(P + 1).data_ptr(), i(T * k).data_ptr(),
                                                    i(T * k).data_ptr(), None, 0, H, I, S, B.EW_F32, ws_ffn.data_ptr(),
                                                    ws_ffn.numel(), st))


@pytest.mark.parametrize("T,k,P,S,nf", [(64, 6, 128, 2, 0), (256, 6, 384, 2, 0), (200, 4, 48, 0, 4), (31, 2, 300, 1, 1)],
                         ids=["decode64", "decode256", "nf4-no-shared", "nf1"])
def test_one_launch_for_both_products_equals_two(ew, T, k, P, S, nf):
    """Decode shapes run both products in one launch, second-product items waiting for the activation rows they read:
    bit for bit the two-launch result, on repeated calls (the completion counters are rebuilt by every plan)."""
    rng = np.random.default_rng(T * 3 + P)
    H, I = 512, 384
    ids = np.stack([rng.choice(P, k, replace=False) for _ in range(T)]).astype(np.int32)
    flat = ids.reshape(-1)
    por = np.argsort(flat, kind="stable").astype(np.int32)
    counts = np.bincount(flat, minlength=P).astype(np.int32)
    offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    dev = lambda a: torch.from_numpy(a).cuda()
    bf = lambda *shape, scale=1.0: (torch.from_numpy(rng.standard_normal(shape, dtype=np.float32)) * scale).cuda().bfloat16()
    x, w13, w2 = bf(T, H), bf(P, 2 * I, H, scale=0.04), bf(P, H, I, scale=0.04)
    s13, s2 = (bf(S, 2 * I, H, scale=0.04), bf(S, H, I, scale=0.04)) if S else (None, None)

    def run(two_launches):
        ew.binding.tune_ffn(path=3 if nf else 0, ws_frags=nf, ws_two_launches=two_launches)
        try:
            if S:
                y = ew.binding.moe_grouped_ffn_with_shared(x, k, I, P, dev(counts), dev(offsets), dev(por), w13, w2, s13, s2)
            else:
                y = ew.moe_grouped_ffn(x, k, I, P, dev(counts), dev(offsets), dev(por), w13, w2)
            torch.cuda.synchronize()
        finally:
            ew.binding.tune_ffn()
        return y

    ref = run(True)
    for _ in range(3):
        assert torch.equal(run(False), ref)
    got, xs = to_f64(ref), to_f64(x)
    for s in np.nonzero(counts)[0][:12]:
        r0, r1 = offsets[s], offsets[s + 1]
        want = moe.expert_ffn(xs[por[r0:r1] // k], to_f64(w13[s]), to_f64(w2[s]))
        assert rel_l2(got[r0:r1], want) <= FFN_REL_L2 and max_abs(got[r0:r1], want) <= FFN_MAX_ABS, f"slot {s}"


def test_one_launch_equals_two_on_random_decode_shapes(ew):
    """Twenty random decode-sized calls (token count, top-k, slots, shared experts, skew all drawn): the one-launch
    result equals the two-launch result bit for bit every time, with and without a row map."""
    rng = np.random.default_rng(20250817)
    H, I = 256, 128
    dev = lambda a: torch.from_numpy(a).cuda()
    bf = lambda *shape, scale=1.0: (torch.from_numpy(rng.standard_normal(shape, dtype=np.float32)) * scale).cuda().bfloat16()
    for case in range(20):
        T = int(rng.integers(1, 300))
        k = int(rng.integers(1, 7))
        P = int(rng.integers(k, 200))
        S = int(rng.integers(0, 3))
        hot = rng.random() < 0.5
        ids = np.stack([rng.choice(P, k, replace=False) for _ in range(T)]).astype(np.int32)
        if hot:
            ids[:, 0] = np.where(rng.random(T) < 0.7, 0, ids[:, 0])          # most tokens also visit slot 0 (a repeat is fine here)
        flat = ids.reshape(-1)
        por = np.argsort(flat, kind="stable").astype(np.int32)
        counts = np.bincount(flat, minlength=P).astype(np.int32)
        offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
        x, w13, w2 = bf(T, H), bf(P, 2 * I, H, scale=0.05), bf(P, H, I, scale=0.05)
        s13, s2 = (bf(S, 2 * I, H, scale=0.05), bf(S, H, I, scale=0.05)) if S else (None, None)
        outs = []
        for two in (True, False, False):
            ew.binding.tune_ffn(ws_two_launches=two)
            try:
                if S:
                    y = ew.binding.moe_grouped_ffn_with_shared(x, k, I, P, dev(counts), dev(offsets), dev(por), w13, w2, s13, s2)
                else:
                    y = ew.moe_grouped_ffn(x, k, I, P, dev(counts), dev(offsets), dev(por), w13, w2)
                torch.cuda.synchronize()
            finally:
                ew.binding.tune_ffn()
            outs.append(y)
        assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2]), f"case {case}: T={T} k={k} P={P} S={S} hot={hot}"
        assert torch.isfinite(outs[0].float()).all()
        s = int(np.argmax(counts))
        r0, r1 = offsets[s], offsets[s + 1]
        want = moe.expert_ffn(to_f64(x)[por[r0:r1] // k], to_f64(w13[s]), to_f64(w2[s]))
        got = to_f64(outs[1])[r0:r1]
        assert rel_l2(got, want) <= FFN_REL_L2 and max_abs(got, want) <= FFN_MAX_ABS, f"case {case}: slot {s}"


def test_unpermute_exact_combination(ew):
    """moe_unpermute alone, f32: inputs chosen so fp32 arithmetic is exact."""
    rng = np.random.default_rng(0)
    T, k, H, S = 37, 3, 64, 2
    y = rng.integers(-8, 9, size=(T * k, H)).astype(np.float32)
    w = rng.choice([0.25, 0.5, 1.0, 2.0], size=(T, k)).astype(np.float32)
    sh = rng.integers(-4, 5, size=(S, T, H)).astype(np.float32)
    rop = rng.permutation(T * k).astype(np.int32)
    ref = moe.unpermute(y, rop, w, sh.sum(0))
    dev = lambda a: torch.from_numpy(a).cuda()
    np.testing.assert_array_equal(to_f64(ew.moe_unpermute(dev(y), dev(rop), dev(w), dev(sh))), ref)
    np.testing.assert_array_equal(to_f64(ew.moe_unpermute(dev(y), dev(rop), dev(w), None)), moe.unpermute(y, rop, w))
    yb, shb = dev(y).bfloat16(), dev(sh).bfloat16()                        # small integers: exact in bf16 too
    got = to_f64(ew.moe_unpermute(yb, dev(rop), dev(w), shb))
    np.testing.assert_allclose(got, ref, rtol=2 ** -8)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("T,k,H,S", [(37, 3, 2048, 2), (5, 6, 4104, 0), (64, 2, 256, 1)])
def test_unpermute_rmsnorm_equals_the_two_calls(ew, dtype, T, k, H, S):
    """The fused combine + normalisation: bit for bit the two separate calls, and the oracle's values."""
    rng = np.random.default_rng(T * 7 + H)
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    dev = lambda a: torch.from_numpy(a).cuda()
    y = dev(rng.standard_normal((T * k, H), dtype=np.float32)).to(td)
    w = dev(rng.random((T, k), dtype=np.float32))
    sh = dev(rng.standard_normal((S, T, H), dtype=np.float32)).to(td) if S else None
    res = dev(rng.standard_normal((T, H), dtype=np.float32)).to(td)
    rop_np = rng.permutation(T * k).astype(np.int32)
    rop, eps = dev(rop_np), 1e-6
    out2 = ew.moe_unpermute(y, rop, w, sh, residual=res)
    normed2 = ew.binding.moe_rmsnorm(out2, eps)
    out1, normed1 = ew.binding.moe_unpermute_rmsnorm(y, rop, w, eps, shared_out=sh, residual=res)
    torch.cuda.synchronize()
    assert torch.equal(out1, out2) and torch.equal(normed1, normed2)
    ref = moe.unpermute(to_f64(y), rop_np, w.cpu().numpy(), to_f64(sh).sum(0) if S else None) + to_f64(res)
    tol = 2.0 ** -8 if dtype == "bf16" else 2.0 ** -20
    assert max_abs(to_f64(out1), ref) <= tol * np.abs(ref).max()
    ref_n = moe.rmsnorm(to_f64(out1), eps)
    assert max_abs(to_f64(normed1), ref_n) <= tol * np.abs(ref_n).max()
    with pytest.raises(ew.EWError):
        ew.binding.moe_unpermute_rmsnorm(y, rop, w, eps, shared_out=sh, out=out1, normed_out=out1)


@pytest.mark.parametrize("cfg_index", [0, 1])
def test_gate_logits(ew, cfg_index):
    cfg = wl.get_config(cfg_index).with_(gate_bias=2.0)
    tuned = wl.tuned_sets(cfg)
    x, Wg, aid = wl.tokens(cfg), wl.gate_weight(cfg), wl.adapter_ids(cfg)
    bias = wl.logit_bias_table(cfg, tuned)
    dev = lambda a: torch.from_numpy(a).cuda()
    got = ew.moe_gate_logits(to_torch(x), dev(Wg), dev(aid), dev(bias)).cpu().numpy()
    ref = moe.gate_logits(x, Wg, aid, bias)
    np.testing.assert_allclose(got, ref, rtol=1e-4, atol=2e-5)
    got0 = ew.moe_gate_logits(to_torch(x), dev(Wg)).cpu().numpy()
    np.testing.assert_allclose(got0, moe.gate_logits(x, Wg), rtol=1e-4, atol=2e-5)


def _run_layer_through_pool(ew, cfg, inp, logits, flags=0, aid=None):
    from paper_2508_17624_amd.layer import MoELayer, load_layer
    dt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    el = 2 if cfg.dtype == "bf16" else 4
    pool = ew.ExpertPool(1, cfg.M, cfg.N, cfg.E_max, 2 * cfg.I * cfg.H * el, cfg.H * cfg.I * el, flags=flags)
    t = lambda a: torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a)   # host tensors: H2D copy inside map
    load_layer(pool, 0, (t(inp["base"][0]), t(inp["base"][1])), [(t(a), t(b)) for a, b in inp["adapters"]], inp["tuned"])
    emap = pool.expert_map_host(0).numpy()
    np.testing.assert_array_equal(emap, moe.build_expert_map(cfg.M, cfg.N, cfg.E_max, inp["tuned"]))
    sh13, sh2 = (to_torch(inp["shared"][0]), to_torch(inp["shared"][1])) if cfg.S else (None, None)
    layer = MoELayer(pool, 0, torch.from_numpy(inp["Wg"]).cuda(), sh13, sh2, cfg.k, cfg.I, cfg.T, dt)
    aid_t = torch.from_numpy(inp["aid"] if aid is None else aid).cuda()
    out = layer.forward(to_torch(inp["x"]), aid_t, torch.from_numpy(logits).cuda()).clone()
    torch.cuda.synchronize()
    return pool, layer, out


def test_layer_c0_f32(ew):
    """Config 0 end to end in fp32 through a VMM pool."""
    cfg = wl.get_config(0)
    inp = layer_inputs(cfg)
    logits = moe.gate_logits(inp["x"], inp["Wg"])
    ref = _oracle_layer(cfg, inp, logits)
    pool, layer, out = _run_layer_through_pool(ew, cfg, inp, logits)
    np.testing.assert_array_equal(layer.ids.cpu().numpy(), ref["ids"])
    np.testing.assert_array_equal(layer.slot.cpu().numpy(), ref["slot"])
    np.testing.assert_array_equal(layer.por.cpu().numpy(), ref["pair_of_row"])
    assert rel_l2(to_f64(out), ref["out"]) <= 1e-5                          # fp32 arithmetic, K <= 256
    assert rel_l2(to_f64(layer.y), ref["y_sorted"]) <= 1e-5
    st = pool.stats()
    assert st["experts_loaded"] == cfg.M + sum(len(J) for J in inp["tuned"])
    pool.close()


def test_layer_c1_bf16_vmm_and_merge_equivalence(ew):
    """Config 1 (DeepSeek-V2-Lite decode shape) end to end through a VMM pool; also against the
    merged-model path of the oracle (the paper's accuracy claim) and a base-only batch."""
    cfg = wl.get_config(1)
    inp = layer_inputs(cfg)
    logits = moe.gate_logits(inp["x"], inp["Wg"])
    ref = _oracle_layer(cfg, inp, logits)
    pool, layer, out = _run_layer_through_pool(ew, cfg, inp, logits)
    for name, got in (("ids", layer.ids), ("slot", layer.slot), ("counts", layer.counts), ("offsets", layer.offsets),
                      ("pair_of_row", layer.por), ("row_of_pair", layer.rop)):
        np.testing.assert_array_equal(got.cpu().numpy().reshape(ref[name].shape), ref[name], err_msg=name)
    got = to_f64(out)
    assert rel_l2(to_f64(layer.y), ref["y_sorted"]) <= FFN_REL_L2 and max_abs(to_f64(layer.y), ref["y_sorted"]) <= FFN_MAX_ABS
    assert rel_l2(got, ref["out"]) <= FFN_REL_L2 and max_abs(got, ref["out"]) <= FFN_MAX_ABS
    merged = moe.merged_model_layer(inp["x"], logits, inp["aid"], cfg.k, cfg.M, inp["tuned"], inp["base"], inp["adapters"], inp["shared"])
    assert rel_l2(got, merged) <= FFN_REL_L2
    # base-only batch on the same pool: slots == ids, adapter slots untouched
    aid0 = np.zeros_like(inp["aid"])
    out0 = layer.forward(to_torch(inp["x"]), torch.from_numpy(aid0).cuda(), torch.from_numpy(logits).cuda()).clone()
    ref0 = _oracle_layer(cfg, inp, logits, aid0)
    assert torch.equal(layer.slot, layer.ids) and int(layer.counts[cfg.M:].sum()) == 0
    assert rel_l2(to_f64(out0), ref0["out"]) <= FFN_REL_L2
    # gate kernel feeding the fused router: ids agree wherever the k-th/(k+1)-th margin is clear
    lg = ew.moe_gate_logits(to_torch(inp["x"]), torch.from_numpy(inp["Wg"]).cuda())
    srt = np.sort(logits, axis=1)[:, ::-1]
    clear = (srt[:, :cfg.k] - srt[:, 1:cfg.k + 1]).min(axis=1) > 1e-4
    ids_g, _ = ew.moe_route_topk(lg, cfg.k)
    np.testing.assert_array_equal(ids_g.cpu().numpy()[clear], ref["ids"][clear])
    pool.close()


@pytest.fixture(scope="module")
def c2(ew):
    """Configuration 2 loaded once for the tests below: inputs, VMM pool, layer, oracle-side logits."""
    cfg = wl.get_config(2)
    inp = layer_inputs(cfg)
    logits = moe.gate_logits(inp["x"], inp["Wg"], inp["aid"], inp["bias"])
    pool, layer, out = _run_layer_through_pool(ew, cfg, inp, logits)
    yield dict(cfg=cfg, inp=inp, logits=logits, pool=pool, layer=layer, out=out)
    pool.close()


def _compare_full(cfg, layer, out, ref, T, what):
    """Integer stages bit for bit, combine weights, then every FFN row and every output row."""
    n = T * cfg.k
    for name, got in (("ids", layer.ids[:T]), ("slot", layer.slot[:T]), ("counts", layer.counts), ("offsets", layer.offsets),
                      ("pair_of_row", layer.por[:n]), ("row_of_pair", layer.rop[:n])):
        np.testing.assert_array_equal(got.cpu().numpy().reshape(ref[name].shape), ref[name], err_msg=f"{what}: {name}")
    np.testing.assert_allclose(layer.w[:T].cpu().numpy(), ref["w"], rtol=2e-5, atol=1e-9)
    y = to_f64(layer.y[:n])
    assert np.isfinite(y).all(), f"{what}: a slot without an expert was read"
    assert rel_l2(y, ref["y_sorted"]) <= FFN_REL_L2 and max_abs(y, ref["y_sorted"]) <= FFN_MAX_ABS, what
    # row by row, so that one wrong row of one chunk, fragment or feature group cannot hide in the norm
    err = np.linalg.norm(y - ref["y_sorted"], axis=1) / (np.linalg.norm(ref["y_sorted"], axis=1) + 1e-3)
    assert err.max() <= 3e-2, f"{what}: sorted row {int(err.argmax())} is off by {err.max():.3e}"
    got = to_f64(out)
    assert rel_l2(got, ref["out"]) <= FFN_REL_L2 and max_abs(got, ref["out"]) <= FFN_MAX_ABS, what
    err = np.linalg.norm(got - ref["out"], axis=1) / (np.linalg.norm(ref["out"], axis=1) + 1e-3)
    assert err.max() <= 3e-2, f"{what}: token {int(err.argmax())} is off by {err.max():.3e}"


def test_layer_c2_full_size(ew, c2):
    """Configuration 2 at full size (8192-token prefill, 20 adapters, Zipf classes, biased gates), in the launch
    configuration the benchmark times: every integer output bit for bit, every one of the 49 152 FFN rows and 8192
    output rows against the oracle."""
    cfg, inp, logits, layer = c2["cfg"], c2["inp"], c2["logits"], c2["layer"]
    ref = _oracle_layer(cfg, inp, logits)
    _compare_full(cfg, layer, c2["out"], ref, cfg.T, "c2")
    assert int((ref["counts"] > 0).sum()) > 200                      # the regime of many active slots
    # the gate kernel at this shape (bias per class included)
    lg = ew.moe_gate_logits(to_torch(inp["x"]), torch.from_numpy(inp["Wg"]).cuda(), torch.from_numpy(inp["aid"]).cuda(),
                            torch.from_numpy(inp["bias"]).cuda()).cpu().numpy()
    np.testing.assert_allclose(lg, logits, rtol=1e-4, atol=3e-5)
    # base-only traffic on the same pool (what the overhead is measured against)
    aid0 = np.zeros_like(inp["aid"])
    logits0 = moe.gate_logits(inp["x"], inp["Wg"])
    out0 = layer.forward(to_torch(inp["x"]), torch.from_numpy(aid0).cuda(), torch.from_numpy(logits0).cuda()).clone()
    torch.cuda.synchronize()
    _compare_full(cfg, layer, out0, _oracle_layer(cfg, inp, logits0, aid0), cfg.T, "c2 base-only")


@pytest.mark.parametrize("T,n_adapters,alpha", [(512, 5, 1.0), (512, 5, 0.1), (512, 20, 1.0), (512, 20, 0.1),
                                                (2048, 5, 1.0), (2048, 5, 0.1), (2048, 20, 1.0), (2048, 20, 0.1)])
def test_second_workload_parity(ew, c2, T, n_adapters, alpha):
    """Chunked-prefill sizes with skewed adapter popularity on the configuration-2 layer (Sec. 5.1: per-adapter
    request shares from a power law with shape alpha; Sec. 5.2: 5 to 20 adapters), the points the benchmark's
    sweep times: all outputs against the oracle."""
    cfg, inp, layer = c2["cfg"], c2["inp"], c2["layer"]
    aid = wl.adapter_ids_powerlaw(cfg, T, n_adapters, alpha)
    assert aid.min() >= 1 and aid.max() <= n_adapters
    sub = dict(inp, x=inp["x"][:T], aid=aid)
    logits = moe.gate_logits(sub["x"], inp["Wg"], aid, inp["bias"])
    out = layer.forward(to_torch(sub["x"]), torch.from_numpy(aid).cuda(), torch.from_numpy(logits).cuda()).clone()
    torch.cuda.synchronize()
    ref = _oracle_layer(cfg, sub, logits)
    _compare_full(cfg, layer, out, ref, T, f"T={T} n={n_adapters} alpha={alpha}")


def test_layer_c1_padded_pool_matches_oracle_and_vmm(ew):
    """The padding approach of Sec. 3.1 on the real VMM backend (every slot backed): same outputs as the oracle, and
    bit-identical to the sparse virtual tensor's (the kernels never learn which pool they run on)."""
    cfg = wl.get_config(1)
    inp = layer_inputs(cfg)
    logits = moe.gate_logits(inp["x"], inp["Wg"])
    ref = _oracle_layer(cfg, inp, logits)
    outs, stats = {}, {}
    for mode, flags in (("vmm", ew.EW_POOL_VMM), ("padded", ew.EW_POOL_PADDED)):
        pool, layer, out = _run_layer_through_pool(ew, cfg, inp, logits, flags=flags)
        _compare_full(cfg, layer, out, ref, cfg.T, mode)
        outs[mode], stats[mode] = (out, layer.y[:cfg.T * cfg.k].clone()), pool.stats()
        pool.close()
    assert torch.equal(outs["vmm"][0], outs["padded"][0]) and torch.equal(outs["vmm"][1], outs["padded"][1])
    el = 2 * 3 * cfg.H * cfg.I
    assert stats["padded"]["pages_mapped"] * stats["padded"]["page_bytes"] >= cfg.P * el
    assert stats["vmm"]["pages_mapped"] < stats["padded"]["pages_mapped"]
    assert stats["vmm"]["f_mem"] == pytest.approx(cfg.P / (cfg.M + sum(len(J) for J in inp["tuned"])))


def test_ffn_argument_errors(ew):
    x = torch.zeros((4, 100), dtype=torch.bfloat16, device="cuda")
    c = torch.zeros(2, dtype=torch.int32, device="cuda")
    with pytest.raises(ew.EWError) as e:
        ew.moe_grouped_ffn(x, 1, 128, 2, c, c, c, x, x)
    assert e.value.code == -6


def test_fused_entry_points_empty_batch_and_argument_errors(ew):
    """T = 0 is a no-op (counts zeroed by the permutation call); bad arguments come back as error codes, never as a launch."""
    B = ew.binding
    lib, st = B.lib(), B._stream()
    i32 = dict(dtype=torch.int32, device="cuda")
    H, I, E, N, P, k, S = 256, 128, 8, 1, 12, 2, 1
    counts, offsets = torch.full((P,), 7, **i32), torch.full((P + 1,), 7, **i32)
    emap = torch.arange(E, **i32).repeat(N + 1, 1).contiguous()
    dummy = torch.zeros(4096, dtype=torch.bfloat16, device="cuda")
    ws = B._workspace(max(lib.moe_grouped_ffn_workspace_bytes(1, k + S, H, I, P + S, B.EW_BF16), 256), "cuda")
    assert lib.moe_route_reroute_permute_plan(None, None, emap.data_ptr(), 0, E, k, N, P, 0, None, None, dummy.data_ptr(),
                                              counts.data_ptr(), offsets.data_ptr(), dummy.data_ptr(), None, None, 0, H, I, S,
                                              B.EW_BF16, None, 0, st) == 0
    torch.cuda.synchronize()
    assert int(counts.abs().sum()) == 0 and int(offsets.abs().sum()) == 0
    for fn in (lib.moe_grouped_ffn_planned, lib.moe_grouped_ffn_with_shared):
        assert fn(None, B.EW_BF16, 0, k, H, I, P, S, None, None, None, None, None, None, None, None, None, 0, st) == 0
    assert lib.moe_unpermute_rmsnorm(None, None, None, None, 0, None, 0, k, H, B.EW_BF16, None, 1e-6, None, st) == 0
    # errors: S < 1 for the shared variant, a negative S, H not a multiple of 128, a workspace that is too small
    args = lambda S_, H_, ws_bytes: (dummy.data_ptr(), B.EW_BF16, 1, k, H_, I, P, S_, counts.data_ptr(), offsets.data_ptr(), None,
                                     dummy.data_ptr(), dummy.data_ptr(), dummy.data_ptr(), dummy.data_ptr(), dummy.data_ptr(),
                                     ws.data_ptr(), ws_bytes, st)
    assert lib.moe_grouped_ffn_with_shared(*args(0, H, ws.numel())) == -1          # EW_ERR_INVALID_ARG
    assert lib.moe_grouped_ffn_planned(*args(-1, H, ws.numel())) == -1
    assert lib.moe_grouped_ffn_with_shared(*args(S, 192, ws.numel())) == -6        # EW_ERR_UNSUPPORTED
    assert lib.moe_grouped_ffn_planned(*args(S, H, 256)) == lib.moe_grouped_ffn_with_shared(*args(S, H, 256)) != 0
    assert "workspace" in lib.ew_last_error().decode()
    assert lib.moe_unpermute_rmsnorm(dummy.data_ptr(), counts.data_ptr(), dummy.data_ptr(), None, 0, None, 1, k, H, B.EW_BF16,
                                     dummy.data_ptr(), 1e-6, dummy.data_ptr(), st) == -1   # normed_out must not be out
    torch.cuda.synchronize()
