"""GPU parity: router top-k, batched rerouting, permutation -- bit-exact against the oracle."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import moe

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ew():
    import paper_2508_17624_amd as m
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    m.lib()
    return m


def _expert_map(cfg, layer=0):
    tuned = wl.tuned_sets(cfg, layer)
    return tuned, moe.build_expert_map(cfg.M, cfg.N, cfg.E_max, tuned)


def _check_permutation(got, ref_slot, P):
    slot, counts, offsets, por, rop = (t.cpu().numpy() for t in got)
    rc, ro, rp, rr = moe.permute(ref_slot, P)
    np.testing.assert_array_equal(slot, ref_slot)
    np.testing.assert_array_equal(counts, rc)
    np.testing.assert_array_equal(offsets, ro)
    np.testing.assert_array_equal(por, rp)
    np.testing.assert_array_equal(rop, rr)


@pytest.mark.parametrize("T,E,k", [(64, 8, 2), (64, 64, 6), (1000, 64, 6), (33, 160, 8), (7, 1024, 64), (1, 5, 5)])
@pytest.mark.parametrize("renorm", [False, True])
def test_route_topk(ew, T, E, k, renorm):
    rng = np.random.default_rng(T * 7 + E)
    logits = (rng.standard_normal((T, E)) * 1.5).astype(np.float32)
    ids, w = ew.moe_route_topk(torch.from_numpy(logits).cuda(), k, renorm)
    rids, rw = moe.route_topk(logits, k, renorm)
    np.testing.assert_array_equal(ids.cpu().numpy(), rids)
    np.testing.assert_allclose(w.cpu().numpy(), rw, rtol=2e-5, atol=1e-9)


def test_route_topk_ties_and_signed_zero(ew):
    rng = np.random.default_rng(5)
    logits = rng.integers(-2, 3, size=(512, 64)).astype(np.float32)       # many exact ties
    z = logits == 0
    logits[z] = np.where(rng.random(z.sum()) < 0.5, 0.0, -0.0)
    logits[0, :] = 1.25                                                    # all equal -> 0..k-1
    ids, w = ew.moe_route_topk(torch.from_numpy(logits).cuda(), 6)
    rids, rw = moe.route_topk(logits, 6)
    np.testing.assert_array_equal(ids.cpu().numpy(), rids)
    assert ids[0].tolist() == [0, 1, 2, 3, 4, 5]
    np.testing.assert_allclose(w.cpu().numpy(), rw, rtol=2e-5)


@pytest.mark.parametrize("T", [1, 64, 256, 341, 342, 682, 683, 1366, 2048, 2049, 5000])
def test_reroute_permute_configs(ew, T):
    """C2/C3-shaped: k=6, E=64, N=20, P=384.  T=341 is the last size of the single-block permutation
    (2048 pairs at most), 342 the first multi-block one; 2048 tokens fill one block's 12288 pairs
    exactly and 2049 spill into a second; 5000 spans several blocks with a ragged tail."""
    cfg = wl.get_config(3)
    tuned, emap = _expert_map(cfg)
    ids = wl.distinct_topk_ids(cfg, T)
    aid = wl.adapter_ids(cfg, T)
    got = ew.moe_reroute_permute(torch.from_numpy(ids).cuda(), torch.from_numpy(aid).cuda(),
                                 torch.from_numpy(emap).cuda(), cfg.N, cfg.P)
    _check_permutation(got, moe.reroute(ids, aid, emap), cfg.P)
    base = aid == 0
    assert np.array_equal(got[0].cpu().numpy()[base], ids[base])            # base tokens unchanged


@pytest.mark.parametrize("T,k,E,N,P", [(300, 1, 4, 0, 4), (100, 64, 64, 1, 128), (4000, 3, 2048, 0, 2048),
                                       (50, 2, 8, 2, 12), (9000, 5, 16, 3, 1)])
def test_reroute_permute_shapes_with_duplicates(ew, T, k, E, N, P):
    """Arbitrary expert maps (duplicate slots inside a token allowed): the sort stays stable."""
    rng = np.random.default_rng(T + k + P)
    ids = rng.integers(0, E, size=(T, k)).astype(np.int32)
    aid = rng.integers(0, N + 1, size=T).astype(np.int32)
    emap = rng.integers(0, P, size=(N + 1, E)).astype(np.int32)
    got = ew.moe_reroute_permute(torch.from_numpy(ids).cuda(), torch.from_numpy(aid).cuda(),
                                 torch.from_numpy(emap).cuda(), N, P)
    _check_permutation(got, moe.reroute(ids, aid, emap), P)


def test_reroute_permute_all_to_one_slot_and_skip_inverse(ew):
    T, k, P = 3000, 4, 16
    ids = np.zeros((T, k), np.int32); aid = np.zeros(T, np.int32)
    emap = np.full((1, 1), 7, np.int32)
    slot, counts, offsets, por, rop = ew.moe_reroute_permute(torch.from_numpy(ids).cuda(), torch.from_numpy(aid).cuda(),
                                                             torch.from_numpy(emap).cuda(), 0, P, want_row_of_pair=False)
    assert rop is None and counts[7].item() == T * k and counts.sum().item() == T * k
    np.testing.assert_array_equal(por.cpu().numpy(), np.arange(T * k))


def test_empty_batch(ew):
    cfg = wl.get_config(1)
    _, emap = _expert_map(cfg)
    z = lambda *s: torch.zeros(s, dtype=torch.int32, device="cuda")
    slot, counts, offsets, por, rop = ew.moe_reroute_permute(z(0, 6), z(0), torch.from_numpy(emap).cuda(), cfg.N, cfg.P)
    assert counts.tolist() == [0] * cfg.P and offsets.tolist() == [0] * (cfg.P + 1)


@pytest.mark.parametrize("cfg_index,T", [(0, 64), (1, 64), (2, 300), (2, 341), (2, 342), (2, 2049), (2, 8192), (4, 256)])
def test_fused_route_reroute_permute(ew, cfg_index, T):
    cfg = wl.get_config(cfg_index)
    tuned, emap = _expert_map(cfg)
    rng = np.random.default_rng(cfg.seed)
    aid = wl.adapter_ids(cfg, T)
    logits = (rng.standard_normal((T, cfg.M)) * 0.9).astype(np.float32)
    if cfg.gate_bias:
        logits += wl.logit_bias_table(cfg, tuned)[aid]
    ids, w, *perm = ew.moe_route_reroute_permute(torch.from_numpy(logits).cuda(), torch.from_numpy(aid).cuda(),
                                                 torch.from_numpy(emap).cuda(), cfg.k, cfg.N, cfg.P)
    rids, rw = moe.route_topk(logits, cfg.k)
    np.testing.assert_array_equal(ids.cpu().numpy(), rids)
    np.testing.assert_allclose(w.cpu().numpy(), rw, rtol=2e-5, atol=1e-9)
    _check_permutation(perm, moe.reroute(rids, aid, emap), cfg.P)
    # same answer as the two stand-alone calls
    ids2, w2 = ew.moe_route_topk(torch.from_numpy(logits).cuda(), cfg.k)
    assert torch.equal(ids, ids2) and torch.equal(w, w2)


def test_c3_full_size(ew):
    """Config 3 at full size (1,048,576 tokens x top-6): every output bit-exact."""
    cfg = wl.get_config(3)
    tuned, emap = _expert_map(cfg)
    ids = wl.distinct_topk_ids(cfg)
    aid = wl.adapter_ids(cfg)
    got = ew.moe_reroute_permute(torch.from_numpy(ids).cuda(), torch.from_numpy(aid).cuda(),
                                 torch.from_numpy(emap).cuda(), cfg.N, cfg.P)
    torch.cuda.synchronize()
    _check_permutation(got, moe.reroute(ids, aid, emap), cfg.P)


@pytest.mark.parametrize("cfg_index,T", [(1, 64), (2, 8192), (3, 100000)])
def test_reroute_singleop_matches_fused(ew, cfg_index, T):
    """The unfused three-operator rerouting (paper Sec. 5.3 baseline) gives the oracle's slots bit for bit, and a
    permutation of those slots through an identity map equals the fused kernel's."""
    cfg = wl.get_config(cfg_index)
    tuned, emap = _expert_map(cfg)
    ids = wl.distinct_topk_ids(cfg, T)
    aid = wl.adapter_ids(cfg, T)
    d = lambda a: torch.from_numpy(a).cuda()
    slot = ew.moe_reroute_singleop(d(ids), d(aid), d(emap), cfg.N)
    ref = moe.reroute(ids, aid, emap)
    np.testing.assert_array_equal(slot.cpu().numpy(), ref)
    ident = torch.arange(cfg.P, dtype=torch.int32, device="cuda").reshape(1, cfg.P)
    zero = torch.zeros(T, dtype=torch.int32, device="cuda")
    two_step = ew.moe_reroute_permute(slot, zero, ident, 0, cfg.P)
    fused = ew.moe_reroute_permute(d(ids), d(aid), d(emap), cfg.N, cfg.P)
    for a, b in zip(two_step, fused):
        assert torch.equal(a, b)


def test_argument_errors(ew):
    z = torch.zeros((4, 2), dtype=torch.int32, device="cuda")
    a = torch.zeros(4, dtype=torch.int32, device="cuda")
    m = torch.zeros((1, 8), dtype=torch.int32, device="cuda")
    with pytest.raises(ew.EWError) as e:
        ew.moe_reroute_permute(z, a, m, 0, 5000)
    assert e.value.code == -6
    with pytest.raises(ew.EWError) as e:
        ew.moe_route_topk(torch.zeros((4, 8), device="cuda"), 9)
    assert e.value.code == -1
