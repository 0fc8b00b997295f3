"""GPU parity of configuration 4: 26 stacked DeepSeek-V2-Lite-shaped MoE layers over one VMM pool,
one 256-token decode step with 20 adapters, against the fp64 oracle with teacher forcing: the oracle
of layer l is fed the GPU's own input h_l and the GPU's fp32 gate logits, so that a single top-k flip
or rounding difference cannot cascade through the stack.  Layers are chained as a pre-norm residual
stream, h_{l+1} = h_l + MoE_l(rmsnorm(h_l)) in bf16 (no attention): without the normalisation the
activations of random-initialised SwiGLU layers grow quadratically from layer to layer."""
import time

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import moe
from gpu_common import FFN_MAX_ABS, FFN_REL_L2, max_abs, rel_l2, to_torch

pytestmark = pytest.mark.gpu

SAMPLE_TOKENS = 32          # tokens per layer whose FFN outputs the oracle recomputes (8 expert FFNs each) ...
FULL_LAYERS = (0, 12, 25)   # ... and the layers where it recomputes all 256 tokens


def _bits(t: torch.Tensor) -> np.ndarray:
    """bf16 tensor -> uint16 bit patterns on the host (what the oracle widens exactly)."""
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def _host(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a)


def test_c4_stack_teacher_forced():
    import paper_2508_17624_amd as ew
    from paper_2508_17624_amd.layer import MoEStack, load_layer
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    ew.lib()
    cfg = wl.get_config(4)
    L, T, k = cfg.L, cfg.T, cfg.k
    t0 = time.time()
    pool = ew.ExpertPool(L, cfg.M, cfg.N, cfg.E_max, 2 * cfg.I * cfg.H * 2, cfg.H * cfg.I * 2)
    gates_np = [wl.gate_weight(cfg, l) for l in range(L)]
    shared_np = [wl.shared_weights(cfg, l) for l in range(L)]
    gates = [torch.from_numpy(g).cuda() for g in gates_np]
    shared = [(to_torch(a), to_torch(b)) for a, b in shared_np]
    stack = MoEStack(pool, gates, shared, k, cfg.I, T, torch.bfloat16)
    aid_np = wl.adapter_ids(cfg)
    aid = torch.from_numpy(aid_np).cuda()
    h = to_torch(wl.tokens(cfg))
    h0 = h.clone()
    hidden = []                     # h_1 .. h_L of the layer-by-layer pass
    active_total = 0
    for l in range(L):
        tuned = wl.tuned_sets(cfg, l)
        base = wl.stacked_expert_weights(cfg, l, 0, cfg.M)
        adapters = [wl.stacked_expert_weights(cfg, l, a + 1, len(tuned[a])) for a in range(cfg.N)]
        load_layer(pool, l, (_host(base[0]), _host(base[1])), [(_host(a), _host(b)) for a, b in adapters], tuned)
        layer = stack.layers[l]
        h_next = stack.forward(h, aid, first=l, last=l + 1).clone()
        torch.cuda.synchronize()
        # integer stages: bit-exact against the oracle run on the GPU's own logits
        logits = layer.logits[:T].cpu().numpy()
        ids, w = moe.route_topk(logits, k)
        emap = moe.build_expert_map(cfg.M, cfg.N, cfg.E_max, tuned)
        np.testing.assert_array_equal(pool.expert_map_host(l).numpy(), emap, err_msg=f"layer {l} expert map")
        slot = moe.reroute(ids, aid_np, emap)
        counts, offsets, por, rop = moe.permute(slot, cfg.P)
        for name, got, ref in (("ids", layer.ids, ids), ("slot", layer.slot, slot), ("counts", layer.counts, counts),
                               ("offsets", layer.offsets, offsets), ("pair_of_row", layer.por, por),
                               ("row_of_pair", layer.rop, rop)):
            np.testing.assert_array_equal(got.cpu().numpy().reshape(ref.shape), ref, err_msg=f"layer {l} {name}")
        np.testing.assert_allclose(layer.w.cpu().numpy(), w, rtol=2e-5, atol=1e-9)
        active_total += int((counts > 0).sum())
        # the normalisation and the gate kernel, each against the oracle on the GPU's own input
        n_bits = _bits(stack.normed[:T])
        ref_n = moe.rmsnorm(_bits(h))
        assert max_abs(moe.as_f64(n_bits), ref_n) <= 2.0 ** -8 * np.abs(ref_n).max(), f"layer {l} rmsnorm"   # one bf16 rounding
        h_bits = n_bits
        ref_logits = moe.gate_logits(h_bits, gates_np[l])
        np.testing.assert_allclose(logits, ref_logits, rtol=1e-4, atol=5e-5, err_msg=f"layer {l} gate logits")
        # FFN outputs on a per-layer sample of tokens that holds every class present in the batch (the base model
        # and each adapter, a different token of each from layer to layer); all tokens in FULL_LAYERS
        rng = np.random.default_rng(1000 + l)
        per_class = [np.nonzero(aid_np == a)[0] for a in np.unique(aid_np)]
        sample = np.array([c[l % len(c)] for c in per_class])
        rest = np.setdiff1d(np.arange(T), sample)
        sample = np.sort(np.concatenate([sample, rng.choice(rest, max(0, SAMPLE_TOKENS - len(sample)), replace=False)]))
        if l in FULL_LAYERS:
            sample = np.arange(T)
        assert len(sample) >= SAMPLE_TOKENS and set(aid_np[sample].tolist()) == set(aid_np.tolist())
        ref = moe.moe_layer(h_bits[sample], logits[sample], aid_np[sample], k, cfg.M, cfg.N, cfg.E_max, tuned, base, adapters,
                            shared_np[l])
        pairs = (sample[:, None] * k + np.arange(k)).reshape(-1)
        got_y = layer.y.detach().to(torch.float64).cpu().numpy()[rop[pairs]]
        ref_y = ref["y_sorted"][ref["row_of_pair"]]
        assert rel_l2(got_y, ref_y) <= FFN_REL_L2 and max_abs(got_y, ref_y) <= FFN_MAX_ABS, f"layer {l} FFN rows"
        # residual stream: h_{l+1} = bf16(h_l + MoE_l(h_l)); the rounding of the sum adds half a bf16 ulp of |h|
        got_h = h_next.to(torch.float64).cpu().numpy()[sample]
        ref_h = moe.as_f64(_bits(h)[sample]) + ref["out"]
        half_ulp = 2.0 ** (np.floor(np.log2(np.abs(ref_h).max())) - 8)
        assert rel_l2(got_h, ref_h) <= FFN_REL_L2 and max_abs(got_h, ref_h) <= FFN_MAX_ABS + half_ulp, f"layer {l} output"
        hidden.append(h_next)
        h = h_next
        print(f"layer {l}: active slots {int((counts > 0).sum())}, {time.time() - t0:.0f} s", flush=True)
        del base, adapters

    st = pool.stats()
    assert st["experts_loaded"] == sum(cfg.M + sum(len(J) for J in wl.tuned_sets(cfg, l)) for l in range(L))
    # the whole stack in one pass reproduces the layer-by-layer hidden states bit for bit (deterministic kernels)
    out = stack.forward(h0, aid).clone()
    torch.cuda.synchronize()
    assert torch.equal(out, hidden[-1])
    # base-only traffic on the same pools: no adapter slot is touched in any layer
    aid0 = torch.zeros_like(aid)
    h = h0
    for l in range(L):
        h = stack.forward(h, aid0, first=l, last=l + 1)
        assert int(stack.layers[l].counts[cfg.M:].sum()) == 0 and torch.equal(stack.layers[l].slot, stack.layers[l].ids)
    torch.cuda.synchronize()
    assert torch.isfinite(h.float()).all()
    print(f"stack: {active_total} active (layer, slot) pairs with 20 adapters vs {L * cfg.M} base-only; pool {st}", flush=True)
    pool.close()
