"""GPU check of moe_reroute_permute_static, the entry point that allocates nothing (its scratch is a device
array built into the library): same outputs as moe_reroute_permute, bit for bit, on calls in a row that share
the built-in buffer -- a large batch, then smaller ones -- and a clear error beyond the buffer's size."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import moe

pytestmark = pytest.mark.gpu


def test_static_scratch_variant_matches_workspace_variant():
    import paper_2508_17624_amd as ew
    from paper_2508_17624_amd import binding as B
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    lib = ew.lib()
    cfg = wl.get_config(3)
    k, P, N, E = cfg.k, cfg.P, cfg.N, cfg.M
    emap_np = moe.build_expert_map(cfg.M, cfg.N, cfg.E_max, wl.tuned_sets(cfg))
    emap = torch.from_numpy(emap_np).cuda()
    T_max = 40000
    ids_all = torch.from_numpy(wl.distinct_topk_ids(cfg, T_max)).cuda()
    aid_all = torch.from_numpy(wl.adapter_ids(cfg, T_max)).cuda()
    i32 = dict(dtype=torch.int32, device="cuda")
    assert lib.moe_reroute_permute_static_max_bytes() == 4 << 20
    # two calls in a row on the multi-block path (the second smaller: it must not see the first one's table),
    # then a batch small enough for the single-block path, then the large one again
    for T in (T_max, 3000, 300, T_max):
        ids, aid = ids_all[:T].contiguous(), aid_all[:T].contiguous()
        assert lib.moe_reroute_permute_workspace_bytes(T, k, P) <= lib.moe_reroute_permute_static_max_bytes()
        out = (torch.full((T, k), -1, **i32), torch.full((P,), -1, **i32), torch.full((P + 1,), -1, **i32),
               torch.full((T * k,), -1, **i32), torch.full((T * k,), -1, **i32))
        before = torch.cuda.memory_allocated()
        B.moe_reroute_permute_static(ids, aid, emap, N, P, out)
        assert torch.cuda.memory_allocated() == before               # nothing came from torch's allocator either
        torch.cuda.synchronize()
        ref = B.moe_reroute_permute(ids, aid, emap, N, P)
        torch.cuda.synchronize()
        for name, a, b in zip(("slot", "counts", "offsets", "pair_of_row", "row_of_pair"), out, ref):
            assert torch.equal(a, b), f"T={T}: {name} differs from moe_reroute_permute"
        # and both equal the oracle
        slot = moe.reroute(ids.cpu().numpy(), aid.cpu().numpy(), emap_np)
        counts, offsets, por, rop = moe.permute(slot, P)
        for name, a, b in zip(("slot", "counts", "offsets", "pair_of_row", "row_of_pair"), out, (slot, counts, offsets, por, rop)):
            np.testing.assert_array_equal(a.cpu().numpy().reshape(b.shape), b, err_msg=f"T={T}: {name}")
    # beyond the built-in buffer: a clear error, nothing launched (host-side check, no device memory touched)
    T_big = 1 << 22
    assert lib.moe_reroute_permute_workspace_bytes(T_big, k, 2048) > lib.moe_reroute_permute_static_max_bytes()
    rc = lib.moe_reroute_permute_static(None, None, None, T_big, k, E, N, 2048, None, None, None, None, None, None)
    assert rc == -6 and b"built-in buffer" in lib.ew_last_error()
