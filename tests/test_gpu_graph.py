"""A layer step and a small stack of layers captured in a HIP graph: the library's calls on the bf16 path enqueue
kernels only (no allocation, no memset node, no host synchronisation, no second stream), so a serving loop can replay
them.  Every replay must reproduce the eager result bit for bit, with eager work of the program in between."""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_common import layer_inputs, to_torch

pytestmark = pytest.mark.gpu


def _host(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a)


def test_layer_step_and_stack_replay_from_a_graph():
    import paper_2508_17624_amd as ew
    from paper_2508_17624_amd.layer import MoEStack, load_layer
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    ew.lib()
    L = 3
    cfg = wl.get_config(1).with_(index=71, L=L, T=48)
    pool = ew.ExpertPool(L, cfg.M, cfg.N, cfg.E_max, 2 * cfg.I * cfg.H * 2, cfg.H * cfg.I * 2)
    gates, shared = [], []
    for l in range(L):
        inp = layer_inputs(cfg, l)
        load_layer(pool, l, (_host(inp["base"][0]), _host(inp["base"][1])), [(_host(a), _host(b)) for a, b in inp["adapters"]],
                   inp["tuned"])
        gates.append(torch.from_numpy(inp["Wg"]).cuda())
        shared.append((to_torch(inp["shared"][0]), to_torch(inp["shared"][1])))
    stack = MoEStack(pool, gates, shared, cfg.k, cfg.I, cfg.T, torch.bfloat16)
    x = to_torch(wl.tokens(cfg))
    aid = torch.from_numpy(wl.adapter_ids(cfg)).cuda()
    aid2 = torch.roll(aid, 5)

    eager = stack.forward(x, aid).clone()            # also warms up everything a first call sets up
    eager2 = stack.forward(x, aid2).clone()
    torch.cuda.synchronize()
    assert not torch.equal(eager, eager2)

    # static inputs of the graph: x_in and aid_in are overwritten between replays
    x_in, aid_in = x.clone(), aid.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        stack.forward(x_in, aid_in)                  # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        out_ref = stack.forward(x_in, aid_in)
    torch.cuda.synchronize()

    for i, (a, want) in enumerate([(aid, eager), (aid2, eager2), (aid, eager), (aid2, eager2)]):
        aid_in.copy_(a)
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_ref, want), f"replay {i} differs from the eager result"
        # eager work between the replays, on the same buffers
        again = stack.forward(x, aid2 if i % 2 == 0 else aid)
        torch.cuda.synchronize()
        assert torch.equal(again, eager2 if i % 2 == 0 else eager)
    pool.close()
