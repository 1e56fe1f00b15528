"""The propagation calls enqueue kernels only (no allocation, no wait, no memset), so a caller can
record them into a HIP graph.  Replays, with eager work and synchronizations in between, must
reproduce the eager result bit for bit every time."""
import numpy as np
import pytest
import torch

from parity import to_device
from workloads import make_config, make_edge_weights

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("weighted", [False, True])
def test_propagate_fwd_bwd_replayed_from_a_graph(weighted):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2511_20564_amd.device as dev
    dev.B.load_library()
    c = make_config(2, scale=0.2)
    K, dt, F = c["K"], c["dtype"], c["F"]
    u, i = torch.from_numpy(c["users"]).cuda(), torch.from_numpy(c["items"]).cuda()
    if weighted:
        g = dev.build_weighted_graph(c["n_users"], c["n_items"], u, i,
                                     torch.from_numpy(make_edge_weights(c["users"].size, seed=1)).cuda())
    else:
        g = dev.build_graph(c["n_users"], c["n_items"], u, i)
    X0, gY = to_device(c["X0"], dt), to_device(c["gY"], dt)
    ws = dev.propagate_workspace(g, X0.dtype, F, K)
    out_f, out_b = torch.empty_like(X0), torch.empty_like(X0)
    eager_f = dev.propagate_fwd(g, X0, K).clone()
    eager_b = dev.propagate_bwd(g, gY, K).clone()
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(s):
        dev.propagate_fwd(g, X0, K, out=out_f, ws=ws)        # warm-up on the capture stream
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=s):
            dev.propagate_fwd(g, X0, K, out=out_f, ws=ws)
            dev.propagate_bwd(g, gY, K, out=out_b, ws=ws)
    torch.cuda.current_stream().wait_stream(s)
    for rep in range(4):
        out_f.zero_()
        out_b.zero_()
        scratch = dev.propagate_fwd(g, gY, 1)               # eager work between replays, other buffers
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_f, eager_f), rep
        assert torch.equal(out_b, eager_b), rep
        del scratch
