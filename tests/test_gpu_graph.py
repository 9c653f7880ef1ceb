"""The four calls only enqueue kernels on the caller's stream, so a caller may capture an iteration into a HIP graph
(worth it when the step is launch-bound, as for the Tiny configuration).  Every replay is checked against eager."""
import pytest
import torch

from paper_2502_11058_amd import workloads as W

pytestmark = pytest.mark.gpu


def test_graph_replays_match_eager_bit_for_bit():
    from paper_2502_11058_amd.harness import DeviceReplica
    assert torch.cuda.is_available(), "no GPU visible"
    w = W.tiny()                                   # SGD-momentum: no per-step scalars baked into the launch
    H = w.period
    eager, graphed = DeviceReplica(w, 0), DeviceReplica(w, 0)
    for rep in (eager, graphed):
        rep.init_params()
    graphs = []
    side = torch.cuda.Stream()
    for slot in range(H):
        g = torch.cuda.CUDAGraph()
        snap = (graphed.a_sync.clone(), graphed.a_s0.clone())
        with torch.cuda.graph(g, stream=side):
            graphed.step(slot)
        graphed.a_sync.copy_(snap[0])              # capture does not run the kernels, but be explicit about state
        graphed.a_s0.copy_(snap[1])
        graphs.append(g)
    for r in range(4 * H):
        for rep in (eager, graphed):               # fresh inputs written in place between replays: eager torch work
            rep.fill_grads(r)
            n = rep.slot_numel[r % H]
            rep.fill_peers_from(torch.zeros_like(rep.flat), r, n)
        eager.step(r)
        graphs[r % H].replay()
        torch.cuda.synchronize()
        assert torch.equal(eager.a_sync.view(torch.int32), graphed.a_sync.view(torch.int32)), f"params r={r}"
        assert torch.equal(eager.a_s0.view(torch.int32), graphed.a_s0.view(torch.int32)), f"momentum r={r}"
        assert torch.equal(eager.stats, graphed.stats), f"statistics r={r}"
    # launch-bound step: the replay is faster than five eager launches
    e0, e1, e2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
    e0.record()
    for r in range(200):
        eager.step(r)
    e1.record()
    for r in range(200):
        graphs[r % H].replay()
    e2.record()
    torch.cuda.synchronize()
    print(f"tiny step: eager {e0.elapsed_time(e1) / 200 * 1e3:.1f} us, graph replay {e1.elapsed_time(e2) / 200 * 1e3:.1f} us")
    eager.close()
    graphed.close()
