"""ddp_partial_average_static (the averaging entry point whose reduction scratch is a fixed array in the library's
device image) against ddp_partial_average, through the C ABI: same flat_out and layer_stats bit for bit, on two calls in
a row of which the second has the smaller input, so that what the first call left in the shared array cannot leak into
the second result.  Also: a slot beyond the fixed array's capacity is refused before anything is launched."""
import numpy as np
import pytest
import torch

from paper_2502_11058_amd import binding as B
from paper_2502_11058_amd import workloads as W

pytestmark = pytest.mark.gpu


def _both(rep, slot, rank, n):
    """(flat_out, stats) of the existing entry point and of the static one on the same inputs."""
    c, N = rep.ctx, len(rep.peers) + 1
    nl = c.ddp_slot_num_layers(slot)
    out = []
    for fn in (c.ddp_partial_average, c.ddp_partial_average_static):
        dst = torch.full_like(rep.flat, float("nan"))
        stats = torch.full((2 * nl,), -1.0, dtype=torch.float64, device=rep.dev)
        fn(slot, rep.flat, rep.peers, N, rank, dst, stats)
        torch.cuda.synchronize()
        out.append((dst[:n].clone(), stats.clone()))
    return out


@pytest.mark.timeout(300)
def test_static_scratch_matches_the_allocating_entry_point(oracle):
    from paper_2502_11058_amd.harness import DeviceReplica
    assert torch.cuda.is_available(), "no GPU visible"
    # a Llama-shaped model with uneven slots: embedding and head make the first and the last slot the large ones
    w = W.small_llama(n_blocks=6, d=512, ffn=1376, vocab=8000, n_replicas=5, period=3)
    rep = DeviceReplica(w, 0)
    rep.init_params()
    sizes = rep.slot_numel
    big, small = int(np.argmax(sizes)), int(np.argmin([s if s > 0 else 1 << 62 for s in sizes]))
    assert 0 < sizes[small] < sizes[big]
    for call, (slot, rank) in enumerate(((big, 1), (small, 3))):          # second call: the smaller input
        n = sizes[slot]
        rep.ctx.ddp_pack(slot, rep.flat)
        torch.cuda.synchronize()
        rep.fill_peers_from(rep.flat.clone(), call, n)
        (ref_out, ref_st), (got_out, got_st) = _both(rep, slot, rank, n)
        assert torch.equal(got_out.view(torch.int32), ref_out.view(torch.int32)), f"flat_out differs (call {call}, slot {slot})"
        assert torch.equal(got_st.view(torch.int64), ref_st.view(torch.int64)), f"layer_stats differ (call {call}, slot {slot})"
        assert float(ref_st.min()) > 0.0
        # and both equal the oracle's mean of the same buffers (bit for bit) and its statistics (fp64 rounding)
        reps = [p[:n].cpu().numpy() for p in rep.peers]
        reps.insert(rank, rep.flat[:n].cpu().numpy())
        mean_ref = oracle.mean(reps)
        assert np.array_equal(got_out.cpu().numpy().view(np.uint32), mean_ref.view(np.uint32))
        _, _, lid, lbeg = rep.ctx.ddp_slot_layout(slot)
        st = got_st.cpu().numpy()
        for i in range(len(lid)):
            g, m = oracle.layer_stats(reps, mean_ref, int(lbeg[i]), int(lbeg[i + 1]))
            assert st[2 * i] == pytest.approx(g, rel=1e-10) and st[2 * i + 1] == pytest.approx(m, rel=1e-10)
    # without statistics the scratch is not touched and the output is the same
    slot, n = big, sizes[big]
    rep.ctx.ddp_pack(slot, rep.flat)
    a, b = torch.empty_like(rep.flat), torch.empty_like(rep.flat)
    rep.ctx.ddp_partial_average(slot, rep.flat, rep.peers, w.n_replicas, 0, a, None)
    rep.ctx.ddp_partial_average_static(slot, rep.flat, rep.peers, w.n_replicas, 0, b, None)
    torch.cuda.synchronize()
    assert torch.equal(a[:n].view(torch.int32), b[:n].view(torch.int32))
    rep.close()


@pytest.mark.timeout(300)
def test_static_scratch_rejects_what_does_not_fit():
    assert torch.cuda.is_available(), "no GPU visible"
    # one tensor of 2^20 + 8 chunks of 1024 elements: its partial sums alone exceed the fixed array
    n = (B.DDP_STATIC_SCRATCH_BYTES // 16 + 8) * 1024
    buf = torch.zeros(n, dtype=torch.float32, device="cuda:0")
    out = torch.full((n,), 7.0, dtype=torch.float32, device="cuda:0")
    stats = torch.full((2,), -1.0, dtype=torch.float64, device="cuda:0")
    c = B.Context(0)
    c.ddp_set_option("mean_chunk", 1024)
    c.ddp_register_model(1, [0], [n], B.DDP_F32, B.DDP_F32, [buf], None, [buf], [buf], None)   # only the layout matters here
    c.ddp_set_schedule([0, 1], [0])
    with pytest.raises(B.DdpError) as e:
        c.ddp_partial_average_static(0, buf, None, 1, 0, out, stats)
    assert e.value.code == 2 and "fixed scratch" in str(e.value), str(e.value)
    torch.cuda.synchronize()
    assert float(out.min()) == 7.0 and float(stats.max()) == -1.0, "something was launched"
    c.ddp_partial_average_static(0, buf, None, 1, 0, out, None)            # no statistics: no scratch needed, any size passes
    torch.cuda.synchronize()
    assert float(out.abs().max()) == 0.0
    c.ddp_partial_average(0, buf, None, 1, 0, out, stats)                  # the allocating entry point takes the same slot
    torch.cuda.synchronize()
    assert stats.tolist() == [0.0, 0.0]
    c.close()
