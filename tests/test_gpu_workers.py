"""Algorithm 1 with K real workers: K replicas live in the one GPU's HBM, each with its own context, its own
gradients and its own drifting state; a worker's peers are the other workers' packed buffers of the same iteration
(device pointers, no synthetic drift).  Every worker is compared bit for bit with the oracle's K-worker run, and the
method's invariant is checked on the device: right after a layer is synchronised, all replicas hold the same bits."""
import numpy as np
import pytest
import torch

from paper_2502_11058_amd import binding as B
from paper_2502_11058_amd import workloads as W

pytestmark = pytest.mark.gpu


def _np(t):
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def _same_bits(a: np.ndarray, b: np.ndarray) -> bool:
    return a.dtype == b.dtype and a.shape == b.shape and a.tobytes() == b.tobytes()


def run_workers(oracle, w, K, iters, mode, order=0, wire16=False, policy=None):
    """mode: "calls" (pack, average, unpack, update) or "fused" (pack for the peers' sake, then one fused call)."""
    from paper_2502_11058_amd.harness import DeviceReplica
    assert torch.cuda.is_available(), "no GPU visible: the HIP path cannot run (there is no CPU fallback)"
    w.n_replicas = K
    reps = [DeviceReplica(w, 0, policy=policy, wire16=wire16, n_peers=0) for _ in range(K)]
    for rep in reps:
        rep.init_params()                                    # Algorithm 1: every worker starts from the same w_0
    sets, H = reps[0].sets, len(reps[0].sets)
    hyper = dict(lr=w.lr, momentum=w.momentum, beta1=w.beta1, beta2=w.beta2, eps=w.eps, weight_decay=w.weight_decay)
    wks = [oracle.Worker(rep.layer_of, [_np(t) for t in rep.sync], w.optimizer, hyper, rep.bf16) for rep in reps]
    outs = [torch.zeros_like(rep.flat) for rep in reps]
    agreed = np.zeros(w.n_layers, dtype=int)
    for r in range(iters):
        slot, S = r % H, sets[r % H]
        total = reps[0].slot_numel[slot]
        grads = []
        for k, rep in enumerate(reps):
            rep.fill_grads(r, worker=k)
            grads.append([_np(g) for g in rep.grad])
        if order == 1:
            for rep in reps:
                rep.ctx.ddp_local_update(rep.opt_struct(r + 1))
        # every worker puts its scheduled layers on the "wire"
        for rep in reps:
            if wire16:
                rep.ctx.ddp_pack_wire16(slot, rep.flat16)
            else:
                rep.ctx.ddp_pack(slot, rep.flat)
        wire = [rep.flat16 if wire16 else rep.flat for rep in reps]
        for k, rep in enumerate(reps):
            peers = [wire[j] for j in range(K) if j != k]
            rep.stats.fill_(-1.0)
            if mode == "fused":
                rep.ctx.ddp_fused_sync_update_layers(slot, 0, w.n_layers, peers, B.DDP_BF16 if wire16 else B.DDP_F32,
                                                     B.DDP_SYNC_THEN_UPDATE, K, k, rep.stats, rep.opt_struct(r + 1))
            elif wire16:
                rep.ctx.ddp_partial_average_wire16(slot, rep.flat16, peers, K, k, outs[k], rep.stats)
            else:
                rep.ctx.ddp_partial_average(slot, rep.flat, peers, K, k, outs[k], rep.stats)
        if mode == "calls":
            for k, rep in enumerate(reps):
                rep.ctx.ddp_unpack(slot, outs[k])
            torch.cuda.synchronize()
            # the invariant: every replica holds the same bits in the layers just synchronised, and only there
            # (the first synchronisation of a layer in sync-then-update order averages the common start: skip those)
            for l in range(w.n_layers):
                same = all(torch.equal(reps[0].sync[t].view(torch.int32), reps[k].sync[t].view(torch.int32))
                           for k in range(1, K) for t in range(len(w.tensors)) if reps[0].layer_of[t] == l)
                if l in S:
                    assert same, f"layer {l} differs between workers right after its synchronisation (r={r})"
                    agreed[l] += 1
                elif order == 1 or r >= 1:
                    assert not same, f"layer {l} was not synchronised at r={r} but the replicas agree"
            if order == 0:
                for rep in reps:
                    rep.ctx.ddp_local_update(rep.opt_struct(r + 1))
        torch.cuda.synchronize()
        # the oracle's K workers take the same iteration from their own state
        res = oracle.run_workers(wks, r, sets, grads, order=order, wire16=wire16)
        for k, rep in enumerate(reps):
            st = _np(rep.stats)
            for i, (g, m) in enumerate(res[k][1]):
                assert st[2 * i] == pytest.approx(g, rel=1e-10, abs=1e-300), f"gamma worker {k} r={r} layer {S[i]}"
                assert st[2 * i + 1] == pytest.approx(m, rel=1e-10), f"msq worker {k} r={r} layer {S[i]}"
            if mode == "calls" and total:
                assert _same_bits(_np(outs[k][:total]), res[k][0]), f"average worker {k} r={r}"
            for t in range(len(w.tensors)):
                assert _same_bits(_np(rep.sync[t]), wks[k].p[t]), f"param worker {k} r={r} t={t}"
                assert _same_bits(_np(rep.s0[t]), wks[k].s0[t]), f"state0 worker {k} r={r} t={t}"
                if rep.adam:
                    assert _same_bits(_np(rep.s1[t]), wks[k].s1[t]), f"state1 worker {k} r={r} t={t}"
                if rep.bf16:
                    assert _same_bits(_np(rep.model[t]), wks[k].model[t]), f"model worker {k} r={r} t={t}"
    for rep in reps:
        rep.close()
    return agreed


@pytest.mark.parametrize("order", [0, 1])
def test_four_tiny_workers_two_periods(oracle, order):
    w = W.tiny()
    agreed = run_workers(oracle, w, K=4, iters=2 * w.period, mode="calls", order=order)
    assert agreed.tolist() == [2] * w.n_layers            # Definition 1: every layer exactly once per period


@pytest.mark.parametrize("mode,wire16", [("calls", False), ("fused", False), ("calls", True), ("fused", True)])
def test_llama_shaped_workers(oracle, mode, wire16):
    w = W.small_llama(n_replicas=3, period=3)
    run_workers(oracle, w, K=3, iters=7, mode=mode, wire16=wire16)


def test_eight_workers_update_then_sync_with_bubble_filling(oracle):
    w = W.small_llama(n_blocks=6, n_replicas=8, period=4)
    agreed = run_workers(oracle, w, K=8, iters=8, mode="calls", order=1, policy="enp+fill")
    assert agreed.min() >= 2                              # filled layers are synchronised more than once per period


def test_two_contexts_on_two_streams_do_not_interfere():
    # contexts own their tables and reduction scratch: two workers stepping at the same time on their own streams
    # end with the bits they get when they run one after the other
    from paper_2502_11058_amd.harness import DeviceReplica
    assert torch.cuda.is_available(), "no GPU visible: the HIP path cannot run (there is no CPU fallback)"
    w = W.small_llama(n_replicas=4, period=2)

    def make(worker):
        rep = DeviceReplica(w, 0)
        rep.init_params()
        rep.ctx.ddp_pack(0, rep.flat)
        torch.cuda.synchronize()
        rep.fill_peers_from(rep.flat, worker, rep.flat.numel())
        return rep

    together = [make(0), make(1)]
    apart = [make(0), make(1)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for r in range(6):
        for k in range(2):
            together[k].fill_grads(r, worker=k)
            apart[k].fill_grads(r, worker=k)
        torch.cuda.synchronize()
        for k in range(2):                                   # both in flight at once, fused and four-call alternating
            with torch.cuda.stream(streams[k]):
                (together[k].fused_step if (r + k) % 2 else together[k].step)(r, local_rank=k, stream=streams[k])
        for k in range(2):
            (apart[k].fused_step if (r + k) % 2 else apart[k].step)(r, local_rank=k)
            torch.cuda.synchronize()
        torch.cuda.synchronize()
        for k in range(2):
            for x, y in ((together[k].a_sync, apart[k].a_sync), (together[k].a_s0, apart[k].a_s0), (together[k].a_s1, apart[k].a_s1)):
                assert torch.equal(x.view(torch.int32), y.view(torch.int32)), f"worker {k} r={r}"
            assert torch.equal(together[k].a_model.view(torch.int16), apart[k].a_model.view(torch.int16))
            assert torch.equal(together[k].stats, apart[k].stats)
    for rep in together + apart:
        rep.close()
