"""Sec. 3.2 end to end on one GPU: a real torch model (its forward and backward are the user's, not the library's)
trains with its parameters and gradients living in the worker's arenas; autograd hooks launch each layer's fused
synchronisation + update on a side stream as soon as that layer's gradient exists.  The oracle worker is fed the very
gradients autograd produced and the same peer buffers; the state must agree bit for bit after every iteration."""
import numpy as np
import pytest
import torch

from paper_2502_11058_amd import workloads as W

pytestmark = pytest.mark.gpu

VOCAB, D, F, NB, T = 512, 128, 352, 3, 64


def _workload(n_replicas, period, policy):
    ts = [W.TensorSpec("embed", 0, VOCAB * D)]
    for b in range(NB):
        ts += [W.TensorSpec(f"block{b}.norm", 1 + b, D), W.TensorSpec(f"block{b}.up", 1 + b, D * F),
               W.TensorSpec(f"block{b}.down", 1 + b, F * D)]
    ts += [W.TensorSpec("norm", 1 + NB, D), W.TensorSpec("head", 1 + NB, VOCAB * D)]
    return W.Workload("hooked_mlp", ts, n_replicas=n_replicas, period=period, optimizer="adamw", param_dtype="bf16", lr=1e-3,
                      sigma_drift=1e-4, iterations=6, policy=policy)


def _rms(x, g):
    return x * torch.rsqrt(x.float().pow(2).mean(-1, keepdim=True) + 1e-5).to(x.dtype) * g


def _loss(p, tokens, targets):
    x = torch.nn.functional.embedding(tokens, p[0].view(VOCAB, D))
    for b in range(NB):
        g, up, down = p[1 + 3 * b], p[2 + 3 * b].view(D, F), p[3 + 3 * b].view(F, D)
        x = x + torch.nn.functional.silu(_rms(x, g) @ up) @ down
    logits = _rms(x, p[-2]) @ p[-1].view(VOCAB, D).t()
    return torch.nn.functional.cross_entropy(logits.float(), targets)


def _np(t):
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


@pytest.mark.parametrize("wire16,order,policy,side_cus", [(False, 0, "enp", 0), (True, 0, "round_robin", 0), (False, 1, "enp+fill", 0),
                                                          (False, 0, "enp", 32), (True, 1, "enp+fill", 64)])
def test_autograd_hooks_drive_the_layerwise_calls(oracle, wire16, order, policy, side_cus):
    # side_cus > 0: the chip is divided, the side stream on that many compute units, forward and backward on the others
    from paper_2502_11058_amd.harness import DeviceReplica
    from paper_2502_11058_amd.overlap import BackwardOverlap
    assert torch.cuda.is_available(), "no GPU visible: the HIP path cannot run (there is no CPU fallback)"
    w = _workload(4, 3, policy)
    rep = DeviceReplica(w, 0, wire16=wire16)
    rep.init_params()
    ov = BackwardOverlap(rep, side_cus=side_cus)
    hyper = dict(lr=w.lr, momentum=w.momentum, beta1=w.beta1, beta2=w.beta2, eps=w.eps, weight_decay=w.weight_decay)
    wk = oracle.Worker(rep.layer_of, [_np(t) for t in rep.sync], w.optimizer, hyper, True)
    gen = torch.Generator(device=rep.dev)
    gen.manual_seed(5)
    N, H = w.n_replicas, len(rep.sets)
    losses = []
    for r in range(w.iterations):
        S, rank = rep.sets[r % H], r % N
        off, order_t, total = oracle.slot_offsets(rep.layer_of, rep.numel, S)
        base = torch.cat([rep.sync[t] for t in order_t]) if total else rep.flat[:0]
        if wire16:
            rep.fill_peers16_from(base, r, total)
            peers_host = [_np(p[:total]) for p in rep.peers16]
        else:
            rep.fill_peers_from(base, r, total)
            peers_host = [_np(p[:total]) for p in rep.peers]
        tokens = torch.randint(0, VOCAB, (T,), device=rep.dev, generator=gen)
        targets = torch.randint(0, VOCAB, (T,), device=rep.dev, generator=gen)
        rep.stats.fill_(-1.0)
        torch.cuda.synchronize()            # the inputs above were produced on the default stream
        with torch.cuda.stream(ov.main_stream):
            ov.begin(r, local_rank=rank, wire16=wire16, order=order)
            loss = _loss(ov.params, tokens, targets)
            loss.backward()
            ov.end()
        torch.cuda.synchronize()
        losses.append(float(loss.detach()))
        # back-propagation finishes the output side first, and every layer got exactly one call
        assert ov.launch_order[0] == w.n_layers - 1 and sorted(ov.launch_order) == list(range(w.n_layers))
        grads = [_np(g) for g in rep.grad]
        assert any(np.any(g != 0) for g in grads)
        if order == 1:
            wk.local_update(grads, r + 1)
            _, ref_stats = wk.sync(S, peers_host, rank, wire16=wire16)
        else:
            _, ref_stats = wk.sync(S, peers_host, rank, wire16=wire16)
            wk.local_update(grads, r + 1)
        st = _np(rep.stats)
        for i, (g, m) in enumerate(ref_stats):
            assert st[2 * i] == pytest.approx(g, rel=1e-10, abs=1e-300) and st[2 * i + 1] == pytest.approx(m, rel=1e-10)
        for t in range(len(w.tensors)):
            assert np.array_equal(_np(rep.sync[t]).view(np.uint32), wk.p[t].view(np.uint32)), f"param r={r} t={t}"
            assert np.array_equal(_np(rep.s0[t]).view(np.uint32), wk.s0[t].view(np.uint32)), f"m r={r} t={t}"
            assert np.array_equal(_np(rep.s1[t]).view(np.uint32), wk.s1[t].view(np.uint32)), f"v r={r} t={t}"
            assert np.array_equal(_np(rep.model[t]), wk.model[t]), f"model copy r={r} t={t}"
    assert all(np.isfinite(losses))
    ov.close()
    rep.close()


def test_profiled_layer_times_feed_the_scheduler(oracle):
    """Sec. 3.2-3.3 as a loop: profile the per-layer backward times of the user's model, hand them (with communication
    times from the layers' wire bytes and an assumed bandwidth) to ddp_schedule, install the result at a period boundary
    and go on training.  The schedule must be the exhaustive optimum for the measured times, and the trajectory must stay
    bit-identical to the oracle's, which is told the same sets."""
    from paper_2502_11058_amd import binding as B
    from paper_2502_11058_amd.harness import DeviceReplica
    from paper_2502_11058_amd.overlap import BackwardOverlap
    assert torch.cuda.is_available(), "no GPU visible: the HIP path cannot run (there is no CPU fallback)"
    w = _workload(4, 3, "enp")
    L, H, N = w.n_layers, w.period, w.n_replicas
    rep = DeviceReplica(w, 0, flat_capacity=w.n_params)         # room for any schedule, even all layers in one slot
    rep.init_params()
    ov = BackwardOverlap(rep)
    hyper = dict(lr=w.lr, momentum=w.momentum, beta1=w.beta1, beta2=w.beta2, eps=w.eps, weight_decay=w.weight_decay)
    wk = oracle.Worker(rep.layer_of, [_np(t) for t in rep.sync], w.optimizer, hyper, True)
    gen = torch.Generator(device=rep.dev)
    gen.manual_seed(11)
    profiles = []

    def iteration(r, profile):
        S, rank = rep.sets[r % H], r % N
        off, order_t, total = oracle.slot_offsets(rep.layer_of, rep.numel, S)
        base = torch.cat([rep.sync[t] for t in order_t]) if total else rep.flat[:0]
        rep.fill_peers_from(base, r, total)
        peers_host = [_np(p[:total]) for p in rep.peers]
        tokens = torch.randint(0, VOCAB, (T,), device=rep.dev, generator=gen)
        targets = torch.randint(0, VOCAB, (T,), device=rep.dev, generator=gen)
        torch.cuda.synchronize()
        ov.begin(r, local_rank=rank, profile=profile)
        ov.backward(_loss(ov.params, tokens, targets))
        ov.end()
        torch.cuda.synchronize()
        if profile:
            profiles.append(ov.layer_bp_ns())
        wk.sync(S, peers_host, rank)
        wk.local_update([_np(g) for g in rep.grad], r + 1)
        for t in range(len(w.tensors)):
            assert np.array_equal(_np(rep.sync[t]).view(np.uint32), wk.p[t].view(np.uint32)), f"param r={r} t={t}"
            assert np.array_equal(_np(rep.s1[t]).view(np.uint32), wk.s1[t].view(np.uint32)), f"v r={r} t={t}"
            assert np.array_equal(_np(rep.model[t]), wk.model[t]), f"model copy r={r} t={t}"

    for r in range(H):                                           # the first period on the initial ENP schedule, profiled after a warm-up
        iteration(r, profile=r > 0)
    bp = np.median(np.asarray(profiles, dtype=np.int64), axis=0).astype(np.int64)
    assert bp.shape == (L,) and (bp > 0).all(), bp               # every layer took part and took time
    # communication: wire bytes of a layer over a bandwidth that makes the whole model cost two backward passes, so that the
    # optimum is neither "everything at once" nor trivial
    nbytes = np.asarray(rep.layer_wire_bytes(), dtype=np.float64)
    comm = np.rint(nbytes * (2.0 * bp.sum() / nbytes.sum())).astype(np.int64)
    _, sp, sl, cost = B.ddp_schedule("opt", L, H, None, bp, comm)
    sets = B.sets_from_csr(sp, sl)
    assert sets == oracle.schedule("opt", L, H, bp, comm)        # exhaustive search on the measured times
    assert cost <= B.ddp_schedule("enp", L, H, None, bp, comm)[3]
    rep.install_schedule(sp, sl)
    assert rep.sets == sets and sorted(l for S in sets for l in S) == list(range(L))
    for r in range(H, 3 * H):                                    # two more periods on the new schedule
        iteration(r, profile=False)
    ov.close()
    rep.close()
