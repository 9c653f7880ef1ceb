"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration bench.py times.

TinyLlama-1.1B: two whole periods, every element of every stage, against the oracle (default order and fp32 wire; and
two iterations through the fused entry point with bf16 on the wire in the update-then-sync order), plus 16 iterations
with a million carried samples.
Llama-2-7B and Llama-3-8B (N = 16, ragged schedule): every element of one full iteration against the oracle, streamed
layer by layer through the host (run_all_elements), and whole trajectories (8 iterations) with ~1.1 M sampled parameters
carried by the oracle (random positions plus every tensor boundary and chunk boundaries), where on top every element of
pack, average and unpack is checked on the device against independent gathers / sequential torch sums (those stages are
exact, so they must agree bit for bit at any size).
Edge shapes at full size: the whole 7B model in one slot, and a single tensor of more than 2^31 elements.
"""
import gc

import numpy as np
import pytest
import torch

from paper_2502_11058_amd import workloads as W
from test_gpu_parity import Tally, _bits, _need_gpu, _np, assert_bf16_within_one_ulp, assert_close_fp32, progress, run_trajectory

pytestmark = pytest.mark.gpu


@pytest.mark.timeout(1500)
def test_tinyllama_full_trajectory(oracle):
    # every element of every stage against the oracle, two full periods (H = 4: every slot twice, the second time with
    # optimizer state and drifted parameters behind it); the CPU oracle is the slow side here, the 16-iteration horizon
    # is covered by the sampled run below
    t = run_trajectory(oracle, W.tinyllama_1b(), iters=8, check_every=4)
    assert t.frac() == 1.0


@pytest.mark.timeout(900)
def test_tinyllama_bf16_wire_update_then_sync_every_element(oracle):
    # the other branch of every choice the step has, at 1.1 G parameters, every element against the oracle: the fused
    # entry point, bf16 on the wire, and Eq. (5)'s printed order (optimizer step first, then the average)
    t = run_trajectory(oracle, W.tinyllama_1b(), iters=2, check_every=2, fused=True, wire16=True, order=1)
    assert t.frac() == 1.0


@pytest.mark.timeout(900)
def test_tinyllama_sampled_16_iterations(oracle):
    # four periods with a million carried samples: the update's tolerance is stated after 16 iterations
    assert run_sampled(oracle, W.tinyllama_1b(), iters=16) == 1.0


def _sample_positions(rep, n_random, seed):
    P = int(rep.offsets[-1] - rep.offsets[0])
    rng = np.random.default_rng(seed)
    pos = [rng.integers(0, P, n_random, dtype=np.int64)]
    starts = rep.offsets[:-1] - rep.offsets[0]
    for d in range(-4, 5):                                   # both sides of every tensor boundary
        pos.append(np.clip(starts + d, 0, P - 1))
    big = np.argsort(rep.numel)[-6:]                          # chunk boundaries inside the largest tensors
    for t in big:
        k = rng.integers(1, max(2, rep.numel[t] // 8192), 64)
        for d in range(-2, 3):
            pos.append(np.clip(starts[t] + k * 8192 + d, 0, P - 1))
    pos.append(np.array([0, 1, 2, 3, P - 4, P - 3, P - 2, P - 1]))
    return np.unique(np.concatenate(pos)) + int(rep.offsets[0])


def run_sampled(oracle, w, iters, n_random=1 << 20, stats_layer_cap=260_000_000, fused=False, wire16=False, placement=None,
                layerwise=0):
    from paper_2502_11058_amd.harness import DeviceReplica
    _need_gpu()
    oracle.set_threads(16)
    gc.collect()
    torch.cuda.empty_cache()
    free, total_mem = torch.cuda.mem_get_info()
    progress(f"[{w.name}] HBM free {free / 1e9:.1f} GB of {total_mem / 1e9:.1f} GB")
    rep = DeviceReplica(w, 0, wire16=wire16, placement_probe=placement)
    if placement:
        progress(f"[{w.name}] placement {rep.placement}")
    rep.init_params()
    N, H = w.n_replicas, w.period
    dev = rep.dev
    o_mean, o_stats = (oracle.mean_wire16, oracle.layer_stats_wire16) if wire16 else (oracle.mean, oracle.layer_stats)
    gi_host = _sample_positions(rep, n_random, 7)
    gi = torch.from_numpy(gi_host).to(dev)
    tensor_of = np.searchsorted(rep.offsets, gi_host, side="right") - 1
    p_s = _np(rep.a_sync[gi])
    m_s, v_s = np.zeros_like(p_s), np.zeros_like(p_s)
    model_s = oracle.bf16_rne(p_s)
    assert np.array_equal(_np(rep.a_model[gi]), model_s)
    inv_n = torch.tensor(1.0 / N, dtype=torch.float32, device=dev)
    n_exact = n_total = 0
    side = torch.cuda.Stream() if layerwise else None

    for r in range(iters):
        slot, S, rank = r % H, rep.sets[r % H], r % N
        off, order_t, total = oracle.slot_offsets(rep.layer_of, rep.numel, S)
        tid, toff, lid, lbeg = rep.ctx.ddp_slot_layout(slot)
        assert rep.ctx.ddp_slot_numel(slot) == total and tid.tolist() == order_t.tolist()
        assert toff.tolist() == [int(off[t]) for t in order_t] and lid.tolist() == list(S)
        # which samples are scheduled, and where they sit in the flat buffer
        sel_host = off[tensor_of] >= 0
        fi_host = (off[tensor_of] + (gi_host - rep.offsets[tensor_of]))[sel_host]
        fi, gsel = torch.from_numpy(fi_host).to(dev), torch.from_numpy(gi_host[sel_host]).to(dev)
        rep.fill_grads(r)
        g_s = _np(rep.a_grad[gi])
        if total == 0:
            # an empty slot (FULL schedule outside its one iteration): the calls are no-ops, only the update acts
            rep.stats.fill_(-1.0)
            if fused:
                rep.fused_step(r, rank, wire16=wire16)
            else:
                rep.step(r, rank, wire16=wire16)
            oracle.adamw(p_s, g_s, m_s, v_s, model_s, w.lr, w.beta1, w.beta2, w.eps, w.weight_decay, r + 1)
            gp, gm, gv = _np(rep.a_sync[gi]), _np(rep.a_s0[gi]), _np(rep.a_s1[gi])
            assert float(rep.stats.max()) == -1.0, "statistics written for an empty slot"
            for a_, b_, what in ((gp, p_s, "param"), (gm, m_s, "m"), (gv, v_s, "v")):
                assert np.array_equal(_bits(a_), _bits(b_)), f"{what} r={r} (empty slot)"
                n_total += a_.size
                n_exact += a_.size
            assert np.array_equal(_np(rep.a_model[gi]), model_s), f"model r={r} (empty slot)"
            progress(f"[{w.name}] r={r} slot {slot} is empty: update only, ok")
            continue
        base = torch.cat([rep.sync[t] for t in order_t])       # independent gather (harness), the peers' base
        if wire16:
            rep.fill_peers16_from(base, r, total)
        else:
            rep.fill_peers_from(base, r, total)
        wire = rep.peers16 if wire16 else rep.peers                      # what the peers put on the wire ...
        local = (lambda x: oracle.bf16_rne(_np(x))) if wire16 else _np   # ... and what the local replica contributes
        if fused or wire16:
            # the end state and the statistics; with the four bf16 calls also every element of pack and average
            x_s = [_np(p[fi]) for p in wire]
            reps_s = x_s[:rank] + [local(base[fi])] + x_s[rank:]
            mean_s = o_mean(reps_s)
            unsched_before = None
            i = int(np.argmin([int(lbeg[j + 1] - lbeg[j]) for j in range(len(S))]))
            b, e = int(lbeg[i]), int(lbeg[i + 1])
            layer_reps = None
            if e - b <= stats_layer_cap:
                xs = [_np(p[b:e]) for p in wire]
                layer_reps = xs[:rank] + [local(base[b:e])] + xs[rank:]
            rep.stats.fill_(-1.0)
            if fused:
                del base
                if layerwise:
                    # buckets of layers on a side stream, the way a backward pass would release them (gradients are
                    # already in place here, so the "backward" of a layer is empty)
                    rep.layerwise_step(r, side, backward=lambda l: None, bucket=layerwise, local_rank=rank, wire16=wire16)
                elif wire16:
                    rep.ctx.ddp_fused_sync_update_wire16(slot, rep.peers16, N, rank, rep.stats, rep.opt_struct(r + 1))
                else:
                    rep.ctx.ddp_fused_sync_update(slot, rep.peers, N, rank, rep.stats, rep.opt_struct(r + 1))
            else:
                rep.flat16.view(torch.int16).fill_(-1)
                rep.ctx.ddp_pack_wire16(slot, rep.flat16)
                step_n = 1 << 28
                for b0 in range(0, total, step_n):      # torch's fp32 -> bf16 cast is round-to-nearest-even as well
                    e0 = min(total, b0 + step_n)
                    assert torch.equal(rep.flat16[b0:e0].view(torch.int16), base[b0:e0].to(torch.bfloat16).view(torch.int16)), f"pack16 r={r} at {b0}"
                assert np.array_equal(_np(rep.flat16[fi]), local(base[fi])), f"pack16 (oracle samples) r={r}"
                del base
                rep.ctx.ddp_partial_average_wire16(slot, rep.flat16, rep.peers16, N, rank, rep.flat, rep.stats)
                seq = rep.peers16[:rank] + [rep.flat16] + rep.peers16[rank:]
                for b0 in range(0, total, step_n):      # widening is exact: an independent fp32 sum of every element
                    e0 = min(total, b0 + step_n)
                    acc = seq[0][b0:e0].float()
                    for k in range(1, N):
                        acc.add_(seq[k][b0:e0].float())
                    acc.mul_(inv_n)
                    assert torch.equal(rep.flat[b0:e0].view(torch.int32), acc.view(torch.int32)), f"mean16 (all elements) r={r} at {b0}"
                del acc, seq
                assert np.array_equal(_bits(_np(rep.flat[fi])), _bits(mean_s)), f"mean16 (oracle samples) r={r}"
                rep.ctx.ddp_unpack(slot, rep.flat)
                rep.ctx.ddp_local_update(rep.opt_struct(r + 1))
            if layer_reps is not None:
                st = _np(rep.stats)
                g, m = o_stats(layer_reps, o_mean(layer_reps), 0, e - b)
                assert st[2 * i] == pytest.approx(g, rel=1e-10), f"fused gamma r={r} layer {S[i]}"
                assert st[2 * i + 1] == pytest.approx(m, rel=1e-10), f"fused msq r={r} layer {S[i]}"
                del layer_reps, xs
            p_s[sel_host] = mean_s
            model_s[sel_host] = oracle.bf16_rne(mean_s)
            oracle.adamw(p_s, g_s, m_s, v_s, model_s, w.lr, w.beta1, w.beta2, w.eps, w.weight_decay, r + 1)
            gp, gm, gv = _np(rep.a_sync[gi]), _np(rep.a_s0[gi]), _np(rep.a_s1[gi])
            assert_close_fp32(gp, p_s, f"fused param r={r}", 1e-9)
            assert_close_fp32(gm, m_s, f"fused m r={r}", 1e-12)
            assert_close_fp32(gv, v_s, f"fused v r={r}", 1e-16)
            assert_bf16_within_one_ulp(_np(rep.a_model[gi]), model_s, f"fused model r={r}")
            for a_, b_ in ((gp, p_s), (gm, m_s), (gv, v_s)):
                n_total += a_.size
                n_exact += int((_bits(a_) == _bits(b_)).sum())
            progress(f"[{w.name}] fused r={r} slot {slot} ({total} elements) ok")
            continue
        # pack: every element against the gather
        rep.flat.fill_(float("nan"))
        rep.ctx.ddp_pack(slot, rep.flat)
        assert torch.equal(rep.flat[:total].view(torch.int32), base.view(torch.int32)), f"pack r={r}"
        x_s = [_np(p[fi]) for p in rep.peers]
        loc_s = _np(base[fi])
        reps_s = x_s[:rank] + [loc_s] + x_s[rank:]
        rep.stats.fill_(-1.0)
        rep.ctx.ddp_partial_average(slot, rep.flat, rep.peers, N, rank, rep.flat, rep.stats)
        # sequential torch sum in rank order, piecewise: an independent fp32 evaluation of every element
        seq = rep.peers[:rank] + [base] + rep.peers[rank:]
        step_n = 1 << 28
        for b0 in range(0, total, step_n):
            e0 = min(total, b0 + step_n)
            acc = seq[0][b0:e0].clone()
            for k in range(1, N):
                acc.add_(seq[k][b0:e0])
            acc.mul_(inv_n)
            assert torch.equal(rep.flat[b0:e0].view(torch.int32), acc.view(torch.int32)), f"mean (all elements) r={r} at {b0}"
        del base, seq, acc
        mean_s = oracle.mean(reps_s)
        assert np.array_equal(_bits(_np(rep.flat[fi])), _bits(mean_s)), f"mean (oracle samples) r={r}"
        # statistics: the oracle on one whole layer, a device-side fp64 evaluation on all layers
        st = _np(rep.stats)
        sizes = [int(lbeg[i + 1] - lbeg[i]) for i in range(len(S))]
        for i in range(len(S)):
            b, e = int(lbeg[i]), int(lbeg[i + 1])
            g64 = torch.zeros((), dtype=torch.float64, device=dev)
            for k in range(N):
                if k != rank:
                    xk = rep.peers[k - (k > rank)][b:e]
                else:       # averaged in place: the local values are still in the model tensors until unpack
                    xk = torch.cat([rep.sync[t] for t in order_t if rep.layer_of[t] == S[i]])
                d = (rep.flat[b:e] - xk).double()
                g64 += (d * d).sum()
            m64 = (rep.flat[b:e].double() ** 2).sum()
            assert st[2 * i] == pytest.approx(float(g64) / N, rel=1e-9), f"gamma (device fp64) r={r} layer {S[i]}"
            assert st[2 * i + 1] == pytest.approx(float(m64), rel=1e-9), f"msq (device fp64) r={r} layer {S[i]}"
        i = int(np.argmin(sizes))
        if sizes[i] <= stats_layer_cap:
            b, e = int(lbeg[i]), int(lbeg[i + 1])
            loc = _np(torch.cat([rep.sync[t] for t in order_t if rep.layer_of[t] == S[i]]))
            xs = [_np(p[b:e]) for p in rep.peers]
            layer_reps = xs[:rank] + [loc] + xs[rank:]
            g, m = oracle.layer_stats(layer_reps, _np(rep.flat[b:e]), 0, e - b)
            assert st[2 * i] == pytest.approx(g, rel=1e-10), f"gamma (oracle) r={r} layer {S[i]}"
            assert st[2 * i + 1] == pytest.approx(m, rel=1e-10), f"msq (oracle) r={r} layer {S[i]}"
            del loc, xs, layer_reps
        # unpack: every scheduled tensor equals its flat range, its model copy the bf16 rounding; others untouched
        unsched_before = _np(rep.a_sync[gi])[~sel_host]
        rep.ctx.ddp_unpack(slot, rep.flat)
        for t in order_t:
            assert torch.equal(rep.sync[t].view(torch.int32), rep.flat[int(off[t]): int(off[t]) + rep.numel[t]].view(torch.int32)), f"unpack r={r} t={t}"
        assert torch.equal(rep.a_model[gsel].view(torch.int16).cpu(), torch.from_numpy(oracle.bf16_rne(mean_s).view(np.int16))), f"model copy r={r}"
        assert np.array_equal(_bits(_np(rep.a_sync[gi])[~sel_host]), _bits(unsched_before)), f"unscheduled tensors moved r={r}"
        # the oracle's carried samples take the same step
        p_s[sel_host] = mean_s
        model_s[sel_host] = oracle.bf16_rne(mean_s)
        rep.ctx.ddp_local_update(rep.opt_struct(r + 1))
        oracle.adamw(p_s, g_s, m_s, v_s, model_s, w.lr, w.beta1, w.beta2, w.eps, w.weight_decay, r + 1)
        gp, gm, gv = _np(rep.a_sync[gi]), _np(rep.a_s0[gi]), _np(rep.a_s1[gi])
        assert_close_fp32(gp, p_s, f"param r={r}", 1e-9)
        assert_close_fp32(gm, m_s, f"m r={r}", 1e-12)
        assert_close_fp32(gv, v_s, f"v r={r}", 1e-16)
        assert_bf16_within_one_ulp(_np(rep.a_model[gi]), model_s, f"model r={r}")
        for a, b_ in ((gp, p_s), (gm, m_s), (gv, v_s)):
            n_total += a.size
            n_exact += int((_bits(a) == _bits(b_)).sum())
        progress(f"[{w.name}] r={r} slot {slot} ({total} elements, {len(S)} layers) ok")
    progress(f"[{w.name}] {gi_host.size} sampled parameters, optimizer state bit-identical in {100.0 * n_exact / n_total:.4f}%")
    rep.close()
    return n_exact / n_total


@pytest.mark.timeout(1500)
def test_llama2_7b_sampled_trajectory(oracle):
    # the slab placed the way bench.py places it (placement search, front pad), default launch options
    assert run_sampled(oracle, W.llama2_7b(), iters=8, placement="search") == 1.0


@pytest.mark.timeout(1500)
def test_llama2_7b_fused_sampled_trajectory(oracle):
    assert run_sampled(oracle, W.llama2_7b(), iters=8, fused=True) == 1.0


@pytest.mark.timeout(1500)
def test_llama2_7b_layerwise_fused_sampled_trajectory(oracle):
    # the fused step as 12 launches of three layers each on a side stream (Sec. 3.2 granularity) instead of one call
    assert run_sampled(oracle, W.llama2_7b(), iters=4, fused=True, layerwise=3) == 1.0


@pytest.mark.timeout(1500)
@pytest.mark.parametrize("fused", [False, True])
def test_llama2_7b_bf16_wire_sampled_trajectory(oracle, fused):
    assert run_sampled(oracle, W.llama2_7b(), iters=4, fused=fused, wire16=True) == 1.0


@pytest.mark.timeout(1500)
@pytest.mark.parametrize("fused", [False, True])
def test_llama2_7b_whole_model_in_one_slot(oracle, fused):
    # Eq. (2) at full size: FULL schedule with H = 2 and N = 2, so the second iteration synchronises all 6.7 G
    # parameters in one slot: flat offsets beyond 2^31 elements and 2^34 bytes, 6.6 M chunks per launch
    w = W.llama2_7b()
    w.n_replicas, w.period, w.policy = 2, 2, "full"
    assert run_sampled(oracle, w, iters=2, fused=fused) == 1.0


@pytest.mark.timeout(1500)
def test_llama3_8b_ragged_schedule_sampled_trajectory(oracle):
    w = W.llama3_8b()
    _need_gpu()
    gc.collect()
    torch.cuda.empty_cache()
    free, total = torch.cuda.mem_get_info()
    # state 16 B/param, flat + 15 peers + the gathered base of the largest slot (1.834 G elements), 2 % slack
    need = (16 * w.n_params + 4 * 17 * 1_834_000_000 + (3 << 30)) * 1.02
    if free < need:
        pytest.skip(f"needs {need / 1e9:.0f} GB of free HBM, {free / 1e9:.0f} GB available")
    assert run_sampled(oracle, w, iters=8) == 1.0


# ----------------------------------------------------------------------------------------------------------------
# every element of one full-size iteration against the oracle, streamed layer by layer
# ----------------------------------------------------------------------------------------------------------------

class _Stager:
    """Device -> host copies through two small pinned buffers, double-buffered: the copy of one piece runs while the
    previous piece is moved into ordinary (pageable) host memory.  Only 512 MiB are ever pinned, and they are released
    at the end: pinning the whole host copy (100 GB and more, which torch's host allocator then keeps cached for the
    life of the process) leaves the GPU runtime without pinnable memory for its own queues and signals."""
    PIECE = 256 << 20

    def __init__(self):
        try:
            self.bufs = [torch.empty(self.PIECE, dtype=torch.uint8, pin_memory=True) for _ in range(2)]
        except RuntimeError:
            self.bufs = [torch.empty(self.PIECE, dtype=torch.uint8) for _ in range(2)]
        self.done = [torch.cuda.Event(), torch.cuda.Event()]

    def fetch(self, t: torch.Tensor) -> np.ndarray:
        src = t.contiguous().view(torch.uint8)
        n = src.numel()
        out = np.empty(n, dtype=np.uint8)
        pieces = [(o, min(self.PIECE, n - o)) for o in range(0, n, self.PIECE)]

        def take(k):
            o, l = pieces[k]
            self.done[k % 2].synchronize()
            out[o:o + l] = self.bufs[k % 2][:l].numpy()

        for k, (o, l) in enumerate(pieces):
            self.bufs[k % 2][:l].copy_(src[o:o + l], non_blocking=True)      # its previous content was taken in round k - 1
            self.done[k % 2].record()
            if k >= 1:
                take(k - 1)
        if pieces:
            take(len(pieces) - 1)
        dt = {torch.float32: np.float32, torch.bfloat16: np.uint16, torch.float64: np.float64}[t.dtype]
        return out.view(dt)

    def release(self):
        torch.cuda.synchronize()
        self.bufs = []
        gc.collect()
        if hasattr(torch._C, "_host_emptyCache"):
            torch._C._host_emptyCache()


def run_all_elements(oracle, w, warm=2, placement=None, stats_layer_cap=260_000_000, both_paths=True):
    """One iteration at full size in bench.py's launch configuration, EVERY element of its result against the oracle.

    After `warm` iterations through the GPU path (so that the optimizer state is what a run holds, not zeros) the state
    before iteration r = warm is copied to the host layer by layer, the GPU takes the step over the whole model in its
    usual launches, and then the oracle takes the same step one layer at a time on the host copy - pack, rank-order
    mean with that layer's range of the peer buffers, statistics, unpack, optimizer - and all of the layer's parameters,
    moments and bf16 model copy are compared with what the GPU holds, bit for bit.  The oracle never sees a value the
    GPU path computed in this iteration.

    both_paths: replica A takes the four calls and a second replica B, seeded and warmed identically, takes the fused entry
    point with A's peer buffers.  A is compared with the oracle as described; B is compared with A on the device, every
    element of parameters, moments and model copy bit for bit (and its statistics with the oracle's), which makes B
    equal to the oracle on every element as well without a second pass over the host.  Otherwise (the model is too
    large for two replicas) the one replica takes the fused entry point."""
    import time
    from paper_2502_11058_amd.harness import DeviceReplica
    _need_gpu()
    oracle.set_threads(16)
    gc.collect()
    torch.cuda.empty_cache()
    clock = {"host copy": 0.0, "oracle": 0.0, "compare": 0.0}
    stager = _Stager()
    _to_host = stager.fetch
    t_start = time.perf_counter()
    A = DeviceReplica(w, 0, placement_probe=placement)
    A.init_params()
    Bf = None
    if both_paths:
        Bf = DeviceReplica(w, 0, placement_probe=False, n_peers=0)
        Bf.init_params()
    N, H, L = w.n_replicas, w.period, w.n_layers
    hyper = dict(lr=w.lr, momentum=w.momentum, beta1=w.beta1, beta2=w.beta2, eps=w.eps, weight_decay=w.weight_decay)
    fused_only = not both_paths

    def stage(r):
        """Inputs of iteration r: fresh gradients, peers = an independent gather of the slot's tensors + drift."""
        S = A.sets[r % H]
        off, order_t, total = oracle.slot_offsets(A.layer_of, A.numel, S)
        assert A.ctx.ddp_slot_numel(r % H) == total
        A.fill_grads(r)
        if Bf is not None:
            Bf.a_grad.copy_(A.a_grad)
        if total:
            base = torch.cat([A.sync[t] for t in order_t])
            A.fill_peers_from(base, r, total)
            del base
        return S, total

    def gpu_step(r, rank):
        if fused_only:
            A.fused_step(r, rank)
        else:
            A.step(r, rank)
        if Bf is not None:
            Bf.ctx.ddp_fused_sync_update(r % H, A.peers, N, rank, Bf.stats, Bf.opt_struct(r + 1))

    for r in range(warm):
        stage(r)
        gpu_step(r, r % N)
    r = warm
    rank = r % N
    S, total = stage(r)
    assert total > 0, "pick an iteration whose slot is not empty"
    tid, toff, lid, lbeg = A.ctx.ddp_slot_layout(r % H)
    assert lid.tolist() == list(S)
    torch.cuda.synchronize()
    if Bf is not None:      # the two replicas have taken the warm-up iterations through different entry points
        for x, y in ((A.a_sync, Bf.a_sync), (A.a_s0, Bf.a_s0), (A.a_s1, Bf.a_s1), (A.a_model, Bf.a_model)):
            assert torch.equal(x.view(torch.int16), y.view(torch.int16)), "four calls and fused entry point differ after the warm-up"

    # element range of every layer in the arenas (tensors lie back to back in registration order)
    first = [None] * L
    last = [None] * L
    for t, l in enumerate(A.layer_of):
        first[l] = t if first[l] is None else first[l]
        last[l] = t
    rng = [(int(A.offsets[first[l]]), int(A.offsets[last[l]]) + A.numel[last[l]]) for l in range(L)]

    t0 = time.perf_counter()
    before = {}
    for l in range(L):
        lo, hi = rng[l]
        before[l] = tuple(_to_host(a[lo:hi]) for a in (A.a_sync, A.a_s0, A.a_s1, A.a_grad))
    clock["host copy"] += time.perf_counter() - t0
    progress(f"[{w.name}] state before iteration {r} on the host ({sum(x.nbytes for b in before.values() for x in b) / 1e9:.0f} GB, "
             f"{time.perf_counter() - t0:.0f} s)")
    A.stats.fill_(-1.0)
    if Bf is not None:
        Bf.stats.fill_(-1.0)
    gpu_step(r, rank)
    torch.cuda.synchronize()
    stats = _np(A.stats)
    if Bf is not None:
        stats_b = _np(Bf.stats)
        t0 = time.perf_counter()
        for x, y, what in ((A.a_sync, Bf.a_sync, "param"), (A.a_s0, Bf.a_s0, "m"), (A.a_s1, Bf.a_s1, "v"), (A.a_model, Bf.a_model, "model copy")):
            assert torch.equal(x.view(torch.int16), y.view(torch.int16)), f"fused entry point: {what} differs from the four calls"
        clock["compare"] += time.perf_counter() - t0
    n_exact = n_total = n_model = 0
    for l in range(L):
        lo, hi = rng[l]
        p0, m0, v0, g = before.pop(l)
        ts = list(range(first[l], last[l] + 1))
        cuts = np.cumsum([0] + [A.numel[t] for t in ts])
        split = lambda a: [a[cuts[j]:cuts[j + 1]] for j in range(len(ts))]
        t0 = time.perf_counter()
        # the oracle's worker on this layer, working in place on the host copy of the state the run holds
        wk = oracle.Worker([0] * len(ts), [np.zeros(1, dtype=np.float32)] * len(ts), w.optimizer, hyper, False)
        wk.p, wk.numel, wk.s0, wk.s1 = split(p0), [A.numel[t] for t in ts], split(m0), split(v0)
        model_ref = np.empty(hi - lo, dtype=np.uint16)
        wk.model = split(model_ref)                                           # written by unpack and by the update
        clock["oracle"] += time.perf_counter() - t0
        if l in S:
            i = list(S).index(l)
            b, e = int(lbeg[i]), int(lbeg[i + 1])
            assert e - b == hi - lo
            t0 = time.perf_counter()
            peers = [_to_host(x[b:e]) for x in A.peers]
            clock["host copy"] += time.perf_counter() - t0
            t0 = time.perf_counter()
            if e - b <= stats_layer_cap:
                mean_ref, st_ref = wk.sync([0], peers, rank)
            else:      # the oracle's statistics loop is serial: on the largest layers only the mean is taken
                flat, off_l, order_l, _ = wk.pack_slot([0])
                mean_ref, st_ref = oracle.mean(list(peers[:rank]) + [flat] + list(peers[rank:])), None
                wk.unpack_slot(mean_ref, off_l, order_l)
            clock["oracle"] += time.perf_counter() - t0
            if not fused_only:                                                 # the four-call path leaves the mean in the flat buffer
                assert np.array_equal(_bits(_to_host(A.flat[b:e])), _bits(mean_ref)), f"mean of layer {l}"
            if st_ref is not None:
                for sv in ((stats,) if Bf is None else (stats, stats_b)):
                    assert sv[2 * i] == pytest.approx(st_ref[0][0], rel=1e-10), f"gamma of layer {l}"
                    assert sv[2 * i + 1] == pytest.approx(st_ref[0][1], rel=1e-10), f"mean norm of layer {l}"
            del peers, mean_ref
        t0 = time.perf_counter()
        wk.local_update(split(g), r + 1)
        clock["oracle"] += time.perf_counter() - t0
        for name, arena, ref, atol in (("param", A.a_sync, p0, 1e-9), ("m", A.a_s0, m0, 1e-12), ("v", A.a_s1, v0, 1e-16)):
            t0 = time.perf_counter()
            got = _to_host(arena[lo:hi])
            clock["host copy"] += time.perf_counter() - t0
            t0 = time.perf_counter()
            n_total += got.size
            if np.array_equal(_bits(got), _bits(ref)):
                n_exact += got.size
            else:
                assert_close_fp32(got, ref, f"{name} of layer {l}", atol)      # the benchmark spec's bar ...
                n_exact += int((_bits(got) == _bits(ref)).sum())               # ... and how many are the same bits
            clock["compare"] += time.perf_counter() - t0
        got = _to_host(A.a_model[lo:hi])
        assert np.array_equal(got, model_ref), f"model copy of layer {l}"
        n_model += got.size
        del wk, p0, m0, v0, g, got, model_ref
        if l % 8 == 0 or l == L - 1:
            progress(f"[{w.name}] r={r}: layers 0..{l} compared, every element ({time.perf_counter() - t_start:.0f} s; "
                     + ", ".join(f"{k} {v:.0f} s" for k, v in clock.items()) + ")")
    assert n_total == 3 * w.n_params and n_model == w.n_params
    progress(f"[{w.name}] {'fused' if fused_only else 'four calls' + (' and fused' if Bf is not None else '')}: "
             f"{n_total + n_model} values compared with the oracle, {100.0 * n_exact / n_total:.6f}% bit-identical")
    stager.release()
    A.close()
    if Bf is not None:
        Bf.close()
    return n_exact / n_total


@pytest.mark.timeout(900)
def test_llama2_7b_every_element_of_one_iteration(oracle):
    # both replicas allocated the way bench.py allocates its timed one (first allocation, no placement search);
    # iteration 2 synchronises slot 2 (four blocks)
    assert run_all_elements(oracle, W.llama2_7b(), warm=2, placement=False, both_paths=True) == 1.0


@pytest.mark.timeout(900)
def test_llama3_8b_every_element_of_one_iteration(oracle):
    assert run_all_elements(oracle, W.llama3_8b(), warm=2, placement=False, both_paths=False) == 1.0


@pytest.mark.timeout(600)
@pytest.mark.parametrize("dense_path", [1, 0])
def test_single_tensor_beyond_2_31_elements(oracle, dense_path):
    """One tensor of 2^31 + 4099 fp32 elements (an embedding of a very large model has that many): element indices inside
    a tensor, chunk starts and flat offsets all pass 2^31.  Four calls and then the fused entry point, table-free and
    table-driven; every element against independent device-side evaluations (exact for pack / average / unpack, and
    for SGD-momentum written as separate torch operations), samples against the oracle."""
    from paper_2502_11058_amd.harness import DeviceReplica
    _need_gpu()
    gc.collect()
    torch.cuda.empty_cache()
    big = (1 << 31) + 4099
    ts = [W.TensorSpec("small.w", 0, 1000), W.TensorSpec("huge.w", 1, big), W.TensorSpec("huge.b", 1, 3)]
    w = W.Workload("huge_tensor", ts, n_replicas=2, period=2, optimizer="sgdm", param_dtype="f32", lr=0.01, momentum=0.9,
                   sigma_drift=1e-3, sigma_grad=1e-2, iterations=2, policy="round_robin")
    rep = DeviceReplica(w, 0, options={"dense_path": dense_path}, placement_probe=False)
    rep.init_params()
    dev = rep.dev
    P = w.n_params
    rng = np.random.default_rng(3)
    gi_host = np.unique(np.concatenate([rng.integers(0, P, 200_000), np.arange(0, 2000), np.arange(P - 2000, P),
                                        np.arange((1 << 31) - 3000, min(P, (1 << 31) + 6000))]))
    assert 0 <= gi_host.min() and gi_host.max() < P          # torch's device gather does not check bounds
    gi = torch.from_numpy(gi_host).to(dev)
    p_s, b_s = _np(rep.a_sync[gi]), np.zeros(gi_host.size, dtype=np.float32)
    half = torch.tensor(0.5, dtype=torch.float32, device=dev)
    for r in range(4):
        fused = r >= 2
        slot, S, rank = r % 2, rep.sets[r % 2], r % 2
        off, order_t, total = oracle.slot_offsets(rep.layer_of, rep.numel, S)
        assert rep.ctx.ddp_slot_numel(slot) == total
        rep.fill_grads(r)
        g_s = _np(rep.a_grad[gi])
        # where the samples sit in the flat buffer (arenas are dense: tensor t starts at rep.offsets[t])
        tensor_of = np.searchsorted(rep.offsets, gi_host, side="right") - 1
        sel = off[tensor_of] >= 0
        fi = torch.from_numpy((off[tensor_of] + (gi_host - rep.offsets[tensor_of]))[sel]).to(dev)
        base = torch.cat([rep.sync[t] for t in order_t])
        rep.fill_peers_from(base, r, total)
        peer = rep.peers[0]
        seq = [peer[:total], base] if rank == 1 else [base, peer[:total]]
        mean_dev = (seq[0] + seq[1]) * half                                    # N = 2: one add, one exact halving
        x_s = [_np(t_[fi]) for t_ in seq]
        mean_s = oracle.mean(x_s)
        assert np.array_equal(_bits(_np(mean_dev[fi])), _bits(mean_s))         # the device evaluation agrees with the oracle where sampled
        before_p, before_b = rep.a_sync.clone(), rep.a_s0.clone()
        if fused:
            del base
            rep.fused_step(r, rank)
        else:
            rep.flat.fill_(float("nan"))
            rep.ctx.ddp_pack(slot, rep.flat)
            assert torch.equal(rep.flat[:total].view(torch.int32), base.view(torch.int32)), f"pack r={r}"
            del base
            rep.ctx.ddp_partial_average(slot, rep.flat, rep.peers, 2, rank, rep.flat, rep.stats)
            assert torch.equal(rep.flat[:total].view(torch.int32), mean_dev.view(torch.int32)), f"mean r={r}"
            rep.ctx.ddp_unpack(slot, rep.flat)
            rep.ctx.ddp_local_update(rep.opt_struct(r + 1))
        # every element: synchronised tensors take the mean, then everything takes buf = mu*buf + g; p = p - lr*buf
        for t in order_t:
            before_p[int(rep.offsets[t]): int(rep.offsets[t]) + rep.numel[t]] = mean_dev[int(off[t]): int(off[t]) + rep.numel[t]]
        del mean_dev
        before_b.mul_(w.momentum).add_(rep.a_grad)
        before_p.sub_(before_b * w.lr)
        assert torch.equal(rep.a_s0.view(torch.int32), before_b.view(torch.int32)), f"momentum buffer r={r}"
        assert torch.equal(rep.a_sync.view(torch.int32), before_p.view(torch.int32)), f"parameters r={r}"
        del before_p, before_b
        # samples through the oracle
        p_s[sel] = mean_s
        oracle.sgdm(p_s, g_s, b_s, w.lr, w.momentum)
        assert np.array_equal(_bits(_np(rep.a_sync[gi])), _bits(p_s)), f"oracle samples, parameters r={r}"
        assert np.array_equal(_bits(_np(rep.a_s0[gi])), _bits(b_s)), f"oracle samples, momentum r={r}"
        progress(f"[huge_tensor dense_path={dense_path}] r={r} {'fused' if fused else 'four calls'} slot {slot} ({total} elements) ok")
    rep.close()
