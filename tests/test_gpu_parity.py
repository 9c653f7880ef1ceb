"""GPU parity: the HIP library against the CPU oracle, element by element, on the same seeded inputs.

Bars: schedule, pack offsets, tensor and layer ids, packed bytes, unpacked bytes and the fp32 average are
bit-exact; per-layer statistics agree to 1e-10 relative (fp64 sums in a different order); optimizer results
agree within 1e-6 relative (fp32) and the bf16 model copy within 1 bf16 ulp, after every iteration.
"""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

from paper_2502_11058_amd import workloads as W

pytestmark = pytest.mark.gpu

RTOL = 1e-6


def _need_gpu():
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: the HIP path cannot run (there is no CPU fallback)")


def _np(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def _bits(a: np.ndarray) -> np.ndarray:
    return a.view(np.uint32) if a.dtype == np.float32 else a


def progress(msg: str) -> None:
    """Progress line from the work itself: printed, and appended to the file named by DDP_TEST_PROGRESS_FILE (if set), so
    that a long test can be followed from outside even when pytest captures the output."""
    print(msg, flush=True)
    path = os.environ.get("DDP_TEST_PROGRESS_FILE")
    if path:
        try:
            with open(path, "a") as f:
                f.write(msg + "\n")
        except OSError:
            pass


def assert_close_fp32(got: np.ndarray, ref: np.ndarray, what: str, atol: float):
    """1e-6 relative, per tensor in the 2-norm and per element; atol guards elements that cancel to ~0."""
    if got.shape == ref.shape and np.array_equal(_bits(got), _bits(ref)):
        return
    g64, r64 = got.astype(np.float64), ref.astype(np.float64)
    nrm = np.linalg.norm(r64)
    assert np.linalg.norm(g64 - r64) <= RTOL * nrm + 1e-30, what
    bad = np.abs(g64 - r64) > RTOL * np.abs(r64) + atol
    assert not bad.any(), (what, int(bad.sum()), got[bad][:4], ref[bad][:4])


def assert_bf16_within_one_ulp(got: np.ndarray, ref: np.ndarray, what: str):
    # bf16 bit patterns are ordered like sign-magnitude integers; map to a monotone integer line first
    def line(u):
        u = u.astype(np.int32)
        return np.where(u & 0x8000, -(u & 0x7fff), u & 0x7fff)
    d = np.abs(line(got) - line(ref))
    assert d.max(initial=0) <= 1, (what, int((d > 1).sum()))


class Tally:
    def __init__(self):
        self.n = 0
        self.exact = 0

    def add(self, a, b):
        self.n += a.size
        self.exact += int((_bits(a) == _bits(b)).sum())

    def frac(self):
        return self.exact / max(self.n, 1)


def run_trajectory(oracle, w, policy=None, iters=None, arena_offset=0, options=None, order=0, grad_dtype=None,
                   check_every=1, threads=16, fused=False, wire16=False, layerwise=0):
    from paper_2502_11058_amd.harness import DeviceReplica
    _need_gpu()
    oracle.set_threads(threads)
    iters = iters or w.iterations
    rep = DeviceReplica(w, 0, options=options, arena_offset=arena_offset, grad_dtype=grad_dtype, policy=policy, wire16=wire16)
    rep.init_params()
    N, H = w.n_replicas, w.period
    fp, bp, comm = W.synthetic_times(w)
    policy = policy or w.policy

    # schedule: bit-exact against the oracle's own search
    import math
    if policy != "opt" or math.comb(w.n_layers + H - 1, H - 1) < 3e7:
        assert rep.sets == oracle.schedule(policy, w.n_layers, H, bp, comm)
    sets = rep.sets

    hyper = dict(lr=w.lr, momentum=w.momentum, beta1=w.beta1, beta2=w.beta2, eps=w.eps, weight_decay=w.weight_decay)
    wk = oracle.Worker(rep.layer_of, [_np(t) for t in rep.sync], w.optimizer, hyper, rep.bf16)
    if rep.bf16:
        for a, b in zip(rep.model, wk.model):
            assert np.array_equal(_np(a), b)
    out = torch.zeros_like(rep.flat)
    if layerwise:
        side = torch.cuda.Stream()
        busy = torch.randn(1024, 1024, device=rep.dev)
        busy_w = torch.eye(1024, device=rep.dev)
    tally = Tally()
    atol_p, atol_s0, atol_s1 = 1e-9, 1e-12, 1e-16

    def update_both(r):
        rep.fill_grads(r)
        grads = [_np(g) for g in rep.grad]
        rep.ctx.ddp_local_update(rep.opt_struct(r + 1))
        wk.local_update(grads, r + 1)

    for r in range(iters):
        slot, S = r % H, sets[r % H]
        rank = r % N
        if order == 1 and not fused:
            update_both(r)
        # layout: offsets, tensor ids, layer ids
        off, order_t, total = oracle.slot_offsets(rep.layer_of, rep.numel, S)
        tid, toff, lid, lbeg = rep.ctx.ddp_slot_layout(slot)
        assert rep.ctx.ddp_slot_numel(slot) == total
        assert tid.tolist() == order_t.tolist() and toff.tolist() == [int(off[t]) for t in order_t]
        assert lid.tolist() == list(S)
        ranges = wk.layer_ranges(S, off, order_t)
        assert lbeg.tolist() == [b for b, _ in ranges] + [total]
        if fused:
            # one call does average + update; peers from an independent gather, statistics and state against the oracle
            dev_flat = torch.cat([rep.sync[t] for t in order_t]) if total else rep.flat[:0]
            local_host = _np(dev_flat)
            if wire16:
                local_host = oracle.bf16_rne(local_host)          # what the local replica contributes
                rep.fill_peers16_from(dev_flat, r, total)
                peers_host = [_np(p[:total]) for p in rep.peers16]
            else:
                rep.fill_peers_from(dev_flat, r, total)
                peers_host = [_np(p[:total]) for p in rep.peers]
            rep.stats.fill_(-1.0)
            if layerwise:
                # gradients appear layer by layer on the main stream, after some unrelated work; each bucket of
                # layers is synchronised and updated on the side stream as soon as its gradients exist
                rep.a_grad.zero_()

                def backward(l):
                    busy.copy_(busy @ busy_w)
                    rep.fill_grads_layer(r, l)
                rep.layerwise_step(r, side, backward=backward, bucket=layerwise, local_rank=rank, wire16=wire16, order=order)
                torch.cuda.synchronize()
                grads = [_np(g) for g in rep.grad]
            else:
                rep.fill_grads(r)
                grads = [_np(g) for g in rep.grad]
            if layerwise:
                pass
            elif order == 1:
                rep.fused_step(r, rank, wire16=wire16, order=1)
            elif wire16:
                rep.ctx.ddp_fused_sync_update_wire16(slot, rep.peers16, N, rank, rep.stats, rep.opt_struct(r + 1))
            else:
                rep.ctx.ddp_fused_sync_update(slot, rep.peers, N, rank, rep.stats, rep.opt_struct(r + 1))
            st = _np(rep.stats)
            if order == 1:
                # Eq. (5) as printed: the carried oracle worker steps, then averages its stepped values with the peers
                wk.local_update(grads, r + 1)
                _, ref_stats = wk.sync(S, peers_host, rank, wire16=wire16)
            else:
                reps = peers_host[:rank] + [local_host] + peers_host[rank:]
                o_mean, o_stats = (oracle.mean_wire16, oracle.layer_stats_wire16) if wire16 else (oracle.mean, oracle.layer_stats)
                mean_ref = o_mean(reps) if total else np.zeros(0, np.float32)
                ref_stats = [o_stats(reps, mean_ref, b, e) for (b, e) in ranges]
                wk.sync(S, peers_host, rank, wire16=wire16)
                wk.local_update(grads, r + 1)
            for i, (g, m) in enumerate(ref_stats):
                assert st[2 * i] == pytest.approx(g, rel=1e-10, abs=1e-300), f"fused gamma r={r} layer {S[i]}"
                assert st[2 * i + 1] == pytest.approx(m, rel=1e-10), f"fused msq r={r} layer {S[i]}"
        elif wire16:
            # bf16 on the wire: pack rounds, the average widens; every stage against the oracle on the same bytes
            dev_flat = torch.cat([rep.sync[t] for t in order_t]) if total else rep.flat[:0]
            local16 = oracle.bf16_rne(_np(dev_flat))
            rep.flat16.view(torch.int16).fill_(-1)
            rep.ctx.ddp_pack_wire16(slot, rep.flat16)
            assert np.array_equal(_np(rep.flat16[:total]), local16), f"pack16 r={r}"
            assert np.array_equal(oracle.pack_wire16([_np(rep.sync[t]) for t in order_t], [off[t] for t in order_t], total), local16)
            assert int(rep.flat16.view(torch.int16)[total:].ne(-1).sum()) == 0, "pack16 wrote past the slot"
            rep.fill_peers16_from(dev_flat, r, total)
            peers_host = [_np(p[:total]) for p in rep.peers16]
            out.fill_(float("nan"))
            rep.stats.fill_(-1.0)
            rep.ctx.ddp_partial_average_wire16(slot, rep.flat16, rep.peers16, N, rank, out, rep.stats)
            reps = peers_host[:rank] + [local16] + peers_host[rank:]
            mean_ref = oracle.mean_wire16(reps) if total else np.zeros(0, np.float32)
            assert np.array_equal(_bits(_np(out[:total])), _bits(mean_ref)), f"mean16 r={r}"
            st = _np(rep.stats)
            for i, (b, e) in enumerate(ranges):
                g, m = oracle.layer_stats_wire16(reps, mean_ref, b, e)
                assert st[2 * i] == pytest.approx(g, rel=1e-10, abs=1e-300), f"gamma16 r={r} layer {S[i]}"
                assert st[2 * i + 1] == pytest.approx(m, rel=1e-10), f"msq16 r={r} layer {S[i]}"
            rep.ctx.ddp_unpack(slot, out)
            wk.sync(S, peers_host, rank, wire16=True)
            if order == 0:
                update_both(r)
        else:
            # pack: against an independent gather of the same device tensors (torch.cat in the oracle's order)
            dev_flat = torch.cat([rep.sync[t] for t in order_t]) if total else rep.flat[:0]
            local_host = _np(dev_flat)
            rep.flat.fill_(float("nan"))
            rep.ctx.ddp_pack(slot, rep.flat)
            assert np.array_equal(_bits(_np(rep.flat[:total])), _bits(local_host)), f"pack r={r}"
            assert np.array_equal(_bits(oracle.pack([_np(rep.sync[t]) for t in order_t], [off[t] for t in order_t], total)),
                                  _bits(local_host))
            # peers: gathered local values + seeded drift; the same bytes go to both sides
            rep.fill_peers_from(dev_flat, r, total)
            peers_host = [_np(p[:total]) for p in rep.peers]
            # average + statistics: bit-exact given the same inputs
            out.fill_(float("nan"))
            rep.stats.fill_(-1.0)
            rep.ctx.ddp_partial_average(slot, rep.flat, rep.peers, N, rank, out, rep.stats)
            reps = peers_host[:rank] + [local_host] + peers_host[rank:]
            mean_ref = oracle.mean(reps) if total else local_host
            assert np.array_equal(_bits(_np(out[:total])), _bits(mean_ref)), f"mean r={r}"
            st = _np(rep.stats)
            with ThreadPoolExecutor(max_workers=8) as pool:      # one oracle call per layer; ctypes releases the GIL
                ref_stats = list(pool.map(lambda be: oracle.layer_stats(reps, mean_ref, be[0], be[1]), ranges))
            for i, (g, m) in enumerate(ref_stats):
                assert st[2 * i] == pytest.approx(g, rel=1e-10, abs=1e-300), f"gamma r={r} layer {S[i]}"
                assert st[2 * i + 1] == pytest.approx(m, rel=1e-10), f"msq r={r} layer {S[i]}"
            # in-place variant (flat_out == flat_local) gives the same bits
            rep.ctx.ddp_partial_average(slot, rep.flat, rep.peers, N, rank, rep.flat, None)
            assert torch.equal(rep.flat[:total].view(torch.int32), out[:total].view(torch.int32)), f"in-place mean r={r}"
            # unpack: the scheduled tensors now hold the average, the model copy its bf16 rounding, nothing else moved
            before = rep.a_sync.clone()
            rep.ctx.ddp_unpack(slot, out)
            expect = before
            for t in order_t:
                expect[int(rep.offsets[t]): int(rep.offsets[t]) + rep.numel[t]] = out[int(off[t]): int(off[t]) + rep.numel[t]]
            assert torch.equal(rep.a_sync.view(torch.int32), expect.view(torch.int32)), f"unpack r={r}"
            if rep.bf16:
                for t in order_t:
                    assert np.array_equal(_np(rep.model[t]), oracle.bf16_rne(mean_ref[int(off[t]): int(off[t]) + rep.numel[t]])), f"model copy r={r} t={t}"
            # the carried oracle worker takes the same step from its own state
            wk.sync(S, peers_host, rank)
            if order == 0:
                update_both(r)
        if (r + 1) % check_every == 0 or r == iters - 1:
            for t in range(len(rep.sync)):
                gp, gs0 = _np(rep.sync[t]), _np(rep.s0[t])
                assert_close_fp32(gp, wk.p[t], f"param r={r} t={t}", atol_p)
                assert_close_fp32(gs0, wk.s0[t], f"state0 r={r} t={t}", atol_s0)
                tally.add(gp, wk.p[t])
                tally.add(gs0, wk.s0[t])
                if rep.adam:
                    gs1 = _np(rep.s1[t])
                    assert_close_fp32(gs1, wk.s1[t], f"state1 r={r} t={t}", atol_s1)
                    tally.add(gs1, wk.s1[t])
                if rep.bf16:
                    assert_bf16_within_one_ulp(_np(rep.model[t]), wk.model[t], f"model r={r} t={t}")
        if w.n_params > 50_000_000:
            progress(f"[{w.name}] iteration {r} slot {slot} ({total} elements) ok")
    # arena bytes outside the tensors were never written
    if arena_offset:
        assert float(rep.a_sync[:arena_offset].abs().sum()) == 0.0
    progress(f"[{w.name}] optimizer state bit-identical to the oracle in {100 * tally.frac():.4f}% of {tally.n} values")
    rep.close()
    return tally


def test_tiny_enp_16_iterations(oracle):
    t = run_trajectory(oracle, W.tiny())
    assert t.frac() == 1.0          # same operations in the same order: the fp32 update is reproduced exactly


def test_tiny_update_then_sync_order(oracle):
    run_trajectory(oracle, W.tiny(), order=1)


def test_tiny_round_robin(oracle):
    run_trajectory(oracle, W.tiny(), policy="round_robin")


@pytest.mark.parametrize("policy", ["full", "every"])
def test_tiny_degenerate_schedules(oracle, policy):
    run_trajectory(oracle, W.tiny(), policy=policy, iters=8)


@pytest.mark.parametrize("arena_offset", [0, 1, 2, 3])
@pytest.mark.parametrize("opt,dtype,N", [("adamw", "bf16", 3), ("sgdm", "f32", 5), ("adamw", "f32", 8), ("sgdm", "bf16", 16)])
def test_odd_shapes_and_alignments(oracle, arena_offset, opt, dtype, N):
    w = W.odd(optimizer=opt, param_dtype=dtype, n_replicas=N, period=2)
    run_trajectory(oracle, w, arena_offset=arena_offset, options={"update_chunk": 4096, "mean_chunk": 2048, "copy_chunk": 1024})


def test_odd_shapes_fp32_gradients_with_bf16_model(oracle):
    run_trajectory(oracle, W.odd(n_replicas=17, period=3), grad_dtype="f32", arena_offset=1)


@pytest.mark.parametrize("nt", [0, 1])
def test_small_llama_opt_schedule(oracle, nt):
    run_trajectory(oracle, W.small_llama(), options={"nontemporal": nt})


def test_small_llama_alg2_schedule_many_replicas(oracle):
    run_trajectory(oracle, W.small_llama(n_replicas=33, period=5), policy="alg2", iters=10)


@pytest.mark.parametrize("fused,wire16", [(False, False), (True, False), (True, True)])
def test_maximum_replica_count(oracle, fused, wire16):
    # N = DDP_MAX_REPLICAS: the run-time replica loop at its limit, four calls and fused
    from paper_2502_11058_amd import binding as B
    t = run_trajectory(oracle, W.odd(n_replicas=B.DDP_MAX_REPLICAS, period=2), fused=fused, wire16=wire16, arena_offset=0)
    assert t.frac() == 1.0


@pytest.mark.parametrize("n_replicas", [1, 2, 6, 7, 9, 10, 11, 12, 13, 14, 15, 17, 18, 24, 32])
def test_every_compiled_and_run_time_replica_count(oracle, n_replicas):
    # the averaging kernel is compiled for N = 1..16 and the fused kernels for N = 2, 4, 8, 16; every other count takes the
    # run-time loop that stages the replicas in LDS.  Four calls, fused, and bf16 on the wire, on ragged shapes.
    w = W.odd(optimizer="adamw", param_dtype="bf16", n_replicas=n_replicas, period=2)
    for fused, wire16 in ((False, False), (True, False), (False, True), (True, True)):
        t = run_trajectory(oracle, w, fused=fused, wire16=wire16, iters=2, arena_offset=n_replicas % 4)
        assert t.frac() == 1.0
    w = W.small_llama(n_replicas=n_replicas, period=2)      # dense arenas: the table-free fused path where it applies
    for fused in (False, True):
        t = run_trajectory(oracle, w, fused=fused, iters=2)
        assert t.frac() == 1.0


@pytest.mark.parametrize("fused", [False, True])
def test_many_small_layers(oracle, fused):
    # 240 layers of two small tensors each: long tables, one statistics row per layer, slots of 48 layers
    ts = []
    for l in range(240):
        ts += [W.TensorSpec(f"l{l}.w", l, 64 * 64 + (l % 3)), W.TensorSpec(f"l{l}.b", l, 64)]
    w = W.Workload("many_layers", ts, n_replicas=4, period=5, optimizer="adamw", param_dtype="bf16", lr=1e-3, sigma_drift=1e-4,
                   sigma_grad=1e-3, iterations=6, policy="opt", time_noise=True)
    t = run_trajectory(oracle, w, fused=fused)
    assert t.frac() == 1.0


def test_small_llama_bubble_filled_schedule(oracle):
    # Sec. 3.4: after filling, top layers sit in several slots; the comm-light synthetic times make filling happen
    w = W.small_llama()
    w.extra["comm_ns_per_byte"] = 0.4
    fp, bp, comm = W.synthetic_times(w)
    sets = oracle.schedule("enp+fill", w.n_layers, w.period, bp, comm)
    assert sum(len(S) for S in sets) > w.n_layers          # some layer really is synchronised twice per period
    t = run_trajectory(oracle, w, policy="enp+fill", iters=8)
    assert t.frac() == 1.0


@pytest.mark.parametrize("name,kw", [("tiny", {}), ("small_llama", {}), ("small_llama", {"n_replicas": 5, "period": 3}),
                                     ("small_llama", {"n_replicas": 16})])
def test_fused_sync_update_equals_the_four_calls(oracle, name, kw):
    w = W.WORKLOADS[name](**kw)
    t = run_trajectory(oracle, w, fused=True, iters=8)
    assert t.frac() == 1.0


@pytest.mark.parametrize("arena_offset", [0, 1, 3])
def test_fused_odd_shapes(oracle, arena_offset):
    w = W.odd(optimizer="adamw", param_dtype="bf16", n_replicas=4, period=2)
    t = run_trajectory(oracle, w, fused=True, arena_offset=arena_offset, options={"update_chunk": 1024})
    assert t.frac() == 1.0
    w = W.odd(optimizer="sgdm", param_dtype="f32", n_replicas=3, period=3)
    run_trajectory(oracle, w, fused=True, arena_offset=arena_offset, policy="full")


@pytest.mark.parametrize("bucket,wire16", [(1, False), (2, False), (3, True), (100, False)])
@pytest.mark.parametrize("name,kw", [("tiny", {}), ("small_llama", {}), ("small_llama", {"n_replicas": 5, "period": 3})])
def test_layerwise_launches_on_a_side_stream_equal_the_whole_step(oracle, name, kw, bucket, wire16):
    # Sec. 3.2: a layer is synchronised as soon as its backward pass is done; the result cannot depend on that
    w = W.WORKLOADS[name](**kw)
    t = run_trajectory(oracle, w, fused=True, layerwise=bucket, wire16=wire16, iters=8)
    assert t.frac() == 1.0


@pytest.mark.parametrize("wire16", [False, True])
@pytest.mark.parametrize("name,kw,layerwise", [("tiny", {}, 0), ("small_llama", {}, 0), ("small_llama", {"n_replicas": 5, "period": 3}, 2),
                                               ("small_llama", {"n_replicas": 16}, 0), ("small_llama", {"n_replicas": 4, "period": 2}, 1)])
def test_fused_update_then_sync_is_eq5_as_printed(oracle, name, kw, layerwise, wire16):
    # the local value takes the optimizer step, then the stepped values are averaged (Eq. (5), Algorithm 1)
    w = W.WORKLOADS[name](**kw)
    t = run_trajectory(oracle, w, fused=True, order=1, wire16=wire16, layerwise=layerwise, iters=8)
    assert t.frac() == 1.0


@pytest.mark.parametrize("arena_offset", [0, 1, 2, 3])
def test_fused_update_then_sync_odd_shapes(oracle, arena_offset):
    w = W.odd(optimizer="adamw", param_dtype="bf16", n_replicas=4, period=2)
    t = run_trajectory(oracle, w, fused=True, order=1, arena_offset=arena_offset, options={"update_chunk": 1024})
    assert t.frac() == 1.0
    w = W.odd(optimizer="sgdm", param_dtype="f32", n_replicas=3, period=3)
    run_trajectory(oracle, w, fused=True, order=1, wire16=True, arena_offset=arena_offset, policy="full")


def test_local_update_by_layer_ranges_equals_the_whole_update(oracle):
    from paper_2502_11058_amd.harness import DeviceReplica
    _need_gpu()
    w = W.small_llama()
    a, b = DeviceReplica(w, 0), DeviceReplica(w, 0)
    for rep in (a, b):
        rep.init_params()
    L = w.n_layers
    for r in range(3):
        for rep in (a, b):
            rep.fill_grads(r)
        a.ctx.ddp_local_update(a.opt_struct(r + 1))
        for lo, n in ((4, L - 4), (0, 1), (1, 0), (1, 3)):            # a partition of [0, L), out of order, one empty range
            b.ctx.ddp_local_update_layers(lo, n, b.opt_struct(r + 1))
        torch.cuda.synchronize()
        for x, y in ((a.a_sync, b.a_sync), (a.a_s0, b.a_s0), (a.a_s1, b.a_s1)):
            assert torch.equal(x.view(torch.int32), y.view(torch.int32))
        assert torch.equal(a.a_model.view(torch.int16), b.a_model.view(torch.int16))
    # and the whole update follows the oracle (carried separately in the trajectory tests); here: ranges are checked
    with pytest.raises(Exception) as e:
        b.ctx.ddp_local_update_layers(L - 1, 2, b.opt_struct(4))
    assert "layer range" in str(e.value)
    with pytest.raises(Exception):
        b.ctx.ddp_fused_sync_update_layers(0, -1, 1, b.peers, 0, 0, w.n_replicas, 0, None, b.opt_struct(4))
    with pytest.raises(Exception):
        b.ctx.ddp_fused_sync_update_layers(0, 0, 1, b.peers, 0, 2, w.n_replicas, 0, None, b.opt_struct(4))       # bad order
    c = DeviceReplica(w, 0, options={"dispatch_ways": 4})
    with pytest.raises(Exception) as e:
        c.ctx.ddp_local_update_layers(0, 1, c.opt_struct(1))
    assert "dispatch_ways" in str(e.value)
    c.ctx.ddp_local_update_layers(0, L, c.opt_struct(1))               # the whole range is fine in any dispatch order
    torch.cuda.synchronize()
    for rep in (a, b, c):
        rep.close()


def test_layerwise_with_a_bubble_filled_schedule_and_odd_shapes(oracle):
    t = run_trajectory(oracle, W.small_llama(n_blocks=6), policy="enp+fill", fused=True, layerwise=1, iters=8)
    assert t.frac() == 1.0
    w = W.odd(optimizer="adamw", param_dtype="bf16", n_replicas=4, period=2)
    t = run_trajectory(oracle, w, fused=True, layerwise=1, arena_offset=3, options={"update_chunk": 1024})
    assert t.frac() == 1.0


@pytest.mark.parametrize("fused", [False, True])
@pytest.mark.parametrize("name,kw", [("tiny", {}), ("small_llama", {}), ("small_llama", {"n_replicas": 5, "period": 3}),
                                     ("small_llama", {"n_replicas": 16}), ("small_llama", {"n_replicas": 4, "period": 2})])
def test_bf16_wire_matches_the_oracle(oracle, name, kw, fused):
    w = W.WORKLOADS[name](**kw)
    t = run_trajectory(oracle, w, fused=fused, wire16=True, iters=8)
    assert t.frac() == 1.0


@pytest.mark.parametrize("fused", [False, True])
@pytest.mark.parametrize("arena_offset", [0, 1, 2, 3])
def test_bf16_wire_odd_shapes(oracle, arena_offset, fused):
    w = W.odd(optimizer="adamw", param_dtype="bf16", n_replicas=4, period=2)
    t = run_trajectory(oracle, w, fused=fused, wire16=True, arena_offset=arena_offset, options={"update_chunk": 1024, "mean_chunk": 2048})
    assert t.frac() == 1.0
    w = W.odd(optimizer="sgdm", param_dtype="f32", n_replicas=3, period=3)
    run_trajectory(oracle, w, fused=fused, wire16=True, arena_offset=arena_offset, policy="full")


@pytest.mark.parametrize("options", [
    {"dense_path": 0}, {"dense_path": 0, "update_chunk": 1024}, {"dense_path": 1, "update_chunk": 4096, "nontemporal": 0},
    {"dispatch_ways": 8}, {"dispatch_ways": 3, "update_chunk": 1024, "mean_chunk": 2048, "copy_chunk": 4096},
    {"update_lds": 0, "mean_lds": 0, "copy_lds": 0, "nontemporal": 0}, {"update_chunk": 1048576, "mean_chunk": 1048576, "copy_chunk": 1048576},
    {"update_wg_per_cu": 4, "mean_wg_per_cu": 0, "copy_wg_per_cu": 1}, {"update_wg_per_cu": 32, "mean_wg_per_cu": 3, "copy_wg_per_cu": 16},
])
def test_launch_options_do_not_change_results(oracle, options):
    t = run_trajectory(oracle, W.odd(n_replicas=8), options=options, arena_offset=2)
    assert t.frac() == 1.0
    t = run_trajectory(oracle, W.odd(n_replicas=8), options=options, arena_offset=0)      # dense arenas: the table-free update
    assert t.frac() == 1.0
    t = run_trajectory(oracle, W.small_llama(), options=options, iters=4)
    assert t.frac() == 1.0
    t = run_trajectory(oracle, W.small_llama(), options=options, fused=True, iters=4)
    assert t.frac() == 1.0


def test_single_replica_is_identity(oracle):
    w = W.tiny()
    w.n_replicas = 1
    run_trajectory(oracle, w, iters=4)


def test_gpt2_small_16_iterations(oracle):
    t = run_trajectory(oracle, W.gpt2_small(), check_every=4)
    assert t.frac() == 1.0


def test_determinism_two_runs_same_bits(oracle):
    from paper_2502_11058_amd.harness import DeviceReplica
    _need_gpu()
    w = W.small_llama()
    snaps = []
    for _ in range(2):
        rep = DeviceReplica(w, 0, policy="opt")
        rep.init_params()
        stats_all = []
        for r in range(8):
            rep.fill_grads(r)
            n = rep.slot_numel[r % w.period]
            rep.fill_peers_from(torch.zeros_like(rep.flat), r, n)
            rep.step(r, local_rank=r % w.n_replicas)
            stats_all.append(rep.stats.clone())
        torch.cuda.synchronize()
        snaps.append((rep.a_sync.clone(), rep.a_model.clone(), rep.a_s0.clone(), rep.a_s1.clone(), torch.stack(stats_all)))
        rep.close()
    for a, b in zip(*snaps):
        assert torch.equal(a, b)
