"""Device-side harness: allocates one worker's state for a workload in HBM, registers it with the library and
drives the four calls of an iteration.  Allocation, seeding and call order only; all arithmetic of the method
happens inside the library.

HBM layout: ONE slab per worker, cut into 2 MiB-aligned regions: one flat arena per stream (fp32 master/params,
optimizer state 0 and 1, gradient, bf16 model copy), then the flat buffer of the largest slot, the N-1 peer
buffers and the statistics.  Every tensor is a view at its dense offset in registration order, so a kernel sees
a handful of long contiguous streams rather than hundreds of separate allocations.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

from . import binding as B
from . import workloads as W


class DeviceReplica:
    def __init__(self, w: W.Workload, device: int = 0, options: Optional[Dict[str, int]] = None, arena_offset: int = 0,
                 grad_dtype: Optional[str] = None, policy: Optional[str] = None, n_peers: Optional[int] = None,
                 region_skew: int = 0, placement_probe=None, wire16: bool = False, front_pad: int = 0, flat_capacity: int = 0):
        """Schedules, allocates, registers.  arena_offset: elements skipped at the start of every arena (tests use
        it to break 16-byte alignment).  policy: schedule policy (default: the workload's).  region_skew: extra bytes
        (multiple of 256) by which each successive region of the slab is shifted off its 2 MiB boundary.
        placement_probe: time the update kernel on the freshly zeroed slab and, if a re-allocation lands on
        physical memory that streams faster, keep that one (default: on for models of a billion parameters or more).
        front_pad: bytes (multiple of 2 MiB) left unused at the start of the slab; placement_probe="search" tries
        several values and keeps the one whose physical placement streams fastest.
        flat_capacity: elements the flat and peer buffers hold at least (default: the largest slot of the initial schedule);
        a worker that will be re-scheduled (install_schedule) reserves the largest slot it may ever get.
        wire16: also allocate bf16 flat and peer buffers for the bf16-on-the-wire entry points (step/fused_step then
        take wire16=True)."""
        self.wire16 = wire16
        self.front_pad = int(front_pad)
        self.w = w
        self.dev = torch.device("cuda", device)
        torch.cuda.set_device(self.dev)
        self.ctx = B.Context(device)
        for k, v in (options or {}).items():
            self.ctx.ddp_set_option(k, v)
        P = w.n_params
        self.bf16 = w.param_dtype == "bf16"
        self.grad_bf16 = (grad_dtype or ("bf16" if self.bf16 else "f32")) == "bf16"
        self.adam = w.optimizer == "adamw"
        self.layer_of = [t.layer for t in w.tensors]
        self.numel = [t.numel for t in w.tensors]

        # schedule first (CPU): the slot sizes decide how much flat / peer space the slab needs
        fp, bp, comm = W.synthetic_times(w)
        pol = policy or w.policy
        _, sp, sl, self.cost = B.ddp_schedule(pol.split("+")[0], w.n_layers, w.period, fp, bp, comm)
        if pol.endswith("+fill"):      # Sec. 3.4: top layers synchronised more often where the network idles
            sp, sl, _ = B.ddp_schedule_fill_bubbles(bp, comm, sp, sl)
        self.set_ptr, self.set_layers = sp, sl
        self.sets = B.sets_from_csr(sp, sl)
        lay = w.layer_numel()
        smax = max(max(sum(lay[l] for l in S) for S in self.sets), 4, int(flat_capacity))
        n_peers = w.n_replicas - 1 if n_peers is None else n_peers
        max_layers = max(len(S) for S in self.sets)

        self._regions_args = (P, arena_offset, smax, n_peers, max_layers, region_skew, sp, sl, device, options)
        self.placement = {"probe_GBps": []}
        self._build()
        if placement_probe is None:
            placement_probe = P >= 1_000_000_000
        if placement_probe == "search":
            # Where the slab lands physically depends on the size of the allocation and on the offset of the data
            # inside it; the kernels' rates vary by a few per cent with it (same kernels, same virtual layout).
            # Try a few unused front pads, time one pass of the four-call step over all slots on each, keep the fastest.
            GiB = 1 << 30
            body = self.slab.numel() - self.front_pad
            total = torch.cuda.get_device_properties(self.dev).total_memory
            tried = []
            tried.append((self._probe_step(), self.front_pad))      # the slab built above is the first candidate
            for pad in (0, 16 * GiB, 24 * GiB, 32 * GiB, 40 * GiB):
                if pad == tried[0][1] or body + pad + 6 * GiB > total:
                    continue
                self._release()
                self.front_pad = pad
                self._build()
                tried.append((self._probe_step(), pad))
            best_rate, best_pad = max(tried)
            if self.front_pad != best_pad:
                self._release()
                self.front_pad = best_pad
                self._build()
                tried.append((self._probe_step(), best_pad))
            self.placement = {"probe_GBps": [r for r, _ in tried], "front_pad_GiB": [p // GiB for _, p in tried], "kept_GiB": best_pad // GiB}
        elif placement_probe:
            # Successive allocations of a slab this large alternate between two physical placements whose DRAM
            # efficiency differs by ~10 % (same kernel, same virtual layout, same TLB behaviour; the slower one
            # shows more read-credit stalls at the memory interface).  Take two, keep the faster.
            first = self._probe()
            self._release()
            self._build()
            second = self._probe()
            self.placement["probe_GBps"] = [first, second]
            if second < 0.995 * first:
                self._release()
                self._build()
                self.placement["probe_GBps"].append(self._probe())

    def _release(self) -> None:
        import gc
        self.ctx.close()
        self.ctx._keep = []
        for name in ("slab", "a_sync", "a_s0", "a_s1", "a_grad", "a_model", "flat", "stats", "peers", "flat16", "peers16", "sync", "model", "grad", "s0", "s1"):
            setattr(self, name, None)
        gc.collect()
        torch.cuda.empty_cache()
        self.ctx = B.Context(self._regions_args[8])
        for k, v in (self._regions_args[9] or {}).items():
            self.ctx.ddp_set_option(k, v)

    def _probe(self) -> float:
        """GB/s of the update kernel on the zeroed slab (zeros stay zeros under SGD-m and AdamW)."""
        stream = torch.cuda.current_stream()
        P = self._regions_args[0]
        per = (2 if self.grad_bf16 else 4) + (24 if self.adam else 16) + (2 if self.bf16 else 0)
        evs = []
        for r in range(5):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            self.ctx.ddp_local_update(self.opt_struct(r + 1))
            e1.record(stream)
            evs.append((e0, e1))
        torch.cuda.synchronize()
        ms = sorted(a.elapsed_time(b) for a, b in evs[1:])
        return per * P / (ms[len(ms) // 2] * 1e-3) / 1e9

    def _probe_step(self) -> float:
        """GB/s of the whole four-call step on the zeroed slab, one pass over the slots (zeros stay zeros)."""
        stream = torch.cuda.current_stream()
        P = self._regions_args[0]
        per = (2 if self.grad_bf16 else 4) + (24 if self.adam else 16) + (2 if self.bf16 else 0)
        N = len(self.peers) + 1
        self.step(0)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        nbytes = 0.0
        for r in range(len(self.sets)):
            self.step(r)
            nbytes += per * P + (8 + 4 * (N + 1) + (10 if self.bf16 else 8)) * self.slot_numel[r]
        e1.record(stream)
        torch.cuda.synchronize()
        return nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9

    def _build(self) -> None:
        P, arena_offset, smax, n_peers, max_layers, region_skew, sp, sl, _, _ = self._regions_args
        w = self.w
        # one slab for everything this worker owns on the device; every region starts on a 2 MiB boundary
        o = arena_offset
        regions = [("sync", torch.float32, P + o), ("s0", torch.float32, P + o)]
        if self.adam:
            regions.append(("s1", torch.float32, P + o))
        regions.append(("grad", torch.bfloat16 if self.grad_bf16 else torch.float32, P + o))
        if self.bf16:
            regions.append(("model", torch.bfloat16, P + o))
        regions.append(("flat", torch.float32, smax))
        regions += [(f"peer{k}", torch.float32, smax) for k in range(n_peers)]
        if self.wire16:
            regions.append(("flat16", torch.bfloat16, smax))
            regions += [(f"peer16_{k}", torch.bfloat16, smax) for k in range(n_peers)]
        regions.append(("stats", torch.float64, 2 * max(max_layers, w.n_layers) + 2))
        ALIGN = 2 << 20
        pos, place = self.front_pad, {}
        for j, (name, dt, n) in enumerate(regions):
            nbytes = n * torch.empty((), dtype=dt).element_size()
            place[name] = (pos + j * region_skew, nbytes, dt)
            pos += (nbytes + ALIGN - 1) // ALIGN * ALIGN
        pos += len(regions) * region_skew
        self.slab = torch.zeros(pos, dtype=torch.uint8, device=self.dev)

        def region(name):
            if name not in place:
                return None
            start, nbytes, dt = place[name]
            return self.slab[start:start + nbytes].view(dt)

        self.a_sync, self.a_s0, self.a_s1 = region("sync"), region("s0"), region("s1")
        self.a_grad, self.a_model = region("grad"), region("model")
        self.flat, self.stats = region("flat"), region("stats")
        self.peers = [region(f"peer{k}") for k in range(n_peers)]
        self.flat16 = region("flat16")
        self.peers16 = [region(f"peer16_{k}") for k in range(n_peers)] if self.wire16 else []
        # the pointer arrays the entry points take, marshalled once
        self._peers_arr = B.device_pointer_array(self.peers) if self.peers else None
        self._peers16_arr = B.device_pointer_array(self.peers16) if self.peers16 else None
        self.offsets = np.concatenate([[0], np.cumsum(self.numel)]).astype(np.int64) + o

        def views(a):
            return None if a is None else [a[int(self.offsets[i]): int(self.offsets[i]) + n] for i, n in enumerate(self.numel)]

        self.sync, self.model, self.grad = views(self.a_sync), views(self.a_model), views(self.a_grad)
        self.s0, self.s1 = views(self.a_s0), views(self.a_s1)
        self.ctx.ddp_register_model(w.n_layers, self.layer_of, self.numel, B.DDP_BF16 if self.bf16 else B.DDP_F32,
                                    B.DDP_BF16 if self.grad_bf16 else B.DDP_F32, self.sync, self.model, self.grad, self.s0, self.s1)
        self.ctx.ddp_set_schedule(sp, sl)
        self.slot_numel = [self.ctx.ddp_slot_numel(s) for s in range(len(self.sets))]
        assert max(max(self.slot_numel), 4) <= smax

    # -- seeded inputs (harness work, outside any timed region) ---------------------------------------------
    def init_params(self) -> None:
        w = self.w
        for i in range(len(w.tensors)):
            W.normal_(self.sync[i], w.sigma_param, W.seed_for(w.base_seed, w.name, "param", 0, 0, i))
        if self.bf16:
            self.a_model.copy_(self.a_sync)        # torch's cast is round-to-nearest-even
        self.a_s0.zero_()
        if self.a_s1 is not None:
            self.a_s1.zero_()

    def fill_grads(self, iteration: int, worker: int = 0) -> None:
        w = self.w
        for i in range(len(w.tensors)):
            W.normal_(self.grad[i], w.sigma_grad, W.seed_for(w.base_seed, w.name, "grad", iteration, worker, i))

    def fill_grads_layer(self, iteration: int, layer: int, worker: int = 0) -> None:
        """The draws of fill_grads for the tensors of one layer (what a backward hook of that layer would leave)."""
        w = self.w
        for i in range(len(w.tensors)):
            if self.layer_of[i] == layer:
                W.normal_(self.grad[i], w.sigma_grad, W.seed_for(w.base_seed, w.name, "grad", iteration, worker, i))

    def fill_peers_from(self, base_flat: torch.Tensor, iteration: int, n: int) -> None:
        """peer k = base_flat[:n] + N(0, sigma_drift), a fresh seeded draw per (iteration, peer)."""
        w = self.w
        for k, p in enumerate(self.peers):
            W.normal_(p[:n], w.sigma_drift, W.seed_for(w.base_seed, w.name, "peer", iteration, k, 0))
            p[:n].add_(base_flat[:n])

    def fill_peers16_from(self, base_flat: torch.Tensor, iteration: int, n: int) -> None:
        """bf16 peer k = bf16_rne(base_flat[:n] + N(0, sigma_drift)): the fp32 peers of fill_peers_from, rounded
        (torch's cast is round-to-nearest-even).  Leaves the fp32 peer buffers holding the unrounded values."""
        self.fill_peers_from(base_flat, iteration, n)
        for p, q in zip(self.peers, self.peers16):
            q[:n].copy_(p[:n])

    # -- the iteration ----------------------------------------------------------------------------------------
    def opt_struct(self, step: int) -> B.ddp_opt:
        w = self.w
        return B.make_opt(w.optimizer, w.lr, step, momentum=w.momentum, beta1=w.beta1, beta2=w.beta2, eps=w.eps,
                          weight_decay=w.weight_decay)

    def step(self, r: int, local_rank: int = 0, with_stats: bool = True, stream=None, wire16: bool = False) -> None:
        """Iteration r (0-based): pack -> partial average -> unpack -> local update, all enqueued on one stream."""
        slot = r % len(self.sets)
        c = self.ctx
        if wire16:
            c.ddp_pack_wire16(slot, self.flat16, stream)
            c.ddp_partial_average_wire16(slot, self.flat16, self._peers16_arr, len(self.peers16) + 1, local_rank, self.flat,
                                         self.stats if with_stats else None, stream)
            c.ddp_unpack(slot, self.flat, stream)
            c.ddp_local_update(self.opt_struct(r + 1), stream)
            return
        c.ddp_pack(slot, self.flat, stream)
        c.ddp_partial_average(slot, self.flat, self._peers_arr, len(self.peers) + 1, local_rank, self.flat,
                              self.stats if with_stats else None, stream)
        c.ddp_unpack(slot, self.flat, stream)
        c.ddp_local_update(self.opt_struct(r + 1), stream)

    def fused_step(self, r: int, local_rank: int = 0, with_stats: bool = True, stream=None, wire16: bool = False,
                   order: int = B.DDP_SYNC_THEN_UPDATE) -> None:
        """Iteration r through the fused entry point: same result, no flat round trip for the local replica."""
        slot = r % len(self.sets)
        if order != B.DDP_SYNC_THEN_UPDATE:
            peers = self.peers16 if wire16 else self.peers
            self.ctx.ddp_fused_sync_update_layers(slot, 0, self.w.n_layers, peers, B.DDP_BF16 if wire16 else B.DDP_F32, order,
                                                  len(peers) + 1, local_rank, self.stats if with_stats else None,
                                                  self.opt_struct(r + 1), stream)
            return
        if wire16:
            self.ctx.ddp_fused_sync_update_wire16(slot, self._peers16_arr, len(self.peers16) + 1, local_rank,
                                                  self.stats if with_stats else None, self.opt_struct(r + 1), stream)
            return
        self.ctx.ddp_fused_sync_update(slot, self._peers_arr, len(self.peers) + 1, local_rank, self.stats if with_stats else None,
                                       self.opt_struct(r + 1), stream)

    def layerwise_step(self, r: int, side_stream, backward=None, bucket: int = 1, local_rank: int = 0, with_stats: bool = True,
                       wire16: bool = False, order: int = B.DDP_SYNC_THEN_UPDATE) -> None:
        """Iteration r the way Sec. 3.2 overlaps it: backward(l) runs on the current stream for l = L-1 .. 0 and ends
        with layer l's gradient written (default: the seeded draw); after every `bucket` layers an event is recorded,
        the side stream waits for it and takes the fused sync + update of exactly those layers, so it runs under the
        backward pass of the layers below.  The current stream finally waits for the side stream."""
        slot = r % len(self.sets)
        main = torch.cuda.current_stream()
        backward = backward or (lambda l: self.fill_grads_layer(r, l))
        peers = self.peers16 if wire16 else self.peers
        opt = self.opt_struct(r + 1)
        side_stream.wait_stream(main)          # everything already queued (peers, statistics buffer) is visible to the side stream
        hi = self.w.n_layers
        while hi > 0:
            lo = max(0, hi - bucket)
            for l in range(hi - 1, lo - 1, -1):
                backward(l)
            ready = torch.cuda.Event()
            ready.record(main)
            side_stream.wait_event(ready)
            self.ctx.ddp_fused_sync_update_layers(slot, lo, hi - lo, peers, B.DDP_BF16 if wire16 else B.DDP_F32, order, len(peers) + 1,
                                                  local_rank, self.stats if with_stats else None, opt, side_stream)
            hi = lo
        main.wait_stream(side_stream)

    def install_schedule(self, set_ptr, set_layers) -> None:
        """Replace the schedule (output of ddp_schedule, e.g. after re-profiling the layer times): ddp_set_schedule rebuilds
        the per-slot tables.  The flat and peer buffers must hold the largest new slot (flat_capacity)."""
        sets = B.sets_from_csr(set_ptr, set_layers)
        lay = self.w.layer_numel()
        need = max(sum(lay[l] for l in S) for S in sets)
        if need > self.flat.numel():
            raise ValueError(f"the new schedule has a slot of {need} elements, the flat and peer buffers hold {self.flat.numel()}")
        if max(len(S) for S in sets) * 2 > self.stats.numel():
            raise ValueError("the statistics buffer is too small for the new schedule")
        self.ctx.ddp_set_schedule(set_ptr, set_layers)
        self.set_ptr, self.set_layers, self.sets = set_ptr, set_layers, sets
        self.slot_numel = [self.ctx.ddp_slot_numel(s) for s in range(len(sets))]

    def layer_wire_bytes(self, wire16: bool = False) -> List[int]:
        """Bytes each layer puts on the wire when it is synchronised (what its communication time is proportional to)."""
        return [(2 if wire16 else 4) * n for n in self.w.layer_numel()]

    def close(self) -> None:
        self.ctx.close()
