"""Device-side harness: allocates one worker's state for a workload in HBM, registers it with the library and
drives the four calls of an iteration.  Allocation, seeding and call order only; all arithmetic of the method
happens inside the library.

HBM layout: one flat arena per stream (fp32 master/params, bf16 model copy, gradient, optimizer state 0 and 1),
every tensor a view at its dense offset in registration order, so a kernel sees a handful of long contiguous
streams rather than hundreds of separate allocations.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

from . import binding as B
from . import workloads as W


class DeviceReplica:
    def __init__(self, w: W.Workload, device: int = 0, options: Optional[Dict[str, int]] = None, arena_offset: int = 0,
                 grad_dtype: Optional[str] = None):
        """arena_offset: elements skipped at the start of every arena (tests use it to break 16-byte alignment)."""
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
        o = arena_offset
        self.a_sync = torch.zeros(P + o, dtype=torch.float32, device=self.dev)
        self.a_model = torch.zeros(P + o, dtype=torch.bfloat16, device=self.dev) if self.bf16 else None
        self.a_grad = torch.zeros(P + o, dtype=torch.bfloat16 if self.grad_bf16 else torch.float32, device=self.dev)
        self.a_s0 = torch.zeros(P + o, dtype=torch.float32, device=self.dev)
        self.a_s1 = torch.zeros(P + o, dtype=torch.float32, device=self.dev) if self.adam else None
        self.offsets = np.concatenate([[0], np.cumsum([t.numel for t in w.tensors])]).astype(np.int64) + o

        def views(a):
            return None if a is None else [a[int(self.offsets[i]): int(self.offsets[i]) + t.numel] for i, t in enumerate(w.tensors)]

        self.sync, self.model, self.grad = views(self.a_sync), views(self.a_model), views(self.a_grad)
        self.s0, self.s1 = views(self.a_s0), views(self.a_s1)
        self.layer_of = [t.layer for t in w.tensors]
        self.numel = [t.numel for t in w.tensors]
        self.ctx.ddp_register_model(w.n_layers, self.layer_of, self.numel, B.DDP_BF16 if self.bf16 else B.DDP_F32,
                                    B.DDP_BF16 if self.grad_bf16 else B.DDP_F32, self.sync, self.model, self.grad, self.s0, self.s1)
        self.sets: List[List[int]] = []
        self.flat: Optional[torch.Tensor] = None
        self.peers: List[torch.Tensor] = []
        self.stats: Optional[torch.Tensor] = None

    # -- schedule -------------------------------------------------------------------------------------------
    def set_schedule(self, policy: Optional[str] = None) -> None:
        w = self.w
        fp, bp, comm = W.synthetic_times(w)
        _, sp, sl, self.cost = B.ddp_schedule(policy or w.policy, w.n_layers, w.period, fp, bp, comm)
        self.set_ptr, self.set_layers = sp, sl
        self.sets = B.sets_from_csr(sp, sl)
        self.ctx.ddp_set_schedule(sp, sl)
        self.slot_numel = [self.ctx.ddp_slot_numel(s) for s in range(len(self.sets))]
        smax = max(max(self.slot_numel), 4)
        self.flat = torch.zeros(smax, dtype=torch.float32, device=self.dev)
        self.stats = torch.zeros(2 * max(len(S) for S in self.sets) + 2, dtype=torch.float64, device=self.dev)

    def alloc_peers(self, n_peers: Optional[int] = None) -> None:
        n = self.w.n_replicas - 1 if n_peers is None else n_peers
        smax = max(max(self.slot_numel), 4)
        self.peers = [torch.zeros(smax, dtype=torch.float32, device=self.dev) for _ in range(n)]

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

    def fill_peers_from(self, base_flat: torch.Tensor, iteration: int, n: int) -> None:
        """peer k = base_flat[:n] + N(0, sigma_drift), a fresh seeded draw per (iteration, peer)."""
        w = self.w
        for k, p in enumerate(self.peers):
            W.normal_(p[:n], w.sigma_drift, W.seed_for(w.base_seed, w.name, "peer", iteration, k, 0))
            p[:n].add_(base_flat[:n])

    # -- the iteration ----------------------------------------------------------------------------------------
    def opt_struct(self, step: int) -> B.ddp_opt:
        w = self.w
        return B.make_opt(w.optimizer, w.lr, step, momentum=w.momentum, beta1=w.beta1, beta2=w.beta2, eps=w.eps,
                          weight_decay=w.weight_decay)

    def step(self, r: int, local_rank: int = 0, with_stats: bool = True, stream=None) -> None:
        """Iteration r (0-based): pack -> partial average -> unpack -> local update, all enqueued on one stream."""
        slot = r % len(self.sets)
        c = self.ctx
        c.ddp_pack(slot, self.flat, stream)
        c.ddp_partial_average(slot, self.flat, self.peers, len(self.peers) + 1, local_rank, self.flat,
                              self.stats if with_stats else None, stream)
        c.ddp_unpack(slot, self.flat, stream)
        c.ddp_local_update(self.opt_struct(r + 1), stream)

    def close(self) -> None:
        self.ctx.close()
