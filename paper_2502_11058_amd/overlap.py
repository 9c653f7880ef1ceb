"""Layer-wise overlap of synchronisation + update with a torch model's backward pass (Sec. 3.2 of the paper: a layer's
synchronisation is launched as soon as its backward pass has produced its gradient, while the layers below are still
in BP).  Plumbing only: parameters and gradients of the model are views of the worker's registered arenas, autograd
hooks record an event per finished layer, and a side stream takes that layer's fused sync + update call.  All of the
method's arithmetic happens inside the library call.
"""
from __future__ import annotations

import functools
from typing import List, Optional

import torch

from . import binding as B
from .harness import DeviceReplica


class BackwardOverlap:
    """Couples a DeviceReplica to a torch model.

    `params[i]` is a 1-D `torch.nn.Parameter` over registered tensor i (the bf16 model copy if there is one, else the
    fp32 parameters); the model reshapes it with `.view(...)`.  Its `.grad` is the registered gradient tensor, so
    autograd accumulates straight into the memory the library reads.  Per iteration: `begin(r)`, the model's forward
    and backward (one backward call per iteration), `end()`.

    A layer's parameters are rewritten as soon as its gradients are complete.  That is safe when nothing later in the
    same backward pass reads them again (every kernel of the layer's own backward is already queued ahead of the
    event); a model that recomputes activations of that layer afterwards, or shares the layer's weights with a layer
    below, must not be driven this way.
    """

    def __init__(self, rep: DeviceReplica, side_stream: Optional[torch.cuda.Stream] = None, side_cus: int = 0):
        """side_cus > 0: divide the chip.  The side stream is confined to that many compute units and `main_stream`
        to the others (ddp_stream_create_cu_range); the caller runs forward and backward under
        `torch.cuda.stream(ov.main_stream)`.  A backward kernel that fills every CU otherwise leaves the side stream no
        slot until it ends, and nothing is hidden.  Default: an ordinary side stream, `main_stream` = the current one."""
        self.rep = rep
        self._owned = []
        if side_cus > 0 and side_stream is None:
            ncu = B.ddp_device_cu_count(rep.dev.index)
            if not 0 < side_cus < ncu:
                raise ValueError(f"side_cus must be in (0, {ncu})")
            self._owned = [B.ddp_stream_create_cu_range(rep.dev.index, 0, side_cus),
                           B.ddp_stream_create_cu_range(rep.dev.index, side_cus, ncu - side_cus)]
            self.side = torch.cuda.ExternalStream(self._owned[0], device=rep.dev)
            self.main_stream = torch.cuda.ExternalStream(self._owned[1], device=rep.dev)
        else:
            self.side = side_stream or torch.cuda.Stream(device=rep.dev)
            self.main_stream = torch.cuda.current_stream(rep.dev)
        self.params: List[torch.nn.Parameter] = []
        self._tensors_in_layer = [0] * rep.w.n_layers
        for i, l in enumerate(rep.layer_of):
            # .data: same memory, but a version counter of its own.  The arenas are views of one slab and share the
            # slab's counter, so any in-place torch op on the slab (autograd's own gradient accumulation included)
            # would otherwise look like a modification of every tensor saved for backward.
            src = (rep.model[i] if rep.bf16 else rep.sync[i]).data
            p = torch.nn.Parameter(src, requires_grad=True)
            p.grad = rep.grad[i].data
            p.register_post_accumulate_grad_hook(functools.partial(self._on_grad, i))
            self.params.append(p)
            self._tensors_in_layer[l] += 1
        self._left: Optional[List[int]] = None
        self._launched: List[bool] = []
        self.launch_order: List[int] = []       # layers in the order their calls were enqueued (last iteration)

    def close(self) -> None:
        """Release the CU-range streams made here (after their work is complete)."""
        if self._owned:
            torch.cuda.synchronize(self.rep.dev)
            for h in self._owned:
                B.ddp_stream_destroy(h)
            self._owned = []

    def begin(self, r: int, local_rank: int = 0, with_stats: bool = True, wire16: bool = False,
              order: int = B.DDP_SYNC_THEN_UPDATE) -> None:
        """Start iteration r (0-based): clear the gradients (autograd accumulates) and arm the hooks.  Whatever is
        already queued on the current stream (peer buffers, the previous iteration) is ordered before the side
        stream's work."""
        rep = self.rep
        rep.a_grad.zero_()
        self._slot = r % len(rep.sets)
        self._opt = rep.opt_struct(r + 1)
        self._rank, self._stats = local_rank, (rep.stats if with_stats else None)
        self._peers = rep.peers16 if wire16 else rep.peers
        self._wire = B.DDP_BF16 if wire16 else B.DDP_F32
        self._order = order
        self._left = list(self._tensors_in_layer)
        self._launched = [False] * rep.w.n_layers
        self.launch_order = []
        self.side.wait_stream(torch.cuda.current_stream())

    def _on_grad(self, i: int, _param) -> None:
        if self._left is None:
            return                                       # backward outside begin()/end(): nothing to overlap
        l = self.rep.layer_of[i]
        self._left[l] -= 1
        if self._left[l] == 0:
            self._launch(l)

    def _launch(self, l: int) -> None:
        # the hook runs on the stream the backward pass runs on: everything that produced this layer's gradients
        # precedes the event
        ready = torch.cuda.Event()
        ready.record(torch.cuda.current_stream())
        self.side.wait_event(ready)
        self.rep.ctx.ddp_fused_sync_update_layers(self._slot, l, 1, self._peers, self._wire, self._order, len(self._peers) + 1,
                                                  self._rank, self._stats, self._opt, self.side)
        self._launched[l] = True
        self.launch_order.append(l)

    def end(self) -> None:
        """After backward: layers whose parameters took no part in the graph get their call now (their gradient is
        zero), then the current stream waits for the side stream, so the next forward sees the new parameters."""
        for l in range(self.rep.w.n_layers - 1, -1, -1):
            if not self._launched[l]:
                self._launch(l)
        self._left = None
        torch.cuda.current_stream().wait_stream(self.side)
