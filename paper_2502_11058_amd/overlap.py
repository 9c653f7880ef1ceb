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
        self._profile = False
        self._stamps = {}
        self._stamp_order: List[int] = []
        self._bp_start = None
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
              order: int = B.DDP_SYNC_THEN_UPDATE, profile: bool = False) -> None:
        """Start iteration r (0-based): clear the gradients (autograd accumulates) and arm the hooks.  Whatever is
        already queued on the current stream (peer buffers, the previous iteration) is ordered before the side
        stream's work.

        profile=True makes this a profiling iteration (the paper's profiler, Sec. 3.2: per-layer backward times are the
        scheduler's input): the hooks only time-stamp each layer's finished gradient, and every layer's sync + update call
        is made in end(), after the backward pass, so that nothing runs beside the backward kernels while they are timed.
        The result of the iteration is the same.  Call backward through `self.backward(loss)` so that the start is
        stamped too, then read `layer_bp_ns()` after `end()`."""
        rep = self.rep
        self._profile = profile
        self._stamps = {}
        self._bp_start = None
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

    def backward(self, loss: torch.Tensor) -> None:
        """loss.backward() with the start of the backward pass time-stamped on the current stream (profiling iterations)."""
        if self._profile:
            self._bp_start = torch.cuda.Event(enable_timing=True)
            self._bp_start.record(torch.cuda.current_stream())
        loss.backward()

    def layer_bp_ns(self) -> List[int]:
        """Per-layer backward time of the last profiling iteration in integer nanoseconds, indexed by layer id: the time
        between the completion of a layer's gradients and the completion of the layer finished before it (for the first
        one: since the start of the backward pass).  Synchronises the device.  Layers that took no part in the graph get 0."""
        if not self._stamps or self._bp_start is None:
            raise RuntimeError("no profiling iteration recorded: begin(profile=True), backward(loss), end()")
        torch.cuda.synchronize(self.rep.dev)
        out = [0] * self.rep.w.n_layers
        prev = self._bp_start
        for l in self._stamp_order:
            out[l] = max(0, int(round(prev.elapsed_time(self._stamps[l]) * 1e6)))
            prev = self._stamps[l]
        return out

    def _launch(self, l: int) -> None:
        if self._profile and self._left is not None:
            # profiling iteration: time-stamp the finished gradient, the call itself waits for end()
            ev = torch.cuda.Event(enable_timing=True)
            ev.record(torch.cuda.current_stream())
            self._stamps[l] = ev
            return
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
        self._stamp_order = list(self._stamps)      # dicts keep insertion order: the order the layers finished in
        self._left = None                           # from here on _launch makes the calls, also in a profiling iteration
        for l in range(self.rep.w.n_layers - 1, -1, -1):
            if not self._launched[l]:
                self._launch(l)
        torch.cuda.current_stream().wait_stream(self.side)
