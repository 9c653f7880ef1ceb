"""Thin ctypes binding of libdreamddp.so: same names as the C ABI (include/dreamddp.h), argument marshalling only.

Every step of the path runs in the library's own kernels; torch tensors are used for device memory and streams.
There is no fallback: if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("DREAMDDP_LIB") or os.path.join(_HERE, "lib", "libdreamddp.so")

DDP_F32, DDP_BF16 = 0, 1
DDP_OPT_SGDM, DDP_OPT_ADAMW = 0, 1
DDP_SYNC_THEN_UPDATE, DDP_UPDATE_THEN_SYNC = 0, 1
DDP_MAX_REPLICAS = 64
DDP_STATIC_SCRATCH_BYTES = 16 << 20
POLICIES = {"enp": 0, "round_robin": 1, "full": 2, "every": 3, "opt": 4, "alg2": 5}
STATUS = {0: "DDP_OK", 1: "DDP_EINVAL", 2: "DDP_ESHAPE", 3: "DDP_EALIGN", 4: "DDP_ENOMEM", 5: "DDP_EHIP", 6: "DDP_ESCHED",
          7: "DDP_ESTATE"}

EXPORTS = [
    "ddp_schedule", "ddp_schedule_cost", "ddp_schedule_alg2_solutions", "ddp_schedule_fill_bubbles", "ddp_schedule_time_model", "ddp_create", "ddp_destroy", "ddp_set_option",
    "ddp_register_model", "ddp_set_schedule", "ddp_slot_numel", "ddp_slot_num_layers", "ddp_slot_num_tensors",
    "ddp_slot_layout", "ddp_pack", "ddp_partial_average", "ddp_unpack", "ddp_local_update", "ddp_fused_sync_update",
    "ddp_pack_wire16", "ddp_partial_average_wire16", "ddp_fused_sync_update_wire16",
    "ddp_local_update_layers", "ddp_fused_sync_update_layers", "ddp_partial_average_static", "ddp_stream_probe", "ddp_device_cu_count", "ddp_stream_create_cu_range", "ddp_stream_destroy", "ddp_last_error",
]


class DdpError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"{STATUS.get(code, code)}: {msg}")
        self.code = code


class ddp_opt(C.Structure):
    _fields_ = [("kind", C.c_int32), ("lr", C.c_float), ("momentum", C.c_float), ("beta1", C.c_float),
                ("beta2", C.c_float), ("eps", C.c_float), ("weight_decay", C.c_float), ("step", C.c_int64)]


_lib = None


def lib():
    """Load the library built in-tree (python -m paper_2502_11058_amd.build, or __graft_entry__.build())."""
    global _lib
    if _lib is None:
        # torch first: the library must share torch's HIP runtime (streams and device pointers come from torch),
        # and whichever copy of libamdhip64 is loaded first serves every later library of the process
        import torch  # noqa: F401
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: build it first (python __graft_entry__.py)")
        l = C.CDLL(LIB_PATH)
        l.ddp_slot_numel.restype = C.c_int64
        l.ddp_last_error.restype = C.c_char_p
        l.ddp_last_error.argtypes = [C.c_void_p]
        l.ddp_slot_numel.argtypes = [C.c_void_p, C.c_int]
        l.ddp_slot_num_layers.argtypes = [C.c_void_p, C.c_int]
        l.ddp_slot_num_tensors.argtypes = [C.c_void_p, C.c_int]
        l.ddp_slot_layout.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        l.ddp_create.argtypes = [C.POINTER(C.c_void_p), C.c_int]
        l.ddp_destroy.argtypes = [C.c_void_p]
        l.ddp_set_option.argtypes = [C.c_void_p, C.c_char_p, C.c_int64]
        l.ddp_register_model.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_int] + [C.c_void_p] * 5
        l.ddp_set_schedule.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
        l.ddp_pack.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
        l.ddp_unpack.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
        l.ddp_partial_average.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]
        l.ddp_partial_average_static.argtypes = l.ddp_partial_average.argtypes
        l.ddp_local_update.argtypes = [C.c_void_p, C.POINTER(ddp_opt), C.c_void_p]
        l.ddp_fused_sync_update.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.POINTER(ddp_opt), C.c_void_p]
        l.ddp_pack_wire16.argtypes = l.ddp_pack.argtypes
        l.ddp_partial_average_wire16.argtypes = l.ddp_partial_average.argtypes
        l.ddp_fused_sync_update_wire16.argtypes = l.ddp_fused_sync_update.argtypes
        l.ddp_local_update_layers.argtypes = [C.c_void_p, C.c_int, C.c_int, C.POINTER(ddp_opt), C.c_void_p]
        l.ddp_fused_sync_update_layers.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int,
                                                   C.c_void_p, C.POINTER(ddp_opt), C.c_void_p]
        l.ddp_device_cu_count.argtypes = [C.c_int, C.POINTER(C.c_int)]
        l.ddp_stream_create_cu_range.argtypes = [C.c_int, C.c_int, C.c_int, C.POINTER(C.c_void_p)]
        l.ddp_stream_destroy.argtypes = [C.c_void_p]
        l.ddp_stream_probe.argtypes = [C.c_int, C.c_int, C.c_int64, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p]
        l.ddp_schedule.argtypes = [C.c_int, C.c_int, C.c_int] + [C.c_void_p] * 7
        l.ddp_schedule_cost.argtypes = [C.c_int, C.c_int] + [C.c_void_p] * 5
        l.ddp_schedule_alg2_solutions.argtypes = [C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]
        l.ddp_schedule_fill_bubbles.argtypes = [C.c_int, C.c_int] + [C.c_void_p] * 7
        l.ddp_schedule_time_model.argtypes = [C.c_int, C.c_int] + [C.c_void_p] * 8
        _lib = l
    return _lib


def _check(rc: int, ctx=None) -> None:
    if rc != 0:
        raise DdpError(rc, lib().ddp_last_error(ctx).decode())


def _i64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int64))


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _np_ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data


# ------------------------------------------------------------------------------------------------------------
# scheduling (CPU)
# ------------------------------------------------------------------------------------------------------------

def ddp_schedule(policy: str, L: int, H: int, t_fp=None, t_bp=None, t_comm=None) -> Tuple[np.ndarray, np.ndarray, np.ndarray, int]:
    """-> (slot_of_layer[L], set_ptr[H+1], set_layers, cost_ns or -1)."""
    fp = None if t_fp is None else _i64(t_fp)
    bp = None if t_bp is None else _i64(t_bp)
    cm = None if t_comm is None else _i64(t_comm)
    slot = np.zeros(max(L, 0), dtype=np.int32)
    set_ptr = np.zeros(max(H, 0) + 1, dtype=np.int32)
    cap = max(L, 0) * (max(H, 1) if policy == "every" else 1)
    set_layers = np.zeros(max(cap, 1), dtype=np.int32)
    cost = C.c_int64(-1)
    rc = lib().ddp_schedule(POLICIES[policy] if isinstance(policy, str) else policy, L, H, _np_ptr(fp), _np_ptr(bp), _np_ptr(cm),
                            slot.ctypes.data, set_ptr.ctypes.data, set_layers.ctypes.data, C.addressof(cost))
    _check(rc)
    return slot, set_ptr, set_layers[: set_ptr[H]].copy(), int(cost.value)


def ddp_schedule_cost(t_bp, t_comm, set_ptr, set_layers) -> int:
    bp, cm, sp, sl = _i64(t_bp), _i64(t_comm), _i32(set_ptr), _i32(set_layers)
    cost = C.c_int64(-1)
    _check(lib().ddp_schedule_cost(len(bp), len(sp) - 1, bp.ctypes.data, cm.ctypes.data, sp.ctypes.data, sl.ctypes.data, C.addressof(cost)))
    return int(cost.value)


def ddp_schedule_alg2_solutions(t_bp, t_comm, H: int) -> int:
    bp, cm = _i64(t_bp), _i64(t_comm)
    n = C.c_int64(0)
    _check(lib().ddp_schedule_alg2_solutions(len(bp), H, bp.ctypes.data, cm.ctypes.data, C.addressof(n)))
    return int(n.value)


def ddp_schedule_fill_bubbles(t_bp, t_comm, set_ptr, set_layers) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """-> (set_ptr[H+1], set_layers, extra[H]) of the schedule after Eq. (12)'s bubble filling."""
    bp, cm, sp, sl = _i64(t_bp), _i64(t_comm), _i32(set_ptr), _i32(set_layers)
    L, H = len(bp), len(sp) - 1
    if len(sl) == 0:
        sl = np.zeros(1, dtype=np.int32)
    osp = np.zeros(H + 1, dtype=np.int32)
    osl = np.zeros(max(L * H, 1), dtype=np.int32)
    ext = np.zeros(H, dtype=np.int32)
    _check(lib().ddp_schedule_fill_bubbles(L, H, bp.ctypes.data, cm.ctypes.data, sp.ctypes.data, sl.ctypes.data,
                                           osp.ctypes.data, osl.ctypes.data, ext.ctypes.data))
    return osp, osl[: osp[H]].copy(), ext


def ddp_schedule_time_model(t_fp, t_bp, t_comm, set_ptr, set_layers) -> Tuple[np.ndarray, np.ndarray, int]:
    """-> (iteration time [H], exposed communication [H], period total) under Eq. (7)."""
    fp = None if t_fp is None else _i64(t_fp)
    bp, cm, sp, sl = _i64(t_bp), _i64(t_comm), _i32(set_ptr), _i32(set_layers)
    H = len(sp) - 1
    if len(sl) == 0:
        sl = np.zeros(1, dtype=np.int32)
    it = np.zeros(H, dtype=np.int64)
    ex = np.zeros(H, dtype=np.int64)
    per = C.c_int64(0)
    _check(lib().ddp_schedule_time_model(len(bp), H, _np_ptr(fp), bp.ctypes.data, cm.ctypes.data, sp.ctypes.data, sl.ctypes.data,
                                         it.ctypes.data, ex.ctypes.data, C.addressof(per)))
    return it, ex, int(per.value)


def csr_from_sets(sets) -> Tuple[np.ndarray, np.ndarray]:
    sp = np.cumsum([0] + [len(S) for S in sets]).astype(np.int32)
    sl = np.asarray([l for S in sets for l in S], dtype=np.int32)
    return sp, sl


def sets_from_csr(set_ptr, set_layers) -> List[List[int]]:
    return [list(map(int, set_layers[set_ptr[s]: set_ptr[s + 1]])) for s in range(len(set_ptr) - 1)]


# ------------------------------------------------------------------------------------------------------------
# context
# ------------------------------------------------------------------------------------------------------------

def _stream_handle(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _dev_ptrs(tensors) -> "C.Array":
    arr = (C.c_void_p * len(tensors))()
    for i, t in enumerate(tensors):
        arr[i] = None if t is None else (t if isinstance(t, int) else t.data_ptr())
    return arr


def device_pointer_array(tensors) -> "C.Array":
    """The host array of device pointers that the peers arguments take, built once; a caller that passes the same
    buffers every iteration hands this to the entry points instead of the list of tensors."""
    return _dev_ptrs(list(tensors))


def _peers_arg(peers):
    if not peers:
        return None
    return peers if isinstance(peers, C.Array) else _dev_ptrs(list(peers))


def ddp_stream_probe(read_tensors, write_tensors, nbytes: int, chunk_bytes: int = 8192, lds_pad: int = 65536, stream=None) -> None:
    """Enqueue the read/write reference kernel over the first nbytes of every given tensor (see the header)."""
    rd = _dev_ptrs(list(read_tensors)) if read_tensors else None
    wr = _dev_ptrs(list(write_tensors)) if write_tensors else None
    _check(lib().ddp_stream_probe(len(read_tensors or []), len(write_tensors or []), int(nbytes), None if rd is None else C.addressof(rd),
                                  None if wr is None else C.addressof(wr), chunk_bytes, lds_pad, _stream_handle(stream)))


def ddp_device_cu_count(device: int = 0) -> int:
    n = C.c_int(0)
    _check(lib().ddp_device_cu_count(device, C.byref(n)))
    return n.value


def ddp_stream_create_cu_range(device: int, cu_first: int, cu_count: int) -> int:
    """-> hipStream_t handle (an int) of a stream confined to those compute units; wrap it with
    torch.cuda.ExternalStream(handle) to run torch work on it, release it with ddp_stream_destroy."""
    h = C.c_void_p()
    _check(lib().ddp_stream_create_cu_range(device, cu_first, cu_count, C.byref(h)))
    return int(h.value)


def ddp_stream_destroy(handle: int) -> None:
    _check(lib().ddp_stream_destroy(C.c_void_p(handle)))


class Context:
    """Owns a ddp_ctx.  Methods carry the names of the C entry points and only marshal arguments."""

    def __init__(self, device: int = 0):
        h = C.c_void_p()
        _check(lib().ddp_create(C.byref(h), device))
        self._h = h
        self._keep = []          # registered tensors, kept alive

    def close(self) -> None:
        if self._h:
            lib().ddp_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def ddp_set_option(self, name: str, value: int) -> None:
        _check(lib().ddp_set_option(self._h, name.encode(), int(value)), self._h)

    def ddp_register_model(self, L: int, layer_of: Sequence[int], numel: Sequence[int], param_dtype: int, grad_dtype: int,
                           sync, model, grad, state0, state1) -> None:
        """sync/model/grad/state0/state1: sequences of torch tensors (or raw device addresses); model and state1 may be None."""
        T = len(layer_of)
        lo, ne = _i32(layer_of), _i64(numel)
        arrays = [None if x is None else _dev_ptrs(x) for x in (sync, model, grad, state0, state1)]
        self._keep = [sync, model, grad, state0, state1]
        _check(lib().ddp_register_model(self._h, L, T, lo.ctypes.data, ne.ctypes.data, param_dtype, grad_dtype,
                                        *[None if a is None else C.addressof(a) for a in arrays]), self._h)

    def ddp_set_schedule(self, set_ptr, set_layers) -> None:
        sp, sl = _i32(set_ptr), _i32(set_layers)
        if len(sl) == 0:
            sl = np.zeros(1, dtype=np.int32)
        _check(lib().ddp_set_schedule(self._h, len(sp) - 1, sp.ctypes.data, sl.ctypes.data), self._h)

    def ddp_slot_numel(self, slot: int) -> int:
        n = lib().ddp_slot_numel(self._h, slot)
        if n < 0:
            _check(int(-n), self._h)
        return int(n)

    def ddp_slot_num_layers(self, slot: int) -> int:
        n = lib().ddp_slot_num_layers(self._h, slot)
        if n < 0:
            _check(-n, self._h)
        return n

    def ddp_slot_num_tensors(self, slot: int) -> int:
        n = lib().ddp_slot_num_tensors(self._h, slot)
        if n < 0:
            _check(-n, self._h)
        return n

    def ddp_slot_layout(self, slot: int):
        """-> (tensor_ids, tensor_off, layer_ids, layer_begin[n_layers+1])."""
        nt, nl = self.ddp_slot_num_tensors(slot), self.ddp_slot_num_layers(slot)
        tid = np.zeros(max(nt, 1), dtype=np.int32)
        off = np.zeros(max(nt, 1), dtype=np.int64)
        lid = np.zeros(max(nl, 1), dtype=np.int32)
        lb = np.zeros(nl + 1, dtype=np.int64)
        _check(lib().ddp_slot_layout(self._h, slot, tid.ctypes.data, off.ctypes.data, lid.ctypes.data, lb.ctypes.data), self._h)
        return tid[:nt], off[:nt], lid[:nl], lb

    def ddp_pack(self, slot: int, flat_local, stream=None) -> None:
        _check(lib().ddp_pack(self._h, slot, flat_local.data_ptr(), _stream_handle(stream)), self._h)

    def ddp_partial_average(self, slot: int, flat_local, peers, N: int, local_rank: int, flat_out, layer_stats=None, stream=None) -> None:
        arr = _peers_arg(peers)
        _check(lib().ddp_partial_average(self._h, slot, flat_local.data_ptr(), None if arr is None else C.addressof(arr), N, local_rank,
                                         flat_out.data_ptr(), None if layer_stats is None else layer_stats.data_ptr(),
                                         _stream_handle(stream)), self._h)

    def ddp_partial_average_static(self, slot: int, flat_local, peers, N: int, local_rank: int, flat_out, layer_stats=None,
                                   stream=None) -> None:
        arr = _peers_arg(peers)
        _check(lib().ddp_partial_average_static(self._h, slot, flat_local.data_ptr(), None if arr is None else C.addressof(arr), N,
                                                local_rank, flat_out.data_ptr(),
                                                None if layer_stats is None else layer_stats.data_ptr(), _stream_handle(stream)), self._h)

    def ddp_unpack(self, slot: int, flat, stream=None) -> None:
        _check(lib().ddp_unpack(self._h, slot, flat.data_ptr(), _stream_handle(stream)), self._h)

    def ddp_local_update(self, opt: ddp_opt, stream=None) -> None:
        _check(lib().ddp_local_update(self._h, C.byref(opt), _stream_handle(stream)), self._h)

    def ddp_fused_sync_update(self, slot: int, peers, N: int, local_rank: int, layer_stats, opt: ddp_opt, stream=None) -> None:
        arr = _peers_arg(peers)
        _check(lib().ddp_fused_sync_update(self._h, slot, None if arr is None else C.addressof(arr), N, local_rank,
                                           None if layer_stats is None else layer_stats.data_ptr(), C.byref(opt),
                                           _stream_handle(stream)), self._h)

    def ddp_pack_wire16(self, slot: int, flat_local16, stream=None) -> None:
        _check(lib().ddp_pack_wire16(self._h, slot, flat_local16.data_ptr(), _stream_handle(stream)), self._h)

    def ddp_partial_average_wire16(self, slot: int, flat_local16, peers16, N: int, local_rank: int, flat_out, layer_stats=None,
                                   stream=None) -> None:
        arr = _peers_arg(peers16)
        _check(lib().ddp_partial_average_wire16(self._h, slot, flat_local16.data_ptr(), None if arr is None else C.addressof(arr), N,
                                                local_rank, flat_out.data_ptr(),
                                                None if layer_stats is None else layer_stats.data_ptr(), _stream_handle(stream)), self._h)

    def ddp_fused_sync_update_wire16(self, slot: int, peers16, N: int, local_rank: int, layer_stats, opt: ddp_opt, stream=None) -> None:
        arr = _peers_arg(peers16)
        _check(lib().ddp_fused_sync_update_wire16(self._h, slot, None if arr is None else C.addressof(arr), N, local_rank,
                                                  None if layer_stats is None else layer_stats.data_ptr(), C.byref(opt),
                                                  _stream_handle(stream)), self._h)

    def ddp_local_update_layers(self, layer_first: int, layer_count: int, opt: ddp_opt, stream=None) -> None:
        _check(lib().ddp_local_update_layers(self._h, layer_first, layer_count, C.byref(opt), _stream_handle(stream)), self._h)

    def ddp_fused_sync_update_layers(self, slot: int, layer_first: int, layer_count: int, peers, wire_dtype: int, order: int, N: int,
                                     local_rank: int, layer_stats, opt: ddp_opt, stream=None) -> None:
        arr = _peers_arg(peers)
        _check(lib().ddp_fused_sync_update_layers(self._h, slot, layer_first, layer_count, None if arr is None else C.addressof(arr),
                                                  wire_dtype, order, N, local_rank,
                                                  None if layer_stats is None else layer_stats.data_ptr(), C.byref(opt),
                                                  _stream_handle(stream)), self._h)

    def last_error(self) -> str:
        return lib().ddp_last_error(self._h).decode()


def make_opt(kind: str, lr: float, step: int, momentum: float = 0.0, beta1: float = 0.9, beta2: float = 0.95, eps: float = 1e-8,
             weight_decay: float = 0.0) -> ddp_opt:
    return ddp_opt(DDP_OPT_SGDM if kind == "sgdm" else DDP_OPT_ADAMW, lr, momentum, beta1, beta2, eps, weight_decay, step)
