"""Python face of the CPU oracle (test infrastructure only; see plsgd_oracle.c for what is followed).

The arithmetic lives in plsgd_oracle.c (plain C loops).  This file builds that C file with gcc, wraps its
functions for numpy arrays, and strings them together into the iteration of Algorithm 1 for one worker and
for K workers in one process.  It imports nothing from the GPU package.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "plsgd_oracle.c")
_LIB = os.path.join(_HERE, "libplsgd_oracle.so")
_lib = None

SYNC_THEN_UPDATE = 0   # Sec. 3.2: a layer's synchronisation follows its backward pass, before the optimizer step
UPDATE_THEN_SYNC = 1   # Algorithm 1 as printed: update to w_{r+1/2}, then average


def build(force: bool = False) -> str:
    """Compile the oracle.  -ffp-contract=off keeps every product and sum a separate fp32 operation."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_slot_offsets.restype = C.c_int64
        _lib.orc_sched_cost.restype = C.c_int64
        _lib.orc_sched_brute.restype = C.c_int64
        _lib.orc_sched_alg2.restype = C.c_int64
        _lib.orc_eq7_summand.restype = C.c_int64
        _lib.orc_iteration_timeline.restype = C.c_int64
    return _lib


def set_threads(n: int) -> None:
    """Number of OpenMP threads for the elementwise loops (1 = the plain serial loops)."""
    omp = C.CDLL("libgomp.so.1")
    omp.omp_set_num_threads(int(n))


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _ptr_array(arrs: Sequence[Optional[np.ndarray]]):
    out = (C.c_void_p * len(arrs))()
    for i, a in enumerate(arrs):
        out[i] = None if a is None else a.ctypes.data
    return out


def _chk(a: np.ndarray, dtype) -> np.ndarray:
    assert a.dtype == dtype and a.flags["C_CONTIGUOUS"], (a.dtype, dtype)
    return a


# ------------------------------------------------------------------------------------------------------------
# elementwise pieces
# ------------------------------------------------------------------------------------------------------------

def bf16_rne(x: np.ndarray) -> np.ndarray:
    x = _chk(np.ascontiguousarray(x), np.float32)
    out = np.empty(x.shape, dtype=np.uint16)
    lib().orc_bf16_rne(_p(x), _p(out), C.c_int64(x.size))
    return out


def bf16_widen(h: np.ndarray) -> np.ndarray:
    h = _chk(np.ascontiguousarray(h), np.uint16)
    out = np.empty(h.shape, dtype=np.float32)
    lib().orc_bf16_widen(_p(h), _p(out), C.c_int64(h.size))
    return out


def slot_offsets(layer_of: Sequence[int], numel: Sequence[int], set_layers: Sequence[int]) -> Tuple[np.ndarray, np.ndarray, int]:
    """(dst_off[T] with -1 for unscheduled tensors, tensor ids in flat order, total elements)."""
    T = len(layer_of)
    lo = np.asarray(layer_of, dtype=np.int32)
    ne = np.asarray(numel, dtype=np.int64)
    sl = np.asarray(set_layers, dtype=np.int32)
    off = np.empty(T, dtype=np.int64)
    order = np.empty(max(T, 1), dtype=np.int32)
    n_order = C.c_int32(0)
    total = lib().orc_slot_offsets(T, _p(lo), _p(ne), len(sl), _p(sl), _p(off), _p(order), C.byref(n_order))
    return off, order[: n_order.value].copy(), int(total)


def pack(tensors: Sequence[np.ndarray], off: Sequence[int], total: int) -> np.ndarray:
    flat = np.zeros(total, dtype=np.float32)
    ts = [_chk(t, np.float32) for t in tensors]
    ne = np.asarray([t.size for t in ts], dtype=np.int64)
    of = np.asarray(off, dtype=np.int64)
    lib().orc_pack(len(ts), _ptr_array(ts), _p(ne), _p(of), _p(flat))
    return flat


def unpack(flat: np.ndarray, tensors: Sequence[np.ndarray], models: Optional[Sequence[Optional[np.ndarray]]],
           off: Sequence[int]) -> None:
    ts = [_chk(t, np.float32) for t in tensors]
    ne = np.asarray([t.size for t in ts], dtype=np.int64)
    of = np.asarray(off, dtype=np.int64)
    mp = None
    if models is not None:
        for m in models:
            if m is not None:
                _chk(m, np.uint16)
        mp = _ptr_array(models)
    lib().orc_unpack(len(ts), _ptr_array(ts), mp, _p(ne), _p(of), _p(_chk(flat, np.float32)))


def mean(replicas: Sequence[np.ndarray]) -> np.ndarray:
    """Average of N flat buffers given in global rank order (Eq. (5), second case)."""
    xs = [_chk(x, np.float32) for x in replicas]
    n = xs[0].size
    assert all(x.size == n for x in xs)
    out = np.empty(n, dtype=np.float32)
    lib().orc_mean(len(xs), _ptr_array(xs), C.c_int64(n), _p(out))
    return out


def layer_stats(replicas: Sequence[np.ndarray], mean_: np.ndarray, begin: int, end: int) -> Tuple[float, float]:
    xs = [_chk(x, np.float32) for x in replicas]
    g = C.c_double(0.0)
    m = C.c_double(0.0)
    lib().orc_layer_stats(len(xs), _ptr_array(xs), _p(_chk(mean_, np.float32)), C.c_int64(begin), C.c_int64(end),
                          C.byref(g), C.byref(m))
    return g.value, m.value


def pack_wire16(tensors: Sequence[np.ndarray], off: Sequence[int], total: int) -> np.ndarray:
    flat = np.zeros(total, dtype=np.uint16)
    ts = [_chk(t, np.float32) for t in tensors]
    ne = np.asarray([t.size for t in ts], dtype=np.int64)
    of = np.asarray(off, dtype=np.int64)
    lib().orc_pack_wire16(len(ts), _ptr_array(ts), _p(ne), _p(of), _p(flat))
    return flat


def mean_wire16(replicas: Sequence[np.ndarray]) -> np.ndarray:
    """Average of N flat bf16 buffers (bit patterns, uint16) in rank order; fp32 result."""
    xs = [_chk(x, np.uint16) for x in replicas]
    n = xs[0].size
    assert all(x.size == n for x in xs)
    out = np.empty(n, dtype=np.float32)
    lib().orc_mean_wire16(len(xs), _ptr_array(xs), C.c_int64(n), _p(out))
    return out


def layer_stats_wire16(replicas: Sequence[np.ndarray], mean_: np.ndarray, begin: int, end: int) -> Tuple[float, float]:
    xs = [_chk(x, np.uint16) for x in replicas]
    g = C.c_double(0.0)
    m = C.c_double(0.0)
    lib().orc_layer_stats_wire16(len(xs), _ptr_array(xs), _p(_chk(mean_, np.float32)), C.c_int64(begin), C.c_int64(end),
                                 C.byref(g), C.byref(m))
    return g.value, m.value


def sgdm(p: np.ndarray, g: np.ndarray, buf: np.ndarray, lr: float, mu: float) -> None:
    """In place on p and buf."""
    assert p.size == g.size == buf.size
    lib().orc_sgdm(_p(_chk(p, np.float32)), _p(_chk(g, np.float32)), _p(_chk(buf, np.float32)), C.c_int64(p.size),
                   C.c_float(lr), C.c_float(mu))


def adamw(p: np.ndarray, g: np.ndarray, m: np.ndarray, v: np.ndarray, model: Optional[np.ndarray], lr: float,
          beta1: float, beta2: float, eps: float, wd: float, step: int) -> None:
    """In place on p, m, v (and model).  g is fp32 or bf16 bit patterns (uint16)."""
    assert p.size == g.size == m.size == v.size
    g32 = g if g.dtype == np.float32 else None
    g16 = g if g.dtype == np.uint16 else None
    assert (g32 is None) != (g16 is None)
    assert g.flags["C_CONTIGUOUS"]
    if model is not None:
        _chk(model, np.uint16)
    lib().orc_adamw(_p(_chk(p, np.float32)), _p(g32), _p(g16), _p(_chk(m, np.float32)), _p(_chk(v, np.float32)),
                    _p(model), C.c_int64(p.size), C.c_float(lr), C.c_float(beta1), C.c_float(beta2), C.c_float(eps),
                    C.c_float(wd), C.c_int64(step))


def adamw_scalars(lr: float, beta1: float, beta2: float, wd: float, step: int) -> np.ndarray:
    out = np.empty(5, dtype=np.float32)
    lib().orc_adamw_scalars(C.c_float(lr), C.c_float(beta1), C.c_float(beta2), C.c_float(wd), C.c_int64(step), _p(out))
    return out


# ------------------------------------------------------------------------------------------------------------
# scheduling
# ------------------------------------------------------------------------------------------------------------

def sched_cost(bp: Sequence[int], comm: Sequence[int], sizes: Sequence[int]) -> int:
    """Eq. (8) for the cut of the BP-ordered layer sequence given by `sizes` (one entry per set)."""
    b = np.asarray(bp, dtype=np.int64)
    c = np.asarray(comm, dtype=np.int64)
    s = np.asarray(sizes, dtype=np.int32)
    assert int(s.sum()) == len(b) == len(c)
    return int(lib().orc_sched_cost(len(b), len(s), _p(b), _p(c), _p(s)))


def sched_brute(bp: Sequence[int], comm: Sequence[int], H: int) -> Tuple[List[int], int, int]:
    """(sizes, cost, number of cuts enumerated) of the exhaustive optimum of Eq. (8)."""
    b = np.asarray(bp, dtype=np.int64)
    c = np.asarray(comm, dtype=np.int64)
    best = np.zeros(H, dtype=np.int32)
    cnt = C.c_int64(0)
    cost = lib().orc_sched_brute(len(b), H, _p(b), _p(c), _p(best), C.byref(cnt))
    return best.tolist(), int(cost), int(cnt.value)


def sched_alg2(bp: Sequence[int], comm: Sequence[int], H: int, cap: int = 1 << 16) -> Tuple[List[int], int, List[List[int]]]:
    """(sizes, cost, Omega) of Algorithm 2's pruned DFS."""
    b = np.asarray(bp, dtype=np.int64)
    c = np.asarray(comm, dtype=np.int64)
    best = np.zeros(H, dtype=np.int32)
    omega = np.zeros((cap, H), dtype=np.int32)
    cost = C.c_int64(0)
    n = lib().orc_sched_alg2(len(b), H, _p(b), _p(c), _p(best), C.byref(cost), _p(omega), C.c_int64(cap))
    assert n <= cap, "solution set larger than the buffer"
    return best.tolist(), int(cost.value), omega[:n].tolist()


def sched_enp(L: int, H: int) -> List[int]:
    s = np.zeros(H, dtype=np.int32)
    lib().orc_sched_enp(L, H, _p(s))
    return s.tolist()


def eq7_summand(bp: Sequence[int], comm: Sequence[int], pos: int, size: int) -> int:
    """One summand of Eq. (7) as printed, for the contiguous set at BP positions [pos, pos+size)."""
    b = np.asarray(bp, dtype=np.int64)
    c = np.asarray(comm, dtype=np.int64)
    return int(lib().orc_eq7_summand(len(b), _p(b), _p(c), pos, size))


def iteration_timeline(bp: Sequence[int], comm: Sequence[int], layers: Sequence[int]) -> Tuple[int, int]:
    """(end of backward + communication, exposed communication) of one iteration that synchronises `layers`."""
    b = np.asarray(bp, dtype=np.int64)
    c = np.asarray(comm, dtype=np.int64)
    ls = np.asarray(layers, dtype=np.int32)
    ex = C.c_int64(0)
    t = lib().orc_iteration_timeline(len(b), _p(b), _p(c), len(ls), _p(ls), C.byref(ex))
    return int(t), int(ex.value)


def time_model(fp: Sequence[int], bp: Sequence[int], comm: Sequence[int], sets: Sequence[Sequence[int]]) -> Tuple[List[int], List[int], int]:
    """Eq. (7) for one period: per-iteration time (forward + backward/communication), exposed communication per
    iteration, and the period total."""
    f = int(np.sum(np.asarray(fp, dtype=np.int64)))
    it, ex = [], []
    for S in sets:
        t, e = iteration_timeline(bp, comm, S)
        it.append(f + t)
        ex.append(e)
    return it, ex, int(sum(it))


def fill_bubbles(bp: Sequence[int], comm: Sequence[int], sizes: Sequence[int]) -> Tuple[List[int], List[List[int]]]:
    """Eq. (12): (number of top layers added per set, the resulting sets in BP order)."""
    b = np.asarray(bp, dtype=np.int64)
    c = np.asarray(comm, dtype=np.int64)
    s = np.asarray(sizes, dtype=np.int32)
    extra = np.zeros(len(s), dtype=np.int32)
    lib().orc_fill_bubbles(len(b), len(s), _p(b), _p(c), _p(s), _p(extra))
    L = len(b)
    base = sets_from_sizes(L, sizes)
    return extra.tolist(), [[L - 1 - j for j in range(e)] + S for e, S in zip(extra.tolist(), base)]


def sets_from_sizes(L: int, sizes: Sequence[int]) -> List[List[int]]:
    """Cut sizes -> per-set layer lists in BP order (descending layer id)."""
    sets, pos = [], 0
    for s in sizes:
        sets.append([L - 1 - j for j in range(pos, pos + s)])
        pos += s
    assert pos == L
    return sets


def schedule(policy: str, L: int, H: int, bp: Optional[Sequence[int]] = None, comm: Optional[Sequence[int]] = None) -> List[List[int]]:
    """Per-slot layer lists.  Slot p is used at 0-based iteration r with r mod H == p.
    A policy name followed by "+fill" applies Eq. (12)'s bubble filling to the cut."""
    if policy.endswith("+fill"):
        base = schedule(policy[:-5], L, H, bp, comm)
        return fill_bubbles(bp, comm, [len(S) for S in base])[1]
    if policy == "enp":
        return sets_from_sizes(L, sched_enp(L, H))
    if policy == "round_robin":
        return [[l for l in range(L - 1, -1, -1) if l % H == p] for p in range(H)]
    if policy == "full":       # Eq. (2): everything when (r+1) % H == 0
        return [[] for _ in range(H - 1)] + [list(range(L - 1, -1, -1))]
    if policy == "every":      # all layers every iteration (per-step model averaging)
        return [list(range(L - 1, -1, -1)) for _ in range(H)]
    if policy == "opt":
        return sets_from_sizes(L, sched_brute(bp, comm, H)[0])
    if policy == "alg2":
        return sets_from_sizes(L, sched_alg2(bp, comm, H)[0])
    raise ValueError(policy)


# ------------------------------------------------------------------------------------------------------------
# one worker, and K workers in one process
# ------------------------------------------------------------------------------------------------------------

class Worker:
    """State of one replica: per-tensor fp32 params (master), optional bf16 model copy, optimizer state."""

    def __init__(self, layer_of: Sequence[int], params: Sequence[np.ndarray], optimizer: str, hyper: dict,
                 bf16_model: bool):
        self.layer_of = list(layer_of)
        self.p = [np.array(x, dtype=np.float32, copy=True) for x in params]
        self.numel = [x.size for x in self.p]
        self.optimizer = optimizer
        self.hyper = dict(hyper)
        self.s0 = [np.zeros_like(x) for x in self.p]                       # momentum buffer or m
        self.s1 = [np.zeros_like(x) for x in self.p] if optimizer == "adamw" else None
        self.model = [bf16_rne(x) for x in self.p] if bf16_model else None

    def pack_slot(self, set_layers: Sequence[int], wire16: bool = False):
        off, order, total = slot_offsets(self.layer_of, self.numel, set_layers)
        fn = pack_wire16 if wire16 else pack
        flat = fn([self.p[t] for t in order], [off[t] for t in order], total)
        return flat, off, order, total

    def unpack_slot(self, flat: np.ndarray, off, order) -> None:
        models = [self.model[t] for t in order] if self.model is not None else None
        unpack(flat, [self.p[t] for t in order], models, [off[t] for t in order])

    def local_update(self, grads: Sequence[np.ndarray], step: int) -> None:
        h = self.hyper
        for t in range(len(self.p)):
            if self.optimizer == "sgdm":
                g = grads[t] if grads[t].dtype == np.float32 else bf16_widen(grads[t])   # widening is exact
                sgdm(self.p[t], g, self.s0[t], h["lr"], h["momentum"])
                if self.model is not None:
                    self.model[t][...] = bf16_rne(self.p[t])
            else:
                adamw(self.p[t], grads[t], self.s0[t], self.s1[t], None if self.model is None else self.model[t],
                      h["lr"], h["beta1"], h["beta2"], h["eps"], h["weight_decay"], step)

    def layer_ranges(self, set_layers, off, order):
        """Flat [begin, end) of each scheduled layer, in set order."""
        out = []
        for l in set_layers:
            ts = [t for t in order if self.layer_of[t] == l]
            if ts:
                out.append((int(off[ts[0]]), int(off[ts[-1]] + self.numel[ts[-1]])))
            else:
                out.append((0, 0))
        return out

    def sync(self, set_layers: Sequence[int], peers: Sequence[np.ndarray], local_rank: int, wire16: bool = False):
        """pack -> average with the peers (rank order, local buffer at position local_rank) -> unpack.
        Returns (flat mean, [(Gamma^l, ||mean^l||^2) per scheduled layer]).  wire16: bf16 buffers on the wire."""
        flat, off, order, total = self.pack_slot(set_layers, wire16)
        reps = list(peers[:local_rank]) + [flat] + list(peers[local_rank:])
        out = (mean_wire16 if wire16 else mean)(reps)
        st = layer_stats_wire16 if wire16 else layer_stats
        stats = [st(reps, out, b, e) for (b, e) in self.layer_ranges(set_layers, off, order)]
        self.unpack_slot(out, off, order)
        return out, stats

    def step(self, r: int, sets: Sequence[Sequence[int]], peers: Sequence[np.ndarray], local_rank: int,
             grads: Sequence[np.ndarray], order: int = SYNC_THEN_UPDATE):
        """Iteration r (0-based) of Algorithm 1 for this worker; slot = r mod H; optimizer step count r+1."""
        S = sets[r % len(sets)]
        if order == UPDATE_THEN_SYNC:
            self.local_update(grads, r + 1)
            return self.sync(S, peers, local_rank)
        res = self.sync(S, peers, local_rank)
        self.local_update(grads, r + 1)
        return res


def run_workers(workers: List[Worker], r: int, sets, grads_per_worker, order: int = SYNC_THEN_UPDATE, wire16: bool = False):
    """One iteration of Algorithm 1 for K workers held in this process: each worker's peers are the other
    workers' packed buffers of the same iteration (bf16 buffers with wire16)."""
    K = len(workers)
    S = sets[r % len(sets)]
    if order == UPDATE_THEN_SYNC:
        for k in range(K):
            workers[k].local_update(grads_per_worker[k], r + 1)
    flats = [w.pack_slot(S, wire16)[0] for w in workers]
    results = []
    for k in range(K):
        peers = [flats[j] for j in range(K) if j != k]
        results.append(workers[k].sync(S, peers, k, wire16))
    if order == SYNC_THEN_UPDATE:
        for k in range(K):
            workers[k].local_update(grads_per_worker[k], r + 1)
    return results
