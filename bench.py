#!/usr/bin/env python3
"""Benchmark of one worker's partial-sync + update step (pack -> partial average -> unpack -> local update).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload llama2_7b]

A "step" is one iteration of Algorithm 1 for one worker: the four library calls for slot r mod H, with the
N-1 peer buffers, the gradients and all optimizer state already resident in HBM.  Inputs are seeded and
synthetic (shapes of the named model, Gaussian values).  Prints ONE JSON line.

  value      = algorithmic bytes of the K timed steps / wall time of the K steps, in GB/s (whole step, launch
               gaps included); also given as a fraction of the 8 TB/s peak and as parameters per second.  For models of
               a billion parameters or more the timed slab is the one the harness's placement search kept; the same K
               steps on the plain first allocation are measured first and reported as no_placement_search.
  roofline   = the dominant kernel (the fused optimizer update): algorithmic bytes per launch / its average
               duration measured with events on the launch stream in a second pass of K steps; traffic = HBM bytes per
               launch from an earlier rocprofv3 counter run (profiles/traffic.json).
  cpu_baseline = the CPU oracle timed on this machine's host cores on a bounded sample (one transformer block), with one
               thread and with all cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0     # MI355X HBM3E, published peak

TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic.json")


def measured_traffic(workload: str, kernel: str, options: dict):
    """HBM bytes per launch of `kernel` as rocprofv3's FETCH_SIZE + WRITE_SIZE counters read them in an earlier,
    separate profiling run (python -m paper_2502_11058_amd.profile_summary writes the file from that run's output and
    records the commit and the command).  None if there is no reading for this workload with default library options:
    a counter run cannot share a process with the timed run, so this is never a live figure."""
    if options:
        return None
    try:
        with open(TRAFFIC_FILE) as f:
            rec = json.load(f).get(workload, {}).get(kernel)
    except (OSError, ValueError):
        return None
    return rec


def algorithmic_bytes(w, S: int):
    """Bytes the method must move in one step with S scheduled elements and P parameters (fp32 on the wire)."""
    P, N = w.n_params, w.n_replicas
    bf16 = w.param_dtype == "bf16"
    pack = 8 * S
    mean = 4 * (N + 1) * S
    unpack = (10 if bf16 else 8) * S
    if w.optimizer == "adamw":
        g = 2 if bf16 else 4
        update = (g + 12 + 12 + (2 if bf16 else 0)) * P      # read g,p,m,v; write p,m,v(,model)
    else:
        g = 2 if bf16 else 4
        update = (g + 8 + 8 + (2 if bf16 else 0)) * P        # read g,p,buf; write p,buf(,model)
    return {"pack": pack, "partial_average": mean, "unpack": unpack, "local_update": update}


def cpu_baseline(rep, w):
    """The oracle on the host cores, on one transformer block of the same workload (the bytes the device holds), in two
    legs: one thread, and every core this process may use.  Each piece of the step (pack, average, statistics, unpack,
    optimizer) is timed on its own so that the serial statistics loop of the oracle does not hide what the others do."""
    import numpy as np
    from oracle import plsgd as oracle
    cores = len(os.sched_getaffinity(0))
    cores = max(1, min(cores, int(os.environ.get("OMP_NUM_THREADS", cores))))
    layer = 1 if w.n_layers > 2 else 0
    ids = [i for i, t in enumerate(w.tensors) if t.layer == layer]

    def host(t):
        import torch
        if t.dtype == torch.bfloat16:
            return t.view(torch.int16).cpu().numpy().view(np.uint16)
        return t.cpu().numpy()

    params = [host(rep.sync[i]) for i in ids]
    grads = [host(rep.grad[i]) for i in ids]
    numel = [x.size for x in params]
    S = int(sum(numel))
    N = w.n_replicas
    off, order, total = oracle.slot_offsets([0] * len(ids), numel, [0])
    rng = np.random.default_rng(0)
    flat0 = oracle.pack(params, [off[t] for t in order], total)
    peers = [flat0 + (rng.standard_normal(S, dtype=np.float32) * np.float32(w.sigma_drift)) for _ in range(N - 1)]
    sub = type(w)(name="sample", tensors=[w.tensors[i] for i in ids], n_replicas=N, period=1, optimizer=w.optimizer,
                  param_dtype=w.param_dtype, lr=w.lr)
    ab = algorithmic_bytes(sub, S)
    models = [np.empty(n, dtype=np.uint16) for n in numel] if rep.bf16 else None
    s0 = [np.zeros(n, dtype=np.float32) for n in numel]
    s1 = [np.zeros(n, dtype=np.float32) for n in numel]
    state = {}

    def do_pack():
        state["flat"] = oracle.pack(params, [off[t] for t in order], total)

    def do_mean():
        state["mean"] = oracle.mean([state["flat"]] + peers)

    def do_stats():
        oracle.layer_stats([state["flat"]] + peers, state["mean"], 0, total)

    def do_unpack():
        oracle.unpack(state["mean"], params, models, [off[t] for t in order])

    def do_update():
        for j in range(len(ids)):
            if w.optimizer == "adamw":
                oracle.adamw(params[j], grads[j], s0[j], s1[j], None if models is None else models[j], w.lr, w.beta1, w.beta2,
                             w.eps, w.weight_decay, state["step"])
            else:
                g = grads[j] if grads[j].dtype == np.float32 else oracle.bf16_widen(grads[j])
                oracle.sgdm(params[j], g, s0[j], w.lr, w.momentum)
        state["step"] += 1

    pieces = (("pack", do_pack, ab["pack"]), ("partial_average", do_mean, ab["partial_average"]), ("layer_statistics", do_stats, 0),
              ("unpack", do_unpack, ab["unpack"]), ("local_update", do_update, ab["local_update"]))
    state["step"] = 1
    for _, fn, _ in pieces:        # untimed first pass: page in every buffer the pieces write
        fn()
    legs = {}
    for threads in ([1, cores] if cores > 1 else [1]):
        oracle.set_threads(threads)
        leg = {}
        total_s = 0.0
        for name, fn, nbytes in pieces:
            t0 = time.perf_counter()
            fn()
            dt = time.perf_counter() - t0
            total_s += dt
            leg[name] = {"s": dt, "GB/s": nbytes / dt / 1e9 if nbytes else None, "elements_per_s": S / dt}
        leg["step_s"] = total_s
        leg["GB/s"] = sum(ab.values()) / total_s / 1e9
        leg["params_per_s"] = S / total_s
        legs[str(threads)] = leg
    oracle.set_threads(cores)
    best = legs[str(cores)]
    return {"value": best["GB/s"], "unit": "GB/s", "cores": cores, "kind": "oracle",
            "sample": f"one transformer block of {w.name} ({S} parameters, N={N}): pack, average, per-layer statistics, unpack and "
                      f"{w.optimizer} update, each timed once after an untimed first pass; {best['step_s']:.2f} s with {cores} threads, "
                      f"{legs['1']['step_s']:.2f} s with 1 (the statistics loop of the oracle is serial in both)",
            "params_per_s": best["params_per_s"], "single_thread": {"value": legs["1"]["GB/s"], "cores": 1, "params_per_s": legs["1"]["params_per_s"]},
            "pieces": legs}


def reference_rates(gib: float):
    """GB/s of ddp_stream_probe for mixes of read and write streams, in the launch shape of the update / average
    kernels (8 KiB of every stream per workgroup, two workgroups per CU) and of pack / unpack (six per CU)."""
    import torch
    from paper_2502_11058_amd import binding as B
    nbytes = int(gib * (1 << 30)) // 4096 * 4096
    dev = torch.device("cuda", 0)
    bufs = [torch.zeros(nbytes // 4, dtype=torch.float32, device=dev) for _ in range(20)]
    for i, b in enumerate(bufs[:16]):
        b.normal_(0.0, 0.02 * (i + 1))
    rd, wr = bufs[:16], bufs[16:]
    stream = torch.cuda.current_stream()
    rows = []
    mixes = [(1, 0), (2, 0), (4, 0), (8, 0), (16, 0), (0, 1), (0, 2), (0, 4), (1, 1), (2, 1), (4, 1), (8, 1), (16, 1), (3, 3), (4, 4), (8, 4)]
    for lds_pad in (65536, 24576):
        for nr, nw in mixes:
            times = []
            for rep_i in range(7):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                B.ddp_stream_probe(rd[:nr], wr[:nw], nbytes, 8192, lds_pad)
                e1.record(stream)
                times.append((e0, e1))
            torch.cuda.synchronize()
            ms = sorted(a.elapsed_time(b) for a, b in times[2:])
            med = ms[len(ms) // 2]
            rows.append({"reads": nr, "writes": nw, "workgroups_per_cu": 2 if lds_pad == 65536 else 6, "ms": med,
                         "GB/s": (nr + nw) * nbytes / (med * 1e-3) / 1e9})
    return {"reference_rates": rows, "bytes_per_stream": nbytes, "peak_GBps": HBM_PEAK_GBS, "clocks": gpu_clocks()}


def gpu_clocks():
    """Clock / performance state of the first AMD GPU from sysfs, read after the run (plain file reads: no child
    process is started from a process that holds the GPU).  None if the files are not there."""
    import glob
    for dev in sorted(glob.glob("/sys/class/drm/card*/device")):
        try:
            if open(os.path.join(dev, "vendor")).read().strip() != "0x1002":
                continue
            out = {}
            for key, name in (("sclk", "pp_dpm_sclk"), ("mclk", "pp_dpm_mclk"), ("fclk", "pp_dpm_fclk")):
                path = os.path.join(dev, name)
                if os.path.exists(path):
                    cur = [ln.split(":", 1)[1].replace("*", "").strip() for ln in open(path).read().splitlines() if ln.strip().endswith("*")]
                    if cur:
                        out[key] = cur[0]
            path = os.path.join(dev, "power_dpm_force_performance_level")
            if os.path.exists(path):
                out["performance_level"] = open(path).read().strip()
            if out:
                return out
        except OSError:
            continue
    return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=16)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="llama2_7b")
    ap.add_argument("--policy", default=None)
    ap.add_argument("--replicas", type=int, default=None, metavar="N",
                    help="override the workload's replica count (e.g. 17 to measure the kernels for run-time replica counts)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-stats", action="store_true", help="skip the per-layer statistics in the average")
    ap.add_argument("--option", action="append", default=[], help="library option name=value (repeatable)")
    ap.add_argument("--wire16", action="store_true",
                    help="also time the bf16-on-the-wire entry points (four calls and fused); reported in an extra "
                         "\"wire16\" object, never in value")
    ap.add_argument("--overlap", action="store_true",
                    help="also time the layer-wise launches of Sec. 3.2 on a side stream under a synthetic backward pass "
                         "(bf16 matrix products standing in for each layer's BP); extra \"overlap\" object, never in value")
    ap.add_argument("--overlap-side-cus", default="16,32,48,64,96,128", metavar="R,R,..",
                    help="with --overlap: also run with the side stream confined to R compute units and the backward pass to the "
                         "others (ddp_stream_create_cu_range), for each R in the list")
    ap.add_argument("--overlap-mm", type=int, default=4096, metavar="D",
                    help="edge of the square bf16 products of --overlap (4096: one product fills the 256 CUs)")
    ap.add_argument("--front-pad-gib", type=int, default=None, metavar="G",
                    help="leave G GiB unused at the start of the worker's slab (default 0)")
    ap.add_argument("--no-placement-search", action="store_true",
                    help="measure on the plain first allocation only.  Default for models of a billion parameters or more: measure that "
                         "first (reported as no_placement_search / value_no_placement_search), then re-allocate the slab by the "
                         "harness's placement search and measure value there")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run 4 plain copies of 1 GiB (ddp_stream_probe, one read and one write stream) before the timed "
                         "region, as the known-size reference for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE readings")
    ap.add_argument("--reference-rates", action="store_true",
                    help="instead of the benchmark: time ddp_stream_probe (a kernel of the library's launch shape that only reads R "
                         "streams and writes W streams) for a list of (R, W) mixes and print the GB/s of each: the practical "
                         "ceilings the kernels' rates are compared with")
    ap.add_argument("--reference-gib", type=float, default=2.0, metavar="G", help="bytes per stream of --reference-rates, in GiB")
    ap.add_argument("--placement-study", type=int, default=0, metavar="M",
                    help="instead of the benchmark: allocate the slab M times in a row, time the update kernel on each "
                         "(zeroed state) and print the GB/s list; shows the two physical placements a slab alternates between")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (peers are staged in HBM; there are no collectives). "
              "Run with --gpus 1.", file=sys.stderr)
        return 2

    import torch
    from paper_2502_11058_amd import workloads as W
    from paper_2502_11058_amd.harness import DeviceReplica

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 3
    w = W.get(args.workload)
    options = {k: int(v) for k, v in (o.split("=") for o in args.option)}
    if args.reference_rates:
        print(json.dumps(reference_rates(args.reference_gib)))
        return 0
    if args.replicas is not None:
        w.n_replicas = args.replicas
    if args.placement_study:
        import gc
        res = []
        for _ in range(args.placement_study):
            rep = DeviceReplica(w, 0, options=options, policy=args.policy, placement_probe=False,
                                front_pad=(args.front_pad_gib or 0) << 30)
            res.append(round(rep._probe(), 1))
            rep.close()
            rep._release()
            rep.ctx.close()
            del rep
            gc.collect()
            torch.cuda.empty_cache()
        print(json.dumps({"placement_study_update_GBps": res, "workload": w.name, "front_pad_GiB": args.front_pad_gib or 0}))
        return 0
    def stage_inputs(rep):
        rep.init_params()
        rep.fill_grads(0)
        # peers: slot 0's packed local values + seeded drift; later slots reuse the staged bytes (same distribution)
        rep.ctx.ddp_pack(0, rep.flat)
        torch.cuda.synchronize()
        if args.wire16:
            rep.fill_peers16_from(rep.flat, 0, rep.flat.numel())
        else:
            rep.fill_peers_from(rep.flat, 0, rep.flat.numel())
        torch.cuda.synchronize()

    with_stats = not args.no_stats

    def plain_measurement(rep):
        """W warm-up and K timed steps of the four calls, then of the fused entry point, on the wall clock; the update
        kernel's own rate from events around its K launches."""
        Hn = len(rep.sets)
        for r in range(args.warmup):
            rep.step(r, with_stats=with_stats)
        torch.cuda.synchronize()
        stream = torch.cuda.current_stream()
        evs = []
        t0 = time.perf_counter()
        for r in range(args.warmup, args.warmup + args.steps):
            slot = r % Hn
            c = rep.ctx
            c.ddp_pack(slot, rep.flat)
            c.ddp_partial_average(slot, rep.flat, rep._peers_arr, len(rep.peers) + 1, 0, rep.flat, rep.stats if with_stats else None)
            c.ddp_unpack(slot, rep.flat)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            c.ddp_local_update(rep.opt_struct(r + 1))
            e1.record(stream)
            evs.append((e0, e1))
        torch.cuda.synchronize()
        wall4 = time.perf_counter() - t0
        nbytes = float(sum(sum(algorithmic_bytes(w, rep.slot_numel[r % Hn]).values()) for r in range(args.warmup, args.warmup + args.steps)))
        upd_ms = sum(a.elapsed_time(b) for a, b in evs) / len(evs)
        for r in range(Hn):
            rep.fused_step(r, with_stats=with_stats)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for r in range(Hn, Hn + args.steps):
            rep.fused_step(r, with_stats=with_stats)
        torch.cuda.synchronize()
        wallf = time.perf_counter() - t0
        upd_bytes = algorithmic_bytes(w, 0)["local_update"]
        return {"value": nbytes / wall4 / 1e9, "unit": "GB/s", "pct_of_peak": 100.0 * nbytes / wall4 / 1e9 / HBM_PEAK_GBS,
                "ms_per_step": 1e3 * wall4 / args.steps, "fused_ms_per_step": 1e3 * wallf / args.steps,
                "local_update_GBps": upd_bytes / (upd_ms * 1e-3) / 1e9, "local_update_frac_of_peak": upd_bytes / (upd_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                "placement": "first allocation of the slab, nothing left unused, no probing"}

    # First the plain way: one slab, first allocation, nothing left unused, no probing of the physical placement.  For
    # models of a billion parameters or more the timed replica is then re-allocated by the harness's placement search
    # (0 / 16 / 24 / 32 / 40 GiB left unused in front of the data, the placement that streams fastest is kept): `value`
    # is measured on that one, and the plain figures are reported beside it as `no_placement_search`.
    use_search = w.n_params >= 1_000_000_000 and not args.no_placement_search and args.front_pad_gib is None
    rep = DeviceReplica(w, 0, options=options, policy=args.policy, wire16=args.wire16, placement_probe=False,
                        front_pad=(args.front_pad_gib or 0) << 30)
    stage_inputs(rep)
    first = None
    if use_search:
        first = plain_measurement(rep)
        rep.close()
        rep._release()
        rep.ctx.close()
        del rep
        import gc
        gc.collect()
        torch.cuda.empty_cache()
        rep = DeviceReplica(w, 0, options=options, policy=args.policy, wire16=args.wire16, placement_probe="search")
        stage_inputs(rep)

    if args.calibrate_copy:
        from paper_2502_11058_amd import binding as B
        src = torch.full((1 << 28,), 1.5, dtype=torch.float32, device=rep.dev)      # 1 GiB read, 1 GiB written per copy
        dst = torch.empty_like(src)
        for _ in range(4):
            B.ddp_stream_probe([src], [dst], 1 << 30, 8192, 65536)
        torch.cuda.synchronize()
        del src, dst

    H = len(rep.sets)
    for r in range(args.warmup):
        rep.step(r, with_stats=with_stats)
    torch.cuda.synchronize()

    # ---- pass 1: K steps, wall clock ------------------------------------------------------------------------------
    r0 = args.warmup
    t0 = time.perf_counter()
    for r in range(r0, r0 + args.steps):
        rep.step(r, with_stats=with_stats)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    step_bytes = [sum(algorithmic_bytes(w, rep.slot_numel[r % H]).values()) for r in range(r0, r0 + args.steps)]
    total_bytes = float(sum(step_bytes))
    gbs = total_bytes / wall / 1e9

    # ---- pass 2: the same K steps with an event between the calls (per-kernel durations on the launch stream) -----
    stream = torch.cuda.current_stream()
    names = ["pack", "partial_average", "unpack", "local_update"]
    evs = []
    r1 = r0 + args.steps
    for r in range(r1, r1 + args.steps):
        slot = r % H
        e = [torch.cuda.Event(enable_timing=True) for _ in range(5)]
        c = rep.ctx
        e[0].record(stream)
        c.ddp_pack(slot, rep.flat)
        e[1].record(stream)
        c.ddp_partial_average(slot, rep.flat, rep.peers, len(rep.peers) + 1, 0, rep.flat, rep.stats if with_stats else None)
        e[2].record(stream)
        c.ddp_unpack(slot, rep.flat)
        e[3].record(stream)
        c.ddp_local_update(rep.opt_struct(r + 1))
        e[4].record(stream)
        evs.append((slot, e))
    torch.cuda.synchronize()
    kern = {n: {"ms": 0.0, "bytes": 0.0, "launches": 0} for n in names}
    step_ms = sorted(e[0].elapsed_time(e[4]) for _, e in evs)           # one step = first to last event of its four calls
    for slot, e in evs:
        ab = algorithmic_bytes(w, rep.slot_numel[slot])
        for i, n in enumerate(names):
            kern[n]["ms"] += e[i].elapsed_time(e[i + 1])
            kern[n]["bytes"] += ab[n]
            kern[n]["launches"] += 1
    kernels = {}
    for n in names:
        k = kern[n]
        ms = k["ms"] / max(k["launches"], 1)
        kernels[n] = {"avg_ms": ms, "GB/s": (k["bytes"] / (k["ms"] * 1e-3) / 1e9) if k["ms"] > 0 else None,
                      "alg_bytes_per_launch": k["bytes"] / max(k["launches"], 1)}
    dom = "local_update"
    achieved = kernels[dom]["GB/s"]
    traffic = measured_traffic(w.name, dom, options)
    roofline = {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBS, "traffic": traffic["bytes_per_launch"] if traffic else None,
                "traffic_source": (f"{os.path.relpath(TRAFFIC_FILE, ROOT)}: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run "
                                   f"(commit {traffic.get('commit')}), not this run") if traffic else None,
                "alg_bytes_per_launch": kernels[dom]["alg_bytes_per_launch"], "avg_launch_ms": kernels[dom]["avg_ms"]}

    # ---- pass 3: the fused entry point (both cases of Eq. (5) in one pass), K steps, wall clock --------------------
    r2 = r1 + args.steps
    for r in range(r2, r2 + H):
        rep.fused_step(r, with_stats=with_stats)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for r in range(r2 + H, r2 + H + args.steps):
        rep.fused_step(r, with_stats=with_stats)
    torch.cuda.synchronize()
    wall_f = time.perf_counter() - t0
    upd_per_param = algorithmic_bytes(w, 0)["local_update"] / w.n_params
    fused_bytes = float(sum(4 * (w.n_replicas - 1) * rep.slot_numel[r % H] + upd_per_param * w.n_params
                            for r in range(r2 + H, r2 + H + args.steps)))
    fused = {"entry_point": "ddp_fused_sync_update", "ms_per_step": 1e3 * wall_f / args.steps,
             "value_vs_4call_bytes": total_bytes / wall_f / 1e9, "own_alg_bytes_per_step_avg": fused_bytes / args.steps,
             "GB/s_on_own_bytes": fused_bytes / wall_f / 1e9, "params_per_s": w.n_params * args.steps / wall_f}

    # ---- optional pass 4: bf16 on the wire (2 bytes per peer element instead of 4) ---------------------------------
    wire16 = None
    if args.wire16:
        wire16 = {}
        r3 = r2 + H + args.steps
        for name, fn in (("four_calls", rep.step), ("fused", rep.fused_step)):
            for r in range(r3, r3 + H):
                fn(r, with_stats=with_stats, wire16=True)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for r in range(r3 + H, r3 + H + args.steps):
                fn(r, with_stats=with_stats, wire16=True)
            torch.cuda.synchronize()
            wl = time.perf_counter() - t0
            S_sum = float(sum(rep.slot_numel[r % H] for r in range(r3 + H, r3 + H + args.steps)))
            upd = upd_per_param * w.n_params * args.steps
            # four calls: pack 4S+2S, average 2NS+4S, unpack 4S + (4+2)S; fused: 2(N-1)S on top of the update
            own = (6 + 2 * w.n_replicas + 4 + 4 + 4 + (2 if rep.bf16 else 0)) * S_sum + upd if name == "four_calls" \
                else 2 * (w.n_replicas - 1) * S_sum + upd
            wire16[name] = {"ms_per_step": 1e3 * wl / args.steps, "own_alg_bytes_per_step_avg": own / args.steps,
                            "GB/s_on_own_bytes": own / wl / 1e9, "params_per_s": w.n_params * args.steps / wl}

    # ---- optional pass 5: layer-wise launches under a synthetic backward pass (Sec. 3.2) ----------------------------
    overlap = None
    if args.overlap:
        side = torch.cuda.Stream()
        D = args.overlap_mm
        A = torch.randn(D, D, device=rep.dev, dtype=torch.bfloat16)
        Bm = torch.randn(D, D, device=rep.dev, dtype=torch.bfloat16)
        Cm = torch.empty(D, D, device=rep.dev, dtype=torch.bfloat16)
        lay = w.layer_numel()
        # stand-in for a layer's BP: 4 flop per parameter and token, 4096 tokens, as D^3 products
        n_mm = [max(1, round(4 * n * 4096 / (2 * 4096 ** 3))) for n in lay]

        def bp(l):
            for _ in range(n_mm[l]):
                torch.mm(A, Bm, out=Cm)

        def timed(fn):
            for r in range(H):
                fn(r)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for r in range(args.steps):
                fn(r)
            torch.cuda.synchronize()
            return 1e3 * (time.perf_counter() - t0) / args.steps

        r4 = 10_000
        bp_ms = timed(lambda r: [bp(l) for l in range(w.n_layers - 1, -1, -1)])
        fused_ms = timed(lambda r: rep.fused_step(r4 + r, with_stats=with_stats))
        serial_ms = timed(lambda r: rep.layerwise_step(r4 + r, torch.cuda.current_stream(), backward=lambda l: None,
                                                       with_stats=with_stats))
        both_ms = timed(lambda r: rep.layerwise_step(r4 + r, side, backward=bp, with_stats=with_stats))
        overlap = {"synthetic_bp_ms": bp_ms, "fused_one_launch_ms": fused_ms, "fused_layerwise_same_stream_ms": serial_ms,
                   "bp_with_layerwise_sync_on_side_stream_ms": both_ms,
                   "hidden_fraction_of_sync_update": (bp_ms + serial_ms - both_ms) / serial_ms,
                   "bp_flop_per_step": float(sum(n_mm)) * 2 * D ** 3, "product_edge": D}
        # The same with the chip divided between the two streams: the side stream (sync + update of the layers whose
        # gradients are ready) owns R compute units, the backward pass the others.  What is reported against the undivided
        # chip: how much longer the backward pass takes on fewer CUs, how long sync + update take on R CUs alone, and the
        # time of the two together; "hidden" = time saved against running them one after the other on the whole chip.
        from paper_2502_11058_amd import binding as B
        ncu = B.ddp_device_cu_count(0)
        rows = []
        for R in [int(x) for x in args.overlap_side_cus.split(",") if x]:
            if R <= 0 or R >= ncu:
                continue
            side_h = B.ddp_stream_create_cu_range(0, 0, R)
            main_h = B.ddp_stream_create_cu_range(0, R, ncu - R)
            side_r, main_r = torch.cuda.ExternalStream(side_h), torch.cuda.ExternalStream(main_h)
            with torch.cuda.stream(main_r):
                bp_r = timed(lambda r: [bp(l) for l in range(w.n_layers - 1, -1, -1)])
                both_r = timed(lambda r: rep.layerwise_step(r4 + r, side_r, backward=bp, with_stats=with_stats))
            with torch.cuda.stream(side_r):
                alone_r = timed(lambda r: rep.layerwise_step(r4 + r, side_r, backward=lambda l: None, with_stats=with_stats))
            torch.cuda.synchronize()
            B.ddp_stream_destroy(side_h)
            B.ddp_stream_destroy(main_h)
            rows.append({"side_cus": R, "backward_cus": ncu - R, "bp_ms": bp_r, "bp_slowdown": bp_r / bp_ms,
                         "sync_update_alone_ms": alone_r, "sync_update_GBps": fused["own_alg_bytes_per_step_avg"] / alone_r / 1e6,
                         "bp_and_sync_update_ms": both_r,
                         "hidden_fraction_of_sync_update": (bp_ms + serial_ms - both_r) / serial_ms})
        overlap["cu_partition"] = rows

    cpu = None if args.no_cpu_baseline else cpu_baseline(rep, w)

    out = {
        "metric": "partial-sync+update step: achieved HBM GB/s & % of peak; params/s",
        "value": gbs, "unit": "GB/s", "pct_of_peak": 100.0 * gbs / HBM_PEAK_GBS,
        "params_per_s": w.n_params * args.steps / wall,
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": 1e3 * wall / args.steps,
        "step_ms_event_timed": {"median": step_ms[len(step_ms) // 2], "min": step_ms[0], "max": step_ms[-1]},
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: P={w.n_params}, N={w.n_replicas}, H={w.period}, {w.param_dtype} params, "
                               f"{w.optimizer}, schedule {args.policy or w.policy}, slot sizes {rep.slot_numel}",
                   "alg_bytes_per_step_avg": total_bytes / args.steps, "layer_stats": with_stats, "options": options,
                   "placement": (f"harness placement search: kept {rep.placement.get('kept_GiB', 0)} GiB unused in front of the "
                                 f"data, tried {rep.placement.get('front_pad_GiB')} GiB, zero-slab probe readings "
                                 f"{[round(x, 1) for x in rep.placement['probe_GBps']]} GB/s; the plain first allocation is in no_placement_search")
                   if first is not None else ("first allocation, no search" if args.front_pad_gib is None else f"front pad {args.front_pad_gib} GiB"),
                   "placement_kept_GiB": rep.placement.get("kept_GiB", 0) if first is not None else (args.front_pad_gib or 0)},
        "kernels": kernels, "roofline": roofline, "fused": fused,
    }
    if first is not None:
        out["value_no_placement_search"] = first["value"]
        out["no_placement_search"] = first
    out["config"]["clocks"] = gpu_clocks()
    if wire16 is not None:
        out["wire16"] = wire16
    if overlap is not None:
        out["overlap"] = overlap
    if cpu is not None:
        out["cpu_baseline"] = cpu
    print(json.dumps(out))
    rep.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
