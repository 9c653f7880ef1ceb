#!/usr/bin/env python3
"""Benchmark of one worker's partial-sync + update step (pack -> partial average -> unpack -> local update).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload llama2_7b]

A "step" is one iteration of Algorithm 1 for one worker: the four library calls for slot r mod H, with the
N-1 peer buffers, the gradients and all optimizer state already resident in HBM.  Inputs are seeded and
synthetic (shapes of the named model, Gaussian values).  Prints ONE JSON line.

  value      = algorithmic bytes of the K timed steps / wall time of the K steps, in GB/s (whole step, launch
               gaps included); also given as a fraction of the 8 TB/s peak and as parameters per second.
  roofline   = the dominant kernel (the fused optimizer update): algorithmic bytes per launch / its average
               duration measured with events on the launch stream in a second pass of K steps.
  cpu_baseline = the CPU oracle timed on this machine's host cores on a bounded sample (one transformer block).
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

# HBM bytes per launch of the update kernel measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by what
# the same counters read for a plain copy of known size (profiles/llama2_7b_step_kernels.txt); None if not measured
# (other workloads, or library options that differ from the defaults the measurement was taken with).
MEASURED_TRAFFIC_BYTES = {"llama2_7b": 188.681e9}


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


def cpu_baseline(rep, w, seconds_budget: float = 20.0):
    """Oracle on the host cores, on one transformer block of the same workload (same bytes as on the device)."""
    import numpy as np
    from oracle import plsgd as oracle
    cores = len(os.sched_getaffinity(0))
    cores = min(cores, int(os.environ.get("OMP_NUM_THREADS", cores)))
    oracle.set_threads(cores)
    layer = 1 if w.n_layers > 2 else 0
    ids = [i for i, t in enumerate(w.tensors) if t.layer == layer]

    def host(t):
        import torch
        if t.dtype == torch.bfloat16:
            return t.view(torch.int16).cpu().numpy().view(np.uint16)
        return t.cpu().numpy()

    hyper = dict(lr=w.lr, momentum=w.momentum, beta1=w.beta1, beta2=w.beta2, eps=w.eps, weight_decay=w.weight_decay)
    wk = oracle.Worker([0] * len(ids), [host(rep.sync[i]) for i in ids], w.optimizer, hyper, rep.bf16)
    grads = [host(rep.grad[i]) for i in ids]
    S = sum(rep.numel[i] for i in ids)
    rng = np.random.default_rng(0)
    flat0 = wk.pack_slot([0])[0]
    peers = [flat0 + (rng.standard_normal(S, dtype=np.float32) * np.float32(w.sigma_drift)) for _ in range(w.n_replicas - 1)]
    sub = type(w)(name="sample", tensors=[w.tensors[i] for i in ids], n_replicas=w.n_replicas, period=1, optimizer=w.optimizer,
                  param_dtype=w.param_dtype, lr=w.lr)
    nbytes = sum(algorithmic_bytes(sub, S).values())
    reps, t_total = 0, 0.0
    while reps < 2 or (t_total < seconds_budget / 2 and reps < 8):
        t0 = time.perf_counter()
        wk.step(reps, [[0]], peers, 0, grads)
        t_total += time.perf_counter() - t0
        reps += 1
    sec = t_total / reps
    return {"value": nbytes / sec / 1e9, "unit": "GB/s", "cores": cores, "kind": "oracle",
            "sample": f"one transformer block of {w.name} ({S} parameters, N={w.n_replicas}): pack + average + unpack + "
                      f"{w.optimizer} update, {reps} repetitions, {sec:.3f} s each",
            "params_per_s": S / sec}


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
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-stats", action="store_true", help="skip the per-layer statistics in the average")
    ap.add_argument("--option", action="append", default=[], help="library option name=value (repeatable)")
    ap.add_argument("--wire16", action="store_true",
                    help="also time the bf16-on-the-wire entry points (four calls and fused); reported in an extra "
                         "\"wire16\" object, never in value")
    ap.add_argument("--overlap", action="store_true",
                    help="also time the layer-wise launches of Sec. 3.2 on a side stream under a synthetic backward pass "
                         "(bf16 matrix products standing in for each layer's BP); extra \"overlap\" object, never in value")
    ap.add_argument("--overlap-mm", type=int, default=4096, metavar="D",
                    help="edge of the square bf16 products of --overlap (4096: one product fills the 256 CUs)")
    ap.add_argument("--front-pad-gib", type=int, default=None, metavar="G",
                    help="leave G GiB unused at the start of the worker's slab (default: let the harness search a few values "
                         "and keep the physical placement that streams fastest)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run 4 plain elementwise copies of 1 GiB (torch.add(src, 0, out=dst)) before the timed region, "
                         "as the known-size reference for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE readings")
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
    if args.front_pad_gib is None:
        rep = DeviceReplica(w, 0, options=options, policy=args.policy, wire16=args.wire16,
                            placement_probe="search" if w.n_params >= 1_000_000_000 else None)
    else:
        rep = DeviceReplica(w, 0, options=options, policy=args.policy, wire16=args.wire16, front_pad=args.front_pad_gib << 30)
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

    if args.calibrate_copy:
        src = torch.full((1 << 28,), 1.5, dtype=torch.float32, device=rep.dev)      # 1 GiB read, 1 GiB written per copy
        dst = torch.empty_like(src)
        for _ in range(4):
            torch.add(src, 0.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    H = len(rep.sets)
    with_stats = not args.no_stats
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
    roofline = {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBS, "traffic": MEASURED_TRAFFIC_BYTES.get(w.name) if not options else None,
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
                   "placement_probe_GBps": [round(x, 1) for x in rep.placement["probe_GBps"]],
                   "placement_front_pad_GiB": rep.placement.get("front_pad_GiB"), "placement_kept_GiB": rep.placement.get("kept_GiB", 0)},
        "kernels": kernels, "roofline": roofline, "fused": fused,
    }
    out["config"]["clocks"] = gpu_clocks()
    if wire16 is not None:
        out["wire16"] = wire16
    if overlap is not None:
        out["overlap"] = overlap
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(rep, w)
    print(json.dumps(out))
    rep.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
