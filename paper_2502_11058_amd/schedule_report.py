"""Schedule quality on synthetic profiles, after the paper's Fig. 15: communication time that is not hidden by
the backward pass, for the equal-number partition, Algorithm 2 and the exact optimum of Eq. (8), as the number
of layers grows (H = 5) and as the bandwidth changes; and, after its Fig. 16, the size of Algorithm 2's solution set
and the search times against the number of cuts a brute-force search visits.  CPU only; uses the library's scheduler
entry points.

    python -m paper_2502_11058_amd.schedule_report
"""
from __future__ import annotations

import numpy as np

from . import binding as B
from . import workloads as W


def exposed(policy: str, fp, bp, comm, H: int, fill: bool = False):
    """(Eq. (8) cost, exposed communication per period under Eq. (7), period time)."""
    L = len(bp)
    _, sp, sl, cost = B.ddp_schedule(policy, L, H, fp, bp, comm)
    if fill:
        sp, sl, _ = B.ddp_schedule_fill_bubbles(bp, comm, sp, sl)
    it, ex, period = B.ddp_schedule_time_model(fp, bp, comm, sp, sl)
    return cost, int(ex.sum()), period


def layers_sweep(H: int = 5, trials: int = 200, seed: int = 0):
    rng = np.random.default_rng(seed)
    rows = []
    for L in (6, 10, 14, 18, 22, 26, 30):
        same = worse = 0
        tot = {"enp": 0.0, "alg2": 0.0, "opt": 0.0}
        for _ in range(trials):
            nbytes = rng.integers(1 << 18, 1 << 24, L).astype(np.float64)
            bp = np.rint(2.0 * nbytes * rng.uniform(0.8, 1.2, L)).astype(np.int64)
            fp = bp // 2
            comm = np.rint(rng.uniform(2.0, 10.0) * nbytes).astype(np.int64)
            c = {p: exposed(p, fp, bp, comm, H) for p in tot}
            base = H * int(bp.sum())
            for p in tot:
                tot[p] += (c[p][0] - base) / base          # Eq. (8) excess relative to the backward time of a period
            same += c["alg2"][0] == c["opt"][0]
            worse += c["alg2"][0] > c["opt"][0]
        rows.append((L, tot["enp"] / trials, tot["alg2"] / trials, tot["opt"] / trials, same / trials))
    return rows


def bandwidth_sweep(name: str = "gpt2_small"):
    w = W.get(name)
    rows = []
    for ns_per_byte in (64.0, 16.0, 8.0, 4.0, 2.0, 1.0, 0.5):
        w.extra["comm_ns_per_byte"] = ns_per_byte
        fp, bp, comm = W.synthetic_times(w)
        r = {p: exposed(p, fp, bp, comm, w.period) for p in ("full", "enp", "alg2", "opt")}
        rows.append((8.0 / ns_per_byte, *(r[p][2] / 1e6 for p in ("full", "enp", "alg2", "opt"))))
    return rows


def complexity_sweep(trials: int = 20, seed: int = 1):
    """Per (L, H): cuts a brute force visits, C(L+H-1, H-1); the bound 2^min(L-1, H-1) on Algorithm 2's solution set;
    the largest solution set seen over random profiles; median search time of Algorithm 2 and of the exact DP."""
    import math
    import time
    rng = np.random.default_rng(seed)
    rows = []
    for L, H in ((8, 4), (16, 4), (32, 4), (32, 8), (64, 8), (128, 8), (128, 16), (256, 16)):
        sizes, t_alg2, t_opt = [], [], []
        for _ in range(trials):
            nbytes = rng.integers(1 << 18, 1 << 24, L).astype(np.float64)
            bp = np.rint(2.0 * nbytes * rng.uniform(0.8, 1.2, L)).astype(np.int64)
            comm = np.rint(rng.uniform(2.0, 10.0) * nbytes).astype(np.int64)
            sizes.append(B.ddp_schedule_alg2_solutions(bp, comm, H))
            for pol, acc in (("alg2", t_alg2), ("opt", t_opt)):
                t0 = time.perf_counter()
                B.ddp_schedule(pol, L, H, bp // 2, bp, comm)
                acc.append(time.perf_counter() - t0)
        rows.append((L, H, math.comb(L + H - 1, H - 1), 2 ** min(L - 1, H - 1), max(sizes), 1e6 * float(np.median(t_alg2)),
                     1e6 * float(np.median(t_opt))))
    return rows


def main() -> None:
    print("Excess of Eq. (8) over H backward passes (mean over 200 random profiles, H = 5), relative to H*t_BP")
    print(f"{'L':>3s} {'ENP':>8s} {'ALG2':>8s} {'OPT':>8s}  ALG2 == OPT")
    for L, e, a, o, same in layers_sweep():
        print(f"{L:3d} {e:8.4f} {a:8.4f} {o:8.4f}  {100 * same:5.1f} %")
    print("\nGPT-2-small-shaped profile, period time under Eq. (7) in ms vs bandwidth (Gbit/s)")
    print(f"{'Gbps':>6s} {'FULL':>9s} {'ENP':>9s} {'ALG2':>9s} {'OPT':>9s}")
    for g, f, e, a, o in bandwidth_sweep():
        print(f"{g:6.2f} {f:9.1f} {e:9.1f} {a:9.1f} {o:9.1f}")
    print("\nSearch effort: brute-force cuts, bound and largest observed size of Algorithm 2's solution set, search times")
    print(f"{'L':>4s} {'H':>3s} {'brute-force cuts':>18s} {'2^min(L-1,H-1)':>15s} {'max |Omega|':>12s} {'ALG2 us':>9s} {'OPT us':>9s}")
    for L, H, cuts, bound, size, ta, to in complexity_sweep():
        print(f"{L:4d} {H:3d} {cuts:18.3e} {bound:15d} {size:12d} {ta:9.1f} {to:9.1f}")


if __name__ == "__main__":
    main()
