"""Seeded random configurations through the whole path: random layer / tensor structure with sizes around every
vector, chunk and power-of-two boundary, random replica count, period, schedule policy, optimizer, precision, arena
alignment, chunk sizes, entry point (four calls / fused), wire precision and update order.  Each case runs three
iterations against the oracle, every element, bit for bit."""
import numpy as np
import pytest

from paper_2502_11058_amd import workloads as W
from test_gpu_parity import run_trajectory

pytestmark = pytest.mark.gpu

SIZES = [1, 2, 3, 4, 5, 7, 8, 9, 63, 64, 65, 255, 256, 257, 1023, 1024, 1025, 2047, 2048, 2049, 4095, 4096, 4097, 8191, 8193,
         65535, 65536, 65537, 100_003, 262_144, 500_001, 1_048_577]


def _case(seed):
    rng = np.random.default_rng(1000 + seed)
    L = int(rng.integers(1, 7))
    ts = []
    for l in range(L):
        for j in range(int(rng.integers(1, 5))):
            ts.append(W.TensorSpec(f"l{l}.t{j}", l, int(rng.choice(SIZES))))
    adam = bool(rng.integers(0, 2))
    bf16 = bool(rng.integers(0, 2))
    H = int(rng.integers(1, 5))
    policy = str(rng.choice(["enp", "round_robin", "full", "every", "opt", "alg2", "enp+fill", "opt+fill"]))
    w = W.Workload(f"fuzz{seed}", ts, n_replicas=int(rng.choice([1, 2, 3, 4, 5, 8, 11, 16, 19, 32])), period=H,
                   optimizer="adamw" if adam else "sgdm", param_dtype="bf16" if bf16 else "f32", lr=3e-4 if adam else 0.01,
                   sigma_drift=1e-4, sigma_grad=1e-3, iterations=3, policy=policy, time_noise=True)
    w.extra["comm_ns_per_byte"] = float(rng.choice([0.3, 2.0, 8.0]))          # light communication leaves bubbles to fill
    fused = bool(rng.integers(0, 2))
    kw = dict(arena_offset=int(rng.integers(0, 4)), fused=fused, wire16=bool(rng.integers(0, 2)),
              order=int(rng.integers(0, 2)) if fused else 0,
              options={"update_chunk": int(rng.choice([1024, 2048, 4096])), "mean_chunk": int(rng.choice([1024, 2048, 8192])),
                       "copy_chunk": int(rng.choice([1024, 2048, 4096])), "dense_path": int(rng.integers(0, 2))})
    return w, kw


@pytest.mark.parametrize("seed", range(128))
def test_random_configuration(oracle, seed):
    w, kw = _case(seed)
    t = run_trajectory(oracle, w, iters=3, **kw)
    assert t.frac() == 1.0, (w.name, kw)
