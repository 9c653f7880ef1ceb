"""Pins for the oracle's replica average (Eq. (5), second case) and the per-layer divergence Gamma."""
import numpy as np
import pytest


def _rand(n, seed, scale=0.02):
    return (np.random.default_rng(seed).standard_normal(n) * scale).astype(np.float32)


@pytest.mark.parametrize("N", [1, 2, 4])
def test_identical_replicas_are_unchanged_up_to_four(oracle, N):
    # x, 2x are exact; 3x rounds by at most 2 ulp(x), and adding x lands on 4x again (ties fall on 4x too)
    x = _rand(100003, 1)
    out = oracle.mean([x.copy() for _ in range(N)])
    assert np.array_equal(out.view(np.uint32), x.view(np.uint32))


@pytest.mark.parametrize("N", [2, 4, 8, 16, 32])
def test_identical_short_mantissa_replicas_are_unchanged(oracle, N):
    # 10-bit integers over 64: every partial sum k*x (k <= 32) is exact in fp32, so averaging is the identity
    x = (np.arange(-512, 512, dtype=np.float32) / 64.0)
    out = oracle.mean([x.copy() for _ in range(N)])
    assert np.array_equal(out.view(np.uint32), x.view(np.uint32))


@pytest.mark.parametrize("N", [3, 5, 8, 16])
def test_identical_replicas_general_within_rounding(oracle, N):
    # partial sums k*x round; the result stays within N/2 ulp of x
    x = _rand(10007, 2)
    out = oracle.mean([x.copy() for _ in range(N)])
    ulp = np.spacing(np.abs(x))
    assert np.all(np.abs(out.astype(np.float64) - x) <= 0.5 * N * ulp)


def test_dyadic_closed_form(oracle):
    # values k/64 and a per-replica shift j/8 are exact in fp32, sums stay exact: mean = x + (N-1)/16
    N = 8
    base = (np.arange(-500, 500, dtype=np.float32) / 64.0)
    reps = [base + np.float32(j / 8.0) for j in range(N)]
    out = oracle.mean(reps)
    expect = base + np.float32(sum(j / 8.0 for j in range(N)) / N)
    assert np.array_equal(out, expect)


def test_sum_is_taken_in_rank_order(oracle):
    # ((1e8 + 1) - 1e8) = 0 in fp32 because 1e8 + 1 rounds back to 1e8; any order that cancels the big
    # terms first would give 1.  Divisor 4 keeps the scaling exact.
    a, b, c, d = np.float32([1e8]), np.float32([1.0]), np.float32([-1e8]), np.float32([0.0])
    assert oracle.mean([a, b, c, d])[0] == 0.0
    assert oracle.mean([a, c, b, d])[0] == 0.25
    assert oracle.mean([b, a, c, d])[0] == 0.0
    assert oracle.mean([a, c, d, b])[0] == 0.25


@pytest.mark.parametrize("N", [2, 3, 4, 7, 8, 16])
def test_close_to_exact_mean(oracle, N):
    reps = [_rand(4099, 10 + k) for k in range(N)]
    out = oracle.mean(reps).astype(np.float64)
    exact = np.mean(np.stack([r.astype(np.float64) for r in reps]), axis=0)
    # N-1 additions and one multiply (plus 1/N rounding for non powers of two), each within half an ulp
    bound = (N + 1) * np.finfo(np.float32).eps * np.max(np.abs(np.stack(reps)), axis=0) * 1.0 + 1e-30
    assert np.all(np.abs(out - exact) <= bound)


def test_mean_may_alias_an_input(oracle):
    import ctypes as C
    reps = [_rand(1000, 20 + k) for k in range(4)]
    expect = oracle.mean(reps)
    ptrs = (C.c_void_p * 4)(*[r.ctypes.data for r in reps])
    oracle.lib().orc_mean(4, ptrs, C.c_int64(1000), reps[2].ctypes.data_as(C.c_void_p))
    assert np.array_equal(reps[2], expect)


def test_stats_match_direct_fp64_definition(oracle):
    N, n = 5, 3001
    reps = [_rand(n, 30 + k) for k in range(N)]
    m = oracle.mean(reps)
    g, msq = oracle.layer_stats(reps, m, 100, 2900)
    X = np.stack(reps)[:, 100:2900]
    d = (m[None, 100:2900] - X).astype(np.float64)          # difference formed in fp32, as the definition says
    assert g == pytest.approx(float((d * d).sum() / N), rel=1e-13)
    assert msq == pytest.approx(float((m[100:2900].astype(np.float64) ** 2).sum()), rel=1e-13)


def test_stats_zero_for_identical_replicas_and_empty_range(oracle):
    x = _rand(513, 3)
    reps = [x.copy() for _ in range(4)]
    m = oracle.mean(reps)
    g, msq = oracle.layer_stats(reps, m, 0, 513)
    assert g == 0.0 and msq > 0.0
    assert oracle.layer_stats(reps, m, 7, 7) == (0.0, 0.0)


def test_stats_variance_decomposition(oracle):
    # (1/N) sum_k ||x_k - mean||^2 = (1/N) sum_k ||x_k||^2 - ||mean||^2, evaluated independently in fp64
    N, n = 8, 20000
    reps = [_rand(n, 40 + k, 1.0) for k in range(N)]
    m = oracle.mean(reps)
    g, msq = oracle.layer_stats(reps, m, 0, n)
    X = np.stack(reps).astype(np.float64)
    rhs = (X * X).sum() / N - (X.mean(axis=0) ** 2).sum()
    assert g == pytest.approx(rhs, rel=1e-5)


def test_gamma_expectation_for_drifted_peers(oracle):
    # local + iid N(0, s^2) drift on the N-1 peers.  Per element the replicas are {0, d_1..d_{N-1}} + local:
    # (1/N) sum d_j^2 - (sum d_j / N)^2 has expectation s^2 (N-1)/N - s^2 (N-1)/N^2 = s^2 (N-1)^2 / N^2
    N, n, s = 8, 400000, 1e-3
    local = _rand(n, 50)
    rng = np.random.default_rng(51)
    reps = [local] + [local + (rng.standard_normal(n) * s).astype(np.float32) for _ in range(N - 1)]
    m = oracle.mean(reps)
    g, _ = oracle.layer_stats(reps, m, 0, n)
    assert g == pytest.approx(n * s * s * (N - 1) ** 2 / N ** 2, rel=0.02)


def test_stats_running_sums_do_not_drift(oracle):
    # Gamma is a mathematical sum (Sec. 3.4); the oracle's accumulators are extended precision so that 3e7 terms
    # agree with numpy's pairwise fp64 sum to 1e-12 (a plain fp64 running sum is off by ~3e-11 here and by
    # 5e-10 at the size of a 65 M-element layer)
    N, n = 8, 4_000_000
    rng = np.random.default_rng(60)
    loc = (rng.standard_normal(n) * 0.02).astype(np.float32)
    reps = [loc] + [loc + (rng.standard_normal(n) * 1e-4).astype(np.float32) for _ in range(N - 1)]
    m = oracle.mean(reps)
    g, msq = oracle.layer_stats(reps, m, 0, n)
    d = (m[None, :] - np.stack(reps)).astype(np.float64)
    assert g == pytest.approx(float((d * d).sum() / N), rel=1e-12)
    assert msq == pytest.approx(float((m.astype(np.float64) ** 2).sum()), rel=1e-12)
