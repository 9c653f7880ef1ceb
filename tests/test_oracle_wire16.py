"""Pins for the oracle's bf16-on-the-wire averaging: it must be the pinned fp32 average applied to the pinned
bf16 rounding of every replica (the local one included), nothing else."""
import numpy as np
import pytest


def _rand(n, seed, scale=0.02):
    return (np.random.default_rng(seed).standard_normal(n) * scale).astype(np.float32)


@pytest.mark.parametrize("N", [1, 2, 3, 8, 16])
def test_wire16_mean_is_fp32_mean_of_rounded_replicas(oracle, N):
    reps = [_rand(20011, 70 + k) for k in range(N)]
    wire = [oracle.bf16_rne(r) for r in reps]
    out = oracle.mean_wire16(wire)
    ref = oracle.mean([oracle.bf16_widen(w) for w in wire])
    assert np.array_equal(out.view(np.uint32), ref.view(np.uint32))


def test_wire16_identical_replicas_give_the_rounded_value(oracle):
    # k * (8-bit mantissa value) is exact in fp32 for k <= 64, so the average of identical replicas is the bf16 value
    x = _rand(30011, 80)
    w = oracle.bf16_rne(x)
    for N in (2, 4, 8, 64):
        out = oracle.mean_wire16([w.copy() for _ in range(N)])
        assert np.array_equal(out.view(np.uint32), oracle.bf16_widen(w).view(np.uint32))
    # and it is NOT the unrounded value: the wire is lossy by design
    assert not np.array_equal(oracle.mean_wire16([w, w]), x)


def test_wire16_pack_rounds_each_element_and_keeps_the_layout(oracle):
    ts = [_rand(5, 81), _rand(257, 82), _rand(1, 83)]
    off = [3, 8, 300]
    flat = oracle.pack_wire16(ts, off, 301)
    for t, o in zip(ts, off):
        assert np.array_equal(flat[o:o + t.size], oracle.bf16_rne(t))
    assert flat[:3].tolist() == [0, 0, 0]


def test_wire16_stats_against_direct_evaluation(oracle):
    N, n = 4, 5003
    wire = [oracle.bf16_rne(_rand(n, 90 + k)) for k in range(N)]
    m = oracle.mean_wire16(wire)
    g, msq = oracle.layer_stats_wire16(wire, m, 10, 5000)
    X = np.stack([oracle.bf16_widen(w) for w in wire])[:, 10:5000]
    d = (m[None, 10:5000] - X).astype(np.float64)
    assert g == pytest.approx(float((d * d).sum() / N), rel=1e-13)
    assert msq == pytest.approx(float((m[10:5000].astype(np.float64) ** 2).sum()), rel=1e-13)


def test_wire16_workers_agree_after_sync(oracle):
    # K workers, each averaging the same K wire buffers: bit-identical results although every local value was rounded
    K, n = 4, 4096
    layer_of = [0]
    workers = [oracle.Worker(layer_of, [_rand(n, 100 + k)], "sgdm", dict(lr=0.01, momentum=0.9), True) for k in range(K)]
    flats = [w.pack_slot([0], wire16=True)[0] for w in workers]
    res = [workers[k].sync([0], [flats[j] for j in range(K) if j != k], k, wire16=True) for k in range(K)]
    for k in range(1, K):
        assert np.array_equal(res[0][0], res[k][0]) and res[0][1] == res[k][1]
        assert np.array_equal(workers[0].p[0], workers[k].p[0]) and np.array_equal(workers[0].model[0], workers[k].model[0])
