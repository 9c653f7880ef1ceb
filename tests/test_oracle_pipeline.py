"""Pins for the oracle's iteration (Algorithm 1, Definition 1 / Eq. (5)) using K workers in one process:
the two limits of partial synchronisation, the once-per-period property, and the flat layout."""
import numpy as np
import pytest
import torch

from paper_2502_11058_amd import workloads as W


def _init(w, oracle, K, seed_kind="param", optimizer=None, hyper=None, bf16=None):
    params = []
    for i, t in enumerate(w.tensors):
        x = torch.empty(t.numel, dtype=torch.float32)
        W.normal_(x, w.sigma_param, W.seed_for(w.base_seed, w.name, seed_kind, 0, 0, i))
        params.append(x.numpy())
    layer_of = [t.layer for t in w.tensors]
    hyper = hyper or dict(lr=w.lr, momentum=w.momentum, beta1=w.beta1, beta2=w.beta2, eps=w.eps,
                          weight_decay=w.weight_decay)
    opt = optimizer or w.optimizer
    bf = (w.param_dtype == "bf16") if bf16 is None else bf16
    return [oracle.Worker(layer_of, params, opt, hyper, bf) for _ in range(K)]


def _grads(w, r, k):
    out = []
    for i, t in enumerate(w.tensors):
        x = torch.empty(t.numel, dtype=torch.float32)
        W.normal_(x, w.sigma_grad, W.seed_for(w.base_seed, w.name, "grad", r, k, i))
        out.append(x.numpy())
    return out


def test_tiny_shape_and_offsets(oracle):
    w = W.tiny()
    assert w.n_params == 526336 and w.n_layers == 8
    sets = oracle.schedule("enp", 8, 4)
    assert sets == [[7, 6], [5, 4], [3, 2], [1, 0]]
    layer_of = [t.layer for t in w.tensors]
    numel = [t.numel for t in w.tensors]
    for S in sets:
        off, order, total = oracle.slot_offsets(layer_of, numel, S)
        assert total == 131584
        # brute force: walk the set, then the tensors, and count
        expect, o = {}, 0
        for l in S:
            for t in range(len(numel)):
                if layer_of[t] == l:
                    expect[t] = o
                    o += numel[t]
        assert order.tolist() == list(expect.keys())
        assert all(off[t] == expect.get(t, -1) for t in range(len(numel)))


def test_model_sizes():
    assert W.gpt2_small().n_params == 124355328 and W.gpt2_small().n_layers == 14
    assert W.gpt2_small(with_biases=True).n_params == 124439808
    assert W.tinyllama_1b().n_params == 1100048384 and W.tinyllama_1b().n_layers == 24
    assert W.llama2_7b().n_params == 6738415616 and W.llama2_7b().n_layers == 34
    assert W.llama3_8b().n_params == 8030261248 and W.llama3_8b().n_layers == 34


@pytest.mark.parametrize("policy", ["enp", "round_robin", "full", "opt", "alg2"])
def test_every_layer_synchronised_once_per_period(oracle, policy):
    w = W.small_llama()
    _, bp, comm = W.synthetic_times(w)
    for H in (1, 2, 3, 4, 6):
        sets = oracle.schedule(policy, w.n_layers, H, bp, comm)
        assert len(sets) == H
        flat = [l for S in sets for l in S]
        assert sorted(flat) == list(range(w.n_layers))


def test_pack_unpack_roundtrip_and_untouched_tensors(oracle):
    w = W.odd(optimizer="sgdm", param_dtype="bf16")
    wk = _init(w, oracle, 1)[0]
    before = [p.copy() for p in wk.p]
    S = [4, 1, 3]
    flat, off, order, total = wk.pack_slot(S)
    assert total == sum(t.numel for t in w.tensors if t.layer in S)
    # flat is the plain concatenation in set order
    cat = np.concatenate([before[i] for l in S for i, t in enumerate(w.tensors) if t.layer == l])
    assert np.array_equal(flat, cat)
    wk.unpack_slot(flat + np.float32(1.0), off, order)
    for i, t in enumerate(w.tensors):
        if t.layer in S:
            assert np.array_equal(wk.p[i], before[i] + np.float32(1.0))
            assert np.array_equal(wk.model[i], oracle.bf16_rne(wk.p[i]))
        else:
            assert np.array_equal(wk.p[i], before[i])
            assert np.array_equal(wk.model[i], oracle.bf16_rne(before[i]))


def test_every_iteration_sync_without_momentum_is_synchronous_sgd(oracle):
    # Eq. (1): w <- w - eta * mean_k g_k.  Averaging the K locally updated models equals this up to rounding,
    # and all workers hold bit-identical models after every iteration.
    w = W.tiny()
    K, R = 4, 6
    hyper = dict(lr=0.01, momentum=0.0)
    workers = _init(w, oracle, K, hyper=hyper)
    ref = [p.astype(np.float64) for p in workers[0].p]
    sets = oracle.schedule("every", w.n_layers, w.period)
    for r in range(R):
        grads = [_grads(w, r, k) for k in range(K)]
        oracle.run_workers(workers, r, sets, grads, order=oracle.UPDATE_THEN_SYNC)
        for i in range(len(ref)):
            ref[i] = ref[i] - float(np.float32(0.01)) * np.mean([g[i].astype(np.float64) for g in grads], axis=0)
        for k in range(1, K):
            for a, b in zip(workers[0].p, workers[k].p):
                assert np.array_equal(a, b)
    for a, b in zip(workers[0].p, ref):
        assert np.allclose(a, b, rtol=0, atol=R * 4 * 6e-8 * 0.1)


@pytest.mark.parametrize("mu", [0.0, 0.9])
def test_full_schedule_is_local_sgd(oracle, mu):
    # Eq. (2) written directly on whole-model vectors, no layers, no packing: local step every iteration,
    # replace by the rank-ordered average when (r+1) % H == 0.
    w = W.tiny()
    K, H, R = 4, 4, 9
    hyper = dict(lr=0.01, momentum=mu)
    workers = _init(w, oracle, K, hyper=hyper)
    vec = [np.concatenate(wk.p) for wk in workers]
    buf = [np.zeros_like(v) for v in vec]
    sets = oracle.schedule("full", w.n_layers, H)
    f = np.float32
    for r in range(R):
        grads = [_grads(w, r, k) for k in range(K)]
        oracle.run_workers(workers, r, sets, grads, order=oracle.UPDATE_THEN_SYNC)
        for k in range(K):
            g = np.concatenate(grads[k])
            buf[k] = f(mu) * buf[k] + g
            vec[k] = vec[k] - f(0.01) * buf[k]
        if (r + 1) % H == 0:
            acc = vec[0].copy()
            for k in range(1, K):
                acc = acc + vec[k]
            avg = acc * f(1.0 / K)
            vec = [avg.copy() for _ in range(K)]
        for k in range(K):
            assert np.array_equal(np.concatenate(workers[k].p), vec[k]), (r, k)


@pytest.mark.parametrize("order", [0, 1])
def test_partial_sync_layers_agree_once_per_period_and_gamma_clears(oracle, order):
    w = W.tiny()
    K, H = 4, 4
    workers = _init(w, oracle, K)
    sets = oracle.schedule("enp", w.n_layers, H)
    layer_of = [t.layer for t in w.tensors]
    agree_count = np.zeros(w.n_layers, dtype=int)
    for k in range(K):                                   # replicas start from the same point: let them drift
        workers[k].local_update(_grads(w, 99, k), 1)
    for r in range(2 * H):
        grads = [_grads(w, r, k) for k in range(K)]
        if order == oracle.UPDATE_THEN_SYNC:
            res = oracle.run_workers(workers, r, sets, grads, order=order)
            state = [[p.copy() for p in wk.p] for wk in workers]
        else:
            # look at the models between the synchronisation and the update
            flats = [wk.pack_slot(sets[r % H])[0] for wk in workers]
            res = []
            for k in range(K):
                res.append(workers[k].sync(sets[r % H], [flats[j] for j in range(K) if j != k], k))
            state = [[p.copy() for p in wk.p] for wk in workers]
            for k in range(K):
                workers[k].local_update(grads[k], r + 1)
        # every worker computed the same average, bit for bit, and reports the same statistics
        for k in range(1, K):
            assert np.array_equal(res[0][0], res[k][0])
            assert res[0][1] == res[k][1]
        for l in range(w.n_layers):
            same = all(np.array_equal(state[0][i], state[k][i]) for k in range(1, K)
                       for i in range(len(layer_of)) if layer_of[i] == l)
            assert same == (l in sets[r % H]), (r, l)
            agree_count[l] += same
        # divergence of the synchronised layers, recomputed after the synchronisation, is exactly zero
        S = sets[r % H]
        off, order_t, total = oracle.slot_offsets(layer_of, [t.numel for t in w.tensors], S)
        after = [oracle.pack([st[t] for t in order_t], [off[t] for t in order_t], total) for st in state]
        m = oracle.mean(after)
        g, _ = oracle.layer_stats(after, m, 0, total)
        assert g == 0.0
        assert all(s[0] > 0.0 for s in res[0][1])           # and it was not zero before
    assert np.all(agree_count == 2)


def test_update_touches_every_layer_each_iteration(oracle):
    w = W.tiny()
    wk = _init(w, oracle, 1)[0]
    sets = oracle.schedule("enp", w.n_layers, w.period)
    before = [p.copy() for p in wk.p]
    flat = wk.pack_slot(sets[0])[0]
    wk.step(0, sets, [flat.copy() for _ in range(3)], 0, _grads(w, 0, 0))
    assert all(not np.array_equal(a, b) for a, b in zip(before, wk.p))
