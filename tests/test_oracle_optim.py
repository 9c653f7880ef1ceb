"""Pins for the oracle's local update (Eq. (5), first case; Algorithm 1 "update model"): closed forms, the
momentum-free special case of Sec. 2.1, and torch.optim on CPU as an independent witness."""
import numpy as np
import pytest
import torch


def _rand(n, seed, scale):
    return (np.random.default_rng(seed).standard_normal(n) * scale).astype(np.float32)


def test_sgdm_zero_momentum_is_plain_sgd(oracle):
    p0, g = _rand(5000, 1, 0.02), _rand(5000, 2, 0.01)
    p, buf = p0.copy(), _rand(5000, 3, 1.0)          # stale buffer content must not matter when mu = 0
    oracle.sgdm(p, g, buf, 0.01, 0.0)
    assert np.array_equal(p, p0 - np.float32(0.01) * g)   # w - eta * grad, each op rounded once in fp32
    assert np.array_equal(buf, g + np.float32(0.0) * 0)


def test_sgdm_constant_gradient_closed_form(oracle):
    # buf_t = g (1 - mu^t)/(1 - mu);  p_t = p_0 - lr g sum_{j<=t} (1 - mu^j)/(1 - mu)
    lr, mu, T = 0.01, 0.9, 25
    p0, g = _rand(3000, 4, 0.02), _rand(3000, 5, 0.01)
    p, buf = p0.copy(), np.zeros_like(p0)
    for _ in range(T):
        oracle.sgdm(p, g, buf, lr, mu)
    mu32, lr32 = float(np.float32(mu)), float(np.float32(lr))
    coef = sum((1 - mu32 ** j) / (1 - mu32) for j in range(1, T + 1))
    expect = p0.astype(np.float64) - lr32 * g.astype(np.float64) * coef
    # 25 steps of fp32 rounding at |p| <= 0.1 (half an ulp = 3.7e-9 each); a wrong term would show at ~1e-4
    assert np.allclose(p, expect, rtol=0, atol=1e-7)
    assert np.allclose(buf, g.astype(np.float64) * (1 - mu32 ** T) / (1 - mu32), rtol=2e-6)


def test_sgdm_hand_values(oracle):
    # dyadic numbers: every operation exact.  mu=0.5, lr=0.25, g=1: buf 1, 1.5, 1.75; p 8 -> 7.75 -> 7.375 -> 6.9375
    p, g, buf = np.float32([8.0]), np.float32([1.0]), np.float32([0.0])
    seen = []
    for _ in range(3):
        oracle.sgdm(p, g, buf, 0.25, 0.5)
        seen.append((float(buf[0]), float(p[0])))
    assert seen == [(1.0, 7.75), (1.5, 7.375), (1.75, 6.9375)]


def test_sgdm_matches_torch_optim(oracle):
    n, T = 4096, 16
    p0 = _rand(n, 6, 0.02)
    tp = torch.nn.Parameter(torch.from_numpy(p0.copy()))
    opt = torch.optim.SGD([tp], lr=0.01, momentum=0.9)
    p, buf = p0.copy(), np.zeros_like(p0)
    for t in range(T):
        g = _rand(n, 100 + t, 0.01)
        tp.grad = torch.from_numpy(g.copy())
        opt.step()
        oracle.sgdm(p, g, buf, 0.01, 0.9)
    ref = tp.detach().numpy()
    assert np.allclose(p, ref, rtol=1e-6, atol=1e-9)


def test_adamw_first_step_closed_form(oracle):
    # m = (1-b1) g, v = (1-b2) g^2: bias corrections cancel, p_1 = p_0 (1 - lr wd) - lr g / (|g| + eps)
    lr, b1, b2, eps, wd = 3e-4, 0.9, 0.95, 1e-8, 0.1
    p0, g = _rand(5000, 7, 0.02), _rand(5000, 8, 1e-3)
    p, m, v = p0.copy(), np.zeros_like(p0), np.zeros_like(p0)
    oracle.adamw(p, g, m, v, None, lr, b1, b2, eps, wd, 1)
    g64 = g.astype(np.float64)
    expect = p0.astype(np.float64) * (1 - lr * wd) - lr * g64 / (np.abs(g64) + eps)
    assert np.allclose(p, expect, rtol=1e-6, atol=1e-9)
    assert np.allclose(m, (1 - b1) * g64, rtol=1e-6)
    assert np.allclose(v, (1 - b2) * g64 * g64, rtol=1e-6)


def test_adamw_constant_gradient_no_decay_walks_by_lr(oracle):
    # with constant g: m_t = g (1 - b1^t), v_t = g^2 (1 - b2^t), so mhat/sqrt(vhat) = sign(g) each step
    lr, T = 1e-3, 20
    p0 = _rand(2000, 9, 0.02)
    g = np.where(np.arange(2000) % 2 == 0, 1e-2, -3e-3).astype(np.float32)
    p, m, v = p0.copy(), np.zeros_like(p0), np.zeros_like(p0)
    for t in range(1, T + 1):
        oracle.adamw(p, g, m, v, None, lr, 0.9, 0.95, 1e-8, 0.0, t)
    expect = p0.astype(np.float64) - T * lr * np.sign(g)
    assert np.allclose(p, expect, rtol=0, atol=T * lr * 2e-5)


def test_adamw_scalars(oracle):
    lr, b1, b2, wd, t = 3e-4, 0.9, 0.95, 0.1, 7
    s = oracle.adamw_scalars(lr, b1, b2, wd, t)
    f = np.float32
    b1d, b2d = float(f(b1)), float(f(b2))
    assert s[0] == f(1) - f(b1) and s[1] == f(1) - f(b2)
    assert s[2] == f(1) - f(lr) * f(wd)
    assert s[3] == f(lr) * f(1.0 / (1.0 - b1d ** t))
    assert s[4] == f(1.0 / np.sqrt(1.0 - b2d ** t))


@pytest.mark.parametrize("wd", [0.0, 0.1])
def test_adamw_matches_torch_optim(oracle, wd):
    n, T = 4096, 16
    p0 = _rand(n, 10, 0.02)
    tp = torch.nn.Parameter(torch.from_numpy(p0.copy()))
    opt = torch.optim.AdamW([tp], lr=3e-4, betas=(0.9, 0.95), eps=1e-8, weight_decay=wd)
    p, m, v = p0.copy(), np.zeros_like(p0), np.zeros_like(p0)
    for t in range(1, T + 1):
        g = _rand(n, 200 + t, 1e-3)
        tp.grad = torch.from_numpy(g.copy())
        opt.step()
        oracle.adamw(p, g, m, v, None, 3e-4, 0.9, 0.95, 1e-8, wd, t)
    ref = tp.detach().numpy()
    assert np.allclose(p, ref, rtol=2e-6, atol=2e-9)


def test_adamw_bf16_gradient_and_model_copy(oracle):
    n = 3000
    p0, g = _rand(n, 11, 0.02), _rand(n, 12, 1e-3)
    g16 = oracle.bf16_rne(g)
    pa, ma, va = p0.copy(), np.zeros_like(p0), np.zeros_like(p0)
    pb, mb, vb = p0.copy(), np.zeros_like(p0), np.zeros_like(p0)
    model = np.zeros(n, dtype=np.uint16)
    oracle.adamw(pa, g16, ma, va, model, 3e-4, 0.9, 0.95, 1e-8, 0.1, 1)
    oracle.adamw(pb, oracle.bf16_widen(g16), mb, vb, None, 3e-4, 0.9, 0.95, 1e-8, 0.1, 1)
    assert np.array_equal(pa, pb) and np.array_equal(ma, mb) and np.array_equal(va, vb)   # widening is exact
    assert np.array_equal(model, oracle.bf16_rne(pa))


def test_threads_do_not_change_results(oracle):
    n = 100003
    p0, g = _rand(n, 13, 0.02), _rand(n, 14, 1e-3)
    outs = []
    for th in (1, 4):
        oracle.set_threads(th)
        p, m, v = p0.copy(), np.zeros_like(p0), np.zeros_like(p0)
        for t in (1, 2, 3):
            oracle.adamw(p, g, m, v, None, 3e-4, 0.9, 0.95, 1e-8, 0.1, t)
        outs.append((p, m, v))
    oracle.set_threads(1)
    for a, b in zip(*outs):
        assert np.array_equal(a, b)


def test_adamw_hand_worked_dyadic_values(oracle):
    # Values chosen so that every intermediate is a dyadic rational that fp32 holds exactly: the result is fixed by the
    # AdamW definition alone, bit for bit, whatever the operation order.  beta1 = 1/2, beta2 = 3/4, step 1:
    #   m = g/2, v = g^2/4, 1/(1-beta1) = 2, 1/sqrt(1-beta2) = 2, so m/(sqrt(v)*2 + eps) = (g/2)/(|g| + eps)
    # with lr = 1/2, eps = 0, weight_decay = 1/4: p' = p*(1 - 1/8) - (1/2*2) * sign(g)/2 = 7p/8 - sign(g)/2
    g = np.array([1.0, -2.0, 0.25, -8.0, 3.0], dtype=np.float32)
    p0 = np.array([1.0, 16.0, -4.0, 0.5, 8.0], dtype=np.float32)
    p, m, v = p0.copy(), np.zeros_like(p0), np.zeros_like(p0)
    oracle.adamw(p, g, m, v, None, 0.5, 0.5, 0.75, 0.0, 0.25, 1)
    assert np.array_equal(m, g / 2) and np.array_equal(v, g * g / 4)
    assert np.array_equal(p, np.array([0.375, 14.5, -4.0, 0.9375, 6.5], dtype=np.float32))
    # eps = 1 with g = +-1: (1/2)/(1 + 1) = 1/4, so p' = 7p/8 - sign(g)/4 ... and a second step from hand-set moments:
    # step 2 would need 1/(1 - 1/4) = 4/3, not dyadic; instead pin the moment recurrences alone (they do not use it)
    g1 = np.array([1.0, -1.0], dtype=np.float32)
    p, m, v = np.array([8.0, 8.0], dtype=np.float32), np.zeros(2, dtype=np.float32), np.zeros(2, dtype=np.float32)
    oracle.adamw(p, g1, m, v, None, 0.5, 0.5, 0.75, 1.0, 0.25, 1)
    assert np.array_equal(p, np.array([6.75, 7.25], dtype=np.float32))
    oracle.adamw(p, 2 * g1, m, v, None, 0.5, 0.5, 0.75, 1.0, 0.25, 2)
    assert np.array_equal(m, np.array([1.25, -1.25], dtype=np.float32))       # 1/2 * 1/2 + 1/2 * 2
    assert np.array_equal(v, np.array([1.1875, 1.1875], dtype=np.float32))    # 3/4 * 1/4 + 1/4 * 4


def test_adamw_against_the_textbook_division_form(oracle):
    # The AdamW of the literature divides by the bias corrections: mhat = m/(1-b1^t), vhat = v/(1-b2^t),
    # p' = p(1 - lr wd) - lr mhat/(sqrt(vhat) + eps).  Evaluated in fp64 from the same fp32 state each step, it must
    # agree with the oracle's fp32 step to a few units in the last place of p: 12 roundings of at most 2^-24 relative
    # each on terms no larger than |p| + lr.
    lr, b1, b2, eps, wd, n = 3e-4, 0.9, 0.95, 1e-8, 0.1, 20000
    p, m, v = _rand(n, 21, 0.02), np.zeros(n, dtype=np.float32), np.zeros(n, dtype=np.float32)
    b1d, b2d, lrd, wdd, epsd = (float(np.float32(x)) for x in (b1, b2, lr, wd, eps))
    for t in range(1, 9):
        g = _rand(n, 300 + t, 1e-3)
        p64, m64, v64, g64 = (x.astype(np.float64) for x in (p, m, v, g))
        m_ref = b1d * m64 + (1 - b1d) * g64
        v_ref = b2d * v64 + (1 - b2d) * g64 * g64
        p_ref = p64 * (1 - lrd * wdd) - lrd * (m_ref / (1 - b1d ** t)) / (np.sqrt(v_ref / (1 - b2d ** t)) + epsd)
        oracle.adamw(p, g, m, v, None, lr, b1, b2, eps, wd, t)
        assert np.max(np.abs(m - m_ref) / (np.abs(b1d * m64) + np.abs((1 - b1d) * g64) + 1e-30)) < 3 * 2.0 ** -24   # the two terms may cancel
        assert np.max(np.abs(v - v_ref) / np.maximum(np.abs(v_ref), 1e-30)) < 4 * 2.0 ** -24
        assert np.max(np.abs(p - p_ref) / (np.abs(p_ref) + lrd)) < 4 * 2.0 ** -24


def test_adamw_bitwise_against_an_array_evaluation(oracle):
    # A second evaluation of the documented operation sequence, written with whole-array fp32 operations (numpy rounds
    # every fp32 operation, sqrt and division included, correctly): the bits must be the same.  A dropped or fused
    # operation, a changed association or a different constant in the loop of the oracle fails this.
    f = np.float32
    lr, b1, b2, eps, wd, n = f(3e-4), f(0.9), f(0.95), f(1e-8), f(0.1), 50000
    p, m, v = _rand(n, 31, 0.02), np.zeros(n, dtype=np.float32), np.zeros(n, dtype=np.float32)
    pr, mr, vr = p.copy(), m.copy(), v.copy()
    for t in range(1, 6):
        g = _rand(n, 400 + t, 1e-3)
        oracle.adamw(p, g, m, v, None, float(lr), float(b1), float(b2), float(eps), float(wd), t)
        step_size = lr * f(1.0 / (1.0 - float(b1) ** t))
        rs2 = f(1.0 / np.sqrt(1.0 - float(b2) ** t))
        mr = b1 * mr + (f(1) - b1) * g
        vr = b2 * vr + ((f(1) - b2) * g) * g
        pr = pr * (f(1) - lr * wd) - step_size * (mr / (np.sqrt(vr) * rs2 + eps))
        for a, b in ((p, pr), (m, mr), (v, vr)):
            assert a.dtype == b.dtype == np.float32 and np.array_equal(a.view(np.uint32), b.view(np.uint32))
