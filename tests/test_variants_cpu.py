"""Variants of the update: pins of the Nesterov oracle (torch.optim.SGD, rational arithmetic),
the learning-rate schedule of Section 5 (closed forms from the paper's numbers), and the
library's host-side schedule against the oracle.  No GPU."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from oracle import schedule
import pins
from paper_1711_00705_amd import mc
from paper_1711_00705_amd import workloads as wl


def test_nesterov_against_rational_arithmetic():
    rng = np.random.Generator(np.random.PCG64(21))
    N = 500
    L = oracle.Layout([N], 2)
    x0 = rng.integers(-50, 51, size=N).astype(np.float32)
    x1 = rng.integers(-50, 51, size=N).astype(np.float32)
    w0 = rng.integers(-64, 65, size=N).astype(np.float32)
    v0 = rng.integers(-64, 65, size=N).astype(np.float32)
    w, v = w0.copy(), v0.copy()
    g = oracle.reduce_update_nesterov(L, [x0, x1], w, v, 0.5, 0.25, 0.125)
    for i in range(N):
        G = Fraction(int(x0[i]) + int(x1[i]))
        W, V = Fraction(int(w0[i])), Fraction(int(v0[i]))
        D = G + Fraction(1, 8) * W
        Vn = Fraction(1, 4) * V + D
        Wn = W - Fraction(1, 2) * (D + Fraction(1, 4) * Vn)
        assert Fraction(float(g[i])) == G and Fraction(float(v[i])) == Vn and Fraction(float(w[i])) == Wn


def test_nesterov_against_torch_sgd():
    import torch
    sizes = [1000, 24, 3000]
    N = sum(sizes)
    lr, mu, wd = 0.1, 0.9, 1e-4
    L = oracle.Layout(sizes, 4)
    w = oracle.pack(L, wl.weight_tensors(sizes))
    v = np.zeros(N, np.float32)
    param = torch.nn.Parameter(torch.from_numpy(w.copy()))
    opt = torch.optim.SGD([param], lr=lr, momentum=mu, weight_decay=wd, dampening=0, nesterov=True)
    for step in range(3):
        xs = [oracle.pack(L, wl.contribution_tensors(sizes, p, step=step)) for p in range(4)]
        w_old, v_old = w.copy(), v.copy()
        g = oracle.reduce_update_nesterov(L, xs, w, v, lr, mu, wd, order=wl.rotation_order(4, 4))
        param.grad = torch.from_numpy(g.copy())
        opt.step()
        tw = param.detach().numpy()
        tv = opt.state[param]["momentum_buffer"].numpy()
        band_v = 1e-6 * (np.abs(mu * v_old) + np.abs(g) + np.abs(wd * w_old)) + 1e-30
        band_w = 1e-6 * (np.abs(w_old) + np.abs(lr * g) + np.abs(lr * mu * tv)) + 1e-30
        assert np.all(np.abs(v - tv) <= band_v), step
        assert np.all(np.abs(w - tw) <= band_w), step
        w[:] = tw
        v[:] = tv


def test_nesterov_reduces_to_plain_sgd_without_momentum():
    # mu = 0: look-ahead term vanishes, both variants give w' = w - lr*d
    sizes = [700, 68]
    L = oracle.Layout(sizes, 3)
    N = L.N
    xs = [oracle.pack(L, wl.contribution_tensors(sizes, p)) for p in range(3)]
    w0 = oracle.pack(L, wl.weight_tensors(sizes))
    w1, v1 = w0.copy(), np.zeros(N, np.float32)
    w2, v2 = w0.copy(), np.zeros(N, np.float32)
    g1 = oracle.reduce_update(L, xs, w1, v1, 0.1, 0.0, 1e-3)
    g2 = oracle.reduce_update_nesterov(L, xs, w2, v2, 0.1, 0.0, 1e-3)
    pins.assert_bits_equal(g1, g2, "g")
    pins.assert_bits_equal(v1, v2, "v")
    nz = v1 != 0            # d + 0*v' = d unless d is a signed zero
    pins.assert_bits_equal(w1[nz], w2[nz], "w")


def test_schedule_oracle_against_the_papers_numbers():
    # Section 5: start 0.1; target 0.1*k*n/256; /10 after every 30 epochs; 90 epochs.
    # 256-GPU run, batch 32 per GPU: target 0.1*32*256/256 = 3.2
    f = lambda e: schedule.lr_at(e, 0.1, 32, 256, 5.0, 30.0)
    assert f(0.0) == pytest.approx(0.1, rel=1e-12)
    assert f(5.0) == pytest.approx(3.2, rel=1e-12)
    assert f(2.5) == pytest.approx((0.1 + 3.2) / 2, rel=1e-12)          # linear ramp: midpoint
    assert f(29.999) == pytest.approx(3.2, rel=1e-12)
    assert f(30.0) == pytest.approx(0.32, rel=1e-12)
    assert f(59.999) == pytest.approx(0.32, rel=1e-12)
    assert f(60.0) == pytest.approx(0.032, rel=1e-12)
    assert f(89.999) == pytest.approx(0.032, rel=1e-12)
    # 32 nodes x 4 GPUs, batch 64 per GPU: 0.1*64*128/256 = 3.2 ; 8 nodes x 4: 0.8
    assert schedule.target_lr(0.1, 64, 128) == pytest.approx(3.2)
    assert schedule.target_lr(0.1, 64, 32) == pytest.approx(0.8)
    # 256 images in total: nothing to scale (k*n = 256 -> target == base)
    assert schedule.target_lr(0.1, 64, 4) == pytest.approx(0.1)
    assert schedule.lr_at(3.0, 0.1, 64, 4, 5.0, 30.0) == pytest.approx(0.1)
    # the ramp is monotone and continuous at its end
    es = np.linspace(0, 5, 101)
    vals = [f(float(e)) for e in es]
    assert all(b >= a for a, b in zip(vals, vals[1:]))
    assert f(4.999999) == pytest.approx(3.2, rel=1e-5)
    # no ramp at all
    assert schedule.lr_at(0.0, 0.1, 32, 256, 0.0, 30.0) == pytest.approx(3.2)


def test_library_schedule_matches_oracle():
    rng = np.random.Generator(np.random.PCG64(2))
    for _ in range(500):
        k = int(rng.choice([16, 32, 64, 128]))
        n = int(rng.choice([4, 8, 32, 64, 128, 256, 512]))
        warm = float(rng.choice([0.0, 1.0, 5.0, 2.5]))
        drop = float(rng.choice([30.0, 10.0, 7.5]))
        e = float(np.float32(rng.uniform(0, 90)))
        base = float(np.float32(rng.choice([0.1, 0.05, 0.4])))
        got = mc.lr_schedule(base, k, n, warm, drop, e)
        want = schedule.lr_at(e, base, k, n, warm, drop)
        assert got == pytest.approx(want, rel=2e-7), (k, n, warm, drop, e)
    for e, want in ((0.0, 0.1), (5.0, 3.2), (30.0, 0.32), (60.0, 0.032)):
        assert mc.lr_schedule(0.1, 32, 256, 5.0, 30.0, e) == pytest.approx(want, rel=2e-7)


def test_library_schedule_and_spec_reject():
    import ctypes
    out = ctypes.c_float()
    f = mc.lib.mc_lr_schedule
    assert f(0.1, 32, 256, 5.0, 30.0, 1.0, None) == mc.ERR_INVALID_ARG
    for bad in ((0.0, 32, 256, 5.0, 30.0, 1.0), (0.1, 0, 256, 5.0, 30.0, 1.0), (0.1, 32, 0, 5.0, 30.0, 1.0),
                (0.1, 32, 256, -1.0, 30.0, 1.0), (0.1, 32, 256, 5.0, 0.0, 1.0), (0.1, 32, 256, 5.0, 30.0, -1.0),
                (float("nan"), 32, 256, 5.0, 30.0, 1.0), (0.1, 32, 256, 5.0, 30.0, float("inf"))):
        assert f(*bad, ctypes.byref(out)) == mc.ERR_INVALID_ARG, bad
    L = mc.Layout([1000, 24], 2)
    B = 0x10000000
    x = [B, B + (1 << 20)]
    g, w, v = B + (8 << 20), B + (9 << 20), B + (10 << 20)

    def code(fn, *a, **kw):
        try:
            fn(*a, **kw)
        except mc.McError as e:
            return e.code
        return mc.OK
    assert code(mc.reduce_update_ex, L, x, None, g, w, v, None) == mc.ERR_INVALID_ARG
    assert code(mc.reduce_update_ex, L, x, None, g, w, v, mc.update_spec(0.1, 0.9, 0.0, nesterov=2)) == mc.ERR_INVALID_ARG
    assert code(mc.reduce_update_ex, L, x, None, g, w, v, mc.update_spec(0.1, 0.9, 0.0, state_policy=3)) == mc.ERR_INVALID_ARG
    assert code(mc.reduce_update_ex, L, x, None, g, w, v, mc.update_spec(0.1, 0.9, 0.0, state_policy=-1)) == mc.ERR_INVALID_ARG
    assert code(mc.reduce_update_ex, L, x, None, g, w, v, mc.update_spec(0.1, 0.9, 0.0, sweep=3)) == mc.ERR_INVALID_ARG
    assert code(mc.reduce_update_ex, L, x, None, g, w, v, mc.update_spec(hyper_dev_ptr=B + 2)) == mc.ERR_ALIGN
    assert code(mc.reduce_update_ex, L, x, None, g, w + 4, v, mc.update_spec(0.1, 0.9, 0.0)) == mc.ERR_ALIGN
    assert code(mc.reduce_update_ex, L, x, None, g, w, v, mc.update_spec(0.1, 0.9, 0.0), elem_begin=100) == mc.ERR_INVALID_ARG
    assert code(mc.hyper_write, None, 0.1, 0.9, 0.0) == mc.ERR_INVALID_ARG
    assert code(mc.hyper_write, B + 1, 0.1, 0.9, 0.0) == mc.ERR_ALIGN
    assert mc.lib.mc_fused_step_ex(L.handle, None, 1, None, None, None, None, None, None, None, None) == mc.ERR_INVALID_ARG


def test_planted_mistakes_in_the_nesterov_step_are_caught():
    """Plant plausible mistakes in wrappers around the Nesterov oracle (on the CPU) and demand
    that the rational-arithmetic pin or the torch pin fails."""
    import types
    real = oracle.reduce_update_nesterov

    def look_ahead_with_old_momentum(L, xs, w, v, lr, mu, wd, order=None):
        w_old, v_old = w.copy(), v.copy()
        g = real(L, xs, w, v, lr, mu, wd, order=order)
        d = v - np.float32(mu) * v_old
        w[:] = w_old - np.float32(lr) * (d + np.float32(mu) * v_old)
        return g

    def plain_step(L, xs, w, v, lr, mu, wd, order=None):
        return oracle.reduce_update(L, xs, w, v, lr, mu, wd, order=order)

    def look_ahead_twice(L, xs, w, v, lr, mu, wd, order=None):
        w_old = w.copy()
        g = real(L, xs, w, v, lr, mu, wd, order=order)
        w[:] = w_old - np.float32(lr) * (v + np.float32(mu) * v)
        return g

    for mutant in (look_ahead_with_old_momentum, plain_step, look_ahead_twice):
        oracle.reduce_update_nesterov = mutant
        try:
            caught = 0
            for t in (test_nesterov_against_rational_arithmetic, test_nesterov_against_torch_sgd):
                try:
                    t()
                except AssertionError:
                    caught += 1
            assert caught >= 1, mutant.__name__
        finally:
            oracle.reduce_update_nesterov = real
