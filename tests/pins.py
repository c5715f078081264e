"""Pins for the CPU oracle: checks against what the paper and the mathematics fix.

Every check takes an implementation object `impl` with the oracle's Python interface
(Layout, pack, unpack, reduce_update, reduce_update_colour).  test_oracle_pins.py runs
them on the oracle; test_oracle_mutants.py runs them on deliberately broken variants of
the oracle (on the CPU) and demands that each planted mistake is caught.

None of the expected values below comes from the oracle or from the GPU path: they are
closed forms, exact integer / rational arithmetic, numpy or torch library routines, or
the pure-Python brute force in brute.py.
"""
from fractions import Fraction

import numpy as np

import brute
from paper_1711_00705_amd import workloads as wl


def u32(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


def assert_bits_equal(a, b, what=""):
    a, b = u32(a), u32(b)
    assert a.shape == b.shape, what
    bad = np.nonzero(a != b)[0]
    assert bad.size == 0, f"{what}: {bad.size} words differ, first at {bad[:5]}"


def _flats(impl, L, tensor_lists):
    return [impl.pack(L, ts) for ts in tensor_lists]


# ---------------------------------------------------------------------------------------
# layout: Section 4.2 says only "split into k chunks"; the properties any reading must
# have, plus the ones our reading (equal, 256-aligned chunks, last short) adds.
# ---------------------------------------------------------------------------------------
def check_layout_properties(impl):
    rng = np.random.Generator(np.random.PCG64(11))
    cases = [([5], 1), ([0], 3), ([0, 0, 7, 0], 2), ([256], 1), ([257], 2), ([1024], 4),
             ([1025], 4), ([100, 200, 300], 7), ([1], 5), ([255, 1], 1), ([70000, 1, 3], 3)]
    for _ in range(40):
        n = int(rng.integers(1, 9))
        cases.append(([int(s) for s in rng.integers(0, 5000, size=n)], int(rng.integers(1, 12))))
    for sizes, k in cases:
        L = impl.Layout(sizes, k)
        N = sum(sizes)
        # dense concatenation: offsets are running totals, nothing in between
        assert L.off[0] == 0 and L.N == N and L.off[-1] == N
        run = 0
        for t, s in enumerate(sizes):
            assert L.off[t] == run
            run += s
        b = L.bounds
        assert len(b) == k + 1 and b[0] == 0 and b[k] == N
        assert all(b[c] <= b[c + 1] for c in range(k))              # contiguous partition
        lens = [int(b[c + 1] - b[c]) for c in range(k)]
        assert sum(lens) == N
        nonempty = [x for x in lens if x > 0]
        if nonempty:
            C = nonempty[0]
            assert C % 256 == 0 or len(nonempty) == 1                # aligned chunk length
            assert all(x == C for x in nonempty[:-1])                # equal except the last
            assert nonempty[-1] <= C
            assert all(x == 0 for x in lens[len(nonempty):])         # empties only trail
            if len(nonempty) > 1 or C % 256 == 0:
                # minimality: one alignment unit less would not cover N with k chunks
                assert (C - 256) * k < N
        for c in range(k):
            assert b[c] % 256 == 0 or b[c] == N                      # starts are aligned


# ---------------------------------------------------------------------------------------
# P1: brute force on tiny inputs
# ---------------------------------------------------------------------------------------
def check_brute_force(impl, n_cases=60, seed=5):
    rng = np.random.Generator(np.random.PCG64(seed))
    for case in range(n_cases):
        n = int(rng.integers(1, 6))
        sizes = [int(s) for s in rng.choice([0, 1, 2, 3, 5, 17, 64, 130, 255, 256, 257, 300], size=n)]
        while sum(sizes) > 700:
            sizes[int(np.argmax(sizes))] = 3
        N = sum(sizes)
        P = int(rng.integers(1, 5))
        k = int(rng.choice([1, 2, 3, 5, max(N, 1), N + 3]))
        lr, mu, wd = [float(x) for x in rng.choice([0.1, 0.9, 1e-4, 0.01, 0.5, 0.0], size=3)]
        order = None if case % 3 == 0 else wl.random_order(k, P, seed=1000 + case)
        contrib_t = [[(rng.standard_normal(s, dtype=np.float32) * np.float32(1e-3)) for s in sizes]
                     for _ in range(P)]
        w_t = [rng.standard_normal(s, dtype=np.float32) * np.float32(0.05) for s in sizes]
        v_t = [rng.standard_normal(s, dtype=np.float32) * np.float32(0.01) for s in sizes]

        L = impl.Layout(sizes, k)
        xs = _flats(impl, L, contrib_t)
        w = impl.pack(L, w_t)
        v = impl.pack(L, v_t)
        g = impl.reduce_update(L, xs, w, v, lr, mu, wd, order=order)

        bx = [brute.pack([[float(e) for e in t] for t in ts]) for ts in contrib_t]
        bw = brute.pack([[float(e) for e in t] for t in w_t])
        bv = brute.pack([[float(e) for e in t] for t in v_t])
        for p in range(P):
            assert_bits_equal(xs[p], np.array(bx[p], dtype=np.float32), f"pack case {case}")
        bg, bwn, bvn = brute.step(bx, bw, bv, k, lr, mu, wd, order=order)
        tag = f"case {case}: sizes={sizes} P={P} k={k}"
        assert_bits_equal(g, np.array(bg, dtype=np.float32), "g " + tag)
        assert_bits_equal(w, np.array(bwn, dtype=np.float32), "w " + tag)
        assert_bits_equal(v, np.array(bvn, dtype=np.float32), "v " + tag)
        # unpack against the running-counter unpack
        outs = impl.unpack(L, w)
        bouts = brute.unpack(bwn, sizes)
        assert len(outs) == len(bouts)
        for a, b_ in zip(outs, bouts):
            assert_bits_equal(a, np.array(b_, dtype=np.float32), "unpack " + tag)


# ---------------------------------------------------------------------------------------
# P2: integer-valued contributions -> every partial sum is exact -> g is THE integer sum,
# whatever the order and whatever k.
# ---------------------------------------------------------------------------------------
def check_exact_integers(impl):
    sizes = [300, 1, 0, 4097, 1023, 77]
    N = sum(sizes)
    for P in (1, 2, 5, 32):
        ts = [wl.integer_tensors(sizes, seed=900 + p) for p in range(P)]
        exact = np.zeros(N, dtype=np.int64)
        for p in range(P):
            exact += np.concatenate(ts[p]).astype(np.int64)
        for k in (1, 3, 8, N + 3):
            for order in (None, wl.rotation_order(k, P), wl.random_order(k, P, seed=k * 31 + P)):
                L = impl.Layout(sizes, k)
                xs = _flats(impl, L, ts)
                w = np.zeros(N, dtype=np.float32)
                v = np.zeros(N, dtype=np.float32)
                g = impl.reduce_update(L, xs, w, v, 0.0, 0.0, 0.0, order=order)
                assert np.array_equal(g.astype(np.int64), exact), (P, k)
                assert np.array_equal(g, exact.astype(np.float32))
                # with mu = wd = 0 the new momentum is g itself; lr = 0 leaves w alone
                assert_bits_equal(v, g + np.float32(0.0), "v = g")
                assert not w.any()


# ---------------------------------------------------------------------------------------
# P3: identity-coded pack: word j of tensor t holds the integer off_t + j.
# ---------------------------------------------------------------------------------------
def check_identity_pack(impl):
    for sizes in ([7, 0, 1, 300, 4096, 5, 0, 123], [1], [0, 0, 2], list(wl.tiny_sizes()[0])):
        N = sum(sizes)
        ts, run = [], 0
        for s in sizes:
            # keep the top exponent bit clear so no word is a NaN/Inf pattern
            ts.append((np.arange(run, run + s, dtype=np.uint32) & np.uint32(0x3FFFFFFF)).view(np.float32))
            run += s
        L = impl.Layout(sizes, 3)
        flat = impl.pack(L, ts)
        assert np.array_equal(flat.view(np.uint32), np.arange(N, dtype=np.uint32))
        back = impl.unpack(L, flat)
        assert len(back) == len(ts)
        for a, b in zip(back, ts):
            assert_bits_equal(a, b, "unpack(pack(T))")
        assert_bits_equal(impl.pack(L, back), flat, "pack(unpack(F))")
        # arbitrary bit patterns (including NaN payloads) survive both ways
        rng = np.random.Generator(np.random.PCG64(3))
        raw = rng.integers(0, 2**32, size=N, dtype=np.uint64).astype(np.uint32).view(np.float32)
        assert_bits_equal(impl.pack(L, impl.unpack(L, raw)), raw, "raw bits")


# ---------------------------------------------------------------------------------------
# P4: identity order -> g does not depend on k, and k = 1 is the plain sequential sum.
# The sequential sum is numpy's binary32 add (a library routine), not the oracle's loop.
# ---------------------------------------------------------------------------------------
def check_k_invariance(impl):
    sizes = [1000, 333, 2048, 1, 5000]
    N = sum(sizes)
    P = 5
    ts = [wl.contribution_tensors(sizes, p, heavy_tail=True) for p in range(P)]
    wt = wl.weight_tensors(sizes)
    ref_g = None
    for k in (1, 2, 3, 4, 8, N, N + 3):
        L = impl.Layout(sizes, k)
        xs = _flats(impl, L, ts)
        w = impl.pack(L, wt)
        v = np.zeros(N, dtype=np.float32)
        g = impl.reduce_update(L, xs, w, v, 0.1, 0.9, 1e-4)
        if ref_g is None:
            acc = np.concatenate(ts[0]).copy()
            for p in range(1, P):
                acc += np.concatenate(ts[p])
            assert acc.dtype == np.float32
            ref_g, ref_w, ref_v = acc, w.copy(), v.copy()
            assert_bits_equal(g, acc, "k=1 vs plain sequential sum")
        else:
            assert_bits_equal(g, ref_g, f"g k={k}")
            assert_bits_equal(w, ref_w, f"w k={k}")
            assert_bits_equal(v, ref_v, f"v k={k}")


# ---------------------------------------------------------------------------------------
# P5: the order table is honoured -- closed form with 2^24, 1, -2^24.
#   (2^24 + 1) ties to even = 2^24, then - 2^24 -> 0
#   (2^24 - 2^24) = 0, then + 1 -> 1
#   (1 - 2^24) = -16777215 exactly, then + 2^24 -> 1
# ---------------------------------------------------------------------------------------
def check_order_closed_form(impl):
    big = float(2 ** 24)
    sizes = [700, 68]                       # N = 768 = 3 chunks of 256
    N = sum(sizes)
    L = impl.Layout(sizes, 3)
    assert list(L.bounds) == [0, 256, 512, 768]
    xs = [np.full(N, val, dtype=np.float32) for val in (big, 1.0, -big)]
    order = np.array([[0, 1, 2], [0, 2, 1], [1, 2, 0]], dtype=np.int32)
    w = np.zeros(N, dtype=np.float32)
    v = np.zeros(N, dtype=np.float32)
    g = impl.reduce_update(L, xs, w, v, 0.0, 0.0, 0.0, order=order)
    expect = np.concatenate([np.full(256, 0.0), np.full(256, 1.0), np.full(256, 1.0)]).astype(np.float32)
    assert_bits_equal(g, expect, "per-colour order")
    # identity order everywhere -> 0 everywhere; reversed everywhere -> (-2^24+1)+2^24 = 1
    g0 = impl.reduce_update(L, xs, w.copy(), v.copy(), 0.0, 0.0, 0.0)
    assert_bits_equal(g0, np.zeros(N, dtype=np.float32), "identity order")
    rev = np.array([[2, 1, 0]] * 3, dtype=np.int32)
    g1 = impl.reduce_update(L, xs, w.copy(), v.copy(), 0.0, 0.0, 0.0, order=rev)
    assert_bits_equal(g1, np.ones(N, dtype=np.float32), "reversed order")
    # left-to-right association with 4 terms: ((1 + 2^24) + 1) + 1 = 2^24 (each +1 is lost),
    # whereas a pairwise tree (1+2^24) + (1+1) = 2^24 + 2
    xs4 = [np.full(N, val, dtype=np.float32) for val in (1.0, big, 1.0, 1.0)]
    g4 = impl.reduce_update(L, xs4, w.copy(), v.copy(), 0.0, 0.0, 0.0)
    assert_bits_equal(g4, np.full(N, big, dtype=np.float32), "left-to-right, 4 terms")


# ---------------------------------------------------------------------------------------
# P6: the binary32 result is a legitimate rounding of the real sum (heavy-tailed inputs)
# ---------------------------------------------------------------------------------------
def check_error_bound(impl):
    sizes = [4096, 3000, 10000]
    N = sum(sizes)
    P, k = 8, 8
    ts = [wl.contribution_tensors(sizes, p, heavy_tail=True) for p in range(P)]
    L = impl.Layout(sizes, k)
    xs = _flats(impl, L, ts)
    for order in (None, wl.rotation_order(k, P)):
        g = impl.reduce_update(L, xs, np.zeros(N, np.float32), np.zeros(N, np.float32),
                               0.0, 0.0, 0.0, order=order)
        S = np.zeros(N, dtype=np.float64)
        A = np.zeros(N, dtype=np.float64)
        for x in xs:
            S += x.astype(np.float64)
            A += np.abs(x.astype(np.float64))
        bound = (P - 1) * 2.0 ** -24 * A * (1 + 1e-6) + 1e-45
        assert np.all(np.abs(g.astype(np.float64) - S) <= bound)
        assert np.any(g != 0)


# ---------------------------------------------------------------------------------------
# P7: the update, against rational arithmetic and closed forms
# ---------------------------------------------------------------------------------------
def check_update_exact_dyadic(impl):
    # dyadic hyper-parameters and small integers: every product and sum is exact
    rng = np.random.Generator(np.random.PCG64(77))
    N = 600
    L = impl.Layout([N], 2)
    lr, mu, wd = 0.5, 0.25, 0.125
    x0 = rng.integers(-50, 51, size=N).astype(np.float32)
    x1 = rng.integers(-50, 51, size=N).astype(np.float32)
    w0 = rng.integers(-64, 65, size=N).astype(np.float32)
    v0 = rng.integers(-64, 65, size=N).astype(np.float32)
    w, v = w0.copy(), v0.copy()
    g = impl.reduce_update(L, [x0, x1], w, v, lr, mu, wd)
    for i in range(N):
        G = Fraction(int(x0[i])) + Fraction(int(x1[i]))
        W, V = Fraction(int(w0[i])), Fraction(int(v0[i]))
        Vn = Fraction(1, 4) * V + G + Fraction(1, 8) * W
        Wn = W - Fraction(1, 2) * Vn
        assert Fraction(float(g[i])) == G
        assert Fraction(float(v[i])) == Vn, i
        assert Fraction(float(w[i])) == Wn, i


def check_update_special_cases(impl):
    sizes = [513, 100]
    N = sum(sizes)
    L = impl.Layout(sizes, 2)
    xs = _flats(impl, L, [wl.contribution_tensors(sizes, p) for p in range(3)])
    w0 = impl.pack(L, wl.weight_tensors(sizes))
    rng = np.random.Generator(np.random.PCG64(8))
    v0 = rng.standard_normal(N, dtype=np.float32) * np.float32(0.01)
    gref = (xs[0] + xs[1]) + xs[2]

    # (ii) mu = 0, wd = 0: plain SGD, w' = w - lr*g with one multiply and one subtract
    w, v = w0.copy(), v0.copy()
    g = impl.reduce_update(L, xs, w, v, 0.1, 0.0, 0.0)
    assert_bits_equal(g, gref, "g")
    # 0*v + (g + 0*w): adding a zero never changes a nonzero value
    nz = gref != 0
    assert_bits_equal(v[nz], gref[nz], "v' = g when mu = wd = 0")
    assert_bits_equal(w, w0 - np.float32(0.1) * v, "w' = w - lr*v'")

    # (iii) lr = 0: weights untouched bit for bit; v' = mu*v + (g + wd*w)
    w, v = w0.copy(), v0.copy()
    impl.reduce_update(L, xs, w, v, 0.0, 0.9, 1e-4)
    assert_bits_equal(w, w0, "lr = 0 leaves w alone")
    expect_v = np.float32(0.9) * v0 + (gref + np.float32(1e-4) * w0)
    assert_bits_equal(v, expect_v, "v' with lr = 0")

    # zero momentum buffer on the first step: v' = d exactly
    w, v = w0.copy(), np.zeros(N, dtype=np.float32)
    impl.reduce_update(L, xs, w, v, 0.1, 0.9, 1e-4)
    d = gref + np.float32(1e-4) * w0
    nzd = d != 0
    assert_bits_equal(v[nzd], d[nzd], "first step v' = d")
    # weight decay pulls towards zero: with g = 0 contributions, |w'| < |w|
    zeros = [np.zeros(N, dtype=np.float32)]
    w, v = w0.copy(), np.zeros(N, dtype=np.float32)
    impl.reduce_update(L, zeros, w, v, 0.1, 0.0, 0.5)
    big_enough = np.abs(w0) > 1e-6
    assert np.all(np.abs(w[big_enough]) < np.abs(w0[big_enough]))
    assert np.all(np.sign(w[big_enough]) == np.sign(w0[big_enough]))


def check_update_geometric(impl):
    # (iv) constant g, wd = 0, w0 = v0 = 0: v_T = g (1 - mu^T)/(1 - mu), w_T = -lr sum_t v_t
    N, T = 300, 25
    lr, mu = 0.1, 0.9
    L = impl.Layout([N], 1)
    gval = np.linspace(-2.0, 2.0, N).astype(np.float32)
    w = np.zeros(N, dtype=np.float32)
    v = np.zeros(N, dtype=np.float32)
    lr32, mu32 = float(np.float32(lr)), float(np.float32(mu))
    G = gval.astype(np.float64)
    wsum = np.zeros(N)
    for t in range(1, T + 1):
        impl.reduce_update(L, [gval], w, v, lr, mu, 0.0)
        vt = G * (1 - mu32 ** t) / (1 - mu32)
        wsum += vt
        tol = (4 * t) * 2.0 ** -24 * np.maximum(np.abs(vt), 1e-30) * 10
        assert np.all(np.abs(v.astype(np.float64) - vt) <= tol), t
        wt = -lr32 * wsum
        tolw = (8 * t) * 2.0 ** -24 * np.maximum(np.abs(wt), 1e-30) * 10
        assert np.all(np.abs(w.astype(np.float64) - wt) <= tolw), t


# ---------------------------------------------------------------------------------------
# P8: the textbook routine -- torch.optim.SGD on CPU, three successive steps from v = 0
# ---------------------------------------------------------------------------------------
def check_against_torch_sgd(impl):
    import torch
    sizes = [1000, 24, 3000]
    N = sum(sizes)
    lr, mu, wd = 0.1, 0.9, 1e-4
    L = impl.Layout(sizes, 4)
    w = impl.pack(L, wl.weight_tensors(sizes))
    v = np.zeros(N, dtype=np.float32)
    param = torch.nn.Parameter(torch.from_numpy(w.copy()))
    opt = torch.optim.SGD([param], lr=lr, momentum=mu, weight_decay=wd, dampening=0, nesterov=False)
    for step in range(3):
        xs = _flats(impl, L, [wl.contribution_tensors(sizes, p, step=step) for p in range(4)])
        w_old, v_old = w.copy(), v.copy()
        g = impl.reduce_update(L, xs, w, v, lr, mu, wd)
        gt = ((xs[0] + xs[1]) + xs[2]) + xs[3]
        assert_bits_equal(g, gt, "g")
        param.grad = torch.from_numpy(gt.copy())
        opt.step()
        tw = param.detach().numpy()
        tv = opt.state[param]["momentum_buffer"].numpy()
        # relative to the operands (w - lr*v' may cancel); torch may fuse a multiply-add
        band_v = 1e-6 * (np.abs(mu * v_old) + np.abs(gt) + np.abs(wd * w_old)) + 1e-30
        band_w = 1e-6 * (np.abs(w_old) + np.abs(lr * tv)) + 1e-30
        assert np.all(np.abs(v - tv) <= band_v), step
        assert np.all(np.abs(w - tw) <= band_w), step
        # keep torch's state as the running state so that differences do not accumulate
        w[:] = tw
        v[:] = tv


# ---------------------------------------------------------------------------------------
# P9: colours are independent (Section 4.2): any colour order, run twice -> same bits
# ---------------------------------------------------------------------------------------
def check_colour_independence(impl):
    sizes = [3000, 500, 1200]
    N = sum(sizes)
    P, k = 4, 5
    L = impl.Layout(sizes, k)
    xs = _flats(impl, L, [wl.contribution_tensors(sizes, p) for p in range(P)])
    w0 = impl.pack(L, wl.weight_tensors(sizes))
    order = wl.rotation_order(k, P)
    w1, v1 = w0.copy(), np.zeros(N, np.float32)
    g1 = impl.reduce_update(L, xs, w1, v1, 0.1, 0.9, 1e-4, order=order)
    w2, v2 = w0.copy(), np.zeros(N, np.float32)
    g2 = impl.reduce_update(L, xs, w2, v2, 0.1, 0.9, 1e-4, order=order)
    assert_bits_equal(g1, g2, "run twice")
    w3, v3 = w0.copy(), np.zeros(N, np.float32)
    g3 = np.zeros(N, np.float32)
    for c in reversed(range(k)):
        impl.reduce_update_colour(L, c, xs, g3, w3, v3, 0.1, 0.9, 1e-4, seq=order[c])
    assert_bits_equal(g1, g3, "colours in reverse")
    assert_bits_equal(w1, w3, "w colours in reverse")
    assert_bits_equal(v1, v3, "v colours in reverse")
    # a colour touches only its own range
    w4, v4 = w0.copy(), np.zeros(N, np.float32)
    g4 = np.full(N, 7.0, np.float32)
    impl.reduce_update_colour(L, 1, xs, g4, w4, v4, 0.1, 0.9, 1e-4, seq=order[1])
    lo, hi = int(L.bounds[1]), int(L.bounds[2])
    outside = np.ones(N, bool)
    outside[lo:hi] = False
    assert np.all(g4[outside] == 7.0) and np.array_equal(w4[outside], w0[outside])
    assert not v4[outside].any()
    assert_bits_equal(g4[lo:hi], g1[lo:hi], "colour 1 range")


# ---------------------------------------------------------------------------------------
# F1/F2: signed zero, denormals, NaN/Inf
# ---------------------------------------------------------------------------------------
def check_ieee_corner_cases(impl):
    N = 512
    L = impl.Layout([N], 2)
    nzero = np.full(N, -0.0, dtype=np.float32)
    # the accumulator starts from the first term: (-0) + (-0) = -0, never +0
    g = impl.reduce_update(L, [nzero, nzero.copy()], np.zeros(N, np.float32), np.zeros(N, np.float32),
                           0.0, 0.0, 0.0)
    assert np.all(u32(g) == 0x80000000)
    g = impl.reduce_update(L, [nzero], np.zeros(N, np.float32), np.zeros(N, np.float32), 0.0, 0.0, 0.0)
    assert np.all(u32(g) == 0x80000000)
    # denormals are kept: 3 * 2^-149 from three smallest denormals; 2^-126 - 2^-149
    tiny = np.full(N, 2.0 ** -149, dtype=np.float32)
    g = impl.reduce_update(L, [tiny, tiny.copy(), tiny.copy()], np.zeros(N, np.float32),
                           np.zeros(N, np.float32), 0.0, 0.0, 0.0)
    assert np.all(u32(g) == 3)
    a = np.full(N, 2.0 ** -126, dtype=np.float32)
    b = np.full(N, -(2.0 ** -149), dtype=np.float32)
    g = impl.reduce_update(L, [a, b], np.zeros(N, np.float32), np.zeros(N, np.float32), 0.0, 0.0, 0.0)
    assert np.all(u32(g) == 0x007FFFFF)
    # denormal products in the update: w = 2^-140, wd = 0.5 -> wd*w = 2^-141 (denormal, exact)
    w = np.full(N, 2.0 ** -140, dtype=np.float32)
    v = np.zeros(N, np.float32)
    impl.reduce_update(L, [np.zeros(N, np.float32)], w, v, 0.0, 0.0, 0.5)
    assert np.all(v == np.float32(2.0 ** -141)) and np.all(v != 0)
    # NaN / Inf propagate
    x = np.zeros(N, np.float32)
    x[3] = np.inf
    x[5] = np.nan
    y = np.zeros(N, np.float32)
    y[3] = -np.inf
    y[7] = np.inf
    w = np.ones(N, np.float32)
    v = np.zeros(N, np.float32)
    g = impl.reduce_update(L, [x, y], w, v, 0.1, 0.9, 0.0)
    assert np.isnan(g[3]) and np.isnan(g[5]) and np.isposinf(g[7])
    assert np.isnan(w[3]) and np.isnan(w[5]) and np.isneginf(w[7])
    assert np.all(np.isfinite(np.delete(g, [3, 5, 7])))


ALL_CHECKS = [
    check_layout_properties,
    check_brute_force,
    check_exact_integers,
    check_identity_pack,
    check_k_invariance,
    check_order_closed_form,
    check_error_bound,
    check_update_exact_dyadic,
    check_update_special_cases,
    check_update_geometric,
    check_against_torch_sgd,
    check_colour_independence,
    check_ieee_corner_cases,
]
