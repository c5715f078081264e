"""Per-colour roles in the oracle: the per-rank pieces, composed over the trees of Section
4.2, give the plain sum of all contributions (Section 3, Algorithm 1) and identical weights
on every node.  CPU only."""
import numpy as np
import pytest

import oracle
from oracle import trees
import allreduce_sim as sim
import pins


def _oracle_call(L):
    def call(contrib, n_terms, do_update, g, w, v, lr, mu, wd, order):
        oracle.reduce_update_roles(L, contrib, n_terms, do_update, g, w, v, lr, mu, wd, order=order)
    call.bounds = L.bounds
    return call


@pytest.mark.parametrize("n_nodes,k,m", [(8, 4, 4), (5, 2, 2), (9, 4, 1), (16, 4, 2), (3, 2, 3), (1, 2, 2)])
def test_whole_allreduce_equals_plain_sum(n_nodes, k, m):
    sizes = [700, 33, 1500]
    L = oracle.Layout(sizes, k)
    N = L.N
    parents = trees.colour_trees(n_nodes, k)
    rng = np.random.Generator(np.random.PCG64(100 + n_nodes))
    # integer-valued: every partial sum exact, so the result must be THE sum of all n*m terms
    local = [[rng.integers(-500, 501, size=N).astype(np.float32) for _ in range(m)] for _ in range(n_nodes)]
    exact = np.zeros(N, np.int64)
    for node in local:
        for x in node:
            exact += x.astype(np.int64)
    w0 = rng.standard_normal(N, dtype=np.float32)
    v0 = rng.standard_normal(N, dtype=np.float32)
    g, w, v = sim.simulate(_oracle_call(L), parents, m, local, w0, v0, N, k, 0.1, 0.9, 1e-4)
    assert np.array_equal(g.astype(np.int64), exact)
    # every node ends with the same weights, and they are the single-rank update with g
    wr, vr = w0.copy(), v0.copy()
    oracle.reduce_update(L, [exact.astype(np.float32)], wr, vr, 0.1, 0.9, 1e-4)
    for node in range(n_nodes):
        pins.assert_bits_equal(w[node], wr, f"w on node {node}")
        pins.assert_bits_equal(v[node], vr, f"v on node {node}")


def test_whole_allreduce_fp32_follows_tree_order():
    n_nodes, k, m = 8, 4, 2
    sizes = [1000, 24]
    L = oracle.Layout(sizes, k)
    N = L.N
    parents = trees.colour_trees(n_nodes, k)
    rng = np.random.Generator(np.random.PCG64(7))
    local = [[rng.standard_normal(N, dtype=np.float32) for _ in range(m)] for _ in range(n_nodes)]
    z = np.zeros(N, np.float32)
    g, w, v = sim.simulate(_oracle_call(L), parents, m, local, z, z, N, k, 0.0, 0.0, 0.0)
    for c in range(k):
        lo, hi = int(L.bounds[c]), int(L.bounds[c + 1])
        pins.assert_bits_equal(g[lo:hi], sim.tree_order_sum(parents[c], m, local, lo, hi), f"colour {c}")


def test_roles_leave_skipped_colours_alone_and_match_uniform_call():
    sizes = [3000, 77]
    k, P = 4, 5
    L = oracle.Layout(sizes, k)
    N = L.N
    rng = np.random.Generator(np.random.PCG64(3))
    xs = [rng.standard_normal(N, dtype=np.float32) for _ in range(P)]
    w0 = rng.standard_normal(N, dtype=np.float32)
    v0 = rng.standard_normal(N, dtype=np.float32)
    # all colours, all terms, all updating == the uniform call
    g1 = np.zeros(N, np.float32)
    w1, v1 = w0.copy(), v0.copy()
    oracle.reduce_update_roles(L, xs, [P] * k, [1] * k, g1, w1, v1, 0.1, 0.9, 1e-3)
    w2, v2 = w0.copy(), v0.copy()
    g2 = oracle.reduce_update(L, xs, w2, v2, 0.1, 0.9, 1e-3)
    pins.assert_bits_equal(g1, g2, "g")
    pins.assert_bits_equal(w1, w2, "w")
    pins.assert_bits_equal(v1, v2, "v")
    # mixed: colour 0 skipped, colour 1 three terms sum-only, colour 2 all terms + update, colour 3 one term
    g = np.full(N, 7.0, np.float32)
    w, v = w0.copy(), v0.copy()
    oracle.reduce_update_roles(L, xs, [0, 3, P, 1], [1, 0, 1, 0], g, w, v, 0.1, 0.9, 1e-3)
    b = [int(x) for x in L.bounds]
    assert np.all(g[b[0]:b[1]] == 7.0)
    pins.assert_bits_equal(g[b[1]:b[2]], ((xs[0] + xs[1]) + xs[2])[b[1]:b[2]], "three terms")
    pins.assert_bits_equal(g[b[2]:b[3]], g2[b[2]:b[3]], "all terms")
    pins.assert_bits_equal(g[b[3]:b[4]], xs[0][b[3]:b[4]], "one term")
    for lo, hi, updated in ((b[0], b[1], False), (b[1], b[2], False), (b[2], b[3], True), (b[3], b[4], False)):
        ref_w, ref_v = (w2, v2) if updated else (w0, v0)
        pins.assert_bits_equal(w[lo:hi], ref_w[lo:hi], "w range")
        pins.assert_bits_equal(v[lo:hi], ref_v[lo:hi], "v range")


def test_oracle_range_partition_equals_whole_call():
    sizes = [3000, 77, 1200]
    k, P = 3, 4
    L = oracle.Layout(sizes, k)
    N = L.N
    rng = np.random.Generator(np.random.PCG64(9))
    xs = [rng.standard_normal(N, dtype=np.float32) for _ in range(P)]
    w0 = rng.standard_normal(N, dtype=np.float32)
    v0 = rng.standard_normal(N, dtype=np.float32)
    order = np.array([[1, 0, 3, 2], [3, 2, 1, 0], [0, 1, 2, 3]], np.int32)
    w1, v1 = w0.copy(), v0.copy()
    g1 = oracle.reduce_update(L, xs, w1, v1, 0.1, 0.9, 1e-3, order=order)
    for packet in (256, 768, 5000):
        g2, w2, v2 = np.zeros(N, np.float32), w0.copy(), v0.copy()
        cuts = list(range(0, N, packet)) + [N]
        for b, e in reversed(list(zip(cuts[:-1], cuts[1:]))):
            oracle.reduce_update_range(L, xs, g2, w2, v2, 0.1, 0.9, 1e-3, b, e, order=order)
        pins.assert_bits_equal(g2, g1, "g")
        pins.assert_bits_equal(w2, w1, "w")
        pins.assert_bits_equal(v2, v1, "v")
    # one packet leaves everything else alone
    g3, w3, v3 = np.full(N, 5.0, np.float32), w0.copy(), v0.copy()
    oracle.reduce_update_range(L, xs, g3, w3, v3, 0.1, 0.9, 1e-3, 1024, 2048, order=order)
    out = np.ones(N, bool)
    out[1024:2048] = False
    assert np.all(g3[out] == 5.0) and np.array_equal(w3[out], w0[out]) and np.array_equal(v3[out], v0[out])
    pins.assert_bits_equal(g3[1024:2048], g1[1024:2048], "packet g")
