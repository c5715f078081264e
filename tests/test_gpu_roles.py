"""GPU parity of mc_reduce_update_roles (per-colour term counts and update flags) against
the oracle, directly and composed into a whole simulated Allreduce over the paper's trees."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle  # noqa: E402
from oracle import trees  # noqa: E402
from paper_1711_00705_amd import mc  # noqa: E402
from paper_1711_00705_amd import workloads as wl  # noqa: E402
import allreduce_sim as sim  # noqa: E402
import gpu_harness as gh  # noqa: E402


def _gpu_call(L):
    """Adapter with the oracle's signature: uploads, calls the library, downloads."""
    def call(contrib, n_terms, do_update, g, w, v, lr, mu, wd, order):
        s = gh.stream_handle()
        xs = [gh.to_dev(x) for x in contrib]
        gd = gh.to_dev(g)
        wd_ = gh.to_dev(w) if w is not None else None
        vd = gh.to_dev(v) if v is not None else None
        mc.reduce_update_roles(L, [x.data_ptr() for x in xs], order, n_terms, do_update, gd.data_ptr(),
                               wd_.data_ptr() if w is not None else None,
                               vd.data_ptr() if v is not None else None, lr, mu, wd, s)
        torch.cuda.synchronize()
        g[:] = gd.cpu().numpy()
        if w is not None:
            w[:] = wd_.cpu().numpy()
            v[:] = vd.cpu().numpy()
    call.bounds = L.colour_bounds()
    return call


def _oracle_call(O):
    def call(contrib, n_terms, do_update, g, w, v, lr, mu, wd, order):
        oracle.reduce_update_roles(O, contrib, n_terms, do_update, g, w, v, lr, mu, wd, order=order)
    call.bounds = O.bounds
    return call


@pytest.mark.parametrize("k,P", [(4, 5), (8, 8), (3, 12), (40, 6)])
def test_mixed_roles_match_oracle(k, P):
    sizes = [30000, 77, 4099]
    L = mc.Layout(sizes, k)
    O = oracle.Layout(sizes, k)
    N = L.N
    rng = np.random.Generator(np.random.PCG64(k * 100 + P))
    xs = [rng.standard_normal(N, dtype=np.float32) * np.float32(1e-3) for _ in range(P)]
    w0 = rng.standard_normal(N, dtype=np.float32) * np.float32(0.05)
    v0 = rng.standard_normal(N, dtype=np.float32) * np.float32(0.01)
    n_terms = rng.integers(0, P + 1, size=k).astype(np.int32)
    do_update = rng.integers(0, 2, size=k).astype(np.uint8)
    n_terms[0], do_update[0] = P, 1
    if k > 2:
        n_terms[1], n_terms[2], do_update[2] = 0, 1, 0
    order = wl.random_order(k, P, seed=5)
    print(f"roles k={k} P={P} n_terms={n_terms.tolist()[:8]} upd={do_update.tolist()[:8]}", flush=True)
    g_ref = np.full(N, 7.0, np.float32)
    w_ref, v_ref = w0.copy(), v0.copy()
    oracle.reduce_update_roles(O, xs, n_terms, do_update, g_ref, w_ref, v_ref, 0.1, 0.9, 1e-4, order=order)
    g, w, v = np.full(N, 7.0, np.float32), w0.copy(), v0.copy()
    _gpu_call(L)(xs, n_terms, do_update, g, w, v, 0.1, 0.9, 1e-4, order)
    gh.assert_bits(g, g_ref, "g")
    gh.assert_bits(w, w_ref, "w")
    gh.assert_bits(v, v_ref, "v")


def test_sum_only_needs_no_weights_and_update_only_needs_no_grad_out():
    sizes = [10000, 3]
    k, P = 2, 3
    L = mc.Layout(sizes, k)
    O = oracle.Layout(sizes, k)
    N = L.N
    rng = np.random.Generator(np.random.PCG64(1))
    xs_h = [rng.standard_normal(N, dtype=np.float32) for _ in range(P)]
    xs = [gh.to_dev(x) for x in xs_h]
    g = gh.dev_empty(N)
    mc.reduce_update_roles(L, [x.data_ptr() for x in xs], None, [P, 2], [0, 0], g.data_ptr(), None, None,
                           0.1, 0.9, 0.0, gh.stream_handle())
    torch.cuda.synchronize()
    g_ref = np.empty(N, np.float32)
    oracle.reduce_update_roles(O, xs_h, [P, 2], [0, 0], g_ref, None, None, 0.1, 0.9, 0.0)
    gh.assert_bits(g.cpu().numpy(), g_ref, "sum only")
    w0 = rng.standard_normal(N, dtype=np.float32)
    w, v = gh.to_dev(w0), gh.dev_empty(N, fill=0)
    mc.reduce_update_roles(L, [x.data_ptr() for x in xs], None, [P, P], [1, 1], None, w.data_ptr(), v.data_ptr(),
                           0.1, 0.9, 0.0, gh.stream_handle())
    torch.cuda.synchronize()
    wr, vr = w0.copy(), np.zeros(N, np.float32)
    oracle.reduce_update(O, xs_h, wr, vr, 0.1, 0.9, 0.0)
    gh.assert_bits(w.cpu().numpy(), wr, "update only w")
    gh.assert_bits(v.cpu().numpy(), vr, "update only v")


@pytest.mark.parametrize("n_nodes,k,m", [(8, 4, 4), (5, 2, 2), (9, 4, 1)])
def test_whole_allreduce_on_gpu_matches_oracle_and_plain_sum(n_nodes, k, m):
    sizes = [9000, 33, 2500]
    L = mc.Layout(sizes, k)
    O = oracle.Layout(sizes, k)
    N = L.N
    # the library's own trees drive the GPU side, the oracle's the CPU side
    parents_gpu = mc.colour_trees(n_nodes, k).tolist()
    parents_ref = trees.colour_trees(n_nodes, k)
    assert parents_gpu == parents_ref
    rng = np.random.Generator(np.random.PCG64(50 + n_nodes))
    local = [[rng.standard_normal(N, dtype=np.float32) * np.float32(1e-3) for _ in range(m)]
             for _ in range(n_nodes)]
    w0 = rng.standard_normal(N, dtype=np.float32) * np.float32(0.05)
    v0 = np.zeros(N, np.float32)
    print(f"allreduce sim n={n_nodes} k={k} m={m}", flush=True)
    g1, w1, v1 = sim.simulate(_gpu_call(L), parents_gpu, m, local, w0, v0, N, k, 0.1, 0.9, 1e-4)
    g2, w2, v2 = sim.simulate(_oracle_call(O), parents_ref, m, local, w0, v0, N, k, 0.1, 0.9, 1e-4)
    gh.assert_bits(g1, g2, "g_total")
    for node in range(n_nodes):
        gh.assert_bits(w1[node], w2[node], f"w node {node}")
        gh.assert_bits(v1[node], v2[node], f"v node {node}")
        gh.assert_bits(w1[node], w1[0], "all nodes agree")
    for c in range(k):
        lo, hi = int(O.bounds[c]), int(O.bounds[c + 1])
        gh.assert_bits(g1[lo:hi], sim.tree_order_sum(parents_ref[c], m, local, lo, hi), f"tree order colour {c}")


def _fused_call(L, O, sizes):
    """The same adapter through mc_fused_step_ex: every contribution, the weights and the
    momentum live in separate per-layer tensors (odd layers misaligned), g is flat."""
    def call(contrib, n_terms, do_update, g, w, v, lr, mu, wd, order):
        s = gh.stream_handle()
        mis = [0, 0, 1]
        dev_x = [gh.place_tensors(oracle.unpack(O, np.ascontiguousarray(x)), mis)[0] for x in contrib]
        sets = [mc.TensorSet(L, gh.ptrs(d)) for d in dev_x]
        gd = gh.to_dev(g)
        wset = vset = None
        if w is not None:
            dev_w, _ = gh.place_tensors(oracle.unpack(O, w), mis)
            dev_v, _ = gh.place_tensors(oracle.unpack(O, v), mis)
            wset, vset = mc.TensorSet(L, gh.ptrs(dev_w)), mc.TensorSet(L, gh.ptrs(dev_v))
        mc.fused_step_ex(L, sets, order, gd.data_ptr(), wset, vset, mc.update_spec(lr, mu, wd), s,
                         n_terms=n_terms, do_update=do_update)
        torch.cuda.synchronize()
        g[:] = gd.cpu().numpy()
        if w is not None:
            w[:] = oracle.pack(O, [t.cpu().numpy() for t in dev_w])
            v[:] = oracle.pack(O, [t.cpu().numpy() for t in dev_v])
    call.bounds = L.colour_bounds()
    return call


@pytest.mark.parametrize("sizes", [[9000, 32, 2500], [9001, 33, 2503]], ids=["aligned", "odd"])
def test_fused_roles_match_oracle_and_compose_to_an_allreduce(sizes):
    n_nodes, k, m = 8, 4, 2
    L = mc.Layout(sizes, k)
    O = oracle.Layout(sizes, k)
    N = L.N
    rng = np.random.Generator(np.random.PCG64(5))
    # one mixed-role call against the oracle
    P = 5
    xs = [rng.standard_normal(N, dtype=np.float32) * np.float32(1e-3) for _ in range(P)]
    w0 = rng.standard_normal(N, dtype=np.float32) * np.float32(0.05)
    v0 = rng.standard_normal(N, dtype=np.float32) * np.float32(0.01)
    n_terms, do_update = [P, 0, 2, 3], [1, 1, 0, 1]
    order = wl.random_order(k, P, seed=1)
    g1, w1, v1 = np.full(N, 7.0, np.float32), w0.copy(), v0.copy()
    _fused_call(L, O, sizes)(xs, n_terms, do_update, g1, w1, v1, 0.1, 0.9, 1e-4, order)
    g2, w2, v2 = np.full(N, 7.0, np.float32), w0.copy(), v0.copy()
    oracle.reduce_update_roles(O, xs, n_terms, do_update, g2, w2, v2, 0.1, 0.9, 1e-4, order=order)
    gh.assert_bits(g1, g2, "fused roles g")
    gh.assert_bits(w1, w2, "fused roles w")
    gh.assert_bits(v1, v2, "fused roles v")
    # sum-only call needs no weights
    g3 = np.zeros(N, np.float32)
    _fused_call(L, O, sizes)(xs, [2, 2, 2, 2], [0, 0, 0, 0], g3, None, None, 0.1, 0.9, 1e-4, None)
    gh.assert_bits(g3, xs[0] + xs[1], "fused sum only")
    # the whole Allreduce composed from fused role calls
    parents = mc.colour_trees(n_nodes, k).tolist()
    local = [[rng.standard_normal(N, dtype=np.float32) * np.float32(1e-3) for _ in range(m)] for _ in range(n_nodes)]
    print(f"fused allreduce sim sizes={sizes}", flush=True)
    ga, wa, va = sim.simulate(_fused_call(L, O, sizes), parents, m, local, w0, np.zeros(N, np.float32), N, k, 0.1, 0.9, 1e-4)
    gb, wb, vb = sim.simulate(_oracle_call(O), parents, m, local, w0, np.zeros(N, np.float32), N, k, 0.1, 0.9, 1e-4)
    gh.assert_bits(ga, gb, "g_total")
    for node in range(n_nodes):
        gh.assert_bits(wa[node], wb[node], f"w node {node}")
        gh.assert_bits(va[node], vb[node], f"v node {node}")
