"""GPU parity of the update variants: Nesterov step, hyper-parameters read from device memory,
a captured step replayed with a changing learning rate, and a ring-ordered reduction."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle  # noqa: E402
from oracle import schedule  # noqa: E402
from paper_1711_00705_amd import mc  # noqa: E402
from paper_1711_00705_amd import workloads as wl  # noqa: E402
import gpu_harness as gh  # noqa: E402

CNN_SIZES = [64, 64, 36864, 64, 16384, 4096, 256, 147456, 512, 1000]


def _flat_inputs(O, sizes, P, seed=3):
    xs = [oracle.pack(O, wl.contribution_tensors(sizes, p, heavy_tail=True)) for p in range(P)]
    w = oracle.pack(O, wl.weight_tensors(sizes))
    rng = np.random.Generator(np.random.PCG64(seed))
    v = rng.standard_normal(O.N, dtype=np.float32) * np.float32(0.01)
    return xs, w, v


@pytest.mark.parametrize("sizes", [list(wl.workload("tiny").sizes), CNN_SIZES], ids=["tiny", "cnn"])
@pytest.mark.parametrize("nesterov", [0, 1])
@pytest.mark.parametrize("from_device", [False, True])
def test_reduce_update_ex(sizes, nesterov, from_device):
    k, P = 3, 4
    L, O = mc.Layout(sizes, k), oracle.Layout(sizes, k)
    N = L.N
    xs, w0, v0 = _flat_inputs(O, sizes, P)
    order = wl.rotation_order(k, P)
    lr, mu, wd = 0.1, 0.9, 1e-4
    s = gh.stream_handle()
    xd = [gh.to_dev(x) for x in xs]
    g, w, v = gh.dev_empty(N), gh.to_dev(w0), gh.to_dev(v0)
    if from_device:
        hyper = gh.dev_empty(3)
        mc.hyper_write(hyper.data_ptr(), lr, mu, wd, s)
        spec = mc.update_spec(7.0, 7.0, 7.0, hyper_dev_ptr=hyper.data_ptr(), nesterov=nesterov)  # immediates ignored
    else:
        spec = mc.update_spec(lr, mu, wd, nesterov=nesterov)
    print(f"reduce_update_ex N={N} nesterov={nesterov} from_device={from_device}", flush=True)
    mc.reduce_update_ex(L, [x.data_ptr() for x in xd], order, g.data_ptr(), w.data_ptr(), v.data_ptr(), spec, s)
    torch.cuda.synchronize()
    wr, vr = w0.copy(), v0.copy()
    fn = oracle.reduce_update_nesterov if nesterov else oracle.reduce_update
    gr = fn(O, xs, wr, vr, lr, mu, wd, order=order)
    gh.assert_bits(g.cpu().numpy(), gr, "g")
    gh.assert_bits(v.cpu().numpy(), vr, "v")
    gh.assert_bits(w.cpu().numpy(), wr, "w")


@pytest.mark.parametrize("nesterov", [0, 1])
def test_fused_step_ex(nesterov):
    sizes, k, P = CNN_SIZES, 3, 4
    L, O = mc.Layout(sizes, k), oracle.Layout(sizes, k)
    N = L.N
    host_x = [wl.contribution_tensors(sizes, p, heavy_tail=True) for p in range(P)]
    host_w = wl.weight_tensors(sizes)
    dev_x = [gh.place_tensors(h)[0] for h in host_x]
    dev_w, _ = gh.place_tensors(host_w)
    dev_v, _ = gh.place_tensors(wl.zero_tensors(sizes))
    sets = [mc.TensorSet(L, gh.ptrs(d)) for d in dev_x]
    wset, vset = mc.TensorSet(L, gh.ptrs(dev_w)), mc.TensorSet(L, gh.ptrs(dev_v))
    g = gh.dev_empty(N)
    hyper = gh.dev_empty(3)
    s = gh.stream_handle()
    mc.hyper_write(hyper.data_ptr(), 0.05, 0.8, 1e-3, s)
    mc.fused_step_ex(L, sets, None, g.data_ptr(), wset, vset,
                     mc.update_spec(hyper_dev_ptr=hyper.data_ptr(), nesterov=nesterov), s)
    torch.cuda.synchronize()
    wr, vr = oracle.pack(O, host_w), np.zeros(N, np.float32)
    fn = oracle.reduce_update_nesterov if nesterov else oracle.reduce_update
    gr = fn(O, [oracle.pack(O, h) for h in host_x], wr, vr, 0.05, 0.8, 1e-3)
    gh.assert_bits(g.cpu().numpy(), gr, "g")
    for a, b in zip(dev_w, oracle.unpack(O, wr)):
        gh.assert_bits(a.cpu().numpy(), b, "w")
    for a, b in zip(dev_v, oracle.unpack(O, vr)):
        gh.assert_bits(a.cpu().numpy(), b, "v")


def test_captured_step_replays_with_the_scheduled_learning_rate():
    """One fused step captured into a graph (kernel nodes only) reads {lr, mu, wd} from device
    memory; between replays the host advances the Section 5 schedule with mc_hyper_write.  Every
    replay is checked against the oracle carrying state, with eager work and synchronisation
    between replays."""
    sizes, k, P = CNN_SIZES, 4, 4
    L, O = mc.Layout(sizes, k), oracle.Layout(sizes, k)
    N = L.N
    order = wl.rotation_order(k, P)
    host_x = [wl.contribution_tensors(sizes, p) for p in range(P)]
    host_w = wl.weight_tensors(sizes)
    dev_x = [gh.place_tensors(h)[0] for h in host_x]
    dev_w, _ = gh.place_tensors(host_w)
    dev_v, _ = gh.place_tensors(wl.zero_tensors(sizes))
    sets = mc.set_table([mc.TensorSet(L, gh.ptrs(d)) for d in dev_x])
    wset, vset = mc.TensorSet(L, gh.ptrs(dev_w)), mc.TensorSet(L, gh.ptrs(dev_v))
    g = gh.dev_empty(N)
    hyper = gh.dev_empty(3)
    spec = mc.update_spec(hyper_dev_ptr=hyper.data_ptr(), nesterov=1)
    mu, wd = 0.9, 1e-4
    main = torch.cuda.current_stream()
    mc.hyper_write(hyper.data_ptr(), 0.0, 0.0, 0.0, int(main.cuda_stream))   # lr = mu = wd = 0: a dry run
    cap = torch.cuda.Stream()
    cap.wait_stream(main)
    with torch.cuda.stream(cap):
        mc.fused_step_ex(L, sets, order, g.data_ptr(), wset, vset, spec, int(cap.cuda_stream))
    torch.cuda.synchronize()
    # the dry run left w alone and set v = g (mu = wd = 0): restore v
    for t in dev_v:
        t.zero_()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=cap):
        mc.fused_step_ex(L, sets, order, g.data_ptr(), wset, vset, spec,
                         int(torch.cuda.current_stream().cuda_stream))
    torch.cuda.synchronize()
    # capture must not have executed anything
    for a, b in zip(dev_w, host_w):
        gh.assert_bits(a.cpu().numpy(), b, "weights changed during capture")
    wr, vr = oracle.pack(O, host_w), np.zeros(N, np.float32)
    xs = [oracle.pack(O, h) for h in host_x]
    for i, epoch in enumerate((0.0, 1.25, 2.5, 5.0, 31.0)):
        lr_lib = mc.lr_schedule(0.1, 32, 256, 5.0, 30.0, epoch)
        assert lr_lib == pytest.approx(schedule.lr_at(epoch, 0.1, 32, 256, 5.0, 30.0), rel=2e-7)
        mc.hyper_write(hyper.data_ptr(), lr_lib, mu, wd, int(main.cuda_stream))
        graph.replay()
        torch.cuda.synchronize()
        gr = oracle.reduce_update_nesterov(O, xs, wr, vr, lr_lib, mu, wd, order=order)
        print(f"replay {i}: epoch {epoch} lr {lr_lib}", flush=True)
        gh.assert_bits(g.cpu().numpy(), gr, f"g replay {i}")
        for a, b in zip(dev_w, oracle.unpack(O, wr)):
            gh.assert_bits(a.cpu().numpy(), b, f"w replay {i}")
        for a, b in zip(dev_v, oracle.unpack(O, vr)):
            gh.assert_bits(a.cpu().numpy(), b, f"v replay {i}")
        # eager work of the program between replays
        _ = (dev_w[2] * 1.0).sum().item()


def test_ring_ordered_reduction():
    """The paper's ring baseline (Section 5.1) reduces along the ring to one root: every node adds
    its own m replicas to the partial sum that arrived from its predecessor.  With one colour that
    is a per-rank call with m or m+1 terms; composed over the ring it must give the exact sum
    (integer inputs) and the same bits as the oracle doing the same walk."""
    sizes, n_nodes, m = [5000, 33, 2048], 5, 2
    L, O = mc.Layout(sizes, 1), oracle.Layout(sizes, 1)
    N = L.N
    rng = np.random.Generator(np.random.PCG64(77))
    local_int = [[rng.integers(-500, 501, size=N).astype(np.float32) for _ in range(m)] for _ in range(n_nodes)]
    local_f = [[rng.standard_normal(N, dtype=np.float32) for _ in range(m)] for _ in range(n_nodes)]
    w0 = rng.standard_normal(N, dtype=np.float32)
    s = gh.stream_handle()
    for local, exact in ((local_int, True), (local_f, False)):
        # GPU walk: node n-1 starts, node 0 is the root and applies the update
        incoming_d, incoming_h = None, None
        w, v = gh.to_dev(w0), gh.dev_empty(N, fill=0)
        wr, vr = w0.copy(), np.zeros(N, np.float32)
        for node in range(n_nodes - 1, -1, -1):
            terms_h = list(local[node]) + ([incoming_h] if incoming_h is not None else [np.zeros(N, np.float32)])
            terms_d = [gh.to_dev(t) for t in terms_h]
            n_terms = [m + (1 if incoming_h is not None else 0)]
            root = node == 0
            out_d = gh.dev_empty(N)
            mc.reduce_update_roles(L, [t.data_ptr() for t in terms_d], None, n_terms, [1 if root else 0],
                                   out_d.data_ptr(), w.data_ptr(), v.data_ptr(), 0.1, 0.9, 1e-4, s)
            torch.cuda.synchronize()
            out_h = np.zeros(N, np.float32)
            oracle.reduce_update_roles(O, terms_h, n_terms, [1 if root else 0], out_h, wr, vr, 0.1, 0.9, 1e-4)
            gh.assert_bits(out_d.cpu().numpy(), out_h, f"partial at node {node}")
            incoming_d, incoming_h = out_d, out_h
        if exact:
            total = np.zeros(N, np.int64)
            for node in local:
                for x in node:
                    total += x.astype(np.int64)
            assert np.array_equal(incoming_h.astype(np.int64), total)
        gh.assert_bits(w.cpu().numpy(), wr, "w at the root")
        gh.assert_bits(v.cpu().numpy(), vr, "v at the root")
