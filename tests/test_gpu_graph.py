"""Every step entry point launches kernels only, so a step can be captured into a graph once
the layout is prepared.  The staged step (P packs, reduce_update, unpack) is captured and
replayed several times, with the program's own eager work and synchronisation between replays,
and every replay is checked against the oracle carrying state."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle  # noqa: E402
from paper_1711_00705_amd import mc  # noqa: E402
from paper_1711_00705_amd import workloads as wl  # noqa: E402
import gpu_harness as gh  # noqa: E402


def test_staged_step_in_a_graph():
    sizes = [64, 64, 36864, 64, 16385, 4096, 255, 147456, 512, 1000]     # odd sizes: unaligned gather too
    k, P = 3, 3
    L = mc.Layout(sizes, k)
    O = oracle.Layout(sizes, k)
    N = L.N
    L.prepare()                                      # the only allocation happens before capture
    order = wl.rotation_order(k, P)
    host_x = [wl.contribution_tensors(sizes, p) for p in range(P)]
    host_w = wl.weight_tensors(sizes)
    dev_x = [gh.place_tensors(h)[0] for h in host_x]
    dev_w, _ = gh.place_tensors(host_w)
    tabs = [mc.ptr_table(gh.ptrs(d)) for d in dev_x]
    w_tab = mc.ptr_table(gh.ptrs(dev_w))
    flats = [gh.dev_empty(N) for _ in range(P)]
    flat_tab = mc.ptr_table([f.data_ptr() for f in flats])
    w, v, g = gh.dev_empty(N), gh.dev_empty(N, fill=0), gh.dev_empty(N)
    main = torch.cuda.current_stream()
    mc.pack(L, w_tab, w.data_ptr(), int(main.cuda_stream))

    def step(sh):
        for p in range(P):
            mc.pack(L, tabs[p], flats[p].data_ptr(), sh)
        mc.reduce_update(L, flat_tab, order, g.data_ptr(), w.data_ptr(), v.data_ptr(), 0.1, 0.9, 1e-4, sh)
        mc.unpack(L, w.data_ptr(), w_tab, sh)

    cap = torch.cuda.Stream()
    cap.wait_stream(main)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=cap):
        step(int(torch.cuda.current_stream().cuda_stream))
    torch.cuda.synchronize()
    # capture executed nothing
    assert np.all(g.cpu().numpy().view(np.uint32) == 0xFFFFFFFF)
    xs = [oracle.pack(O, h) for h in host_x]
    wr, vr = oracle.pack(O, host_w), np.zeros(N, np.float32)
    for rep in range(4):
        graph.replay()
        torch.cuda.synchronize()
        gr = oracle.reduce_update(O, xs, wr, vr, 0.1, 0.9, 1e-4, order=order)
        gh.assert_bits(g.cpu().numpy(), gr, f"g replay {rep}")
        gh.assert_bits(w.cpu().numpy(), wr, f"w replay {rep}")
        gh.assert_bits(v.cpu().numpy(), vr, f"v replay {rep}")
        for a, b in zip(dev_w, oracle.unpack(O, wr)):
            gh.assert_bits(a.cpu().numpy(), b, f"unpacked w replay {rep}")
        # eager work between replays: new contributions for the next replay, on the main stream
        host_x = [wl.contribution_tensors(sizes, p, step=rep + 1) for p in range(P)]
        for d, h in zip(dev_x, host_x):
            for t, a in zip(d, h):
                if a.size:
                    t.copy_(torch.from_numpy(a))
        xs = [oracle.pack(O, h) for h in host_x]
        torch.cuda.synchronize()


def test_captured_pair_of_sweep_directions():
    """A graph replays the kernel arguments it captured, the walking direction among them.  A
    caller whose state exceeds the memory-side cache captures the fused step twice, once per
    explicit direction (mc_update_spec.sweep), and alternates the two graphs; every replay must
    give the oracle's bits, and the automatic direction must behave the same eagerly."""
    sizes = [20_000_000, 12, 4100, 14_000_004]        # 34 M elements: 272 MB of weights + momentum
    k, P = 4, 2
    L = mc.Layout(sizes, k)
    O = oracle.Layout(sizes, k)
    N = L.N
    assert 8 * N > (256 << 20)
    L.prepare()
    order = wl.rotation_order(k, P)
    host_x = [wl.contribution_tensors(sizes, p) for p in range(P)]
    host_w = wl.weight_tensors(sizes)
    dev_x = [gh.place_tensors(h)[0] for h in host_x]
    dev_w, _ = gh.place_tensors(host_w)
    dev_v, _ = gh.place_tensors(wl.zero_tensors(sizes))
    sets = mc.set_table([mc.TensorSet(L, gh.ptrs(d)) for d in dev_x])
    wset, vset = mc.TensorSet(L, gh.ptrs(dev_w)), mc.TensorSet(L, gh.ptrs(dev_v))
    g = gh.dev_empty(N)
    main = torch.cuda.current_stream()
    graphs = {}
    for name, sweep in (("forward", mc.SWEEP_FORWARD), ("backward", mc.SWEEP_BACKWARD)):
        spec = mc.update_spec(0.01, 0.9, 5e-4, state_policy=mc.STATE_RESIDENT, sweep=sweep)
        cap = torch.cuda.Stream()
        cap.wait_stream(main)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=cap):
            mc.fused_step_ex(L, sets, order, g.data_ptr(), wset, vset, spec, int(torch.cuda.current_stream().cuda_stream))
        torch.cuda.synchronize()
        graphs[name] = graph
    assert np.all(g.cpu().numpy().view(np.uint32) == 0xFFFFFFFF), "capture executed nothing"
    xs = [oracle.pack(O, h) for h in host_x]
    wr, vr = oracle.pack(O, host_w), np.zeros(N, np.float32)

    def check(what):
        gr = oracle.reduce_update(O, xs, wr, vr, 0.01, 0.9, 5e-4, order=order)
        gh.assert_bits(g.cpu().numpy(), gr, f"g {what}")
        for a, b in zip(dev_w, oracle.unpack(O, wr)):
            gh.assert_bits(a.cpu().numpy(), b, f"w {what}")
        for a, b in zip(dev_v, oracle.unpack(O, vr)):
            gh.assert_bits(a.cpu().numpy(), b, f"v {what}")

    for rep in range(4):
        name = "forward" if rep % 2 == 0 else "backward"
        print(f"replay {rep}: {name}", flush=True)
        graphs[name].replay()
        torch.cuda.synchronize()
        check(f"replay {rep} ({name})")
        g.view(torch.int32).fill_(-1)                 # eager work between replays
        torch.cuda.synchronize()
    # the automatic direction, eagerly, with resident state: two more steps from the same state
    spec = mc.update_spec(0.01, 0.9, 5e-4, state_policy=mc.STATE_RESIDENT)
    for rep in range(2):
        mc.fused_step_ex(L, sets, order, g.data_ptr(), wset, vset, spec, int(main.cuda_stream))
        torch.cuda.synchronize()
        check(f"eager automatic direction, step {rep}")
