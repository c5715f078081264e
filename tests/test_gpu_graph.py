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
