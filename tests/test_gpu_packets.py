"""GPU parity of mc_reduce_update_range: the step cut into packets (Section 4.2's pipelined
reductions), in any order and on two streams, against the oracle."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle  # noqa: E402
from paper_1711_00705_amd import mc  # noqa: E402
from paper_1711_00705_amd import workloads as wl  # noqa: E402
import gpu_harness as gh  # noqa: E402


def _setup(sizes, k, P, seed=1):
    L = mc.Layout(sizes, k)
    O = oracle.Layout(sizes, k)
    N = L.N
    rng = np.random.Generator(np.random.PCG64(seed))
    xs = [rng.standard_normal(N, dtype=np.float32) * np.float32(1e-3) for _ in range(P)]
    w = rng.standard_normal(N, dtype=np.float32) * np.float32(0.05)
    v = rng.standard_normal(N, dtype=np.float32) * np.float32(0.01)
    return L, O, N, xs, w, v


def test_one_packet_touches_only_its_range():
    sizes = [5000, 1000, 3003]
    k, P = 3, 4
    L, O, N, xs, w0, v0 = _setup(sizes, k, P)
    order = wl.rotation_order(k, P)
    xd = [gh.to_dev(x) for x in xs]
    for begin, end in ((0, 256), (2816, 6400), (8960, N), (512, 512), (0, N)):
        g, w, v = gh.dev_empty(N), gh.to_dev(w0), gh.to_dev(v0)
        mc.reduce_update_range(L, [x.data_ptr() for x in xd], order, g.data_ptr(), w.data_ptr(), v.data_ptr(),
                               0.1, 0.9, 1e-4, begin, end, gh.stream_handle())
        torch.cuda.synchronize()
        gr = np.full(N, np.nan, np.float32)
        gr.view(np.uint32)[:] = 0xFFFFFFFF
        wr, vr = w0.copy(), v0.copy()
        oracle.reduce_update_range(O, xs, gr, wr, vr, 0.1, 0.9, 1e-4, begin, end, order=order)
        assert np.array_equal(g.cpu().numpy().view(np.uint32), gr.view(np.uint32)), (begin, end)
        gh.assert_bits(w.cpu().numpy(), wr, f"w [{begin},{end})")
        gh.assert_bits(v.cpu().numpy(), vr, f"v [{begin},{end})")


@pytest.mark.parametrize("packet", [256, 1024, 7936, 99840])
def test_packets_in_any_order_on_two_streams_equal_the_whole_step(packet):
    sizes = [70000, 12345, 4099, 30000]
    k, P = 4, 5
    L, O, N, xs, w0, v0 = _setup(sizes, k, P, seed=packet)
    order = wl.random_order(k, P, seed=3)
    xd = [gh.to_dev(x) for x in xs]
    g, w, v = gh.dev_empty(N), gh.to_dev(w0), gh.to_dev(v0)
    cuts = list(range(0, N, packet)) + [N]
    packets = list(zip(cuts[:-1], cuts[1:]))
    rng = np.random.Generator(np.random.PCG64(8))
    rng.shuffle(packets)
    print(f"packet={packet}: {len(packets)} packets", flush=True)
    main = torch.cuda.current_stream()
    side = torch.cuda.Stream()
    side.wait_stream(main)
    for i, (b, e) in enumerate(packets):
        st = side if i % 2 else main
        mc.reduce_update_range(L, [x.data_ptr() for x in xd], order, g.data_ptr(), w.data_ptr(), v.data_ptr(),
                               0.1, 0.9, 1e-4, b, e, int(st.cuda_stream))
    main.wait_stream(side)
    torch.cuda.synchronize()
    wr, vr = w0.copy(), v0.copy()
    gr = oracle.reduce_update(O, xs, wr, vr, 0.1, 0.9, 1e-4, order=order)
    gh.assert_bits(g.cpu().numpy(), gr, "g")
    gh.assert_bits(w.cpu().numpy(), wr, "w")
    gh.assert_bits(v.cpu().numpy(), vr, "v")


def test_packets_with_roles():
    sizes = [20000, 4000]
    k, P = 4, 6
    L, O, N, xs, w0, v0 = _setup(sizes, k, P, seed=5)
    n_terms = np.array([6, 2, 0, 3], np.int32)
    do_update = np.array([1, 0, 1, 0], np.uint8)
    xd = [gh.to_dev(x) for x in xs]
    g, w, v = gh.dev_empty(N, fill=0), gh.to_dev(w0), gh.to_dev(v0)
    for b in range(0, N, 2048):
        mc.reduce_update_range(L, [x.data_ptr() for x in xd], None, g.data_ptr(), w.data_ptr(), v.data_ptr(),
                               0.1, 0.9, 1e-4, b, min(N, b + 2048), gh.stream_handle(),
                               n_terms=n_terms, do_update=do_update)
    torch.cuda.synchronize()
    gr, wr, vr = np.zeros(N, np.float32), w0.copy(), v0.copy()
    oracle.reduce_update_roles(O, xs, n_terms, do_update, gr, wr, vr, 0.1, 0.9, 1e-4)
    gh.assert_bits(g.cpu().numpy(), gr, "g")
    gh.assert_bits(w.cpu().numpy(), wr, "w")
    gh.assert_bits(v.cpu().numpy(), vr, "v")
