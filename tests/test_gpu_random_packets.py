"""Randomised parity of the packet forms: seeded layouts, colour counts, contribution counts and
sequences; every colour cut into packets of a random 256-aligned length; the packets taken in a
random order.  Each case goes through mc_reduce_update_range (one call per packet, two streams)
and through the resident mc_reduce_update_packets (a random number of workgroups; flags raised
beforehand, or packets delivered on a second stream while the reducer polls), and must give the
bits of the oracle's whole step.  Every wait in the reducer is bounded by its poll budget.
MC_RANDOM_CASES raises the number of cases."""
import os

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle  # noqa: E402
from paper_1711_00705_amd import mc  # noqa: E402
from paper_1711_00705_amd import workloads as wl  # noqa: E402
import gpu_harness as gh  # noqa: E402

N_CASES = max(12, int(os.environ.get("MC_RANDOM_CASES", "24")) // 2)


def _case(seed):
    rng = np.random.Generator(np.random.PCG64(88000 + seed))
    if rng.integers(0, 2):
        sizes = [int(4 * rng.integers(1, 60000)) for _ in range(int(rng.integers(1, 12)))]
    else:
        sizes = [int(rng.integers(0, 90000)) for _ in range(int(rng.integers(1, 12)))]
    if sum(sizes) == 0:
        sizes.append(5)
    k = int(rng.choice([1, 2, 3, 4, 8, 32]))
    P = int(rng.choice([1, 2, 3, 4, 5, 8, 9]))
    if k * P > 256:
        P = 256 // k
    order = [None, wl.rotation_order(k, P), wl.random_order(k, P, seed=seed)][int(rng.integers(0, 3))]
    return sizes, k, P, order, rng


@pytest.mark.parametrize("seed", range(N_CASES))
def test_random_packets(seed):
    sizes, k, P, order, rng = _case(seed)
    L = mc.Layout(sizes, k)
    O = oracle.Layout(sizes, k)
    N = L.N
    bounds = [int(b) for b in L.colour_bounds()]
    pk = []
    for c in range(k):
        lo, hi = bounds[c], bounds[c + 1]
        b = lo
        while b < hi:
            e = min(hi, b + 256 * int(rng.integers(1, 200)))
            pk.append((b, e))
            b = e
    pk = [pk[i] for i in rng.permutation(len(pk))]
    n_blocks = int(rng.choice([1, 7, 64, 256, 512]))
    n_blocks = min(n_blocks, 2 * torch.cuda.get_device_properties(0).multi_processor_count)   # the entry point's limit
    deliver = bool(rng.integers(0, 2)) and P >= 2
    lr, mu, wd = 0.1, 0.9, 1e-4
    print(f"random packets {seed}: n={len(sizes)} N={N} k={k} P={P} packets={len(pk)} blocks={n_blocks} "
          f"delivered={deliver}", flush=True)
    xs = [rng.standard_normal(N, dtype=np.float32) * np.float32(1e-3) for _ in range(P)]
    w0 = rng.standard_normal(N, dtype=np.float32) * np.float32(0.05)
    v0 = rng.standard_normal(N, dtype=np.float32) * np.float32(0.01)
    w_ref, v_ref = w0.copy(), v0.copy()
    g_ref = oracle.reduce_update(O, xs, w_ref, v_ref, lr, mu, wd, order=order)

    main, side = torch.cuda.current_stream(), torch.cuda.Stream()
    s, ss = int(main.cuda_stream), int(side.cuda_stream)
    xd = [gh.to_dev(x) for x in xs]
    ptrs = [x.data_ptr() for x in xd]

    # one range call per packet, alternating between two streams (packets are disjoint)
    g, w, v = gh.dev_empty(N), gh.to_dev(w0), gh.to_dev(v0)
    side.wait_stream(main)
    for j, (b, e) in enumerate(pk):
        mc.reduce_update_range(L, ptrs, order, g.data_ptr(), w.data_ptr(), v.data_ptr(), lr, mu, wd, b, e,
                               ss if j % 2 else s)
    main.wait_stream(side)
    torch.cuda.synchronize()
    gh.assert_bits(g.cpu().numpy()[:N], g_ref, f"range case {seed}: g")
    gh.assert_bits(w.cpu().numpy()[:N], w_ref, f"range case {seed}: w")
    gh.assert_bits(v.cpu().numpy()[:N], v_ref, f"range case {seed}: v")

    # the resident reducer
    g, w, v = gh.dev_empty(N), gh.to_dev(w0), gh.to_dev(v0)
    pk_dev = torch.tensor(np.array(pk, dtype=np.int64).reshape(-1), device="cuda")
    ready = torch.full((len(pk),), 0x5A5A, dtype=torch.int32, device="cuda")
    progress = torch.full((n_blocks + mc.PACKETS_STATUS_WORDS,), 9, dtype=torch.int32, device="cuda")
    spec = mc.update_spec(lr, mu, wd)
    arriving = list(range(P // 2, P)) if deliver else []
    src = {p: xd[p] for p in arriving}
    x_run = [gh.dev_empty(N) if p in arriving else xd[p] for p in range(P)]        # NaN canaries until delivered
    arrivals = len(arriving) if deliver else 1

    def reducer(limit):
        mc.reduce_update_packets(L, [x.data_ptr() for x in x_run], order, g.data_ptr(), w.data_ptr(), v.data_ptr(),
                                 spec, pk_dev.data_ptr(), len(pk), ready.data_ptr(), arrivals, limit,
                                 progress.data_ptr(), n_blocks, s)

    mc.packets_reset(ready.data_ptr(), len(pk), progress.data_ptr(), n_blocks, s)
    if deliver:
        side.wait_stream(main)
        reducer(20000)
        for j, (b, e) in enumerate(pk):
            for p in arriving:
                mc.packet_deliver(x_run[p].data_ptr() + 4 * b, src[p].data_ptr() + 4 * b, e - b,
                                  ready.data_ptr() + 4 * j, ss)
        done = torch.cuda.Event()
        done.record(side)
        main.wait_event(done)
        reducer(20000)
    else:
        for j, (b, e) in enumerate(pk):
            mc.packet_signal(ready.data_ptr(), j, e - b, s)
        reducer(1000)
    torch.cuda.synchronize()
    pr = progress.cpu().numpy()
    assert np.all(pr[:n_blocks] == len(pk)) and pr[n_blocks + 1] == 0, f"packets case {seed}: not every packet done"
    gh.assert_bits(g.cpu().numpy()[:N], g_ref, f"packets case {seed}: g")
    gh.assert_bits(w.cpu().numpy()[:N], w_ref, f"packets case {seed}: w")
    gh.assert_bits(v.cpu().numpy()[:N], v_ref, f"packets case {seed}: v")
