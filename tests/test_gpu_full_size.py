"""GPU parity at the full sizes of the measured configurations, in the default launch
configuration (the one bench.py times).  The oracle is fast enough to check every element."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle  # noqa: E402
from paper_1711_00705_amd import mc  # noqa: E402
from paper_1711_00705_amd import workloads as wl  # noqa: E402
import gpu_harness as gh  # noqa: E402


@pytest.mark.parametrize("name,order_kind", [
    ("resnet50", "identity"), ("resnet50", "rotation"),
    ("resnet50_heavy", "identity"), ("resnet50_heavy", "rotation"),
    ("vgg16", "rotation"),
])
def test_full_size_step(name, order_kind):
    cfg = wl.workload(name)
    print(f"full size {name} N={cfg.total} P={cfg.P} k={cfg.k} order={order_kind}", flush=True)
    order = None if order_kind == "identity" else wl.rotation_order(cfg.k, cfg.P)
    st = gh.Step(cfg.sizes, cfg.k)
    xs = [wl.contribution_tensors(cfg.sizes, p, heavy_tail=cfg.heavy_tail) for p in range(cfg.P)]
    w = wl.weight_tensors(cfg.sizes)
    v = wl.zero_tensors(cfg.sizes)
    gpu, ref = st.run(xs, w, v, cfg.lr, cfg.mu, cfg.wd, order=order)
    st.check(gpu, ref, cfg.lr, cfg.mu, cfg.wd, name)
    torch.cuda.empty_cache()


def test_full_size_odd_layout_staged():
    """ResNet-50 with every tensor one element longer through mc_pack x P, mc_reduce_update and
    mc_unpack: every flat offset after the first tensor is misaligned against the 16-byte aligned
    tensors, so pack and unpack run their 32-bit path on the tensor side at full size."""
    base = wl.workload("resnet50")
    sizes = [s + 1 for s in base.sizes]
    print(f"full size staged, odd layout N={sum(sizes)}", flush=True)
    st = gh.Step(sizes, base.k)
    xs = [wl.contribution_tensors(sizes, p) for p in range(base.P)]
    gpu, ref = st.run(xs, wl.weight_tensors(sizes), wl.zero_tensors(sizes), base.lr, base.mu, base.wd,
                      order=wl.rotation_order(base.k, base.P))
    st.check(gpu, ref, base.lr, base.mu, base.wd, "staged odd layout")
    torch.cuda.empty_cache()


def test_googlenet_hundred_steps_carry_state():
    cfg = wl.workload("googlenet")
    L = mc.Layout(cfg.sizes, cfg.k)
    O = oracle.Layout(cfg.sizes, cfg.k)
    N = L.N
    order = wl.rotation_order(cfg.k, cfg.P)
    s = gh.stream_handle()
    w_layers, _ = gh.place_tensors(wl.weight_tensors(cfg.sizes))
    w = gh.gpu_pack(L, w_layers)
    v = gh.dev_empty(N, fill=0)
    g = gh.dev_empty(N)
    wr = oracle.pack(O, wl.weight_tensors(cfg.sizes))
    vr = np.zeros(N, np.float32)
    flats = [gh.dev_empty(N) for _ in range(cfg.P)]
    for step in range(cfg.steps):
        host = [wl.contribution_tensors(cfg.sizes, p, step=step) for p in range(cfg.P)]
        keep = []
        for p in range(cfg.P):
            dts, _ = gh.place_tensors(host[p])
            keep.append(dts)
            mc.pack(L, gh.ptrs(dts), flats[p].data_ptr(), s)
        mc.reduce_update(L, [f.data_ptr() for f in flats], order, g.data_ptr(), w.data_ptr(),
                         v.data_ptr(), cfg.lr, cfg.mu, cfg.wd, s)
        torch.cuda.synchronize()
        gr = oracle.reduce_update(O, [oracle.pack(O, ts) for ts in host], wr, vr,
                                  cfg.lr, cfg.mu, cfg.wd, order=order)
        if step + 1 in (1, 2, 50, 100):
            print(f"googlenet step {step + 1}", flush=True)
            gh.assert_bits(g.cpu().numpy(), gr, f"g after step {step + 1}")
            gh.assert_bits(w.cpu().numpy(), wr, f"w after step {step + 1}")
            gh.assert_bits(v.cpu().numpy(), vr, f"v after step {step + 1}")
    mc.unpack(L, w.data_ptr(), gh.ptrs(w_layers), s)
    torch.cuda.synchronize()
    for a, b in zip(w_layers, oracle.unpack(O, wr)):
        gh.assert_bits(a.cpu().numpy(), b, "unpacked final weights")


def test_full_size_roles_nesterov_device_hyper():
    """ResNet-50 size through the most general entry point: per-colour term counts, update only
    on two colours, Nesterov step, {lr, mu, wd} read from device memory."""
    cfg = wl.workload("resnet50_heavy")
    k, P = cfg.k, cfg.P
    L = mc.Layout(cfg.sizes, k)
    O = oracle.Layout(cfg.sizes, k)
    N = L.N
    print(f"full size roles/nesterov N={N} P={P} k={k}", flush=True)
    rng = np.random.Generator(np.random.PCG64(11))
    xs_h = [oracle.pack(O, wl.contribution_tensors(cfg.sizes, p, heavy_tail=True)) for p in range(P)]
    w_h = oracle.pack(O, wl.weight_tensors(cfg.sizes))
    v_h = rng.standard_normal(N, dtype=np.float32) * np.float32(0.01)
    s = gh.stream_handle()
    xd = [gh.to_dev(x) for x in xs_h]
    w, v, g = gh.to_dev(w_h), gh.to_dev(v_h), gh.dev_empty(N)
    hyper = gh.dev_empty(3)
    mc.hyper_write(hyper.data_ptr(), cfg.lr, cfg.mu, cfg.wd, s)
    # uniform call, Nesterov, device hyper-parameters
    mc.reduce_update_ex(L, [x.data_ptr() for x in xd], wl.rotation_order(k, P), g.data_ptr(), w.data_ptr(),
                        v.data_ptr(), mc.update_spec(hyper_dev_ptr=hyper.data_ptr(), nesterov=1), s)
    torch.cuda.synchronize()
    wr, vr = w_h.copy(), v_h.copy()
    gr = oracle.reduce_update_nesterov(O, xs_h, wr, vr, cfg.lr, cfg.mu, cfg.wd, order=wl.rotation_order(k, P))
    gh.assert_bits(g.cpu().numpy(), gr, "g (nesterov)")
    gh.assert_bits(w.cpu().numpy(), wr, "w (nesterov)")
    gh.assert_bits(v.cpu().numpy(), vr, "v (nesterov)")
    # roles on top of that state: colours 0 and 5 update with all terms, colour 2 is skipped, the rest sum 4 terms
    n_terms = np.array([P, 4, 0, 4, 4, P, 4, 4], np.int32)
    do_update = np.array([1, 0, 1, 0, 0, 1, 0, 0], np.uint8)
    mc.reduce_update_roles(L, [x.data_ptr() for x in xd], None, n_terms, do_update, g.data_ptr(), w.data_ptr(),
                           v.data_ptr(), cfg.lr, cfg.mu, cfg.wd, s)
    torch.cuda.synchronize()
    oracle.reduce_update_roles(O, xs_h, n_terms, do_update, gr, wr, vr, cfg.lr, cfg.mu, cfg.wd)
    gh.assert_bits(g.cpu().numpy(), gr, "g (roles)")
    gh.assert_bits(w.cpu().numpy(), wr, "w (roles)")
    gh.assert_bits(v.cpu().numpy(), vr, "v (roles)")


def test_full_size_roles_on_per_layer_tensors():
    """ResNet-50 size through mc_fused_step_ex with a rank's roles (the paper's 8-node, 4-colour
    example, 4 local replicas): the root of colour 0 adds 8 buffers there and 4 elsewhere and updates
    only its own colour; an inner node adds 7 and 4 and updates nothing; then the other colours are
    updated from a broadcast sum.  State is carried from call to call and checked every time."""
    cfg = wl.workload("resnet50")
    k, m = cfg.k, cfg.P
    P = m + k
    L = mc.Layout(cfg.sizes, k)
    O = oracle.Layout(cfg.sizes, k)
    N = L.N
    print(f"full size fused roles N={N} P={P} k={k}", flush=True)
    rng = np.random.Generator(np.random.PCG64(23))
    xs_layers = [wl.contribution_tensors(cfg.sizes, p) for p in range(P)]
    xs_h = [oracle.pack(O, t) for t in xs_layers]
    w_layers = wl.weight_tensors(cfg.sizes)
    v_layers = [rng.standard_normal(s, dtype=np.float32) * np.float32(0.01) for s in cfg.sizes]
    wr, vr = oracle.pack(O, w_layers), oracle.pack(O, v_layers)
    gr = np.zeros(N, np.float32)
    s = gh.stream_handle()
    dev_x = [gh.place_tensors(t)[0] for t in xs_layers]
    dev_w, _ = gh.place_tensors(w_layers)
    dev_v, _ = gh.place_tensors(v_layers)
    sets = mc.set_table([mc.TensorSet(L, gh.ptrs(d)) for d in dev_x])
    wset, vset = mc.TensorSet(L, gh.ptrs(dev_w)), mc.TensorSet(L, gh.ptrs(dev_v))
    g = gh.dev_empty(N, fill=0)
    spec = mc.update_spec(cfg.lr, cfg.mu, cfg.wd)

    def check(what):
        torch.cuda.synchronize()
        gh.assert_bits(g.cpu().numpy(), gr, f"g ({what})")
        for a, b in zip(dev_w, oracle.unpack(O, wr)):
            gh.assert_bits(a.cpu().numpy(), b, f"w ({what})")
        for a, b in zip(dev_v, oracle.unpack(O, vr)):
            gh.assert_bits(a.cpu().numpy(), b, f"v ({what})")

    for what, n_terms, do_update in (("root of colour 0", [8, 4, 4, 4], [1, 0, 0, 0]),
                                     ("inner node of colour 0", [7, 4, 4, 4], [0, 0, 0, 0]),
                                     ("two children here, one there", [6, 5, 4, 4], [0, 1, 0, 0])):
        mc.fused_step_ex(L, sets, None, g.data_ptr(), wset, vset, spec, s, n_terms=n_terms, do_update=do_update)
        oracle.reduce_update_roles(O, xs_h, n_terms, do_update, gr, wr, vr, cfg.lr, cfg.mu, cfg.wd)
        check(what)
    # the non-root colours updated from a broadcast sum (one contribution), colour 0 skipped
    bcast = mc.set_table([mc.TensorSet(L, gh.ptrs(dev_x[5]))])
    mc.fused_step_ex(L, bcast, None, g.data_ptr(), wset, vset, spec, s, n_terms=[0, 1, 1, 1], do_update=[1, 1, 1, 1])
    oracle.reduce_update_roles(O, [xs_h[5]], [0, 1, 1, 1], [1, 1, 1, 1], gr, wr, vr, cfg.lr, cfg.mu, cfg.wd)
    check("update from a broadcast sum")
    torch.cuda.empty_cache()


def test_full_size_packet_pipeline_two_steps():
    """The packet pipeline as bench.py drives it, at ResNet-50 size: two of the four contributions
    land in 16 packets (colours interleaved) on a second stream, paced by mc_delay, while one
    resident reducer of 256 workgroups sums each packet when its flag is complete; then the ordered
    second call.  Two steps in a row (flags and progress reset in between, state carried)."""
    cfg = wl.workload("resnet50")
    k, P = cfg.k, cfg.P
    L = mc.Layout(cfg.sizes, k)
    O = oracle.Layout(cfg.sizes, k)
    N = L.N
    order = wl.rotation_order(k, P)
    n_blocks = min(256, 2 * torch.cuda.get_device_properties(0).multi_processor_count)
    bounds = [int(b) for b in L.colour_bounds()]
    per_colour = []
    for c in range(k):
        lo, hi = bounds[c], bounds[c + 1]
        step = -(-(-(-(hi - lo) // 4)) // 256) * 256
        per_colour.append([(b, min(hi, b + step)) for b in range(lo, hi, step)])
    pk = [p[j] for j in range(max(len(p) for p in per_colour)) for p in per_colour if j < len(p)]
    print(f"full size packet pipeline N={N} packets={len(pk)}", flush=True)
    pk_dev = torch.tensor(np.array(pk, dtype=np.int64).reshape(-1), device="cuda")
    ready = torch.zeros(len(pk), dtype=torch.int32, device="cuda")
    progress = torch.zeros(n_blocks + mc.PACKETS_STATUS_WORDS, dtype=torch.int32, device="cuda")
    main, prod = torch.cuda.current_stream(), torch.cuda.Stream()
    s, ps = int(main.cuda_stream), int(prod.cuda_stream)
    arriving = [2, 3]
    w_h = oracle.pack(O, wl.weight_tensors(cfg.sizes))
    v_h = np.zeros(N, np.float32)
    w, v, g = gh.to_dev(w_h), gh.to_dev(v_h), gh.dev_empty(N)
    spec = mc.update_spec(cfg.lr, cfg.mu, cfg.wd)
    x_dev = [gh.dev_empty(N) for _ in range(P)]
    for step_no in range(2):
        xs_h = [oracle.pack(O, wl.contribution_tensors(cfg.sizes, p, step=step_no)) for p in range(P)]
        src = {p: gh.to_dev(xs_h[p]) for p in arriving}
        for p in range(P):
            if p in arriving:
                x_dev[p].view(torch.int32).fill_(-1)          # NaN canaries until the packets land
            else:
                x_dev[p].copy_(torch.from_numpy(xs_h[p]))
        torch.cuda.synchronize()

        def reducer():
            mc.reduce_update_packets(L, [x.data_ptr() for x in x_dev], order, g.data_ptr(), w.data_ptr(), v.data_ptr(),
                                     spec, pk_dev.data_ptr(), len(pk), ready.data_ptr(), len(arriving), 200000,
                                     progress.data_ptr(), n_blocks, s)
        mc.packets_reset(ready.data_ptr(), len(pk), progress.data_ptr(), n_blocks, s)
        prod.wait_stream(main)
        reducer()
        for j, (b, e) in enumerate(pk):
            mc.delay(20, ps)
            for p in arriving:
                mc.packet_deliver(x_dev[p].data_ptr() + 4 * b, src[p].data_ptr() + 4 * b, e - b,
                                  ready.data_ptr() + 4 * j, ps)
        done = torch.cuda.Event()
        done.record(prod)
        main.wait_event(done)
        reducer()
        torch.cuda.synchronize()
        pr = progress.cpu().numpy()
        assert np.all(pr[:n_blocks] == len(pk)) and pr[n_blocks + 1] == 0, f"step {step_no}: not every packet done"
        print(f"step {step_no}: workgroups that gave up in the first call: {int(pr[n_blocks])}", flush=True)
        g_ref = oracle.reduce_update(O, xs_h, w_h, v_h, cfg.lr, cfg.mu, cfg.wd, order=order)
        gh.assert_bits(g.cpu().numpy(), g_ref, f"step {step_no}: g")
        gh.assert_bits(w.cpu().numpy(), w_h, f"step {step_no}: w")
        gh.assert_bits(v.cpu().numpy(), v_h, f"step {step_no}: v")
