"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by
element, on the same seeded host bytes.  Bar: bit-exact for packed words and the reduced
gradient; weights and momentum within 1e-6 relative to their operands (and, because the
kernel does not contract multiply-adds, bit-exact as well)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle  # noqa: E402
from paper_1711_00705_amd import mc  # noqa: E402
from paper_1711_00705_amd import workloads as wl  # noqa: E402
import gpu_harness as gh  # noqa: E402


@pytest.fixture(autouse=True)
def _restore_options():
    keep = {o: mc.get_option(o) for o in (mc.OPT_RU_SHAPE, mc.OPT_STATE_POLICY, mc.OPT_PACK_NONTEMPORAL, mc.OPT_STATE_STORE_SC1)}
    yield
    for o, v in keep.items():
        mc.set_option(o, v)
    torch.cuda.synchronize()


def _inputs(sizes, P, step=0, heavy=False, v_zero=True, seed_v=5):
    xs = [wl.contribution_tensors(sizes, p, step=step, heavy_tail=heavy) for p in range(P)]
    w = wl.weight_tensors(sizes)
    if v_zero:
        v = wl.zero_tensors(sizes)
    else:
        rng = np.random.Generator(np.random.PCG64(seed_v))
        v = [rng.standard_normal(int(s), dtype=np.float32) * np.float32(0.01) for s in sizes]
    return xs, w, v


# ---------------------------------------------------------------------------------------
# the Tiny configuration: arbitrary sizes -> misaligned offsets, scalar tails
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("order_kind", ["identity", "rotation", "random"])
@pytest.mark.parametrize("misalign", [None, [1, 2, 3, 0]])
def test_tiny_config(order_kind, misalign):
    cfg = wl.workload("tiny")
    order = {"identity": None, "rotation": wl.rotation_order(cfg.k, cfg.P),
             "random": wl.random_order(cfg.k, cfg.P, seed=4)}[order_kind]
    st = gh.Step(cfg.sizes, cfg.k)
    xs, w, v = _inputs(cfg.sizes, cfg.P)
    print(f"tiny N={cfg.total} order={order_kind} misalign={misalign}", flush=True)
    gpu, ref = st.run(xs, w, v, cfg.lr, cfg.mu, cfg.wd, order=order, misalign=misalign)
    st.check(gpu, ref, cfg.lr, cfg.mu, cfg.wd, "tiny")


@pytest.mark.parametrize("unroll", [1, 2])
@pytest.mark.parametrize("nt", [0, 1])
@pytest.mark.parametrize("pack_nt", [0, 1, 2, 3])
def test_launch_shapes_do_not_change_bits(unroll, nt, pack_nt):
    mc.set_option(mc.OPT_STATE_STORE_SC1, (unroll + nt + pack_nt) % 2)
    mc.set_option(mc.OPT_RU_SHAPE, unroll)
    mc.set_option(mc.OPT_PACK_NONTEMPORAL, pack_nt)
    mc.set_option(mc.OPT_STATE_POLICY, 1 + nt)
    sizes = [30000, 1, 4097, 12345, 70001]      # several tiles of every shape + ragged tail
    st = gh.Step(sizes, 3)
    xs, w, v = _inputs(sizes, 5, v_zero=False)
    print(f"shapes unroll={unroll} nt={nt} pack_nt={pack_nt}", flush=True)
    gpu, ref = st.run(xs, w, v, 0.1, 0.9, 1e-4, order=wl.rotation_order(3, 5), misalign=[0, 1, 0, 3])
    st.check(gpu, ref, 0.1, 0.9, 1e-4, f"unroll={unroll} nt={nt} pack_nt={pack_nt}")


@pytest.mark.parametrize("P", [1, 2, 3, 4, 5, 6, 7, 8, 9, 16, 32])
def test_every_contribution_count(P):
    sizes = [5000, 3, 2049, 8191]
    k = 4
    st = gh.Step(sizes, k)
    xs, w, v = _inputs(sizes, P, v_zero=False)
    print(f"P={P}", flush=True)
    for order in (None, wl.random_order(k, P, seed=P)):
        gpu, ref = st.run(xs, w, v, 0.05, 0.8, 1e-3, order=order, unpack_outputs=False)
        st.check(gpu, ref, 0.05, 0.8, 1e-3, f"P={P}")


def test_the_same_contribution_twice():
    """Contributions are only read, so one buffer may be given more than once (x + x + y)."""
    sizes = [5000, 3, 2049, 8191]
    k = 2
    L = mc.Layout(sizes, k)
    O = oracle.Layout(sizes, k)
    xs, w, v = _inputs(sizes, 2, v_zero=False)
    xf = [oracle.pack(O, t) for t in xs]
    wf, vf = oracle.pack(O, w), oracle.pack(O, v)
    xd = [gh.to_dev(x) for x in xf]
    wd_, vd, gd = gh.to_dev(wf), gh.to_dev(vf), gh.dev_empty(L.N)
    mc.reduce_update(L, [xd[0].data_ptr(), xd[0].data_ptr(), xd[1].data_ptr()], None, gd.data_ptr(),
                     wd_.data_ptr(), vd.data_ptr(), 0.1, 0.9, 1e-4, gh.stream_handle())
    torch.cuda.synchronize()
    g = oracle.reduce_update(O, [xf[0], xf[0], xf[1]], wf, vf, 0.1, 0.9, 1e-4)
    gh.assert_bits(gd[:L.N].cpu().numpy(), g, "g")
    gh.assert_bits(wd_.cpu().numpy(), wf, "w")
    gh.assert_bits(vd.cpu().numpy(), vf, "v")


@pytest.mark.parametrize("sizes,k", [
    ([1], 1), ([1], 5), ([3], 2), ([4], 1), ([255], 1), ([256], 2), ([257], 2), ([1023, 1], 3),
    ([0, 5, 0, 0, 7], 2), ([1024], 1024), ([2000], 2003), ([777, 0, 1], 9), ([8192], 1),
    ([8191], 1), ([8193], 1), ([100] * 50, 7),
])
def test_edge_sizes(sizes, k):
    st = gh.Step(sizes, k)
    P = 3
    xs, w, v = _inputs(sizes, P, v_zero=False)
    print(f"edge sizes={sizes[:6]} k={k}", flush=True)
    gpu, ref = st.run(xs, w, v, 0.1, 0.9, 1e-4, order=wl.rotation_order(k, P), misalign=[3, 1])
    st.check(gpu, ref, 0.1, 0.9, 1e-4, f"sizes={sizes[:6]} k={k}")


def test_many_colours_span_several_launches():
    sizes = [40000, 20001]
    k, P = 100, 8                     # 32 colours per launch at most
    st = gh.Step(sizes, k)
    xs, w, v = _inputs(sizes, P, heavy=True, v_zero=False)
    gpu, ref = st.run(xs, w, v, 0.1, 0.9, 1e-4, order=wl.random_order(k, P, seed=9))
    st.check(gpu, ref, 0.1, 0.9, 1e-4, "k=100")
    k, P = 40, 32                     # 8 colours per launch at P = 32
    st = gh.Step(sizes, k)
    xs, w, v = _inputs(sizes, P, v_zero=False)
    gpu, ref = st.run(xs, w, v, 0.1, 0.9, 1e-4, order=wl.rotation_order(k, P), unpack_outputs=False)
    st.check(gpu, ref, 0.1, 0.9, 1e-4, "k=40 P=32")


def test_many_tensors_span_several_pack_launches():
    rng = np.random.Generator(np.random.PCG64(12))
    sizes = [int(s) for s in rng.choice([0, 1, 2, 3, 4, 5, 16, 63, 64, 100, 1000, 5000], size=700)]
    st = gh.Step(sizes, 5)
    xs, w, v = _inputs(sizes, 2, v_zero=False)
    for mis in (None, [0, 1, 2, 3, 2]):
        gpu, ref = st.run(xs, w, v, 0.1, 0.9, 1e-4, misalign=mis)
        st.check(gpu, ref, 0.1, 0.9, 1e-4, "700 tensors")


def test_pack_unpack_identity_coded_and_guards():
    """Word j of tensor t holds off_t + j; flat must read 0,1,2,...  Guard words around every
    destination must stay untouched."""
    cfg = wl.workload("tiny")
    sizes = list(cfg.sizes)
    L = mc.Layout(sizes, 3)
    N = L.N
    ts, run = [], 0
    for s in sizes:
        ts.append((np.arange(run, run + s, dtype=np.uint32) & np.uint32(0x3FFFFFFF)).view(np.float32))
        run += s
    for mis in (None, [1, 3, 2, 0, 1]):
        dts, arena = gh.place_tensors(ts, mis)
        G = 64
        buf = gh.dev_empty(N + 2 * G)
        flat = buf[G:G + N]
        assert flat.data_ptr() % 16 == 0
        mc.pack(L, gh.ptrs(dts), flat.data_ptr(), gh.stream_handle())
        torch.cuda.synchronize()
        host = buf.cpu().numpy().view(np.uint32)
        assert np.all(host[:G] == 0xFFFFFFFF) and np.all(host[G + N:] == 0xFFFFFFFF), "pack wrote outside flat"
        assert np.array_equal(host[G:G + N], np.arange(N, dtype=np.uint32))
        # unpack into a fresh guarded arena
        outs, arena2 = gh.place_tensors([np.zeros(s, np.float32) for s in sizes], mis or [0])
        before = arena2.cpu().numpy().view(np.uint32).copy()
        mc.unpack(L, flat.data_ptr(), gh.ptrs(outs), gh.stream_handle())
        torch.cuda.synchronize()
        after = arena2.cpu().numpy().view(np.uint32)
        touched = np.zeros(after.size, bool)
        base = arena2.data_ptr()
        for o, t in zip(outs, ts):
            lo = (o.data_ptr() - base) // 4
            touched[lo:lo + t.size] = True
            gh.assert_bits(o.cpu().numpy(), t, "unpack")
        assert np.array_equal(after[~touched], before[~touched]), "unpack wrote outside its tensors"


@pytest.mark.parametrize("mis", [[0], [1], [2], [3], [3, 1, 2]])
def test_shifted_tensors_many_whole_tiles(mis):
    """Tensors of many tiles whose addresses sit 1, 2 or 3 elements off the 16-byte grid relative
    to their flat offsets (every combination: the odd sizes shift the offsets too): the tiles
    move as realigned vectors, the first and last tile of each tensor element by element.  Word
    j of tensor t holds off_t + j; nothing outside the tensors may change."""
    sizes = [1, 3000, 2, 2050, 5, 777, 4099, 1280, 256, 260, 263, 515]
    L = mc.Layout(sizes, 4)
    N = L.N
    ts, run = [], 0
    for s in sizes:
        ts.append(np.arange(run, run + s, dtype=np.uint32).view(np.float32))
        run += s
    print(f"shifted tensors mis={mis} N={N}", flush=True)
    dts, _arena = gh.place_tensors(ts, mis)
    G = 64
    buf = gh.dev_empty(N + 2 * G)
    flat = buf[G:G + N]
    mc.pack(L, gh.ptrs(dts), flat.data_ptr(), gh.stream_handle())
    torch.cuda.synchronize()
    host = buf.cpu().numpy().view(np.uint32)
    assert np.all(host[:G] == 0xFFFFFFFF) and np.all(host[G + N:] == 0xFFFFFFFF), "pack wrote outside flat"
    assert np.array_equal(host[G:G + N], np.arange(N, dtype=np.uint32))
    outs, arena2 = gh.place_tensors([np.zeros(s, np.float32) for s in sizes], mis)
    before = arena2.cpu().numpy().view(np.uint32).copy()
    mc.unpack(L, flat.data_ptr(), gh.ptrs(outs), gh.stream_handle())
    torch.cuda.synchronize()
    after = arena2.cpu().numpy().view(np.uint32)
    touched = np.zeros(after.size, bool)
    for o, t in zip(outs, ts):
        lo = (o.data_ptr() - arena2.data_ptr()) // 4
        touched[lo:lo + t.size] = True
        gh.assert_bits(o.cpu().numpy(), t, "unpack")
    assert np.array_equal(after[~touched], before[~touched]), "unpack wrote outside its tensors"


def test_arbitrary_bit_patterns_survive_pack_unpack():
    sizes = [1000, 37, 5000, 2]
    L = mc.Layout(sizes, 2)
    rng = np.random.Generator(np.random.PCG64(3))
    ts = [rng.integers(0, 2 ** 32, size=s, dtype=np.uint64).astype(np.uint32).view(np.float32) for s in sizes]
    dts, _ = gh.place_tensors(ts, [2, 0, 1])
    flat = gh.gpu_pack(L, dts)
    outs, _ = gh.place_tensors([np.zeros(s, np.float32) for s in sizes], [1])
    mc.unpack(L, flat.data_ptr(), gh.ptrs(outs), gh.stream_handle())
    torch.cuda.synchronize()
    O = oracle.Layout(sizes, 2)
    gh.assert_bits(flat[:L.N].cpu().numpy(), oracle.pack(O, ts), "pack raw bits")
    for o, t in zip(outs, ts):
        gh.assert_bits(o.cpu().numpy(), t, "unpack raw bits")


def test_reduce_update_does_not_write_outside():
    sizes = [5003]
    L = mc.Layout(sizes, 2)
    N, G = L.N, 64
    rng = np.random.Generator(np.random.PCG64(1))
    bufs = []
    for _ in range(3):  # g, w, v with guards
        b = gh.dev_empty(N + 2 * G)
        bufs.append(b)
    xs = [gh.to_dev(rng.standard_normal(N, dtype=np.float32)) for _ in range(3)]
    w0 = rng.standard_normal(N, dtype=np.float32)
    bufs[1][G:G + N].copy_(torch.from_numpy(w0))
    bufs[2][G:G + N].zero_()
    mc.reduce_update(L, [x.data_ptr() for x in xs], None, bufs[0][G:].data_ptr(), bufs[1][G:].data_ptr(),
                     bufs[2][G:].data_ptr(), 0.1, 0.9, 0.0, gh.stream_handle())
    torch.cuda.synchronize()
    for b in bufs:
        h = b.cpu().numpy().view(np.uint32)
        assert np.all(h[:G] == 0xFFFFFFFF) and np.all(h[G + N:] == 0xFFFFFFFF)
        assert not np.any(h[G:G + N] == 0xFFFFFFFF)


def test_grad_out_null_gives_same_update():
    sizes = [9000, 513]
    st = gh.Step(sizes, 3)
    xs, w, v = _inputs(sizes, 4, v_zero=False)
    gpu, ref = st.run(xs, w, v, 0.1, 0.9, 1e-4, want_g=False)
    assert gpu["g"] is None
    st.check(gpu, ref, 0.1, 0.9, 1e-4, "grad_out = NULL")


def test_order_closed_form_on_gpu():
    # 2^24 + 1 - 2^24 in three different sequences: 0, 1, 1 (left-to-right, ties-to-even)
    big = float(2 ** 24)
    N = 768
    L = mc.Layout([700, 68], 3)
    assert list(L.colour_bounds()) == [0, 256, 512, 768]
    xs = [gh.to_dev(np.full(N, val, np.float32)) for val in (big, 1.0, -big)]
    order = np.array([[0, 1, 2], [0, 2, 1], [1, 2, 0]], np.int32)
    g = gh.dev_empty(N)
    w = gh.dev_empty(N, fill=0)
    v = gh.dev_empty(N, fill=0)
    mc.reduce_update(L, [x.data_ptr() for x in xs], order, g.data_ptr(), w.data_ptr(), v.data_ptr(),
                     0.0, 0.0, 0.0, gh.stream_handle())
    torch.cuda.synchronize()
    expect = np.concatenate([np.zeros(256), np.ones(256), np.ones(256)]).astype(np.float32)
    gh.assert_bits(g.cpu().numpy(), expect, "closed form per colour")


def test_ieee_corner_cases_on_gpu():
    N = 1000
    sizes = [N]
    st = gh.Step(sizes, 2)
    nz = np.full(N, -0.0, np.float32)
    tiny = np.full(N, 2.0 ** -149, np.float32)
    zeros = [np.zeros(N, np.float32)]
    # signed zero: (-0) + (-0) = -0
    gpu, ref = st.run([[nz], [nz.copy()]], zeros, zeros, 0.0, 0.0, 0.0)
    assert np.all(gpu["g"].view(np.uint32) == 0x80000000)
    st.check(gpu, ref, 0.0, 0.0, 0.0, "signed zero")
    # denormals are kept in sums ...
    gpu, ref = st.run([[tiny], [tiny.copy()], [tiny.copy()]], zeros, zeros, 0.0, 0.0, 0.0)
    assert np.all(gpu["g"].view(np.uint32) == 3)
    st.check(gpu, ref, 0.0, 0.0, 0.0, "denormal sum")
    # ... and in the update's products: 0.5 * 2^-140 = 2^-141
    w = [np.full(N, 2.0 ** -140, np.float32)]
    gpu, ref = st.run([zeros[0:1]], w, zeros, 0.25, 0.5, 0.5)
    assert np.all(gpu["v"] == np.float32(2.0 ** -141))
    st.check(gpu, ref, 0.25, 0.5, 0.5, "denormal product")
    # a mix of denormal-range values through the whole update
    rng = np.random.Generator(np.random.PCG64(6))
    xs = [[(rng.standard_normal(N, dtype=np.float32) * np.float32(1e-40))] for _ in range(4)]
    w = [rng.standard_normal(N, dtype=np.float32) * np.float32(1e-38)]
    v = [rng.standard_normal(N, dtype=np.float32) * np.float32(1e-39)]
    gpu, ref = st.run(xs, w, v, 0.1, 0.9, 1e-4)
    st.check(gpu, ref, 0.1, 0.9, 1e-4, "denormal range")
    # NaN / Inf propagate (payload bits are not pinned: compare as "both NaN")
    x = np.zeros(N, np.float32)
    y = np.zeros(N, np.float32)
    x[3], x[5], y[3], y[7] = np.inf, np.nan, -np.inf, np.inf
    gpu, ref = st.run([[x], [y]], [np.ones(N, np.float32)], zeros, 0.1, 0.9, 0.0)
    st.check(gpu, ref, 0.1, 0.9, 0.0, "nan/inf", nan_ok=True)
    assert np.isnan(gpu["g"][3]) and np.isnan(gpu["g"][5]) and np.isposinf(gpu["g"][7])


def test_exact_integer_sums_any_order():
    sizes = [300, 1, 0, 4097, 1023, 77]
    N = sum(sizes)
    P, k = 32, 8
    ts = [wl.integer_tensors(sizes, seed=900 + p) for p in range(P)]
    exact = np.zeros(N, np.int64)
    for p in range(P):
        exact += np.concatenate(ts[p]).astype(np.int64)
    st = gh.Step(sizes, k)
    z = wl.zero_tensors(sizes)
    for order in (None, wl.rotation_order(k, P), wl.random_order(k, P, seed=2)):
        gpu, ref = st.run(ts, z, z, 0.0, 0.0, 0.0, order=order, unpack_outputs=False)
        assert np.array_equal(gpu["g"].astype(np.int64), exact)
        st.check(gpu, ref, 0.0, 0.0, 0.0, "integers")


def test_replay_is_deterministic_and_state_carries():
    """Three successive steps carrying (w, v) on the GPU, against the oracle carrying state;
    the whole sequence run twice gives identical bits."""
    sizes = [20000, 777, 4096]
    k, P = 4, 4
    L = mc.Layout(sizes, k)
    O = oracle.Layout(sizes, k)
    N = L.N
    results = []
    for rep in range(2):
        w = gh.to_dev(oracle.pack(O, wl.weight_tensors(sizes)))
        v = gh.dev_empty(N, fill=0)
        g = gh.dev_empty(N)
        wr = oracle.pack(O, wl.weight_tensors(sizes))
        vr = np.zeros(N, np.float32)
        for step in range(3):
            xs_h = [oracle.pack(O, wl.contribution_tensors(sizes, p, step=step)) for p in range(P)]
            xs = [gh.to_dev(x) for x in xs_h]
            mc.reduce_update(L, [x.data_ptr() for x in xs], wl.rotation_order(k, P), g.data_ptr(),
                             w.data_ptr(), v.data_ptr(), 0.1, 0.9, 1e-4, gh.stream_handle())
            torch.cuda.synchronize()
            gr = oracle.reduce_update(O, xs_h, wr, vr, 0.1, 0.9, 1e-4, order=wl.rotation_order(k, P))
            gh.assert_bits(g.cpu().numpy(), gr, f"g step {step}")
            gh.assert_bits(w.cpu().numpy(), wr, f"w step {step}")
            gh.assert_bits(v.cpu().numpy(), vr, f"v step {step}")
        results.append((w.cpu().numpy(), v.cpu().numpy()))
    gh.assert_bits(results[0][0], results[1][0], "replay w")
    gh.assert_bits(results[0][1], results[1][1], "replay v")


def test_non_default_stream():
    sizes = [50000, 30]
    st = gh.Step(sizes, 2)
    xs, w, v = _inputs(sizes, 3)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        gpu, ref = st.run(xs, w, v, 0.1, 0.9, 1e-4)
    st.check(gpu, ref, 0.1, 0.9, 1e-4, "side stream")


def test_copy_yardstick_copies():
    n = 1_000_003 * 4
    src = torch.arange(n, dtype=torch.int32, device="cuda").view(torch.float32)
    buf = gh.dev_empty(n + 128)
    dst = buf[64:64 + n]
    mc.copy(dst.data_ptr(), src.data_ptr(), 4 * n, gh.stream_handle())
    torch.cuda.synchronize()
    h = buf.cpu().numpy().view(np.uint32)
    assert np.all(h[:64] == 0xFFFFFFFF) and np.all(h[64 + n:] == 0xFFFFFFFF)
    assert np.array_equal(h[64:64 + n], np.arange(n, dtype=np.uint32))


def test_pack_and_unpack_through_tensor_sets_with_thousands_of_tensors():
    """The set forms take the pointers from a device table: one launch for 5000 tensors (the
    pointer-array forms need twenty), same words either way."""
    rng = np.random.Generator(np.random.PCG64(31))
    sizes = [int(s) for s in rng.choice([0, 1, 3, 4, 16, 17, 64, 100, 255, 1024], size=5000)]
    L = mc.Layout(sizes, 7)
    O = oracle.Layout(sizes, 7)
    N = L.N
    host = [rng.integers(0, 2 ** 32, size=s, dtype=np.uint64).astype(np.uint32).view(np.float32) for s in sizes]
    for mis in ([0], [1, 0, 3, 2, 0, 0, 1]):
        dts, _ = gh.place_tensors(host, mis)
        tset = mc.TensorSet(L, gh.ptrs(dts))
        G = 64
        buf = gh.dev_empty(N + 2 * G)
        flat = buf[G:G + N]
        mc.pack_set(L, tset, flat.data_ptr(), gh.stream_handle())
        flat2 = gh.dev_empty(N)
        mc.pack(L, gh.ptrs(dts), flat2.data_ptr(), gh.stream_handle())
        torch.cuda.synchronize()
        h = buf.cpu().numpy().view(np.uint32)
        assert np.all(h[:G] == 0xFFFFFFFF) and np.all(h[G + N:] == 0xFFFFFFFF)
        want = oracle.pack(O, host)
        gh.assert_bits(h[G:G + N].view(np.float32), want, "pack_set")
        gh.assert_bits(flat2[:N].cpu().numpy(), want, "pack (20 launches)")
        outs, arena = gh.place_tensors([np.zeros(s, np.float32) for s in sizes], mis)
        oset = mc.TensorSet(L, gh.ptrs(outs))
        before = arena.cpu().numpy().view(np.uint32).copy()
        mc.unpack_set(L, flat.data_ptr(), oset, gh.stream_handle())
        torch.cuda.synchronize()
        after = arena.cpu().numpy().view(np.uint32)
        touched = np.zeros(after.size, bool)
        for o, t in zip(outs, host):
            lo = (o.data_ptr() - arena.data_ptr()) // 4
            touched[lo:lo + t.size] = True
            gh.assert_bits(o.cpu().numpy(), t, "unpack_set")
        assert np.array_equal(after[~touched], before[~touched]), "unpack_set wrote outside its tensors"
        # a set must not overlap the flat buffer it is packed into
        alias = mc.TensorSet(L, [flat.data_ptr() + 4 * int(o) for o in L.tensor_offsets()[:-1]])
        with pytest.raises(mc.McError) as e:
            mc.pack_set(L, alias, flat.data_ptr(), gh.stream_handle())
        assert e.value.code == mc.ERR_OVERLAP
        for s_ in (tset, oset, alias):
            s_.destroy()


@pytest.mark.parametrize("alternate", [0, 1])
def test_sweep_direction_does_not_change_bits(alternate):
    """Successive whole-payload calls with resident state larger than the memory-side cache walk the
    payload in opposite directions (a cache-reuse measure); the same step repeated from the same
    state must give the same bits whichever direction it happens to get, in both forms of the step."""
    keep = {o: mc.get_option(o) for o in (mc.OPT_ALTERNATE_SWEEP, mc.OPT_STATE_POLICY)}
    mc.set_option(mc.OPT_ALTERNATE_SWEEP, alternate)
    mc.set_option(mc.OPT_STATE_POLICY, mc.STATE_RESIDENT)
    try:
        # above 32 Mi elements (256 MB of weights + momentum) the calls alternate when enabled
        sizes = [30000, 12, 4099, 70001] if alternate == 0 else [20_000_000, 12, 4099, 14_000_001]
        st = gh.Step(sizes, 3)
        fs = gh.FusedStep(sizes, 3)
        xs, w, v = _inputs(sizes, 2, v_zero=False)
        order = wl.rotation_order(3, 2)
        for rep in range(3 if alternate == 0 else 2):      # the layouts persist across repetitions
            gpu, ref = st.run(xs, w, v, 0.1, 0.9, 1e-4, order=order)
            st.check(gpu, ref, 0.1, 0.9, 1e-4, f"staged rep {rep}")
            gpu, ref = fs.run(xs, w, v, 0.1, 0.9, 1e-4, order=order, misalign=[0])
            fs.check(gpu, ref, f"fused rep {rep}")
    finally:
        for o, val in keep.items():
            mc.set_option(o, val)


@pytest.mark.parametrize("policy", [mc.STATE_DEFAULT, mc.STATE_RESIDENT, mc.STATE_STREAMING])
@pytest.mark.parametrize("sweep", [mc.SWEEP_AUTO, mc.SWEEP_FORWARD, mc.SWEEP_BACKWARD])
@pytest.mark.parametrize("shape", [1, 2])
def test_state_policy_and_sweep_do_not_change_bits(policy, sweep, shape):
    """The spec's state_policy and sweep fields choose cache treatment and walking direction only:
    every combination must give the oracle's bits, several tiles per colour plus ragged ends."""
    keep = mc.get_option(mc.OPT_RU_SHAPE)
    mc.set_option(mc.OPT_RU_SHAPE, shape)
    try:
        sizes = [30000, 12, 4099, 70001, 5]
        k, P = 3, 3
        L = mc.Layout(sizes, k)
        O = oracle.Layout(sizes, k)
        xs, w, v = _inputs(sizes, P, v_zero=False)
        order = wl.rotation_order(k, P)
        xf = [oracle.pack(O, t) for t in xs]
        wf, vf = oracle.pack(O, w), oracle.pack(O, v)
        xd = [gh.to_dev(x) for x in xf]
        wd_, vd = gh.to_dev(wf), gh.to_dev(vf)
        gd = gh.dev_empty(L.N)
        print(f"spec policy={policy} sweep={sweep} shape={shape}", flush=True)
        mc.reduce_update_ex(L, [x.data_ptr() for x in xd], order, gd.data_ptr(), wd_.data_ptr(), vd.data_ptr(),
                            mc.update_spec(0.1, 0.9, 1e-4, state_policy=policy, sweep=sweep), gh.stream_handle())
        torch.cuda.synchronize()
        g = oracle.reduce_update(O, xf, wf, vf, 0.1, 0.9, 1e-4, order=order)
        gh.assert_bits(gd[:L.N].cpu().numpy(), g, "g")
        gh.assert_bits(wd_.cpu().numpy(), wf, "w")
        gh.assert_bits(vd.cpu().numpy(), vf, "v")
        # the fused form with the same spec
        fs = gh.FusedStep(sizes, k)
        gpu, ref = fs.run(xs, w, v, 0.1, 0.9, 1e-4, order=order, misalign=[0],
                          spec=mc.update_spec(0.1, 0.9, 1e-4, state_policy=policy, sweep=sweep))
        fs.check(gpu, ref, "fused with spec")
    finally:
        mc.set_option(mc.OPT_RU_SHAPE, keep)


@pytest.mark.parametrize("run", [2, 5, 16, 64])
def test_tile_order_does_not_change_bits(run):
    """With MC_OPT_XCD_RUN every kernel permutes its tiles so that each die walks `run`
    neighbouring tiles; tiles are independent, so pack, sum, update and unpack must give the
    plain order's bits.  Sizes: several permuted spans plus a ragged rest, several colours."""
    keep = mc.get_option(mc.OPT_XCD_RUN)
    mc.set_option(mc.OPT_XCD_RUN, run)
    try:
        sizes = [300_000, 12, 4099, 700_001, 0, 1_000_000, 37]
        xs, w, v = _inputs(sizes, 3, v_zero=False)
        order = wl.rotation_order(5, 3)
        st = gh.Step(sizes, 5)
        gpu, ref = st.run(xs, w, v, 0.1, 0.9, 1e-4, order=order)
        st.check(gpu, ref, 0.1, 0.9, 1e-4, f"staged xcd_run {run}")
        fs = gh.FusedStep(sizes, 5)
        gpu, ref = fs.run(xs, w, v, 0.1, 0.9, 1e-4, order=order, misalign=[0])
        fs.check(gpu, ref, f"fused xcd_run {run}")
    finally:
        mc.set_option(mc.OPT_XCD_RUN, keep)
