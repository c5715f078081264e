"""Randomised parity of a rank's role-dependent step: per-colour term counts (0 = colour skipped,
up to P) and update flags drawn at random, over seeded layouts (CNN-like, arbitrary, many tiny
tensors), misaligned per-layer tensors, colour counts, sequences, hyper-parameters from the call
or from device memory and launch options, through mc_reduce_update_roles on flat buffers and
mc_fused_step_ex on per-layer tensors, against the oracle.  MC_RANDOM_CASES raises the number
of cases."""
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
OPTS = (mc.OPT_RU_SHAPE, mc.OPT_STATE_POLICY, mc.OPT_STATE_STORE_SC1, mc.OPT_XCD_RUN, mc.OPT_DIRECT_TILES,
        mc.OPT_LDS_CAP_UPDATE)


@pytest.fixture(autouse=True)
def _restore_options():
    keep = {o: mc.get_option(o) for o in OPTS}
    yield
    for o, v in keep.items():
        mc.set_option(o, v)
    torch.cuda.synchronize()


def _case(seed):
    rng = np.random.Generator(np.random.PCG64(77000 + seed))
    kind = int(rng.integers(0, 3))
    if kind == 0:      # CNN-like: multiples of four, a few big ones
        sizes = [int(4 * rng.integers(1, 20000)) for _ in range(int(rng.integers(1, 25)))]
    elif kind == 1:    # arbitrary
        sizes = [int(rng.integers(0, 40000)) for _ in range(int(rng.integers(1, 25)))]
    else:              # many small and empty tensors around a large one
        sizes = [int(rng.choice([0, 1, 3, 5, 64, 255, 256, 257, 513])) for _ in range(int(rng.integers(5, 300)))]
        sizes.append(int(rng.integers(1, 300000)))
        rng.shuffle(sizes)
    if sum(sizes) == 0:
        sizes.append(11)
    k = int(rng.choice([1, 2, 3, 4, 8, 13, 32, 40]))
    P = int(rng.choice([1, 2, 3, 4, 5, 6, 7, 8, 9, 12]))
    n_terms = rng.integers(0, P + 1, size=k).astype(np.int32)
    if rng.integers(0, 2):                       # the shape of a tree rank: one colour with more terms
        n_terms[:] = min(P, int(rng.integers(1, 5)))
        n_terms[int(rng.integers(0, k))] = P
    do_update = rng.integers(0, 2, size=k).astype(np.uint8)
    order = [None, wl.rotation_order(k, P), wl.random_order(k, P, seed=seed)][int(rng.integers(0, 3))]
    misalign = [[0], [0, 0, 1], [int(x) for x in rng.integers(0, 4, size=5)]][int(rng.integers(0, 3))]
    opts = {mc.OPT_RU_SHAPE: int(rng.choice([0, 1, 2])), mc.OPT_STATE_POLICY: int(rng.integers(1, 3)),
            mc.OPT_STATE_STORE_SC1: int(rng.integers(0, 2)), mc.OPT_XCD_RUN: int(rng.choice([0, 0, 2, 8])),
            mc.OPT_DIRECT_TILES: int(rng.integers(0, 3)), mc.OPT_LDS_CAP_UPDATE: int(rng.choice([-1, 0, 8192, 40960]))}
    hyper = [float(x) for x in (rng.choice([0.1, 0.01, 0.5]), rng.choice([0.9, 0.0, 0.5]), rng.choice([1e-4, 0.0, 5e-4]))]
    from_device = int(rng.integers(0, 2))
    return sizes, k, P, n_terms, do_update, order, misalign, opts, hyper, from_device, rng


@pytest.mark.parametrize("seed", range(N_CASES))
def test_random_roles(seed):
    sizes, k, P, n_terms, do_update, order, misalign, opts, (lr, mu, wd), from_device, rng = _case(seed)
    for o, v in opts.items():
        mc.set_option(o, v)
    L = mc.Layout(sizes, k)
    O = oracle.Layout(sizes, k)
    N = L.N
    print(f"random roles {seed}: n={len(sizes)} N={N} k={k} P={P} terms={n_terms.tolist()[:10]} upd={do_update.tolist()[:10]} "
          f"hyper_from_device={from_device} misalign={misalign} opts={list(opts.values())}", flush=True)
    xs = [rng.standard_normal(N, dtype=np.float32) * np.float32(1e-3) for _ in range(P)]
    w0 = rng.standard_normal(N, dtype=np.float32) * np.float32(0.05)
    v0 = rng.standard_normal(N, dtype=np.float32) * np.float32(0.01)
    g_ref, w_ref, v_ref = np.full(N, 7.0, np.float32), w0.copy(), v0.copy()
    oracle.reduce_update_roles(O, xs, n_terms, do_update, g_ref, w_ref, v_ref, lr, mu, wd, order=order)
    s = gh.stream_handle()
    if from_device:
        hyper = gh.dev_empty(3)
        mc.hyper_write(hyper.data_ptr(), lr, mu, wd, s)
        spec = mc.update_spec(hyper_dev_ptr=hyper.data_ptr())
    else:
        spec = mc.update_spec(lr, mu, wd)

    # flat buffers
    xd = [gh.to_dev(x) for x in xs]
    g, w, v = gh.to_dev(np.full(N, 7.0, np.float32)), gh.to_dev(w0), gh.to_dev(v0)
    mc.reduce_update_roles(L, [x.data_ptr() for x in xd], order, n_terms, do_update, g.data_ptr(), w.data_ptr(),
                           v.data_ptr(), lr, mu, wd, s)
    torch.cuda.synchronize()
    gh.assert_bits(g.cpu().numpy()[:N], g_ref, f"flat case {seed}: g")
    gh.assert_bits(w.cpu().numpy()[:N], w_ref, f"flat case {seed}: w")
    gh.assert_bits(v.cpu().numpy()[:N], v_ref, f"flat case {seed}: v")

    # per-layer tensors, misaligned
    dev_x = [gh.place_tensors(oracle.unpack(O, x), misalign)[0] for x in xs]
    dev_w, w_arena = gh.place_tensors(oracle.unpack(O, w0), misalign)
    dev_v, v_arena = gh.place_tensors(oracle.unpack(O, v0), misalign)
    w_before = w_arena.cpu().numpy().view(np.uint32).copy()
    sets = [mc.TensorSet(L, gh.ptrs(d)) for d in dev_x]
    wset, vset = mc.TensorSet(L, gh.ptrs(dev_w)), mc.TensorSet(L, gh.ptrs(dev_v))
    g2 = gh.to_dev(np.full(N, 7.0, np.float32))
    mc.fused_step_ex(L, sets, order, g2.data_ptr(), wset, vset, spec, s, n_terms=n_terms, do_update=do_update)
    torch.cuda.synchronize()
    gh.assert_bits(g2.cpu().numpy()[:N], g_ref, f"fused case {seed}: g")
    gh.assert_bits(oracle.pack(O, [t.cpu().numpy() for t in dev_w]), w_ref, f"fused case {seed}: w")
    gh.assert_bits(oracle.pack(O, [t.cpu().numpy() for t in dev_v]), v_ref, f"fused case {seed}: v")
    # nothing between the per-layer weight tensors may change
    after = w_arena.cpu().numpy().view(np.uint32)
    touched = np.zeros(after.size, bool)
    for t in dev_w:
        lo = (t.data_ptr() - w_arena.data_ptr()) // 4
        touched[lo:lo + t.numel()] = True
    assert np.array_equal(after[~touched], w_before[~touched]), f"fused case {seed}: wrote outside the weight tensors"
