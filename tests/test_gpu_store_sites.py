"""Regression guard for the 128-bit write-through store (csrc/mc_mem.h): every kernel that issues
it, in every workgroup shape it is built in (the update kernels' optional two-vector shape included),
on a payload of 16.8 M elements: large enough for the large-payload choices of the launch code, small
enough to check in a second.  A store whose data registers are rewritten too early shows up as
scattered wrong words, so every word is compared."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle  # noqa: E402
from paper_1711_00705_amd import mc  # noqa: E402
import gpu_harness as gh  # noqa: E402

SIZES = [9_000_000, 64, 7_800_000, 1000, 36]        # 16,801,100 elements, just above 2^24
OPTS = (mc.OPT_RU_SHAPE, mc.OPT_STATE_POLICY, mc.OPT_STATE_STORE_SC1, mc.OPT_PACK_NONTEMPORAL)


@pytest.fixture(autouse=True)
def _restore_options():
    keep = {o: mc.get_option(o) for o in OPTS}
    yield
    for o, v in keep.items():
        mc.set_option(o, v)
    torch.cuda.synchronize()


def _words(n, salt):
    w = (np.arange(n, dtype=np.uint64) * 2654435761 + salt) & 0x7F7FFFFF
    return w.astype(np.uint32).view(np.float32)


def test_pack_unpack_and_copy_store_sites():
    L = mc.Layout(SIZES, 4)
    O = oracle.Layout(SIZES, 4)
    assert L.N >= 1 << 24
    host = [_words(s, 17 * t) for t, s in enumerate(SIZES)]
    dev, _ = gh.place_tensors(host)
    s = gh.stream_handle()
    for pack_nt in (3, 0):                                  # write-through stores on / off
        mc.set_option(mc.OPT_PACK_NONTEMPORAL, pack_nt)
        print(f"store sites: pack/unpack pack_nt={pack_nt} N={L.N}", flush=True)
        flat = gh.gpu_pack(L, dev)                          # flat side of pack
        gh.assert_bits(flat[:L.N].cpu().numpy(), oracle.pack(O, host), "pack")
        back = [torch.zeros_like(t) for t in dev]
        mc.unpack(L, flat.data_ptr(), gh.ptrs(back), s)     # tensor side of unpack
        torch.cuda.synchronize()
        for a, b in zip(back, host):
            gh.assert_bits(a.cpu().numpy(), b, "unpack")
    dst = gh.dev_empty(L.N)
    n_bytes = (L.N // 4) * 16
    mc.copy(dst.data_ptr(), flat.data_ptr(), n_bytes, s)
    torch.cuda.synchronize()
    gh.assert_bits(dst[:n_bytes // 4].cpu().numpy(), flat[:n_bytes // 4].cpu().numpy(), "mc_copy")
    small = mc.Layout([300_000, 12, 70_000], 2)             # a small payload (the launch code's other branch)
    hs = [_words(s_, 5 + t) for t, s_ in enumerate([300_000, 12, 70_000])]
    ds, _ = gh.place_tensors(hs)
    mc.set_option(mc.OPT_PACK_NONTEMPORAL, 3)
    fl = gh.gpu_pack(small, ds)
    torch.cuda.synchronize()
    gh.assert_bits(fl[:small.N].cpu().numpy(), oracle.pack(oracle.Layout([300_000, 12, 70_000], 2), hs), "pack, one vector")


@pytest.mark.parametrize("shape", [1, 2])
@pytest.mark.parametrize("policy", [mc.STATE_RESIDENT, mc.STATE_STREAMING])
def test_state_store_sites(shape, policy):
    """Updated weights and momentum, both forms of the step, both tile shapes, both policies."""
    mc.set_option(mc.OPT_RU_SHAPE, shape)
    mc.set_option(mc.OPT_STATE_POLICY, policy)
    mc.set_option(mc.OPT_STATE_STORE_SC1, 1)
    k, P = 4, 2
    rng = np.random.Generator(np.random.PCG64(99))
    xs = [[rng.standard_normal(s, dtype=np.float32) * np.float32(1e-3) for s in SIZES] for _ in range(P)]
    w = [rng.standard_normal(s, dtype=np.float32) * np.float32(0.05) for s in SIZES]
    v = [rng.standard_normal(s, dtype=np.float32) * np.float32(0.01) for s in SIZES]
    print(f"store sites: update shape={shape} policy={policy}", flush=True)
    st = gh.Step(SIZES, k)
    gpu, ref = st.run(xs, w, v, 0.1, 0.9, 1e-4)
    st.check(gpu, ref, 0.1, 0.9, 1e-4, "staged")
    fs = gh.FusedStep(SIZES, k)
    gpu, ref = fs.run(xs, w, v, 0.1, 0.9, 1e-4)
    fs.check(gpu, ref, "fused")
