"""mc_pack_noalloc (the pack for callers that cannot allocate device memory) against mc_pack:
same words bit for bit, on two calls in a row of which the second is the smaller one, so that
whatever the first call left in the library's fixed table array must not leak into the second.
Also checked against the oracle's pack, like every other pack test."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle  # noqa: E402
from paper_1711_00705_amd import mc  # noqa: E402
from paper_1711_00705_amd import workloads as wl  # noqa: E402
import gpu_harness as gh  # noqa: E402


def _coded_tensors(sizes, salt):
    """Every word distinct and recognisable: (tensor, position) coded into the bits (exponent
    kept away from all-ones so that no word is a NaN)."""
    out = []
    for t, s in enumerate(sizes):
        words = (np.arange(int(s), dtype=np.uint64) * 2654435761 + t * 40503 + salt) & 0x7F7FFFFF
        out.append(words.astype(np.uint32).view(np.float32))
    return out


def _both_packs(sizes, k, salt, misalign=None):
    L = mc.Layout(sizes, k)
    host = _coded_tensors(sizes, salt)
    dev, _arena = gh.place_tensors(host, misalign)
    s = gh.stream_handle()
    G = 64
    ref_flat = gh.dev_empty(L.N)
    mc.pack(L, gh.ptrs(dev), ref_flat.data_ptr() if L.N else None, s)
    buf = gh.dev_empty(L.N + 2 * G)
    print(f"mc_pack_noalloc n={L.n} N={L.N} k={k} misalign={misalign}", flush=True)
    mc.pack_noalloc(L, gh.ptrs(dev), buf[G:].data_ptr() if L.N else None, s)
    torch.cuda.synchronize()
    got = buf.cpu().numpy().view(np.uint32)
    assert np.all(got[:G] == 0xFFFFFFFF) and np.all(got[G + L.N:] == 0xFFFFFFFF), "wrote outside the flat buffer"
    gh.assert_bits(got[G:G + L.N].view(np.float32), ref_flat[:L.N].cpu().numpy(), "mc_pack_noalloc vs mc_pack")
    gh.assert_bits(got[G:G + L.N].view(np.float32), oracle.pack(oracle.Layout(sizes, k), host),
                   "mc_pack_noalloc vs the oracle")
    for a, b in zip(dev, host):
        gh.assert_bits(a.cpu().numpy(), b, "a source tensor changed")


def test_two_calls_in_a_row_second_smaller():
    big = wl.workload("googlenet")                        # 116 tensors, 6,998,552 elements: several thousand tiles
    _both_packs(big.sizes, big.k, salt=1)
    small = wl.workload("tiny")                           # 12 odd-sized tensors, 250,093 elements, ragged tail
    _both_packs(small.sizes, small.k, salt=2, misalign=[1, 2, 3, 0])
    _both_packs([5, 0, 3, 1, 0, 257], 3, salt=3)          # smaller again: one tile, empty tensors
    _both_packs(big.sizes, big.k, salt=4)                 # and back to the large one


def test_same_stream_calls_do_not_disturb_each_other():
    """Two different layouts queued back to back on one stream without a synchronisation in
    between: the second call's table rebuild must wait for the first call's gather."""
    a = wl.workload("googlenet")
    b = wl.workload("tiny")
    La, Lb = mc.Layout(a.sizes, a.k), mc.Layout(b.sizes, b.k)
    ha, hb = _coded_tensors(a.sizes, 7), _coded_tensors(b.sizes, 8)
    da, _ = gh.place_tensors(ha)
    db, _ = gh.place_tensors(hb)
    fa, fb, fa2 = gh.dev_empty(La.N), gh.dev_empty(Lb.N), gh.dev_empty(La.N)
    s = gh.stream_handle()
    print("mc_pack_noalloc back to back: googlenet, tiny, googlenet", flush=True)
    mc.pack_noalloc(La, gh.ptrs(da), fa.data_ptr(), s)
    mc.pack_noalloc(Lb, gh.ptrs(db), fb.data_ptr(), s)
    mc.pack_noalloc(La, gh.ptrs(da), fa2.data_ptr(), s)
    torch.cuda.synchronize()
    gh.assert_bits(fa[:La.N].cpu().numpy(), oracle.pack(oracle.Layout(a.sizes, a.k), ha), "first call")
    gh.assert_bits(fb[:Lb.N].cpu().numpy(), oracle.pack(oracle.Layout(b.sizes, b.k), hb), "second call")
    gh.assert_bits(fa2[:La.N].cpu().numpy(), oracle.pack(oracle.Layout(a.sizes, a.k), ha), "third call")


def test_full_resnet50_payload():
    cfg = wl.workload("resnet50")
    _both_packs(cfg.sizes, cfg.k, salt=5)


def test_limits_are_errors_and_touch_nothing():
    sizes = [4] * (mc.NOALLOC_MAX_TENSORS + 1)
    L = mc.Layout(sizes, 2)
    dev = [gh.dev_empty(4) for _ in sizes]
    flat = gh.dev_empty(L.N)
    with pytest.raises(mc.McError) as e:
        mc.pack_noalloc(L, gh.ptrs(dev), flat.data_ptr(), gh.stream_handle())
    assert e.value.code == mc.ERR_LIMIT
    torch.cuda.synchronize()
    assert np.all(flat.cpu().numpy().view(np.uint32) == 0xFFFFFFFF)
