"""Plumbing for the GPU parity tests: torch supplies device memory and the stream, the
library under test does all the work, the oracle supplies the expected bits."""
import numpy as np
import torch

import oracle
from paper_1711_00705_amd import mc


def stream_handle() -> int:
    return int(torch.cuda.current_stream().cuda_stream)


def to_dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def dev_empty(n: int, fill=None) -> torch.Tensor:
    # at least one element so that data_ptr() is a real address; 0xFF.. canary by default
    t = torch.empty(max(int(n), 1), dtype=torch.float32, device="cuda")
    t.view(torch.int32).fill_(-1 if fill is None else fill)
    return t


def place_tensors(host_tensors, misalign=None):
    """Upload per-layer tensors.  With `misalign` (a list of element shifts 0..3) they are
    carved out of one arena so that tensor t starts 4*misalign[t % len] bytes past a
    16-byte boundary.  Returns (list of device views, arena or None)."""
    if misalign is None:
        return [to_dev(t) if t.size else torch.empty(0, dtype=torch.float32, device="cuda")
                for t in host_tensors], None
    total = sum(((t.size + 3) // 4 + 2) * 4 for t in host_tensors) + 8
    arena = dev_empty(total)
    views, cur = [], 0
    for i, t in enumerate(host_tensors):
        cur = (cur + 3) // 4 * 4 + misalign[i % len(misalign)]
        v = arena[cur:cur + t.size]
        if t.size:
            v.copy_(torch.from_numpy(t))
        views.append(v)
        cur += t.size
    return views, arena


def ptrs(tensors):
    return [t.data_ptr() if t.numel() else None for t in tensors]


def gpu_pack(L: mc.Layout, dev_tensors) -> torch.Tensor:
    flat = dev_empty(L.N)
    mc.pack(L, ptrs(dev_tensors), flat.data_ptr() if L.N else None, stream_handle())
    return flat


def bits_equal(a: np.ndarray, b: np.ndarray):
    a = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    b = np.ascontiguousarray(b, dtype=np.float32).view(np.uint32)
    return a.shape == b.shape and bool(np.array_equal(a, b))


def assert_bits(a, b, what):
    a = np.ascontiguousarray(a, dtype=np.float32)
    b = np.ascontiguousarray(b, dtype=np.float32)
    assert a.shape == b.shape, what
    ua, ub = a.view(np.uint32), b.view(np.uint32)
    bad = np.nonzero(ua != ub)[0]
    if bad.size:
        i = int(bad[0])
        raise AssertionError(f"{what}: {bad.size} of {a.size} words differ; first at {i}: "
                             f"got {a[i]!r} (0x{ua[i]:08x}) expected {b[i]!r} (0x{ub[i]:08x})")


def assert_bits_or_both_nan(a, b, what):
    a = np.ascontiguousarray(a, dtype=np.float32)
    b = np.ascontiguousarray(b, dtype=np.float32)
    both_nan = np.isnan(a) & np.isnan(b)
    a2, b2 = a.copy(), b.copy()
    a2[both_nan] = 0
    b2[both_nan] = 0
    assert_bits(a2, b2, what)


def assert_update_band(w_gpu, v_gpu, w_ref, v_ref, w_old, v_old, g_ref, lr, mu, wd, what):
    """The 1e-6 bar, relative to the operands of the last subtraction / addition (w - lr*v'
    may cancel, so a per-element |delta|/|ref| is not meaningful)."""
    lr, mu, wd = np.float32(lr), np.float32(mu), np.float32(wd)
    band_v = 1e-6 * (np.abs(mu * v_old) + np.abs(g_ref) + np.abs(wd * w_old)).astype(np.float64)
    band_w = 1e-6 * (np.abs(w_old) + np.abs(lr * v_ref)).astype(np.float64)
    dv = np.abs(v_gpu.astype(np.float64) - v_ref.astype(np.float64))
    dw = np.abs(w_gpu.astype(np.float64) - w_ref.astype(np.float64))
    assert np.all(dv <= band_v), f"{what}: momentum outside the 1e-6 band at {int(np.argmax(dv - band_v))}"
    assert np.all(dw <= band_w), f"{what}: weights outside the 1e-6 band at {int(np.argmax(dw - band_w))}"


class Step:
    """One full step on the GPU from host per-layer tensors, with the oracle's answer."""

    def __init__(self, sizes, k):
        self.sizes = [int(s) for s in sizes]
        self.L = mc.Layout(self.sizes, k)
        self.O = oracle.Layout(self.sizes, k)

    def run(self, contrib_tensors, w_tensors, v_tensors, lr, mu, wd, order=None, want_g=True,
            misalign=None, unpack_outputs=True):
        """Returns dict(gpu=..., ref=...) of numpy arrays g, w, v (flat) and, optionally, the
        unpacked weights per layer."""
        L, O = self.L, self.O
        P = len(contrib_tensors)
        s = stream_handle()
        # ---- GPU: pack x P, pack w and v, reduce+update, unpack w'
        keep = []
        x_flat = []
        for ts in contrib_tensors:
            dts, arena = place_tensors(ts, misalign)
            keep.append((dts, arena))
            x_flat.append(gpu_pack(L, dts))
        w_dev, _a = place_tensors(w_tensors, misalign)
        v_dev, _b = place_tensors(v_tensors, misalign)
        w_flat = gpu_pack(L, w_dev)
        v_flat = gpu_pack(L, v_dev)
        g_flat = dev_empty(L.N) if want_g else None
        mc.reduce_update(L, [x.data_ptr() for x in x_flat], order,
                         g_flat.data_ptr() if want_g else None,
                         w_flat.data_ptr(), v_flat.data_ptr(), lr, mu, wd, s)
        out_layers = None
        if unpack_outputs:
            mc.unpack(L, w_flat.data_ptr(), ptrs(w_dev), s)
            out_layers = [t.cpu().numpy() for t in w_dev]
        torch.cuda.synchronize()
        N = L.N
        gpu = dict(x=[x[:N].cpu().numpy() for x in x_flat],
                   g=g_flat[:N].cpu().numpy() if want_g else None,
                   w=w_flat[:N].cpu().numpy(), v=v_flat[:N].cpu().numpy(), layers=out_layers)
        # ---- oracle on the same host bytes
        xs = [oracle.pack(O, ts) for ts in contrib_tensors]
        w = oracle.pack(O, w_tensors)
        v = oracle.pack(O, v_tensors)
        w_old, v_old = w.copy(), v.copy()
        g = oracle.reduce_update(O, xs, w, v, lr, mu, wd, order=order, want_g=True)
        ref = dict(x=xs, g=g, w=w, v=v, w_old=w_old, v_old=v_old, layers=oracle.unpack(O, w))
        return gpu, ref

    def check(self, gpu, ref, lr, mu, wd, what, nan_ok=False):
        cmp = assert_bits_or_both_nan if nan_ok else assert_bits
        for p, (a, b) in enumerate(zip(gpu["x"], ref["x"])):
            assert_bits(a, b, f"{what}: packed contribution {p}")
        if gpu["g"] is not None:
            cmp(gpu["g"], ref["g"], f"{what}: reduced gradient")
        if not nan_ok:
            assert_update_band(gpu["w"], gpu["v"], ref["w"], ref["v"], ref["w_old"], ref["v_old"],
                               ref["g"], lr, mu, wd, what)
        # the update is written without contraction, so it is expected to be bit-exact too
        cmp(gpu["v"], ref["v"], f"{what}: momentum")
        cmp(gpu["w"], ref["w"], f"{what}: weights")
        if gpu["layers"] is not None:
            assert len(gpu["layers"]) == len(ref["layers"])
            for t, (a, b) in enumerate(zip(gpu["layers"], ref["layers"])):
                cmp(a, b, f"{what}: unpacked weights of tensor {t}")


class FusedStep:
    """mc_fused_step from host per-layer tensors, with the oracle's answer composed from its
    pack, reduce_update and unpack."""

    def __init__(self, sizes, k):
        self.sizes = [int(s) for s in sizes]
        self.L = mc.Layout(self.sizes, k)
        self.O = oracle.Layout(self.sizes, k)

    def run(self, contrib_tensors, w_tensors, v_tensors, lr, mu, wd, order=None, want_g=True,
            misalign=None, misalign_w=None, spec=None):
        """spec: an mc.UpdateSpec carrying the same lr, mu, wd -> mc_fused_step_ex instead of
        mc_fused_step (the oracle's answer is the same)."""
        L, O = self.L, self.O
        s = stream_handle()
        placed = [place_tensors(ts, misalign) for ts in contrib_tensors]
        w_dev, w_arena = place_tensors(w_tensors, misalign_w if misalign_w is not None else misalign)
        v_dev, v_arena = place_tensors(v_tensors, misalign_w if misalign_w is not None else misalign)
        sets = [mc.TensorSet(L, ptrs(d)) for d, _ in placed]
        wset = mc.TensorSet(L, ptrs(w_dev))
        vset = mc.TensorSet(L, ptrs(v_dev))
        G = 64
        gbuf = dev_empty(L.N + 2 * G) if want_g else None
        g_ptr = gbuf[G:].data_ptr() if want_g else None
        arenas_before = [a.cpu().numpy().view(np.uint32).copy() if a is not None else None
                         for a in (w_arena, v_arena)]
        if spec is None:
            mc.fused_step(L, sets, order, g_ptr if L.N else None, wset, vset, lr, mu, wd, s)
        else:
            mc.fused_step_ex(L, sets, order, g_ptr if L.N else None, wset, vset, spec, s)
        torch.cuda.synchronize()
        N = L.N
        gpu = dict(g=gbuf[G:G + N].cpu().numpy() if want_g else None,
                   w_layers=[t.cpu().numpy() for t in w_dev], v_layers=[t.cpu().numpy() for t in v_dev])
        if want_g:
            h = gbuf.cpu().numpy().view(np.uint32)
            assert np.all(h[:G] == 0xFFFFFFFF) and np.all(h[G + N:] == 0xFFFFFFFF), "g guard words overwritten"
        # nothing outside the tensors of an arena may change
        for arena, before, devs in ((w_arena, arenas_before[0], w_dev), (v_arena, arenas_before[1], v_dev)):
            if arena is None:
                continue
            after = arena.cpu().numpy().view(np.uint32)
            touched = np.zeros(after.size, bool)
            for t in devs:
                lo = (t.data_ptr() - arena.data_ptr()) // 4
                touched[lo:lo + t.numel()] = True
            assert np.array_equal(after[~touched], before[~touched]), "wrote outside the weight / momentum tensors"
        # contributions are read-only
        for (d, _), ts in zip(placed, contrib_tensors):
            for a, b in zip(d, ts):
                assert_bits(a.cpu().numpy(), b, "a contribution tensor changed")
        for st in sets + [wset, vset]:
            st.destroy()
        # ---- oracle
        xs = [oracle.pack(O, ts) for ts in contrib_tensors]
        w = oracle.pack(O, w_tensors)
        v = oracle.pack(O, v_tensors)
        g = oracle.reduce_update(O, xs, w, v, lr, mu, wd, order=order, want_g=True)
        ref = dict(g=g, w_layers=oracle.unpack(O, w), v_layers=oracle.unpack(O, v))
        return gpu, ref

    @staticmethod
    def check(gpu, ref, what, nan_ok=False):
        cmp = assert_bits_or_both_nan if nan_ok else assert_bits
        if gpu["g"] is not None:
            cmp(gpu["g"], ref["g"], f"{what}: reduced gradient")
        for key in ("w_layers", "v_layers"):
            assert len(gpu[key]) == len(ref[key])
            for t, (a, b) in enumerate(zip(gpu[key], ref[key])):
                cmp(a, b, f"{what}: {key}[{t}]")
