"""Randomised calls of the C ABI with valid-shaped but arbitrary arguments, on the CPU: every
call must come back with one of the documented codes (never crash, never hang), and calls that
pass validation may only fail with MC_ERR_HIP here (there is no GPU to launch on)."""
import ctypes

import numpy as np
import pytest

from paper_1711_00705_amd import mc


def _gpu_present() -> bool:
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


# The addresses below are made up.  Without a GPU a call that passes validation fails in the HIP
# runtime; WITH one it would launch on them, so this file must never run where a GPU is visible.
pytestmark = pytest.mark.skipif(_gpu_present(), reason="made-up device addresses: CPU-only test")

CODES = {mc.OK, mc.ERR_INVALID_ARG, mc.ERR_ALIGN, mc.ERR_OVERLAP, mc.ERR_ALLOC, mc.ERR_HIP}


def _code(fn, *a, **kw):
    try:
        fn(*a, **kw)
    except mc.McError as e:
        return e.code
    return mc.OK


def test_random_calls_return_documented_codes():
    rng = np.random.Generator(np.random.PCG64(99))
    seen = set()
    for it in range(1500):
        n = int(rng.integers(1, 12))
        sizes = [int(s) for s in rng.choice([0, 1, 3, 4, 255, 256, 257, 1000, 4096, 70000], size=n)]
        k = int(rng.choice([1, 2, 3, 8, 40]))
        L = mc.Layout(sizes, k)
        N = L.N
        P = int(rng.choice([1, 2, 4, 8, 32, 33, 0]))
        base = 0x10000000

        def addr():
            a = base + int(rng.integers(0, 64)) * (1 << 22)
            if rng.random() < 0.15:
                a += int(rng.choice([4, 8, 12, 2]))
            return None if rng.random() < 0.05 else a
        x = [addr() for _ in range(max(P, 0))]
        order = None
        if P > 0 and rng.random() < 0.5:
            order = np.stack([rng.permutation(P) for _ in range(k)]).astype(np.int32)
            if rng.random() < 0.2:
                order[int(rng.integers(0, k)), int(rng.integers(0, P))] = int(rng.integers(-2, P + 2))
        g, w, v = addr(), addr(), addr()
        c = _code(mc.reduce_update, L, x, order, g, w, v, 0.1, 0.9, 1e-4)
        assert c in CODES, c
        seen.add(c)
        if P > 0:
            nt = rng.integers(-1, P + 2, size=k).astype(np.int32)
            du = rng.integers(0, 2, size=k).astype(np.uint8)
            c = _code(mc.reduce_update_roles, L, x, order, nt, du, g, w, v, 0.1, 0.9, 1e-4)
            assert c in CODES, c
            b = int(rng.integers(-2, N // 256 + 3)) * 256
            e = int(rng.choice([N, b + 256 * int(rng.integers(0, 5)), N + 1, b - 256]))
            c = _code(mc.reduce_update_range, L, x, order, g, w, v, 0.1, 0.9, 1e-4, b, e)
            assert c in CODES, c
            spec = mc.update_spec(0.1, 0.9, 0.0, hyper_dev_ptr=addr() if rng.random() < 0.3 else None,
                                  nesterov=int(rng.choice([0, 1, 2, -1])))
            c = _code(mc.reduce_update_ex, L, x, order, g, w, v, spec)
            assert c in CODES, c
        tens = [addr() for _ in range(n)]
        assert _code(mc.pack, L, tens, g) in CODES
        assert _code(mc.unpack, L, g, tens) in CODES
        out = ctypes.c_void_p()
        rc = mc.lib.mc_tensor_set_create(L.handle, mc.ptr_table(tens), ctypes.byref(out))
        assert rc in CODES and (rc == mc.OK) == bool(out.value)
        if out.value:
            mc.lib.mc_tensor_set_destroy(out)
        L.destroy()
    assert {mc.ERR_INVALID_ARG, mc.ERR_ALIGN, mc.ERR_OVERLAP} <= seen
