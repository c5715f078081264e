"""Host-side checks of the C-ABI library that need no GPU: exported symbols, layout tables
against the oracle, and argument validation (which must reject before any launch)."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
from paper_1711_00705_amd import mc
from paper_1711_00705_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "mc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mc_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = _declared_functions()
    assert len(names) >= 28
    raw = ctypes.CDLL(mc.LIBRARY_PATH)
    for n in names:
        assert hasattr(raw, n), f"{n} declared in mc.h but not exported"
    assert sorted(mc.SIGNATURES) == names, "binding and header list different entry points"


def test_error_strings():
    for code in (0, -1, -2, -3, -4, -5, -6, -99):
        assert isinstance(mc.strerror(code), str) and mc.strerror(code)
    assert len({mc.strerror(code) for code in (0, -1, -2, -3, -4, -5, -6, -99)}) == 8


def test_pack_noalloc_rejects_before_touching_the_gpu():
    """The capacity limits and the argument checks of mc_pack_noalloc come before its first HIP
    call, so they can be exercised without a GPU."""
    f = mc.lib.mc_pack_noalloc
    too_many = mc.Layout([4] * (mc.NOALLOC_MAX_TENSORS + 1), 2)
    tab = mc.ptr_table([0x1000] * too_many.n)
    assert f(too_many.handle, tab, 0x10000, None) == mc.ERR_LIMIT
    too_long = mc.Layout([mc.NOALLOC_MAX_ELEMS, 1], 4)
    assert f(too_long.handle, mc.ptr_table([0x1000, 0x2000]), 0x10000, None) == mc.ERR_LIMIT
    L = mc.Layout([8, 0, 8], 2)
    assert f(None, mc.ptr_table([0x1000, None, 0x2000]), 0x10000, None) == mc.ERR_INVALID_ARG
    assert f(L.handle, None, 0x10000, None) == mc.ERR_INVALID_ARG
    assert f(L.handle, mc.ptr_table([0x1000, None, 0x2000]), None, None) == mc.ERR_INVALID_ARG
    assert f(L.handle, mc.ptr_table([0x1000, None, 0x2000]), 0x10008, None) == mc.ERR_ALIGN
    assert f(L.handle, mc.ptr_table([0x1000, None, None]), 0x10000, None) == mc.ERR_INVALID_ARG
    assert f(L.handle, mc.ptr_table([0x1002, None, 0x2000]), 0x10000, None) == mc.ERR_ALIGN
    assert f(L.handle, mc.ptr_table([0x10010, None, 0x2000]), 0x10000, None) == mc.ERR_OVERLAP
    empty = mc.Layout([0, 0], 3)
    assert f(empty.handle, mc.ptr_table([None, None]), None, None) == mc.OK


LAYOUT_CASES = [([5], 1), ([0], 3), ([0, 0, 7, 0], 2), ([256], 1), ([257], 2), ([1024], 4),
                ([1025], 4), ([100, 200, 300], 7), ([1], 5), ([3, 1], 900)]


@pytest.mark.parametrize("sizes,k", LAYOUT_CASES)
def test_layout_matches_oracle_small(sizes, k):
    L = mc.Layout(sizes, k)
    O = oracle.Layout(sizes, k)
    assert L.N == O.N
    assert np.array_equal(L.tensor_offsets(), O.off)
    assert np.array_equal(L.colour_bounds(), O.bounds)
    L.destroy()


@pytest.mark.parametrize("name", wl.WORKLOADS)
def test_layout_matches_oracle_workloads(name):
    cfg = wl.workload(name)
    for k in (1, cfg.k, 7, 64):
        L = mc.Layout(cfg.sizes, k)
        O = oracle.Layout(cfg.sizes, k)
        assert L.N == O.N == cfg.total
        assert np.array_equal(L.tensor_offsets(), O.off)
        assert np.array_equal(L.colour_bounds(), O.bounds)


def test_layout_random_matches_oracle():
    rng = np.random.Generator(np.random.PCG64(2))
    for _ in range(200):
        n = int(rng.integers(1, 40))
        sizes = [int(s) for s in rng.integers(0, 20000, size=n)]
        k = int(rng.integers(1, 70))
        L = mc.Layout(sizes, k)
        O = oracle.Layout(sizes, k)
        assert np.array_equal(L.tensor_offsets(), O.off)
        assert np.array_equal(L.colour_bounds(), O.bounds)


def test_layout_create_rejects():
    out = ctypes.c_void_p(123)
    arr = (ctypes.c_int64 * 2)(4, 5)
    f = mc.lib.mc_layout_create
    assert f(None, 2, 1, ctypes.byref(out)) == mc.ERR_INVALID_ARG and not out.value
    assert f(arr, 0, 1, ctypes.byref(out)) == mc.ERR_INVALID_ARG
    assert f(arr, 2, 0, ctypes.byref(out)) == mc.ERR_INVALID_ARG
    assert f(arr, 2, 1, None) == mc.ERR_INVALID_ARG
    neg = (ctypes.c_int64 * 2)(4, -1)
    out = ctypes.c_void_p(123)
    assert f(neg, 2, 1, ctypes.byref(out)) == mc.ERR_INVALID_ARG and not out.value
    huge = (ctypes.c_int64 * 2)(2 ** 40, 1)
    assert f(huge, 2, 1, ctypes.byref(out)) == mc.ERR_INVALID_ARG
    assert mc.lib.mc_layout_destroy(None) == mc.OK
    assert mc.lib.mc_layout_total(None, None) == mc.ERR_INVALID_ARG


def _code(fn, *a, **kw):
    try:
        fn(*a, **kw)
    except mc.McError as e:
        return e.code
    return mc.OK


def test_reduce_update_rejects_before_launch():
    L = mc.Layout([1000, 24], 2)
    N = L.N
    B = 0x10000000                     # made-up, 16-byte aligned device addresses, 1 MiB apart
    x = [B + (i << 20) for i in range(4)]
    g, w, v = B + (8 << 20), B + (9 << 20), B + (10 << 20)
    ru = mc.reduce_update
    assert _code(ru, L, [], None, g, w, v, .1, .9, 0.) == mc.ERR_INVALID_ARG            # P = 0
    assert _code(ru, L, [x[0]] * 33, None, g, w, v, .1, .9, 0.) == mc.ERR_INVALID_ARG   # P > MAX_P
    assert _code(ru, L, [x[0], None], None, g, w, v, .1, .9, 0.) == mc.ERR_INVALID_ARG
    assert _code(ru, L, x, None, g, None, v, .1, .9, 0.) == mc.ERR_INVALID_ARG
    assert _code(ru, L, x, None, g, w, None, .1, .9, 0.) == mc.ERR_INVALID_ARG
    bad = np.array([[0, 1, 2, 3], [0, 1, 1, 3]], np.int32)
    assert _code(ru, L, x, bad, g, w, v, .1, .9, 0.) == mc.ERR_INVALID_ARG
    bad = np.array([[0, 1, 2, 4], [0, 1, 2, 3]], np.int32)
    assert _code(ru, L, x, bad, g, w, v, .1, .9, 0.) == mc.ERR_INVALID_ARG
    bad = np.array([[0, 1, 2, -1], [0, 1, 2, 3]], np.int32)
    assert _code(ru, L, x, bad, g, w, v, .1, .9, 0.) == mc.ERR_INVALID_ARG
    assert _code(ru, L, [x[0], x[1] + 4], None, g, w, v, .1, .9, 0.) == mc.ERR_ALIGN
    assert _code(ru, L, x, None, g + 8, w, v, .1, .9, 0.) == mc.ERR_ALIGN
    assert _code(ru, L, x, None, g, w + 4, v, .1, .9, 0.) == mc.ERR_ALIGN
    assert _code(ru, L, x, None, g, w, v + 12, .1, .9, 0.) == mc.ERR_ALIGN
    assert _code(ru, L, x, None, x[2], w, v, .1, .9, 0.) == mc.ERR_OVERLAP
    assert _code(ru, L, x, None, g, w, w, .1, .9, 0.) == mc.ERR_OVERLAP
    assert _code(ru, L, x, None, g, w, w + 4 * N - 16, .1, .9, 0.) == mc.ERR_OVERLAP     # last vector
    assert _code(ru, L, x, None, None, x[1] + 16, v, .1, .9, 0.) == mc.ERR_OVERLAP
    rc = mc.lib.mc_reduce_update(None, None, 4, None, None, None, None, 0., 0., 0., None)
    assert rc == mc.ERR_INVALID_ARG


def test_pack_rejects_before_launch():
    L = mc.Layout([1000, 0, 24], 2)
    B = 0x10000000
    ts = [B, None, B + (1 << 20)]
    flat = B + (4 << 20)
    for fn in (lambda t, f: mc.pack(L, t, f), lambda t, f: mc.unpack(L, f, t)):
        assert _code(fn, ts, None) == mc.ERR_INVALID_ARG
        assert _code(fn, ts, flat + 4) == mc.ERR_ALIGN
        assert _code(fn, [B, None, None], flat) == mc.ERR_INVALID_ARG      # non-empty tensor, NULL
        assert _code(fn, [B + 2, None, B + (1 << 20)], flat) == mc.ERR_ALIGN
        assert _code(fn, [flat + 400, None, B], flat) == mc.ERR_OVERLAP
        assert _code(fn, [B, None, flat - 8], flat) == mc.ERR_OVERLAP
    # two destination tensors of an unpack that overlap each other (fine as sources of a pack)
    assert _code(lambda t, f: mc.unpack(L, f, t), [B, None, B + 3996], flat) == mc.ERR_OVERLAP
    assert mc.lib.mc_pack(None, None, None, None) == mc.ERR_INVALID_ARG
    assert mc.lib.mc_unpack(None, None, None, None) == mc.ERR_INVALID_ARG
    assert mc.lib.mc_layout_prepare(None) == mc.ERR_INVALID_ARG


def test_empty_payload_is_a_no_op():
    L = mc.Layout([0, 0], 3)
    assert L.N == 0 and list(L.colour_bounds()) == [0, 0, 0, 0]
    mc.pack(L, [None, None], None)
    mc.unpack(L, None, [None, None])
    mc.reduce_update(L, [None], None, None, None, None, 0.1, 0.9, 0.0)


def test_options():
    assert mc.get_option(mc.OPT_RU_SHAPE) in (0, 1, 2)
    for opt, good, bad in ((mc.OPT_RU_SHAPE, (0, 1, 2), (-1, 3, 4)),
                           (mc.OPT_STATE_POLICY, (1, 2), (-1, 0, 3)),
                           (mc.OPT_PACK_NONTEMPORAL, (0, 1, 2, 3), (-1, 4)),
                           (mc.OPT_STATE_STORE_SC1, (0, 1), (-1, 2)),
                           (mc.OPT_ALTERNATE_SWEEP, (0, 1), (-1, 2)),
                           (mc.OPT_XCD_RUN, (0, 1, 8, 64), (-1, 65)),
                           (mc.OPT_XCD_RUN_PACK, (-1, 0, 16, 64), (-2, 65)),
                           (mc.OPT_XCD_RUN_UNPACK, (-1, 0, 16, 64), (-2, 65)),
                           (mc.OPT_DIRECT_TILES, (0, 1, 2), (-1, 3)),
                           (mc.OPT_LDS_CAP_UPDATE, (-1, 0, 20480, 65536), (-2, 65537)),
                           (mc.OPT_LDS_CAP_PACK, (-1, 0, 20480, 65536), (-2, 65537))):
        keep = mc.get_option(opt)
        for g in good:
            mc.set_option(opt, g)
            assert mc.get_option(opt) == g
        for b in bad:
            assert _code(mc.set_option, opt, b) == mc.ERR_INVALID_ARG
        mc.set_option(opt, keep)
    assert _code(mc.set_option, 99, 0) == mc.ERR_INVALID_ARG
    assert _code(mc.get_option, 99) == mc.ERR_INVALID_ARG


def test_copy_rejects_before_launch():
    B = 0x10000000
    assert _code(mc.copy, B, B + 4096, 0) == mc.OK                      # nothing to do
    assert _code(mc.copy, B, B + 4096, 100) == mc.ERR_INVALID_ARG       # not a multiple of 16
    assert _code(mc.copy, B, B + 4096, -16) == mc.ERR_INVALID_ARG
    assert _code(mc.copy, None, B, 1024) == mc.ERR_INVALID_ARG
    assert _code(mc.copy, B, None, 1024) == mc.ERR_INVALID_ARG
    assert _code(mc.copy, B + 8, B + 4096, 1024) == mc.ERR_ALIGN
    assert _code(mc.copy, B, B + 512, 1024) == mc.ERR_OVERLAP


def test_reduce_update_roles_rejects_before_launch():
    L = mc.Layout([1000, 24], 2)
    B = 0x10000000
    x = [B + (i << 20) for i in range(4)]
    g, w, v = B + (8 << 20), B + (9 << 20), B + (10 << 20)
    rr = mc.reduce_update_roles
    assert _code(rr, L, x, None, [4, 5], [1, 1], g, w, v, .1, .9, 0.) == mc.ERR_INVALID_ARG   # n_terms > P
    assert _code(rr, L, x, None, [4, -1], [1, 1], g, w, v, .1, .9, 0.) == mc.ERR_INVALID_ARG
    assert _code(rr, L, x, None, [4, 2], [1, 0], None, w, v, .1, .9, 0.) == mc.ERR_INVALID_ARG  # sum-only needs g
    assert _code(rr, L, x, None, [4, 2], [1, 0], g, None, v, .1, .9, 0.) == mc.ERR_INVALID_ARG  # update needs w
    assert _code(rr, L, x, None, [4, 2], [1, 0], g, w, None, .1, .9, 0.) == mc.ERR_INVALID_ARG
    assert _code(rr, L, x, None, [4, 2], [1, 0], g + 4, w, v, .1, .9, 0.) == mc.ERR_ALIGN
    assert _code(rr, L, x, None, [4, 2], [1, 0], x[0], w, v, .1, .9, 0.) == mc.ERR_OVERLAP
    rc = mc.lib.mc_reduce_update_roles(L.handle, mc.ptr_table(x), 4, None, None, None, g, w, v, 0., 0., 0., None)
    assert rc == mc.ERR_INVALID_ARG
    # every colour skipped: nothing to do, nothing needed
    assert _code(rr, L, x, None, [0, 0], [1, 0], None, None, None, .1, .9, 0.) in (mc.OK, mc.ERR_HIP)


@pytest.mark.parametrize("first", ["torch", "mc"])
def test_one_hip_runtime_whatever_the_import_order(first):
    """torch bundles its own HIP runtime; the binding must end up sharing it, or the second
    runtime in the process would see no device."""
    import subprocess
    import sys
    code = (
        "import sys; sys.path.insert(0, %r)\n"
        "%s\n"
        "libs = sorted(set(l.split()[-1] for l in open('/proc/self/maps') if 'libamdhip64' in l))\n"
        "print(len(libs), libs)\n"
    ) % (ROOT, "import torch; from paper_1711_00705_amd import mc" if first == "torch"
         else "from paper_1711_00705_amd import mc; import torch")
    out = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=300)
    assert out.returncode == 0, out.stderr
    assert out.stdout.split()[0] == "1", out.stdout


def test_tensor_set_rejects_before_touching_the_gpu():
    import ctypes
    L = mc.Layout([1000, 0, 24], 2)
    B = 0x10000000
    out = ctypes.c_void_p(5)
    f = mc.lib.mc_tensor_set_create
    assert f(None, mc.ptr_table([B, None, B + 8192]), ctypes.byref(out)) == mc.ERR_INVALID_ARG and not out.value
    assert f(L.handle, None, ctypes.byref(out)) == mc.ERR_INVALID_ARG
    assert f(L.handle, mc.ptr_table([B, None, B + 8192]), None) == mc.ERR_INVALID_ARG
    assert f(L.handle, mc.ptr_table([B, None, None]), ctypes.byref(out)) == mc.ERR_INVALID_ARG
    assert f(L.handle, mc.ptr_table([B + 1, None, B + 8192]), ctypes.byref(out)) == mc.ERR_ALIGN
    assert f(L.handle, mc.ptr_table([B, None, B + 3996]), ctypes.byref(out)) == mc.ERR_OVERLAP
    assert mc.lib.mc_tensor_set_destroy(None) == mc.OK
    assert mc.lib.mc_pack_set(L.handle, None, B, None) == mc.ERR_INVALID_ARG
    assert mc.lib.mc_unpack_set(None, B, None, None) == mc.ERR_INVALID_ARG
    assert mc.lib.mc_fused_step(L.handle, None, 1, None, None, None, None, 0., 0., 0., None) == mc.ERR_INVALID_ARG


def test_reduce_update_range_rejects_before_launch():
    L = mc.Layout([1000, 24], 2)          # N = 1024, bounds 0, 512, 1024
    B = 0x10000000
    x = [B + (i << 20) for i in range(2)]
    g, w, v = B + (8 << 20), B + (9 << 20), B + (10 << 20)
    rr = mc.reduce_update_range
    assert _code(rr, L, x, None, g, w, v, .1, .9, 0., -256, 512) == mc.ERR_INVALID_ARG
    assert _code(rr, L, x, None, g, w, v, .1, .9, 0., 512, 256) == mc.ERR_INVALID_ARG
    assert _code(rr, L, x, None, g, w, v, .1, .9, 0., 0, 1025) == mc.ERR_INVALID_ARG
    assert _code(rr, L, x, None, g, w, v, .1, .9, 0., 100, 512) == mc.ERR_INVALID_ARG     # begin unaligned
    assert _code(rr, L, x, None, g, w, v, .1, .9, 0., 0, 700) == mc.ERR_INVALID_ARG       # end unaligned, not N
    assert _code(rr, L, x, None, g, w, v, .1, .9, 0., 256, 256) == mc.OK                  # empty packet
    assert _code(rr, L, x, None, g, w + 4, v, .1, .9, 0., 0, 256) == mc.ERR_ALIGN
    assert _code(rr, L, x, None, g, w, v, .1, .9, 0., 0, 256, 0, [2, 3], [1, 1]) == mc.ERR_INVALID_ARG  # n_terms > P
    L2 = mc.Layout([1000], 1)             # N = 1000: a range may end at N (and then must be aligned)
    assert _code(rr, L2, x, None, g, w + 4, v, .1, .9, 0., 768, 1000, 0) == mc.ERR_ALIGN
    assert _code(rr, L2, x, None, g, w, v, .1, .9, 0., 768, 999, 0) == mc.ERR_INVALID_ARG
