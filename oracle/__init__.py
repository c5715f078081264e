"""CPU oracle (test infrastructure): numpy-facing wrapper around ``mc_oracle.c``.

Only ``tests/``, ``__graft_entry__.smoke()`` and the CPU-baseline leg of ``bench.py`` may
import this package.  It never imports the GPU package, and the GPU package never
imports it.  All arithmetic is in ``mc_oracle.c`` (plain loops); this file only builds
the shared object with gcc and marshals numpy arrays into pointers.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mc_oracle.c")
_LIB = os.path.join(_HERE, "libmc_oracle.so")
_CFLAGS = ["-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC", "-Wall"]

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (a second or so).  Returns the path of the library."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", *_CFLAGS, "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64p = ctypes.POINTER(ctypes.c_int64)
        i32p = ctypes.POINTER(ctypes.c_int32)
        vpp = ctypes.POINTER(ctypes.c_void_p)
        lib.mco_layout.argtypes = [i64p, ctypes.c_int32, ctypes.c_int32, i64p, i64p]
        lib.mco_layout.restype = ctypes.c_int
        lib.mco_pack.argtypes = [i64p, ctypes.c_int32, vpp, ctypes.c_void_p]
        lib.mco_pack.restype = None
        lib.mco_unpack.argtypes = [i64p, ctypes.c_int32, ctypes.c_void_p, vpp]
        lib.mco_unpack.restype = None
        lib.mco_reduce_update_colour.argtypes = [
            ctypes.c_int64, ctypes.c_int64, vpp, ctypes.c_int32, i32p,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_float, ctypes.c_float, ctypes.c_float]
        lib.mco_reduce_update_colour.restype = None
        lib.mco_reduce_update_colour_nesterov.argtypes = lib.mco_reduce_update_colour.argtypes
        lib.mco_reduce_update_colour_nesterov.restype = None
        lib.mco_reduce_update.argtypes = [
            i64p, ctypes.c_int32, vpp, ctypes.c_int32, i32p,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_float, ctypes.c_float, ctypes.c_float]
        lib.mco_reduce_update.restype = ctypes.c_int
        lib.mco_reduce_update_roles.argtypes = [
            i64p, ctypes.c_int32, vpp, ctypes.c_int32, i32p, i32p, ctypes.POINTER(ctypes.c_uint8),
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_float, ctypes.c_float, ctypes.c_float]
        lib.mco_reduce_update_roles.restype = ctypes.c_int
        _lib = lib
    return _lib


def _i64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int64)


def _ptr(a: np.ndarray, typ):
    return a.ctypes.data_as(ctypes.POINTER(typ))


def _check_f32(a: np.ndarray, n: Optional[int] = None, name: str = "array") -> None:
    if not (isinstance(a, np.ndarray) and a.dtype == np.float32 and a.flags.c_contiguous
            and a.ndim == 1):
        raise TypeError(f"{name}: need a contiguous 1-d float32 numpy array")
    if n is not None and a.shape[0] != n:
        raise ValueError(f"{name}: length {a.shape[0]} != {n}")


def _ptr_table(arrs: Sequence[np.ndarray]):
    tab = (ctypes.c_void_p * len(arrs))()
    for i, a in enumerate(arrs):
        tab[i] = a.ctypes.data
    return tab


class Layout:
    """Flat offsets ``off`` (n+1) and colour bounds ``bounds`` (k+1) of a tensor list."""

    def __init__(self, numel: Sequence[int], k: int):
        numel = _i64(numel)
        n = int(numel.shape[0])
        self.n = n
        self.k = int(k)
        self.off = np.zeros(n + 1, dtype=np.int64)
        self.bounds = np.zeros(max(self.k, 0) + 1, dtype=np.int64)
        rc = _load().mco_layout(_ptr(numel, ctypes.c_int64), n, self.k,
                                _ptr(self.off, ctypes.c_int64), _ptr(self.bounds, ctypes.c_int64))
        if rc != 0:
            raise ValueError("mco_layout: invalid argument")
        self.N = int(self.off[n])


def pack(layout: Layout, tensors: Sequence[np.ndarray]) -> np.ndarray:
    """Concatenate per-layer tensors into the flat payload (bit copy)."""
    assert len(tensors) == layout.n
    for t, a in enumerate(tensors):
        _check_f32(a, int(layout.off[t + 1] - layout.off[t]), f"tensor {t}")
    flat = np.empty(layout.N, dtype=np.float32)
    _load().mco_pack(_ptr(layout.off, ctypes.c_int64), layout.n, _ptr_table(tensors),
                     flat.ctypes.data)
    return flat


def unpack(layout: Layout, flat: np.ndarray) -> List[np.ndarray]:
    """Split the flat payload back into per-layer tensors (bit copy)."""
    _check_f32(flat, layout.N, "flat")
    outs = [np.empty(int(layout.off[t + 1] - layout.off[t]), dtype=np.float32)
            for t in range(layout.n)]
    _load().mco_unpack(_ptr(layout.off, ctypes.c_int64), layout.n, flat.ctypes.data,
                       _ptr_table(outs))
    return outs


def _order_arg(order, k: int, P: int):
    if order is None:
        return None, None
    o = np.ascontiguousarray(order, dtype=np.int32)
    if o.shape != (k, P):
        raise ValueError(f"order must have shape ({k},{P})")
    for c in range(k):
        if sorted(o[c].tolist()) != list(range(P)):
            raise ValueError(f"order row {c} is not a permutation of 0..{P-1}")
    return o, _ptr(o, ctypes.c_int32)


def reduce_update(layout: Layout, contrib: Sequence[np.ndarray], w: np.ndarray, v: np.ndarray,
                  lr: float, mu: float, wd: float, order=None, want_g: bool = True):
    """Sum the P flat contributions per colour in the given sequence and apply the SGD
    momentum / weight-decay update to ``w`` and ``v`` IN PLACE.  Returns g (or None)."""
    P = len(contrib)
    for p, a in enumerate(contrib):
        _check_f32(a, layout.N, f"contrib {p}")
    _check_f32(w, layout.N, "w")
    _check_f32(v, layout.N, "v")
    o, optr = _order_arg(order, layout.k, P)
    g = np.empty(layout.N, dtype=np.float32) if want_g else None
    rc = _load().mco_reduce_update(_ptr(layout.bounds, ctypes.c_int64), layout.k,
                                   _ptr_table(contrib), P, optr,
                                   g.ctypes.data if want_g else None,
                                   w.ctypes.data, v.ctypes.data,
                                   ctypes.c_float(lr), ctypes.c_float(mu), ctypes.c_float(wd))
    if rc != 0:
        raise ValueError("mco_reduce_update: invalid argument")
    return g


def reduce_update_colour(layout: Layout, c: int, contrib: Sequence[np.ndarray], g, w, v,
                         lr: float, mu: float, wd: float, seq=None) -> None:
    """One colour only (colours are independent, so they may be run in any order or on
    separate host threads; ctypes releases the GIL during the call)."""
    P = len(contrib)
    s = np.arange(P, dtype=np.int32) if seq is None else np.ascontiguousarray(seq, dtype=np.int32)
    assert sorted(s.tolist()) == list(range(P))
    _load().mco_reduce_update_colour(int(layout.bounds[c]), int(layout.bounds[c + 1]),
                                     _ptr_table(contrib), P, _ptr(s, ctypes.c_int32),
                                     None if g is None else g.ctypes.data,
                                     w.ctypes.data, v.ctypes.data,
                                     ctypes.c_float(lr), ctypes.c_float(mu), ctypes.c_float(wd))


def reduce_update_roles(layout: Layout, contrib: Sequence[np.ndarray], n_terms, do_update,
                        g: np.ndarray, w, v, lr: float, mu: float, wd: float, order=None) -> None:
    """Per-colour roles (Section 4.2): colour c adds the first n_terms[c] entries of its
    sequence into ``g`` (IN PLACE; ranges of skipped colours are left alone) and applies the
    SGD step only where do_update[c] is set.  ``w`` / ``v`` may be None if no colour updates."""
    P = len(contrib)
    for p, a in enumerate(contrib):
        _check_f32(a, layout.N, f"contrib {p}")
    _check_f32(g, layout.N, "g")
    nt = np.ascontiguousarray(n_terms, dtype=np.int32)
    du = np.ascontiguousarray(do_update, dtype=np.uint8)
    assert nt.shape == (layout.k,) and du.shape == (layout.k,)
    if w is not None:
        _check_f32(w, layout.N, "w")
        _check_f32(v, layout.N, "v")
    o, optr = _order_arg(order, layout.k, P)
    rc = _load().mco_reduce_update_roles(
        _ptr(layout.bounds, ctypes.c_int64), layout.k, _ptr_table(contrib), P, optr,
        _ptr(nt, ctypes.c_int32), _ptr(du, ctypes.c_uint8), g.ctypes.data,
        None if w is None else w.ctypes.data, None if v is None else v.ctypes.data,
        ctypes.c_float(lr), ctypes.c_float(mu), ctypes.c_float(wd))
    if rc != 0:
        raise ValueError("mco_reduce_update_roles: invalid argument")


def reduce_update_range(layout: Layout, contrib: Sequence[np.ndarray], g, w, v,
                        lr: float, mu: float, wd: float, begin: int, end: int, order=None) -> None:
    """The step restricted to flat elements [begin, end) (one packet of the pipelined
    reduction, Section 4.2): every colour is cut to that range; g, w, v are changed IN PLACE
    there and nowhere else."""
    P = len(contrib)
    for c in range(layout.k):
        lo = max(int(layout.bounds[c]), begin)
        hi = min(int(layout.bounds[c + 1]), end)
        if hi <= lo:
            continue
        seq = np.arange(P, dtype=np.int32) if order is None else np.ascontiguousarray(order[c], dtype=np.int32)
        _load().mco_reduce_update_colour(lo, hi, _ptr_table(contrib), P, _ptr(seq, ctypes.c_int32),
                                         None if g is None else g.ctypes.data, w.ctypes.data, v.ctypes.data,
                                         ctypes.c_float(lr), ctypes.c_float(mu), ctypes.c_float(wd))


def reduce_update_nesterov(layout: Layout, contrib: Sequence[np.ndarray], w: np.ndarray, v: np.ndarray,
                           lr: float, mu: float, wd: float, order=None) -> np.ndarray:
    """reduce_update with the Nesterov look-ahead step; w and v IN PLACE, returns g."""
    P = len(contrib)
    for p, a in enumerate(contrib):
        _check_f32(a, layout.N, f"contrib {p}")
    _check_f32(w, layout.N, "w")
    _check_f32(v, layout.N, "v")
    o, _ = _order_arg(order, layout.k, P)
    g = np.empty(layout.N, dtype=np.float32)
    for c in range(layout.k):
        seq = np.arange(P, dtype=np.int32) if o is None else np.ascontiguousarray(o[c])
        _load().mco_reduce_update_colour_nesterov(
            int(layout.bounds[c]), int(layout.bounds[c + 1]), _ptr_table(contrib), P,
            _ptr(seq, ctypes.c_int32), g.ctypes.data, w.ctypes.data, v.ctypes.data,
            ctypes.c_float(lr), ctypes.c_float(mu), ctypes.c_float(wd))
    return g
