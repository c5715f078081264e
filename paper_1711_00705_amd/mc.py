"""Thin ctypes binding of libmc.so: the same entry points as include/mc.h, argument
marshalling only.  Every step of the path runs in the library's HIP kernels; there is no
fallback of any kind -- a missing or unloadable library raises at import of this module.

Device buffers are passed as integer addresses (e.g. ``torch.Tensor.data_ptr()``), the
stream as the integer ``hipStream_t`` (e.g. ``torch.cuda.current_stream().cuda_stream``).
"""
from __future__ import annotations

import ctypes
from typing import Optional, Sequence

import numpy as np

from . import build as _build

OK = 0
ERR_INVALID_ARG = -1
ERR_ALIGN = -2
ERR_OVERLAP = -3
ERR_ALLOC = -4
ERR_HIP = -5
ERR_LIMIT = -6
MAX_P = 32
NOALLOC_MAX_TENSORS = 256
NOALLOC_MAX_ELEMS = 1 << 28
PACKETS_MAX_COLOURS = 32
PACKETS_MAX_BLOCKS = 4096
PACKETS_STATUS_WORDS = 2
COLOUR_ALIGN_ELEMS = 256
OPT_RU_SHAPE = 1
OPT_STATE_POLICY = 2
OPT_PACK_NONTEMPORAL = 3
OPT_STATE_STORE_SC1 = 4
OPT_ALTERNATE_SWEEP = 5
OPT_XCD_RUN = 6
OPT_XCD_RUN_PACK = 7
OPT_XCD_RUN_UNPACK = 8
OPT_DIRECT_TILES = 9
OPT_LDS_CAP_UPDATE = 10
OPT_LDS_CAP_PACK = 11
STATE_DEFAULT, STATE_RESIDENT, STATE_STREAMING = 0, 1, 2
SWEEP_AUTO, SWEEP_FORWARD, SWEEP_BACKWARD = 0, 1, 2
ROLE_LEAF, ROLE_INNER, ROLE_ROOT = 0, 1, 2

_i64p = ctypes.POINTER(ctypes.c_int64)
_i32p = ctypes.POINTER(ctypes.c_int32)
_vpp = ctypes.POINTER(ctypes.c_void_p)
_vp = ctypes.c_void_p

# name -> (restype, argtypes): one entry per declaration in include/mc.h
SIGNATURES = {
    "mc_layout_create": (ctypes.c_int, [_i64p, ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(_vp)]),
    "mc_layout_destroy": (ctypes.c_int, [_vp]),
    "mc_layout_prepare": (ctypes.c_int, [_vp]),
    "mc_layout_total": (ctypes.c_int, [_vp, _i64p]),
    "mc_layout_counts": (ctypes.c_int, [_vp, _i32p, _i32p]),
    "mc_layout_tensor_offsets": (ctypes.c_int, [_vp, _i64p]),
    "mc_layout_colour_bounds": (ctypes.c_int, [_vp, _i64p]),
    "mc_layout_units": (ctypes.c_int, [_vp, _i32p, _i32p, _i32p]),
    "mc_pack": (ctypes.c_int, [_vp, _vpp, _vp, _vp]),
    "mc_unpack": (ctypes.c_int, [_vp, _vp, _vpp, _vp]),
    "mc_pack_noalloc": (ctypes.c_int, [_vp, _vpp, _vp, _vp]),
    "mc_reduce_update": (ctypes.c_int, [_vp, _vpp, ctypes.c_int32, _i32p, _vp, _vp, _vp,
                                        ctypes.c_float, ctypes.c_float, ctypes.c_float, _vp]),
    "mc_colour_trees": (ctypes.c_int, [ctypes.c_int32, ctypes.c_int32, _i32p]),
    "mc_rank_roles": (ctypes.c_int, [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, _i32p, _i32p, _i32p]),
    "mc_reduce_update_roles": (ctypes.c_int, [_vp, _vpp, ctypes.c_int32, _i32p, _i32p,
                                              ctypes.POINTER(ctypes.c_uint8), _vp, _vp, _vp,
                                              ctypes.c_float, ctypes.c_float, ctypes.c_float, _vp]),
    "mc_reduce_update_range": (ctypes.c_int, [_vp, _vpp, ctypes.c_int32, _i32p, _i32p,
                                              ctypes.POINTER(ctypes.c_uint8), _vp, _vp, _vp,
                                              ctypes.c_float, ctypes.c_float, ctypes.c_float,
                                              ctypes.c_int64, ctypes.c_int64, _vp]),
    "mc_tensor_set_create": (ctypes.c_int, [_vp, _vpp, ctypes.POINTER(_vp)]),
    "mc_tensor_set_destroy": (ctypes.c_int, [_vp]),
    "mc_pack_set": (ctypes.c_int, [_vp, _vp, _vp, _vp]),
    "mc_unpack_set": (ctypes.c_int, [_vp, _vp, _vp, _vp]),
    "mc_fused_step": (ctypes.c_int, [_vp, _vpp, ctypes.c_int32, _i32p, _vp, _vp, _vp,
                                     ctypes.c_float, ctypes.c_float, ctypes.c_float, _vp]),
    "mc_reduce_update_ex": (ctypes.c_int, [_vp, _vpp, ctypes.c_int32, _i32p, _i32p,
                                           ctypes.POINTER(ctypes.c_uint8), _vp, _vp, _vp, _vp,
                                           ctypes.c_int64, ctypes.c_int64, _vp]),
    "mc_fused_step_ex": (ctypes.c_int, [_vp, _vpp, ctypes.c_int32, _i32p, _i32p,
                                        ctypes.POINTER(ctypes.c_uint8), _vp, _vp, _vp, _vp, _vp]),
    "mc_packets_reset": (ctypes.c_int, [_vp, ctypes.c_int32, _vp, ctypes.c_int32, _vp]),
    "mc_packet_signal": (ctypes.c_int, [_vp, ctypes.c_int32, ctypes.c_uint32, _vp]),
    "mc_packet_deliver": (ctypes.c_int, [_vp, _vp, ctypes.c_int64, _vp, _vp]),
    "mc_delay": (ctypes.c_int, [ctypes.c_uint32, _vp]),
    "mc_reduce_update_packets": (ctypes.c_int, [_vp, _vpp, ctypes.c_int32, _i32p, _vp, _vp, _vp, _vp,
                                                _vp, ctypes.c_int32, _vp, ctypes.c_uint32, ctypes.c_uint32,
                                                _vp, ctypes.c_int32, _vp]),
    "mc_hyper_write": (ctypes.c_int, [_vp, ctypes.c_float, ctypes.c_float, ctypes.c_float, _vp]),
    "mc_lr_schedule": (ctypes.c_int, [ctypes.c_float, ctypes.c_int32, ctypes.c_int32, ctypes.c_float,
                                      ctypes.c_float, ctypes.c_float, ctypes.POINTER(ctypes.c_float)]),
    "mc_copy": (ctypes.c_int, [_vp, _vp, ctypes.c_int64, _vp]),
    "mc_strerror": (ctypes.c_char_p, [ctypes.c_int]),
    "mc_last_hip_error": (ctypes.c_int, []),
    "mc_set_option": (ctypes.c_int, [ctypes.c_int, ctypes.c_int]),
    "mc_get_option": (ctypes.c_int, [ctypes.c_int, ctypes.POINTER(ctypes.c_int)]),
}


def _share_torch_hip_runtime() -> None:
    """One process must use ONE HIP runtime.  PyTorch wheels bundle their own libamdhip64
    (same SONAME as the system one, found through torch/lib's RPATH).  If libmc.so pulled in
    the system copy first and torch its bundled copy later, the process would hold two
    runtimes and the second one sees no device.  Device memory and streams come from torch,
    so when torch is installed its copy is loaded here, before libmc.so, whose dependency on
    the SONAME then binds to it; a later `import torch` finds the same file already mapped."""
    import importlib.util
    import os
    try:
        spec = importlib.util.find_spec("torch")
    except (ImportError, ValueError):
        spec = None
    if spec is None or not spec.origin:
        return
    cand = os.path.join(os.path.dirname(spec.origin), "lib", "libamdhip64.so")
    if os.path.exists(cand):
        ctypes.CDLL(cand, mode=ctypes.RTLD_GLOBAL)


def _load() -> ctypes.CDLL:
    path = _build.library_path(build_if_missing=True)
    _share_torch_hip_runtime()
    lib = ctypes.CDLL(path)
    for name, (res, args) in SIGNATURES.items():
        fn = getattr(lib, name)          # AttributeError if the symbol is not exported
        fn.restype = res
        fn.argtypes = args
    return lib


lib = _load()
LIBRARY_PATH = lib._name


class McError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = lib.mc_strerror(code).decode()
        if code == ERR_HIP:
            msg += " (hipError_t %d)" % lib.mc_last_hip_error()
        super().__init__(f"{where}: {msg} [{code}]")


def _check(code: int, where: str) -> None:
    if code != OK:
        raise McError(code, where)


class PtrTable:
    """A host array of device addresses (or handles) that can be passed to the library as is
    and reused across calls (saves rebuilding it on every step)."""

    def __init__(self, ptrs: Sequence[Optional[int]], keep=None):
        self.count = len(ptrs)
        self._array = (ctypes.c_void_p * max(self.count, 1))()
        for i, p in enumerate(ptrs):
            self._array[i] = p
        self._as_parameter_ = ctypes.cast(self._array, ctypes.POINTER(ctypes.c_void_p))  # what ctypes passes
        self.keep = keep                       # objects whose lifetime the table depends on


def ptr_table(ptrs: Sequence[Optional[int]]) -> PtrTable:
    return PtrTable(ptrs)


def _ptr_table(ptrs) -> PtrTable:
    return ptrs if isinstance(ptrs, PtrTable) else PtrTable(ptrs)


def _count(ptrs) -> int:
    return ptrs.count if isinstance(ptrs, PtrTable) else len(ptrs)


class Layout:
    """Owns one ``mc_layout*``."""

    def __init__(self, numel: Sequence[int], k_colours: int):
        arr = np.ascontiguousarray(numel, dtype=np.int64)
        self._h = _vp()
        _check(lib.mc_layout_create(arr.ctypes.data_as(_i64p), int(arr.shape[0]), int(k_colours),
                                    ctypes.byref(self._h)), "mc_layout_create")
        n = ctypes.c_int32()
        k = ctypes.c_int32()
        _check(lib.mc_layout_counts(self._h, ctypes.byref(n), ctypes.byref(k)), "mc_layout_counts")
        self.n, self.k = n.value, k.value
        total = ctypes.c_int64()
        _check(lib.mc_layout_total(self._h, ctypes.byref(total)), "mc_layout_total")
        self.N = total.value

    @property
    def handle(self):
        return self._h

    def tensor_offsets(self) -> np.ndarray:
        off = np.empty(self.n + 1, dtype=np.int64)
        _check(lib.mc_layout_tensor_offsets(self._h, off.ctypes.data_as(_i64p)), "mc_layout_tensor_offsets")
        return off

    def colour_bounds(self) -> np.ndarray:
        b = np.empty(self.k + 1, dtype=np.int64)
        _check(lib.mc_layout_colour_bounds(self._h, b.ctypes.data_as(_i64p)), "mc_layout_colour_bounds")
        return b

    def units(self):
        """(units_per_colour, unit_tensor[k, units_per_colour], unit_first[n + k]); (0, None, None) without a table."""
        upc = ctypes.c_int32()
        _check(lib.mc_layout_units(self._h, ctypes.byref(upc), None, None), "mc_layout_units")
        if upc.value == 0:
            return 0, None, None
        ut = np.empty(self.k * upc.value, dtype=np.int32)
        uf = np.empty(self.n + self.k, dtype=np.int32)
        _check(lib.mc_layout_units(self._h, ctypes.byref(upc), ut.ctypes.data_as(_i32p), uf.ctypes.data_as(_i32p)),
               "mc_layout_units")
        return upc.value, ut.reshape(self.k, upc.value), uf

    def prepare(self) -> None:
        _check(lib.mc_layout_prepare(self._h), "mc_layout_prepare")

    def destroy(self) -> None:
        if self._h:
            h, self._h = self._h, _vp()
            _check(lib.mc_layout_destroy(h), "mc_layout_destroy")

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def layout_create(numel: Sequence[int], k_colours: int) -> Layout:
    return Layout(numel, k_colours)


def pack(layout: Layout, tensor_ptrs: Sequence[Optional[int]], flat_ptr: Optional[int], stream: int = 0) -> None:
    if _count(tensor_ptrs) != layout.n:
        raise ValueError("need one pointer per tensor of the layout")
    _check(lib.mc_pack(layout.handle, _ptr_table(tensor_ptrs), flat_ptr, stream or None), "mc_pack")


def pack_noalloc(layout: Layout, tensor_ptrs: Sequence[Optional[int]], flat_ptr: Optional[int],
                 stream: int = 0) -> None:
    if _count(tensor_ptrs) != layout.n:
        raise ValueError("need one pointer per tensor of the layout")
    _check(lib.mc_pack_noalloc(layout.handle, _ptr_table(tensor_ptrs), flat_ptr, stream or None), "mc_pack_noalloc")


def unpack(layout: Layout, flat_ptr: Optional[int], tensor_ptrs: Sequence[Optional[int]], stream: int = 0) -> None:
    if _count(tensor_ptrs) != layout.n:
        raise ValueError("need one pointer per tensor of the layout")
    _check(lib.mc_unpack(layout.handle, flat_ptr, _ptr_table(tensor_ptrs), stream or None), "mc_unpack")


def reduce_update(layout: Layout, contrib_ptrs: Sequence[Optional[int]], order, grad_out_ptr: Optional[int],
                  weights_ptr: Optional[int], momentum_ptr: Optional[int],
                  lr: float, mu: float, wd: float, stream: int = 0) -> None:
    P = _count(contrib_ptrs)
    optr = None
    if order is not None:
        o = np.ascontiguousarray(order, dtype=np.int32)
        if o.size != layout.k * P:
            raise ValueError("order must hold k_colours * P entries")
        optr = o.ctypes.data_as(_i32p)
    _check(lib.mc_reduce_update(layout.handle, _ptr_table(contrib_ptrs), P, optr, grad_out_ptr,
                                weights_ptr, momentum_ptr, lr, mu, wd, stream or None), "mc_reduce_update")


def reduce_update_roles(layout: Layout, contrib_ptrs, order, n_terms, do_update,
                        grad_out_ptr: Optional[int], weights_ptr: Optional[int],
                        momentum_ptr: Optional[int], lr: float, mu: float, wd: float,
                        stream: int = 0) -> None:
    P = _count(contrib_ptrs)
    optr = None
    if order is not None:
        o = np.ascontiguousarray(order, dtype=np.int32)
        if o.size != layout.k * P:
            raise ValueError("order must hold k_colours * P entries")
        optr = o.ctypes.data_as(_i32p)
    nt = np.ascontiguousarray(n_terms, dtype=np.int32)
    du = np.ascontiguousarray(do_update, dtype=np.uint8)
    if nt.size != layout.k or du.size != layout.k:
        raise ValueError("n_terms and do_update must hold k_colours entries")
    _check(lib.mc_reduce_update_roles(layout.handle, _ptr_table(contrib_ptrs), P, optr,
                                      nt.ctypes.data_as(_i32p),
                                      du.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)),
                                      grad_out_ptr, weights_ptr, momentum_ptr, lr, mu, wd,
                                      stream or None), "mc_reduce_update_roles")


def reduce_update_range(layout: Layout, contrib_ptrs, order, grad_out_ptr: Optional[int],
                        weights_ptr: Optional[int], momentum_ptr: Optional[int],
                        lr: float, mu: float, wd: float, elem_begin: int, elem_end: int,
                        stream: int = 0, n_terms=None, do_update=None) -> None:
    P = _count(contrib_ptrs)
    optr = None
    if order is not None:
        o = np.ascontiguousarray(order, dtype=np.int32)
        if o.size != layout.k * P:
            raise ValueError("order must hold k_colours * P entries")
        optr = o.ctypes.data_as(_i32p)
    ntp = dup = None
    if n_terms is not None or do_update is not None:
        nt = np.ascontiguousarray(n_terms, dtype=np.int32)
        du = np.ascontiguousarray(do_update, dtype=np.uint8)
        if nt.size != layout.k or du.size != layout.k:
            raise ValueError("n_terms and do_update must hold k_colours entries")
        ntp, dup = nt.ctypes.data_as(_i32p), du.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8))
    _check(lib.mc_reduce_update_range(layout.handle, _ptr_table(contrib_ptrs), P, optr, ntp, dup,
                                      grad_out_ptr, weights_ptr, momentum_ptr, lr, mu, wd,
                                      elem_begin, elem_end, stream or None), "mc_reduce_update_range")


def colour_trees(n_nodes: int, k_colours: int) -> np.ndarray:
    """parent[c, r] of every node r in every colour's tree (-1 = root)."""
    out = np.empty((max(k_colours, 0), max(n_nodes, 0)), dtype=np.int32)
    _check(lib.mc_colour_trees(n_nodes, k_colours, out.ctypes.data_as(_i32p)), "mc_colour_trees")
    return out


def rank_roles(n_nodes: int, k_colours: int, rank: int):
    """(role[k], n_children[k], children[k, k]) of one rank."""
    k = max(k_colours, 0)
    role = np.empty(k, dtype=np.int32)
    cnt = np.empty(k, dtype=np.int32)
    ch = np.empty((k, k), dtype=np.int32)
    _check(lib.mc_rank_roles(n_nodes, k_colours, rank, role.ctypes.data_as(_i32p),
                             cnt.ctypes.data_as(_i32p), ch.ctypes.data_as(_i32p)), "mc_rank_roles")
    return role, cnt, ch


class TensorSet:
    """Owns one ``mc_tensor_set*`` (keeps its layout alive)."""

    def __init__(self, layout: Layout, tensor_ptrs):
        if _count(tensor_ptrs) != layout.n:
            raise ValueError("need one pointer per tensor of the layout")
        self._layout = layout
        self._h = _vp()
        _check(lib.mc_tensor_set_create(layout.handle, _ptr_table(tensor_ptrs), ctypes.byref(self._h)),
               "mc_tensor_set_create")

    @property
    def handle(self):
        return self._h

    def destroy(self) -> None:
        if self._h:
            h, self._h = self._h, _vp()
            _check(lib.mc_tensor_set_destroy(h), "mc_tensor_set_destroy")

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def tensor_set_create(layout: Layout, tensor_ptrs) -> TensorSet:
    return TensorSet(layout, tensor_ptrs)


def pack_set(layout: Layout, tensors: TensorSet, flat_ptr: Optional[int], stream: int = 0) -> None:
    _check(lib.mc_pack_set(layout.handle, tensors.handle if tensors is not None else None, flat_ptr,
                           stream or None), "mc_pack_set")


def unpack_set(layout: Layout, flat_ptr: Optional[int], tensors: TensorSet, stream: int = 0) -> None:
    _check(lib.mc_unpack_set(layout.handle, flat_ptr, tensors.handle if tensors is not None else None,
                             stream or None), "mc_unpack_set")


def set_table(sets) -> PtrTable:
    """A host array of tensor-set handles, reusable across calls (keeps the sets alive)."""
    return PtrTable([s.handle.value if s is not None else None for s in sets], keep=list(sets))


def fused_step(layout: Layout, contrib_sets, order, grad_out_ptr: Optional[int], weights: TensorSet,
               momentum: TensorSet, lr: float, mu: float, wd: float, stream: int = 0) -> None:
    tab = contrib_sets if isinstance(contrib_sets, PtrTable) else set_table(contrib_sets)
    P = tab.count
    optr = None
    if order is not None:
        o = np.ascontiguousarray(order, dtype=np.int32)
        if o.size != layout.k * P:
            raise ValueError("order must hold k_colours * P entries")
        optr = o.ctypes.data_as(_i32p)
    _check(lib.mc_fused_step(layout.handle, tab, P, optr, grad_out_ptr,
                             weights.handle if weights is not None else None,
                             momentum.handle if momentum is not None else None,
                             lr, mu, wd, stream or None), "mc_fused_step")


class UpdateSpec(ctypes.Structure):
    """mc_update_spec: immediate {lr, mu, wd} or a device pointer to them, the Nesterov flag, and
    the two choices that change how memory is walked but never a result (STATE_*, SWEEP_*)."""
    _fields_ = [("lr", ctypes.c_float), ("mu", ctypes.c_float), ("wd", ctypes.c_float),
                ("hyper_dev", ctypes.c_void_p), ("nesterov", ctypes.c_int32),
                ("state_policy", ctypes.c_int32), ("sweep", ctypes.c_int32)]


def update_spec(lr: float = 0.0, mu: float = 0.0, wd: float = 0.0, hyper_dev_ptr: Optional[int] = None,
                nesterov: int = 0, state_policy: int = STATE_DEFAULT, sweep: int = SWEEP_AUTO) -> UpdateSpec:
    return UpdateSpec(lr, mu, wd, hyper_dev_ptr, int(nesterov), int(state_policy), int(sweep))


def _order_ptr(order, k: int, P: int):
    if order is None:
        return None, None
    o = np.ascontiguousarray(order, dtype=np.int32)
    if o.size != k * P:
        raise ValueError("order must hold k_colours * P entries")
    return o, o.ctypes.data_as(_i32p)


def reduce_update_ex(layout: Layout, contrib_ptrs, order, grad_out_ptr, weights_ptr, momentum_ptr,
                     spec: UpdateSpec, stream: int = 0, n_terms=None, do_update=None,
                     elem_begin: int = 0, elem_end: int = -1) -> None:
    P = _count(contrib_ptrs)
    _o, optr = _order_ptr(order, layout.k, P)
    ntp = dup = None
    if n_terms is not None or do_update is not None:
        nt = np.ascontiguousarray(n_terms, dtype=np.int32)
        du = np.ascontiguousarray(do_update, dtype=np.uint8)
        if nt.size != layout.k or du.size != layout.k:
            raise ValueError("n_terms and do_update must hold k_colours entries")
        ntp, dup = nt.ctypes.data_as(_i32p), du.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8))
    _check(lib.mc_reduce_update_ex(layout.handle, _ptr_table(contrib_ptrs), P, optr, ntp, dup,
                                   grad_out_ptr, weights_ptr, momentum_ptr,
                                   ctypes.byref(spec) if spec is not None else None,
                                   elem_begin, elem_end, stream or None), "mc_reduce_update_ex")


def fused_step_ex(layout: Layout, contrib_sets, order, grad_out_ptr, weights: "TensorSet",
                  momentum: "TensorSet", spec: UpdateSpec, stream: int = 0, n_terms=None,
                  do_update=None) -> None:
    tab = contrib_sets if isinstance(contrib_sets, PtrTable) else set_table(contrib_sets)
    _o, optr = _order_ptr(order, layout.k, tab.count)
    ntp = dup = None
    if n_terms is not None or do_update is not None:
        nt = np.ascontiguousarray(n_terms, dtype=np.int32)
        du = np.ascontiguousarray(do_update, dtype=np.uint8)
        if nt.size != layout.k or du.size != layout.k:
            raise ValueError("n_terms and do_update must hold k_colours entries")
        ntp, dup = nt.ctypes.data_as(_i32p), du.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8))
    _check(lib.mc_fused_step_ex(layout.handle, tab, tab.count, optr, ntp, dup, grad_out_ptr,
                                weights.handle if weights is not None else None,
                                momentum.handle if momentum is not None else None,
                                ctypes.byref(spec) if spec is not None else None, stream or None),
           "mc_fused_step_ex")


def packets_reset(ready_ptr: Optional[int], n_packets: int, progress_ptr: Optional[int], n_blocks: int,
                  stream: int = 0) -> None:
    _check(lib.mc_packets_reset(ready_ptr, n_packets, progress_ptr, n_blocks, stream or None), "mc_packets_reset")


def packet_signal(ready_ptr: Optional[int], packet: int, value: int, stream: int = 0) -> None:
    _check(lib.mc_packet_signal(ready_ptr, packet, value, stream or None), "mc_packet_signal")


def packet_deliver(dst_ptr: Optional[int], src_ptr: Optional[int], n_elems: int, flag_ptr: Optional[int],
                   stream: int = 0) -> None:
    _check(lib.mc_packet_deliver(dst_ptr, src_ptr, n_elems, flag_ptr, stream or None), "mc_packet_deliver")


def delay(microseconds: int, stream: int = 0) -> None:
    _check(lib.mc_delay(microseconds, stream or None), "mc_delay")


def reduce_update_packets(layout: Layout, contrib_ptrs, order, grad_out_ptr, weights_ptr, momentum_ptr,
                          spec: UpdateSpec, packets_ptr: Optional[int], n_packets: int, ready_ptr: Optional[int],
                          arrivals: int, spin_limit: int, progress_ptr: Optional[int], n_blocks: int,
                          stream: int = 0) -> None:
    P = _count(contrib_ptrs)
    _o, optr = _order_ptr(order, layout.k, P)
    _check(lib.mc_reduce_update_packets(layout.handle, _ptr_table(contrib_ptrs), P, optr, grad_out_ptr,
                                        weights_ptr, momentum_ptr,
                                        ctypes.byref(spec) if spec is not None else None,
                                        packets_ptr, n_packets, ready_ptr, arrivals, spin_limit,
                                        progress_ptr, n_blocks, stream or None), "mc_reduce_update_packets")


def hyper_write(hyper_dev_ptr: Optional[int], lr: float, mu: float, wd: float, stream: int = 0) -> None:
    _check(lib.mc_hyper_write(hyper_dev_ptr, lr, mu, wd, stream or None), "mc_hyper_write")


def lr_schedule(base_lr: float, batch_per_gpu: int, n_workers: int, warmup_epochs: float,
                drop_every_epochs: float, epoch: float) -> float:
    out = ctypes.c_float()
    _check(lib.mc_lr_schedule(base_lr, batch_per_gpu, n_workers, warmup_epochs, drop_every_epochs,
                              epoch, ctypes.byref(out)), "mc_lr_schedule")
    return out.value


def copy(dst_ptr: Optional[int], src_ptr: Optional[int], n_bytes: int, stream: int = 0) -> None:
    _check(lib.mc_copy(dst_ptr, src_ptr, n_bytes, stream or None), "mc_copy")


def set_option(option: int, value: int) -> None:
    _check(lib.mc_set_option(option, value), "mc_set_option")


def get_option(option: int) -> int:
    v = ctypes.c_int()
    _check(lib.mc_get_option(option, ctypes.byref(v)), "mc_get_option")
    return v.value


def strerror(code: int) -> str:
    return lib.mc_strerror(code).decode()
