"""Do the pins bite?  Plant plausible mistakes in (wrappers around) the CPU oracle and
demand that at least one pin fails for each.  Everything here runs on the CPU."""
import types

import numpy as np
import pytest

import oracle
import pins


def _mutant(**overrides):
    m = types.SimpleNamespace(Layout=oracle.Layout, pack=oracle.pack, unpack=oracle.unpack,
                              reduce_update=oracle.reduce_update,
                              reduce_update_colour=oracle.reduce_update_colour)
    for k, f in overrides.items():
        setattr(m, k, f)
    return m


def _caught(impl):
    failed = []
    for chk in pins.ALL_CHECKS:
        try:
            chk(impl)
        except Exception:                       # AssertionError or anything the mutant breaks
            failed.append(chk.__name__)
    return failed


# ---- mutants of the reduction ---------------------------------------------------------
def _drop_last_term(L, xs, w, v, lr, mu, wd, order=None, want_g=True):
    if len(xs) > 2:
        P = len(xs) - 1
        o = None if order is None else np.array([[q for q in row if q != P] for row in order], np.int32)
        return oracle.reduce_update(L, xs[:-1], w, v, lr, mu, wd, order=o, want_g=want_g)
    return oracle.reduce_update(L, xs, w, v, lr, mu, wd, order=order, want_g=want_g)


def _ignore_order(L, xs, w, v, lr, mu, wd, order=None, want_g=True):
    return oracle.reduce_update(L, xs, w, v, lr, mu, wd, order=None, want_g=want_g)


def _order_shifted_by_one_colour(L, xs, w, v, lr, mu, wd, order=None, want_g=True):
    if order is not None:
        order = np.roll(np.asarray(order), 1, axis=0)
    return oracle.reduce_update(L, xs, w, v, lr, mu, wd, order=order, want_g=want_g)


def _reversed_sequence(L, xs, w, v, lr, mu, wd, order=None, want_g=True):
    P = len(xs)
    o = np.tile(np.arange(P, dtype=np.int32), (L.k, 1)) if order is None else np.asarray(order)
    return oracle.reduce_update(L, xs, w, v, lr, mu, wd, order=o[:, ::-1], want_g=want_g)


def _start_from_zero(L, xs, w, v, lr, mu, wd, order=None, want_g=True):
    # accumulate from +0.0 instead of from the first term
    z = np.zeros(L.N, dtype=np.float32)
    P = len(xs)
    o = np.tile(np.arange(P, dtype=np.int32), (L.k, 1)) if order is None else np.asarray(order)
    o2 = np.concatenate([np.full((L.k, 1), P, np.int32), o.astype(np.int32)], axis=1)
    return oracle.reduce_update(L, list(xs) + [z], w, v, lr, mu, wd, order=o2, want_g=want_g)


def _pairwise_sum(L, xs, w, v, lr, mu, wd, order=None, want_g=True):
    # (x0+x1) + (x2+x3) instead of strict left to right, when there are exactly 4 terms
    if len(xs) == 4 and order is None:
        a = xs[0] + xs[1]
        b = xs[2] + xs[3]
        return oracle.reduce_update(L, [a, b], w, v, lr, mu, wd, want_g=want_g)
    return oracle.reduce_update(L, xs, w, v, lr, mu, wd, order=order, want_g=want_g)


def _float64_accumulate(L, xs, w, v, lr, mu, wd, order=None, want_g=True):
    g = oracle.reduce_update(L, xs, w.copy(), v.copy(), lr, mu, wd, order=order, want_g=True)
    acc = np.zeros(L.N, np.float64)
    for x in xs:
        acc += x
    g64 = acc.astype(np.float32)
    oracle.reduce_update(L, [g64], w, v, lr, mu, wd)
    return g64 if want_g else None


# ---- mutants of the update ------------------------------------------------------------
def _no_weight_decay(L, xs, w, v, lr, mu, wd, order=None, want_g=True):
    return oracle.reduce_update(L, xs, w, v, lr, mu, 0.0, order=order, want_g=want_g)


def _ascent(L, xs, w, v, lr, mu, wd, order=None, want_g=True):
    return oracle.reduce_update(L, xs, w, v, -lr, mu, wd, order=order, want_g=want_g)


def _decay_sign(L, xs, w, v, lr, mu, wd, order=None, want_g=True):
    return oracle.reduce_update(L, xs, w, v, lr, mu, -wd, order=order, want_g=want_g)


def _no_momentum(L, xs, w, v, lr, mu, wd, order=None, want_g=True):
    return oracle.reduce_update(L, xs, w, v, lr, 0.0, wd, order=order, want_g=want_g)


def _dampened(L, xs, w, v, lr, mu, wd, order=None, want_g=True):
    # v' = mu*v + (1-mu)*d  (dampening = mu) instead of dampening 0
    v_old = v.copy()
    g = oracle.reduce_update(L, xs, w, v, lr, mu, wd, order=order, want_g=True)
    d = v - np.float32(mu) * v_old
    v[:] = np.float32(mu) * v_old + np.float32(1 - mu) * d
    return g if want_g else None


def _update_uses_old_momentum(L, xs, w, v, lr, mu, wd, order=None, want_g=True):
    # w' = w - lr*v_old instead of lr*v'
    w_old, v_old = w.copy(), v.copy()
    g = oracle.reduce_update(L, xs, w, v, lr, mu, wd, order=order, want_g=True)
    w[:] = w_old - np.float32(lr) * v_old
    return g if want_g else None


def _swap_mu_lr(L, xs, w, v, lr, mu, wd, order=None, want_g=True):
    return oracle.reduce_update(L, xs, w, v, mu, lr, wd, order=order, want_g=want_g)


# ---- mutants of layout / pack ---------------------------------------------------------
class _UnalignedLayout(oracle.Layout):
    def __init__(self, numel, k):
        super().__init__(numel, k)
        N = self.N
        c = -(-N // k) if k > 0 else 0
        self.bounds = np.array([min(N, i * c) for i in range(k + 1)], dtype=np.int64)


class _FloorChunkLayout(oracle.Layout):
    def __init__(self, numel, k):
        super().__init__(numel, k)
        N = self.N
        c = (N // k + 255) // 256 * 256
        self.bounds = np.array([min(N, i * c) for i in range(k)] + [N], dtype=np.int64)


def _pack_reversed_tensors(L, tensors):
    flat = oracle.pack(L, tensors)
    if L.n >= 2 and L.off[1] - L.off[0] == L.off[2] - L.off[1] and L.off[1] > 0:
        return flat
    # swap the first two tensors' places when both are non-empty
    s0, s1 = int(L.off[1] - L.off[0]), int(L.off[2] - L.off[1]) if L.n >= 2 else 0
    if s0 and s1:
        out = flat.copy()
        out[:s1] = flat[s0:s0 + s1]
        out[s1:s0 + s1] = flat[:s0]
        return out
    return flat


def _pack_float_roundtrip(L, tensors):
    # moving words as floating-point VALUES through a wider type quiets signalling NaNs /
    # loses payloads on some paths; emulate with a value-level pass that normalises NaNs
    flat = oracle.pack(L, tensors)
    out = flat.copy()
    out[np.isnan(out)] = np.float32(np.nan)
    return out


def _unpack_off_by_one(L, flat):
    outs = oracle.unpack(L, flat)
    if L.n >= 2 and outs[1].size and outs[0].size:
        outs[1] = outs[1].copy()
        outs[1][0] = outs[0][-1]
    return outs


MUTANTS = {
    "drop_last_term": _mutant(reduce_update=_drop_last_term),
    "ignore_order": _mutant(reduce_update=_ignore_order),
    "order_rows_shifted": _mutant(reduce_update=_order_shifted_by_one_colour),
    "reversed_sequence": _mutant(reduce_update=_reversed_sequence),
    "start_from_zero": _mutant(reduce_update=_start_from_zero),
    "pairwise_sum": _mutant(reduce_update=_pairwise_sum),
    "float64_accumulate": _mutant(reduce_update=_float64_accumulate),
    "no_weight_decay": _mutant(reduce_update=_no_weight_decay),
    "ascent": _mutant(reduce_update=_ascent),
    "decay_sign": _mutant(reduce_update=_decay_sign),
    "no_momentum": _mutant(reduce_update=_no_momentum),
    "dampened": _mutant(reduce_update=_dampened),
    "update_uses_old_momentum": _mutant(reduce_update=_update_uses_old_momentum),
    "swap_mu_lr": _mutant(reduce_update=_swap_mu_lr),
    "unaligned_chunks": _mutant(Layout=_UnalignedLayout),
    "floor_chunks": _mutant(Layout=_FloorChunkLayout),
    "pack_swaps_tensors": _mutant(pack=_pack_reversed_tensors),
    "pack_as_values": _mutant(pack=_pack_float_roundtrip),
    "unpack_off_by_one": _mutant(unpack=_unpack_off_by_one),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_mutant_is_caught(name):
    failed = _caught(MUTANTS[name])
    assert failed, f"no pin noticed the planted mistake '{name}'"


def test_unmutated_passes_everything():
    assert _caught(_mutant()) == []
