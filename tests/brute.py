"""Brute-force, per-element re-statement of the step for TINY inputs (pure Python).

A pin for the C oracle, written to share nothing with it: no offsets table (tensors are
walked with a running counter), the colour of a flat index is found by scanning chunk
by chunk, and binary32 rounding is done by packing a Python float (binary64) into 4
bytes.  For +, - and * of two binary32 values, rounding the binary64 result to binary32
equals the correctly rounded binary32 operation (53 >= 2*24+2), so this is exact
binary32 arithmetic by a different mechanism than C's float type.

Follows Section 3, Algorithm 1 (sum of all contributions, then SGD) and Section 4.2
(payload cut into k chunks that are summed independently).
"""
import struct


def f32(x: float) -> float:
    """Round a Python float to the nearest binary32 (ties to even), returned as a float."""
    return struct.unpack("<f", struct.pack("<f", x))[0]


def bits(x: float) -> int:
    return struct.unpack("<I", struct.pack("<f", x))[0]


def chunk_len(N: int, k: int, align: int = 256) -> int:
    """Smallest multiple of `align` whose k-fold covers N (found by search, not by formula)."""
    c = 0
    while c * k < N:
        c += align
    return c


def colour_of(i: int, N: int, k: int) -> int:
    c_len = chunk_len(N, k)
    c, start = 0, 0
    while not (start <= i < start + c_len):
        start += c_len
        c += 1
    assert c < k
    return c


def pack(tensors):
    flat = []
    for t in tensors:
        for val in t:
            flat.append(val)
    return flat


def unpack(flat, sizes):
    out, cursor = [], 0
    for n in sizes:
        cur = []
        for _ in range(n):
            cur.append(flat[cursor])
            cursor += 1
        out.append(cur)
    assert cursor == len(flat)
    return out


def step(contrib_flat, w, v, k, lr, mu, wd, order=None):
    """contrib_flat: list of P lists (binary32-representable floats).  Returns (g, w', v')."""
    P = len(contrib_flat)
    N = len(w)
    lr, mu, wd = f32(lr), f32(mu), f32(wd)
    g, wn, vn = [], [], []
    for i in range(N):
        c = colour_of(i, N, k)
        seq = list(range(P)) if order is None else [int(s) for s in order[c]]
        acc = contrib_flat[seq[0]][i]
        for q in seq[1:]:
            acc = f32(acc + contrib_flat[q][i])
        d = f32(acc + f32(wd * w[i]))
        vv = f32(f32(mu * v[i]) + d)
        ww = f32(w[i] - f32(lr * vv))
        g.append(acc)
        vn.append(vv)
        wn.append(ww)
    return g, wn, vn
