"""Tiny pure-Python re-derivations used to pin the C oracle (exact rationals, brute force).

Nothing here is used by the product or by the oracle itself; these are independent second
opinions for small inputs only.
"""
from fractions import Fraction

import numpy as np

EMPTY = 0xFFFFFFFF


def encode_exact(x):
    """Sec. 3.1 encoding with exact rational arithmetic.  x: 1-D float32 -> (pos bits, strong bits)."""
    x = np.asarray(x, dtype=np.float32)
    fr = [Fraction(float(v)) for v in x]          # float32 -> exact rational
    tau = sum(abs(f) for f in fr) / len(fr)
    pos = [1 if f > 0 else 0 for f in fr]
    strong = [1 if abs(f) > tau else 0 for f in fr]
    return pos, strong


def pack(pos, strong):
    d = len(pos)
    W = (d + 63) // 64
    code = [0] * (2 * W)
    for i in range(d):
        if pos[i]:
            code[i // 64] |= 1 << (i % 64)
        if strong[i]:
            code[W + i // 64] |= 1 << (i % 64)
    return np.array(code, dtype=np.uint64)


def unpack(code, d):
    W = (d + 63) // 64
    code = [int(c) for c in code]
    pos = [(code[i // 64] >> (i % 64)) & 1 for i in range(d)]
    strong = [(code[W + i // 64] >> (i % 64)) & 1 for i in range(d)]
    return pos, strong


def signed_levels(code, d):
    """Signed level vector: +-(1 + strong)."""
    pos, strong = unpack(code, d)
    return np.array([(1 + s) * (1 if p else -1) for p, s in zip(pos, strong)], dtype=np.int64)


def distance_by_levels(ca, cb, d):
    """d(a,b) = (<|a|,|b|> - <a,b>) / 2 on signed levels: differing signs contribute the product of levels."""
    a = signed_levels(ca, d)
    b = signed_levels(cb, d)
    num = int(np.dot(np.abs(a), np.abs(b)) - np.dot(a, b))
    assert num % 2 == 0
    return num // 2


def popcount_forms(ca, cb, d):
    """The two word-level forms a fast implementation may use; returns both values."""
    W = (d + 63) // 64
    ca = [int(c) for c in ca]
    cb = [int(c) for c in cb]
    f1 = f2 = 0
    for w in range(W):
        X = ca[w] ^ cb[w]
        sa, sb = ca[W + w], cb[W + w]
        pc = lambda v: bin(v).count("1")
        f1 += pc(X) + pc(X & (sa | sb)) + 2 * pc(X & sa & sb)
        f2 += pc(X) + pc(X & sa) + pc(X & sb) + pc(X & sa & sb)
    return f1, f2


def bfs_reachable(adj, entry):
    seen = {int(entry)}
    frontier = [int(entry)]
    while frontier:
        nxt = []
        for u in frontier:
            for v in adj[u]:
                v = int(v)
                if v != EMPTY and v not in seen:
                    seen.add(v)
                    nxt.append(v)
        frontier = nxt
    return seen
