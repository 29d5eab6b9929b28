"""Hand-crafted inputs shared by the CPU pins and the GPU parity tests (inputs only, no arithmetic of the method)."""
from __future__ import annotations

import numpy as np


def batch_starts(n_min: int, bs_min: int):
    """First batch boundary of the batch-synchronous construction (batches of max(1, done // 50) nodes)
    at or after n_min whose batch holds at least bs_min nodes.  Returns (done, batch size)."""
    done = 0
    while True:
        bs = max(1, done // 50)
        if done >= n_min and bs >= bs_min:
            return done, bs
        done += bs


def hub_crowd_codes(seed: int = 11, d: int = 128):
    """Sign-Magnitude codes for the hub-cap case of the construction.

    n0 ordinary nodes with random codes (node 0 = the hub, which is also the entry node), then one whole batch:
      * 191 nodes "A": the hub's code with the same 10 weak sign bits flipped, plus one or two more weak sign
        flips of their own -> distance 11 or 12 to the hub, at most 4 to each other;
      * 5 nodes "B1..B5": the hub's code with 4, 5, 6, 7, 8 strong sign bits flipped (disjoint sets) ->
        distance 16, 20, 24, 28, 32 to the hub, and far from every A and from each other.
    Every new node's nearest node is the hub, so all 196 select it in the same batch; by (distance, id) the
    hub's new in-edge candidates are the 191 A's, then B1 (rank 192), B2 (rank 193), ...
    Returns (codes [n][4] uint64, n0, ids of A, ids of B).
    """
    rng = np.random.default_rng(seed)
    W = d // 64
    n0, bs = batch_starts(9_800, 196)
    codes = rng.integers(0, 2 ** 63, size=(n0, 2 * W), dtype=np.uint64) * np.uint64(2) + \
        rng.integers(0, 2, size=(n0, 2 * W), dtype=np.uint64)
    # magnitude plane with ~42 % strong bits, like encoded Gaussian data
    strong = rng.random((n0, d)) < 0.42
    for w in range(W):
        word = np.zeros(n0, dtype=np.uint64)
        for b in range(64):
            word |= strong[:, 64 * w + b].astype(np.uint64) << np.uint64(b)
        codes[:, W + w] = word
    hub = codes[0].copy()
    is_strong = [(int(hub[W + i // 64]) >> (i % 64)) & 1 for i in range(d)]
    weak = [i for i in range(d) if not is_strong[i]]
    strong_dims = [i for i in range(d) if is_strong[i]]
    assert len(weak) >= 40 and len(strong_dims) >= 30

    def flipped(dims):
        c = hub.copy()
        for i in dims:
            c[i // 64] ^= np.uint64(1) << np.uint64(i % 64)
        return c

    common, rest = weak[:10], weak[10:]
    own = [(a,) for a in rest] + [(a, b) for ai, a in enumerate(rest) for b in rest[ai + 1:]]
    own = [own[i] for i in rng.permutation(len(own))[:191]]
    A = [flipped(common + list(o)) for o in own]
    B, at = [], 0
    for cnt in (4, 5, 6, 7, 8):
        B.append(flipped(strong_dims[at:at + cnt]))
        at += cnt
    crowd = A + B
    order = rng.permutation(len(crowd))          # ids must not follow the distance order
    crowd = [crowd[i] for i in order]
    ids = {int(src): n0 + pos for pos, src in enumerate(order)}
    all_codes = np.concatenate([codes, np.stack(crowd)])
    assert len(crowd) <= bs
    return all_codes, n0, [ids[i] for i in range(191)], [ids[191 + j] for j in range(5)]
