"""Arrival-order model of a multipath transport: spray, reorder, retransmit.

Stands in for the paper's network: the sender sprays chunks of one connection over
many paths (Section 3.2, 256 paths per connection; Section 4.1, random spraying),
each path delivers in FIFO order, paths interleave arbitrarily, and a chunk that
was only delayed may be retransmitted (Section 3.2, fast / timeout retransmission),
which is where duplicates come from.  In-flight data is bounded (Section 5, maximum
congestion window), modelled as a reorder window W.

Only integer bookkeeping lives here; payload bytes are never touched.
"""
from collections import deque

import numpy as np

from .payload import rng


def gen_arrivals(seed: int, n: int, paths: int, window=None, dup: float = 0.0, stream: int = 0):
    """Arrival sequence for a phase whose logical chunks are seq 0..n-1.

    Sender, in seq order: each chunk goes on a uniformly random path.  With
    probability ``dup`` a byte-identical retransmission is scheduled: once seq
    ``min(s + 1 + U{0..W-1}, n-1)`` has been sent, copy 1 of ``s`` is sent on a
    different path (when there is more than one).

    Receiver: ``base`` = lowest seq of which no copy has been delivered.  A path is
    eligible when its FIFO head has ``seq < base + W``.  One eligible path is chosen
    uniformly, its head is delivered.  The FIFO holding ``base``'s original only has
    earlier-sent (hence eligible) entries ahead of it, so delivery always progresses.

    Returns ``(seq, copy, path)`` int64 arrays in arrival order; every seq appears
    once or twice.
    """
    n = int(n)
    P = int(paths)
    W = n if window is None else int(window)
    W = max(W, 1)
    if n == 0:
        z = np.zeros(0, dtype=np.int64)
        return z, z.copy(), z.copy()
    g = rng(seed, 0xA5510000 + stream)
    path0 = g.integers(0, P, n)
    is_dup = g.random(n) < dup
    delay = g.integers(0, W, n)
    hop = g.integers(1, P, n) if P > 1 else np.zeros(n, dtype=np.int64)

    fifos = [deque() for _ in range(P)]
    pending = {}
    for s in range(n):
        fifos[path0[s]].append((s, 0))
        if is_dup[s]:
            pending.setdefault(min(s + 1 + int(delay[s]), n - 1), []).append(s)
        for s2 in pending.pop(s, ()):
            fifos[(path0[s2] + hop[s2]) % P].append((s2, 1))
    assert not pending
    total = n + int(is_dup.sum())

    big = np.iinfo(np.int64).max
    head = np.array([f[0][0] if f else big for f in fifos], dtype=np.int64)
    delivered = np.zeros(n, dtype=bool)
    base = 0
    pick = g.random(total)
    seq = np.empty(total, dtype=np.int64)
    cpy = np.empty(total, dtype=np.int64)
    pth = np.empty(total, dtype=np.int64)
    for k in range(total):
        elig = np.flatnonzero(head < base + W)
        p = int(elig[int(pick[k] * len(elig))])
        s, c = fifos[p].popleft()
        head[p] = fifos[p][0][0] if fifos[p] else big
        seq[k], cpy[k], pth[k] = s, c, p
        delivered[s] = True
        while base < n and delivered[base]:
            base += 1
    assert base == n and all(not f for f in fifos)
    return seq, cpy, pth


def identity_arrivals(n: int):
    """In-order, duplicate-free arrival (the degenerate single-path case)."""
    seq = np.arange(int(n), dtype=np.int64)
    return seq, np.zeros_like(seq), np.zeros_like(seq)


def merge_streams(seed: int, lengths, stream: int = 0) -> np.ndarray:
    """Seeded uniform interleave of several independent arrival streams.

    Returns an int64 array of stream ids, one per merged arrival, in which stream
    ``i`` occurs ``lengths[i]`` times and each stream's own order is preserved by
    the caller consuming its items front to back.  Every interleaving that keeps
    the per-stream orders is equally likely (a uniformly shuffled multiset).
    """
    ids = np.repeat(np.arange(len(lengths), dtype=np.int64), np.asarray(lengths, dtype=np.int64))
    rng(seed, 0xA5520000 + stream).shuffle(ids)
    return ids
