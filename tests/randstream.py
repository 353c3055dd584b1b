"""Random small record streams with every feature mixed: odd lengths, zero lengths, duplicates
(adjacent and far), forwarding / no forwarding / forward-only, scattered non-overlapping
destinations.  Used by the brute-force pin of the oracle and by the GPU fuzz test."""
import numpy as np

from synth import payload as pl
from synth.layout import DESC, NO_FORWARD, FORWARD_ONLY, ELEM_SIZE, COPY


def random_stream(seed, dtype, op, max_chunks=40, max_len=5000):
    g = pl.rng(seed, 0xF022)
    es = ELEM_SIZE[dtype]
    n = int(g.integers(1, max_chunks + 1))
    lens = g.integers(0, max_len // es + 1, n) * es
    lens[g.random(n) < 0.1] = 0
    m = g.random(n) < 0.2                          # some lengths are whole 16-byte vectors
    lens[m] = np.minimum(g.integers(1, 40, n)[m] * 16, max(16, max_len // 16 * 16))
    pitch = ((int(lens.max()) + 15) // 16 + 1) * 16
    dst_slot = g.permutation(n + 3)[:n]            # scattered, with gaps
    out_slot = g.permutation(n + 2)[:n]
    kind = g.integers(0, 3, n)                     # 0 keep only, 1 forward, 2 forward-only
    if op == COPY:
        kind = np.minimum(kind, 1)                 # a relay of a copy is allowed too, keep it simpler
    copies = 1 + (g.random(n) < 0.35) * g.integers(1, 4, n)
    arr = np.repeat(np.arange(n), copies)
    arr = arr[g.permutation(len(arr))] if g.random() < 0.8 else arr   # sometimes adjacent duplicates
    d = np.zeros(len(arr), dtype=DESC)
    d["src_off"] = np.arange(len(arr), dtype=np.uint64) * pitch
    d["dst_off"] = dst_slot[arr].astype(np.uint64) * pitch
    off = out_slot[arr].astype(np.uint64) * pitch
    d["out_off"] = np.where(kind[arr] == 0, NO_FORWARD, np.where(kind[arr] == 2, off | FORWARD_ONLY, off))
    d["len"] = lens[arr]
    d["seq"] = arr
    nel = lambda slots: slots * pitch // es
    draw = {0: lambda s, k: pl.uniform_f32(seed, s, k) * 4, 1: lambda s, k: pl.normal_bf16(seed, s, k),
            2: lambda s, k: pl.uniform_f16(seed, s, k, 8.0),
            3: lambda s, k: pl.uniform_i32(seed, s, k)}[dtype]
    uniq = draw(1, nel(n)).reshape(n, -1)
    recv = uniq[arr].reshape(-1).copy()
    acc = draw(2, nel(n + 3))
    return dict(descs=d, recv=recv, acc=acc, out_bytes=(n + 2) * pitch, n_bits=n, dtype=dtype, op=op)
