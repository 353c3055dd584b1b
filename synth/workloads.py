"""Synthetic receive-side workloads: one rank's share of a multipath collective.

A workload is what the (simulated) control path would hand the GPU: a receive
staging pool filled in ARRIVAL order, and per phase a list of 32-byte records
(synth.layout.DESC) saying where each arrival belongs.  Shapes follow the paper's
evaluation sweeps (1 MB-1 GB messages, 32 KB default chunks, 16 KB minimum, 4 KB
MTU, 256 paths per connection: Sections 3.2, 3.3, 6 and Table 1); the chunk streams
themselves are seeded stand-ins for the NCCL-tests / RCCL-tests traffic the paper
measured on, none of which is reproduced here.

Ring schedule (standard ring allreduce, rank r of R, segment j = j-th R-th of the
message): reduce-scatter step s receives segment (r-s-1) mod R and combines it
into the local accumulator; allgather step s receives the fully reduced segment
(r-s) mod R and overwrites.  What a step produces is what the rank sends in the
next step, so it is also written to the outbound staging buffer, except for the
very last step.  This module only lays out offsets and copies payload bytes; it
never combines two payload values.
"""
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

from . import payload as pl
from .arrivals import gen_arrivals, identity_arrivals, merge_streams
from .layout import (DESC, GATHER_DESC, MAX_SOURCES, NO_FORWARD, FORWARD_ONLY, ELEM_SIZE, SUM, COPY, F32, BF16,
                     F16, I32)

LOGICAL = np.dtype([("seq", "<u4"), ("dst_off", "<u8"), ("out_off", "<u8"), ("len", "<u4")])


@dataclass
class Phase:
    name: str
    op: int
    descs: np.ndarray            # DESC records in arrival order
    n_unique: int                # distinct seqs in descs
    payload_bytes: int           # sum of len over distinct seqs
    algo_bytes: int              # algorithmic HBM bytes (single pass byte model)


@dataclass
class Workload:
    name: str
    dtype: int
    acc: np.ndarray              # initial accumulator (fp32, or uint16 bf16 bit patterns)
    recv_stage: np.ndarray       # arrival-order slot pool, same storage dtype
    out_bytes: int               # size of the outbound staging buffer (0 = none)
    n_bits: int                  # dedup bitmap size in bits
    phases: List[Phase] = field(default_factory=list)
    note: str = ""
    extra: dict = field(default_factory=dict)  # builder-specific facts tests may assert on

    @property
    def es(self) -> int:
        return ELEM_SIZE[self.dtype]


def byte_model(op: int, logical: np.ndarray, n_arrivals: int) -> int:
    """Algorithmic HBM bytes: reduce reads src+acc, copy reads src; every unique
    chunk writes acc and, when it forwards, the staging copy; every arrival costs
    its 32-byte record and one 4-byte bitmap word update."""
    ln = logical["len"].astype(np.int64)
    fwd = logical["out_off"] != NO_FORWARD
    relay = fwd & ((logical["out_off"] & FORWARD_ONLY) != 0)  # forwarded but not written back
    reads = ln if op == COPY else 2 * ln
    writes = np.where(relay, 0, ln) + np.where(fwd, ln, 0)
    return int(reads.sum() + writes.sum()) + 36 * int(n_arrivals)


def ring_logical(R: int, M: int, C: int, rank: int = 0, allgather: bool = True,
                 forward_last_rs: Optional[bool] = None, seq_base: int = 0,
                 acc_base: int = 0, out_base: int = 0, relay: bool = False):
    """Logical chunks one rank receives in a ring allreduce (or reduce-scatter).

    Returns (rs, ag, n_out_chunks): LOGICAL arrays in sender order.  Sequence
    numbers run step-major over both phases; forwarded chunks get consecutive
    C-byte slots of the staging buffer.  ``forward_last_rs`` defaults to
    ``allgather`` (an allreduce sends the finished segment on; a bare
    reduce-scatter keeps it).  With ``relay`` the intermediate reduce-scatter steps
    (all but the last) carry the forward-only flag: their partial sums are needed by
    the next rank only and are not written back to the accumulator.
    """
    assert M % R == 0
    if forward_last_rs is None:
        forward_last_rs = allgather
    S = M // R
    cps = -(-S // C)
    n_out = 0

    def build(steps, seg_of, fwd_of, seq0, relay_of=lambda s: False):
        nonlocal n_out
        rec = np.zeros(steps * cps, dtype=LOGICAL)
        k = 0
        for s in range(steps):
            seg = seg_of(s) % R
            for c in range(cps):
                ln = min(C, S - c * C)
                rec[k]["seq"] = seq0 + s * cps + c
                rec[k]["dst_off"] = acc_base + seg * S + c * C
                rec[k]["len"] = ln
                if fwd_of(s):
                    rec[k]["out_off"] = np.uint64(out_base + n_out * C) | (FORWARD_ONLY if relay_of(s) else np.uint64(0))
                    n_out += 1
                else:
                    rec[k]["out_off"] = NO_FORWARD
                k += 1
        return rec

    rs = build(R - 1, lambda s: rank - s - 1, lambda s: s < R - 2 or forward_last_rs, seq_base,
               lambda s: relay and s < R - 2)
    if allgather:
        ag = build(R - 1, lambda s: rank - s, lambda s: s < R - 2, seq_base + (R - 1) * cps)
    else:
        ag = np.zeros(0, dtype=LOGICAL)
    return rs, ag, n_out


def materialize(logical: np.ndarray, arr_idx: np.ndarray, slot0: int, slot_bytes: int) -> np.ndarray:
    """DESC records in arrival order: arrival k (index arr_idx[k] into ``logical``)
    occupies receive slot slot0 + k."""
    d = np.zeros(len(arr_idx), dtype=DESC)
    lg = logical[arr_idx]
    d["src_off"] = (slot0 + np.arange(len(arr_idx), dtype=np.uint64)) * np.uint64(slot_bytes)
    d["dst_off"] = lg["dst_off"]
    d["out_off"] = lg["out_off"]
    d["len"] = lg["len"]
    d["seq"] = lg["seq"]
    return d


def fill_slots(recv_stage: np.ndarray, unique_payload: np.ndarray, arr_idx: np.ndarray, slot0: int):
    """Copy logical chunk arr_idx[k]'s payload into slot slot0 + k (duplicates are
    byte-identical copies in slots of their own)."""
    per = unique_payload.shape[1]
    view = recv_stage.reshape(-1, per)
    blk = 2048
    for lo in range(0, len(arr_idx), blk):
        hi = min(len(arr_idx), lo + blk)
        view[slot0 + lo: slot0 + hi] = unique_payload[arr_idx[lo:hi]]


def _draw(dist: str, dtype: int, seed: int, stream: int, n: int) -> np.ndarray:
    if dist == "uniform":
        if dtype == F16:
            return pl.uniform_f16(seed, stream, n, 4.0)
        if dtype == I32:
            return pl.uniform_i32(seed, stream, n)
        return pl.uniform_f32(seed, stream, n) if dtype == F32 else pl.uniform_bf16(seed, stream, n)
    if dist == "normal":
        assert dtype == BF16
        return pl.normal_bf16(seed, stream, n)
    if dist == "ones":
        return pl.ints_as(np.ones(n, dtype=np.int64), dtype)
    if dist == "smallint":
        return pl.ints_as(pl.small_int(seed, stream, n), dtype)
    raise ValueError(dist)


def ring_share(name: str, seed: int, R: int, M: int, C: int, dtype: int, paths: int,
               window, dup: float, dist: str, allgather: bool = True, op: int = SUM,
               identity: bool = False, arrival_seed=None, arrivals=None, relay: bool = False) -> Workload:
    """One rank's receive share of a ring allreduce (allgather=True) or ring
    reduce-scatter, with i.i.d. payload values from ``dist``.

    Payload values depend on ``seed`` only; the arrival order depends on
    ``arrival_seed`` (default: ``seed``), or is given outright as ``arrivals`` (one
    index array per phase, each logical chunk at least once), so the same logical
    stream can be replayed under different interleavings."""
    es = ELEM_SIZE[dtype]
    assert C % 16 == 0 and (M // R) % es == 0
    rs, ag, n_out = ring_logical(R, M, C, allgather=allgather, relay=relay)
    acc = _draw(dist, dtype, seed, 1, M // es)
    phases_l = [("reduce-scatter", op, rs)] + ([("allgather", COPY, ag)] if allgather else [])
    arrs = []
    for i, (_, _, lg) in enumerate(phases_l):
        if arrivals is not None:
            a = np.asarray(arrivals[i], dtype=np.int64)
        elif identity:
            a = identity_arrivals(len(lg))[0]
        else:
            a = gen_arrivals(seed if arrival_seed is None else arrival_seed, len(lg), paths,
                             window, dup, stream=i)[0]
        arrs.append(a)
    n_slots = sum(len(a) for a in arrs)
    recv = np.zeros(n_slots * (C // es), dtype=pl.np_dtype(dtype))
    phases, slot0 = [], 0
    for i, ((pname, pop, lg), a) in enumerate(zip(phases_l, arrs)):
        uniq = _draw(dist, dtype, seed, 10 + i, len(lg) * (C // es)).reshape(len(lg), C // es)
        fill_slots(recv, uniq, a, slot0)
        del uniq
        d = materialize(lg, a, slot0, C)
        phases.append(Phase(pname, pop, d, len(lg), int(lg["len"].astype(np.int64).sum()),
                            byte_model(pop, lg, len(a))))
        slot0 += len(a)
    n_bits = len(rs) + len(ag)
    w = Workload(name, dtype, acc, recv, n_out * C, n_bits, phases,
                 note=f"R={R} M={M} C={C} paths={paths} window={window} dup={dup} dist={dist}")
    w.extra["logical"] = [lg for (_, _, lg) in phases_l]
    w.extra["arrivals"] = arrs
    return w


def two_pass_records(w: Workload, arrival_bytes: int, group: int = 1):
    """The paper's literal form of the receive path (Section 3.1): first a scattered memcpy of the
    arrivals into an in-order transport buffer, then the reduction from the transport buffer.
    For a ring workload ``w`` whose arrivals are ``arrival_bytes`` long, returns per phase a pair
    (scatter records, reduce records) and the transport buffer's size.  The scatter records place
    arrival ``seq`` at ``(seq - first seq of the phase) * arrival_bytes`` and never forward; the
    reduce records read the transport buffer in pieces of ``group`` arrivals (with packet-sized
    arrivals, the collective's own chunk) and carry the phase's destinations.  Records only: the
    two passes are run by whoever calls this."""
    pairs, seq0, most = [], 0, 0
    for ph, lg in zip(w.phases, w.extra["logical"]):
        first = ph.descs.copy()
        first["dst_off"] = (first["seq"].astype(np.uint64) - np.uint64(seq0)) * np.uint64(arrival_bytes)
        first["out_off"] = NO_FORWARD
        assert len(lg) % group == 0 and np.all(lg["len"] == arrival_bytes), "whole groups of full arrivals"
        head = lg[::group]
        second = np.zeros(len(head), dtype=DESC)
        second["src_off"] = np.arange(len(head), dtype=np.uint64) * np.uint64(arrival_bytes * group)
        second["dst_off"], second["out_off"], second["len"] = head["dst_off"], head["out_off"], arrival_bytes * group
        second["seq"] = head["seq"]
        if group > 1:  # the arrivals of a group are consecutive in the accumulator and in the staging buffer
            nxt = lg[1::group]
            assert np.all(nxt["dst_off"] == head["dst_off"] + np.uint64(arrival_bytes))
            fwd = head["out_off"] != NO_FORWARD
            assert np.all(nxt["out_off"][fwd] == head["out_off"][fwd] + np.uint64(arrival_bytes))
        pairs.append((first, second))
        seq0 += len(lg)
        most = max(most, len(lg))
    return pairs, most * arrival_bytes


def alltoall_dispatch(name: str, seed: int, n_src: int, row_bytes: int, max_bytes: int, C: int,
                      paths: int, dup: float, dtype: int = BF16, lengths=None) -> Workload:
    """All-to-all dispatch receive side: ``n_src`` remote sources each send
    L_p = row_bytes * U{0..max_bytes // row_bytes} bytes, chunked at C; the
    destination is the concatenation in source order (exclusive prefix sum of L_p).
    Per-source streams are generated independently and merged by a seeded uniform
    interleave.  No reduction, no forwarding."""
    es = ELEM_SIZE[dtype]
    g = pl.rng(seed, 0xA2A)
    if lengths is None:
        lengths = row_bytes * g.integers(0, max_bytes // row_bytes + 1, n_src)
    lengths = np.asarray(lengths, dtype=np.int64)
    nchunks = -(-lengths // C)
    dst_base = np.concatenate([[0], np.cumsum(lengths)])
    seq_base = np.concatenate([[0], np.cumsum(nchunks)])
    logical = np.zeros(int(nchunks.sum()), dtype=LOGICAL)
    per_src_arr = []
    for p in range(n_src):
        n = int(nchunks[p])
        lo = int(seq_base[p])
        c = np.arange(n, dtype=np.int64)
        logical["seq"][lo:lo + n] = lo + c
        logical["dst_off"][lo:lo + n] = dst_base[p] + c * C
        logical["len"][lo:lo + n] = np.minimum(C, lengths[p] - c * C)
        logical["out_off"][lo:lo + n] = NO_FORWARD
        per_src_arr.append(lo + gen_arrivals(seed, n, paths, None, dup, stream=100 + p)[0])
    order = merge_streams(seed, [len(a) for a in per_src_arr])
    cursor = [0] * n_src
    arr = np.empty(len(order), dtype=np.int64)
    for k, p in enumerate(order):
        arr[k] = per_src_arr[p][cursor[p]]
        cursor[p] += 1
    total = int(lengths.sum())
    acc = np.zeros(total // es, dtype=pl.np_dtype(dtype))
    recv = np.zeros(len(arr) * (C // es), dtype=pl.np_dtype(dtype))
    uniq = _draw("normal" if dtype == BF16 else "uniform", dtype, seed, 10,
                 len(logical) * (C // es)).reshape(len(logical), C // es)
    fill_slots(recv, uniq, arr, 0)
    d = materialize(logical, arr, 0, C)
    ph = Phase("scatter", COPY, d, len(logical), total, byte_model(COPY, logical, len(arr)))
    w = Workload(name, dtype, acc, recv, 0, len(logical), [ph],
                 note=f"sources={n_src} lengths={lengths.tolist()} C={C} paths={paths} dup={dup}")
    # what each source sent, as bytes: its chunks' payloads back to back, tail trimmed
    ub = uniq.view(np.uint8).reshape(len(logical), C)
    w.extra["sources"] = [
        ub[int(seq_base[p]): int(seq_base[p + 1])].reshape(-1)[: int(lengths[p])].copy()
        for p in range(n_src)
    ]
    w.extra["lengths"] = lengths
    return w


def direct_reduce_scatter(name: str, seed: int, R: int, M: int, C: int, dtype: int, paths: int, dup: float,
                          dist: str, op: int = SUM, reissue: float = 0.02) -> Workload:
    """Direct (one-hop) reduce-scatter receive side: each of the R-1 peers sends its copy
    of this rank's segment (M/R bytes, chunked at C) over its own multipath connection; the
    streams interleave at the receiver.  The control path emits one gather record per
    destination chunk at the moment the last of its R-1 source chunks has arrived, listing
    the first-arrived slot of every source in source-rank order; retransmitted source chunks
    occupy slots but produce no record.  With probability ``reissue`` a record is emitted a
    second time later on (a repeated hand-over the GPU must drop).  workload.phases[0].descs
    holds GATHER_DESC records; the accumulator is the rank's own segment."""
    es = ELEM_SIZE[dtype]
    n_src = R - 1
    assert 1 <= n_src <= MAX_SOURCES and M % R == 0
    S = M // R
    n = -(-S // C)
    per_src = [gen_arrivals(seed, n, paths, None, dup, stream=200 + p)[0] for p in range(n_src)]
    order = merge_streams(seed, [len(a) for a in per_src], stream=7)
    cursor = [0] * n_src
    first_slot = np.full((n_src, n), -1, dtype=np.int64)
    have = np.zeros(n, dtype=np.int64)
    src_of_slot, chunk_of_slot, emit = [], [], []
    for k, p in enumerate(order):
        c = int(per_src[p][cursor[p]])
        cursor[p] += 1
        src_of_slot.append(p)
        chunk_of_slot.append(c)
        if first_slot[p, c] < 0:
            first_slot[p, c] = k
            have[c] += 1
            if have[c] == n_src:
                emit.append(c)
    g = pl.rng(seed, 0xD1D)
    again = [c for c in emit if g.random() < reissue]
    seq_list = list(emit)
    for c in again:  # somewhere after the original
        at = seq_list.index(c) + 1 + int(g.integers(0, max(1, len(seq_list) // 4)))
        seq_list.insert(min(at, len(seq_list)), c)
    d = np.zeros(len(seq_list), dtype=GATHER_DESC)
    for i, c in enumerate(seq_list):
        d[i]["dst_off"] = c * C
        d[i]["out_off"] = NO_FORWARD
        d[i]["len"] = min(C, S - c * C)
        d[i]["seq"] = c
        d[i]["n_src"] = n_src
        d[i]["src_off"][:n_src] = first_slot[:, c] * C
    per = C // es
    recv = np.zeros(len(order) * per, dtype=pl.np_dtype(dtype))
    view = recv.reshape(-1, per)
    sos, cos = np.array(src_of_slot), np.array(chunk_of_slot)
    for p in range(n_src):
        uq = _draw(dist, dtype, seed, 300 + p, n * per).reshape(n, per)
        idx = np.flatnonzero(sos == p)
        view[idx] = uq[cos[idx]]
    acc = _draw(dist, dtype, seed, 1, S // es)
    ln = np.minimum(C, S - np.arange(n, dtype=np.int64) * C)
    algo = int((n_src + 1) * ln.sum() + ln.sum()) + (160 + 4) * len(d)
    ph = Phase("gather-reduce", op, d, n, int(n_src * ln.sum()), algo)
    return Workload(name, dtype, acc, recv, 0, n, [ph],
                    note=f"direct reduce-scatter R={R} M={M} C={C} paths={paths} dup={dup} dist={dist}")


def small_messages(name: str, seed: int, n_msgs: int, R: int, C: int, paths: int, dup: float,
                   lo_bytes: int = 64 << 10, hi_bytes: int = 1 << 20, dtype: int = F32,
                   dist: str = "uniform"):
    """Small-message regime: ``n_msgs`` independent ring allreduces with
    log-uniform sizes in [lo_bytes, hi_bytes), each rounded down to a multiple of
    16*R bytes so that segments stay 16-byte aligned.  All messages live in shared
    arenas (acc, recv_stage, out_stage, bitmap) at consecutive offsets, so a caller
    may apply one message per call or many per call.

    Returns (workload, per_msg) where workload.phases is empty and per_msg is a
    list of dicts {size, rs: DESC[], ag: DESC[], n_unique, payload_bytes,
    algo_bytes}; the caller concatenates records of the messages it batches.
    """
    es = ELEM_SIZE[dtype]
    g = pl.rng(seed, 0x5A11)
    u = g.random(n_msgs)
    sizes = (lo_bytes * (hi_bytes / lo_bytes) ** u).astype(np.int64)
    sizes -= sizes % (16 * R)
    acc_base = np.concatenate([[0], np.cumsum(sizes)])
    per_msg, slot0, out0, bit0 = [], 0, 0, 0
    all_arr = []
    for m in range(n_msgs):
        rs, ag, n_out = ring_logical(R, int(sizes[m]), C, seq_base=bit0,
                                     acc_base=int(acc_base[m]), out_base=out0 * C)
        a_rs = gen_arrivals(seed, len(rs), paths, None, dup, stream=2 * m)[0]
        a_ag = gen_arrivals(seed, len(ag), paths, None, dup, stream=2 * m + 1)[0]
        d_rs = materialize(rs, a_rs, slot0, C)
        d_ag = materialize(ag, a_ag, slot0 + len(a_rs), C)
        all_arr.append((slot0, len(rs), a_rs, len(ag), a_ag))
        per_msg.append(dict(size=int(sizes[m]), rs=d_rs, ag=d_ag, n_unique=len(rs) + len(ag),
                            payload_bytes=int(rs["len"].astype(np.int64).sum() + ag["len"].astype(np.int64).sum()),
                            algo_bytes=byte_model(SUM, rs, len(a_rs)) + byte_model(COPY, ag, len(a_ag))))
        slot0 += len(a_rs) + len(a_ag)
        out0 += n_out
        bit0 += len(rs) + len(ag)
    per = C // es
    recv = np.zeros(slot0 * per, dtype=pl.np_dtype(dtype))
    gp = pl.rng(seed, 77)
    view = recv.reshape(-1, per)
    for (s0, n_rs, a_rs, n_ag, a_ag) in all_arr:
        for n, a, base in ((n_rs, a_rs, s0), (n_ag, a_ag, s0 + len(a_rs))):
            if n == 0:
                continue
            x = gp.random((n, per), dtype=np.float32)
            x *= np.float32(2.0)
            x -= np.float32(1.0)
            uq = x if dtype == F32 else (x.view(np.uint32) >> np.uint32(16)).astype(np.uint16)
            view[base: base + len(a)] = uq[a]
    acc = _draw(dist, dtype, seed, 1, int(acc_base[-1]) // es)
    w = Workload(name, dtype, acc, recv, out0 * C, bit0, [],
                 note=f"msgs={n_msgs} R={R} C={C} paths={paths} dup={dup}")
    return w, per_msg


# ---------------------------------------------------------------------------
# The five named configurations (full sizes) and reduced shapes of the same recipe
# ---------------------------------------------------------------------------

def config1(seed: int = 1, **kw) -> Workload:
    a = dict(R=8, M=4 << 20, C=64 << 10, dtype=F32, paths=4, window=None, dup=0.01, dist="uniform")
    a.update(kw)
    return ring_share("allreduce-4MiB-f32", seed, **a)


def config2(seed: int = 1, **kw) -> Workload:
    a = dict(R=16, M=256 << 20, C=32 << 10, dtype=BF16, paths=256, window=1024, dup=0.02, dist="normal")
    a.update(kw)
    return ring_share("allreduce-256MiB-bf16", seed, **a)


def config3(seed: int = 1, **kw) -> Workload:
    a = dict(R=8, M=1 << 30, C=128 << 10, dtype=F32, paths=64, window=256, dup=0.005,
             dist="uniform", allgather=False)
    a.update(kw)
    return ring_share("reduce-scatter-1GiB-f32", seed, **a)


def config4(seed: int = 1, **kw) -> Workload:
    a = dict(n_src=7, row_bytes=7168 * 2, max_bytes=16 << 20, C=16 << 10, paths=128, dup=0.01)
    a.update(kw)
    return alltoall_dispatch("alltoall-dispatch-bf16", seed, **a)


def config5(seed: int = 1, **kw):
    a = dict(n_msgs=10000, R=8, C=4 << 10, paths=32, dup=0.03)
    a.update(kw)
    return small_messages("small-allreduce-f32", seed, **a)
