"""Host-side checks of the synthetic input generators (no oracle, no GPU)."""
import numpy as np
import pytest

from synth import workloads as wl
from synth.arrivals import gen_arrivals, merge_streams
from synth.layout import DESC, NO_FORWARD, COPY, SUM, F32, BF16


@pytest.mark.parametrize("n,P,W,d", [(500, 8, 16, 0.1), (64, 1, None, 0.5), (1000, 256, 64, 0.02), (1, 4, 3, 1.0)])
def test_arrival_model_invariants(n, P, W, d):
    seq, cpy, pth = gen_arrivals(3, n, P, W, d)
    counts = np.bincount(seq, minlength=n)
    assert counts.min() >= 1 and counts.max() <= 2  # every chunk arrives, at most one retransmission
    assert np.array_equal(np.sort(seq[cpy == 0]), np.arange(n))
    # reorder window: when seq s arrives, every seq <= s - W has already arrived
    w = n if W is None else W
    first = np.full(n, -1)
    for k, s in enumerate(seq):
        if first[s] < 0:
            first[s] = k
    for k, s in enumerate(seq):
        if s - w >= 0:
            assert first[: s - w + 1].max() < k and first[: s - w + 1].min() >= 0
    # each path delivers originals in the order they were sent
    for p in range(P):
        s_p = seq[(pth == p) & (cpy == 0)]
        assert np.all(np.diff(s_p) > 0)
    # a retransmission travels on another path
    if P > 1:
        for s in np.flatnonzero(counts == 2):
            assert len(set(pth[seq == s])) == 2
    # same seed, same stream
    assert np.array_equal(seq, gen_arrivals(3, n, P, W, d)[0])


def test_arrivals_are_actually_reordered_and_duplicated():
    seq, cpy, _ = gen_arrivals(1, 4000, 256, 1024, 0.02)
    assert 40 <= cpy.sum() <= 130
    assert np.count_nonzero(np.diff(seq) < 0) > 1000
    assert np.abs(seq - np.arange(len(seq))).max() > 100


def test_merge_keeps_counts():
    ids = merge_streams(2, [5, 0, 7])
    assert np.array_equal(np.bincount(ids, minlength=3), [5, 0, 7])


def test_ring_share_layout_config2_shape():
    """Reduced message, same recipe as the 256 MiB configuration."""
    w = wl.config2(M=16 << 20)
    rs, ag = w.phases
    assert rs.op == SUM and ag.op == COPY
    assert rs.n_unique == 15 * 32 and ag.n_unique == 15 * 32
    assert w.n_bits == 2 * 15 * 32 and w.out_bytes == (15 + 14) * 32 * (32 << 10)
    d = np.concatenate([rs.descs, ag.descs])
    assert d.dtype == DESC
    assert np.array_equal(d["src_off"], np.arange(len(d), dtype=np.uint64) * (32 << 10))
    assert np.all(d["len"] == 32 << 10) and np.all(d["dst_off"] % 16 == 0)
    # reduce-scatter never touches the rank's own segment 0; allgather never touches segment 1
    S = (16 << 20) // 16
    assert not np.any(rs.descs["dst_off"] < S)
    assert not np.any((ag.descs["dst_off"] >= S) & (ag.descs["dst_off"] < 2 * S))
    assert np.all(rs.descs["out_off"] != NO_FORWARD)
    assert np.count_nonzero(np.unique(ag.descs[ag.descs["out_off"] == NO_FORWARD]["seq"])) == 32
    # byte model: 4 C per reduced+forwarded chunk, 3 C / 2 C for allgather, + 36 B per arrival
    C = 32 << 10
    assert rs.algo_bytes == 4 * C * 480 + 36 * len(rs.descs)
    assert ag.algo_bytes == 3 * C * 448 + 2 * C * 32 + 36 * len(ag.descs)
    # duplicates are byte-identical copies in their own slots
    per = C // 2
    slots = w.recv_stage.reshape(-1, per)
    _, first, cnt = np.unique(d["seq"], return_index=True, return_counts=True)
    assert (cnt == 2).any()
    for s in np.unique(d["seq"])[cnt == 2][:8]:
        k = np.flatnonzero(d["seq"] == s)
        assert np.array_equal(slots[k[0]], slots[k[1]]) and k[0] != k[1]


def test_full_size_shapes_without_building_payloads():
    rs, ag, n_out = wl.ring_logical(16, 256 << 20, 32 << 10)
    assert len(rs) == 7680 and len(ag) == 7680 and n_out == 14848
    rs, ag, n_out = wl.ring_logical(8, 1 << 30, 128 << 10, allgather=False)
    assert len(rs) == 7168 and len(ag) == 0 and n_out == 6144
    assert np.count_nonzero(rs["out_off"] == NO_FORWARD) == 1024


def test_alltoall_layout():
    w = wl.config4(max_bytes=1 << 20)
    d = w.phases[0].descs
    L = w.extra["lengths"]
    assert np.all(L % 14336 == 0) and len(L) == 7
    assert np.all(d["out_off"] == NO_FORWARD) and np.all(d["len"] % 2048 == 0) and np.all(d["len"] > 0)
    u = np.unique(d["seq"])
    assert len(u) == w.n_bits == int(np.sum(-(-L // (16 << 10))))
    assert w.acc.nbytes == int(L.sum())


def test_small_messages_layout():
    w, msgs = wl.config5(n_msgs=40)
    sizes = np.array([m["size"] for m in msgs])
    assert sizes.min() >= (64 << 10) - 128 and sizes.max() < (1 << 20) and np.all(sizes % 128 == 0)
    assert w.acc.nbytes == sizes.sum()
    allseq = np.concatenate([np.concatenate([m["rs"]["seq"], m["ag"]["seq"]]) for m in msgs])
    assert len(np.unique(allseq)) == w.n_bits
    # messages do not share destination ranges
    ends = np.cumsum(sizes)
    for m, lo, hi in zip(msgs, ends - sizes, ends):
        assert m["rs"]["dst_off"].min() >= lo and (m["rs"]["dst_off"] + m["rs"]["len"]).max() <= hi


def test_control_header_fields_roundtrip():
    """Section 3.1: 8 + 7 + 8 + 1 + 8 bits; every field survives packing, fields do not overlap."""
    from synth import header as hd
    from synth import payload as pl
    g = pl.rng(5, 5)
    n = 5000
    f = dict(conn=g.integers(0, 256, n), msg=g.integers(0, 128, n), csn=g.integers(0, 256, n),
             last=g.integers(0, 2, n), spare=g.integers(0, 256, n))
    h = hd.pack(**f)
    assert h.dtype == np.uint32
    back = hd.unpack(h)
    for k in f:
        assert np.array_equal(back[k], f[k]), k
    # one field at its maximum, the others zero: exactly that field's bits are set
    widths = dict(conn=8, msg=7, csn=8, last=1, spare=8)
    seen = 0
    for k, bits in widths.items():
        one = int(hd.pack(**{x: ((1 << bits) - 1 if x == k else 0) for x in widths}))
        assert bin(one).count("1") == bits and one & seen == 0
        seen |= one
    assert seen == 0xFFFFFFFF
    assert hd.MESSAGES_IN_FLIGHT == 128 and hd.CHUNKS_PER_MESSAGE == 256
    assert np.array_equal(hd.seq_of(h), f["msg"] * 256 + f["csn"])
    with pytest.raises(AssertionError):
        hd.pack(0, 128, 0, 0)
    hs = hd.pack(3, [5, 5, 9], [0, 41, 7], [0, 1, 0])
    c = hd.chunk_counts(hs)
    assert c[5] == 42 and c[9] == 0 and c.sum() == 42
