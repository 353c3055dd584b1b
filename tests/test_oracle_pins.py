"""Pins for the CPU oracle: every check compares it with something that is NOT the
oracle -- closed forms, integer arithmetic, numpy as a third opinion, exact
rounding done by brute force, hand-derived tie cases, invariants of the problem.

Each pin is written so that a plausible slip in the oracle (double apply, dropped
duplicate test, wrong offset field, swapped src/dst, missing forward, wrong
rounding direction, wrong ring segment index) fails at least one assertion.
"""
import os

import numpy as np
import pytest

import oracle
from synth import payload as pl
from synth import workloads as wl
from synth.arrivals import gen_arrivals
from synth.layout import (DESC, NO_FORWARD, FORWARD_ONLY, F32, BF16, F16, I32, SUM, MAX, MIN, COPY, PROD,
                          ELEM_SIZE)

from ringloop import closed_loop_allreduce

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def run_workload(w, check=True, split=None):
    """Oracle over every phase of a workload; returns (acc, out_stage bytes, bitmap words)."""
    acc = w.acc.copy()
    out = np.full(w.out_bytes, 0xA5, dtype=np.uint8) if w.out_bytes else None
    seen = oracle.new_seen(w.n_bits)
    for ph in w.phases:
        cuts = [0, len(ph.descs)] if split is None else [0] + sorted(split(len(ph.descs))) + [len(ph.descs)]
        for lo, hi in zip(cuts[:-1], cuts[1:]):
            oracle.apply(acc, out, w.recv_stage, ph.descs[lo:hi], seen, w.dtype, ph.op, check=check)
    return acc, out, oracle.pack_bitmap(seen)


# --- P1: exactly once, closed form ---------------------------------------------

@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("seed", [1, 2, 3])
def test_exactly_once_all_ones(dtype, seed):
    """acc = 0, every payload element = 1, SUM: any reorder / duplication must leave
    exactly 1 in every covered element (2 = applied twice, 0 = lost)."""
    R, C, es = 4, 256, ELEM_SIZE[dtype]
    M = R * 5 * C - R * 64  # ragged: last chunk of each segment is short
    w = wl.ring_share("p1", seed, R=R, M=M, C=C, dtype=dtype, paths=5, window=7, dup=0.4,
                      dist="ones", allgather=False)
    w.acc[:] = 0
    guard = w.acc.copy()
    acc, out, bm = run_workload(w)
    one = pl.ints_as(np.array([1]), dtype)[0]
    S = M // R // es
    covered = np.ones(M // es, dtype=bool)
    covered[0:S] = False  # rank 0 never receives its own segment 0 in reduce-scatter
    assert np.all(acc[covered] == one)
    assert np.array_equal(acc[~covered], guard[~covered])
    seqs = np.unique(w.phases[0].descs["seq"])
    assert sum(bin(int(x)).count("1") for x in bm) == len(seqs) == w.phases[0].n_unique
    for s in range(w.n_bits):
        assert bool(bm[s >> 5] >> (s & 31) & 1) == (s in set(seqs.tolist()))
    assert len(w.phases[0].descs) > len(seqs), "the stream must contain duplicates"


def test_exactly_once_many_copies_any_position():
    """One seq repeated 9 times (first, middle, last, adjacent) is applied once."""
    C, n = 64, 6
    recv_rows = []
    d = np.zeros(0, dtype=DESC)
    order = [3, 0, 3, 3, 1, 2, 3, 4, 3, 5, 3, 3, 0, 3, 3]
    d = np.zeros(len(order), dtype=DESC)
    recv = np.zeros(len(order) * C // 4, dtype=np.float32)
    for k, s in enumerate(order):
        d[k] = (k * C, s * C, NO_FORWARD, C, s)
        recv[k * C // 4:(k + 1) * C // 4] = s + 1  # same seq -> same payload
    acc = np.full(n * C // 4, 100.0, dtype=np.float32)
    seen = oracle.new_seen(n)
    applied = oracle.apply(acc, None, recv, d, seen, F32, SUM)
    assert applied == n
    expect = 100.0 + np.repeat(np.arange(1, n + 1), C // 4)
    assert np.array_equal(acc, expect.astype(np.float32))
    # a second call with the same records is all duplicates
    assert oracle.apply(acc, None, recv, d, seen, F32, SUM) == 0
    assert np.array_equal(acc, expect.astype(np.float32))


# --- P2: independence of path interleaving ------------------------------------

@pytest.mark.parametrize("dtype,dist", [(F32, "uniform"), (BF16, "normal")])
def test_interleaving_invariance(dtype, dist):
    kw = dict(R=4, M=4 * 6 * 512, C=512, dtype=dtype, paths=8, window=5, dup=0.3, dist=dist)
    base = wl.ring_share("p2", 7, **kw)
    ref = run_workload(base)
    n = [len(lg) for lg in base.extra["logical"]]
    variants = [wl.ring_share("p2", 7, arrival_seed=s, **kw) for s in (11, 12, 13)]
    # reversed arrival order, and "every duplicate first, then the originals"
    variants.append(wl.ring_share("p2", 7, arrivals=[a[::-1] for a in base.extra["arrivals"]], **kw))
    dups_first = []
    for a, m in zip(base.extra["arrivals"], n):
        _, first = np.unique(a, return_index=True)
        mask = np.ones(len(a), dtype=bool)
        mask[first] = False
        dups_first.append(np.concatenate([a[mask], a[~mask][::-1]]))
    variants.append(wl.ring_share("p2", 7, arrivals=dups_first, **kw))
    variants.append(wl.ring_share("p2", 7, identity=True, **kw))
    for v in variants:
        got = run_workload(v)
        for a, b in zip(ref, got):
            assert np.array_equal(a, b)
    # cutting a call into many calls at arbitrary points changes nothing
    g = pl.rng(5, 5)
    got = run_workload(base, check=False,
                       split=lambda m: g.choice(np.arange(1, m), size=min(6, m - 1), replace=False).tolist())
    for a, b in zip(ref, got):
        assert np.array_equal(a, b)


# --- P3: closed loop equals the textbook ring, and the exact integer sum -----------

class OracleBackend:
    def make_rank(self, acc_init, out_bytes, n_bits):
        return dict(acc=acc_init, out=np.zeros(out_bytes, dtype=np.uint8), seen=oracle.new_seen(n_bits))

    def apply(self, h, recv, descs, dtype, op):
        oracle.apply(h["acc"], h["out"], recv, descs, h["seen"], dtype, op)

    def read_out(self, h, off, nbytes):
        return h["out"][off:off + nbytes].copy()

    def read_acc(self, h):
        return h["acc"]


class OracleBackendWithSegment(OracleBackend):
    """The same, with the first hop's chunks produced by the oracle's sender-side segmentation."""

    def segment(self, h, off, nbytes, C):
        stage = np.zeros(-(-nbytes // C) * (C + 32), dtype=np.uint8)
        d = oracle.segment(stage, h["acc"].view(np.uint8), off, nbytes, C, 0, C + 32)
        return [stage[o:o + n].copy() for o, n in zip(d["stage_off"], d["len"])]


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("R,n,C", [(2, 64, 16), (3, 96, 32), (4, 512, 64), (8, 4096, 48)])
def test_closed_loop_small_integers_exact(dtype, R, n, C):
    """Integer-valued inputs in [-8, 8]: every partial sum is exact in fp32 and in
    bf16 (|sum| <= 64), so the allreduce must equal the int64 column sum -- a result
    that does not depend on fold order or on any rounding rule."""
    n = n * (2 if dtype == BF16 else 1)
    vals = pl.small_int(3, R, R * n).reshape(R, n)
    x = pl.ints_as(vals, dtype)
    got = closed_loop_allreduce(OracleBackend(), x, dtype, C, seed=9, paths=3, window=4, dup=0.25)
    expect = pl.ints_as(vals.sum(axis=0), dtype)
    for r in range(R):
        assert np.array_equal(got[r], expect)


def test_closed_loop_with_segmented_first_hop():
    """Step 0 of the ring sends each rank's own segment: cut into chunks by the sender-side path
    instead of host slicing, the closed loop still equals the textbook ring (ragged last chunk)."""
    R, n, C = 4, 4 * 100, 48
    x = pl.uniform_f32(15, 3, R * n).reshape(R, n)
    got = closed_loop_allreduce(OracleBackendWithSegment(), x, F32, C, seed=3, paths=3, window=4, dup=0.2)
    assert np.array_equal(got, oracle.ring_allreduce(x, F32, SUM))


@pytest.mark.parametrize("dtype,op", [(F32, SUM), (BF16, SUM), (F32, MAX), (BF16, MIN)])
def test_closed_loop_matches_textbook_ring(dtype, op):
    """General values: the chunked, reordered, duplicated transport must give
    bit-for-bit what an in-order ring without any transport gives."""
    R, n, C = 5, 5 * 200, 112
    x = (pl.uniform_f32(4, 4, R * n) * 3).reshape(R, n) if dtype == F32 else pl.normal_bf16(4, 4, R * n).reshape(R, n)
    got = closed_loop_allreduce(OracleBackend(), x, dtype, C, seed=2, paths=6, window=None, dup=0.2, op=op)
    expect = oracle.ring_allreduce(x, dtype, op)
    assert np.array_equal(got, expect)
    assert all(np.array_equal(expect[0], expect[r]) for r in range(R))


def test_textbook_ring_itself():
    """The in-order ring reference against numpy: R=2 is one correctly rounded add per
    element; integer inputs give the exact column sum; MAX gives the column maximum;
    and for fp32 the value of segment j is the left fold starting at rank j."""
    a = pl.uniform_f32(1, 1, 2 * 64).reshape(2, 64)
    r = oracle.ring_allreduce(a, F32, SUM)
    assert np.array_equal(r[0], a[0] + a[1]) and np.array_equal(r[1], a[0] + a[1])
    vals = pl.small_int(2, 2, 7 * 70).reshape(7, 70)
    for dt in (F32, BF16):
        r = oracle.ring_allreduce(pl.ints_as(vals, dt), dt, SUM)
        assert all(np.array_equal(r[k], pl.ints_as(vals.sum(axis=0), dt)) for k in range(7))
    x = pl.uniform_f32(3, 3, 6 * 60).reshape(6, 60)
    assert np.array_equal(oracle.ring_allreduce(x, F32, MAX)[2], x.max(axis=0))
    assert np.array_equal(oracle.ring_allreduce(x, F32, MIN)[5], x.min(axis=0))
    r = oracle.ring_allreduce(x, F32, SUM)
    for j in range(6):
        fold = x[j, j * 10:(j + 1) * 10].copy()
        for h in range(1, 6):
            fold = fold + x[(j + h) % 6, j * 10:(j + 1) * 10]  # numpy fp32 add: one rounding each
        assert np.array_equal(r[0, j * 10:(j + 1) * 10], fold)


# --- P4: in-order, duplicate-free special case = slice arithmetic in numpy --------

@pytest.mark.parametrize("op", [SUM, MAX, MIN, COPY])
def test_identity_stream_is_slicewise_numpy(op):
    C = 320
    w = wl.ring_share("p4", 5, R=4, M=4 * 3 * C + 4 * 64, C=C, dtype=F32, paths=1, window=None,
                      dup=0.0, dist="uniform", allgather=False, op=op, identity=True)
    acc, out, _ = run_workload(w)
    expect = w.acc.copy()
    eout = np.full(w.out_bytes, 0xA5, dtype=np.uint8)
    f = {SUM: np.add, MAX: np.maximum, MIN: np.minimum, COPY: lambda a, b: b}[op]
    for d in w.phases[0].descs:
        n, s, t = d["len"] // 4, d["src_off"] // 4, d["dst_off"] // 4
        expect[t:t + n] = f(expect[t:t + n], w.recv_stage[s:s + n])
        if d["out_off"] != NO_FORWARD:
            eout[int(d["out_off"]):int(d["out_off"]) + int(d["len"])] = expect[t:t + n].view(np.uint8)
    assert np.array_equal(acc, expect)
    assert np.array_equal(out, eout)
    # the last reduce-scatter step keeps its result: some records forward, some do not
    fw = w.phases[0].descs["out_off"] != NO_FORWARD
    assert fw.any() and (~fw).any()


# --- forward-only records: relay the combined value, leave the accumulator alone ---------

def test_forward_only_records_relay_without_write_back():
    C = 256
    w = wl.ring_share("relay", 6, R=4, M=4 * 3 * C + 4 * 32, C=C, dtype=F32, paths=1, window=None,
                      dup=0.0, dist="uniform", allgather=False, identity=True, relay=True)
    d = w.phases[0].descs
    flagged = (d["out_off"] != NO_FORWARD) & ((d["out_off"] & FORWARD_ONLY) != 0)
    assert flagged.any() and (~flagged).any()
    acc, out, bm = run_workload(w)
    expect = w.acc.copy()
    eout = np.full(w.out_bytes, 0xA5, dtype=np.uint8)
    for r, f in zip(d, flagged):
        n, s, t = r["len"] // 4, r["src_off"] // 4, r["dst_off"] // 4
        val = expect[t:t + n] + w.recv_stage[s:s + n]  # numpy fp32 add: one rounding
        if not f:
            expect[t:t + n] = val
        if r["out_off"] != NO_FORWARD:
            o = int(r["out_off"] & ~FORWARD_ONLY)
            eout[o:o + int(r["len"])] = val.view(np.uint8)
    assert np.array_equal(acc, expect) and np.array_equal(out, eout)
    assert sum(bin(int(x)).count("1") for x in bm) == len(d)
    # byte model: a relayed chunk moves 3 bytes per payload byte
    C4 = int(d["len"][flagged].astype(np.int64).sum())
    plain = wl.ring_share("plain", 6, R=4, M=4 * 3 * C + 4 * 32, C=C, dtype=F32, paths=1, window=None,
                          dup=0.0, dist="uniform", allgather=False, identity=True)
    assert plain.phases[0].algo_bytes - w.phases[0].algo_bytes == C4


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_closed_loop_with_relay_equals_textbook_ring(dtype):
    """Not writing intermediate partial sums back must not change the allreduce result:
    those segments are overwritten by the allgather phase."""
    R, n, C = 6, 6 * 160, 96
    x = pl.uniform_f32(4, 5, R * n).reshape(R, n) if dtype == F32 else pl.normal_bf16(4, 5, R * n).reshape(R, n)
    got = closed_loop_allreduce(OracleBackend(), x, dtype, C, seed=3, paths=5, window=4, dup=0.2, relay=True)
    assert np.array_equal(got, oracle.ring_allreduce(x, dtype, SUM))


# --- P5: all-to-all is a placement of the source bytes -----------------------------

@pytest.mark.parametrize("seed", [1, 2])
def test_alltoall_is_concatenation_of_sources(seed):
    w = wl.alltoall_dispatch("p5", seed, n_src=7, row_bytes=224, max_bytes=224 * 40, C=512,
                             paths=6, dup=0.2)
    lengths = w.extra["lengths"]
    total = int(lengths.sum())
    guard = 64
    dst = np.full(total + 2 * guard, 0xEE, dtype=np.uint8)
    seen = oracle.new_seen(w.n_bits)
    ph = w.phases[0]
    applied = oracle.scatter(dst[guard:guard + total], w.recv_stage, ph.descs, seen)
    assert applied == ph.n_unique
    srcs = np.concatenate(w.extra["sources"]) if total else np.zeros(0, np.uint8)
    assert np.array_equal(dst[guard:guard + total], srcs)
    assert np.all(dst[:guard] == 0xEE) and np.all(dst[guard + total:] == 0xEE)
    assert np.array_equal(np.bincount(dst[guard:guard + total], minlength=256), np.bincount(srcs, minlength=256))
    # scatter and apply(COPY, no forward) are the same operation
    acc = np.zeros(total // 2, dtype=np.uint16)
    oracle.apply(acc, None, w.recv_stage, ph.descs, oracle.new_seen(w.n_bits), BF16, COPY)
    assert np.array_equal(acc.view(np.uint8), srcs)


def test_alltoall_empty_source_contributes_nothing():
    w = wl.alltoall_dispatch("p5e", 1, n_src=3, row_bytes=32, max_bytes=0, C=64, paths=2, dup=0.5,
                             lengths=[0, 96, 0])
    assert len(np.unique(w.phases[0].descs["seq"])) == 2
    dst = np.zeros(96, dtype=np.uint8)
    oracle.scatter(dst, w.recv_stage, w.phases[0].descs, oracle.new_seen(w.n_bits))
    assert np.array_equal(dst, w.extra["sources"][1])


# --- P6: numerics --------------------------------------------------------------

def nearest_even_bf16(f32: np.ndarray) -> np.ndarray:
    """binary32 -> bf16 by the definition of round-to-nearest-even, evaluated exactly:
    the two bf16 neighbours of x are its truncation and the next pattern up in
    magnitude; choose the closer in exact (float64) arithmetic, the even one on a tie."""
    u = f32.view(np.uint32)
    lo = (u >> 16).astype(np.uint32)
    hi = lo + 1  # next magnitude; crossing into the exponent is the right neighbour too
    x = f32.astype(np.float64)
    flo = (lo << 16).view(np.float32).astype(np.float64)
    with np.errstate(over="ignore", invalid="ignore"):
        fhi = (hi << 16).view(np.float32).astype(np.float64)
        # beyond the largest finite bf16 the upper neighbour is infinity, standing for 2^128
        fhi = np.where(np.isinf(fhi), np.sign(x) * 2.0 ** 128, fhi)
        dlo, dhi = np.abs(x - flo), np.abs(fhi - x)
    pick_hi = (dhi < dlo) | ((dhi == dlo) & ((lo & 1) == 1))
    return np.where(pick_hi, hi, lo).astype(np.uint16)


def test_bf16_rounding_is_nearest_even_exact():
    g = pl.rng(6, 6)
    u = g.integers(0, 2 ** 32, 300000, dtype=np.uint64).astype(np.uint32)
    # add every pattern whose dropped half is exactly the tie, or one off it
    base = (np.arange(0, 1 << 16, dtype=np.uint32) << 16)
    u = np.concatenate([u, base | 0x8000, base | 0x7FFF, base | 0x8001, base, base | 0xFFFF])
    f = u.view(np.float32)
    finite = np.isfinite(f)
    f = f[finite]
    got = np.array([oracle.f32_to_bf16(v) for v in f[:: max(1, len(f) // 120000)]], dtype=np.uint16)
    expect = nearest_even_bf16(f[:: max(1, len(f) // 120000)])
    assert np.array_equal(got, expect)


def _f32_arg(bits: int):
    """A ctypes float holding exactly these bits: passing a Python float instead would go through
    a double and quiet a signalling NaN on the way, which is the very case under test."""
    import ctypes
    return ctypes.c_float.from_buffer_copy(np.uint32(bits).tobytes())


# signalling and quiet NaNs of both signs; several have mantissa bits only in the part narrowing drops
NAN_BITS = [0x7F800001, 0xFF800001, 0x7FC00000, 0xFFC00000, 0x7FFFFFFF, 0xFFFFFFFF, 0x7F80FFFF, 0xFF801FFF,
            0x7FA00000, 0x7F800100, 0xFF80E000, 0x7FBFFFFF]


def test_narrowing_a_nan_gives_a_quiet_nan_of_the_same_sign():
    """IEEE 754 fixes what a format conversion does with a NaN: the result is a NaN (never an
    infinity, a zero or a finite value, whatever rounding would do to the pattern), quiet, and of
    the same sign.  numpy's binary16 conversion is the third opinion for NaN-ness."""
    for u in NAN_BITS:
        f = np.array([u], dtype=np.uint32).view(np.float32)
        assert np.isnan(f[0])
        sign = (u >> 16) & 0x8000
        b = int(oracle.lib().orc_f32_to_bf16(_f32_arg(u)))
        assert (b & 0x7F80) == 0x7F80 and (b & 0x007F) != 0, hex(u)   # a bf16 NaN
        assert (b & 0x0040) and (b & 0x8000) == sign, hex(u)          # quiet, same sign
        h = int(oracle.lib().orc_f32_to_f16(_f32_arg(u)))
        assert (h & 0x7C00) == 0x7C00 and (h & 0x03FF) != 0, hex(u)   # a binary16 NaN
        assert (h & 0x0200) and (h & 0x8000) == sign, hex(u)
        assert np.isnan(f.astype(np.float16)[0]) and np.isnan(np.array([h], np.uint16).view(np.float16)[0])
    # through the data path: a NaN element stays NaN in every 16-bit sum, whatever the other operand
    for a, r in ((0x7E00, 0x3C00), (0x7C01, 0x0000), (0xFE00, 0x7C00), (0x7C00, 0xFC00)):
        got = np.array([oracle.combine_f16(a, r, SUM), oracle.combine_f16(r, a, SUM)], np.uint16).view(np.float16)
        with np.errstate(invalid="ignore"):
            ref = np.array([a], np.uint16).view(np.float16) + np.array([r], np.uint16).view(np.float16)
        assert np.isnan(ref[0]) and np.all(np.isnan(got)), (hex(a), hex(r))
    for a, r in ((0x7FC0, 0x3F80), (0x7F81, 0x0000), (0xFFC0, 0x7F80), (0x7F80, 0xFF80)):
        got = [oracle.combine_bf16(a, r, SUM), oracle.combine_bf16(r, a, SUM)]
        assert all((g & 0x7F80) == 0x7F80 and (g & 0x7F) for g in got), (hex(a), hex(r))


def test_bf16_golden_ties():
    """Hand-derived cases, one per line: a_bits r_bits expected_bits (hex)."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "bf16_sum_cases.txt")) if l.strip() and l[0] != "#"]
    assert len(rows) >= 10
    for a, r, e in rows:
        assert oracle.combine_bf16(int(a, 16), int(r, 16), SUM) == int(e, 16), (a, r, e)
        assert oracle.combine_bf16(int(r, 16), int(a, 16), SUM) == int(e, 16), (r, a, e)


def test_f16_golden_ties():
    """Hand-derived binary16 cases: ties, overflow threshold, subnormals."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "f16_sum_cases.txt")) if l.strip() and l[0] != "#"]
    assert len(rows) >= 10
    for a, r, e in rows:
        assert oracle.combine_f16(int(a, 16), int(r, 16), SUM) == int(e, 16), (a, r, e)
        assert oracle.combine_f16(int(r, 16), int(a, 16), SUM) == int(e, 16), (r, a, e)


def test_bf16_sum_is_f32_add_then_nearest_even():
    g = pl.rng(8, 8)
    a = pl.normal_bf16(8, 1, 50000)
    r = pl.normal_bf16(8, 2, 50000)
    r[::7] = (a[::7] ^ 0x8000)  # exact cancellation
    r[::11] = a[::11] + 1       # neighbours
    wide = lambda h: (h.astype(np.uint32) << 16).view(np.float32)
    s32 = wide(a) + wide(r)  # numpy: one correctly rounded binary32 add
    expect = nearest_even_bf16(s32)
    got = np.array([oracle.combine_bf16(int(x), int(y), SUM) for x, y in zip(a, r)], dtype=np.uint16)
    assert np.array_equal(got, expect)


def test_f32_sum_is_correctly_rounded_and_keeps_subnormals():
    a = pl.uniform_f32(9, 1, 20000) * np.float32(1e-3)
    r = pl.uniform_f32(9, 2, 20000)
    # float64 holds a+r with >= 2*24+2 bits, so rounding its sum to binary32 is the exact answer
    expect = (a.astype(np.float64) + r.astype(np.float64)).astype(np.float32)
    got = np.array([oracle.combine_f32(float(x), float(y), SUM) for x, y in zip(a, r)], dtype=np.float32)
    assert np.array_equal(got.view(np.uint32), expect.view(np.uint32))
    tiny = np.array([1, 2, 0x007FFFFF, 0x00800000], dtype=np.uint32).view(np.float32)
    for t in tiny:
        got = oracle.combine_f32(float(t), float(tiny[0]), SUM)
        assert got.view(np.uint32) == t.view(np.uint32) + 1  # subnormal spacing is one ulp = 2^-149
    assert oracle.combine_f32(0.0, -0.0, SUM).view(np.uint32) == 0  # +0 + -0 = +0


def test_max_min_select_and_tie_rule():
    assert oracle.combine_f32(1.0, 2.0, MAX) == 2.0 and oracle.combine_f32(2.0, 1.0, MAX) == 2.0
    assert oracle.combine_f32(1.0, 2.0, MIN) == 1.0 and oracle.combine_f32(-3.0, 1.0, MIN) == -3.0
    assert oracle.combine_bf16(0x3F80, 0x4000, MAX) == 0x4000 and oracle.combine_bf16(0xC000, 0x3F80, MIN) == 0xC000
    # defined here (not fixed by the paper): a tie or an unordered pair keeps the local value
    assert oracle.combine_f32(0.0, -0.0, MAX).view(np.uint32) == 0
    assert oracle.combine_f32(-0.0, 0.0, MAX).view(np.uint32) == 0x80000000
    assert np.isnan(oracle.combine_f32(float("nan"), 1.0, MAX)) and oracle.combine_f32(1.0, float("nan"), MAX) == 1.0
    assert oracle.combine_f32(5.0, 7.0, COPY) == 7.0 and oracle.combine_bf16(1, 2, COPY) == 2


# --- binary16, int32, PROD ---------------------------------------------------------------

def test_f16_conversions_against_numpy():
    """numpy's float16 is an independent IEEE binary16: widening must agree on all 65536
    patterns, narrowing (nearest even, gradual underflow, overflow to inf) on every pattern
    around each binary16 boundary and on random binary32 values."""
    allh = np.arange(1 << 16, dtype=np.uint16)
    wide = np.array([oracle.f16_to_f32(int(h)) for h in allh], dtype=np.float32)
    ref = allh.view(np.float16).astype(np.float32)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(wide), nan) and np.array_equal(wide[~nan].view(np.uint32), ref[~nan].view(np.uint32))
    # binary32 patterns: each finite half value's fp32 image, +- a few ulps, and exact midpoints
    base = ref[~nan & np.isfinite(ref)].view(np.uint32)
    cand = np.concatenate([base + np.uint32(d) for d in (0, 1, 0xFFF, 0x1000, 0x1001, 0x1FFF, 0x2000)]
                          + [base - np.uint32(d) for d in (1, 0x1000, 0x1001)]
                          + [pl.rng(2, 2).integers(0, 2 ** 32, 200000, dtype=np.uint64).astype(np.uint32),
                             np.array([0x33000000, 0x33000001, 0x32FFFFFF, 0x33800000, 0x33C00000, 0x477FE000,
                                       0x477FEFFF, 0x477FF000, 0x477FFFFF, 0x47800000, 0x7F7FFFFF, 0x387FC000,
                                       0x387FE000, 0x38800000, 0x387FFFFF], dtype=np.uint32)])
    f = cand.view(np.float32)
    f = f[np.isfinite(f)][::7]
    with np.errstate(over="ignore"):
        expect = f.astype(np.float16).view(np.uint16)
    got = np.array([oracle.f32_to_f16(v) for v in f], dtype=np.uint16)
    assert np.array_equal(got, expect)


@pytest.mark.parametrize("op,npf", [(SUM, np.add), (PROD, np.multiply), (MAX, np.maximum), (MIN, np.minimum)])
def test_f16_i32_f32_ops_against_numpy(op, npf):
    n = 30000
    # binary16: numpy computes in fp32 when given fp32 inputs; round once with astype
    a, r = pl.uniform_f16(5, 1, n, 300.0), pl.uniform_f16(5, 2, n, 300.0)
    r[::9] = a[::9]
    with np.errstate(over="ignore"):
        expect = npf(a.view(np.float16).astype(np.float32), r.view(np.float16).astype(np.float32)).astype(np.float16)
    got = np.array([oracle.combine_f16(int(x), int(y), op) for x, y in zip(a, r)], dtype=np.uint16)
    assert np.array_equal(got, expect.view(np.uint16))
    # int32: wrapping add / multiply, signed max / min
    a, r = pl.uniform_i32(6, 1, n), pl.uniform_i32(6, 2, n)
    with np.errstate(over="ignore"):
        expect = npf(a, r)
    got = np.array([oracle.combine_i32(int(x), int(y), op) for x, y in zip(a, r)], dtype=np.int32)
    assert np.array_equal(got, expect)
    # fp32: one correctly rounded operation
    a, r = pl.uniform_f32(7, 1, n) * 1e3, pl.uniform_f32(7, 2, n)
    got = np.array([oracle.combine_f32(float(x), float(y), op) for x, y in zip(a, r)], dtype=np.float32)
    assert np.array_equal(got.view(np.uint32), npf(a, r).view(np.uint32))


def test_bf16_prod_is_f32_multiply_then_nearest_even():
    a, r = pl.normal_bf16(8, 3, 40000), pl.normal_bf16(8, 4, 40000)
    wide = lambda h: (h.astype(np.uint32) << 16).view(np.float32)
    expect = nearest_even_bf16(wide(a) * wide(r))  # product of two 8-bit significands is exact in fp32
    got = np.array([oracle.combine_bf16(int(x), int(y), PROD) for x, y in zip(a, r)], dtype=np.uint16)
    assert np.array_equal(got, expect)


@pytest.mark.parametrize("dtype,op", [(F16, SUM), (I32, SUM), (I32, PROD), (F16, MAX), (F32, PROD)])
def test_closed_loop_new_types_match_textbook_ring(dtype, op):
    R, n, C = 4, 4 * 192, 80
    x = wl._draw("uniform", dtype, 12, 3, R * n).reshape(R, n)
    got = closed_loop_allreduce(OracleBackend(), x, dtype, C, seed=7, paths=4, window=5, dup=0.2, op=op)
    expect = oracle.ring_allreduce(x, dtype, op)
    assert np.array_equal(got, expect)
    if dtype == I32 and op == SUM:  # wrapping integer sum: independent of order, equals the int64 sum mod 2^32
        assert np.array_equal(expect[0], x.astype(np.int64).sum(axis=0).astype(np.int32))


# --- receiver feedback from the bitmap -----------------------------------------------------

def numpy_ack(bits):
    """Independent reading of the same definition with numpy: first zero, popcount, and runs
    from the positions where the padded bit sequence changes value."""
    n = len(bits)
    zeros = np.flatnonzero(bits == 0)
    cum = int(zeros[0]) if len(zeros) else n
    edges = np.flatnonzero(np.diff(np.concatenate([[0], bits, [0]]).astype(np.int8)))
    runs = edges.reshape(-1, 2)
    runs = runs[runs[:, 0] > 0]
    return cum, int(bits.sum()), runs


def test_ack_report_hand_cases():
    pack = lambda bits: np.packbits(np.array(bits, dtype=np.uint8), bitorder="little").view(np.uint8)
    def words_of(bits):
        b = np.zeros((len(bits) + 31) // 32 * 32, dtype=np.uint8)
        b[:len(bits)] = bits
        return np.packbits(b, bitorder="little").view(np.uint32)
    # 1110 0110 1: cumulative 3, applied 6, runs [5,7) and [8,9)
    ca, na, nr, rg = oracle.ack_report(words_of([1, 1, 1, 0, 0, 1, 1, 0, 1]), 9, 8)
    assert (ca, na, nr) == (3, 6, 2) and rg.tolist() == [[5, 7], [8, 9]]
    ca, na, nr, rg = oracle.ack_report(words_of([0, 1, 1]), 3, 8)
    assert (ca, na, nr) == (0, 2, 1) and rg.tolist() == [[1, 3]]
    ca, na, nr, rg = oracle.ack_report(words_of([1] * 70), 70, 8)
    assert (ca, na, nr) == (70, 70, 0)
    ca, na, nr, rg = oracle.ack_report(words_of([0] * 40), 40, 8)
    assert (ca, na, nr) == (0, 0, 0)
    # a run across a word boundary; garbage above n_bits is ignored; more runs than room
    bits = [1] * 30 + [0] + [1] * 5 + [0, 1, 0, 1, 0, 1]
    w = words_of(bits).copy()
    w[-1] |= np.uint32(0xFFFFFFFF) << np.uint32(len(bits) - 32)
    ca, na, nr, rg = oracle.ack_report(w, len(bits), 2)
    assert (ca, na, nr) == (30, 38, 4) and rg.tolist() == [[31, 36], [37, 38]]
    assert oracle.ack_report(np.zeros(0, np.uint32), 0, 4)[:3] == (0, 0, 0)


@pytest.mark.parametrize("n_bits,density", [(1, 0.5), (31, 0.9), (32, 0.9), (33, 0.5), (1000, 0.97), (5000, 0.5), (4097, 0.999)])
def test_ack_report_against_numpy(n_bits, density):
    g = pl.rng(n_bits, 3)
    for trial in range(6):
        bits = (g.random(n_bits) < density).astype(np.uint8)
        if trial == 0:
            bits[: n_bits // 2] = 1
        b = np.zeros((n_bits + 31) // 32 * 32, dtype=np.uint8)
        b[:n_bits] = bits
        words = np.packbits(b, bitorder="little").view(np.uint32)
        cum, cnt, runs = numpy_ack(bits)
        ca, na, nr, rg = oracle.ack_report(words, n_bits, len(runs) + 3)
        assert (ca, na, nr) == (cum, cnt, len(runs))
        assert np.array_equal(rg.astype(np.int64), runs)


def _slot_words(rows, bits_per_slot):
    """rows: one list of 0/1 per slot (shorter than the window = zero padded)."""
    b = np.zeros((len(rows), bits_per_slot), dtype=np.uint8)
    for i, r in enumerate(rows):
        b[i, :len(r)] = r
    return np.packbits(b.reshape(-1), bitorder="little").view(np.uint32).copy()


def test_message_status_hand_cases():
    """Section 3.2's message window: hand-worked slots of 64 bits."""
    rows = [
        [1, 1, 1, 0, 1],            # count 5 known: cumulative 3, applied 4, incomplete
        [1] * 5,                    # count 5: complete
        [1] * 5 + [1, 1],           # count 5 with stray bits above it: still complete, strays not counted
        [1] * 40,                   # count unknown (0): window-wide reading, never complete
        [],                         # empty slot, count 7
        [1] * 64,                   # full window, count 64
        [0] + [1] * 63,             # first bit missing
        [1] * 33 + [0] + [1] * 4,   # hole right after a word boundary
    ]
    counts = [5, 5, 5, 0, 7, 64, 64, 38]
    w = _slot_words(rows, 64)
    before = w.copy()
    st = oracle.message_status(w, counts, 64)
    assert st.tolist() == [[3, 4, 0, 0], [5, 5, 1, 0], [5, 5, 1, 0], [40, 40, 0, 0], [0, 0, 0, 0],
                           [64, 64, 1, 0], [0, 63, 0, 0], [33, 37, 0, 0]]
    assert np.array_equal(w, before), "without recycling the bitmap is only read"
    st2 = oracle.message_status(w, counts, 64, recycle=True)
    assert np.array_equal(st2, st)
    after = w.view(np.uint64)
    for i in range(len(rows)):
        assert after[i] == (0 if st[i, 2] else before.view(np.uint64)[i]), i   # strays of slot 2 are cleared too
    # a count beyond the window is clamped to the window
    assert oracle.message_status(_slot_words([[1] * 32], 32), [100], 32).tolist() == [[32, 32, 1, 0]]


@pytest.mark.parametrize("bits_per_slot,n_slots", [(32, 5), (256, 128), (96, 7), (2048, 3)])
def test_message_status_against_numpy(bits_per_slot, n_slots):
    """An independent reading of the same definition with array operations."""
    g = pl.rng(bits_per_slot, n_slots)
    for trial in range(4):
        counts = g.integers(0, bits_per_slot + 1, n_slots).astype(np.uint32)
        bits = (g.random((n_slots, bits_per_slot)) < [0.5, 0.9, 0.99, 1.0][trial]).astype(np.uint8)
        bits[::3] = 1                                     # every third slot has everything
        bits[1::3, : bits_per_slot // 3] = 1              # a cumulative prefix
        words = np.packbits(bits.reshape(-1), bitorder="little").view(np.uint32).copy()
        limit = np.where(counts == 0, bits_per_slot, counts)
        below = np.arange(bits_per_slot)[None, :] < limit[:, None]
        seen = bits.astype(bool) & below
        missing = ~bits.astype(bool) & below
        cum = np.where(missing.any(1), missing.argmax(1), limit)
        cnt = seen.sum(1)
        done = (counts != 0) & (cnt == limit)
        st = oracle.message_status(words, counts, bits_per_slot, recycle=True)
        assert np.array_equal(st[:, 0], cum) and np.array_equal(st[:, 1], cnt)
        assert np.array_equal(st[:, 2], done.astype(np.uint32)) and not st[:, 3].any()
        kept = bits.copy()
        kept[done] = 0
        assert np.array_equal(words, np.packbits(kept.reshape(-1), bitorder="little").view(np.uint32))


@pytest.mark.parametrize("dtype,op", [(F32, SUM), (BF16, SUM), (BF16, MAX), (F32, COPY)])
@pytest.mark.parametrize("threads", [1, 3, 16])
def test_threaded_baseline_equals_the_definition(dtype, op, threads):
    """The multi-core CPU baseline is the definition on more cores: same bytes, same bitmap, for a
    reordered stream with duplicates, relayed chunks and a call cut in two."""
    kw = dict(R=4, M=4 * 16 * 256, C=256, dtype=dtype, paths=5, window=9, dup=0.3, dist="uniform")
    for relay in (False, True):
        w = wl.ring_share("thr", 11, relay=relay, **kw)
        a1, o1, s1 = w.acc.copy(), np.zeros(w.out_bytes, np.uint8), oracle.new_seen(w.n_bits)
        a2, o2, s2 = w.acc.copy(), np.zeros(w.out_bytes, np.uint8), oracle.new_seen(w.n_bits)
        for ph in w.phases:
            this_op = COPY if ph.op == COPY else op
            n1 = oracle.apply(a1, o1, w.recv_stage, ph.descs, s1, dtype, this_op)
            cut = len(ph.descs) // 3
            n2 = oracle.apply_threaded(a2, o2, w.recv_stage, ph.descs[:cut], s2, dtype, this_op, threads)
            n2 += oracle.apply_threaded(a2, o2, w.recv_stage, ph.descs[cut:], s2, dtype, this_op, threads)
            assert n1 == n2 == ph.n_unique
        assert np.array_equal(a1.view(np.uint8), a2.view(np.uint8)) and np.array_equal(o1, o2) and np.array_equal(s1, s2)
    d = w.phases[0].descs.copy()
    d["seq"][0] = w.n_bits + 5
    with pytest.raises(oracle.OraclePrecondition):
        oracle.apply_threaded(a2, o2, w.recv_stage, d, oracle.new_seen(w.n_bits), dtype, op, threads)


# --- P7: a chunk that never arrives ------------------------------------------------

def test_missing_chunk_leaves_hole_and_clear_bit():
    kw = dict(R=4, M=4 * 8 * 128, C=128, dtype=F32, paths=3, window=6, dup=0.2, dist="uniform")
    w = wl.ring_share("p7", 4, **kw)
    full = run_workload(w)
    lost = int(w.extra["logical"][0][5]["seq"])
    lg = w.extra["logical"][0][5]
    ph = w.phases[0]
    ph.descs = ph.descs[ph.descs["seq"] != lost]
    acc, out, bm = run_workload(w)
    assert not (bm[lost >> 5] >> (lost & 31)) & 1
    assert sum(bin(int(x)).count("1") for x in bm) == sum(bin(int(x)).count("1") for x in full[2]) - 1
    lo, n = int(lg["dst_off"]) // 4, int(lg["len"]) // 4
    hole = np.zeros(len(acc), dtype=bool)
    hole[lo:lo + n] = True
    # reduce-scatter never revisits the segment, but allgather may overwrite it later:
    ag_dst = w.extra["logical"][1]["dst_off"]
    if not np.any((ag_dst >= lo * 4) & (ag_dst < (lo + n) * 4)):
        assert np.array_equal(acc[hole], w.acc[hole])
    assert np.array_equal(acc[~hole], full[0][~hole])
    oo = int(lg["out_off"])
    assert np.all(out[oo:oo + n * 4] == 0xA5)
    mask = np.ones(len(out), dtype=bool)
    mask[oo:oo + n * 4] = False
    assert np.array_equal(out[mask], full[1][mask])


# --- preconditions the oracle asserts ------------------------------------------------

def _one(src=0, dst=0, out=NO_FORWARD, ln=64, seq=0):
    d = np.zeros(1, dtype=DESC)
    d[0] = (src, dst, out, ln, seq)
    return d


def test_oracle_rejects_bad_records():
    acc = np.zeros(64, np.float32)
    recv = np.zeros(64, np.float32)
    out = np.zeros(256, np.uint8)
    seen = oracle.new_seen(4)
    cases = [(_one(seq=4), -2), (_one(src=8), -3), (_one(dst=4), -3), (_one(ln=62), -3),
             (_one(out=8), -3), (_one(src=256 - 48), -4), (_one(dst=256), -4), (_one(out=224), -4)]
    for d, code in cases:
        with pytest.raises(oracle.OraclePrecondition) as e:
            oracle.apply(acc, out, recv, d, seen, F32, SUM)
        assert e.value.code == code, (d, code)
    with pytest.raises(oracle.OraclePrecondition):
        oracle.apply(acc, None, recv, _one(out=0), seen, F32, SUM)  # forward without a staging buffer
    assert not seen.any() and not acc.any()
    # same seq, different destination / different payload; different seq, overlapping destination
    two = np.concatenate([_one(src=0, dst=0, seq=1), _one(src=64, dst=64, seq=1)])
    with pytest.raises(oracle.OraclePrecondition) as e:
        oracle.apply(acc, out, recv, two, seen, F32, SUM)
    assert e.value.code == -5
    recv2 = recv.copy(); recv2[16] = 1.0
    two = np.concatenate([_one(src=0, dst=0, seq=1), _one(src=64, dst=0, seq=1)])
    with pytest.raises(oracle.OraclePrecondition) as e:
        oracle.apply(acc, out, recv2, two, seen, F32, SUM)
    assert e.value.code == -5
    two = np.concatenate([_one(src=0, dst=0, seq=1), _one(src=64, dst=32, seq=2)])
    with pytest.raises(oracle.OraclePrecondition) as e:
        oracle.apply(acc, out, recv, two, seen, F32, SUM)
    assert e.value.code == -6
    two = np.concatenate([_one(src=0, dst=0, out=0, seq=1), _one(src=64, dst=64, out=16, seq=2)])
    with pytest.raises(oracle.OraclePrecondition) as e:
        oracle.apply(acc, out, recv, two, seen, F32, SUM)
    assert e.value.code == -6
    assert oracle.apply(acc, out, recv, np.zeros(0, dtype=DESC), seen, F32, SUM) == 0


def test_zero_length_and_tail_records():
    acc = np.arange(32, dtype=np.float32)
    recv = np.ones(32, np.float32)
    out = np.zeros(128, np.uint8)
    d = np.concatenate([_one(src=0, dst=0, ln=0, seq=0), _one(src=16, dst=16, out=0, ln=20, seq=1)])
    seen = oracle.new_seen(2)
    assert oracle.apply(acc, out, recv, d, seen, F32, SUM) == 2
    expect = np.arange(32, dtype=np.float32)
    expect[4:9] += 1
    assert np.array_equal(acc, expect) and seen.all()
    assert np.array_equal(out[:20].view(np.float32), expect[4:9]) and not out[20:].any()
