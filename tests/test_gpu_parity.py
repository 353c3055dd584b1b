"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs, element by element.  Integer, placement, dedup and copy results must be
bit-exact; fp32 combine 0 ulp; bf16 SUM is allowed 1 ulp by the stated target but is
asserted bit-exact here because both sides round fp32 -> bf16 once, to nearest even.
"""
import os
import sys

import numpy as np
import pytest
import torch

import oracle
from synth import payload as pl
from synth import workloads as wl
from synth.layout import DESC, NO_FORWARD, F32, BF16, F16, I32, SUM, MAX, MIN, COPY, PROD, ELEM_SIZE

from gpuhelp import DeviceRun, oracle_results, assert_same, to_dev, to_host
from ringloop import closed_loop_allreduce

pytestmark = pytest.mark.gpu

# Launch configurations every case runs under: the library's own choice, then (chunk_bytes, parts)
# pairs forcing one workgroup per record and 2, 5 and 16 workgroups per record (calls of at most
# 2048 single-record tiles; otherwise `parts` is ignored and the call runs unsplit).
LAUNCHES = [None, (0, 1), (0, 2), (0, 5), (0, 16)]


def say(*a):
    print(*a, file=sys.stderr, flush=True)


def check_workload(pkg, w, opts=None, checked=True, split=None):
    eacc, eout, ebm = oracle_results(w)  # first: the oracle also validates the records
    run = DeviceRun(w, opts=opts)
    run.run_phases(checked=checked, split=split)
    acc, out, bm, rej = run.results()
    assert rej == 0
    assert pkg.uccl_claim_timeouts() == 0
    assert_same(bm, ebm, "bitmap")
    assert_same(acc, eacc, "acc")
    if eout is not None:
        assert_same(out, eout, "out_stage")


# ---- the five recipes at sizes the oracle finishes in seconds, every launch configuration ------

@pytest.mark.parametrize("opts", LAUNCHES)
def test_config1_full_size(gpu_lib, opts):
    say("config1 full size, launch", opts)
    check_workload(gpu_lib, wl.config1(seed=1), opts)


@pytest.mark.parametrize("opts", LAUNCHES)
@pytest.mark.parametrize("seed", [1, 2])
def test_config2_recipe_reduced(gpu_lib, opts, seed):
    say("config2 16 MiB, launch", opts, "seed", seed)
    check_workload(gpu_lib, wl.config2(seed=seed, M=16 << 20), opts)


@pytest.mark.parametrize("opts", LAUNCHES)
def test_config3_recipe_reduced(gpu_lib, opts):
    say("config3 32 MiB, launch", opts)
    check_workload(gpu_lib, wl.config3(seed=3, M=32 << 20), opts)


@pytest.mark.parametrize("opts", LAUNCHES)
def test_config4_recipe_reduced(gpu_lib, opts):
    say("config4 max 2 MiB per source, launch", opts)
    w = wl.config4(seed=2, max_bytes=2 << 20)
    dst = torch.full((w.acc.nbytes + 512,), 0xEE, dtype=torch.uint8, device="cuda")
    recv = to_dev(w.recv_stage)
    d = to_dev(w.phases[0].descs)
    bm = torch.zeros((w.n_bits + 31) // 32, dtype=torch.int32, device="cuda")
    rej = torch.zeros(1, dtype=torch.int32, device="cuda")
    if opts is None:
        gpu_lib.uccl_chunk_scatter_checked(dst[256:256 + w.acc.nbytes], recv, d, len(w.phases[0].descs), bm,
                                           n_rejected=rej, n_bits=w.n_bits)
    else:
        gpu_lib.uccl_chunk_scatter_opts(dst[256:256 + w.acc.nbytes], recv, d, len(w.phases[0].descs), bm,
                                        n_rejected=rej, n_bits=w.n_bits, opts=opts)
    torch.cuda.synchronize()
    got = dst.cpu().numpy()
    edst = np.zeros(w.acc.nbytes, dtype=np.uint8)
    seen = oracle.new_seen(w.n_bits)
    oracle.scatter(edst, w.recv_stage, w.phases[0].descs, seen)
    assert rej.item() == 0
    assert_same(got[256:256 + w.acc.nbytes], edst, "dst")
    assert_same(got[256:256 + w.acc.nbytes], np.concatenate(w.extra["sources"]), "dst vs sources")
    assert np.all(got[:256] == 0xEE) and np.all(got[256 + w.acc.nbytes:] == 0xEE)
    assert_same(bm.cpu().numpy().view(np.uint32), oracle.pack_bitmap(seen), "bitmap")


def test_config5_recipe_batched_and_per_message(gpu_lib):
    """Small-message regime: 60 messages, applied (a) one message per pair of calls and
    (b) many messages per call; both must equal the oracle applied message by message."""
    w, msgs = wl.config5(seed=4, n_msgs=60)
    eacc = w.acc.copy()
    eout = np.full(w.out_bytes, 0xA5, dtype=np.uint8)
    seen = oracle.new_seen(w.n_bits)
    for m in msgs:
        oracle.apply(eacc, eout, w.recv_stage, m["rs"], seen, F32, SUM)
        oracle.apply(eacc, eout, w.recv_stage, m["ag"], seen, F32, COPY)
    ebm = oracle.pack_bitmap(seen)
    for mode in ("per-message", "per-message-split", "batched", "batched-hint"):
        say("config5", mode)
        run = DeviceRun(w, opts={"batched-hint": (4096, 0), "per-message-split": (0, 4)}.get(mode))
        if mode.startswith("per-message"):
            for m in msgs:
                run.apply(to_dev(m["rs"]), len(m["rs"]), SUM)
                run.apply(to_dev(m["ag"]), len(m["ag"]), COPY)
        else:
            for lo in range(0, len(msgs), 25):
                rs = np.concatenate([m["rs"] for m in msgs[lo:lo + 25]])
                ag = np.concatenate([m["ag"] for m in msgs[lo:lo + 25]])
                run.apply(to_dev(rs), len(rs), SUM)
                run.apply(to_dev(ag), len(ag), COPY)
        torch.cuda.synchronize()
        acc, out, bm, rej = run.results()
        assert rej == 0 and gpu_lib.uccl_claim_timeouts() == 0
        assert_same(bm, ebm, "bitmap")
        assert_same(acc, eacc, "acc")
        assert_same(out, eout, "out")


@pytest.mark.parametrize("hint,per_segment",
                         [(h, n) for n in (10, 100) for h in (512, 1024, 2048, 4096, 8192, 16384, 1 << 20)] +
                         [(16384, 2800), (1 << 20, 2800)])   # the largest call only where it selects another kernel
def test_every_tile_size(gpu_lib, hint, per_segment):
    """The chunk size given with the call and the record count only choose the kernel and how many
    records a workgroup takes; the result never changes.  Calls of about 35 records (one small
    workgroup per record for chunk sizes up to 16 KiB; records cut into parts for the largest),
    of about 350 records (tiles of 32, 32, 16, 8, 4 records per workgroup; one record per
    workgroup from 16 KiB on), and of about 9 700 records (tiles of 2 records too)."""
    C = 5008
    w = wl.ring_share("tiles", 13, R=4, M=4 * ((per_segment - 1) * C + 1040), C=C, dtype=BF16, paths=5, window=11,
                      dup=0.2, dist="normal")
    check_workload(gpu_lib, w, (hint, 0))


def test_very_many_tiny_records_without_hint(gpu_lib):
    """150 000 records of 64 bytes, no chunk-size hint: the tile grows with the record count
    (every tile size of the heuristic is crossed by cutting the call at 5 000 / 20 000 / 100 000)."""
    n, C = 150000, 64
    g = pl.rng(31, 1)
    seq = np.concatenate([g.permutation(n), g.integers(0, n, 6000)])
    seq = seq[g.permutation(len(seq))]
    d = np.zeros(len(seq), dtype=DESC)
    d["src_off"] = np.arange(len(seq), dtype=np.uint64) * C
    d["dst_off"] = seq.astype(np.uint64) * C
    d["out_off"] = np.where(seq % 2 == 0, seq.astype(np.uint64) * C, NO_FORWARD)
    d["len"], d["seq"] = C, seq
    vals = pl.uniform_f32(31, 2, n * C // 4).reshape(n, C // 4)
    recv = vals[seq].reshape(-1).copy()
    w = wl.Workload("tiny", F32, pl.uniform_f32(31, 3, n * C // 4), recv, n * C, n,
                    [wl.Phase("p", SUM, d, n, n * C, 0)])
    check_workload(gpu_lib, w, None, checked=False, split=lambda m: [5000, 25000, 125000])
    check_workload(gpu_lib, w, None, checked=True)


# ---- ops, dtypes, ragged tails, odd lengths ------------------------------------------

@pytest.mark.parametrize("opts", LAUNCHES)
@pytest.mark.parametrize("dtype", [F32, BF16, F16, I32])
@pytest.mark.parametrize("op", [SUM, MAX, MIN, COPY, PROD])
def test_ops_dtypes_ragged(gpu_lib, opts, dtype, op):
    say("ops ragged", opts, dtype, op)
    C = 20000 - 20000 % 16 + 16  # 20000: many 16-byte vectors plus trips that do not divide evenly
    dist = "normal" if dtype == BF16 else "uniform"
    w = wl.ring_share("ragged", 11, R=4, M=4 * (5 * C + 4112), C=C, dtype=dtype, paths=7, window=9,
                      dup=0.15, dist=dist, op=op, allgather=True)
    check_workload(gpu_lib, w, opts)


def _records(rows):
    d = np.zeros(len(rows), dtype=DESC)
    for k, r in enumerate(rows):
        d[k] = r
    return d


@pytest.mark.parametrize("opts", LAUNCHES)
@pytest.mark.parametrize("dtype,op", [(F32, SUM), (BF16, SUM), (BF16, MAX), (F32, COPY), (BF16, COPY), (F16, PROD),
                                      (I32, MIN)])
def test_lengths_not_multiple_of_16(gpu_lib, opts, dtype, op):
    """len is any multiple of the element size, including 0."""
    es = ELEM_SIZE[dtype]
    lens = [0, es, 2 * es, 16 - es, 16, 16 + es, 48 - es, 1024 + 3 * es, 4096 + 16 - es, 9 * 1024 + es, 70000 + es]
    slot = 70016 + 64
    rows, n = [], len(lens)
    for k, ln in enumerate(lens):
        rows.append((k * slot, ((n - 1 - k) * slot), k * slot if k % 2 else NO_FORWARD, ln, k))
    rows.append((n * slot, (n - 1 - 3) * slot, 3 * slot, lens[3], 3))  # a duplicate of record 3
    d = _records(rows)
    nel = (n + 1) * slot // ELEM_SIZE[dtype]
    acc0 = wl._draw("normal" if dtype == BF16 else "uniform", dtype, 5, 1, nel)
    recv = wl._draw("normal" if dtype == BF16 else "uniform", dtype, 5, 2, nel)
    recv.view(np.uint8)[n * slot:n * slot + lens[3]] = recv.view(np.uint8)[3 * slot:3 * slot + lens[3]]
    w = wl.Workload("odd", dtype, acc0, recv, (n + 1) * slot, n, [wl.Phase("p", op, d, n, sum(lens), 0)])
    check_workload(gpu_lib, w, opts)
    check_workload(gpu_lib, w, opts, checked=False)


@pytest.mark.parametrize("opts", LAUNCHES)
def test_scatter_any_byte_length(gpu_lib, opts):
    """The all-to-all scatter is a byte copy: any length, including odd ones."""
    lens = [0, 1, 2, 3, 15, 16, 17, 31, 33, 1000, 4097, 65535, 70001]
    slot = 70016
    n = len(lens)
    d = _records([(k * slot, (n - 1 - k) * slot, NO_FORWARD, ln, k) for k, ln in enumerate(lens)]
                 + [((n + j) * slot, (n - 1 - 12) * slot, NO_FORWARD, lens[12], 12) for j in range(3)])
    recv = pl.rng(7, 7).integers(0, 256, (n + 3) * slot).astype(np.uint8)
    for j in range(3):
        recv[(n + j) * slot:(n + j) * slot + lens[12]] = recv[12 * slot:12 * slot + lens[12]]
    dst0 = np.full(n * slot, 0x5C, dtype=np.uint8)
    dst = to_dev(dst0)
    bm = torch.zeros(1, dtype=torch.int32, device="cuda")
    for checked in (True, False):
        if opts is not None:
            gpu_lib.uccl_chunk_scatter_opts(dst, to_dev(recv), to_dev(d), len(d), bm, n_bits=n if checked else None,
                                            opts=opts)
        elif checked:
            gpu_lib.uccl_chunk_scatter_checked(dst, to_dev(recv), to_dev(d), len(d), bm, n_bits=n)
        else:
            gpu_lib.uccl_chunk_scatter(dst, to_dev(recv), to_dev(d), len(d), bm)
        torch.cuda.synchronize()
        edst = dst0.copy()
        seen = oracle.new_seen(n)
        assert oracle.scatter(edst, recv, d, seen) == n
        assert_same(dst.cpu().numpy(), edst, "dst")
        assert_same(bm.cpu().numpy().view(np.uint32), oracle.pack_bitmap(seen), "bitmap")
        dst = to_dev(dst0)
        bm.zero_()
    assert gpu_lib.uccl_claim_timeouts() == 0


@pytest.mark.parametrize("opts", LAUNCHES)
@pytest.mark.parametrize("dtype,op", [(BF16, SUM), (F32, MAX), (F32, COPY)])
def test_forward_only_records(gpu_lib, opts, dtype, op):
    """Intermediate reduce-scatter steps flagged forward-only: staging gets the combined
    value, the accumulator keeps its bytes; ragged chunk sizes."""
    C = 12304
    w = wl.ring_share("relay", 17, R=5, M=5 * (4 * C + 2064), C=C, dtype=dtype, paths=6, window=8, dup=0.15,
                      dist="uniform" if dtype == F32 else "normal", op=op, relay=True)
    check_workload(gpu_lib, w, opts)
    check_workload(gpu_lib, w, opts, checked=False)


def test_closed_loop_ring_with_relay(gpu_lib):
    R, n, C = 4, 4 * 5000, 4096
    x = pl.normal_bf16(8, 9, R * n).reshape(R, n)
    got = closed_loop_allreduce(GpuBackend(gpu_lib), x, BF16, C, seed=5, paths=4, window=None, dup=0.1, relay=True)
    assert_same(got, oracle.ring_allreduce(x, BF16, SUM), "closed loop with forward-only steps")


def test_empty_call_and_all_duplicates(gpu_lib):
    w = wl.ring_share("e", 1, R=3, M=3 * 4096, C=1024, dtype=F32, paths=2, window=None, dup=0.5,
                      dist="uniform", allgather=False)
    run = DeviceRun(w)
    run.apply(run.descs[0], 0, SUM)
    torch.cuda.synchronize()
    acc, out, bm, _ = run.results()
    assert_same(acc, w.acc, "acc after empty call")
    assert not bm.any()
    run.run_phases()
    first = run.results()
    run.run_phases()  # the same records again: every one is now a duplicate
    again = run.results()
    for a, b in zip(first[:3], again[:3]):
        if a is not None:
            assert_same(a, b, "second pass changes nothing")
    eacc, eout, ebm = oracle_results(w)
    assert_same(first[0], eacc, "acc")
    # after a reset the records apply again (SUM adds the payload a second time)
    run.reset()
    run.run_phases()
    acc2 = run.results()[0]
    seen = oracle.new_seen(w.n_bits)
    oracle.apply(eacc, eout, w.recv_stage, w.phases[0].descs, seen, F32, SUM)
    assert_same(acc2, eacc, "acc after reset + reapply")


# ---- exactly-once under concurrency ---------------------------------------------------

@pytest.mark.parametrize("opts", LAUNCHES)
@pytest.mark.parametrize("dtype", [F32, BF16])
def test_exactly_once_many_copies_everywhere(gpu_lib, opts, dtype):
    """Payload all ones, acc zero, SUM; every seq is repeated many times: adjacent records
    (same wavefront, same bitmap word), far apart (different workgroups), and across two
    calls.  A double apply shows as 2, a lost chunk as 0.  With records cut into parts, every
    part of every copy has to learn the one decision taken for its record."""
    es = ELEM_SIZE[dtype]
    C, n = 4096, 96
    g = pl.rng(21, LAUNCHES.index(opts))
    arr = np.concatenate([np.repeat(np.arange(n), 3), np.arange(n), g.integers(0, n, 700), np.repeat(np.arange(8), 40)])
    arr = np.concatenate([arr[:300], g.permutation(arr[300:])])
    d = np.zeros(len(arr), dtype=DESC)
    d["src_off"] = np.arange(len(arr), dtype=np.uint64) * C
    d["dst_off"] = arr.astype(np.uint64) * C
    d["out_off"] = arr.astype(np.uint64) * C
    d["len"] = C
    d["seq"] = arr
    one = pl.ints_as(np.ones(1, dtype=np.int64), dtype)[0]
    recv = np.full(len(arr) * C // es, one, dtype=pl.np_dtype(dtype))
    acc0 = np.zeros(n * C // es, dtype=pl.np_dtype(dtype))
    w = wl.Workload("once", dtype, acc0, recv, n * C, n, [wl.Phase("p", SUM, d, n, n * C, 0)])
    run = DeviceRun(w, opts=opts)
    run.run_phases(split=lambda m: [m // 3, m // 2])
    acc, out, bm, rej = run.results()
    assert rej == 0 and gpu_lib.uccl_claim_timeouts() == 0
    assert np.all(acc == one), f"{np.count_nonzero(acc != one)} elements are not exactly 1"
    assert np.array_equal(out.view(acc.dtype), acc)
    assert sum(bin(int(x)).count("1") for x in bm) == n


DIFFER = [(None, 4096), (None, 65536), ((0, 1), 4096), ((0, 1), 65536), ((0, 5), 4096), ((0, 5), 65536),
          ((0, 16), 65536), ((4096, 0), 4096), ((65536, 0), 65536)]


@pytest.mark.parametrize("opts,C", DIFFER)
def test_copies_that_differ_one_wins_whole(gpu_lib, opts, C):
    """Which copy of a retransmitted chunk is applied is not defined; that it is ONE copy, whole, is.
    Here the copies of a chunk break the rule that they are identical: copy j carries the value
    j + 1 everywhere.  With acc zero and SUM every destination chunk must end up constant, equal
    to one of its copies' values (a mix of two copies, or a sum of two, shows), the staging copy
    equal to it; the oracle is not asked (it rejects such input), the check is closed form."""
    n, copies = 48, 3
    g = pl.rng(23, DIFFER.index((opts, C)))
    arr = g.permutation(np.repeat(np.arange(n), copies))
    which = np.zeros(len(arr), dtype=np.int64)            # arrival k is copy which[k] of chunk arr[k]
    seen = np.zeros(n, dtype=np.int64)
    for k, a in enumerate(arr):
        which[k] = seen[a]
        seen[a] += 1
    d = np.zeros(len(arr), dtype=DESC)
    d["src_off"] = np.arange(len(arr), dtype=np.uint64) * C
    d["dst_off"] = arr.astype(np.uint64) * C
    d["out_off"] = arr.astype(np.uint64) * C
    d["len"] = C
    d["seq"] = arr
    recv = np.repeat((which + 1).astype(np.float32), C // 4)
    acc0 = np.zeros(n * C // 4, dtype=np.float32)
    w = wl.Workload("differ", F32, acc0, recv, n * C, n, [wl.Phase("p", SUM, d, n, n * C, 0)])
    run = DeviceRun(w, opts=opts)
    run.run_phases(split=lambda m: [m // 2])
    acc, out, bm, rej = run.results()
    assert rej == 0 and gpu_lib.uccl_claim_timeouts() == 0
    chunks = acc.reshape(n, -1)
    assert np.all(chunks == chunks[:, :1]), "a destination chunk mixes two copies"
    assert set(np.unique(chunks[:, 0]).tolist()) <= {1.0, 2.0, 3.0}, np.unique(chunks[:, 0])
    assert np.array_equal(out.view(np.float32), acc)
    assert sum(bin(int(x)).count("1") for x in bm) == n


@pytest.mark.parametrize("opts", [None, (0, 4)])
def test_split_calls_equal_single_call(gpu_lib, opts):
    w = wl.config2(seed=5, M=8 << 20)
    g = pl.rng(6, 6)
    check_workload(gpu_lib, w, opts, split=lambda m: sorted(g.choice(np.arange(1, m), 5, replace=False).tolist()))


def test_missing_chunk_leaves_hole(gpu_lib):
    w = wl.config1(seed=2)
    lost = int(w.extra["logical"][0][9]["seq"])
    ph = w.phases[0]
    ph.descs = ph.descs[ph.descs["seq"] != lost]
    check_workload(gpu_lib, w)
    run = DeviceRun(w)
    run.run_phases()
    bm = run.results()[2]
    assert not (bm[lost >> 5] >> (lost & 31)) & 1


# ---- checked entry point -----------------------------------------------------------------

def test_checked_rejects_bad_records_and_moves_nothing(gpu_lib):
    n_bits, C = 8, 256
    acc0 = pl.uniform_f32(1, 1, 4 * C // 4)
    recv = pl.uniform_f32(1, 2, 8 * C // 4)
    good = (0, 0, 0, C, 0)
    bad = [
        (C, C, NO_FORWARD, C, 8),            # seq out of range
        (C + 4, C, NO_FORWARD, C, 1),        # misaligned source
        (C, C + 8, NO_FORWARD, C, 1),        # misaligned destination
        (C, C, 8, C, 1),                     # misaligned forward
        (C, C, NO_FORWARD, C - 2, 1),        # len not a multiple of 4
        (8 * C - 16, C, NO_FORWARD, C, 1),   # source runs past recv_stage
        (C, 4 * C - 16, NO_FORWARD, C, 1),   # destination runs past acc
        (C, C, 2 * C - 16, C, 1),            # forward runs past out_stage
        (1 << 62, C, NO_FORWARD, C, 1),      # absurd offsets
        (C, (1 << 64) - 16, NO_FORWARD, 32, 1),
    ]
    d = _records([good] + bad + [(2 * C, 2 * C, C, C, 2)])
    w = wl.Workload("bad", F32, acc0, recv, 2 * C, n_bits, [wl.Phase("p", SUM, d, 2, 2 * C, 0)])
    for opts in LAUNCHES:
        run = DeviceRun(w, opts=opts)
        run.run_phases()
        acc, out, bm, rej = run.results()
        assert rej == len(bad), opts   # a rejected record is counted once however many parts look at it
        assert bm[0] == 0b101
        exp = acc0.copy()
        exp[:C // 4] += recv[:C // 4]
        exp[2 * C // 4:3 * C // 4] += recv[2 * C // 4:3 * C // 4]
        assert_same(acc, exp, "acc")
        assert_same(out.view(np.float32), np.concatenate([exp[:C // 4], exp[2 * C // 4:3 * C // 4]]), "out")
    # a forward with no staging buffer is rejected, not dereferenced; scatter rejects forwards
    run = DeviceRun(wl.Workload("nofwd", F32, acc0, recv, 0, n_bits, [wl.Phase("p", SUM, _records([good]), 1, C, 0)]))
    run.run_phases()
    acc, _, bm, rej = run.results()
    assert rej == 1 and bm[0] == 0
    assert_same(acc, acc0, "acc untouched")
    dst = to_dev(acc0)
    bmt = torch.zeros(1, dtype=torch.int32, device="cuda")
    rejt = torch.zeros(1, dtype=torch.int32, device="cuda")
    gpu_lib.uccl_chunk_scatter_checked(dst, to_dev(recv), to_dev(_records([good])), 1, bmt, n_rejected=rejt, n_bits=8)
    torch.cuda.synchronize()
    assert rejt.item() == 1 and bmt.item() == 0
    assert_same(to_host(dst, np.float32), acc0, "dst untouched")


# ---- numerics special values ---------------------------------------------------------------

def test_special_values_bit_exact(gpu_lib):
    """Subnormals are kept, infinities propagate, +0 + -0 = +0, MAX/MIN tie rule; NaN results
    are compared as NaN-ness only (NaN payloads are not fixed by the method)."""
    f = np.array([0, 0x80000000, 1, 2, 0x007FFFFF, 0x00800000, 0x807FFFFF, 0x3F800000, 0xBF800000,
                  0x7F7FFFFF, 0xFF7FFFFF, 0x7F800000, 0xFF800000, 0x33800000, 0x00000003], dtype=np.uint32)
    a32 = np.repeat(f, len(f)).view(np.float32)
    r32 = np.tile(f, len(f)).view(np.float32)
    h = np.array([0, 0x8000, 1, 2, 0x007F, 0x0080, 0x807F, 0x3F80, 0xBF80, 0x7F7F, 0xFF7F, 0x7F80, 0xFF80,
                  0x3B80, 0x3F81, 0x3B81, 0x3B7F, 0x7B00], dtype=np.uint16)
    a16, r16 = np.repeat(h, len(h)), np.tile(h, len(h))
    q = np.array([0, 0x8000, 1, 2, 0x03FF, 0x0400, 0x83FF, 0x3C00, 0xBC00, 0x7BFF, 0xFBFF, 0x7C00, 0xFC00,
                  0x1400, 0x3C01, 0x1401, 0x13FF, 0x6C00, 0x7BFE], dtype=np.uint16)  # binary16
    aq, rq = np.repeat(q, len(q)), np.tile(q, len(q))
    i = np.array([0, 1, -1, 2 ** 31 - 1, -2 ** 31, 65536, -65536, 46341, 3, -7], dtype=np.int32)
    ai, ri = np.repeat(i, len(i)), np.tile(i, len(i))
    for dtype, a, r in ((F32, a32, r32), (BF16, a16, r16), (F16, aq, rq), (I32, ai, ri)):
        es = ELEM_SIZE[dtype]
        n = len(a)
        pad = (-n * es) % 16
        nb = n * es + pad
        accp = np.zeros(nb // es, dtype=a.dtype); accp[:n] = a
        recvp = np.zeros(nb // es, dtype=a.dtype); recvp[:n] = r
        for op in (SUM, MAX, MIN, PROD):
            d = _records([(0, 0, 0, n * es, 0)])
            w = wl.Workload("sv", dtype, accp, recvp, nb, 1, [wl.Phase("p", op, d, 1, n * es, 0)])
            run = DeviceRun(w)
            run.run_phases()
            acc, out, _, rej = run.results()
            eacc, eout, _ = oracle_results(w)
            assert rej == 0
            wide = {F32: lambda x: x, BF16: lambda x: (x.astype(np.uint32) << 16).view(np.float32),
                    F16: lambda x: x.view(np.float16).astype(np.float32), I32: lambda x: x.astype(np.float32)}[dtype]
            nan = np.isnan(wide(eacc))
            assert np.array_equal(np.isnan(wide(acc)), nan)
            assert_same(acc[~nan], eacc[~nan], f"dtype {dtype} op {op}")
            assert_same(out[:n * es].view(a.dtype)[~nan[:n]], eacc[:n][~nan[:n]], "forward copy")


def test_bf16_sum_dense_pairs(gpu_lib):
    """Every bf16 pattern against 96 partner patterns (6.3 M pairs), bit-exact except NaN payloads."""
    allh = np.arange(1 << 16, dtype=np.uint16)
    partners = np.concatenate([pl.rng(3, 3).integers(0, 1 << 16, 64).astype(np.uint16),
                               np.array([0, 0x8000, 1, 0x8001, 0x7F, 0x80, 0x3F80, 0xBF80, 0x3B80, 0xBB80,
                                         0x7F7F, 0xFF7F, 0x7F80, 0xFF80, 0x3F81, 0x3B7F] * 2, dtype=np.uint16)])
    a = np.tile(allh, len(partners))
    r = np.repeat(partners, 1 << 16)
    n = len(a)
    d = _records([(k * (n // 8) * 2, k * (n // 8) * 2, NO_FORWARD, (n // 8) * 2, k) for k in range(8)])
    w = wl.Workload("pairs", BF16, a, r, 0, 8, [wl.Phase("p", SUM, d, 8, n * 2, 0)])
    run = DeviceRun(w)
    run.run_phases()
    acc = run.results()[0]
    eacc = oracle_results(w)[0]
    nan = np.isnan((eacc.astype(np.uint32) << 16).view(np.float32))
    assert np.array_equal(np.isnan((acc.astype(np.uint32) << 16).view(np.float32)), nan)
    assert_same(acc[~nan], eacc[~nan], "bf16 sum")


# ---- receiver feedback from the bitmap ---------------------------------------------------------

@pytest.mark.parametrize("n_bits,density", [(0, 0.5), (1, 1.0), (31, 0.9), (32, 1.0), (33, 0.5), (1024, 0.98),
                                            (1025, 0.5), (15360, 0.999), (100000, 0.7), (1 << 21, 0.9995)])
def test_ack_report(gpu_lib, n_bits, density):
    g = pl.rng(n_bits + 1, 4)
    for trial in range(3):
        bits = (g.random(n_bits) < density).astype(np.uint8)
        if trial == 1 and n_bits:
            bits[: n_bits * 2 // 3] = 1
        b = np.zeros((n_bits + 31) // 32 * 32 + 32, dtype=np.uint8)
        b[:n_bits] = bits
        b[n_bits:] = 1  # bits past the end must be ignored
        words = np.packbits(b, bitorder="little").view(np.uint32)
        for max_ranges in (0, 3, 4096):
            ca, na, nr, rg = oracle.ack_report(words, n_bits, max_ranges)
            rep = torch.full((32 + 16 * max_ranges + 16,), 0xCD, dtype=torch.uint8, device="cuda")
            gpu_lib.uccl_dedup_report(to_dev(words), n_bits, rep, max_ranges)
            torch.cuda.synchronize()
            raw = rep.cpu().numpy()
            hdr = raw[:32].view(np.uint64)
            assert (int(hdr[0]), int(hdr[1])) == (ca, na), (n_bits, trial)
            assert (int(raw[16:20].view(np.uint32)[0]), int(raw[20:24].view(np.uint32)[0])) == (nr, int(na == n_bits))
            got = raw[32:32 + 16 * min(nr, max_ranges)].view(np.uint64).reshape(-1, 2)
            assert np.array_equal(got, rg), (n_bits, trial, max_ranges)
            assert np.all(raw[32 + 16 * max_ranges:] == 0xCD), "wrote past the room given"


@pytest.mark.parametrize("bits_per_slot,n_slots", [(32, 1), (32, 9), (64, 130), (256, 128), (96, 1000), (2048, 5),
                                                   (1024, 64)])
def test_message_status(gpu_lib, bits_per_slot, n_slots):
    g = pl.rng(bits_per_slot * 7 + n_slots, 6)
    for trial, density in enumerate((0.5, 0.95, 0.999, 1.0)):
        counts = g.integers(0, bits_per_slot + 1, n_slots).astype(np.uint32)
        counts[::5] = bits_per_slot
        if n_slots > 2:
            counts[2] = bits_per_slot + 77  # clamped to the window
        bits = (g.random((n_slots, bits_per_slot)) < density).astype(np.uint8)
        bits[::3] = 1
        bits[1::3, : bits_per_slot // 3] = 1
        words = np.packbits(bits.reshape(-1), bitorder="little").view(np.uint32).copy()
        for recycle in (False, True):
            ewords = words.copy()
            est = oracle.message_status(ewords, counts, bits_per_slot, recycle)
            d_words = torch.cat([to_dev(words).view(torch.int32), torch.full((8,), 0x5A5A5A5A, dtype=torch.int32, device="cuda")])
            st = torch.full((n_slots * 4 + 4,), 0x7B7B7B7B, dtype=torch.int32, device="cuda")
            gpu_lib.uccl_message_status(d_words, to_dev(counts), n_slots, bits_per_slot, st, recycle)
            torch.cuda.synchronize()
            got = st.cpu().numpy().view(np.uint32)
            assert np.array_equal(got[:n_slots * 4].reshape(-1, 4), est), (trial, recycle)
            assert np.all(got[n_slots * 4:] == 0x7B7B7B7B), "wrote past the status rows"
            gw = d_words.cpu().numpy().view(np.uint32)
            assert np.array_equal(gw[:len(words)], ewords), (trial, recycle)
            assert np.all(gw[len(words):] == 0x5A5A5A5A), "wrote past the bitmap"
            if recycle and trial == 3:
                assert est[::5, 2].all() and not ewords.reshape(n_slots, -1)[::5].any()


def test_message_status_into_pinned_host_memory(gpu_lib):
    """The status rows may live in pinned host memory: the control path reads them without a copy."""
    g = pl.rng(55, 5)
    n_slots, per = 128, 256
    counts = g.integers(0, per + 1, n_slots).astype(np.uint32)
    bits = (g.random((n_slots, per)) < 0.97).astype(np.uint8)
    bits[::2] = 1
    words = np.packbits(bits.reshape(-1), bitorder="little").view(np.uint32).copy()
    est = oracle.message_status(words.copy(), counts, per)
    st = torch.zeros(n_slots * 4, dtype=torch.int32, pin_memory=True)
    gpu_lib.uccl_message_status(to_dev(words), to_dev(counts), n_slots, per, st, False)
    torch.cuda.synchronize()
    assert np.array_equal(st.numpy().view(np.uint32).reshape(-1, 4), est)


def test_message_window_over_small_allreduces(gpu_lib):
    """A connection's message window driven the way Section 3.1 lays it out: a message has at
    most 256 chunks and sits in one of 128 slots, the bit index of a chunk is slot * 256 + chunk
    sequence number, the last chunk's mark gives the count, and a slot is reused once its
    message is complete (status with recycling).  Three rounds over the window, each with other
    lengths, some chunks retransmitted, some messages finished only a round later."""
    from synth import header as hd
    C_ = 1024
    g = pl.rng(41, 41)
    n_slots, per = hd.MESSAGES_IN_FLIGHT, hd.CHUNKS_PER_MESSAGE
    acc = pl.uniform_f32(41, 1, n_slots * per * C_ // 4)
    eacc = acc.copy()
    d_acc = to_dev(acc)
    bitmap = torch.zeros(n_slots * per // 32, dtype=torch.int32, device="cuda")
    seen = oracle.new_seen(n_slots * per)
    counts = np.zeros(n_slots, dtype=np.uint32)    # the receiver's knowledge of message lengths
    pending = {}                                   # slot -> (chunks in the message, csns still to come)
    for rnd in range(3):
        held, hdrs = {}, []
        for slot in range(n_slots):
            if slot in pending:                    # the rest of an unfinished message arrives now
                total, missing = pending[slot]
                csn = np.array(sorted(missing), dtype=np.int64)
            else:
                total = int(g.integers(1, per + 1))
                csn = np.arange(total, dtype=np.int64)
                if slot % 17 == rnd:               # hold a quarter of this message back for a round
                    hold = set(g.choice(total, size=max(1, total // 4), replace=False).tolist())
                    held[slot] = (total, hold)
                    csn = np.array([c for c in csn if c not in hold], dtype=np.int64)
            again = csn[g.random(len(csn)) < 0.05]                      # retransmitted copies
            csn = g.permutation(np.concatenate([csn, again]))
            hdrs.append(hd.pack(7, slot, csn, csn == total - 1))
        pending = held
        hdr = np.concatenate(hdrs)
        hdr = hdr[g.permutation(len(hdr))]                              # paths interleave the messages
        seq = hd.seq_of(hdr)
        recv = pl.uniform_f32(41, 10 + rnd, n_slots * per * C_ // 4)    # payload of (slot, csn) at its own place
        d = np.zeros(len(hdr), dtype=DESC)
        d["src_off"] = seq.astype(np.uint64) * C_
        d["dst_off"] = seq.astype(np.uint64) * C_
        d["out_off"] = NO_FORWARD
        d["len"], d["seq"] = C_, seq
        oracle.apply(eacc, None, recv, d, seen, F32, SUM, check=False)
        gpu_lib.uccl_chunk_apply(d_acc, None, to_dev(recv), to_dev(d), len(d), bitmap, F32, SUM)
        counts = np.maximum(counts, hd.chunk_counts(hdr))
        ewords = oracle.pack_bitmap(seen)
        est = oracle.message_status(ewords, counts, per, recycle=True)
        st = torch.zeros(n_slots * 4, dtype=torch.int32, device="cuda")
        gpu_lib.uccl_message_status(bitmap, to_dev(counts), n_slots, per, st, True)
        torch.cuda.synchronize()
        assert np.array_equal(st.cpu().numpy().view(np.uint32).reshape(-1, 4), est), rnd
        assert np.array_equal(bitmap.cpu().numpy().view(np.uint32), ewords), rnd
        assert_same(d_acc.cpu().numpy().view(np.float32), eacc, f"acc after round {rnd}")
        done = est[:, 2] == 1
        assert set(np.flatnonzero(~done).tolist()) == set(pending), "exactly the held-back messages are incomplete"
        seen[:] = np.unpackbits(ewords.view(np.uint8), bitorder="little")[:len(seen)]   # recycled slots start over
        counts[done] = 0


def test_ack_report_after_a_lossy_phase(gpu_lib):
    """Drop some chunks of a reduce-scatter phase, apply the rest, ask for the report into pinned
    host memory: the holes are exactly the complement of cum_ack + ranges."""
    w = wl.config2(seed=8, M=16 << 20)
    ph = w.phases[0]
    lost = {3, 4, 200, 201, 202, 479}
    ph.descs = ph.descs[~np.isin(ph.descs["seq"], list(lost))]
    run = DeviceRun(w)
    run.apply(run.descs[0][:0], 0, SUM)
    run.apply(to_dev(ph.descs), len(ph.descs), SUM)
    rep = torch.zeros(32 + 16 * 16, dtype=torch.uint8, pin_memory=True)
    gpu_lib.uccl_dedup_report(run.bitmap, 480, rep, 16)
    torch.cuda.synchronize()
    raw = rep.numpy()
    cum, applied = int(raw[:8].view(np.uint64)[0]), int(raw[8:16].view(np.uint64)[0])
    nr = int(raw[16:20].view(np.uint32)[0])
    rg = raw[32:32 + 16 * nr].view(np.uint64).reshape(-1, 2)
    assert cum == 3 and applied == 480 - len(lost) and raw[20] == 0
    have = set(range(cum))
    for a, b in rg:
        have |= set(range(int(a), int(b)))
    assert have == set(range(480)) - lost


# ---- closed loop: the GPU path as every rank of a ring ------------------------------------------

class GpuBackend:
    def __init__(self, pkg):
        self.pkg = pkg

    def make_rank(self, acc_init, out_bytes, n_bits):
        return dict(acc=to_dev(acc_init), out=torch.zeros(out_bytes, dtype=torch.uint8, device="cuda"),
                    bm=torch.zeros((n_bits + 31) // 32, dtype=torch.int32, device="cuda"), n_bits=n_bits,
                    like=acc_init.dtype)

    def apply(self, h, recv, descs, dtype, op):
        self.pkg.uccl_chunk_apply_checked(h["acc"], h["out"], to_dev(recv), to_dev(descs), len(descs), h["bm"],
                                          dtype, op, n_bits=h["n_bits"])
        torch.cuda.synchronize()

    def read_out(self, h, off, nbytes):
        return h["out"][off:off + nbytes].cpu().numpy()

    def read_acc(self, h):
        return to_host(h["acc"], h["like"])


@pytest.mark.parametrize("dtype,R,n,C", [(F32, 8, 1 << 20, 64 << 10), (BF16, 4, 4 * 6000, 2048), (F32, 3, 3 * 1000, 528)])
def test_closed_loop_ring_matches_textbook(gpu_lib, dtype, R, n, C):
    """All R ranks run on the GPU path; first case is the 4 MiB fp32 / 64 KiB-chunk shape with
    true ring partial sums as payloads."""
    say("closed loop", dtype, R, n, C)
    x = pl.uniform_f32(8, 8, R * n).reshape(R, n) if dtype == F32 else pl.normal_bf16(8, 8, R * n).reshape(R, n)
    got = closed_loop_allreduce(GpuBackend(gpu_lib), x, dtype, C, seed=3, paths=4, window=None, dup=0.05)
    assert_same(got, oracle.ring_allreduce(x, dtype, SUM), "closed loop vs textbook ring")
    vals = pl.small_int(9, 9, R * n).reshape(R, n)
    got = closed_loop_allreduce(GpuBackend(gpu_lib), pl.ints_as(vals, dtype), dtype, C, seed=4, paths=4, dup=0.05)
    for r in range(R):
        assert_same(got[r], pl.ints_as(vals.sum(axis=0), dtype), "integer inputs: exact column sum")


@pytest.mark.parametrize("opts", [None, (0, 3)])
@pytest.mark.parametrize("scheme", ["window", "swift", "credit"])
def test_stream_from_control_path_model(gpu_lib, opts, scheme):
    """Arrival order from the discrete-event control-path model (power-of-two path choice, loss, fast
    and timeout retransmission; window-, delay- or credit-based sending) instead of the random-spray model."""
    from synth.control_sim import simulated_arrivals
    kw = dict(R=16, M=16 << 20, C=32 << 10, dtype=BF16, paths=256, window=1024, dup=0.02, dist="normal")
    lg = wl.ring_logical(16, 16 << 20, 32 << 10)
    arr = [simulated_arrivals(21, len(l), scheme=scheme, paths=256, loss=1 / 64, jitter_us=12.0, rto_us=90.0, stream=i)[0]
           for i, l in enumerate(lg[:2])]
    w = wl.ring_share("sim", 21, arrivals=arr, **kw)
    assert sum(len(a) for a in arr) > w.n_bits, "the model produced duplicates"
    check_workload(gpu_lib, w, opts)


def test_rejected_calls_leave_buffers_untouched(gpu_lib):
    """Host-side argument errors enqueue nothing: device buffers keep their bytes."""
    w = wl.config2(seed=2, M=4 << 20)
    run = DeviceRun(w)
    lib = gpu_lib.load()
    n = len(w.phases[0].descs)
    args = [run.acc.data_ptr(), run.out.data_ptr(), run.recv.data_ptr(), run.descs[0].data_ptr(), n,
            run.bitmap.data_ptr(), BF16, SUM, None]
    bad = [(0, None), (2, None), (3, None), (5, None), (6, 9), (7, 7), (0, args[0] + 8), (3, args[3] + 16 - 8),
           (5, args[5] + 2)]
    for pos, val in bad:
        a = list(args)
        a[pos] = val
        assert lib.uccl_chunk_apply(*a) in (gpu_lib.UCCL_EINVAL, gpu_lib.UCCL_EALIGN), (pos, val)
    torch.cuda.synchronize()
    acc, out, bm, _ = run.results()
    assert_same(acc, w.acc, "acc"); assert not bm.any() and np.all(out == 0xA5)


def test_c_abi_from_plain_c(gpu_lib):
    """A C program (no Python, no PyTorch) drives the library and checks it against the oracle."""
    import os
    import subprocess
    exe = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c_abi_check")
    assert os.path.exists(exe), "tests/c_abi_check is not built: run __graft_entry__.build()"
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and all(k in r.stdout for k in ("C ABI OK", "MORE OK", "FEED OK")), (r.returncode, r.stdout, r.stderr)
    print(r.stdout.strip())


def test_side_stream(gpu_lib):
    w = wl.config2(seed=9, M=8 << 20)
    run = DeviceRun(w)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    for ph, d in zip(w.phases, run.descs):
        run.apply(d, len(ph.descs), ph.op, stream=s)
    s.synchronize()
    acc, out, bm, rej = run.results()
    eacc, eout, ebm = oracle_results(w)
    assert_same(acc, eacc, "acc"); assert_same(out, eout, "out"); assert_same(bm, ebm, "bitmap")


# ---- randomized mix of every feature --------------------------------------------------------------

@pytest.mark.parametrize("dtype", [F32, BF16, F16, I32])
@pytest.mark.parametrize("parts", [0, 1, 3, 8])
def test_random_streams_all_features(gpu_lib, dtype, parts):
    """200 random small streams per (type, parts): odd and zero lengths, duplicates adjacent
    and far, forward / keep / forward-only, every op, checked and unchecked entry, one call or
    two, with and without a chunk size (so every tile size, and records cut into parts)."""
    from randstream import random_stream
    base = int(os.environ.get("UCCL_TEST_SEED_BASE", "7000"))      # other seeds and more streams for a soak run
    for seed in range(int(os.environ.get("UCCL_TEST_STREAMS", "50"))):
        for op in (SUM, MAX, COPY, PROD):
            s = random_stream(base + 100 * dtype + 17 * seed + op, dtype, op, max_chunks=48, max_len=9000)
            opts = ([0, 1024, 4096, 65536][seed % 4], parts)
            acc, recv = to_dev(s["acc"]), to_dev(s["recv"])
            out = torch.full((s["out_bytes"],), 0x3C, dtype=torch.uint8, device="cuda")
            bm = torch.zeros((s["n_bits"] + 31) // 32, dtype=torch.int32, device="cuda")
            rej = torch.zeros(1, dtype=torch.int32, device="cuda")
            d = to_dev(s["descs"])
            n = len(s["descs"])
            cuts = [0, n] if seed % 3 else [0, n // 2, n]
            for lo, hi in zip(cuts[:-1], cuts[1:]):
                gpu_lib.uccl_chunk_apply_opts(acc, out, recv, d[lo * 32:], hi - lo, bm, dtype, op,
                                              n_rejected=rej if seed % 2 else None,
                                              n_bits=s["n_bits"] if seed % 2 else None, opts=opts)
            torch.cuda.synchronize()
            eacc, eout, seen = s["acc"].copy(), np.full(s["out_bytes"], 0x3C, np.uint8), oracle.new_seen(s["n_bits"])
            oracle.apply(eacc, eout, s["recv"], s["descs"], seen, dtype, op)
            what = f"dtype {dtype} opts {opts} seed {seed} op {op}"
            assert rej.item() == 0, what
            assert_same(bm.cpu().numpy().view(np.uint32), oracle.pack_bitmap(seen), "bitmap " + what)
            got = to_host(acc, s["acc"].dtype)
            if dtype in (F32, BF16, F16):
                wide = {F32: lambda x: x, BF16: lambda x: (x.astype(np.uint32) << 16).view(np.float32),
                        F16: lambda x: x.view(np.float16).astype(np.float32)}[dtype]
                nan = np.isnan(wide(eacc))
                assert np.array_equal(np.isnan(wide(got)), nan), what
                assert_same(got[~nan], eacc[~nan], "acc " + what)
                go, eo = out.cpu().numpy().view(s["acc"].dtype), eout.view(s["acc"].dtype)
                nan_o = np.isnan(wide(eo))
                assert_same(go[~nan_o], eo[~nan_o], "out " + what)
            else:
                assert_same(got, eacc, "acc " + what)
                assert_same(out.cpu().numpy(), eout, "out " + what)
    assert gpu_lib.uccl_claim_timeouts() == 0


def test_same_records_on_two_streams_apply_once(gpu_lib):
    """The whole record list is issued twice, concurrently, on two streams (a retransmitted
    batch handed over by another engine thread): the bitmap atomics decide each chunk once."""
    dtype, C, n = BF16, 16384, 3000
    one = pl.ints_as(np.ones(1, dtype=np.int64), dtype)[0]
    arr = pl.rng(41, 1).permutation(n)
    d = np.zeros(n, dtype=DESC)
    d["src_off"] = np.arange(n, dtype=np.uint64) * C
    d["dst_off"] = d["out_off"] = arr.astype(np.uint64) * C
    d["len"], d["seq"] = C, arr
    recv = np.full(n * C // 2, one, dtype=np.uint16)
    w = wl.Workload("two", dtype, np.zeros(n * C // 2, dtype=np.uint16), recv, n * C, n, [wl.Phase("p", SUM, d, n, n * C, 0)])
    for trial in range(3):
        run = DeviceRun(w)
        s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
        torch.cuda.synchronize()
        run.apply(run.descs[0], n, SUM, stream=s1)
        run.apply(run.descs[0], n, SUM, stream=s2)
        s1.synchronize(); s2.synchronize()
        acc, out, bm, rej = run.results()
        assert rej == 0 and np.all(acc == one), f"trial {trial}: {np.count_nonzero(acc != one)} elements not exactly 1"
        assert np.array_equal(out.view(np.uint16), acc) and sum(int(x).bit_count() for x in bm) == n


@pytest.mark.parametrize("name,dtype", [("bf16_sum_cases.txt", BF16), ("f16_sum_cases.txt", F16)])
def test_hand_derived_rounding_cases_on_the_gpu(gpu_lib, name, dtype):
    """The hand-derived tie / overflow / subnormal cases of tests/golden, through the GPU path:
    one record whose elements are the cases (both operand orders), against the expected bits
    written in the file, not against the oracle."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", name)
    rows = [l.split() for l in open(path) if l.strip() and l[0] != "#"]
    a = np.array([int(x, 16) for x, _, _ in rows] + [int(y, 16) for _, y, _ in rows], dtype=np.uint16)
    r = np.array([int(y, 16) for _, y, _ in rows] + [int(x, 16) for x, _, _ in rows], dtype=np.uint16)
    e = np.array([int(z, 16) for _, _, z in rows] * 2, dtype=np.uint16)
    pad = (-len(a)) % 8                                  # buffers in whole 16-byte vectors; the record is not
    acc = to_dev(np.concatenate([a, np.zeros(pad, np.uint16)]))
    recv = to_dev(np.concatenate([r, np.zeros(pad, np.uint16)]))
    out = torch.zeros_like(acc)
    d = np.zeros(1, dtype=DESC)
    d[0] = (0, 0, 0, 2 * len(a), 0)
    bitmap = torch.zeros(1, dtype=torch.int32, device="cuda")
    for opts in LAUNCHES:
        acc_k = acc.clone()
        bitmap.zero_()
        gpu_lib.uccl_chunk_apply_opts(acc_k, out, recv, to_dev(d), 1, bitmap, dtype, SUM, opts=opts)
        torch.cuda.synchronize()
        got = acc_k.cpu().numpy().view(np.uint16)[:len(a)]
        assert np.array_equal(got, e), (opts, [f"{x:04X}" for x in got], [f"{x:04X}" for x in e])
        assert np.array_equal(out.cpu().numpy().view(np.uint16)[:len(a)], e)


@pytest.mark.parametrize("parts", [0, 4, 16])
def test_cut_records_on_two_streams_apply_once(gpu_lib, parts):
    """Few, large records (so every record is cut into parts), the same list issued concurrently
    on two streams: each stream has its own claim words, the bitmap decides between the streams,
    and every part of every record learns exactly one decision."""
    dtype, C, n = F32, 96 << 10, 120
    arr = pl.rng(43, 1).permutation(n)
    d = np.zeros(n, dtype=DESC)
    d["src_off"] = np.arange(n, dtype=np.uint64) * C
    d["dst_off"] = d["out_off"] = arr.astype(np.uint64) * C
    d["len"], d["seq"] = C, arr
    recv = np.ones(n * C // 4, dtype=np.float32)
    w = wl.Workload("two-cut", dtype, np.zeros(n * C // 4, dtype=np.float32), recv, n * C, n,
                    [wl.Phase("p", SUM, d, n, n * C, 0)])
    for trial in range(3):
        run = DeviceRun(w, opts=(0, parts))
        s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
        torch.cuda.synchronize()
        run.apply(run.descs[0], n, SUM, stream=s1)
        run.apply(run.descs[0], n, SUM, stream=s2)
        run.apply(run.descs[0], n, SUM, stream=s1)
        s1.synchronize(); s2.synchronize()
        acc, out, bm, rej = run.results()
        assert rej == 0 and gpu_lib.uccl_claim_timeouts() == 0
        assert np.all(acc == 1.0), f"trial {trial}: {np.count_nonzero(acc != 1.0)} elements not exactly 1"
        assert np.array_equal(out.view(np.float32), acc) and sum(int(x).bit_count() for x in bm) == n


def test_cut_records_in_a_captured_graph(gpu_lib):
    """A call made under stream capture is never cut into parts (its replays could overlap with
    other work on the claim words), whatever `parts` asks for; replays give the oracle's result."""
    w = wl.config1(seed=5)
    eacc, eout, ebm = oracle_results(w)
    run = DeviceRun(w, opts=(64 << 10, 8))
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(g, stream=side):
        gpu_lib.uccl_dedup_reset(run.bitmap, w.n_bits)
        for ph, dd in zip(w.phases, run.descs):
            run.apply(dd, len(ph.descs), ph.op, checked=False)
    acc0 = run.acc.clone()
    for rep in range(3):
        run.acc.copy_(acc0)
        g.replay()
        torch.cuda.synchronize()
        acc, out, bm, _ = run.results()
        assert_same(bm, ebm, f"bitmap, replay {rep}")
        assert_same(acc, eacc, f"acc, replay {rep}")
        assert_same(out, eout, f"out, replay {rep}")


@pytest.mark.parametrize("packet_bytes", [0, 4096, 8192])
def test_two_pass_form_equals_the_single_pass_definition(gpu_lib, packet_bytes):
    """The paper's literal receive path (Section 3.1: scattered memcpy of the out-of-order payloads
    into the transport buffer, then the original reduction), composed from uccl_chunk_scatter and
    uccl_chunk_apply: its accumulator and staging bytes equal the oracle's single-pass result on
    the same arrivals.  packet_bytes > 0: every arrival is one datagram payload, reassembled into
    the transport buffer and then reduced at the collective's 32 KiB chunk size (Appendix C.4)."""
    C = 32 << 10
    arrival = packet_bytes or C
    w = wl.config2(seed=12, M=16 << 20, C=arrival, window=1024 * C // arrival)
    eacc, eout, _ = oracle_results(w)
    pairs, transport_bytes = wl.two_pass_records(w, arrival, C // arrival)
    run = DeviceRun(w)
    transport = torch.zeros(transport_bytes, dtype=torch.uint8, device="cuda")
    placed = torch.zeros((w.n_bits + 31) // 32, dtype=torch.int32, device="cuda")   # dedup state of the first pass
    for ph, (first, second) in zip(w.phases, pairs):
        gpu_lib.uccl_chunk_scatter_opts(transport, run.recv, to_dev(first), len(first), placed, opts=(arrival, 0))
        gpu_lib.uccl_chunk_apply_opts(run.acc, run.out, transport, to_dev(second), len(second), run.bitmap, w.dtype,
                                      ph.op, opts=(C, 0))
    torch.cuda.synchronize()
    acc, out, bm, _ = run.results()
    assert_same(acc, eacc, "acc"); assert_same(out, eout, "out_stage")
    assert sum(int(x).bit_count() for x in placed.cpu().numpy().view(np.uint32)) == w.n_bits
    # the second pass dedups per collective chunk: one bit per group of arrivals
    assert sum(int(x).bit_count() for x in bm) == w.n_bits // (C // arrival)


def test_more_streams_than_claim_regions(gpu_lib):
    """The claim pool has one region per stream for 64 streams; a call on a stream that finds none is
    launched with one workgroup per record instead.  80 streams, each with a call of few large
    records on buffers of its own: every result is the oracle's."""
    w = wl.ring_share("regions", 61, R=4, M=4 * 6 * (48 << 10), C=48 << 10, dtype=F32, paths=3, window=None, dup=0.1,
                      dist="uniform", allgather=False)
    eacc, eout, ebm = oracle_results(w)
    streams = [torch.cuda.Stream() for _ in range(80)]
    runs = [DeviceRun(w, opts=(48 << 10, 4)) for _ in streams]
    torch.cuda.synchronize()
    for s, run in zip(streams, runs):
        run.apply(run.descs[0], len(w.phases[0].descs), SUM, checked=False, stream=s)
    torch.cuda.synchronize()
    assert gpu_lib.uccl_claim_timeouts() == 0
    for k, run in enumerate(runs):
        acc, out, bm, _ = run.results()
        assert_same(acc, eacc, f"acc, stream {k}"); assert_same(out, eout, f"out, stream {k}"); assert_same(bm, ebm, f"bitmap {k}")


def test_cut_records_from_several_host_threads_on_one_stream(gpu_lib):
    """Four host threads issue calls of few large records (each cut into parts) on ONE stream at the
    same time, each thread on buffers of its own.  The calls share the stream's claim words, and a
    part recognises its own call by a tag that must grow in the order the calls run: tags are drawn
    and launches enqueued under one lock, so no part ever waits for a tag that has been passed."""
    import threading
    w = wl.ring_share("threads", 71, R=4, M=4 * 9 * (40 << 10), C=40 << 10, dtype=F32, paths=3, window=None,
                      dup=0.15, dist="uniform", allgather=False)
    eacc, eout, ebm = oracle_results(w)
    stream = torch.cuda.Stream()
    n_threads, rounds = 4, 25
    runs = [[DeviceRun(w, opts=(40 << 10, 4)) for _ in range(rounds)] for _ in range(n_threads)]
    torch.cuda.synchronize()
    errors = []

    def issue(mine):
        try:
            torch.cuda.set_device(0)
            for run in mine:
                run.apply(run.descs[0], len(w.phases[0].descs), SUM, checked=False, stream=stream)
        except Exception as e:  # noqa: BLE001 - reported by the main thread
            errors.append(e)
    threads = [threading.Thread(target=issue, args=(r,)) for r in runs]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    stream.synchronize()
    assert not errors, errors
    assert gpu_lib.uccl_claim_timeouts() == 0
    for a, mine in enumerate(runs):
        for b, run in enumerate(mine):
            acc, out, bm, _ = run.results()
            assert_same(acc, eacc, f"acc, thread {a} call {b}"); assert_same(out, eout, f"out, thread {a} call {b}")
            assert_same(bm, ebm, f"bitmap, thread {a} call {b}")


def test_prepared_calls_equal_the_marshalled_ones(gpu_lib):
    """pkg.uccl_prepare marshals once; invoking the result makes the same C call again: two
    passes over config 1 (reset + every phase), each checked against the oracle, then an error
    code surfaces as the same exception."""
    pkg = gpu_lib
    w = wl.config1(seed=4)
    say("prepared calls, config1")
    eacc, eout, ebm = oracle_results(w)
    run = DeviceRun(w)
    acc0 = run.acc.clone()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):      # prepared on `side`: that is where every later invocation goes
        reset = pkg.uccl_prepare(pkg.uccl_dedup_reset, run.bitmap, w.n_bits)
        steps = [pkg.uccl_prepare(pkg.uccl_chunk_apply_opts, run.acc, run.out, run.recv, d, len(ph.descs), run.bitmap,
                                  w.dtype, ph.op, n_rejected=run.rejected, n_bits=w.n_bits, opts=(64 << 10, 0))
                 for ph, d in zip(w.phases, run.descs)]
    for rep in range(2):
        run.acc.copy_(acc0)
        run.out.fill_(0xA5)
        side.wait_stream(torch.cuda.current_stream())
        reset()
        for s in steps:
            s()
        side.synchronize()
        acc, out, bm, rej = run.results()
        assert rej == 0 and pkg.uccl_claim_timeouts() == 0
        assert_same(bm, ebm, f"bitmap, pass {rep}")
        assert_same(acc, eacc, f"acc, pass {rep}")
        assert_same(out, eout, f"out_stage, pass {rep}")
    bad = pkg.uccl_prepare(pkg.uccl_chunk_apply, run.acc, run.out, run.recv, run.descs[0], 1, run.bitmap, 99, SUM)
    with pytest.raises(pkg.UcclError) as e:
        bad()
    assert e.value.code == pkg.UCCL_EINVAL
    with pytest.raises(ValueError):    # not exactly one C call
        pkg.uccl_prepare(lambda: None)
