"""Full-size parity, in the launch configuration bench.py times: the unchecked general entry
point, the transport's chunk size given with the call, everything else left to the library.  Every output
element of every configuration is compared with the oracle (the oracle finishes each of
them in seconds, so no sampling is needed)."""
import sys
import time

import numpy as np
import pytest
import torch

import oracle
from synth import workloads as wl
from synth.layout import SUM, COPY, F32

from gpuhelp import DeviceRun, oracle_results, assert_same, to_dev

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, file=sys.stderr, flush=True)


def run_full(pkg, w, chunk):
    run = DeviceRun(w, opts=(chunk, 0))
    run.reset()
    run.run_phases(checked=False)
    assert pkg.uccl_claim_timeouts() == 0
    return run.results()


def test_config1_full_size_as_benchmarked(gpu_lib):
    """4 MiB fp32 in 64 KiB chunks: 57 + 56 records, each cut into parts by the library's own choice."""
    w = wl.config1(seed=1)
    eacc, eout, ebm = oracle_results(w)
    acc, out, bm, _ = run_full(gpu_lib, w, 64 << 10)
    assert_same(bm, ebm, "bitmap")
    assert_same(acc, eacc, "acc")
    assert_same(out, eout, "out_stage")


@pytest.mark.parametrize("name,chunk", [("config2", 32 << 10), ("config3", 128 << 10)])
def test_ring_share_full_size(gpu_lib, name, chunk):
    t0 = time.time()
    w = getattr(wl, name)(seed=1)
    say(f"{name}: built in {time.time() - t0:.1f}s, {sum(len(p.descs) for p in w.phases)} arrivals")
    eacc, eout, ebm = oracle_results(w)
    say(f"{name}: oracle done at {time.time() - t0:.1f}s")
    acc, out, bm, _ = run_full(gpu_lib, w, chunk)
    assert_same(bm, ebm, "bitmap")
    assert_same(acc, eacc, "acc")
    assert_same(out, eout, "out_stage")
    # properties that hold at any size: the untouched segment keeps its initial bytes,
    # every distinct seq has its bit, nothing else has
    S = w.acc.nbytes // (16 if name == "config2" else 8)
    if name == "config3":
        assert_same(acc.view(np.uint8)[:S], w.acc.view(np.uint8)[:S], "segment 0 untouched by reduce-scatter")
    assert sum(int(x).bit_count() for x in bm) == sum(p.n_unique for p in w.phases) == w.n_bits


def test_alltoall_full_size(gpu_lib):
    w = wl.config4(seed=1)
    ph = w.phases[0]
    dst = torch.zeros(w.acc.nbytes, dtype=torch.uint8, device="cuda")
    bm = torch.zeros((w.n_bits + 31) // 32, dtype=torch.int32, device="cuda")
    gpu_lib.uccl_chunk_scatter_opts(dst, to_dev(w.recv_stage), to_dev(ph.descs), len(ph.descs), bm,
                                    opts=(16 << 10, 0))
    torch.cuda.synchronize()
    edst = np.zeros(w.acc.nbytes, dtype=np.uint8)
    seen = oracle.new_seen(w.n_bits)
    assert oracle.scatter(edst, w.recv_stage, ph.descs, seen) == ph.n_unique
    got = dst.cpu().numpy()
    assert_same(got, edst, "dst")
    assert_same(got, np.concatenate(w.extra["sources"]), "dst is the concatenation of the sources")
    assert_same(bm.cpu().numpy().view(np.uint32), oracle.pack_bitmap(seen), "bitmap")


def test_small_messages_all_10000(gpu_lib):
    """All 10000 small allreduces of the recipe (1.57 M unique chunks), 128 messages per call."""
    t0 = time.time()
    w, msgs = wl.config5(seed=1, n_msgs=10000)
    say(f"config5: built {len(msgs)} messages in {time.time() - t0:.1f}s")
    eacc = w.acc.copy()
    eout = np.zeros(w.out_bytes, dtype=np.uint8)
    seen = oracle.new_seen(w.n_bits)
    run = DeviceRun(w, guard=0, opts=(4 << 10, 0))
    for lo in range(0, len(msgs), 128):
        rs = np.concatenate([m["rs"] for m in msgs[lo:lo + 128]])
        ag = np.concatenate([m["ag"] for m in msgs[lo:lo + 128]])
        run.apply(to_dev(rs), len(rs), SUM, checked=False)
        run.apply(to_dev(ag), len(ag), COPY, checked=False)
        oracle.apply(eacc, eout, w.recv_stage, rs, seen, F32, SUM, check=False)
        oracle.apply(eacc, eout, w.recv_stage, ag, seen, F32, COPY, check=False)
        if lo % (128 * 16) == 0:
            say(f"config5: {lo} messages at {time.time() - t0:.0f}s")
    torch.cuda.synchronize()
    acc, out, bm, _ = run.results()
    assert_same(bm, oracle.pack_bitmap(seen), "bitmap")
    assert_same(acc, eacc, "acc")
    assert_same(out, eout, "out_stage")


@pytest.mark.parametrize("dtype,op", [(1, 0), (2, 0), (1, 4), (2, 4)])
def test_16bit_every_pair(gpu_lib, dtype, op):
    """All 65536 x 65536 pairs of bf16 / binary16 bit patterns through SUM and PROD, bit-exact
    against the oracle (NaN results: NaN-ness only, their payload is not fixed by the method)."""
    from synth.layout import DESC, NO_FORWARD
    what = f"{ {1: 'bf16', 2: 'f16'}[dtype]} { {0: 'SUM', 4: 'PROD'}[op]} pairs"
    blk = 2048                                     # a-values per block: 134 M pairs
    n = blk * 65536
    r_np = np.tile(np.arange(65536, dtype=np.uint16), blk)
    r_dev = to_dev(r_np)
    pieces = 64
    d = np.zeros(pieces, dtype=DESC)
    for k in range(pieces):
        d[k] = (k * (n // pieces) * 2, k * (n // pieces) * 2, NO_FORWARD, (n // pieces) * 2, k)
    d_dev = to_dev(d)
    bm = torch.zeros(pieces // 32, dtype=torch.int32, device="cuda")
    wide = (lambda h: (h.astype(np.uint32) << 16).view(np.float32)) if dtype == 1 else \
           (lambda h: h.view(np.float16).astype(np.float32))
    t0 = time.time()
    for b in range(65536 // blk):
        a_np = np.repeat(np.arange(b * blk, (b + 1) * blk, dtype=np.uint16), 65536)
        acc = to_dev(a_np)
        bm.zero_()
        gpu_lib.uccl_chunk_apply(acc, None, r_dev, d_dev, pieces, bm, dtype, op)
        exp = a_np.copy()
        seen = oracle.new_seen(pieces)
        oracle.apply(exp, None, r_np, d, seen, dtype, op, check=False)
        got = acc.cpu().numpy().view(np.uint16)
        if not np.array_equal(got, exp):
            nan = np.isnan(wide(exp))
            assert np.array_equal(np.isnan(wide(got)), nan), f"block {b}: NaN-ness differs"
            bad = np.flatnonzero((got != exp) & ~nan)
            assert len(bad) == 0, (f"block {b}: {len(bad)} mismatches, first a={a_np[bad[0]]:#06x} "
                                   f"r={r_np[bad[0]]:#06x} got={got[bad[0]]:#06x} exp={exp[bad[0]]:#06x}")
        if b % 8 == 7:
            say(f"{what}: block {b + 1}/{65536 // blk} at {time.time() - t0:.0f}s")


def test_direct_reduce_scatter_full_size(gpu_lib):
    """The multi-source fold at the size bench.py times it (R = 8, 1 GiB fp32: seven senders'
    128 MiB copies folded into this rank's segment, 128 KiB chunks), every element against the oracle."""
    t0 = time.time()
    w = wl.direct_reduce_scatter("direct-reduce-scatter-1GiB-f32", 1, R=8, M=1 << 30, C=128 << 10, dtype=F32,
                                 paths=64, dup=0.005, dist="uniform")
    ph = w.phases[0]
    say(f"direct-rs: built in {time.time() - t0:.1f}s, {len(ph.descs)} records")
    eacc, seen = w.acc.copy(), oracle.new_seen(w.n_bits)
    assert oracle.reduce_gather(eacc, None, w.recv_stage, ph.descs, seen, F32, SUM) == ph.n_unique
    say(f"direct-rs: oracle done at {time.time() - t0:.1f}s")
    acc, recv = to_dev(w.acc), to_dev(w.recv_stage)
    bitmap = torch.zeros((w.n_bits + 31) // 32, dtype=torch.int32, device="cuda")
    gpu_lib.uccl_chunk_reduce_gather(acc, None, recv, to_dev(ph.descs), len(ph.descs), bitmap, F32, SUM,
                                     opts=(128 << 10, 0))
    torch.cuda.synchronize()
    assert_same(bitmap.cpu().numpy().view(np.uint32), oracle.pack_bitmap(seen), "bitmap")
    assert_same(acc.cpu().numpy().view(np.float32), eacc, "acc")
