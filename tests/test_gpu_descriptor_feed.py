"""Descriptor feed without per-batch argument changes: records and their count live in a
slot (pinned host memory, mapped into the device) that the control path rewrites; the
library call has fixed arguments, is captured once in a graph and replayed per message."""
import sys

import numpy as np
import pytest
import torch

import oracle
from synth import workloads as wl
from synth.layout import DESC, NO_FORWARD, F32, SUM, COPY

from gpuhelp import DeviceRun, oracle_results, assert_same, to_dev, to_host

pytestmark = pytest.mark.gpu


def pinned(nbytes):
    t = torch.zeros(nbytes, dtype=torch.uint8, pin_memory=True)
    return t, t.numpy()


def test_records_read_from_pinned_host_memory(gpu_lib):
    w = wl.config2(seed=3, M=8 << 20)
    eacc, eout, ebm = oracle_results(w)
    run = DeviceRun(w)
    keep = []
    for ph in w.phases:
        t, v = pinned(ph.descs.nbytes)
        v[:] = ph.descs.view(np.uint8).reshape(-1)
        keep.append(t)
        run.apply(t, len(ph.descs), ph.op)
    torch.cuda.synchronize()
    acc, out, bm, rej = run.results()
    assert rej == 0
    assert_same(acc, eacc, "acc"); assert_same(out, eout, "out"); assert_same(bm, ebm, "bitmap")


def test_indirect_count(gpu_lib):
    w = wl.config2(seed=4, M=8 << 20)
    ph = w.phases[0]
    n = len(ph.descs)
    cnt_t, cnt_v = pinned(4)
    for live in (0, 1, n // 3, n, n + 1000):
        run = DeviceRun(w)
        cnt_v.view(np.uint32)[0] = live
        gpu_lib.uccl_chunk_apply_indirect(run.acc, run.out, run.recv, run.descs[0], cnt_t, n, run.bitmap,
                                          w.dtype, ph.op, n_rejected=run.rejected, n_bits=w.n_bits)
        torch.cuda.synchronize()
        acc, out, bm, rej = run.results()
        eacc, eout, seen = w.acc.copy(), np.full(w.out_bytes, 0xA5, np.uint8), oracle.new_seen(w.n_bits)
        oracle.apply(eacc, eout, w.recv_stage, ph.descs[:min(live, n)], seen, w.dtype, ph.op)
        assert rej == 0
        assert_same(acc, eacc, f"acc live={live}"); assert_same(out, eout, "out")
        assert_same(bm, oracle.pack_bitmap(seen), "bitmap")
    # device-resident count, unchecked call
    run = DeviceRun(w)
    cnt_d = torch.tensor([n // 2], dtype=torch.int32, device="cuda")
    gpu_lib.uccl_chunk_apply_indirect(run.acc, run.out, run.recv, run.descs[0], cnt_d, n, run.bitmap, w.dtype, ph.op)
    torch.cuda.synchronize()
    eacc, eout, seen = w.acc.copy(), np.full(w.out_bytes, 0xA5, np.uint8), oracle.new_seen(w.n_bits)
    oracle.apply(eacc, eout, w.recv_stage, ph.descs[:n // 2], seen, w.dtype, ph.op)
    assert_same(run.results()[0], eacc, "acc")


def test_graph_replay_per_message(gpu_lib):
    """One captured graph (reduce-scatter call + allgather call on fixed arguments) replayed for
    every message after the host rewrote the slot; every replay is checked against the oracle,
    with eager work and synchronisation between replays."""
    w, msgs = wl.config5(seed=6, n_msgs=24)
    cap = max(max(len(m["rs"]), len(m["ag"])) for m in msgs) + 7
    run = DeviceRun(w, guard=0)
    slots = {k: pinned(cap * 32) for k in ("rs", "ag")}
    counts_t, counts_v = pinned(8)
    counts = counts_v.view(np.uint32)
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(g, stream=side):
        gpu_lib.uccl_chunk_apply_indirect(run.acc, run.out, run.recv, slots["rs"][0], counts_t[0:4], cap,
                                          run.bitmap, F32, SUM, n_rejected=run.rejected, n_bits=w.n_bits,
                                          opts=(4096, 0))
        gpu_lib.uccl_chunk_apply_indirect(run.acc, run.out, run.recv, slots["ag"][0], counts_t[4:8], cap,
                                          run.bitmap, F32, COPY, n_rejected=run.rejected, n_bits=w.n_bits,
                                          opts=(4096, 0))
    eacc = w.acc.copy()
    eout = np.zeros(w.out_bytes, dtype=np.uint8)
    seen = oracle.new_seen(w.n_bits)
    scratch = torch.zeros(1 << 16, device="cuda")
    for i, m in enumerate(msgs):
        for j, key in enumerate(("rs", "ag")):
            d = m[key].view(np.uint8).reshape(-1)
            slots[key][1][:len(d)] = d
            slots[key][1][len(d):] = 0xFF  # stale bytes beyond the count must never be used
            counts[j] = len(m[key])
        g.replay()
        torch.cuda.synchronize()
        scratch.add_(1.0).sum().item()  # the program's own eager work between replays
        oracle.apply(eacc, eout, w.recv_stage, m["rs"], seen, F32, SUM)
        oracle.apply(eacc, eout, w.recv_stage, m["ag"], seen, F32, COPY)
        acc, out, bm, rej = run.results()
        assert rej == 0, f"message {i}"
        assert_same(bm, oracle.pack_bitmap(seen), f"bitmap after message {i}")
        assert_same(acc, eacc, f"acc after message {i}")
        assert_same(out, eout, f"out after message {i}")
    counts[:] = 0
    g.replay()  # an empty slot is a no-op
    torch.cuda.synchronize()
    assert_same(run.results()[0], eacc, "acc after empty replay")


@pytest.mark.parametrize("capacity,poll", [(4096, True), (100, True), (37, False), (100000, False)])
def test_host_side_feed_batches_messages(gpu_lib, capacity, poll):
    """Records pushed message by message (reduce-scatter records to lane 0, then allgather
    records to lane 1), with slots far smaller than a message, equal to several messages, or
    larger than everything: the result is the oracle's, and the batcher really batched."""
    w, msgs = wl.config5(seed=8, n_msgs=40)
    run = DeviceRun(w, guard=0)
    feed = gpu_lib.uccl_feed_create(run.acc, run.out, run.recv, run.bitmap, F32, SUM, COPY, capacity, 4)
    try:
        for m in msgs:
            gpu_lib.uccl_feed_push(feed, 0, np.ascontiguousarray(m["rs"]))
            gpu_lib.uccl_feed_push(feed, 1, np.ascontiguousarray(m["ag"]))
            if poll:
                gpu_lib.uccl_feed_poll(feed)
        gpu_lib.uccl_feed_sync(feed)
        stats = gpu_lib.uccl_feed_get_stats(feed)
    finally:
        gpu_lib.uccl_feed_destroy(feed)
    total = sum(len(m["rs"]) + len(m["ag"]) for m in msgs)
    assert stats["records"] == total and stats["flushes"] >= 1 and stats["max_batch"] <= 2 * capacity
    if capacity == 100000 and not poll:
        assert stats["flushes"] == 1
    eacc, eout, seen = w.acc.copy(), np.zeros(w.out_bytes, dtype=np.uint8), oracle.new_seen(w.n_bits)
    for m in msgs:
        oracle.apply(eacc, eout, w.recv_stage, m["rs"], seen, F32, SUM)
        oracle.apply(eacc, eout, w.recv_stage, m["ag"], seen, F32, COPY)
    acc, out, bm, _ = run.results()
    assert_same(bm, oracle.pack_bitmap(seen), "bitmap"); assert_same(acc, eacc, "acc"); assert_same(out, eout, "out")


def test_host_side_feed_large_hand_over(gpu_lib):
    """One hand-over of tens of thousands of records per lane: large batches are copied to device
    memory before the kernel reads them (small ones are read from the pinned slot directly);
    same result either way."""
    w, msgs = wl.config5(seed=9, n_msgs=220)
    run = DeviceRun(w, guard=0)
    feed = gpu_lib.uccl_feed_create(run.acc, run.out, run.recv, run.bitmap, F32, SUM, COPY, 1 << 17, 2)
    try:
        for m in msgs:
            gpu_lib.uccl_feed_push(feed, 0, np.ascontiguousarray(m["rs"]))
            gpu_lib.uccl_feed_push(feed, 1, np.ascontiguousarray(m["ag"]))
        gpu_lib.uccl_feed_sync(feed)
        stats = gpu_lib.uccl_feed_get_stats(feed)
    finally:
        gpu_lib.uccl_feed_destroy(feed)
    assert stats["flushes"] == 1 and stats["max_batch"] > 2 * 16384, stats  # both lanes above the direct-read limit
    eacc, eout, seen = w.acc.copy(), np.zeros(w.out_bytes, dtype=np.uint8), oracle.new_seen(w.n_bits)
    for m in msgs:
        oracle.apply(eacc, eout, w.recv_stage, m["rs"], seen, F32, SUM)
    for m in msgs:
        oracle.apply(eacc, eout, w.recv_stage, m["ag"], seen, F32, COPY)
    acc, out, bm, _ = run.results()
    assert_same(bm, oracle.pack_bitmap(seen), "bitmap"); assert_same(acc, eacc, "acc"); assert_same(out, eout, "out")


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_host_side_feed_random_push_pattern(gpu_lib, seed):
    """Pushes of random sizes into either lane, polls, flushes and syncs in random order, a slot
    capacity that many pushes overflow: every record is handed over exactly once, whatever the
    pattern.  Lane 0 reduces into one half of the accumulator, lane 1 copies into the other, so
    the two lanes never depend on each other and any interleaving has the same result."""
    from synth import payload as pl
    from synth.layout import DESC, NO_FORWARD
    g = pl.rng(900 + seed, 1)
    C_, n = 2048, 3000
    acc = pl.uniform_f32(900 + seed, 2, 2 * n * C_ // 4)
    recv = pl.uniform_f32(900 + seed, 3, 2 * n * C_ // 4)
    lanes = []
    for lane in (0, 1):
        arrivals = np.concatenate([g.permutation(n), g.integers(0, n, n // 10)])     # 10 % retransmitted
        d = np.zeros(len(arrivals), dtype=DESC)
        d["seq"] = arrivals + lane * n
        d["src_off"] = (arrivals + lane * n).astype(np.uint64) * C_
        d["dst_off"] = d["src_off"]
        d["out_off"] = np.where(arrivals % 3 == 0, NO_FORWARD, d["src_off"])
        d["len"] = C_ - 16 * (arrivals % 5)
        lanes.append(d)
    d_acc, d_recv = to_dev(acc), to_dev(recv)
    d_out = torch.zeros(acc.nbytes, dtype=torch.uint8, device="cuda")
    bitmap = torch.zeros((2 * n + 31) // 32, dtype=torch.int32, device="cuda")
    feed = gpu_lib.uccl_feed_create(d_acc, d_out, d_recv, bitmap, F32, SUM, COPY, 257, 3)
    at = [0, 0]
    try:
        while at[0] < len(lanes[0]) or at[1] < len(lanes[1]):
            lane = int(g.integers(0, 2))
            if at[lane] >= len(lanes[lane]):
                lane = 1 - lane
            k = int(min(g.integers(0, 700), len(lanes[lane]) - at[lane]))
            gpu_lib.uccl_feed_push(feed, lane, np.ascontiguousarray(lanes[lane][at[lane]:at[lane] + k]))
            at[lane] += k
            what = int(g.integers(0, 6))
            if what == 0:
                gpu_lib.uccl_feed_flush(feed)
            elif what == 1:
                gpu_lib.uccl_feed_sync(feed)
            elif what < 5:
                gpu_lib.uccl_feed_poll(feed)
        gpu_lib.uccl_feed_sync(feed)
        stats = gpu_lib.uccl_feed_get_stats(feed)
    finally:
        gpu_lib.uccl_feed_destroy(feed)
    assert stats["records"] == len(lanes[0]) + len(lanes[1]) and stats["max_batch"] <= 2 * 257
    eacc, eout, seen = acc.copy(), np.zeros(acc.nbytes, dtype=np.uint8), oracle.new_seen(2 * n)
    assert oracle.apply(eacc, eout, recv, lanes[0], seen, F32, SUM) == n
    assert oracle.apply(eacc, eout, recv, lanes[1], seen, F32, COPY) == n
    assert_same(bitmap.cpu().numpy().view(np.uint32), oracle.pack_bitmap(seen), "bitmap")
    assert_same(d_acc.cpu().numpy().view(np.float32), eacc, "acc")
    assert_same(d_out.cpu().numpy(), eout, "out")


def test_two_feeds_with_different_chunk_sizes_interleaved(gpu_lib):
    """Two connections in one process, one with 4 KiB chunks and one with 128 KiB chunks, each
    with a feed of its own on a stream of its own, pushed alternately from one thread: the
    launch of each hand-over is sized from that feed's own records (nothing process-wide), and
    both results are the oracle's.  The 128 KiB connection hands over few records at a time, so
    its records are cut into parts; both feeds' streams then hold claim regions of their own."""
    from synth.layout import BF16
    small = wl.ring_share("small", 51, R=4, M=4 * 300 * 4096, C=4096, dtype=F32, paths=8, window=64, dup=0.05,
                          dist="uniform")
    large = wl.ring_share("large", 52, R=4, M=4 * 24 * (128 << 10), C=128 << 10, dtype=BF16, paths=8, window=16,
                          dup=0.05, dist="normal")
    runs = [DeviceRun(small, guard=0), DeviceRun(large, guard=0)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for s in streams:
        s.wait_stream(torch.cuda.current_stream())
    feeds = [gpu_lib.uccl_feed_create(r.acc, r.out, r.recv, r.bitmap, r.w.dtype, SUM, COPY, cap, 4, stream=s)
             for r, cap, s in zip(runs, (512, 40), streams)]
    try:
        cursors = [[0, 0], [0, 0]]
        steps = [97, 7]
        busy = True
        while busy:
            busy = False
            for f, (feed, run, step) in enumerate(zip(feeds, runs, steps)):
                for lane, ph in enumerate(run.w.phases):
                    lo = cursors[f][lane]
                    # the allgather lane starts only once the reduce-scatter lane has been pushed completely
                    if lo >= len(ph.descs) or (lane == 1 and cursors[f][0] < len(run.w.phases[0].descs)):
                        continue
                    gpu_lib.uccl_feed_push(feed, lane, np.ascontiguousarray(ph.descs[lo:lo + step]))
                    cursors[f][lane] = lo + step
                    busy = True
                gpu_lib.uccl_feed_poll(feed)
        for feed in feeds:
            gpu_lib.uccl_feed_sync(feed)
    finally:
        for feed in feeds:
            gpu_lib.uccl_feed_destroy(feed)
    assert gpu_lib.uccl_claim_timeouts() == 0
    for run in runs:
        eacc, eout, ebm = oracle_results(run.w, guard=0)
        acc, out, bm, _ = run.results()
        assert_same(bm, ebm, run.w.name + " bitmap")
        assert_same(acc, eacc, run.w.name + " acc")
        assert_same(out, eout, run.w.name + " out")
