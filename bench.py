#!/usr/bin/env python3
"""Benchmark of the receive-side chunk data path on one MI355X.

A step is one pass of the whole hot path over one rank's share of the collective: reset
the dedup bitmap, then one library call per phase over that phase's arrival list (dedup,
place, SUM / COPY, write back, forward).  Inputs are seeded synthetic chunk streams,
resident in HBM before the timed region starts.

Steps rotate over `--sets` identical copies of the buffers (default 4), so that no buffer
is still in the 256 MB last-level cache when its turn comes again: the headline number is
an HBM number.  `--also-warm` adds the same loop over a single buffer set (`warm_cache`).

Prints one JSON line: whole-job reduced-payload GB/s, the HBM-roofline fraction of the
dominant kernel (algorithmic bytes / measured kernel time / 8 TB/s), dense streaming kernels
of the same traffic shape at the same footprint (`stream_ceiling`), and the CPU oracle timed
on the host cores of the same machine as a reported baseline.
"""
import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

PEAK_HBM_GBS = 8000.0  # MI355X published HBM3E peak, GB/s
# Kernel durations are sampled on every EVENT_STRIDE-th timed step: an event pair on a dispatch
# adds a completion signal between kernels (about 5 us each), which would otherwise slow every step.
EVENT_STRIDE = 4
ROOT = os.path.dirname(os.path.abspath(__file__))
METRIC = "reduced payload GB/s (dedup+place+reduce+forward of one rank's chunk stream), 1x MI355X"

# HBM bytes per launch of the dominant kernel from rocprofv3 counters (FETCH_SIZE and WRITE_SIZE,
# each scaled by what it reads for a plain copy of known size, see profiles/): valid only for the
# kernel source it was measured on, identified by the hash of the HIP source files.
MEASURED_TRAFFIC = {
    # (workload, source_hash() of the files under csrc/): bytes per launch
    ("config1", "c123f02476acd1e3"): 14883934,
    ("config2", "c123f02476acd1e3"): 1007972699,
    ("config3", "c123f02476acd1e3"): 3625022876,
    ("config4", "c123f02476acd1e3"): 108173818,
    ("direct-rs", "c123f02476acd1e3"): 1208245583,
}

WORKLOADS = {
    "config1": "allreduce rank share: R=8, 4 MiB fp32 uniform[-1,1], 64 KiB chunks, 4 paths, no window, 1% duplicates",
    "config2": "allreduce rank share: R=16, 256 MiB bf16 normal(0,1), 32 KiB chunks, 256 paths, window 1024, 2% duplicates",
    "config3": "reduce-scatter rank share: R=8, 1 GiB fp32 uniform[-1,1], 128 KiB chunks, 64 paths, window 256, 0.5% duplicates",
    "config4": "all-to-all dispatch: 7 sources x U[0,16 MiB] of 14336-byte bf16 rows, 16 KiB chunks, 128 paths, 1% duplicates",
    "config5": "small allreduces: 10,000 messages, fp32, 64 KiB-1 MiB log-uniform, R=8, 4 KiB chunks, 32 paths, 3% duplicates, 128 messages per call",
    "direct-rs": "direct (one-hop) reduce-scatter: R=8, 1 GiB fp32, 7 senders' copies of this rank's 128 MiB segment "
                 "folded in rank order by gather records, 128 KiB chunks, 64 paths per sender, 0.5% duplicates",
    "config5-single": "small allreduces, one message at a time (two calls per message)",
    "config5-feed": "small allreduces pushed message by message into the library's host-side batcher (uccl_feed): a "
                    "slot is handed to the GPU whenever the previous hand-over has finished (adaptive batching)",
    "config5-graph": "small allreduces, one message at a time: the control path rewrites a pinned descriptor "
                     "slot and replays a captured graph of the two calls (no per-message argument marshalling)",
    "calls": "single calls of n records of C bytes (fp32 SUM with forward, no duplicates, scattered destinations): kernel "
             "time as the library launches them and with the records never cut / cut into 8 / 16 parts",
    "segment": "sender side: this rank's own segment of a ring (config2's shape: 16 MiB in 32 KiB chunks; config3's: "
               "128 MiB in 128 KiB chunks) cut into staged chunks with send records",
}


def source_hash():
    """First 16 hex digits of sha256 over the kernel sources (every file under csrc/, by name order)."""
    d = os.path.join(ROOT, "paper_2504_17307_amd", "csrc")
    h = hashlib.sha256()
    for name in sorted(os.listdir(d)):
        if name.endswith((".hip", ".hpp")):
            with open(os.path.join(d, name), "rb") as f:
                h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()[:16]


def device_info(torch):
    """What the runtime says about the GPU the numbers were taken on (machines of one model differ)."""
    p = torch.cuda.get_device_properties(0)
    info = {"name": p.name, "compute_units": p.multi_processor_count, "memory_GiB": round(p.total_memory / 2**30, 1)}
    for key in ("clock_rate", "memory_clock_rate", "memory_bus_width", "L2_cache_size", "gcnArchName"):
        if hasattr(p, key):
            info[key] = getattr(p, key)
    return info


def cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def call_stats(descs, op):
    """(unique chunks, payload bytes, algorithmic bytes) of one call's record list, by the
    single-pass byte model: a reduce reads slot + accumulator, a copy reads the slot; every
    unique chunk writes the accumulator and, if it forwards, the staging copy; every record
    costs its 32 bytes and one 4-byte bitmap word update."""
    _, first = np.unique(descs["seq"], return_index=True)
    ln = descs["len"][first].astype(np.int64)
    off = descs["out_off"][first]
    fwd = off != np.uint64(0xFFFFFFFFFFFFFFFF)
    relay = fwd & ((off & np.uint64(0x8000000000000000)) != 0)  # forwarded, not written back
    reads = ln if op == 3 else 2 * ln
    algo = int(reads.sum() + ln[~relay].sum() + ln[fwd].sum()) + 36 * len(descs)
    return len(first), int(ln.sum()), algo


def two_pass_calls(w, chunk, group=1):
    """The paper's literal form (Section 3.1) as a call list: per phase a scattered memcpy of the
    arrivals into an in-order transport buffer, then the reduction from it (records from
    synth.workloads.two_pass_records).  Returns the call list and the transport buffer size."""
    from synth import workloads as wl
    from synth.layout import COPY
    pairs, transport_bytes = wl.two_pass_records(w, chunk, group)
    calls = []
    for ph, (d1, d2) in zip(w.phases, pairs):
        _, _, algo = call_stats(d1, COPY)
        calls.append(dict(name=ph.name + ": scatter to transport buffer", op=COPY, descs=d1, n_unique=0,
                          payload_bytes=0, algo_bytes=algo, scatter=True, dst="transport", src="recv", bm="bitmap"))
        u, pay, algo = call_stats(d2, ph.op)
        calls.append(dict(name=ph.name + ": reduce from transport buffer", op=ph.op, descs=d2, n_unique=u,
                          payload_bytes=pay, algo_bytes=algo, scatter=False, dst="acc", src="transport", bm="bitmap2"))
    return calls, transport_bytes


def build_job(name, seed, n_msgs, relay=False, per_call=128, packet_bytes=0, dup=None):
    """Returns (workload, calls, chunk_bytes) with calls = list of dicts
    {name, op, descs (numpy), n_unique, payload_bytes, algo_bytes, scatter}."""
    from synth import workloads as wl
    from synth.layout import SUM, COPY
    if name in ("config1", "config2", "config3"):
        chunk = {"config1": 64 << 10, "config2": 32 << 10, "config3": 128 << 10}[name]
        kw = {} if dup is None else dict(dup=dup)
        if packet_bytes:  # arrivals are MTU-sized packets; the reorder window keeps its size in bytes
            window = {"config1": None, "config2": 1024, "config3": 256}[name]
            kw.update(C=packet_bytes, window=None if window is None else window * chunk // packet_bytes)
        w = getattr(wl, name)(seed=seed, relay=relay, **kw)
        calls = [dict(name=ph.name, op=ph.op, descs=ph.descs, n_unique=ph.n_unique,
                      payload_bytes=ph.payload_bytes, algo_bytes=ph.algo_bytes, scatter=False)
                 for ph in w.phases]
        return w, calls, packet_bytes or chunk
    if name == "direct-rs":
        w = wl.direct_reduce_scatter("direct-reduce-scatter-1GiB-f32", seed, R=8, M=1 << 30, C=128 << 10, dtype=0,
                                     paths=64, dup=0.005, dist="uniform")
        ph = w.phases[0]
        return w, [dict(name="gather-reduce", op=SUM, descs=ph.descs, n_unique=ph.n_unique,
                        payload_bytes=ph.payload_bytes, algo_bytes=ph.algo_bytes, scatter=False, gather=True)], 128 << 10
    if name == "config4":
        w = wl.config4(seed=seed)
        ph = w.phases[0]
        return w, [dict(name="scatter", op=COPY, descs=ph.descs, n_unique=ph.n_unique,
                        payload_bytes=ph.payload_bytes, algo_bytes=ph.algo_bytes, scatter=True)], 16 << 10
    if name in ("config5", "config5-single"):
        w, msgs = wl.config5(seed=seed, n_msgs=n_msgs)
        group = per_call if name == "config5" else 1  # at most 128 messages in flight per connection
        calls = []
        for lo in range(0, len(msgs), group):
            ms = msgs[lo:lo + group]
            for key, op in (("rs", SUM), ("ag", COPY)):
                d = np.concatenate([m[key] for m in ms])
                uniq, pay, algo = call_stats(d, op)
                calls.append(dict(name=key, op=op, descs=d, n_unique=uniq, payload_bytes=pay,
                                  algo_bytes=algo, scatter=False))
        w.extra["n_msgs"] = len(msgs)
        return w, calls, 4 << 10
    raise SystemExit(f"unknown workload {name}; choose from {sorted(WORKLOADS)}")


def to_dev(torch, a, shift=0):
    """Device copy of a numpy buffer as raw bytes, `shift` bytes into a larger allocation."""
    flat = torch.from_numpy(np.ascontiguousarray(a).view(np.uint8).reshape(-1))
    if not shift:
        return flat.cuda()
    t = torch.empty(flat.numel() + shift, dtype=torch.uint8, device="cuda")[shift:]
    t.copy_(flat)
    return t


def headline(workload, args, payload, seconds, steps, warmup, dtype, config):
    """The fields every line carries; `seconds` is the time of one step."""
    return {
        "metric": METRIC, "value": round(payload / seconds / 1e9, 2), "unit": "GB/s", "n_gpus": 1,
        "steps": steps, "warmup": warmup, "ms_per_step": round(seconds * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": dtype, "data": "synthetic",
        "config": {"workload": f"{workload}: {WORKLOADS[workload]}", "seed": args.seed, **config},
    }


def same_bytes(got, expected):
    return all(np.array_equal(np.ascontiguousarray(g).view(np.uint8).reshape(-1),
                              np.ascontiguousarray(e).view(np.uint8).reshape(-1)) for g, e in zip(got, expected))


def finish(result, ok=True):
    print(json.dumps(result))
    if not ok:
        sys.exit(1)


# ---- small messages fed one at a time ------------------------------------------------------------

def small_message_job(args, torch):
    from synth import workloads as wl
    w, msgs = wl.config5(seed=args.seed, n_msgs=args.messages)
    acc, recv = to_dev(torch, w.acc), to_dev(torch, w.recv_stage)
    out = torch.zeros(w.out_bytes, dtype=torch.uint8, device="cuda")
    bitmap = torch.zeros((w.n_bits + 31) // 32, dtype=torch.int32, device="cuda")
    return w, msgs, acc, recv, out, bitmap


def small_message_result(name, args, w, msgs, per_msg, reps, first, extra_config):
    """The JSON line of a one-message-at-a-time feed, with the oracle's single-core time over the
    same messages and the parity of the first pass against it."""
    from synth.layout import SUM, COPY, F32
    payload = sum(m["payload_bytes"] for m in msgs)
    unique = sum(m["n_unique"] for m in msgs)
    algo = sum(m["algo_bytes"] for m in msgs)
    step = per_msg * len(msgs)
    result = headline(name, args, payload, step, reps, 1, "f32",
                      dict(messages=len(msgs), unique_chunks=unique, payload_bytes=payload, algorithmic_bytes=algo,
                           **extra_config))
    result.update({"chunks_per_s": round(unique / step, 1), "us_per_message": round(per_msg * 1e6, 3),
                   "step_hbm_frac": round(algo / step / 1e9 / PEAK_HBM_GBS, 4), "roofline": None})
    ok = True
    if not args.no_cpu_baseline:
        import oracle
        eacc, eout, seen = w.acc.copy(), np.zeros(w.out_bytes, dtype=np.uint8), oracle.new_seen(w.n_bits)
        t0 = time.perf_counter()
        for m in msgs:
            oracle.apply(eacc, eout, w.recv_stage, m["rs"], seen, F32, SUM, check=False)
            oracle.apply(eacc, eout, w.recv_stage, m["ag"], seen, F32, COPY, check=False)
        cpu_t = time.perf_counter() - t0
        result["cpu_baseline"] = {"value": round(payload / cpu_t / 1e9, 3), "unit": "GB/s", "cores": 1,
                                  "kind": "oracle", "sample": f"all {len(msgs)} messages once, {cpu_t:.1f} s"}
        ok = same_bytes(first, (eacc, eout, oracle.pack_bitmap(seen)))
        result["parity_first_pass"] = "bit-exact vs oracle (acc, out_stage, bitmap)" if ok else "MISMATCH"
    return result, ok


def latency_us(samples):
    return {"median": round(float(np.median(samples)) * 1e6, 2), "p99": round(float(np.percentile(samples, 99)) * 1e6, 2)}


def bench_graph_feed(args, pkg, torch):
    """Small-message regime fed through descriptor slots: K pinned slots (records + counts for
    the two phases), one captured graph per slot.  Per message the host copies the records
    into the next slot and replays its graph; a slot is reused only after its previous replay
    has finished.  Also measures the host-observed completion latency of one message."""
    from synth.layout import SUM, COPY, F32
    w, msgs, acc, recv, out, bitmap = small_message_job(args, torch)
    cap = max(max(len(m["rs"]), len(m["ag"])) for m in msgs)
    K = 32
    slots = []
    side = torch.cuda.Stream()
    for _ in range(K):
        d_rs = torch.zeros(cap * 32, dtype=torch.uint8, pin_memory=True)
        d_ag = torch.zeros(cap * 32, dtype=torch.uint8, pin_memory=True)
        cnt = torch.zeros(8, dtype=torch.uint8, pin_memory=True)
        g = torch.cuda.CUDAGraph()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.graph(g, stream=side):
            pkg.uccl_chunk_apply_indirect(acc, out, recv, d_rs, cnt[0:4], cap, bitmap, F32, SUM, opts=(4096, 0))
            pkg.uccl_chunk_apply_indirect(acc, out, recv, d_ag, cnt[4:8], cap, bitmap, F32, COPY, opts=(4096, 0))
        slots.append(dict(rs=d_rs.numpy(), ag=d_ag.numpy(), cnt=cnt.numpy().view(np.uint32), graph=g,
                          done=torch.cuda.Event(), keep=(d_rs, d_ag, cnt)))
    raw = [(m["rs"].view(np.uint8).reshape(-1), m["ag"].view(np.uint8).reshape(-1), len(m["rs"]), len(m["ag"]))
           for m in msgs]

    def feed(i):
        sl = slots[i % K]
        sl["done"].synchronize()
        rs, ag, n_rs, n_ag = raw[i]
        sl["rs"][:len(rs)] = rs
        sl["ag"][:len(ag)] = ag
        sl["cnt"][0], sl["cnt"][1] = n_rs, n_ag
        sl["graph"].replay()
        sl["done"].record()

    def one_pass():
        pkg.uccl_dedup_reset(bitmap, w.n_bits)
        for i in range(len(msgs)):
            feed(i)

    one_pass()
    torch.cuda.synchronize()
    first = (acc.cpu().numpy(), out.cpu().numpy(), bitmap.cpu().numpy().view(np.uint32))
    t0 = time.perf_counter()
    reps = max(1, args.steps // 10)
    for _ in range(reps):
        one_pass()
    torch.cuda.synchronize()
    per_msg = (time.perf_counter() - t0) / reps / len(msgs)

    # completion latency of a single message, host clock: slot write + replay + wait
    lat = []
    pkg.uccl_dedup_reset(bitmap, w.n_bits)
    torch.cuda.synchronize()
    for i in range(min(len(msgs), 300)):
        t0 = time.perf_counter()
        feed(i)
        slots[i % K]["done"].synchronize()
        lat.append(time.perf_counter() - t0)
    # the same with two eager calls per message and device-resident records
    eager = lambda m, k, op: pkg.uccl_prepare(pkg.uccl_chunk_apply, acc, out, recv, to_dev(torch, m[k]), len(m[k]), bitmap, F32, op)
    d_dev = [(eager(m, "rs", SUM), eager(m, "ag", COPY)) for m in msgs[:300]]
    lat_eager = []
    pkg.uccl_dedup_reset(bitmap, w.n_bits)
    torch.cuda.synchronize()
    for a, b in d_dev:
        t0 = time.perf_counter()
        a()
        b()
        torch.cuda.synchronize()
        lat_eager.append(time.perf_counter() - t0)
    result, ok = small_message_result("config5-graph", args, w, msgs, per_msg, reps, first,
                                      dict(slots=K, slot_capacity_records=cap))
    result["completion_latency_us"] = {"graph_slot": latency_us(lat), "two_eager_calls": latency_us(lat_eager)}
    finish(result, ok)


def bench_feed(args, pkg, torch):
    """Small-message regime through uccl_feed: per message two pushes and a poll."""
    from synth.layout import SUM, COPY, F32
    w, msgs, acc, recv, out, bitmap = small_message_job(args, torch)
    feed = pkg.uccl_feed_create(acc, out, recv, bitmap, F32, SUM, COPY, 65536, 8)
    # every push marshalled once (pkg.uccl_prepare): what is timed is the C calls, as a native control path makes them
    recs = [tuple(pkg.uccl_prepare(pkg.uccl_feed_push, feed, lane, np.ascontiguousarray(m[k])) for lane, k in ((0, "rs"), (1, "ag")))
            for m in msgs]
    poll = pkg.uccl_prepare(pkg.uccl_feed_poll, feed)

    def one_pass():
        pkg.uccl_dedup_reset(bitmap, w.n_bits)
        for rs, ag in recs:
            rs()
            ag()
            poll()
        pkg.uccl_feed_sync(feed)

    one_pass()
    first = (acc.cpu().numpy(), out.cpu().numpy(), bitmap.cpu().numpy().view(np.uint32))
    before = pkg.uccl_feed_get_stats(feed)
    reps = max(1, args.steps // 10)
    t0 = time.perf_counter()
    for _ in range(reps):
        one_pass()
    per_msg = (time.perf_counter() - t0) / reps / len(msgs)
    after = pkg.uccl_feed_get_stats(feed)
    lat = []
    pkg.uccl_dedup_reset(bitmap, w.n_bits)
    torch.cuda.synchronize()
    for rs, ag in recs[:300]:
        t0 = time.perf_counter()
        rs()
        ag()
        pkg.uccl_feed_sync(feed)
        lat.append(time.perf_counter() - t0)
    pkg.uccl_feed_destroy(feed)
    flushes = (after["flushes"] - before["flushes"]) / reps
    result, ok = small_message_result("config5-feed", args, w, msgs, per_msg, reps, first,
                                      dict(slots=8, slot_capacity_records=65536))
    result["feed"] = {"hand_overs_per_pass": round(flushes, 1), "messages_per_hand_over": round(len(msgs) / max(flushes, 1), 1),
                      "largest_hand_over_records": after["max_batch"], "slot_waits": after["slot_waits"]}
    result["completion_latency_us"] = latency_us(lat)
    finish(result, ok)


# ---- single kernels ----------------------------------------------------------------------------

def launch_time_us(pkg, torch, launch, reps=30, skip=5, before=None):
    """Median duration of launch(k), from event pairs attached to its dispatch; before(k), if given,
    runs ahead of it untimed (launches of its own, such as a bitmap reset)."""
    evs = []
    for k in range(reps):
        if before is not None:
            before(k)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        b.record()
        pkg.uccl_time_next_launch(a, b)
        launch(k)
        evs.append((a, b))
    torch.cuda.synchronize()
    return float(np.median([a.elapsed_time(b) for a, b in evs[skip:]])) * 1e3


def time_feedback_kernels(pkg, torch, bitmap, n_bits):
    """(acknowledgement report over this workload's bitmap, status of a 128 x 256-bit message window), in us."""
    report = torch.zeros(32 + 16 * 64, dtype=torch.uint8, device="cuda")
    report_us = launch_time_us(pkg, torch, lambda k: pkg.uccl_dedup_report(bitmap, n_bits, report, 64))
    hdr = report.cpu().numpy()
    assert int(hdr[:8].view(np.uint64)[0]) == n_bits and int(hdr[20:24].view(np.uint32)[0]) == 1, \
        "after a full step every chunk is acknowledged"
    # the same bitmap with every 97th chunk missing (a lossy phase): the report then lists ranges
    words = bitmap.cpu().numpy().view(np.uint32).copy()
    holes = np.arange(50, n_bits, 97, dtype=np.int64)
    np.bitwise_and.at(words, holes >> 5, ~(np.uint32(1) << (holes & 31).astype(np.uint32)))
    lossy = torch.from_numpy(words.view(np.int32)).cuda()
    lossy_us = {}
    for max_ranges in (64, 4096):
        rep = torch.zeros(32 + 16 * max_ranges, dtype=torch.uint8, device="cuda")
        lossy_us[max_ranges] = launch_time_us(pkg, torch, lambda k: pkg.uccl_dedup_report(lossy, n_bits, rep, max_ranges))
        h = rep.cpu().numpy()
        if len(holes):
            assert int(h[:8].view(np.uint64)[0]) == 50 and int(h[8:16].view(np.uint64)[0]) == n_bits - len(holes)
            assert int(h[16:20].view(np.uint32)[0]) == len(holes) - (1 if holes[-1] == n_bits - 1 else 0)
    win = torch.zeros(128 * 8, dtype=torch.int32, device="cuda")
    win[: 64 * 8] = -1                                   # half of the slots complete
    n_chunks = torch.full((128,), 200, dtype=torch.int32, device="cuda")
    status = torch.zeros(128 * 4, dtype=torch.int32, device="cuda")
    status_us = launch_time_us(pkg, torch, lambda k: pkg.uccl_message_status(win, n_chunks, 128, 256, status, False))
    assert int(status.view(128, 4)[:, 2].sum()) == 64
    return report_us, status_us, {"holes": int(len(holes)), "median_us_by_max_ranges": {str(k): round(v, 2) for k, v in lossy_us.items()}}


def calibration_copy(torch):
    """One plain 1 GiB device-to-device copy, the known quantity the traffic counters are scaled by."""
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    dst.copy_(src)
    torch.cuda.synchronize()


def bench_segment(args, pkg, torch):
    """Sender side: the rank's own segment cut into staged chunks with send records (the first hop
    of a ring).  One step = one uccl_chunk_segment call; 1 byte read + 1 byte written per payload byte."""
    import oracle
    from synth import payload as pl
    rows = {}
    for shape, seg_bytes, chunk in (("config2", (256 << 20) // 16, 32 << 10), ("config3", (1 << 30) // 8, 128 << 10)):
        n = seg_bytes // chunk
        host = pl.rng(args.seed, 5).integers(0, 256, seg_bytes, dtype=np.uint8)
        sets = [dict(t=to_dev(torch, host), stage=torch.zeros(seg_bytes, dtype=torch.uint8, device="cuda"),
                     recs=torch.zeros(n * 16, dtype=torch.uint8, device="cuda")) for _ in range(max(1, args.sets))]

        def step(k, sets=sets, seg_bytes=seg_bytes, chunk=chunk):
            s = sets[k % len(sets)]
            pkg.uccl_chunk_segment(s["stage"], s["t"], 0, seg_bytes, chunk, 0, chunk, s["recs"], 3, 0, 0)
        step(0)
        torch.cuda.synchronize()
        exp = np.zeros(seg_bytes, dtype=np.uint8)
        exp_d = oracle.segment(exp, host, 0, seg_bytes, chunk, conn_id=3)
        ok = (np.array_equal(sets[0]["stage"].cpu().numpy(), exp) and
              np.array_equal(sets[0]["recs"].cpu().numpy().view(oracle.SEND_DESC), exp_d))
        for k in range(args.warmup):
            step(k)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(args.steps):
            step(k)
        torch.cuda.synchronize()
        per = (time.perf_counter() - t0) / args.steps
        kernel_us = launch_time_us(pkg, torch, lambda k: step(k + 1))
        algo = 2 * seg_bytes + 16 * n
        rows[shape] = dict(segment_bytes=seg_bytes, chunk_bytes=chunk, chunks=n, ms_per_step=round(per * 1e3, 4),
                           payload_GBps=round(seg_bytes / per / 1e9, 1), kernel_us=round(kernel_us, 2),
                           kernel_hbm_frac=round(algo / (kernel_us * 1e-6) / 1e9 / PEAK_HBM_GBS, 4),
                           parity="bit-exact vs oracle (staging, send records)" if ok else "MISMATCH")
        del sets
    big = rows["config3"]
    result = headline("segment", args, big["segment_bytes"], big["ms_per_step"] * 1e-3, args.steps, args.warmup, "u8",
                      dict(buffer_sets=max(1, args.sets)))
    result["segments"] = rows
    algo = 2 * big["segment_bytes"] + 16 * big["chunks"]
    achieved = algo / (big["kernel_us"] * 1e-6) / 1e9
    result["roofline"] = {"bound": "hbm", "kernel": "segment_kernel (config3's shape)", "achieved": round(achieved, 1),
                          "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(achieved / PEAK_HBM_GBS, 4), "traffic": None,
                          "algorithmic_bytes_per_launch": algo, "avg_launch_ms": round(big["kernel_us"] * 1e-3, 5)}
    finish(result, all(r["parity"] != "MISMATCH" for r in rows.values()))


def bench_calls(args, pkg, torch):
    """Where the launch choices of the library come from: kernel time (event pair attached to the
    dispatch, median) of one call of n records of C bytes each, over buffers rotating over four sets.
    `auto` is the library's own choice for (n, C); the other columns force the number of parts."""
    from synth.layout import DESC, F32, SUM
    rng = np.random.default_rng(args.seed)
    sizes = [(4 << 10, (16, 57, 128, 512, 2048)), (8 << 10, (16, 57, 128, 512, 2048, 8192)),
             (16 << 10, (16, 57, 128, 1024, 4096, 8192)), (32 << 10, (8, 32, 57, 128, 512, 1024, 2047, 2048)),
             (64 << 10, (8, 57, 128, 256, 512, 1024, 2048)), (128 << 10, (8, 57, 128, 256, 512, 1024, 2048))]
    most = max(c * max(ns) for c, ns in sizes)
    n_sets = max(1, args.sets)
    sets = [dict(acc=torch.zeros(most, dtype=torch.uint8, device="cuda"), recv=torch.ones(most, dtype=torch.uint8, device="cuda"),
                 out=torch.zeros(most, dtype=torch.uint8, device="cuda"), bm=torch.zeros(8192 // 32, dtype=torch.int32, device="cuda"))
            for _ in range(n_sets)]
    def call_us(call, n_bits):
        """Median kernel time of call(buffer set); the bitmap reset before it is a launch of its own."""
        return round(launch_time_us(pkg, torch, lambda k: call(sets[k % n_sets]), reps=args.steps, skip=args.warmup,
                                    before=lambda k: pkg.uccl_dedup_reset(sets[k % n_sets]["bm"], n_bits)), 2)

    rows = []
    for chunk, counts in sizes:
        for n in counts:
            perm = rng.permutation(n)
            d = np.zeros(n, dtype=DESC)
            d["src_off"] = np.arange(n, dtype=np.uint64) * chunk
            d["dst_off"] = d["out_off"] = perm.astype(np.uint64) * chunk
            d["len"], d["seq"] = chunk, perm
            recs = to_dev(torch, d)
            row = dict(chunk_bytes=chunk, records=n, algorithmic_bytes=n * (4 * chunk + 36), launch=pkg.uccl_launch_plan(n, (chunk, 0)))
            for label, parts in (("auto", 0), ("uncut", 1), ("parts8", 8), ("parts16", 16)):
                if parts > 1 and (chunk < (32 << 10) or n * parts > 4096):
                    continue   # a workgroup takes several records of smaller chunks: parts do not apply
                row[label + "_us"] = call_us(lambda s: pkg.uccl_chunk_apply_opts(
                    s["acc"], s["out"], s["recv"], recs, n, s["bm"], F32, SUM, opts=(chunk, parts)), n)
            rows.append(row)
    # the multi-source fold (seven senders per destination chunk) on calls of few records
    GATHER = np.dtype([("dst_off", "<u8"), ("out_off", "<u8"), ("len", "<u4"), ("seq", "<u4"), ("n_src", "<u4"),
                       ("reserved", "<u4"), ("src_off", "<u8", (16,))])
    n_src, gather_rows = 7, []
    for chunk in (32 << 10, 64 << 10, 128 << 10):
        for n in (1, 8, 32, 128, 512):
            if n * chunk * n_src > most:
                continue
            d = np.zeros(n, dtype=GATHER)
            d["dst_off"] = np.arange(n, dtype=np.uint64) * chunk
            d["out_off"] = np.uint64(0xFFFFFFFFFFFFFFFF)
            d["len"], d["seq"], d["n_src"] = chunk, np.arange(n), n_src
            for j in range(n_src):
                d["src_off"][:, j] = (j * n + np.arange(n, dtype=np.uint64)) * chunk
            recs = to_dev(torch, d)
            row = dict(chunk_bytes=chunk, records=n, sources=n_src, algorithmic_bytes=n * ((n_src + 2) * chunk + 164),
                       launch=pkg.uccl_launch_plan(n, (chunk, 0), gather=True))
            for label, parts in (("auto", 0), ("uncut", 1)):
                row[label + "_us"] = call_us(lambda s: pkg.uccl_chunk_reduce_gather(
                    s["acc"], None, s["recv"], recs, n, s["bm"], F32, SUM, opts=(chunk, parts)), n)
            gather_rows.append(row)
    ok = pkg.uccl_claim_timeouts() == 0
    big = rows[-1]
    result = headline("calls", args, big["records"] * big["chunk_bytes"], big["auto_us"] * 1e-6, args.steps, args.warmup, "f32",
                      dict(buffer_sets=n_sets))
    result["calls"] = rows
    result["gather_calls"] = gather_rows
    result["claim_timeouts"] = pkg.uccl_claim_timeouts()
    result["roofline"] = {"bound": "hbm", "kernel": "the largest call of the sweep", "achieved": round(big["algorithmic_bytes"] / (big["auto_us"] * 1e-6) / 1e9, 1),
                          "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(big["algorithmic_bytes"] / (big["auto_us"] * 1e-6) / 1e9 / PEAK_HBM_GBS, 4),
                          "traffic": None, "algorithmic_bytes_per_launch": big["algorithmic_bytes"], "avg_launch_ms": round(big["auto_us"] * 1e-3, 5)}
    finish(result, ok)


# ---- the CPU oracle beside it ----------------------------------------------------------------------

def cpu_baselines(w, calls, payload, arrivals, first):
    """The oracle as it stands on one host core (about 10 s of repetitions of the whole step) and,
    for plain apply calls, the same definition dealt over the host cores; also the parity of the
    GPU's first pass against the oracle's result.  Returns (fields to add to the line, parity ok)."""
    import oracle
    out = {}
    reps, cpu_t, exp = 0, 0.0, None
    while cpu_t < 10.0 and reps < 64:
        eacc = w.acc.copy()
        eout = np.zeros(max(w.out_bytes, 16), dtype=np.uint8)
        seen = oracle.new_seen(w.n_bits)
        t0 = time.perf_counter()
        for c in calls:
            if c.get("gather"):
                oracle.reduce_gather(eacc, None, w.recv_stage, c["descs"], seen, w.dtype, c["op"])
            elif c["scatter"]:
                oracle.scatter(eacc.view(np.uint8), w.recv_stage, c["descs"], seen, check=False)
            else:
                oracle.apply(eacc, eout, w.recv_stage, c["descs"], seen, w.dtype, c["op"], check=False)
        cpu_t += time.perf_counter() - t0
        reps += 1
        if exp is None:
            exp = (eacc, eout[:w.out_bytes], oracle.pack_bitmap(seen))
    out["cpu_baseline"] = {
        "value": round(payload * reps / cpu_t / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
        "cpu": cpu_model(),
        "sample": f"the whole step ({len(calls)} calls, {arrivals} arrivals, {payload} payload bytes) x {reps} repetitions, {cpu_t:.1f} s",
    }
    # the same definition on all host cores of this machine's share (serial dedup, then the unique
    # chunks dealt to threads); reported beside the single-core figure, only for plain apply calls
    if not any(c.get("gather") or c["scatter"] for c in calls):
        threads = max(1, min(16, os.cpu_count() or 1))
        reps_t, cpu_tt, same_t = 0, 0.0, True
        while cpu_tt < 5.0 and reps_t < 64:
            tacc = w.acc.copy()
            tout = np.zeros(max(w.out_bytes, 16), dtype=np.uint8)
            seen = oracle.new_seen(w.n_bits)
            t0 = time.perf_counter()
            for c in calls:
                oracle.apply_threaded(tacc, tout, w.recv_stage, c["descs"], seen, w.dtype, c["op"], threads)
            cpu_tt += time.perf_counter() - t0
            reps_t += 1
            if reps_t == 1:
                same_t = (np.array_equal(tacc.view(np.uint8), exp[0].view(np.uint8)) and
                          np.array_equal(tout[:w.out_bytes], exp[1]))
        out["cpu_baseline_threaded"] = {
            "value": round(payload * reps_t / cpu_tt / 1e9, 3), "unit": "GB/s", "cores": threads,
            "kind": "oracle, unique chunks dealt to threads after a serial dedup pass",
            "equals_single_core_result": bool(same_t),
            "sample": f"the whole step x {reps_t} repetitions, {cpu_tt:.1f} s",
        }
    ok = same_bytes(first, exp)
    out["parity_first_pass"] = "bit-exact vs oracle (acc, out_stage, bitmap)" if ok else "MISMATCH"
    return out, ok


def two_pass_parity(w, first):
    """The two-pass mode's first pass against the oracle's single-pass definition (acc, out_stage)."""
    import oracle
    eacc, eout, seen = w.acc.copy(), np.zeros(max(w.out_bytes, 16), dtype=np.uint8), oracle.new_seen(w.n_bits)
    for ph in w.phases:
        oracle.apply(eacc, eout, w.recv_stage, ph.descs, seen, w.dtype, ph.op, check=False)
    return (np.array_equal(first[0], eacc.view(np.uint8).reshape(-1)) and
            np.array_equal(first[1], eout[:w.out_bytes]))


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="config2", choices=sorted(WORKLOADS))
    ap.add_argument("--seed", type=int, default=1)
    ap.add_argument("--sets", type=int, default=4, help="buffer sets the steps rotate over")
    ap.add_argument("--messages", type=int, default=10000, help="config5: number of messages")
    ap.add_argument("--duplicates", type=float, default=None, help="config1-3: retransmitted share of the chunks instead of the recipe's")
    ap.add_argument("--no-prepare", action="store_true", help="marshal every call's arguments anew instead of once")
    ap.add_argument("--streams", type=int, default=1,
                    help="config5: issue consecutive message batches round-robin on this many streams "
                         "(batches are independent of each other; the two calls of a batch stay ordered)")
    ap.add_argument("--messages-per-call", type=int, default=128,
                    help="config5: messages batched into one call (128 = in-flight messages of one connection)")
    ap.add_argument("--parts", type=int, default=0,
                    help="workgroups per record for calls of few large records (0 = the library decides, 1 = never cut)")
    ap.add_argument("--no-chunk-hint", action="store_true", help="do not tell the library the chunk size")
    ap.add_argument("--chunk-hint", type=int, default=None, help="override the chunk size given with each call (bytes)")
    ap.add_argument("--records-per-call", type=int, default=0,
                    help="cut every phase into calls of this many records, queued back to back (0 = one call per phase)")
    ap.add_argument("--packet-bytes", type=int, default=0,
                    help="config1-3: arrivals are packets of this many bytes instead of whole chunks (Section 3.1, "
                         "unreliable datagrams: one MTU-sized payload per arrival); with --two-pass the reduction "
                         "reads the transport buffer at the configuration's chunk size")
    ap.add_argument("--relay", action="store_true",
                    help="ring workloads: flag intermediate reduce-scatter steps forward-only (their partial "
                         "sums are not written back to the accumulator: 3 instead of 4 bytes per payload byte)")
    ap.add_argument("--two-pass", action="store_true",
                    help="ring workloads: run the paper's literal two-pass form (scattered memcpy into a transport "
                         "buffer, then reduce) instead of the fused single pass, for comparison")
    ap.add_argument("--graph", action="store_true",
                    help="capture each buffer set's step (reset + calls) in a HIP graph once and replay it: what a "
                         "launch-bound caller does (no per-kernel timing; captured calls are never cut into parts)")
    ap.add_argument("--stagger", type=int, default=0,
                    help="place acc and out_stage 1 and 2 times this many bytes (a multiple of 256) into their "
                         "allocations, to move the streams' relative alignment in the memory channels")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the dense streaming kernels")
    ap.add_argument("--also-warm", action="store_true", help="also time the loop over one buffer set (cache resident)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy (known traffic to scale hardware counters by)")
    return ap.parse_args()


def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: the path is measured as one GPU's share on one GPU; --gpus N>1 is not supported "
              "(the path shards as one independent rank per GPU, there is nothing to aggregate)", file=sys.stderr)
        sys.exit(2)
    if args.stagger % 256:
        raise SystemExit("--stagger must be a multiple of 256")

    import torch
    import paper_2504_17307_amd as pkg
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    pkg.uccl_init()   # loads the library (raises if it is not built) and makes its scratch memory
    if args.workload == "config5-graph":
        return bench_graph_feed(args, pkg, torch)
    if args.workload == "config5-feed":
        return bench_feed(args, pkg, torch)
    if args.workload == "calls":
        return bench_calls(args, pkg, torch)
    if args.workload == "segment":
        return bench_segment(args, pkg, torch)
    t0 = time.time()
    w, calls, chunk_bytes = build_job(args.workload, args.seed, args.messages, args.relay, args.messages_per_call,
                                      args.packet_bytes, args.duplicates)
    collective_chunk = {"config1": 64 << 10, "config2": 32 << 10, "config3": 128 << 10}.get(args.workload, chunk_bytes)
    if args.chunk_hint is not None:
        chunk_bytes = args.chunk_hint
    opts = (0 if args.no_chunk_hint else chunk_bytes, args.parts)   # per-call tuning, passed with every call
    transport_bytes = 0
    if args.two_pass:
        calls, transport_bytes = two_pass_calls(w, chunk_bytes, collective_chunk // chunk_bytes if args.packet_bytes else 1)
    print(f"[bench] built {w.name} in {time.time() - t0:.1f}s: {w.note}", file=sys.stderr, flush=True)

    sets = []
    for _ in range(max(1, args.sets)):
        out = torch.zeros(max(w.out_bytes, 16) + 2 * args.stagger, dtype=torch.uint8, device="cuda")[2 * args.stagger:]
        sets.append(dict(acc=to_dev(torch, w.acc, args.stagger), recv=to_dev(torch, w.recv_stage), out=out,
                         transport=torch.zeros(max(transport_bytes, 16), dtype=torch.uint8, device="cuda")))
    bitmap = torch.zeros((w.n_bits + 31) // 32, dtype=torch.int32, device="cuda")
    bitmap2 = torch.zeros((w.n_bits + 31) // 32, dtype=torch.int32, device="cuda")
    descs = [to_dev(torch, c["descs"]) for c in calls]
    counts = [len(c["descs"]) for c in calls]
    streams = [torch.cuda.Stream() for _ in range(args.streams)] if args.streams > 1 else None

    def call(i, s):
        if streams is not None:  # calls come in (reduce-scatter, allgather) pairs per batch
            with torch.cuda.stream(streams[(i // 2) % len(streams)]):
                return call_on_current(i, s)
        return call_on_current(i, s)

    # arguments are marshalled once per (call, buffer set) (pkg.uccl_prepare), unless the stream changes between calls
    prepared = {} if streams is None and not args.graph and not args.no_prepare else None

    def call_on_current(i, s):
        c = calls[i]
        bm = bitmap2 if c.get("bm") == "bitmap2" else bitmap
        rec = 160 if c.get("gather") else 32
        per = args.records_per_call or counts[i]
        for lo in range(0, counts[i], max(per, 1)):
            if prepared is not None and (i, lo, id(s)) in prepared:
                prepared[(i, lo, id(s))]()
                continue
            n = min(per, counts[i] - lo)
            d = descs[i][lo * rec:(lo + n) * rec]
            if c.get("gather"):
                f = (pkg.uccl_chunk_reduce_gather, s["acc"], None, s["recv"], d, n, bm, w.dtype, c["op"])
            elif c["scatter"]:
                f = (pkg.uccl_chunk_scatter_opts, s[c.get("dst", "acc")], s[c.get("src", "recv")], d, n, bm)
            else:
                f = (pkg.uccl_chunk_apply_opts, s["acc"], s["out"], s[c.get("src", "recv")], d, n, bm, w.dtype, c["op"])
            if prepared is None:
                f[0](*f[1:], opts=opts)
            else:
                prepared[(i, lo, id(s))] = pkg.uccl_prepare(*f, opts=opts)
                prepared[(i, lo, id(s))]()

    def issue(k, timed=None):
        """Enqueue one step on buffer set k % len(sets)."""
        s = sets[k % len(sets)]
        if streams is not None:
            for st in streams:
                torch.cuda.current_stream().wait_stream(st)
        pkg.uccl_dedup_reset(bitmap, w.n_bits)
        if streams is not None:
            for st in streams:
                st.wait_stream(torch.cuda.current_stream())
        if args.two_pass:
            pkg.uccl_dedup_reset(bitmap2, w.n_bits)
        for i in range(len(calls)):
            if timed is not None and i in timed and k % EVENT_STRIDE == 0:
                # a pre-made event pair attached to the dispatch itself: the kernel's own begin and end
                pkg.uccl_time_next_launch(*timed[i][k // EVENT_STRIDE])
            call(i, s)

    # one pass from the pristine state, kept for the parity check against the oracle
    issue(0)
    torch.cuda.synchronize()
    first = (sets[0]["acc"].cpu().numpy(), sets[0]["out"][:w.out_bytes].cpu().numpy(),
             bitmap.cpu().numpy().view(np.uint32))
    for k in range(1, len(sets) if prepared is not None else 0):   # marshal the other sets' calls before anything is timed
        issue(k)

    graphs = None
    if args.graph:
        assert streams is None, "--graph and --streams do not combine"
        graphs, side = [], torch.cuda.Stream()
        for k in range(len(sets)):
            g = torch.cuda.CUDAGraph()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.graph(g, stream=side):
                issue(k)
            graphs.append(g)
        torch.cuda.synchronize()

    def step(k, timed=None):
        if graphs is not None:
            graphs[k % len(graphs)].replay()
        else:
            issue(k, timed)

    # Per-launch durations are taken INSIDE the timed steps (every EVENT_STRIDE-th one): a HIP
    # event pair, made and recorded once beforehand, is attached to the dispatch of the kernel on
    # the stream it runs on (torch's current stream).  Workloads with many calls per step time the
    # largest call of each op.
    by_op = {}
    for i, c in enumerate(calls):
        if c["op"] not in by_op or c["algo_bytes"] > calls[by_op[c["op"]]]["algo_bytes"]:
            by_op[c["op"]] = i
    timed = {}
    if streams is None and not args.records_per_call and graphs is None:
        for i in by_op.values():
            timed[i] = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                        for _ in range((args.steps + EVENT_STRIDE - 1) // EVENT_STRIDE)]
            for a, b in timed[i]:
                a.record()
                b.record()
    torch.cuda.synchronize()

    def timed_loop(n_sets, events=None):
        nonlocal sets, graphs
        keep, keep_g = sets, graphs
        sets, graphs = sets[:n_sets], (graphs[:n_sets] if graphs is not None else None)
        for k in range(args.warmup):
            step(k)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(args.steps):
            step(k, events)
        torch.cuda.synchronize()
        el = time.perf_counter() - t0
        sets, graphs = keep, keep_g
        return el

    elapsed = timed_loop(len(sets), timed)
    warm_elapsed = timed_loop(1) if (args.also_warm and len(sets) > 1) else None
    if not timed:  # overlapping streams, graph replays, or phases cut into several launches: no per-kernel attribution
        timed = {i: [] for i in by_op.values()}
    kernels = []
    for i, evs in timed.items():
        t = np.array([a.elapsed_time(b) for a, b in evs]) if evs else np.array([float("nan")])
        c = calls[i]
        kernels.append(dict(call=c["name"], op=["SUM", "MAX", "MIN", "COPY"][c["op"]], records=counts[i],
                            algorithmic_bytes=c["algo_bytes"], payload_bytes=c["payload_bytes"],
                            avg_ms=round(float(t.mean()), 5), median_ms=round(float(np.median(t)), 5),
                            min_ms=round(float(t.min()), 5),
                            hbm_frac=round(c["algo_bytes"] / (t.mean() * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)))
    dom = max(kernels, key=lambda k: k["algorithmic_bytes"])

    def timed_ms(i):
        evs = timed.get(i) or []
        return float(np.mean([a.elapsed_time(b) for a, b in evs])) if evs else 0.0

    report_us, status_us, lossy_report = time_feedback_kernels(pkg, torch, bitmap, w.n_bits)
    timeouts = pkg.uccl_claim_timeouts()
    stream_ceiling = None
    if not args.no_ceilings:  # last: the dense kernels overwrite the accumulators and staging buffers
        n_src = int(calls[0]["descs"]["n_src"].max()) if calls[0].get("gather") else 0
        reorder_window = {"config2": 1024, "config3": 256}.get(args.workload, 0)   # in chunks, as the recipe states
        from paper_2504_17307_amd.probe import stream_ceilings   # the dense streaming kernels and their driver
        stream_ceiling = stream_ceilings(torch, sets, max(dom["payload_bytes"] // max(n_src, 1), 2048),
                                         max(collective_chunk, 32 << 10), n_src, window_blocks=reorder_window)
    if args.calibration_copy:
        calibration_copy(torch)

    payload = sum(c["payload_bytes"] for c in calls)
    unique = sum(c["n_unique"] for c in calls)
    arrivals = sum(counts)
    algo = sum(c["algo_bytes"] for c in calls)
    per_step = elapsed / args.steps
    per_kernel = not np.isnan(dom["avg_ms"])
    achieved = dom["algorithmic_bytes"] / (dom["avg_ms"] * 1e-3) / 1e9 if per_kernel else algo / per_step / 1e9
    cache_note = ("buffers rotate over %d sets: HBM resident, not cache resident" % len(sets)
                  if (w.acc.nbytes + w.recv_stage.nbytes + w.out_bytes) * len(sets) > (1 << 30)
                  else "working set fits the 256 MB last-level cache: an effective, not an HBM, figure")
    kernel_name = pkg.uccl_launch_plan(args.records_per_call or dom["records"], (opts[0], args.parts), bool(calls[0].get("gather")),
                                       dom["op"] != "COPY")["kernel"]   # what the library says it launches for the dominant call

    result = headline(args.workload, args, payload, per_step, args.steps, args.warmup,
                      {0: "f32", 1: "bf16", 2: "f16", 3: "i32"}[w.dtype],
                      {"unique_chunks": unique, "arrivals": arrivals, "payload_bytes": payload,
                       "algorithmic_bytes": algo, "parts": args.parts, "chunk_hint": opts[0], "buffer_sets": len(sets),
                       "forward_only_intermediate_steps": bool(args.relay), "two_pass": bool(args.two_pass),
                       "packet_bytes": args.packet_bytes or None, "duplicates": args.duplicates, "graph_replay": bool(args.graph),
                       "stagger_bytes": args.stagger or None, "prepared_calls": prepared is not None,
                       "calls_per_step": 1 + sum(-(-n // (args.records_per_call or max(n, 1))) for n in counts),
                       "records_per_call": args.records_per_call or None, "streams": args.streams, "cache": cache_note})
    result.update({
        "chunks_per_s": round(unique / per_step, 1), "arrivals_per_s": round(arrivals / per_step, 1),
        "step_hbm_frac": round(algo / per_step / 1e9 / PEAK_HBM_GBS, 4),
        "warm_cache": None if warm_elapsed is None else {
            "ms_per_step": round(warm_elapsed / args.steps * 1e3, 4),
            "value": round(payload / (warm_elapsed / args.steps) / 1e9, 2),
            "step_hbm_frac": round(algo / (warm_elapsed / args.steps) / 1e9 / PEAK_HBM_GBS, 4),
            "note": "same loop over one buffer set; the accumulator stays in the last-level cache"},
        "roofline": {
            "bound": "hbm",
            "kernel": f"{kernel_name}, {dom['call']} call ({dom['op']})",
            "basis": "the dominant kernel's own duration" if per_kernel else "whole step (no per-kernel attribution in this mode)",
            "achieved": round(achieved, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
            "frac": round(achieved / PEAK_HBM_GBS, 4),
            "traffic": MEASURED_TRAFFIC.get((args.workload, source_hash())),
            "algorithmic_bytes_per_launch": dom["algorithmic_bytes"], "avg_launch_ms": dom["avg_ms"] if per_kernel else None,
        },
        "kernels": kernels if per_kernel else [],
        # the reduce phase alone (its call's unique payload over its kernel's own duration)
        "reduce_phase_payload_GBps": (round(calls[by_op[0]]["payload_bytes"] / (timed_ms(by_op[0]) * 1e-3) / 1e9, 1)
                                      if per_kernel and 0 in by_op and timed_ms(by_op[0]) > 0 else None),
        "stream_ceiling": stream_ceiling,
        "device": device_info(torch),
        "dedup_report": {"n_bits": w.n_bits, "median_us": round(report_us, 2),
                         "what": "ack_report_kernel: cumulative ack, applied count, selective ranges",
                         "every_97th_chunk_missing": lossy_report},
        "message_status": {"slots": 128, "bits_per_slot": 256, "median_us": round(status_us, 2),
                           "what": "message_status_kernel: per-slot cumulative point, applied count, completion"},
        "claim_timeouts": timeouts,
    })
    if args.workload.startswith("config5"):
        result["us_per_message"] = round(per_step * 1e6 / w.extra["n_msgs"], 3)
        result["config"]["messages"] = w.extra["n_msgs"]

    ok = timeouts == 0
    if args.two_pass:
        same = two_pass_parity(w, first)
        result["parity_first_pass"] = ("two-pass result bit-exact vs the oracle's single-pass definition (acc, out_stage)"
                                       if same else "MISMATCH")
        ok = ok and same
    elif not args.no_cpu_baseline:
        extra, same = cpu_baselines(w, calls, payload, arrivals, first)
        result.update(extra)
        ok = ok and same
    finish(result, ok)


if __name__ == "__main__":
    main()
