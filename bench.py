#!/usr/bin/env python3
"""Benchmark of the receive-side chunk data path on one MI355X.

A step is one pass of the whole hot path over one rank's share of the collective: reset
the dedup bitmap, apply the reduce-scatter phase's arrival list (dedup, place, SUM, write
back, forward), apply the allgather phase's list (dedup, place, COPY, forward).  Inputs
are seeded synthetic chunk streams, resident in HBM before the timed region starts.

Prints one JSON line: whole-job reduced-payload GB/s, the HBM-roofline fraction of the
dominant kernel (algorithmic bytes / measured kernel time / 8 TB/s), and the CPU oracle
timed on the host cores of the same box as a reported baseline.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

PEAK_HBM_GBS = 8000.0  # MI355X published HBM3E peak, GB/s


def build_workload(name, seed):
    from synth import workloads as wl
    if name == "config2":
        return wl.config2(seed=seed), "allreduce rank share: R=16, 256 MiB bf16 normal(0,1), 32 KiB chunks, 256 paths, window 1024, 2% duplicates"
    if name == "config1":
        return wl.config1(seed=seed), "allreduce rank share: R=8, 4 MiB fp32 uniform[-1,1], 64 KiB chunks, 4 paths, 1% duplicates"
    if name == "config3":
        return wl.config3(seed=seed), "reduce-scatter rank share: R=8, 1 GiB fp32 uniform[-1,1], 128 KiB chunks, 64 paths, window 256, 0.5% duplicates"
    if name == "config2-small":
        return wl.config2(seed=seed, M=16 << 20), "config2 recipe at 16 MiB (functional check only)"
    raise SystemExit(f"unknown workload {name}")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="config2")
    ap.add_argument("--seed", type=int, default=1)
    ap.add_argument("--shape", type=int, default=0, help="launch shape id (0 = auto)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy (a kernel of known traffic that "
                         "hardware counters of the same run can be scaled by)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU's share on one GPU; --gpus N>1 is not supported "
              "(the path shards as one independent rank per GPU, there is nothing to aggregate)", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2504_17307_amd as pkg
    from synth.layout import COPY

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    pkg.load()
    pkg.uccl_set_launch_shape(args.shape)
    t0 = time.time()
    w, desc_text = build_workload(args.workload, args.seed)
    print(f"[bench] built {w.name} in {time.time() - t0:.1f}s: {w.note}", file=sys.stderr, flush=True)

    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a).view(np.uint8).reshape(-1)).cuda()
    acc = dev(w.acc)
    recv = dev(w.recv_stage)
    out = torch.zeros(max(w.out_bytes, 16), dtype=torch.uint8, device="cuda")
    bitmap = torch.zeros((w.n_bits + 31) // 32, dtype=torch.int32, device="cuda")
    descs = [dev(ph.descs) for ph in w.phases]
    counts = [len(ph.descs) for ph in w.phases]

    def step():
        pkg.uccl_dedup_reset(bitmap, w.n_bits)
        for ph, d, n in zip(w.phases, descs, counts):
            pkg.uccl_chunk_apply(acc, out, recv, d, n, bitmap, w.dtype, ph.op)

    # one pass from the pristine state, kept for the parity check against the oracle
    step()
    torch.cuda.synchronize()
    first = (acc.cpu().numpy(), out[:w.out_bytes].cpu().numpy(), bitmap.cpu().numpy().view(np.uint32))

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3

    # per-kernel durations: HIP events on the stream the kernels are launched on
    # (torch's current stream), one pair per launch
    kernel_ms = []
    for i, (ph, d, n) in enumerate(zip(w.phases, descs, counts)):
        evs = []
        for _ in range(args.steps):
            pkg.uccl_dedup_reset(bitmap, w.n_bits)
            for j, (ph2, d2, n2) in enumerate(zip(w.phases, descs, counts)):
                if j == i:
                    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    a.record()
                    pkg.uccl_chunk_apply(acc, out, recv, d2, n2, bitmap, w.dtype, ph2.op)
                    b.record()
                    evs.append((a, b))
                else:
                    pkg.uccl_chunk_apply(acc, out, recv, d2, n2, bitmap, w.dtype, ph2.op)
        torch.cuda.synchronize()
        t = np.array([a.elapsed_time(b) for a, b in evs])
        kernel_ms.append((float(t.mean()), float(np.median(t)), float(t.min())))

    if args.calibration_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dstc = torch.empty_like(src)
        torch.cuda.synchronize()
        dstc.copy_(src)
        torch.cuda.synchronize()
        del src, dstc

    payload = sum(ph.payload_bytes for ph in w.phases)
    unique = sum(ph.n_unique for ph in w.phases)
    arrivals = sum(counts)
    algo = sum(ph.algo_bytes for ph in w.phases)
    dom = int(np.argmax([ph.algo_bytes for ph in w.phases]))
    dom_ms = kernel_ms[dom][0]
    achieved = w.phases[dom].algo_bytes / (dom_ms * 1e-3) / 1e9

    result = {
        "metric": "reduced payload GB/s (dedup+place+reduce+forward of one rank's chunk stream), 1x MI355X",
        "value": round(payload / elapsed * args.steps / 1e9, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if w.dtype == 1 else "f32",
        "data": "synthetic",
        "config": {"workload": f"{args.workload}: {desc_text}", "seed": args.seed,
                   "unique_chunks": unique, "arrivals": arrivals, "payload_bytes": payload,
                   "algorithmic_bytes": algo, "launch_shape": args.shape,
                   "calls_per_step": "dedup_reset + one uccl_chunk_apply per phase"},
        "chunks_per_s": round(unique / (elapsed / args.steps), 1),
        "arrivals_per_s": round(arrivals / (elapsed / args.steps), 1),
        "step_hbm_frac": round(algo / (elapsed / args.steps) / 1e9 / PEAK_HBM_GBS, 4),
        "roofline": {
            "bound": "hbm",
            "kernel": f"chunk_apply_kernel ({w.phases[dom].name} phase, {'SUM' if w.phases[dom].op == 0 else 'COPY'})",
            "achieved": round(achieved, 1),
            "peak": PEAK_HBM_GBS,
            "unit": "GB/s",
            "frac": round(achieved / PEAK_HBM_GBS, 4),
            "traffic": None,
            "algorithmic_bytes_per_launch": w.phases[dom].algo_bytes,
            "avg_launch_ms": round(dom_ms, 5),
        },
        "kernels": [
            {"phase": ph.name, "records": n, "algorithmic_bytes": ph.algo_bytes, "avg_ms": round(k[0], 5),
             "median_ms": round(k[1], 5), "min_ms": round(k[2], 5),
             "hbm_frac": round(ph.algo_bytes / (k[0] * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}
            for ph, n, k in zip(w.phases, counts, kernel_ms)
        ],
    }

    if not args.no_cpu_baseline:
        import oracle
        reps, cpu_t, exp = 0, 0.0, None
        while cpu_t < 10.0 and reps < 8:
            eacc = w.acc.copy()
            eout = np.zeros(max(w.out_bytes, 16), dtype=np.uint8)
            seen = oracle.new_seen(w.n_bits)
            t0 = time.perf_counter()
            for ph in w.phases:
                oracle.apply(eacc, eout, w.recv_stage, ph.descs, seen, w.dtype, ph.op, check=False)
            cpu_t += time.perf_counter() - t0
            reps += 1
            if exp is None:
                exp = (eacc, eout[:w.out_bytes], oracle.pack_bitmap(seen))
        result["cpu_baseline"] = {
            "value": round(payload * reps / cpu_t / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"the whole step (both phases, {arrivals} arrivals, {payload} payload bytes) x {reps} repetitions, {cpu_t:.1f} s",
        }
        same = all(np.array_equal(np.ascontiguousarray(g).view(np.uint8), np.ascontiguousarray(e).view(np.uint8))
                   for g, e in zip(first, exp))
        result["parity_first_pass"] = "bit-exact vs oracle (acc, out_stage, bitmap)" if same else "MISMATCH"
        if not same:
            print(json.dumps(result))
            sys.exit(1)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
