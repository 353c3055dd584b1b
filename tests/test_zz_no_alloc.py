"""The entry point for callers that cannot allocate (uccl_chunk_apply_noalloc), through the C ABI:
same result as uccl_chunk_apply, bit for bit, on two calls in a row of which the second is smaller
(the array of claim words keeps what the first call left), then replayed from a captured graph."""
import numpy as np
import pytest
import torch

import oracle
from synth import workloads as wl
from synth.layout import F32, BF16

from gpuhelp import DeviceRun, oracle_results, assert_same

pytestmark = pytest.mark.gpu


def run_with(pkg, w, entry):
    """All phases of workload `w` through `entry` (a binding function with uccl_chunk_apply's
    signature), results as numpy arrays."""
    run = DeviceRun(w)
    for ph, d in zip(w.phases, run.descs):
        entry(run.acc, run.out, run.recv, d, len(ph.descs), run.bitmap, w.dtype, ph.op)
    torch.cuda.synchronize()
    return run.results()[:3]


def test_no_alloc_entry_point_equals_the_allocating_one(gpu_lib):
    # 57 + 56 records of 64 KiB, then 21 + 20 records of 24 KiB + a ragged tail: both are cut into parts
    first = wl.config1(seed=11)
    second = wl.ring_share("smaller", 12, R=6, M=6 * (4 * 24576 + 1040), C=24576, dtype=BF16, paths=4, window=None,
                           dup=0.1, dist="normal")
    assert max(len(p.descs) for p in second.phases) < min(len(p.descs) for p in first.phases)
    for w in (first, second):          # two calls in a row, the second with the smaller input
        got = run_with(gpu_lib, w, gpu_lib.uccl_chunk_apply_noalloc)
        ref = run_with(gpu_lib, w, gpu_lib.uccl_chunk_apply)
        for g, r, what in zip(got, ref, ("acc", "out_stage", "bitmap")):
            assert_same(g, r, f"{w.name}: {what} vs uccl_chunk_apply")
        eacc, eout, ebm = oracle_results(w)
        assert_same(got[0], eacc, w.name + ": acc vs oracle")
        assert_same(got[1], eout, w.name + ": out_stage vs oracle")
        assert_same(got[2], ebm, w.name + ": bitmap vs oracle")
    assert gpu_lib.uccl_claim_timeouts() == 0


def test_no_alloc_entry_point_every_duplicate_once(gpu_lib):
    """All-ones payloads, every record several times, adjacent and far apart: every part of every copy
    learns the one decision taken for its record (2 = applied twice, 0 = lost)."""
    C, n = 40 << 10, 48
    arr = np.concatenate([np.repeat(np.arange(n), 2), np.arange(n)[::-1], np.arange(0, n, 3)])
    from synth.layout import DESC, SUM
    d = np.zeros(len(arr), dtype=DESC)
    d["src_off"] = np.arange(len(arr), dtype=np.uint64) * C
    d["dst_off"] = d["out_off"] = arr.astype(np.uint64) * C
    d["len"], d["seq"] = C, arr
    w = wl.Workload("ones", F32, np.zeros(n * C // 4, np.float32), np.ones(len(arr) * C // 4, np.float32), n * C, n,
                    [wl.Phase("p", SUM, d, n, n * C, 0)])
    for _ in range(2):
        acc, out, bm = run_with(gpu_lib, w, gpu_lib.uccl_chunk_apply_noalloc)
        assert np.all(acc == 1.0) and np.array_equal(out.view(np.float32), acc)
        assert sum(int(x).bit_count() for x in bm) == n
    assert gpu_lib.uccl_claim_timeouts() == 0


def test_no_alloc_entry_point_in_a_replayed_graph(gpu_lib):
    """What the entry point is for: captured once, replayed with eager work in between; every
    replay equals the oracle (the claim words are cleared by a fill kernel inside the graph)."""
    w = wl.config1(seed=13)
    eacc, eout, ebm = oracle_results(w)
    gpu_lib.uccl_init()                   # the array's address is looked up before the capture
    run = DeviceRun(w)
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(g, stream=side):
        gpu_lib.uccl_dedup_reset(run.bitmap, w.n_bits)
        for ph, d in zip(w.phases, run.descs):
            gpu_lib.uccl_chunk_apply_noalloc(run.acc, run.out, run.recv, d, len(ph.descs), run.bitmap, w.dtype, ph.op)
    acc0 = run.acc.clone()
    other = torch.zeros(1 << 16, device="cuda")
    for rep in range(4):
        run.acc.copy_(acc0)
        g.replay()
        torch.cuda.synchronize()
        other.add_(1.0).sum().item()      # the program's own eager work between replays
        acc, out, bm, _ = run.results()
        assert_same(bm, ebm, f"bitmap, replay {rep}")
        assert_same(acc, eacc, f"acc, replay {rep}")
        assert_same(out, eout, f"out_stage, replay {rep}")
    assert gpu_lib.uccl_claim_timeouts() == 0


def test_no_alloc_entry_point_rejects_what_it_has_no_room_for(gpu_lib):
    w = wl.config2(seed=3, M=4 << 20)
    run = DeviceRun(w)
    n = gpu_lib.UCCL_NOALLOC_MAX_DESCS + 1
    with pytest.raises(gpu_lib.UcclError) as e:
        gpu_lib.uccl_chunk_apply_noalloc(run.acc, run.out, run.recv, run.descs[0], n, run.bitmap, w.dtype, 0)
    assert e.value.code == gpu_lib.UCCL_ETOOBIG and "too many records" in str(e.value)
    torch.cuda.synchronize()
    acc, out, bm, _ = run.results()
    assert_same(acc, w.acc, "acc untouched") and not bm.any()
