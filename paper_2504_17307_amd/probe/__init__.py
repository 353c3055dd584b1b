"""Measurement aid, not part of the product: dense streaming kernels of the data path's traffic
shapes (stream_probe.hip, a library of its own) and the driver that times them over a workload's
own buffers.  bench.py reports the result as `stream_ceiling` beside the path's own figures."""
import ctypes
import os

import numpy as np

# name -> (mode id of the probe library, streams the shape touches)
PROBE_MODES = {"read_1r": (0, 1), "write_1w": (1, 1), "copy_1r1w": (2, 2), "reduce_forward_2r2w": (3, 4),
               "copy_forward_1r2w": (4, 3), "reduce_keep_2r1w": (5, 3)}


def back_to_back_s(torch, run, reps):
    """Seconds per launch of run(k), k = 0 .. reps-1 queued back to back (after four warm-up launches)."""
    for k in range(4):
        run(k)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for k in range(reps):
        run(k)
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) * 1e-3 / reps


def stream_ceilings(torch, sets, stream_bytes, block_bytes, gather_sources=0, reps=20, window_blocks=0):
    """What the memory system of this GPU delivers for the data path's traffic shapes with nothing
    in the way: dense kernels (no records, no dedup, no scatter; paper_2504_17307_amd/probe) over the
    workload's own buffers, `stream_bytes` per stream (the dominant call's payload), one
    `block_bytes` block per workgroup (the chunk), the same cache policies, rotating over the same
    buffer sets.  GB/s over all streams a shape touches."""
    from paper_2504_17307_amd.build import PROBE_LIB
    if not os.path.exists(PROBE_LIB):
        return {"error": f"{PROBE_LIB} is not built (python -m paper_2504_17307_amd.build)"}
    fn = ctypes.CDLL(PROBE_LIB).uccl_probe_stream
    fn.restype = ctypes.c_int
    fn.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32,
                   ctypes.c_uint32, ctypes.c_void_p, ctypes.c_void_p]
    modes = dict(PROBE_MODES)
    if gather_sources:   # the multi-sender reduce: its sources are consecutive regions of recv_stage, no staging copy
        modes = {f"gather_{gather_sources + 1}r1w": (6, gather_sources + 2), "read_1r": (0, 1)}
        nbytes = min([stream_bytes] + [min(s["recv"].numel() // gather_sources, s["acc"].numel()) for s in sets])
    elif min(s["out"].numel() for s in sets) < 2048:   # nothing is forwarded (all-to-all): slot -> destination only
        modes = {k: PROBE_MODES[k] for k in ("read_1r", "write_1w", "copy_1r1w")}
        nbytes = min([stream_bytes] + [min(s["recv"].numel(), s["acc"].numel()) for s in sets])
    else:
        nbytes = min([stream_bytes] + [min(s["recv"].numel(), s["acc"].numel(), s["out"].numel()) for s in sets])
    nbytes -= nbytes % 2048
    block = max(2048, block_bytes - block_bytes % 2048)
    if nbytes < 2048:
        return {"error": "buffers too small for the probe"}
    stream = torch.cuda.current_stream().cuda_stream
    out = {}
    for name, (mode, n_streams) in modes.items():
        def run(k):
            s = sets[k % len(sets)]
            stage = s["out"] if s["out"].numel() >= nbytes else s["acc"]   # no staging buffer: write the destination
            rc = fn(mode, s["recv"].data_ptr(), s["acc"].data_ptr(), stage.data_ptr(), nbytes, block,
                    gather_sources, None, stream)
            assert rc == 0, f"probe mode {name} refused"
        out[name + "_GBps"] = round(n_streams * nbytes / back_to_back_s(torch, run, reps) / 1e9, 1)
    if window_blocks > 1 and "reduce_forward_2r2w" in modes and nbytes >= 2 * block:
        # the same two forwarding shapes with destinations scattered the way arrivals are: block b of the
        # slot stream goes to a random block of the accumulator / staging streams within its reorder window
        scat = ctypes.CDLL(PROBE_LIB).uccl_probe_scattered
        scat.restype = ctypes.c_int
        scat.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32,
                         ctypes.c_void_p, ctypes.c_void_p]
        n_blocks = nbytes // block
        rng = np.random.default_rng(7)
        perm = np.arange(n_blocks, dtype=np.uint32)
        for lo in range(0, n_blocks, window_blocks):
            rng.shuffle(perm[lo:lo + window_blocks])
        perm_dev = torch.from_numpy(perm.view(np.int32)).cuda()
        for name, mode, n_streams in (("reduce_forward_2r2w_scattered", 3, 4), ("copy_forward_1r2w_scattered", 4, 3)):
            def run_scattered(k):
                s = sets[k % len(sets)]
                rc = scat(mode, s["recv"].data_ptr(), s["acc"].data_ptr(), s["out"].data_ptr(), n_blocks * block, block,
                          perm_dev.data_ptr(), stream)
                assert rc == 0, f"probe mode {name} refused"
            out[name + "_GBps"] = round(n_streams * n_blocks * block / back_to_back_s(torch, run_scattered, reps) / 1e9, 1)
    out["what"] = (f"dense kernels of the path's traffic shapes: {nbytes} bytes per stream, {block}-byte block per "
                   f"workgroup, the workload's own buffers rotating over {len(sets)} sets, same run"
                   + (f"; `_scattered`: destination blocks permuted within windows of {window_blocks} blocks" if window_blocks > 1 else ""))
    return out
