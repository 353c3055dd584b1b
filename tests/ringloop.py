"""Closed-loop ring driver: all R ranks of a ring allreduce stepped together, with
every hop's data cut into chunks, sprayed, reordered and duplicated by the arrival
model.  What rank r-1 wrote to its outbound staging buffer in one step is what rank
r receives in the next.  The driver only moves bytes and builds records; the
per-arrival work is done by the backend under test (the CPU oracle, or the GPU
library), passed in as an object with:

    make_rank(acc_init, out_bytes, n_bits) -> handle
    apply(handle, recv_np, descs_np, dtype, op) -> None
    read_out(handle, off, nbytes) -> np.uint8 array
    read_acc(handle) -> np array (same storage dtype as acc_init)
    segment(handle, off, nbytes, C) -> list of np.uint8 arrays   (optional: the very first step's
        hand-off, the rank's own segment cut into chunks by the backend's sender-side path; without
        it the driver slices the input on the host)
"""
import numpy as np

from synth.arrivals import gen_arrivals
from synth.layout import COPY, ELEM_SIZE, FORWARD_ONLY
from synth.workloads import ring_logical, materialize


def closed_loop_allreduce(backend, x, dtype, C, seed, paths=4, window=None, dup=0.1, op=0, relay=False):
    R, n = x.shape
    es = ELEM_SIZE[dtype]
    M = n * es
    S = M // R
    cps = -(-S // C)
    xb = np.ascontiguousarray(x).view(np.uint8).reshape(R, M)
    plans, ranks = [], []
    for r in range(R):
        rs, ag, n_out = ring_logical(R, M, C, rank=r, relay=relay)
        plans.append((rs, ag))
        ranks.append(backend.make_rank(x[r].copy(), n_out * C, len(rs) + len(ag)))
    prev = [None] * R  # LOGICAL records of what each rank produced in the previous step
    for phase in (0, 1):
        for s in range(R - 1):
            staged = []
            first_hop = phase == 0 and s == 0 and hasattr(backend, "segment")
            sent = [backend.segment(ranks[q], q * S, S, C) for q in range(R)] if first_hop else None
            for r in range(R):
                left = (r - 1) % R
                mine = plans[r][phase][s * cps:(s + 1) * cps]
                # bytes the left neighbour sends: its own raw segment in the very first
                # step, afterwards what its previous step wrote to its staging buffer
                chunks = []
                for c in range(cps):
                    ln = int(mine[c]["len"])
                    if first_hop:
                        assert len(sent[left]) == cps and len(sent[left][c]) == ln
                        chunks.append(sent[left][c])
                    elif phase == 0 and s == 0:
                        o = left * S + c * C
                        chunks.append(xb[left, o:o + ln])
                    else:
                        off = int(prev[left][c]["out_off"]) & ~int(FORWARD_ONLY)  # flag bit is not an address bit
                        chunks.append(backend.read_out(ranks[left], off, ln))
                arr = gen_arrivals(seed, cps, paths, window, dup, stream=(phase * R + s) * R + r)[0]
                recv = np.zeros(len(arr) * C, dtype=np.uint8)
                for k, i in enumerate(arr):
                    recv[k * C:k * C + len(chunks[i])] = chunks[i]
                staged.append((recv, materialize(mine, arr, 0, C), mine))
            for r in range(R):
                recv, descs, mine = staged[r]
                backend.apply(ranks[r], recv, descs, dtype, op if phase == 0 else COPY)
                prev[r] = mine
    return np.stack([backend.read_acc(h) for h in ranks])
