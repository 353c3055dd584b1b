"""Helpers for GPU tests: move a synthetic workload to the device, run it through the
C-ABI library (via the thin binding), and bring the results back as numpy arrays."""
import numpy as np
import torch

import paper_2504_17307_amd as pkg


def to_dev(a: np.ndarray) -> torch.Tensor:
    """Device copy of a numpy buffer as raw bytes (the library is typed by its dtype argument)."""
    return torch.from_numpy(np.ascontiguousarray(a).view(np.uint8).reshape(-1).copy()).cuda()


def to_host(t: torch.Tensor, like_dtype) -> np.ndarray:
    return t.cpu().numpy().view(like_dtype)


class DeviceRun:
    """Device-resident buffers of one workload."""

    def __init__(self, w, guard=0xA5, opts=None):
        self.w = w
        self.opts = opts  # None, or (chunk_bytes, parts): per-call tuning passed to the general entry point
        self.acc = to_dev(w.acc)
        self.recv = to_dev(w.recv_stage)
        self.out = torch.full((w.out_bytes,), guard, dtype=torch.uint8, device="cuda") if w.out_bytes else None
        self.bitmap = torch.zeros((w.n_bits + 31) // 32, dtype=torch.int32, device="cuda")
        self.rejected = torch.zeros(1, dtype=torch.int32, device="cuda")
        self.descs = [to_dev(ph.descs) for ph in w.phases]

    def reset(self):
        pkg.uccl_dedup_reset(self.bitmap, self.w.n_bits)

    def apply(self, descs_dev, n, op, checked=True, stream=None):
        if self.opts is not None:
            pkg.uccl_chunk_apply_opts(self.acc, self.out, self.recv, descs_dev, n, self.bitmap, self.w.dtype, op,
                                      n_rejected=self.rejected if checked else None,
                                      n_bits=self.w.n_bits if checked else None, opts=self.opts, stream=stream)
        elif checked:
            pkg.uccl_chunk_apply_checked(self.acc, self.out, self.recv, descs_dev, n, self.bitmap,
                                         self.w.dtype, op, n_rejected=self.rejected,
                                         n_bits=self.w.n_bits, stream=stream)
        else:
            pkg.uccl_chunk_apply(self.acc, self.out, self.recv, descs_dev, n, self.bitmap,
                                 self.w.dtype, op, stream=stream)

    def run_phases(self, checked=True, split=None):
        for ph, d in zip(self.w.phases, self.descs):
            n = len(ph.descs)
            cuts = [0, n] if split is None else [0] + sorted(split(n)) + [n]
            for lo, hi in zip(cuts[:-1], cuts[1:]):
                self.apply(d[lo * 32:], hi - lo, ph.op, checked)
        torch.cuda.synchronize()

    def results(self):
        acc = to_host(self.acc, self.w.acc.dtype)
        out = self.out.cpu().numpy() if self.out is not None else None
        bm = self.bitmap.cpu().numpy().view(np.uint32)
        return acc, out, bm, int(self.rejected.item())


def oracle_results(w, guard=0xA5):
    import oracle
    acc = w.acc.copy()
    out = np.full(w.out_bytes, guard, dtype=np.uint8) if w.out_bytes else None
    seen = oracle.new_seen(w.n_bits)
    for ph in w.phases:
        oracle.apply(acc, out, w.recv_stage, ph.descs, seen, w.dtype, ph.op)
    return acc, out, oracle.pack_bitmap(seen)


def assert_same(got, exp, what=""):
    """Bit-exact comparison with a useful message (first mismatch, count)."""
    g = np.ascontiguousarray(got).view(np.uint8).reshape(-1)
    e = np.ascontiguousarray(exp).view(np.uint8).reshape(-1)
    assert g.shape == e.shape, (what, g.shape, e.shape)
    if not np.array_equal(g, e):
        bad = np.flatnonzero(g != e)
        raise AssertionError(f"{what}: {len(bad)} bytes differ, first at byte {bad[0]}: "
                             f"got {g[bad[0]]:#x} expected {e[bad[0]]:#x}")
