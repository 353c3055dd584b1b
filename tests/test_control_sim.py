"""The control-path model as a source of arrival orders (host only), and the data path's
results on such streams (oracle here; the GPU run is in test_gpu_parity.py)."""
import numpy as np
import pytest

import oracle
from synth import workloads as wl
from synth.control_sim import ControlPath, ReceiverCredit, SwiftWindow, simulated_arrivals
from synth.layout import BF16, SUM


def test_lossless_quiet_network_has_no_duplicates_and_little_reordering():
    seq, copy, path, cp = simulated_arrivals(1, 600, paths=1, jitter_us=0.0, loss=0.0, rto_us=1e9,
                                             dup_ack_threshold=10 ** 6)
    assert np.array_equal(seq, np.arange(600)) and not copy.any()
    assert cp.stats["retransmitted"] == 0 and cp.stats["duplicates"] == 0


@pytest.mark.parametrize("loss", [0.0, 1 / 256, 1 / 16])
def test_every_chunk_is_delivered_and_duplicates_come_from_retransmission(loss):
    n = 2000
    seq, copy, path, cp = simulated_arrivals(3, n, paths=32, loss=loss, jitter_us=10.0)
    assert np.array_equal(np.unique(seq), np.arange(n))
    assert len(seq) == cp.stats["sent"] - cp.stats["lost"]
    assert cp.stats["sent"] == n + cp.stats["retransmitted"]
    assert cp.stats["duplicates"] == len(seq) - n
    # every copy index that arrived was sent: copy k > 0 only exists if a retransmission happened
    assert copy.max() <= cp.stats["retransmitted"]
    if loss > 0:
        assert cp.stats["lost"] > 0 and cp.stats["retransmitted"] >= cp.stats["lost"]
    # multipath reorders
    assert np.count_nonzero(np.diff(seq) < 0) > n // 20
    # same seed, same run
    seq2 = simulated_arrivals(3, n, paths=32, loss=loss, jitter_us=10.0)[0]
    assert np.array_equal(seq, seq2)


def test_window_bounds_data_in_flight():
    class Watch(ControlPath):
        peak = 0

        def onPacingChunk(self, now):
            Watch.peak = max(Watch.peak, len(self.inflight))
            return super().onPacingChunk(now)

    cp = Watch(5, 1500, paths=16, max_cwnd=64, init_cwnd=64)
    seq = cp.run()[0]
    assert Watch.peak <= 64
    first = np.full(1500, -1)
    for k, s in enumerate(seq):
        if first[s] < 0:
            first[s] = k
    # nothing arrives more than (window + retransmissions) positions ahead of the lowest missing seq
    base = 0
    seen = np.zeros(1500, bool)
    for s in seq:
        assert s < base + 64 + cp.stats["retransmitted"] + 1
        seen[s] = True
        while base < 1500 and seen[base]:
            base += 1


def test_power_of_two_prefers_faster_paths():
    class Count(ControlPath):
        def onSelectPath(self, seq):
            p = super().onSelectPath(seq)
            self.picks[p] += 1
            return p

    cp = Count(7, 4000, paths=8, base_delay_us=(5.0, 60.0), jitter_us=1.0)
    cp.picks = np.zeros(8, int)
    cp.run()
    order = np.argsort(cp.delay)
    assert cp.picks[order[:4]].sum() > 1.5 * cp.picks[order[4:]].sum()


def test_hooks_are_called():
    calls = {}

    class Spy(ControlPath):
        pass

    for name in ("onChunkSize", "onPacingChunk", "onSelectPath", "onTxRtxChunk", "onRxChunk", "onRxRtxChunk",
                 "onRxACK", "onRxCredit"):
        assert callable(getattr(ControlPath, name)), name

    def wrap(name):
        orig = getattr(ControlPath, name)

        def f(self, *a):
            calls[name] = calls.get(name, 0) + 1
            return orig(self, *a)
        return f

    for name in ("onPacingChunk", "onSelectPath", "onTxRtxChunk", "onRxChunk", "onRxRtxChunk", "onRxACK"):
        setattr(Spy, name, wrap(name))
    Spy(9, 800, paths=16, loss=0.02, jitter_us=12.0, rto_us=60.0).run()
    assert all(calls.get(k, 0) > 0 for k in ("onPacingChunk", "onSelectPath", "onTxRtxChunk", "onRxChunk",
                                              "onRxRtxChunk", "onRxACK")), calls


@pytest.mark.parametrize("scheme", ["swift", "credit"])
@pytest.mark.parametrize("loss", [0.0, 1 / 64])
def test_schemes_written_against_the_extension_points(scheme, loss):
    """A delay-based window and a receiver-credit scheme (Section 4), each a subclass that only
    overrides extension points: every chunk is delivered, the books balance, and each scheme
    shows its own signature."""
    n = 3000
    seq, copy, path, cp = simulated_arrivals(5, n, scheme=scheme, paths=32, loss=loss, jitter_us=8.0)
    assert np.array_equal(np.unique(seq), np.arange(n))
    assert len(seq) == cp.stats["sent"] - cp.stats["lost"]
    assert cp.stats["sent"] == n + cp.stats["retransmitted"]
    assert cp.stats["duplicates"] == len(seq) - n
    if scheme == "credit":
        assert isinstance(cp, ReceiverCredit)
        assert cp.credits_seen == len(seq), "one credit per arrival came back to the sender"
        assert cp.credit >= 0
    else:
        assert isinstance(cp, SwiftWindow)
        # the delay target keeps the window, and with it the queueing delay, below the loss-based scheme's
        base = simulated_arrivals(5, n, scheme="window", paths=32, loss=loss, jitter_us=8.0)[3]
        assert cp.stats["retransmitted"] <= base.stats["retransmitted"]


@pytest.mark.parametrize("scheme", ["window", "swift", "credit"])
def test_data_path_result_does_not_depend_on_the_transport(scheme):
    """The same logical stream delivered by the random-spray model and by the control-path
    model (with loss and retransmission, under each scheme) gives byte-identical results."""
    kw = dict(R=4, M=4 * 40 * 512, C=512, dtype=BF16, paths=16, window=32, dup=0.05, dist="normal")
    base = wl.ring_share("spray", 11, **kw)
    arr = [simulated_arrivals(11, len(lg), scheme=scheme, paths=16, loss=0.03, jitter_us=15.0, rto_us=80.0, stream=i)[0]
           for i, lg in enumerate(base.extra["logical"])]
    sim = wl.ring_share("sim", 11, arrivals=arr, **kw)
    assert any(len(a) > len(lg) for a, lg in zip(arr, base.extra["logical"])), "the model must produce duplicates"

    def run(w):
        acc, out, seen = w.acc.copy(), np.zeros(w.out_bytes, np.uint8), oracle.new_seen(w.n_bits)
        for ph in w.phases:
            oracle.apply(acc, out, w.recv_stage, ph.descs, seen, w.dtype, ph.op)
        return acc, out, oracle.pack_bitmap(seen)

    for a, b in zip(run(base), run(sim)):
        assert np.array_equal(a, b)
