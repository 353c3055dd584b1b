"""A small discrete-event model of the paper's host control path, used as a source of
arrival orders with realistic reordering and duplication statistics.

What is modelled (all on the CPU side of the paper; none of it is the GPU data path):
  * multipath over P paths with per-path delay, a FIFO bottleneck queue and chunk loss
    (Section 3.2: 256 paths per connection; Section 6 loss experiment: losing any packet
    loses the whole chunk);
  * path selection by power-of-two choices on the smoothed per-path RTT (Section 4.1);
  * a congestion window in chunks with additive increase and a multiplicative decrease on
    loss (a stand-in for the window-based schemes of Section 4; the maximum window of
    Section 5 bounds the data in flight);
  * TCP-like cumulative + selective acknowledgements, fast retransmission after a raised
    duplicate-ACK threshold, timeout retransmission (Sections 3.2 and 4.3).
A retransmission of a chunk that was only delayed reaches the receiver as a DUPLICATE;
that, and the interleaving of paths, is what the GPU path has to absorb.

The eight extension points the paper lists (Appendix A) appear as overridable methods with
the paper's names; SwiftWindow (delay-based window) and ReceiverCredit (credits granted by the
receiver, in the manner of EQDS) are two extensions written against them, as the paper's own
case studies are.  Only integer / float bookkeeping of the transport lives here; payload
bytes are never touched.
"""
import heapq

import numpy as np

from .payload import rng


class ControlPath:
    """One sender/receiver pair moving chunks 0..n-1 of one phase."""

    def __init__(self, seed, n, paths=32, chunk_us=0.66, base_delay_us=(8.0, 14.0), jitter_us=6.0,
                 loss=0.0, max_cwnd=256, init_cwnd=32, dup_ack_threshold=16, rto_us=120.0, stream=0):
        assert 0.0 <= loss < 0.9, "a path that loses (almost) everything never completes"
        self.g = rng(seed, 0xC7A10000 + stream)
        self.n, self.P = int(n), int(paths)
        self.chunk_us = chunk_us                      # serialisation time of one chunk on one path
        lo, hi = base_delay_us
        self.delay = lo + (hi - lo) * self.g.random(self.P)   # one-way propagation per path
        self.jitter_us, self.loss = jitter_us, loss
        self.max_cwnd, self.cwnd = max_cwnd, float(init_cwnd)
        self.dupthresh, self.rto = dup_ack_threshold, rto_us
        self.srtt = np.full(self.P, 2 * (lo + hi) / 2)        # smoothed RTT estimate per path
        self.busy_until = np.zeros(self.P)                    # FIFO bottleneck per path
        self.stats = dict(sent=0, retransmitted=0, lost=0, duplicates=0, fast=0, timeout=0)

    # ---- the paper's extension points (Appendix A) --------------------------------------
    def onChunkSize(self, seq):            # all chunks of a phase have the configured size here
        return 1

    def onPacingChunk(self, now):          # window check: may another chunk leave now?
        return len(self.inflight) < min(int(self.cwnd), self.max_cwnd)

    def onSelectPath(self, seq):           # power of two choices on the smoothed RTT
        a, b = self.g.integers(0, self.P, 2)
        return int(a if self.srtt[a] <= self.srtt[b] else b)

    def onTxRtxChunk(self, seq, why):      # a retransmission leaves: shrink the window once per event
        self.stats["retransmitted"] += 1
        self.stats[why] += 1
        self.cwnd = max(2.0, self.cwnd * 0.7)

    def onRxChunk(self, seq, copy, path, now):     # receiver: first arrival of seq
        pass

    def onRxRtxChunk(self, seq, copy, path, now):  # receiver: seq had already arrived
        self.stats["duplicates"] += 1

    def onRxACK(self, path, rtt):          # sender: RTT sample, additive increase
        self.srtt[path] += 0.125 * (rtt - self.srtt[path])
        self.cwnd = min(self.max_cwnd, self.cwnd + 1.0 / max(self.cwnd, 1.0))

    def onRxCredit(self, credit):          # sender: a credit from the receiver arrived
        pass

    def creditFor(self, seq, now):         # receiver side of a receiver-driven scheme: credit granted per arrival
        return 0

    # ---- the event loop --------------------------------------------------------------------
    def _send(self, now, seq, copy):
        p = self.onSelectPath(seq)
        self.stats["sent"] += 1
        start = max(now, self.busy_until[p])
        self.busy_until[p] = start + self.chunk_us
        self.inflight[seq] = now
        self.sent_copy[seq] = copy
        if self.g.random() < self.loss:
            self.stats["lost"] += 1
        else:
            arrive = start + self.chunk_us + self.delay[p] + self.jitter_us * self.g.exponential()
            heapq.heappush(self.events, (arrive, self.tick(), "rx", seq, copy, p, now, None))
        heapq.heappush(self.events, (now + self.rto, self.tick(), "rto", seq, copy, p, now, None))

    def tick(self):
        self._tick += 1
        return self._tick

    def run(self):
        """Returns (seq, copy, path, time) arrays in arrival order at the receiver."""
        self.events, self._tick = [], 0
        self.inflight, self.sent_copy = {}, {}
        received = np.zeros(self.n, dtype=bool)
        acked = np.zeros(self.n, dtype=bool)       # sender's view (cumulative + selective)
        last_fast = np.full(self.n, -1e18)
        next_new, now = 0, 0.0
        arrivals = []

        def pump(now):
            nonlocal next_new
            while next_new < self.n and self.onPacingChunk(now):
                self._send(now, next_new, 0)
                next_new += 1

        pump(0.0)
        while self.events:
            now, _, kind, seq, copy, p, sent_at, picture = heapq.heappop(self.events)
            if kind == "rx":
                arrivals.append((seq, copy, p, now))
                if received[seq]:
                    self.onRxRtxChunk(seq, copy, p, now)
                else:
                    received[seq] = True
                    self.onRxChunk(seq, copy, p, now)
                # the ACK carries the receiver's picture at this moment (cumulative + selective ranges)
                heapq.heappush(self.events, (now + self.delay[p], self.tick(), "ack", seq, copy, p, sent_at,
                                             received.copy()))
                grant = self.creditFor(seq, now)
                if grant:
                    heapq.heappush(self.events, (now + self.delay[p], self.tick(), "credit", grant, 0, p, now, None))
            elif kind == "ack":
                self.onRxACK(p, now - sent_at)
                acked |= picture
                for s in [s for s in self.inflight if acked[s]]:
                    del self.inflight[s]
                # fast retransmission: a hole with at least dupthresh acknowledged chunks above it
                holes = np.flatnonzero(~acked[:next_new])
                if len(holes):
                    above = np.cumsum(acked[:next_new][::-1])[::-1]
                    for h in holes[:8]:
                        if above[h] >= self.dupthresh and now - last_fast[h] > self.srtt.mean():
                            last_fast[h] = now
                            self.onTxRtxChunk(h, "fast")
                            self._send(now, int(h), self.sent_copy.get(int(h), 0) + 1)
                pump(now)
            elif kind == "credit":
                self.onRxCredit(seq)               # the amount travels in the seq field of the event
                pump(now)
            elif kind == "rto":
                if not acked[seq] and self.sent_copy.get(seq) == copy:
                    self.onTxRtxChunk(seq, "timeout")
                    self._send(now, seq, copy + 1)
        assert received.all(), "the transport must deliver every chunk eventually"
        a = np.array(arrivals, dtype=np.float64).reshape(-1, 4)
        self.completion_us = float(a[:, 3].max()) if len(a) else 0.0
        return a[:, 0].astype(np.int64), a[:, 1].astype(np.int64), a[:, 2].astype(np.int64), a[:, 3]


class SwiftWindow(ControlPath):
    """Delay-based window in the manner of Swift (Section 4: one of the paper's two sender-driven
    schemes): grow additively while the measured RTT is under a target, shrink in proportion to
    the excess otherwise, at most once per RTT; a retransmission shrinks it like any other."""

    def __init__(self, *a, target_margin_us=12.0, beta=0.8, **kw):
        super().__init__(*a, **kw)
        self.target = float(np.min(self.srtt)) + target_margin_us
        self.beta, self.acks, self.cut_at = beta, 0, -10**9

    def onRxACK(self, path, rtt):
        self.srtt[path] += 0.125 * (rtt - self.srtt[path])
        self.acks += 1                     # the hook gets no clock: cuts are spaced by counting acknowledgements
        if rtt <= self.target:
            self.cwnd = min(self.max_cwnd, self.cwnd + 1.0 / max(self.cwnd, 1.0))
        elif self.acks - self.cut_at >= max(int(self.cwnd), 1):                        # about one RTT of acks
            self.cut_at = self.acks
            self.cwnd = max(2.0, self.cwnd * max(1.0 - self.beta * (rtt - self.target) / rtt, 0.5))


class ReceiverCredit(ControlPath):
    """Receiver-driven scheme in the manner of EQDS (Section 4.2, Appendix B): the sender may use
    an initial allowance without asking, after which every chunk leaves against a credit; the
    receiver grants one credit per arrival, so the sender is clocked at the pace the receiver
    drains.  Retransmissions go out without credit (the request-to-send exchange is not modelled)."""

    def __init__(self, *a, **kw):
        super().__init__(*a, **kw)
        self.credit = float(self.cwnd)     # the initial allowance
        self.credits_seen = 0

    def onPacingChunk(self, now):
        if self.credit >= 1.0 and len(self.inflight) < self.max_cwnd:
            self.credit -= 1.0
            return True
        return False

    def creditFor(self, seq, now):
        return 1

    def onRxCredit(self, credit):
        self.credit += credit
        self.credits_seen += credit

    def onRxACK(self, path, rtt):          # no window to adapt; keep the RTT estimate for path choice
        self.srtt[path] += 0.125 * (rtt - self.srtt[path])

    def onTxRtxChunk(self, seq, why):
        self.stats["retransmitted"] += 1
        self.stats[why] += 1


SCHEMES = {"window": ControlPath, "swift": SwiftWindow, "credit": ReceiverCredit}


def simulated_arrivals(seed, n, scheme="window", **kw):
    """Arrival order of chunks 0..n-1 under the control-path model; same return convention
    as synth.arrivals.gen_arrivals (seq, copy, path), plus the model for its statistics."""
    cp = SCHEMES[scheme](seed, n, **kw)
    seq, copy, path, _ = cp.run()
    return seq, copy, path, cp
