"""The 32-bit control header that travels with every chunk (Section 3.1 of the paper:
connection id 8 bits, message id 7 bits, chunk sequence number 8 bits, a last-chunk mark,
8 bits kept for receiver-driven congestion control), and the rule that turns it into a bit
index of the receiver's dedup bitmap.  Only bit packing lives here; payload is never touched.

The paper fixes the field WIDTHS, not their positions; the positions below are this module's
choice (low bits first: chunk sequence number, last mark, message id, connection id, spare).
"""
import numpy as np

CSN_BITS, LAST_BITS, MSG_BITS, CONN_BITS, SPARE_BITS = 8, 1, 7, 8, 8
assert CSN_BITS + LAST_BITS + MSG_BITS + CONN_BITS + SPARE_BITS == 32

MESSAGES_IN_FLIGHT = 1 << MSG_BITS   # 128 message slots per connection
CHUNKS_PER_MESSAGE = 1 << CSN_BITS   # 256 chunks per message

_CSN, _LAST, _MSG, _CONN, _SPARE = 0, 8, 9, 16, 24


def pack(conn, msg, csn, last, spare=0):
    """Field arrays (or scalars) -> uint32 headers."""
    conn, msg, csn, last, spare = (np.asarray(x, dtype=np.uint32) for x in (conn, msg, csn, last, spare))
    assert np.all(conn < (1 << CONN_BITS)) and np.all(msg < MESSAGES_IN_FLIGHT)
    assert np.all(csn < CHUNKS_PER_MESSAGE) and np.all(last < 2) and np.all(spare < (1 << SPARE_BITS))
    return (csn << np.uint32(_CSN)) | (last << np.uint32(_LAST)) | (msg << np.uint32(_MSG)) | \
           (conn << np.uint32(_CONN)) | (spare << np.uint32(_SPARE))


def unpack(hdr):
    """uint32 headers -> dict of field arrays."""
    h = np.asarray(hdr, dtype=np.uint32)
    f = lambda at, bits: (h >> np.uint32(at)) & np.uint32((1 << bits) - 1)
    return dict(conn=f(_CONN, CONN_BITS), msg=f(_MSG, MSG_BITS), csn=f(_CSN, CSN_BITS),
                last=f(_LAST, LAST_BITS), spare=f(_SPARE, SPARE_BITS))


def seq_of(hdr):
    """Bit index in one connection's dedup bitmap: message slot * 256 + chunk sequence number
    (a bitmap of 128 * 256 bits = 4 KiB per connection)."""
    f = unpack(hdr)
    return f["msg"] * np.uint32(CHUNKS_PER_MESSAGE) + f["csn"]


def chunk_counts(hdr, n_slots=MESSAGES_IN_FLIGHT):
    """What the receiver knows about message lengths from the headers that have arrived: for
    each slot, csn + 1 of a header carrying the last-chunk mark, 0 if none has arrived."""
    f = unpack(hdr)
    out = np.zeros(n_slots, dtype=np.uint32)
    sel = f["last"] == 1
    out[f["msg"][sel]] = f["csn"][sel] + np.uint32(1)
    return out
