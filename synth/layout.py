"""Binary layout of the records that cross the library boundary.

The control path (simulated here) hands the GPU a list of per-arrival records,
the way the paper's receiver CPU hands packet pointers to the fused kernel
through host/device shared memory (Implementation section) in "the right order
given by the receiver CPU" (Section 3.1, reassembly challenge).  This module only
describes bytes; it performs none of the method's arithmetic.
"""
import numpy as np

#: one record per ARRIVAL (not per logical chunk), 32 bytes, little endian
DESC = np.dtype(
    [
        ("src_off", "<u8"),  # byte offset of this arrival's slot in recv_stage
        ("dst_off", "<u8"),  # byte offset in acc (apply) / dst (scatter)
        ("out_off", "<u8"),  # byte offset in out_stage, or NO_FORWARD
        ("len", "<u4"),      # payload bytes
        ("seq", "<u4"),      # bit index in the dedup bitmap = logical chunk id
    ]
)
assert DESC.itemsize == 32

#: one record per DESTINATION chunk with up to 16 source slots (multi-sender reduce), 160 bytes
MAX_SOURCES = 16
GATHER_DESC = np.dtype(
    [
        ("dst_off", "<u8"), ("out_off", "<u8"), ("len", "<u4"), ("seq", "<u4"),
        ("n_src", "<u4"), ("reserved", "<u4"), ("src_off", "<u8", (MAX_SOURCES,)),
    ]
)
assert GATHER_DESC.itemsize == 160

NO_FORWARD = np.uint64(0xFFFFFFFFFFFFFFFF)
FORWARD_ONLY = np.uint64(0x8000000000000000)  # flag in out_off: relay the result, do not write acc

# dtype / op codes shared by every caller (values are part of the C ABI)
F32, BF16, F16, I32 = 0, 1, 2, 3
SUM, MAX, MIN, COPY, PROD = 0, 1, 2, 3, 4

ELEM_SIZE = {F32: 4, BF16: 2, F16: 2, I32: 4}
OFFSET_ALIGN = 16  # every offset in a record is a multiple of this


def bitmap_words(n_bits: int) -> int:
    """Number of 32-bit words a dedup bitmap of n_bits needs."""
    return (int(n_bits) + 31) // 32
