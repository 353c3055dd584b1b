"""Python face of the CPU oracle (chunk_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
package; the GPU library and its binding never do.  The arithmetic is all in the C
file; this module compiles it with gcc and marshals numpy arrays.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_DIR, "chunk_oracle.c")
_SRC_THREADED = os.path.join(_DIR, "chunk_threaded.c")
_LIB = os.path.join(_DIR, "libchunk_oracle.so")

# strict IEEE: no fast-math, no FMA contraction, SSE2 scalar arithmetic
CFLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-fno-fast-math", "-ffp-contract=off",
          "-Wall", "-Wextra"]

F32, BF16, F16, I32 = 0, 1, 2, 3
SUM, MAX, MIN, COPY, PROD = 0, 1, 2, 3, 4
NO_FORWARD = 0xFFFFFFFFFFFFFFFF
FORWARD_ONLY = 0x8000000000000000
ERRORS = {-1: "ARG", -2: "SEQ", -3: "ALIGN", -4: "BOUNDS", -5: "MISMATCH", -6: "OVERLAP"}

DESC = np.dtype([("src_off", "<u8"), ("dst_off", "<u8"), ("out_off", "<u8"),
                 ("len", "<u4"), ("seq", "<u4")])
SEND_DESC = np.dtype([("stage_off", "<u8"), ("len", "<u4"), ("header", "<u4")])
GATHER_DESC = np.dtype([("dst_off", "<u8"), ("out_off", "<u8"), ("len", "<u4"), ("seq", "<u4"),
                        ("n_src", "<u4"), ("reserved", "<u4"), ("src_off", "<u8", (16,))])


class OraclePrecondition(ValueError):
    def __init__(self, code):
        super().__init__(f"oracle precondition violated: {ERRORS.get(code, code)}")
        self.code = code


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (always when force, else when stale).  CHUNK_ORACLE_LIB in the
    environment names another, already built library to load instead: the mutation test uses it to
    run the pins against copies of the oracle with a mistake planted."""
    if os.environ.get("CHUNK_ORACLE_LIB"):
        return os.environ["CHUNK_ORACLE_LIB"]
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < max(
        os.path.getmtime(_SRC), os.path.getmtime(_SRC_THREADED), os.path.getmtime(os.path.join(_DIR, "chunk_oracle.h")))
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", *CFLAGS, "-pthread", _SRC, _SRC_THREADED, "-o", tmp])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        vp, u64, i64 = C.c_void_p, C.c_uint64, C.c_int64
        L.orc_apply.restype = i64
        L.orc_apply.argtypes = [vp, u64, vp, u64, vp, u64, vp, u64, vp, u64, C.c_int, C.c_int]
        L.orc_apply_threaded.restype = i64
        L.orc_apply_threaded.argtypes = [vp, u64, vp, u64, vp, u64, vp, u64, vp, u64, C.c_int, C.c_int, C.c_int]
        L.orc_reduce_gather.restype = i64
        L.orc_reduce_gather.argtypes = [vp, u64, vp, u64, vp, u64, vp, u64, vp, u64, C.c_int, C.c_int]
        L.orc_scatter.restype = i64
        L.orc_scatter.argtypes = [vp, u64, vp, u64, vp, u64, vp, u64]
        L.orc_check_call.restype = i64
        L.orc_check_call.argtypes = [vp, u64, vp, u64]
        L.orc_pack_bitmap.restype = None
        L.orc_pack_bitmap.argtypes = [vp, u64, vp]
        L.orc_message_status.restype = None
        L.orc_message_status.argtypes = [vp, vp, C.c_uint32, C.c_uint32, vp, C.c_int]
        L.orc_ack_report.restype = None
        L.orc_ack_report.argtypes = [vp, u64, vp, vp, vp, vp, C.c_uint32]
        L.orc_segment.restype = i64
        L.orc_segment.argtypes = [vp, u64, vp, u64, u64, u64, C.c_uint32, u64, u64, vp, C.c_uint32, C.c_uint32,
                                  C.c_uint32]
        L.orc_ring_allreduce.restype = C.c_int
        L.orc_ring_allreduce.argtypes = [vp, C.c_uint32, u64, C.c_int, C.c_int, vp]
        L.orc_combine_f32.restype = C.c_float
        L.orc_combine_f32.argtypes = [C.c_float, C.c_float, C.c_int]
        L.orc_combine_bf16.restype = C.c_uint16
        L.orc_combine_bf16.argtypes = [C.c_uint16, C.c_uint16, C.c_int]
        L.orc_f32_to_bf16.restype = C.c_uint16
        L.orc_f32_to_bf16.argtypes = [C.c_float]
        L.orc_combine_f16.restype = C.c_uint16
        L.orc_combine_f16.argtypes = [C.c_uint16, C.c_uint16, C.c_int]
        L.orc_combine_i32.restype = C.c_int32
        L.orc_combine_i32.argtypes = [C.c_int32, C.c_int32, C.c_int]
        L.orc_f32_to_f16.restype = C.c_uint16
        L.orc_f32_to_f16.argtypes = [C.c_float]
        L.orc_f16_to_f32.restype = C.c_float
        L.orc_f16_to_f32.argtypes = [C.c_uint16]
        _lib = L
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data


def _descs(descs):
    d = np.ascontiguousarray(descs)
    assert d.dtype.itemsize == 32 and d.dtype.names == DESC.names, "descriptor layout"
    return d


def new_seen(n_bits: int) -> np.ndarray:
    return np.zeros(int(n_bits), dtype=np.uint8)


def apply(acc, out_stage, recv_stage, descs, seen, dtype, op, check=True) -> int:
    """In-place oracle_apply on numpy buffers; returns the number of records applied."""
    d = _descs(descs)
    for a in (acc, recv_stage, seen) + ((out_stage,) if out_stage is not None else ()):
        assert a.flags.c_contiguous
    if check:
        rc = lib().orc_check_call(_ptr(recv_stage), recv_stage.nbytes, _ptr(d), len(d))
        if rc < 0:
            raise OraclePrecondition(rc)
    rc = lib().orc_apply(_ptr(acc), acc.nbytes, _ptr(out_stage),
                         0 if out_stage is None else out_stage.nbytes, _ptr(recv_stage),
                         recv_stage.nbytes, _ptr(d), len(d), _ptr(seen), len(seen),
                         int(dtype), int(op))
    if rc < 0:
        raise OraclePrecondition(rc)
    return int(rc)


def apply_threaded(acc, out_stage, recv_stage, descs, seen, dtype, op, threads) -> int:
    """oracle.apply on `threads` cores (the benchmark's multi-core CPU baseline); same result."""
    d = _descs(descs)
    rc = lib().orc_apply_threaded(_ptr(acc), acc.nbytes, _ptr(out_stage),
                                  0 if out_stage is None else out_stage.nbytes, _ptr(recv_stage),
                                  recv_stage.nbytes, _ptr(d), len(d), _ptr(seen), len(seen),
                                  int(dtype), int(op), int(threads))
    if rc < 0:
        raise OraclePrecondition(rc)
    return rc


def reduce_gather(acc, out_stage, recv_stage, descs, seen, dtype, op) -> int:
    d = np.ascontiguousarray(descs)
    assert d.dtype.itemsize == 160 and d.dtype.names == GATHER_DESC.names, "gather record layout"
    rc = lib().orc_reduce_gather(_ptr(acc), acc.nbytes, _ptr(out_stage),
                                 0 if out_stage is None else out_stage.nbytes, _ptr(recv_stage),
                                 recv_stage.nbytes, _ptr(d), len(d), _ptr(seen), len(seen), int(dtype), int(op))
    if rc < 0:
        raise OraclePrecondition(rc)
    return int(rc)


def scatter(dst, recv_stage, descs, seen, check=True) -> int:
    d = _descs(descs)
    assert dst.flags.c_contiguous and recv_stage.flags.c_contiguous
    if check:
        rc = lib().orc_check_call(_ptr(recv_stage), recv_stage.nbytes, _ptr(d), len(d))
        if rc < 0:
            raise OraclePrecondition(rc)
    rc = lib().orc_scatter(_ptr(dst), dst.nbytes, _ptr(recv_stage), recv_stage.nbytes,
                           _ptr(d), len(d), _ptr(seen), len(seen))
    if rc < 0:
        raise OraclePrecondition(rc)
    return int(rc)


def pack_bitmap(seen) -> np.ndarray:
    words = np.zeros((len(seen) + 31) // 32, dtype=np.uint32)
    lib().orc_pack_bitmap(_ptr(seen), len(seen), _ptr(words))
    return words


def ack_report(words, n_bits, max_ranges):
    """Returns (cum_ack, n_applied, n_ranges, ranges[min(n_ranges, max_ranges)][2])."""
    words = np.ascontiguousarray(words, dtype=np.uint32)
    assert len(words) * 32 >= n_bits
    ca, na = C.c_uint64(0), C.c_uint64(0)
    nr = C.c_uint32(0)
    ranges = np.zeros((max(max_ranges, 1), 2), dtype=np.uint64)
    lib().orc_ack_report(_ptr(words), int(n_bits), C.addressof(ca), C.addressof(na), C.addressof(nr),
                         _ptr(ranges), int(max_ranges))
    return ca.value, na.value, nr.value, ranges[:min(nr.value, max_ranges)]


def message_status(words, n_chunks, bits_per_slot, recycle=False):
    """Per-slot (cum_ack, n_applied, complete, 0) rows; `words` is updated in place when recycling."""
    assert words.dtype == np.uint32 and words.flags.c_contiguous
    n_chunks = np.ascontiguousarray(n_chunks, dtype=np.uint32)
    assert bits_per_slot % 32 == 0 and len(words) * 32 >= len(n_chunks) * bits_per_slot
    out = np.zeros((len(n_chunks), 4), dtype=np.uint32)
    lib().orc_message_status(_ptr(words), _ptr(n_chunks), len(n_chunks), int(bits_per_slot), _ptr(out),
                             int(bool(recycle)))
    return out


def segment(stage, tensor, tensor_off, nbytes, chunk_bytes, stage_off=0, slot_stride=None, conn_id=0, msg_id=0,
            first_csn=0, want_descs=True):
    """Cut tensor[tensor_off, +nbytes) into staged chunks (in place in ``stage``, a uint8 array);
    returns the send records (SEND_DESC array, or None)."""
    assert stage.flags.c_contiguous and tensor.flags.c_contiguous
    slot_stride = chunk_bytes if slot_stride is None else slot_stride
    n = -(-int(nbytes) // int(chunk_bytes)) if chunk_bytes else 0
    descs = np.zeros(n, dtype=SEND_DESC) if want_descs else None
    rc = lib().orc_segment(_ptr(stage), stage.nbytes, _ptr(tensor), tensor.nbytes, int(tensor_off), int(nbytes),
                           int(chunk_bytes), int(stage_off), int(slot_stride), _ptr(descs), int(conn_id), int(msg_id),
                           int(first_csn))
    if rc < 0:
        raise OraclePrecondition(rc)
    assert rc == n
    return descs


def ring_allreduce(x, dtype, op=SUM) -> np.ndarray:
    """x: (R, n) array (fp32, or uint16 bf16 bits).  Returns every rank's final buffer."""
    x = np.ascontiguousarray(x)
    R, n = x.shape
    out = np.empty_like(x)
    rc = lib().orc_ring_allreduce(_ptr(x), R, n, int(dtype), int(op), _ptr(out))
    if rc:
        raise OraclePrecondition(rc)
    return out


def combine_f32(a, r, op) -> np.float32:
    return np.float32(lib().orc_combine_f32(np.float32(a), np.float32(r), int(op)))


def combine_bf16(a, r, op) -> int:
    return int(lib().orc_combine_bf16(int(a), int(r), int(op)))


def f32_to_bf16(f) -> int:
    return int(lib().orc_f32_to_bf16(np.float32(f)))


def combine_f16(a, r, op) -> int:
    return int(lib().orc_combine_f16(int(a), int(r), int(op)))


def combine_i32(a, r, op) -> int:
    return int(lib().orc_combine_i32(int(a), int(r), int(op)))


def f32_to_f16(f) -> int:
    return int(lib().orc_f32_to_f16(np.float32(f)))


def f16_to_f32(h) -> np.float32:
    return np.float32(lib().orc_f16_to_f32(int(h)))
