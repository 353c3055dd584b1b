"""Thin ctypes binding of libuccl_chunk.so (the C ABI declared in include/uccl_chunk.h).

Argument marshalling only: every step of the data path (dedup, place, combine, write,
forward) runs in the HIP kernels.  Buffers are device memory owned by the caller, passed
as torch tensors (their data_ptr() is used) or as integer device addresses; ``stream`` is
a torch.cuda.Stream, an integer hipStream_t, or None for torch's current stream.

There is no CPU fallback: if the shared library cannot be loaded, load() raises.
"""
import ctypes as C
import os
import threading

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libuccl_chunk.so")
HEADER_PATH = os.path.join(os.path.dirname(_PKG), "include", "uccl_chunk.h")

UCCL_F32, UCCL_BF16, UCCL_F16, UCCL_I32 = 0, 1, 2, 3
UCCL_SUM, UCCL_MAX, UCCL_MIN, UCCL_COPY, UCCL_PROD = 0, 1, 2, 3, 4
UCCL_OK, UCCL_EINVAL, UCCL_EALIGN, UCCL_ELAUNCH, UCCL_ENOMEM, UCCL_ETOOBIG = 0, -1, -2, -3, -4, -5
UCCL_NO_FORWARD = 0xFFFFFFFFFFFFFFFF
DESC_BYTES = 32
UCCL_NOALLOC_MAX_DESCS = 2048
GATHER_DESC_BYTES = 160
UCCL_MAX_SOURCES = 16


class uccl_extents(C.Structure):
    _fields_ = [("acc_bytes", C.c_uint64), ("out_bytes", C.c_uint64),
                ("recv_bytes", C.c_uint64), ("n_bits", C.c_uint64)]


class uccl_launch_opts(C.Structure):
    _fields_ = [("chunk_bytes", C.c_uint32), ("parts", C.c_uint32), ("reserved", C.c_uint32 * 2)]


class uccl_plan(C.Structure):
    _fields_ = [("kernel", C.c_uint32), ("records_per_group", C.c_uint32), ("parts", C.c_uint32),
                ("threads", C.c_uint32), ("groups", C.c_uint32), ("unit_bytes", C.c_uint32), ("reserved", C.c_uint32 * 2)]


KERNEL_NAMES = ("chunk_flat_kernel", "chunk_few_kernel", "chunk_gather_kernel", "chunk_gather_parts_kernel")


class uccl_feed_stats(C.Structure):
    _fields_ = [("flushes", C.c_uint64), ("records", C.c_uint64), ("max_batch", C.c_uint64),
                ("slot_waits", C.c_uint64)]


class UcclError(RuntimeError):
    def __init__(self, code, what):
        detail = ""
        if code == UCCL_ELAUNCH and _lib is not None:
            detail = ": " + _lib.uccl_last_error_detail().decode()
        name = _lib.uccl_strerror(code).decode() if _lib is not None else str(code)
        super().__init__(f"{what} failed: {name} ({code}){detail}")
        self.code = code


_lib = None

_SIGNATURES = {
    "uccl_chunk_apply": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32,
                                   C.c_void_p, C.c_int, C.c_int, C.c_void_p]),
    "uccl_chunk_apply_noalloc": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32,
                                           C.c_void_p, C.c_int, C.c_int, C.c_void_p]),
    "uccl_chunk_apply_checked": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                           C.c_uint32, C.c_void_p, C.c_int, C.c_int,
                                           C.POINTER(uccl_extents), C.c_void_p, C.c_void_p]),
    "uccl_chunk_apply_opts": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                        C.c_uint32, C.c_void_p, C.c_int, C.c_int,
                                        C.POINTER(uccl_extents), C.c_void_p, C.POINTER(uccl_launch_opts),
                                        C.c_void_p]),
    "uccl_chunk_apply_indirect": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                            C.c_void_p, C.c_uint32, C.c_void_p, C.c_int, C.c_int,
                                            C.POINTER(uccl_extents), C.c_void_p, C.POINTER(uccl_launch_opts),
                                            C.c_void_p]),
    "uccl_chunk_reduce_gather": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32,
                                           C.c_void_p, C.c_int, C.c_int, C.POINTER(uccl_extents),
                                           C.c_void_p, C.POINTER(uccl_launch_opts), C.c_void_p]),
    "uccl_chunk_scatter": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p,
                                     C.c_void_p]),
    "uccl_chunk_scatter_checked": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32,
                                             C.c_void_p, C.POINTER(uccl_extents), C.c_void_p,
                                             C.c_void_p]),
    "uccl_chunk_scatter_opts": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p,
                                          C.POINTER(uccl_extents), C.c_void_p, C.POINTER(uccl_launch_opts),
                                          C.c_void_p]),
    "uccl_chunk_segment": (C.c_int, [C.c_void_p, C.c_void_p, C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint64,
                                     C.c_uint64, C.c_void_p, C.c_uint32, C.c_uint32, C.c_uint32, C.c_void_p]),
    "uccl_dedup_reset": (C.c_int, [C.c_void_p, C.c_uint64, C.c_void_p]),
    "uccl_init": (C.c_int, []),
    "uccl_claim_timeouts": (C.c_int, [C.POINTER(C.c_uint64)]),
    "uccl_feed_create": (C.c_int, [C.POINTER(C.c_void_p), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                   C.c_int, C.c_int, C.c_int, C.c_uint32, C.c_uint32, C.c_void_p]),
    "uccl_feed_push": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_uint32]),
    "uccl_feed_poll": (C.c_int, [C.c_void_p]),
    "uccl_feed_flush": (C.c_int, [C.c_void_p]),
    "uccl_feed_sync": (C.c_int, [C.c_void_p]),
    "uccl_feed_get_stats": (C.c_int, [C.c_void_p, C.POINTER(uccl_feed_stats)]),
    "uccl_feed_destroy": (C.c_int, [C.c_void_p]),
    "uccl_dedup_report": (C.c_int, [C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint32, C.c_void_p]),
    "uccl_message_status": (C.c_int, [C.c_void_p, C.c_void_p, C.c_uint32, C.c_uint32, C.c_void_p, C.c_int,
                                      C.c_void_p]),
    "uccl_launch_plan": (C.c_int, [C.c_uint32, C.POINTER(uccl_launch_opts), C.c_int, C.c_int, C.POINTER(uccl_plan)]),
    "uccl_time_next_launch": (C.c_int, [C.c_void_p, C.c_void_p]),
    "uccl_strerror": (C.c_char_p, [C.c_int]),
    "uccl_last_error_detail": (C.c_char_p, []),
    "uccl_version": (C.c_int, []),
}


def load(path: str = None):
    """Load the built library (building it first only if no library file exists)."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or LIB_PATH
    try:
        # PyTorch ships its own HIP runtime under the same soname; it has to be the first
        # one the process loads, or device memory made by torch is unknown to this library.
        import torch  # noqa: F401
    except ImportError:
        pass
    if not os.path.exists(p):
        if path is not None:
            raise RuntimeError(f"{p} does not exist")
        from .build import build
        build()
    elif path is None:
        from .build import sources
        if max(os.path.getmtime(f) for f in sources()) > os.path.getmtime(p):
            raise RuntimeError(f"{p} is older than its sources: rebuild (python -m paper_2504_17307_amd.build)")
    lib = C.CDLL(p)
    for name, (res, args) in _SIGNATURES.items():
        fn = getattr(lib, name)  # AttributeError if the library does not export it
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


def _ptr(x):
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _nbytes(x):
    return 0 if x is None else x.numel() * x.element_size()


def _stream(s):
    if s is None:
        import torch
        return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else None
    if isinstance(s, int):
        return s
    return s.cuda_stream


def _check(code, what):
    if code != UCCL_OK:
        raise UcclError(code, what)


_tls = threading.local()


def _call(name, *cargs):
    """Make the C call with marshalled arguments, or, inside uccl_prepare, hand the call back instead."""
    fn = getattr(load(), name)
    pending = getattr(_tls, "pending", None)
    if pending is not None:
        pending.append((fn, cargs, name))
        return
    _check(fn(*cargs), name)


def uccl_prepare(func, *args, **kwargs):
    """Marshal a call once, enqueue it many times (a control path that issues two small calls per
    message spends as long turning tensors into pointers as the launch itself takes).  ``func`` is
    one of this module's functions that make exactly one C call (uccl_chunk_apply*,
    uccl_chunk_scatter*, uccl_chunk_reduce_gather, uccl_chunk_segment, uccl_dedup_reset,
    uccl_dedup_report, uccl_message_status); the result is a zero-argument callable that makes that
    C call with the same pointers, sizes and stream handle every time: the stream is the one given,
    or torch's current one, WHEN THE CALL WAS PREPARED.  The callable keeps the arguments alive."""
    _tls.pending = []
    try:
        func(*args, **kwargs)
        (fn, cargs, name), = _tls.pending
    finally:
        _tls.pending = None

    def enqueue():
        code = fn(*cargs)
        if code != UCCL_OK:
            raise UcclError(code, name)

    enqueue.keeps = (args, kwargs)
    return enqueue


def _extents(extents, acc, out_stage, recv_stage, n_bits):
    if extents is not None:
        return extents
    if n_bits is None:
        raise ValueError("n_bits is required when extents are derived from tensors")
    return uccl_extents(_nbytes(acc), _nbytes(out_stage), _nbytes(recv_stage), int(n_bits))


_opts_cache = {}


def _opts(opts):
    """None, a uccl_launch_opts, or a (chunk_bytes, parts) pair -> a pointer argument."""
    if opts is None:
        return None
    if isinstance(opts, uccl_launch_opts):
        return C.byref(opts)
    key = (int(opts[0]), int(opts[1]))
    ref = _opts_cache.get(key)
    if ref is None:
        ref = _opts_cache[key] = C.byref(uccl_launch_opts(*key))   # byref keeps the struct alive
    return ref


def uccl_chunk_apply(acc, out_stage, recv_stage, descs, n_descs, dedup_bitmap, dtype, op, stream=None):
    _call("uccl_chunk_apply", _ptr(acc), _ptr(out_stage), _ptr(recv_stage), _ptr(descs), int(n_descs),
          _ptr(dedup_bitmap), int(dtype), int(op), _stream(stream))


def uccl_chunk_apply_noalloc(acc, out_stage, recv_stage, descs, n_descs, dedup_bitmap, dtype, op, stream=None):
    _call("uccl_chunk_apply_noalloc", _ptr(acc), _ptr(out_stage), _ptr(recv_stage), _ptr(descs),
          int(n_descs), _ptr(dedup_bitmap), int(dtype), int(op), _stream(stream))


def uccl_chunk_apply_checked(acc, out_stage, recv_stage, descs, n_descs, dedup_bitmap, dtype, op,
                             extents=None, n_rejected=None, stream=None, n_bits=None):
    """``extents`` is a uccl_extents; when None it is filled from the tensors' sizes and
    ``n_bits`` (the bitmap's valid bit count)."""
    e = _extents(extents, acc, out_stage, recv_stage, n_bits)
    _call("uccl_chunk_apply_checked", _ptr(acc), _ptr(out_stage), _ptr(recv_stage), _ptr(descs),
          int(n_descs), _ptr(dedup_bitmap), int(dtype), int(op), C.byref(e), _ptr(n_rejected),
          _stream(stream))


def uccl_chunk_apply_opts(acc, out_stage, recv_stage, descs, n_descs, dedup_bitmap, dtype, op,
                          extents=None, n_rejected=None, opts=None, stream=None, n_bits=None):
    """The general form.  Checked when ``extents`` or ``n_bits`` is given, unchecked otherwise;
    ``opts`` is None, a uccl_launch_opts, or a (chunk_bytes, parts) pair."""
    e = None
    if extents is not None or n_bits is not None:
        e = C.byref(_extents(extents, acc, out_stage, recv_stage, n_bits))
    _call("uccl_chunk_apply_opts", _ptr(acc), _ptr(out_stage), _ptr(recv_stage), _ptr(descs), int(n_descs),
          _ptr(dedup_bitmap), int(dtype), int(op), e, _ptr(n_rejected), _opts(opts), _stream(stream))


def uccl_chunk_apply_indirect(acc, out_stage, recv_stage, descs, n_descs_ptr, max_descs, dedup_bitmap,
                              dtype, op, extents=None, n_rejected=None, opts=None, stream=None, n_bits=None):
    """``descs`` / ``n_descs_ptr`` may be pinned host tensors.  With ``n_bits`` given (or an
    explicit ``extents``) records are validated on the GPU, otherwise the call is unchecked."""
    e = None
    if extents is not None or n_bits is not None:
        e = C.byref(_extents(extents, acc, out_stage, recv_stage, n_bits))
    _call("uccl_chunk_apply_indirect", _ptr(acc), _ptr(out_stage), _ptr(recv_stage), _ptr(descs),
          _ptr(n_descs_ptr), int(max_descs), _ptr(dedup_bitmap), int(dtype), int(op), e, _ptr(n_rejected),
          _opts(opts), _stream(stream))


def uccl_chunk_reduce_gather(acc, out_stage, recv_stage, descs, n_descs, dedup_bitmap, dtype, op,
                             extents=None, n_rejected=None, opts=None, stream=None, n_bits=None):
    e = None
    if extents is not None or n_bits is not None:
        e = C.byref(_extents(extents, acc, out_stage, recv_stage, n_bits))
    _call("uccl_chunk_reduce_gather", _ptr(acc), _ptr(out_stage), _ptr(recv_stage), _ptr(descs),
          int(n_descs), _ptr(dedup_bitmap), int(dtype), int(op), e, _ptr(n_rejected), _opts(opts),
          _stream(stream))


def uccl_chunk_scatter(dst, recv_stage, descs, n_descs, dedup_bitmap, stream=None):
    _call("uccl_chunk_scatter", _ptr(dst), _ptr(recv_stage), _ptr(descs), int(n_descs), _ptr(dedup_bitmap),
          _stream(stream))


def uccl_chunk_scatter_checked(dst, recv_stage, descs, n_descs, dedup_bitmap, extents=None,
                               n_rejected=None, stream=None, n_bits=None):
    e = _extents(extents, dst, None, recv_stage, n_bits)
    _call("uccl_chunk_scatter_checked", _ptr(dst), _ptr(recv_stage), _ptr(descs), int(n_descs),
          _ptr(dedup_bitmap), C.byref(e), _ptr(n_rejected), _stream(stream))


def uccl_chunk_scatter_opts(dst, recv_stage, descs, n_descs, dedup_bitmap, extents=None, n_rejected=None,
                            opts=None, stream=None, n_bits=None):
    e = None
    if extents is not None or n_bits is not None:
        e = C.byref(_extents(extents, dst, None, recv_stage, n_bits))
    _call("uccl_chunk_scatter_opts", _ptr(dst), _ptr(recv_stage), _ptr(descs), int(n_descs),
          _ptr(dedup_bitmap), e, _ptr(n_rejected), _opts(opts), _stream(stream))


def uccl_init():
    _call("uccl_init")


def uccl_claim_timeouts() -> int:
    n = C.c_uint64(0)
    _call("uccl_claim_timeouts", C.byref(n))
    return n.value


SEND_DESC_BYTES = 16


def uccl_chunk_segment(out_stage, tensor, tensor_off, nbytes, chunk_bytes, stage_off=0, slot_stride=None,
                       send_descs=None, conn_id=0, msg_id=0, first_csn=0, stream=None):
    """``send_descs``: a tensor (device or pinned host) with room for ceil(nbytes / chunk_bytes) 16-byte records, or None."""
    _call("uccl_chunk_segment", _ptr(out_stage), _ptr(tensor), int(tensor_off), int(nbytes),
          int(chunk_bytes), int(stage_off), int(chunk_bytes if slot_stride is None else slot_stride),
          _ptr(send_descs), int(conn_id), int(msg_id), int(first_csn), _stream(stream))


def uccl_dedup_reset(dedup_bitmap, n_bits, stream=None):
    _call("uccl_dedup_reset", _ptr(dedup_bitmap), int(n_bits), _stream(stream))


def uccl_feed_create(acc, out_stage, recv_stage, dedup_bitmap, dtype, lane0_op, lane1_op, capacity_records,
                     n_slots, stream=None):
    """Returns an opaque feed handle (keep the tensors alive for as long as the feed is)."""
    h = C.c_void_p()
    _call("uccl_feed_create", C.byref(h), _ptr(acc), _ptr(out_stage), _ptr(recv_stage), _ptr(dedup_bitmap),
          int(dtype), int(lane0_op), int(lane1_op), int(capacity_records), int(n_slots), _stream(stream))
    return h


def uccl_feed_push(feed, lane, host_records):
    """``host_records``: a contiguous numpy array of 32-byte records in host memory."""
    _call("uccl_feed_push", feed, int(lane), host_records.ctypes.data, len(host_records))


def uccl_feed_poll(feed):
    _call("uccl_feed_poll", feed)


def uccl_feed_flush(feed):
    _call("uccl_feed_flush", feed)


def uccl_feed_sync(feed):
    _call("uccl_feed_sync", feed)


def uccl_feed_get_stats(feed) -> dict:
    s = uccl_feed_stats()
    _call("uccl_feed_get_stats", feed, C.byref(s))
    return {k: getattr(s, k) for k, _ in uccl_feed_stats._fields_}


def uccl_feed_destroy(feed):
    _call("uccl_feed_destroy", feed)


ACK_HEADER_BYTES = 32


def uccl_message_status(dedup_bitmap, n_chunks, n_slots, bits_per_slot, status, recycle=False, stream=None):
    """Per-slot {cum_ack, n_applied, complete, 0} of a connection's message window into `status`."""
    _call("uccl_message_status", _ptr(dedup_bitmap), _ptr(n_chunks), int(n_slots), int(bits_per_slot),
          _ptr(status), int(bool(recycle)), _stream(stream))


def uccl_dedup_report(dedup_bitmap, n_bits, report, max_ranges, stream=None):
    """``report``: a tensor of at least 32 + 16 * max_ranges bytes (device or pinned host)."""
    _call("uccl_dedup_report", _ptr(dedup_bitmap), int(n_bits), _ptr(report), int(max_ranges),
          _stream(stream))


def uccl_launch_plan(n_descs, opts=None, gather=False, reads_acc=True) -> dict:
    """What a call of ``n_descs`` records with these options is launched as (host arithmetic only)."""
    p = uccl_plan()
    _call("uccl_launch_plan", int(n_descs), _opts(opts), int(bool(gather)), int(bool(reads_acc)), C.byref(p))
    d = {k: getattr(p, k) for k, _ in uccl_plan._fields_ if k != "reserved"}
    d["kernel"] = KERNEL_NAMES[p.kernel]
    return d


def uccl_time_next_launch(start_event, stop_event):
    """Events are torch.cuda.Event(enable_timing=True) objects (recorded once before, so
    that their HIP handles exist) or integer hipEvent_t handles."""
    h = lambda e: None if e is None else (e if isinstance(e, int) else e.cuda_event)
    _call("uccl_time_next_launch", h(start_event), h(stop_event))


def uccl_strerror(code) -> str:
    return load().uccl_strerror(int(code)).decode()


def uccl_version() -> int:
    return load().uccl_version()
