/*
 * uccl_chunk.h -- C ABI of the receive-side chunk data path for multipath collectives
 * on AMD Instinct MI355X (gfx950).
 *
 * Problem (paper, Section 2.1 "collectives over RDMA", Section 3.1 "challenge of
 * reassembly", Section 3.2 "handling out-of-order packets", Section 5): chunks of a
 * collective message are sprayed over many network paths and land in GPU memory in
 * ARRIVAL order, possibly more than once (retransmission).  The receiver CPU knows,
 * per arrival, which logical chunk it is and where it belongs, and passes a list of
 * pointers to the GPU kernel through shared memory.  The GPU kernel must put every
 * payload where it belongs and combine it with the tensor buffer (sum, max) or just
 * copy it, and leave the result where the next ring step will send it from.
 *
 * This library is that GPU kernel for one rank's share: for every record, in one
 * pass over the payload,
 *     dedup   - test-and-set bit `seq` of the bitmap; only the first arrival proceeds
 *     place   - src = recv_stage + src_off, dst = acc + dst_off, fwd = out_stage + out_off
 *     combine - t[i] = op(acc[dst+i], recv[src+i])   (COPY: t[i] = recv[src+i])
 *     write   - acc[dst+i] = t[i]; and out_stage[out+i] = t[i] when the record forwards
 *
 * All buffer pointers are DEVICE pointers owned by the caller (the data-path calls never
 * allocate, free or keep them; only the optional uccl_feed object owns memory); `stream`
 * is a hipStream_t passed as void* (NULL = the null stream).  Every call only enqueues
 * work on `stream` and returns: no host
 * synchronisation, no host read of device memory.  Records and buffers must stay valid
 * until the stream has passed the call; receive slots may be recycled after that point
 * (the paper's irecv_free_ptrs moment, Section 5).
 */
#ifndef UCCL_CHUNK_H
#define UCCL_CHUNK_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define UCCL_CHUNK_VERSION 2

/* One record per ARRIVAL, written by the control path in arrival order (Section 3.1:
 * "the right order given by the receiver CPU"; Section 5: packet pointers passed via
 * CPU-GPU shared memory).  32 bytes; the array must be 16-byte aligned. */
typedef struct uccl_chunk_desc {
  uint64_t src_off; /* byte offset of this arrival's slot in recv_stage; multiple of 16 */
  uint64_t dst_off; /* byte offset in acc (apply) / dst (scatter); multiple of 16 */
  uint64_t out_off; /* byte offset in out_stage, multiple of 16; UCCL_NO_FORWARD = do not forward */
  uint32_t len;     /* payload bytes, 0 .. 2^32 - 1; a multiple of the element size (apply) */
  uint32_t seq;     /* logical chunk id = bit index in dedup_bitmap (the role of the chunk
                       sequence number of the control header, Section 3.1) */
} uccl_chunk_desc;

#define UCCL_NO_FORWARD 0xFFFFFFFFFFFFFFFFull
/* OR-ed into out_off: forward the combined value but do NOT write it back to acc (acc is
 * only read).  For intermediate reduce-scatter steps of a ring, whose partial sums are
 * needed by the next rank only: 3 instead of 4 bytes moved per payload byte.  The offset
 * proper is out_off & ~UCCL_FORWARD_ONLY. */
#define UCCL_FORWARD_ONLY 0x8000000000000000ull

typedef enum uccl_dtype { UCCL_F32 = 0, UCCL_BF16 = 1, UCCL_F16 = 2, UCCL_I32 = 3 } uccl_dtype;

/* Section 2.1 names "sum, max"; MIN, PROD and COPY complete the set a collective library
 * offers.  a = accumulator element, r = received element.
 * SUM / PROD f32       : one IEEE-754 binary32 add / multiply (nearest even, subnormals kept).
 * SUM / PROD bf16, f16 : widen both to binary32 (exact), add / multiply, round once to the
 *                        storage type, nearest even; a bf16 NaN result is (bits >> 16) | 0x0040.
 * SUM / PROD i32       : two's complement, wrapping modulo 2^32.
 * MAX / MIN            : strict comparison on the (widened) values, signed for i32; a tie or an
 *                        unordered pair keeps the accumulator's element: MAX(a, r) = r if r > a else a.
 * COPY                 : t = r; the element type is irrelevant and `len` may be any byte count. */
typedef enum uccl_op {
  UCCL_SUM = 0, UCCL_MAX = 1, UCCL_MIN = 2, UCCL_COPY = 3, UCCL_PROD = 4
} uccl_op;

enum {
  UCCL_OK = 0,
  UCCL_EINVAL = -1,  /* null pointer with n_descs > 0, unknown dtype/op, bad launch options, aliasing buffers */
  UCCL_EALIGN = -2,  /* a base pointer is not 16-byte aligned (bitmap / counter: 4-byte) */
  UCCL_ELAUNCH = -3, /* HIP refused the launch; uccl_last_error_detail() has HIP's message */
  UCCL_ENOMEM = -4,  /* uccl_feed_create / uccl_init could not get host, pinned or device memory */
  UCCL_ETOOBIG = -5  /* more records than the entry point's stated maximum: split the call */
};

/* Buffer sizes for the checked entry points (HOST struct, read during the call). */
typedef struct uccl_extents {
  uint64_t acc_bytes;  /* size of acc / dst */
  uint64_t out_bytes;  /* size of out_stage (0 if none) */
  uint64_t recv_bytes; /* size of recv_stage */
  uint64_t n_bits;     /* number of valid bits in dedup_bitmap */
} uccl_extents;

/* Per-call tuning (HOST struct, read during the call; a NULL pointer means all zeros).  Results
 * never depend on it, only speed does.
 *   chunk_bytes  the transport's chunk size (the control path chooses it per connection: 32 KB by
 *                default, Section 3.3 "control coalescing"; Appendix A onChunkSize), 0 = unknown.
 *                Sets how many records a workgroup takes: about 32 KiB of payload per workgroup (calls of
 *                at most 128 records take one workgroup per record, sized to the chunk).
 *   parts        workgroups per record for calls of few, large records (Appendix C.4: small
 *                messages are where the kernel's fixed costs show): 0 = the library decides,
 *                1 = never cut a record, 2..16 = that many.  Honoured only when a workgroup takes
 *                a single record and the call has at most 2048 of them. */
typedef struct uccl_launch_opts {
  uint32_t chunk_bytes;
  uint32_t parts;
  uint32_t reserved[2]; /* 0 */
} uccl_launch_opts;

/*
 * uccl_chunk_apply -- dedup, place, combine, write back and forward (see top of file).
 *
 *   acc          device, read+written: the rank's accumulator / tensor buffer
 *   out_stage    device, written: outbound staging buffer; may be NULL if no record forwards
 *   recv_stage   device, read: arrival-order slot pool (the GPU-resident reorder buffers)
 *   descs        device, read: n_descs records, arrival order
 *   dedup_bitmap device, read+written atomically: bit s set <=> chunk s has been applied
 *                since the last uccl_dedup_reset; persists across calls
 *
 * Exactly one record per distinct `seq` is applied over the bitmap's lifetime, whatever
 * the arrival order and however often a chunk is repeated, within a call or across
 * calls on one stream.  Which of several copies supplies the bytes is unspecified.
 *
 * Preconditions the caller guarantees (the unchecked call cannot verify them):
 *   - seq < number of bits in dedup_bitmap; every offset range lies inside its buffer;
 *   - records with the same seq have identical dst_off, out_off, len and payload bytes;
 *   - within one call, records with different seq touch disjoint ranges of acc and of
 *     out_stage (order between dependent steps is expressed by separate calls);
 *   - recv_stage overlaps neither acc nor out_stage.
 * A record whose offsets are misaligned, whose len is not a multiple of the element size,
 * or which forwards although out_stage is NULL, is skipped (its bit stays clear).
 *
 * Returns UCCL_OK (also for n_descs == 0, which enqueues nothing) or a negative code;
 * on error nothing has been enqueued.  One launch covers the whole call with one workgroup
 * per 1..32 records; a record count whose workgroup count exceeds what the device accepts
 * in one launch comes back as UCCL_ELAUNCH (split the call).
 *
 * Scratch memory.  A call of few large records (at most 16 MiB of payload in chunks above 32 KiB, or at
 * most 32 chunks of 32 KiB; at most 128 records when no chunk size is given) is launched with several
 * workgroups per record so that it fills the machine; those workgroups
 * agree on the record's fate through one 64-bit claim word per record (on a 128-byte line of its
 * own) in a pool the library allocates once per device (16 MiB + 8 bytes, hipMalloc at the first
 * such call or in uccl_init, kept until the process ends).  The pool has one region per stream
 * handle, for the first 64 handles that issue such a call on the device; a region is never given
 * back, so do not destroy a stream while such a call is still running on it (a stream created
 * next may be given the same handle, and with it the region).  If the pool cannot be had, the
 * stream is the 65th or later, or the stream is being
 * captured into a graph, the call is launched with one workgroup per record instead: slower,
 * same result.  Apart from that one-time allocation no data-path call allocates.
 */
int uccl_chunk_apply(void* acc, void* out_stage, const void* recv_stage,
                     const uccl_chunk_desc* descs, uint32_t n_descs, uint32_t* dedup_bitmap,
                     uccl_dtype dtype, uccl_op op, void* stream);

/* Eagerly make the current device's claim pool (see "Scratch memory" above) and look up the
 * address of the array uccl_chunk_apply_noalloc uses, so that no later call allocates or loads
 * anything.  Idempotent; UCCL_OK or a negative code.  Utility, no passage of the paper. */
int uccl_init(void);

/*
 * uccl_chunk_apply_noalloc -- uccl_chunk_apply for callers that cannot allocate device memory:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * operation and result; the claim words of records cut into parts (see "Scratch memory" above)
 * live in an array inside the library's code object instead of the pool: UCCL_NOALLOC_MAX_DESCS
 * lines of 128 bytes + 256 bytes = 256.25 KiB, held by every GPU the library runs on until the
 * process ends.  The call makes no hipMalloc / hipFree and creates no pool; the first call on a device
 * (or uccl_init) looks the array's device address up.
 *   - n_descs > UCCL_NOALLOC_MAX_DESCS returns UCCL_ETOOBIG and enqueues nothing.  (Calls that
 *     large are never cut into parts, so uccl_chunk_apply serves them without any scratch memory.)
 *   - Every call on a GPU shares that GPU's array, whatever the stream: a split call first clears
 *     its own words with a small fill kernel, then runs; the pair may be captured and replayed.
 *     Calls (or replays) that overlap in time on one GPU race on the array: keep them on one
 *     stream, or order them with events.
 */
#define UCCL_NOALLOC_MAX_DESCS 2048
int uccl_chunk_apply_noalloc(void* acc, void* out_stage, const void* recv_stage,
                             const uccl_chunk_desc* descs, uint32_t n_descs, uint32_t* dedup_bitmap,
                             uccl_dtype dtype, uccl_op op, void* stream);

/*
 * uccl_chunk_apply_checked -- same operation; additionally every record is validated ON
 * THE GPU against `extents` before its bit is touched: seq < n_bits, all three ranges
 * inside their buffers, alignment, len granularity, and a forward needs out_stage.  A
 * record that fails is skipped (bit stays clear, no byte moved) and, if `n_rejected`
 * (device uint32_t, caller-zeroed, 4-byte aligned, may be NULL) is given, counted there.
 * On the host, overlapping recv_stage / acc / out_stage extents return UCCL_EINVAL.
 */
int uccl_chunk_apply_checked(void* acc, void* out_stage, const void* recv_stage,
                             const uccl_chunk_desc* descs, uint32_t n_descs,
                             uint32_t* dedup_bitmap, uccl_dtype dtype, uccl_op op,
                             const uccl_extents* extents, uint32_t* n_rejected, void* stream);

/*
 * uccl_chunk_apply_opts -- the general form: uccl_chunk_apply with optional validation
 * (`extents` and `n_rejected` as in uccl_chunk_apply_checked, both may be NULL = unchecked) and
 * optional per-call tuning (`opts`, may be NULL).  UCCL_EINVAL for parts > 16 or non-zero
 * reserved fields.
 */
int uccl_chunk_apply_opts(void* acc, void* out_stage, const void* recv_stage,
                          const uccl_chunk_desc* descs, uint32_t n_descs, uint32_t* dedup_bitmap,
                          uccl_dtype dtype, uccl_op op, const uccl_extents* extents,
                          uint32_t* n_rejected, const uccl_launch_opts* opts, void* stream);

/*
 * uccl_chunk_apply_indirect -- the same operation fed from a descriptor slot the control
 * path refills, with no argument changing between launches (Section 5: the receiver CPU
 * passes the pointer list through CPU-GPU shared memory; Appendix C.4: per-batch kernel
 * launches are what hurts small messages).  `descs` has room for `max_descs` records and
 * `*n_descs_ptr` (uint32_t, 4-byte aligned) says how many are live; both may be pinned
 * host memory mapped into the device (hipHostMalloc) or device memory, and are read when
 * the kernel runs, not when the call is made.  A count above max_descs is capped.  Because
 * every argument is fixed, the call can be captured once in a HIP graph and replayed after
 * the control path has rewritten the slot.  The launch is sized for max_descs.  `extents`
 * and `n_rejected` are as in uccl_chunk_apply_checked; both may be NULL (unchecked); `opts` may
 * be NULL.  A call made while its stream is being captured is never cut into parts.
 */
int uccl_chunk_apply_indirect(void* acc, void* out_stage, const void* recv_stage,
                              const uccl_chunk_desc* descs, const uint32_t* n_descs_ptr,
                              uint32_t max_descs, uint32_t* dedup_bitmap, uccl_dtype dtype,
                              uccl_op op, const uccl_extents* extents, uint32_t* n_rejected,
                              const uccl_launch_opts* opts, void* stream);

/*
 * uccl_chunk_reduce_gather -- several senders' chunks for ONE destination chunk in one
 * record (Section 2.1: the kernel reduces the transport buffers "from multiple sender GPUs"
 * into the tensor buffer; direct reduce-scatter and tree steps have this shape).  For each
 * first-arriving record:
 *     t = acc[dst + i]
 *     for j = 0 .. n_src-1:  t = op(t, recv_stage[src_off[j] + i])      -- in this order
 *     acc[dst + i] = t  (unless UCCL_FORWARD_ONLY);  out_stage[out + i] = t  (if forwarding)
 * SUM / PROD on bf16 and f16 keep t in binary32 across the whole fold and round once at the
 * end; on f32 every step is one binary32 operation; MAX / MIN select as in uccl_chunk_apply.
 * The order of sources is part of the record, so the result does not depend on arrival
 * timing.  COPY is not defined here (UCCL_EINVAL).  The accumulator is read and written
 * once per chunk: (n_src + 1) reads and 1 (+1 forwarding) writes per payload byte of one source.
 * `seq` dedups the record as a whole: the control path issues it when all its sources are
 * in, and may issue it again.  `extents` / `n_rejected` as in uccl_chunk_apply_checked, both
 * may be NULL; `opts` may be NULL.  A call of few records of 32 KiB or more is cut into parts like
 * uccl_chunk_apply's (same claim pool, same fallback under graph capture).  Records: 160 bytes, 16-byte
 * aligned array.
 */
#define UCCL_MAX_SOURCES 16
typedef struct uccl_gather_desc {
  uint64_t dst_off;                    /* byte offset in acc, multiple of 16 */
  uint64_t out_off;                    /* as in uccl_chunk_desc, incl. UCCL_NO_FORWARD / UCCL_FORWARD_ONLY */
  uint32_t len;                        /* payload bytes of each source, multiple of the element size */
  uint32_t seq;                        /* bit index in dedup_bitmap */
  uint32_t n_src;                      /* 1 .. UCCL_MAX_SOURCES */
  uint32_t reserved;
  uint64_t src_off[UCCL_MAX_SOURCES];  /* byte offsets in recv_stage, multiples of 16, fold order */
} uccl_gather_desc;
int uccl_chunk_reduce_gather(void* acc, void* out_stage, const void* recv_stage,
                             const uccl_gather_desc* descs, uint32_t n_descs, uint32_t* dedup_bitmap,
                             uccl_dtype dtype, uccl_op op, const uccl_extents* extents,
                             uint32_t* n_rejected, const uccl_launch_opts* opts, void* stream);

/*
 * uccl_chunk_scatter -- all-to-all receive side (Section 2.1: copy from transport
 * buffers to tensor buffers; Section 3.1: scattered memcpy): dedup + place + byte copy
 * into `dst` at per-source offsets.  No combine, no forward (out_off must be
 * UCCL_NO_FORWARD, other records are skipped), element type irrelevant.
 */
int uccl_chunk_scatter(void* dst, const void* recv_stage, const uccl_chunk_desc* descs,
                       uint32_t n_descs, uint32_t* dedup_bitmap, void* stream);

int uccl_chunk_scatter_checked(void* dst, const void* recv_stage, const uccl_chunk_desc* descs,
                               uint32_t n_descs, uint32_t* dedup_bitmap,
                               const uccl_extents* extents, uint32_t* n_rejected, void* stream);

/* The general form of the scatter: `extents`, `n_rejected` and `opts` may each be NULL. */
int uccl_chunk_scatter_opts(void* dst, const void* recv_stage, const uccl_chunk_desc* descs,
                            uint32_t n_descs, uint32_t* dedup_bitmap, const uccl_extents* extents,
                            uint32_t* n_rejected, const uccl_launch_opts* opts, void* stream);

/*
 * uccl_chunk_segment -- sender side: cut a range of the tensor buffer into chunks in the outbound
 * staging buffer and write one send record per chunk for the control path (Section 2.1: the kernel
 * copies from the tensor buffer to the transport buffer; Section 3.1: the sender CPU gives the
 * address of every data chunk and a 32-bit control header travels with it -- connection id 8 bits,
 * message id 7 bits, chunk sequence number 8 bits, a last-chunk mark; Appendix A: onChunkSize
 * returns the permitted chunk size, then a chunk_desc is built).  A ring's first step sends the
 * rank's own segment this way; every later step sends what uccl_chunk_apply forwarded.
 *
 *   tensor[tensor_off, +bytes) is cut into n = ceil(bytes / chunk_bytes) payloads (the last may be
 *   shorter, of any byte length; bytes == 0 enqueues nothing); payload i is copied to
 *   out_stage + stage_off + i * slot_stride and send_descs[i] = { that offset, its length, its header }.
 *   Chunks are numbered first_csn, first_csn + 1, ...; a message holds 256, so chunk number c is
 *   chunk c mod 256 of message (msg_id + c / 256) mod 128, and the last chunk of every message
 *   (sequence number 255, or the final chunk of the call) carries the mark.  Header layout:
 *   sequence number in bits 0-7, mark in bit 8, message id in bits 9-15, connection id in bits
 *   16-23, bits 24-31 zero (left to receiver-driven congestion control).
 *
 * out_stage, tensor: DEVICE memory, 16-byte aligned; send_descs: device or pinned host memory, room
 * for n records, 8-byte aligned, may be NULL (copy only).  tensor_off, stage_off, chunk_bytes and
 * slot_stride are multiples of 16 (UCCL_EALIGN), chunk_bytes > 0, slot_stride >= chunk_bytes,
 * conn_id < 256, msg_id < 128, at most 2^32 - 1 chunks (UCCL_EINVAL).  A control path that changes the
 * chunk size as it goes (onChunkSize) makes one call per run of equal-sized chunks.  Ranges must lie
 * inside their buffers and must not overlap (not checked).  Stream ordered.
 */
typedef struct uccl_send_desc {
  uint64_t stage_off; /* byte offset of the chunk's payload in out_stage */
  uint32_t len;       /* payload bytes */
  uint32_t header;    /* control header, layout above */
} uccl_send_desc;
int uccl_chunk_segment(void* out_stage, const void* tensor, uint64_t tensor_off, uint64_t bytes,
                       uint32_t chunk_bytes, uint64_t stage_off, uint64_t slot_stride,
                       uccl_send_desc* send_descs, uint32_t conn_id, uint32_t msg_id, uint32_t first_csn,
                       void* stream);

/* Clear the first n_bits bits (rounded up to whole 32-bit words) of the bitmap: starts a
 * new message / connection epoch (Section 3.1: a message id, and with it its chunk sequence
 * numbers, is reused once its message is complete).  Uses a fill kernel, so it may be captured
 * in a graph. */
int uccl_dedup_reset(uint32_t* dedup_bitmap, uint64_t n_bits, void* stream);

/*
 * uccl_dedup_report -- receiver feedback for the control path, read off the bitmap
 * (Section 3.2: seq / ack numbers guide retransmission; Section 4.3: selective
 * retransmission needs to know which chunks above the cumulative point have arrived;
 * Section 3.1: the control header's last-chunk bit marks message completion).
 * Writes to `report` (device memory or pinned host memory, 8-byte aligned, room for
 * sizeof(uccl_ack_report) + max_ranges * 16 bytes):
 *   cum_ack    first clear bit in [0, n_bits), n_bits if none: every chunk below it is applied
 *   n_applied  number of set bits in [0, n_bits)
 *   n_ranges   number of maximal runs of set bits that start above cum_ack (may exceed
 *              max_ranges; only the first max_ranges are written)
 *   complete   1 if n_applied == n_bits
 * followed by the runs in ascending order as pairs {start, end} of uint64_t, end exclusive.
 * Bits at and above n_bits in the last word are ignored.  n_bits < 2^40.  Stream ordered.
 */
typedef struct uccl_ack_report {
  uint64_t cum_ack;
  uint64_t n_applied;
  uint32_t n_ranges;
  uint32_t complete;
  uint64_t reserved;
} uccl_ack_report;
int uccl_dedup_report(const uint32_t* dedup_bitmap, uint64_t n_bits, void* report,
                      uint32_t max_ranges, void* stream);

/*
 * uccl_message_status -- per-message receiver state for one connection's window of in-flight
 * messages (Section 3.1: a 7-bit message id allows 128 messages in flight, an 8-bit chunk
 * sequence number 256 chunks each, and a last-chunk mark tells the receiver the chunk count).
 * The bitmap is read as n_slots windows of bits_per_slot bits; window i holds the chunks of
 * the message in slot i at bits [i * bits_per_slot, + limit), where limit = n_chunks[i]
 * (clamped to bits_per_slot), or bits_per_slot while the count is not known (n_chunks[i] == 0).
 *   status[i].cum_ack    first clear bit of the window below limit, limit if none
 *   status[i].n_applied  set bits below limit
 *   status[i].complete   1 iff n_chunks[i] != 0 and every bit below limit is set
 * recycle != 0: after its status is taken, the whole window of every complete slot is cleared,
 * so that the slot's message id can be reused; only then does the call write the bitmap.
 * dedup_bitmap, n_chunks, status: DEVICE memory (status may be pinned host memory), 4-byte
 * aligned, status 16-byte aligned.  bits_per_slot: multiple of 32 in 32..2048 (UCCL_EINVAL
 * otherwise).  n_slots == 0 is a no-op; more than 2^24 slots is UCCL_EINVAL.  Stream ordered.
 */
typedef struct uccl_msg_status {
  uint32_t cum_ack;
  uint32_t n_applied;
  uint32_t complete;
  uint32_t reserved; /* written as 0 */
} uccl_msg_status;
int uccl_message_status(uint32_t* dedup_bitmap, const uint32_t* n_chunks, uint32_t n_slots,
                        uint32_t bits_per_slot, uccl_msg_status* status, int recycle, void* stream);

/*
 * uccl_feed -- host-side batcher between the control path and the kernels (Appendix C.4:
 * kernel launches per batch hurt small messages; adaptive batching is the remedy).
 * The ONLY part of this library that allocates: `n_slots` (2..1024) slots, each two lanes of
 * `capacity_records` records in pinned host memory plus the same in device memory.
 *   push   copies `n` HOST records into lane 0 or 1 of the current slot; a full lane flushes
 *   flush  hands the current slot over: per non-empty lane one asynchronous record copy and
 *          one uccl_chunk_apply on the feed's stream, lane 0 before lane 1 (so a message whose
 *          reduce-scatter records went to lane 0 before its allgather records went to lane 1
 *          is applied in that order); then moves to the next slot, waiting only if that slot's
 *          previous hand-over has not finished
 *   poll   flushes pending records if the previous hand-over has finished -- the GPU would
 *          otherwise idle -- and keeps batching if it has not
 *   sync   flush, then wait until every hand-over has finished
 *   destroy  waits for the hand-overs in flight, frees the slots; records pushed but not yet
 *          handed over are dropped (call sync first to keep them)
 * Buffers, bitmap and element type are fixed at creation; lane ops are given there too.  Each
 * hand-over is launched with the largest `len` among its lane's records as the chunk size, so
 * feeds of connections with different chunk sizes do not interfere.  The
 * slots live on the device that is current at creation; use the feed with that device current.
 * If a hand-over fails half way (UCCL_ELAUNCH), its records stay in the slot and the next
 * flush offers them again; records already applied are then dropped by the bitmap.
 * A feed is used by one host thread at a time.  All calls return UCCL_OK or a negative code.
 */
typedef struct uccl_feed uccl_feed;
typedef struct uccl_feed_stats {
  uint64_t flushes;    /* hand-overs so far */
  uint64_t records;    /* records handed over */
  uint64_t max_batch;  /* largest hand-over, in records (both lanes) */
  uint64_t slot_waits; /* times push/flush had to wait for a slot to come back */
} uccl_feed_stats;
int uccl_feed_create(uccl_feed** feed, void* acc, void* out_stage, const void* recv_stage,
                     uint32_t* dedup_bitmap, uccl_dtype dtype, uccl_op lane0_op, uccl_op lane1_op,
                     uint32_t capacity_records, uint32_t n_slots, void* stream);
int uccl_feed_push(uccl_feed* feed, int lane, const uccl_chunk_desc* host_records, uint32_t n);
int uccl_feed_poll(uccl_feed* feed);
int uccl_feed_flush(uccl_feed* feed);
int uccl_feed_sync(uccl_feed* feed);
int uccl_feed_get_stats(const uccl_feed* feed, uccl_feed_stats* stats);
int uccl_feed_destroy(uccl_feed* feed);

/* What a call of `n_descs` records with these options is launched as: which kernel, how many
 * records a workgroup takes or how many workgroups a record, the workgroup size, the grid, and the
 * bytes per stream one wavefront moves per trip.  Pure host arithmetic on the arguments (no GPU
 * call, no state; the same rule the data-path calls apply), for tests, tuning and profiling tools.
 * `gather` != 0: uccl_chunk_reduce_gather, else the apply / scatter family; `reads_acc` != 0: the
 * op combines with the accumulator (anything but UCCL_COPY).  `parts` > 1 assumes that claim words
 * are to be had (see "Scratch memory"); a call that finds none is launched with parts = 1.
 * UCCL_EINVAL for a NULL `plan` or options the data-path calls would refuse.  Utility, no passage
 * of the paper. */
enum { UCCL_KERNEL_FLAT = 0, UCCL_KERNEL_FEW = 1, UCCL_KERNEL_GATHER = 2, UCCL_KERNEL_GATHER_PARTS = 3 };
typedef struct uccl_plan {
  uint32_t kernel;            /* UCCL_KERNEL_* */
  uint32_t records_per_group; /* records one workgroup takes (1 when a record is cut into parts) */
  uint32_t parts;             /* workgroups per record */
  uint32_t threads;           /* workgroup size */
  uint32_t groups;            /* workgroups in the launch */
  uint32_t unit_bytes;        /* bytes per stream a wavefront moves per trip */
  uint32_t reserved[2];       /* 0 */
} uccl_plan;
int uccl_launch_plan(uint32_t n_descs, const uccl_launch_opts* opts, int gather, int reads_acc, uccl_plan* plan);

/* Measurement aid: the next apply / scatter / report call made by THIS host thread attaches the
 * two hipEvent_t (either may be NULL) to its kernel dispatch, so that
 * hipEventElapsedTime(start, stop) is that kernel's own execution time on the device,
 * without the queueing and launch gaps an event pair recorded around the call would
 * include.  One-shot: cleared by the launch (also by a launch that fails). */
int uccl_time_next_launch(void* start_event, void* stop_event);

/* Diagnostics: parts of split records that gave up waiting for their record's decision since the
 * pool was made, on the current device (synchronous read-back; always 0 on working hardware). */
int uccl_claim_timeouts(uint64_t* count);

/* Utilities, no passage of the paper: text of a return code; HIP's text for the last
 * UCCL_ELAUNCH on this thread; UCCL_CHUNK_VERSION of the loaded library. */
const char* uccl_strerror(int code);
const char* uccl_last_error_detail(void);
int uccl_version(void);

#ifdef __cplusplus
}
#endif
#endif /* UCCL_CHUNK_H */
