/*
 * CPU oracle for the receive-side chunk data path.  TEST INFRASTRUCTURE ONLY.
 *
 * This is the plain definition of what the GPU library must compute, executed
 * sequentially on one host thread.  It exists so that tests, the smoke check and
 * the benchmark's CPU-baseline leg have something independent to compare the GPU
 * path with.  It shares no code, header or table with the GPU library, and no
 * product code path may call it.
 *
 * What it follows:
 *  - Section 2.1 (collectives over RDMA): the GPU kernel copies between transport
 *    buffers and tensor buffers and reduces (sum, max) transport buffers into the
 *    tensor buffers.
 *  - Section 3.1 (reassembly challenge): out-of-order payloads are copied to where
 *    the receiver CPU says they belong, then the reduction runs.
 *  - Section 3.2 (handling out-of-order packets): sequence numbers identify
 *    chunks, retransmission creates duplicates, reorder buffers live in GPU memory.
 *
 * Parity status: every function is pinned by tests/test_oracle_pins.py (multi-source fold:
 * tests/test_gather_reduce.py; whole definition against a brute-force model:
 * tests/test_oracle_bruteforce.py; sender-side segmentation: tests/test_segment.py) except
 *  - MAX/MIN on NaN or mixed-sign zeros, and which copy of a duplicated sequence
 *    number supplies the bytes: the paper fixes neither ("parity unpinned"; the
 *    behaviour below is a definition made here, see the comments at each).
 */
#ifndef CHUNK_ORACLE_H
#define CHUNK_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
  uint64_t src_off; /* byte offset of the arrival's slot in recv_stage */
  uint64_t dst_off; /* byte offset in acc */
  uint64_t out_off; /* byte offset in out_stage, or ORC_NO_FORWARD */
  uint32_t len;     /* payload bytes */
  uint32_t seq;     /* logical chunk id = index into seen[] */
} orc_desc;

#define ORC_NO_FORWARD 0xFFFFFFFFFFFFFFFFull
/* flag in out_off: the combined value goes to out_stage only, acc is read but not written */
#define ORC_FORWARD_ONLY 0x8000000000000000ull

enum { ORC_F32 = 0, ORC_BF16 = 1, ORC_F16 = 2, ORC_I32 = 3 };
enum { ORC_SUM = 0, ORC_MAX = 1, ORC_MIN = 2, ORC_COPY = 3, ORC_PROD = 4 };

/* negative return codes: a precondition of the problem statement is violated */
enum {
  ORC_E_ARG = -1,      /* bad dtype / op / null pointer */
  ORC_E_SEQ = -2,      /* seq >= n_bits */
  ORC_E_ALIGN = -3,    /* offset not 16-byte aligned or len not a multiple of the element size */
  ORC_E_BOUNDS = -4,   /* a range leaves its buffer, or a forward with no out_stage */
  ORC_E_MISMATCH = -5, /* two records of one seq differ in dst/out/len or payload bytes */
  ORC_E_OVERLAP = -6   /* records of different seq overlap in acc or in out_stage */
};

/* Apply records in array (= arrival) order.  seen[] (one byte per seq) persists
 * across calls; the caller zeroes it to start a new epoch.  Returns the number
 * of records applied (first arrivals), or a negative code with nothing further
 * applied after the offending record. */
int64_t orc_apply(void* acc, uint64_t acc_bytes, void* out_stage, uint64_t out_bytes,
                  const void* recv_stage, uint64_t recv_bytes, const orc_desc* descs,
                  uint64_t n_descs, uint8_t* seen, uint64_t n_bits, int dtype, int op);

/* Several senders' chunks for one destination chunk (Section 2.1: reductions "from multiple
 * sender GPUs"): t = acc; for each source in the listed order t = op(t, source); acc = t.
 * 16-bit SUM / PROD keep t in binary32 over the whole fold and round once at the end. */
#define ORC_MAX_SOURCES 16
typedef struct {
  uint64_t dst_off, out_off;
  uint32_t len, seq, n_src, reserved;
  uint64_t src_off[ORC_MAX_SOURCES];
} orc_gather_desc;
int64_t orc_reduce_gather(void* acc, uint64_t acc_bytes, void* out_stage, uint64_t out_bytes,
                          const void* recv_stage, uint64_t recv_bytes, const orc_gather_desc* descs,
                          uint64_t n_descs, uint8_t* seen, uint64_t n_bits, int dtype, int op);

/* All-to-all scatter: byte copy, no forward, element type irrelevant. */
int64_t orc_scatter(void* dst, uint64_t dst_bytes, const void* recv_stage, uint64_t recv_bytes,
                    const orc_desc* descs, uint64_t n_descs, uint8_t* seen, uint64_t n_bits);

/* Checks the preconditions a single call must satisfy beyond per-record bounds:
 * records sharing a seq are identical (fields and payload); records of different
 * seq touch disjoint acc and out_stage ranges.  0 or a negative code. */
int64_t orc_check_call(const void* recv_stage, uint64_t recv_bytes, const orc_desc* descs,
                       uint64_t n_descs);

/* Pack seen[] into 32-bit words, bit (s & 31) of word (s >> 5) = seen[s]. */
void orc_pack_bitmap(const uint8_t* seen, uint64_t n_bits, uint32_t* words);

/* The same call on n_threads cores (chunk_threaded.c): serial dedup in arrival order, then the
 * chosen records dealt to threads, each applied through orc_apply().  Equals orc_apply() bit
 * for bit when the call's preconditions hold; returns the number applied or a negative code. */
int64_t orc_apply_threaded(void* acc, uint64_t acc_bytes, void* out_stage, uint64_t out_bytes,
                           const void* recv_stage, uint64_t recv_bytes, const orc_desc* descs,
                           uint64_t n_descs, uint8_t* seen, uint64_t n_bits, int dtype, int op,
                           int n_threads);

/* Receiver feedback read off a packed bitmap (Section 3.2 seq/ack, Section 4.3 selective
 * retransmission): cum_ack = first clear bit (n_bits if none); n_applied = set bits;
 * n_ranges = maximal runs of set bits starting above cum_ack, the first max_ranges of them
 * written to ranges[] as {start, end} pairs with end exclusive, ascending. */
void orc_ack_report(const uint32_t* words, uint64_t n_bits, uint64_t* cum_ack, uint64_t* n_applied,
                    uint32_t* n_ranges, uint64_t* ranges, uint32_t max_ranges);

/* Per-message receiver state (Section 3.1: up to 128 messages in flight per connection, each
 * of up to 256 chunks, a last-chunk mark that tells the receiver the chunk count).  The bitmap
 * is n_slots windows of bits_per_slot bits (a multiple of 32); window i holds message slot i
 * at bits [i * bits_per_slot, + limit) with limit = n_chunks[i] clamped to bits_per_slot, or
 * bits_per_slot while n_chunks[i] == 0 (count not known yet).  out[i] = {cum_ack = first clear
 * bit below limit (limit if none), n_applied = set bits below limit, complete = count known and
 * all set, 0}.  recycle != 0 clears the whole window of every complete slot afterwards. */
void orc_message_status(uint32_t* words, const uint32_t* n_chunks, uint32_t n_slots,
                        uint32_t bits_per_slot, uint32_t* out4, int recycle);

/* Sender side (Section 2.1: the kernel copies from the tensor buffer to the transport buffer;
 * Section 3.1: the sender CPU names the address of every data chunk and sends a 32-bit control
 * header with it -- 8-bit connection id, 7-bit message id, 8-bit chunk sequence number, a
 * last-chunk mark; Appendix A: onChunkSize gives the chunk size, then a chunk_desc is built).
 * The bytes tensor[tensor_off, +bytes) are cut into payloads of chunk_bytes (the last may be
 * shorter; none if bytes == 0); payload i is copied to stage + stage_off + i * slot_stride and
 * described by descs[i] = { its staging offset, its length, its header }.  The chunks are numbered
 * first_csn, first_csn + 1, ...: a message holds 256 of them, so chunk number c travels as
 * message (msg_id + c / 256) mod 128 with sequence number c mod 256, and the last chunk of every
 * message (sequence number 255, or the final chunk of the transfer) carries the mark.  Header
 * layout (a choice of this interface): sequence number in bits 0-7, mark in bit 8, message id in
 * bits 9-15, connection id in bits 16-23, bits 24-31 zero.  Returns the number of chunks or a
 * negative code (ORC_E_ALIGN: an offset, chunk_bytes or slot_stride not a multiple of 16, or
 * chunk_bytes == 0; ORC_E_BOUNDS: a range leaves its buffer or slots overlap; ORC_E_ARG). */
typedef struct {
  uint64_t stage_off;
  uint32_t len;
  uint32_t header;
} orc_send_desc;
int64_t orc_segment(void* stage, uint64_t stage_bytes, const void* tensor, uint64_t tensor_bytes,
                    uint64_t tensor_off, uint64_t bytes, uint32_t chunk_bytes, uint64_t stage_off,
                    uint64_t slot_stride, orc_send_desc* descs, uint32_t conn_id, uint32_t msg_id,
                    uint32_t first_csn);

/* Textbook in-order ring allreduce of R vectors of n elements (n % R == 0),
 * no chunks, no transport: x is R*n elements (rank-major), result is R*n
 * elements (every rank's final buffer).  Returns 0 or ORC_E_ARG. */
int orc_ring_allreduce(const void* x, uint32_t R, uint64_t n, int dtype, int op, void* result);

/* One element-wise combine, exposed so tests can pin the numerics directly. */
float orc_combine_f32(float a, float r, int op);
uint16_t orc_combine_bf16(uint16_t a, uint16_t r, int op);
uint16_t orc_combine_f16(uint16_t a, uint16_t r, int op);
int32_t orc_combine_i32(int32_t a, int32_t r, int op);
uint16_t orc_f32_to_bf16(float f);
uint16_t orc_f32_to_f16(float f);
float orc_f16_to_f32(uint16_t h);

#ifdef __cplusplus
}
#endif
#endif
