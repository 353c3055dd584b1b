/*
 * The C ABI used from plain C, no Python and no PyTorch: device memory from hipMalloc, a
 * small deterministic chunk stream built here (reordered, with duplicates), one call of
 * each entry point, results compared byte for byte with the CPU oracle (linked as a
 * separate library); then the remaining entry points, and a stream of small messages through the
 * host-side batcher.  Prints "C ABI OK", "MORE OK" and "FEED OK" and exits 0 on success.
 *
 * Build: hipcc -I include -I oracle tests/c_abi_check.c -L<pkg> -luccl_chunk -L oracle -lchunk_oracle
 */
#define _POSIX_C_SOURCE 199309L
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <time.h>

#include "chunk_oracle.h"
#include "uccl_chunk.h"

#define CK(x)                                                                          \
  do {                                                                                 \
    hipError_t e_ = (x);                                                               \
    if (e_ != hipSuccess) {                                                            \
      fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);   \
      return 2;                                                                        \
    }                                                                                  \
  } while (0)
#define UC(x)                                                                          \
  do {                                                                                 \
    int c_ = (x);                                                                      \
    if (c_ != UCCL_OK) {                                                               \
      fprintf(stderr, "%s at line %d: %s\n", uccl_strerror(c_), __LINE__,              \
              uccl_last_error_detail());                                               \
      return 3;                                                                        \
    }                                                                                  \
  } while (0)

static uint32_t lcg(uint32_t* s) { *s = *s * 1664525u + 1013904223u; return *s >> 8; }

static double now_us(void) {
  struct timespec t;
  clock_gettime(CLOCK_MONOTONIC, &t);
  return t.tv_sec * 1e6 + t.tv_nsec * 1e-3;
}

/*
 * Small allreduces (ring share of R = 8, 4 KiB chunks, 2..32 chunks per segment) pushed message
 * by message into uccl_feed from C: reduce-scatter records to lane 0, allgather records to
 * lane 1, then poll.  Run twice from the same initial state -- once with poll deciding when
 * to hand over (adaptive batching), once flushing after every message -- and each result is
 * compared with the oracle.  Prints the host time per message of both.
 */
static int feed_check(hipStream_t st) {
  enum { M = 400, R = 8, CH = 4096 };
  uint32_t seed = 777u;
  uint32_t cps[M];
  uint64_t acc_off[M], bit_off[M], rec_off[M], n_rec = 0, acc_bytes = 0, n_bits = 0, out_bytes = 0, out_off[M];
  for (int m = 0; m < M; ++m) {
    cps[m] = 2 + lcg(&seed) % 31;
    acc_off[m] = acc_bytes; bit_off[m] = n_bits; rec_off[m] = n_rec; out_off[m] = out_bytes;
    acc_bytes += (uint64_t)R * cps[m] * CH;
    n_bits += 2ull * (R - 1) * cps[m];
    n_rec += 2ull * (R - 1) * cps[m] + 2; /* one retransmitted record per phase */
    out_bytes += (2ull * (R - 1) - 1) * cps[m] * CH;
  }
  const uint64_t recv_bytes = n_rec * CH;
  float* h_acc = (float*)malloc(acc_bytes);
  float* h_recv = (float*)malloc(recv_bytes);
  uccl_chunk_desc* rec = (uccl_chunk_desc*)malloc(sizeof(uccl_chunk_desc) * n_rec);
  if (!h_acc || !h_recv || !rec) return 7;
  for (uint64_t i = 0; i < acc_bytes / 4; ++i) h_acc[i] = (float)(lcg(&seed) % 4001) / 1000.0f - 2.0f;
  for (uint64_t i = 0; i < recv_bytes / 4; ++i) h_recv[i] = (float)(lcg(&seed) % 4001) / 1000.0f - 2.0f;
  /* records of message m: [rec_off, +7 cps + 1) reduce-scatter, then 7 cps + 1 allgather; rank r = 0 */
  for (int m = 0; m < M; ++m) {
    const uint32_t c = cps[m], per = (R - 1) * c;
    for (int phase = 0; phase < 2; ++phase) {
      uccl_chunk_desc* d = rec + rec_off[m] + (uint64_t)phase * (per + 1);
      for (uint32_t k = 0; k < per; ++k) {
        const uint32_t s = k / c, j = k % c;
        const uint32_t seg = phase == 0 ? (2 * R - s - 1) % R : (R - s) % R;
        d[k].dst_off = acc_off[m] + ((uint64_t)seg * c + j) * CH;
        const uint64_t fwd_index = (uint64_t)phase * per + k; /* the last allgather step does not forward */
        d[k].out_off = (phase == 1 && s == R - 2) ? UCCL_NO_FORWARD : out_off[m] + fwd_index * CH;
        d[k].len = CH;
        d[k].seq = (uint32_t)(bit_off[m] + (uint64_t)phase * per + k);
      }
      for (uint32_t k = per - 1; k > 0; --k) { /* arrival order within the phase: shuffled */
        uint32_t j = lcg(&seed) % (k + 1);
        uccl_chunk_desc t = d[k]; d[k] = d[j]; d[j] = t;
      }
      d[per] = d[lcg(&seed) % per]; /* a retransmission of one of them, in a slot of its own */
      for (uint32_t k = 0; k <= per; ++k) d[k].src_off = (rec_off[m] + (uint64_t)phase * (per + 1) + k) * CH;
      /* identical payload for the two copies */
      for (uint32_t k = 0; k < per; ++k)
        if (d[k].seq == d[per].seq) memcpy((char*)h_recv + d[per].src_off, (char*)h_recv + d[k].src_off, CH);
    }
  }

  /* oracle: per message, reduce-scatter records then allgather records */
  float* o_acc = (float*)malloc(acc_bytes);
  unsigned char* o_out = (unsigned char*)calloc(out_bytes, 1);
  uint8_t* seen = (uint8_t*)calloc(n_bits, 1);
  memcpy(o_acc, h_acc, acc_bytes);
  for (int m = 0; m < M; ++m) {
    const uint32_t per = (R - 1) * cps[m];
    const orc_desc* d = (const orc_desc*)(rec + rec_off[m]);
    if (orc_apply(o_acc, acc_bytes, o_out, out_bytes, h_recv, recv_bytes, d, per + 1, seen, n_bits, ORC_F32, ORC_SUM) != per ||
        orc_apply(o_acc, acc_bytes, o_out, out_bytes, h_recv, recv_bytes, d + per + 1, per + 1, seen, n_bits, ORC_F32, ORC_COPY) != per) {
      fprintf(stderr, "feed: oracle refused message %d\n", m);
      return 7;
    }
  }

  void *d_acc, *d_out, *d_recv, *d_bm;
  CK(hipMalloc(&d_acc, acc_bytes)); CK(hipMalloc(&d_out, out_bytes)); CK(hipMalloc(&d_recv, recv_bytes));
  CK(hipMalloc(&d_bm, (n_bits + 31) / 32 * 4));
  CK(hipMemcpy(d_recv, h_recv, recv_bytes, hipMemcpyHostToDevice));
  float* g_acc = (float*)malloc(acc_bytes);
  unsigned char* g_out = (unsigned char*)malloc(out_bytes);
  double us[2];
  uccl_feed_stats stats[2];
  for (int mode = 0; mode < 2; ++mode) { /* 0: adaptive (poll), 1: hand over after every message */
    CK(hipMemcpy(d_acc, h_acc, acc_bytes, hipMemcpyHostToDevice));
    CK(hipMemset(d_out, 0, out_bytes));
    UC(uccl_dedup_reset((uint32_t*)d_bm, n_bits, st));
    CK(hipStreamSynchronize(st));
    uccl_feed* f = NULL;
    UC(uccl_feed_create(&f, d_acc, d_out, d_recv, (uint32_t*)d_bm, UCCL_F32, UCCL_SUM, UCCL_COPY, 1u << 15, 8, st));
    const double t0 = now_us();
    for (int m = 0; m < M; ++m) {
      const uint32_t per = (R - 1) * cps[m];
      UC(uccl_feed_push(f, 0, rec + rec_off[m], per + 1));
      UC(uccl_feed_push(f, 1, rec + rec_off[m] + per + 1, per + 1));
      UC(mode == 0 ? uccl_feed_poll(f) : uccl_feed_flush(f));
    }
    UC(uccl_feed_sync(f));
    us[mode] = (now_us() - t0) / M;
    UC(uccl_feed_get_stats(f, &stats[mode]));
    UC(uccl_feed_destroy(f));
    CK(hipMemcpy(g_acc, d_acc, acc_bytes, hipMemcpyDeviceToHost));
    CK(hipMemcpy(g_out, d_out, out_bytes, hipMemcpyDeviceToHost));
    if (memcmp(g_acc, o_acc, acc_bytes)) { fprintf(stderr, "feed mode %d: acc differs\n", mode); return 8; }
    if (memcmp(g_out, o_out, out_bytes)) { fprintf(stderr, "feed mode %d: out_stage differs\n", mode); return 8; }
  }
  printf("FEED OK: %d messages, %llu records; adaptive %.2f us/message (%llu hand-overs, largest %llu records, "
         "%llu slot waits); one hand-over per message %.2f us/message (%llu hand-overs, %llu slot waits)\n",
         (int)M, (unsigned long long)n_rec, us[0], (unsigned long long)stats[0].flushes,
         (unsigned long long)stats[0].max_batch, (unsigned long long)stats[0].slot_waits, us[1],
         (unsigned long long)stats[1].flushes, (unsigned long long)stats[1].slot_waits);
  return 0;
}


/*
 * The entry points beyond apply / scatter, each once from C against the oracle: a call of few
 * large records through uccl_chunk_apply_noalloc and through uccl_chunk_apply_opts with records
 * cut into parts, uccl_chunk_apply_indirect with the count in device memory, a multi-source fold,
 * sender-side segmentation, and the per-message status with recycling.
 */
static int more_entry_points(hipStream_t st) {
  enum { N = 24, C = 65536, NS = 3, SLOTS = 16, BPS = 64 };
  { /* what the library says it launches for the calls made below (host arithmetic only) */
    const uccl_launch_opts four = {C, 4, {0, 0}};
    uccl_plan pl;
    if (uccl_launch_plan(N + 4, &four, 0, 1, &pl) != UCCL_OK || pl.kernel != UCCL_KERNEL_FEW || pl.parts != 4 ||
        pl.groups != (N + 4) * 4 || uccl_launch_plan(N, NULL, 1, 1, &pl) != UCCL_OK || pl.kernel != UCCL_KERNEL_GATHER_PARTS) {
      printf("launch plan\n");
      return 1;
    }
  }
  const uint64_t bytes = (uint64_t)N * C;
  uint32_t seed = 4242u;
  float* h_recv = (float*)malloc(bytes * NS);
  float* h_acc = (float*)malloc(bytes);
  for (uint64_t i = 0; i < bytes * NS / 4; ++i) h_recv[i] = (float)(lcg(&seed) % 4001) / 1000.0f - 2.0f;
  for (uint64_t i = 0; i < bytes / 4; ++i) h_acc[i] = (float)(lcg(&seed) % 4001) / 2000.0f - 1.0f;
  uccl_chunk_desc h_desc[N + 4];
  for (uint32_t k = 0; k < N + 4; ++k) { /* arrival k < N carries chunk 7 k mod N; the last four repeat chunks 0..3 */
    const uint32_t s = k < N ? (k * 7u) % N : k - N;
    h_desc[k].src_off = (uint64_t)k * C;
    h_desc[k].dst_off = (uint64_t)s * C;
    h_desc[k].out_off = (uint64_t)(N - 1 - s) * C;
    h_desc[k].len = (s == 5) ? C - 1040 : C;
    h_desc[k].seq = s;
  }
  for (uint32_t k = N; k < N + 4; ++k) /* a retransmitted chunk: the same bytes, here read from the same slot */
    for (uint32_t j = 0; j < N; ++j)
      if (h_desc[j].seq == h_desc[k].seq) h_desc[k].src_off = h_desc[j].src_off;

  float* o_acc = (float*)malloc(bytes);
  unsigned char* o_out = (unsigned char*)calloc(bytes, 1);
  uint8_t seen[N];
  uint32_t o_words[1], g_words[1];
  memcpy(o_acc, h_acc, bytes); memset(seen, 0, N);
  if (orc_apply(o_acc, bytes, o_out, bytes, h_recv, bytes, (const orc_desc*)h_desc, N + 4, seen, N, ORC_F32, ORC_SUM) != N) return 7;
  orc_pack_bitmap(seen, N, o_words);

  void *d_acc, *d_out, *d_recv, *d_desc, *d_bm, *d_cnt;
  CK(hipMalloc(&d_acc, bytes)); CK(hipMalloc(&d_out, bytes)); CK(hipMalloc(&d_recv, bytes * NS));
  CK(hipMalloc(&d_desc, sizeof(h_desc))); CK(hipMalloc(&d_bm, 4 * SLOTS * BPS / 32)); CK(hipMalloc(&d_cnt, 4));
  CK(hipMemcpy(d_recv, h_recv, bytes * NS, hipMemcpyHostToDevice));
  CK(hipMemcpy(d_desc, h_desc, sizeof(h_desc), hipMemcpyHostToDevice));
  float* g_acc = (float*)malloc(bytes);
  unsigned char* g_out = (unsigned char*)malloc(bytes);
  UC(uccl_init());
  for (int variant = 0; variant < 3; ++variant) {
    CK(hipMemcpy(d_acc, h_acc, bytes, hipMemcpyHostToDevice));
    CK(hipMemset(d_out, 0, bytes));
    UC(uccl_dedup_reset((uint32_t*)d_bm, N, st));
    if (variant == 0) {
      UC(uccl_chunk_apply_noalloc(d_acc, d_out, d_recv, (const uccl_chunk_desc*)d_desc, N + 4, (uint32_t*)d_bm,
                                  UCCL_F32, UCCL_SUM, st));
    } else if (variant == 1) {
      const uccl_launch_opts opts = {C, 4, {0, 0}};
      UC(uccl_chunk_apply_opts(d_acc, d_out, d_recv, (const uccl_chunk_desc*)d_desc, N + 4, (uint32_t*)d_bm,
                               UCCL_F32, UCCL_SUM, NULL, NULL, &opts, st));
    } else {
      const uint32_t live = N + 4;
      CK(hipMemcpy(d_cnt, &live, 4, hipMemcpyHostToDevice));
      UC(uccl_chunk_apply_indirect(d_acc, d_out, d_recv, (const uccl_chunk_desc*)d_desc, (const uint32_t*)d_cnt,
                                   N + 4, (uint32_t*)d_bm, UCCL_F32, UCCL_SUM, NULL, NULL, NULL, st));
    }
    CK(hipStreamSynchronize(st));
    CK(hipMemcpy(g_acc, d_acc, bytes, hipMemcpyDeviceToHost));
    CK(hipMemcpy(g_out, d_out, bytes, hipMemcpyDeviceToHost));
    CK(hipMemcpy(g_words, d_bm, 4, hipMemcpyDeviceToHost));
    if (memcmp(g_acc, o_acc, bytes) || memcmp(g_out, o_out, bytes) || g_words[0] != o_words[0]) {
      fprintf(stderr, "few-record call, variant %d: differs from the oracle\n", variant);
      return 7;
    }
  }
  uint64_t gave_up = 1;
  UC(uccl_claim_timeouts(&gave_up));
  if (gave_up != 0) { fprintf(stderr, "%llu parts gave up waiting\n", (unsigned long long)gave_up); return 7; }

  /* multi-source fold: chunk s folds source regions 2, 0, 1 in that order */
  uccl_gather_desc h_g[N];
  memset(h_g, 0, sizeof(h_g));
  for (uint32_t s = 0; s < N; ++s) {
    h_g[s].dst_off = (uint64_t)s * C; h_g[s].out_off = UCCL_NO_FORWARD; h_g[s].len = C; h_g[s].seq = s; h_g[s].n_src = NS;
    h_g[s].src_off[0] = 2 * bytes + (uint64_t)s * C; h_g[s].src_off[1] = (uint64_t)s * C; h_g[s].src_off[2] = bytes + (uint64_t)s * C;
  }
  if (sizeof(orc_gather_desc) != sizeof(uccl_gather_desc)) return 8;
  memcpy(o_acc, h_acc, bytes); memset(seen, 0, N);
  if (orc_reduce_gather(o_acc, bytes, NULL, 0, h_recv, bytes * NS, (const orc_gather_desc*)h_g, N, seen, N, ORC_F32, ORC_SUM) != N) return 8;
  void* d_g;
  CK(hipMalloc(&d_g, sizeof(h_g)));
  CK(hipMemcpy(d_g, h_g, sizeof(h_g), hipMemcpyHostToDevice));
  CK(hipMemcpy(d_acc, h_acc, bytes, hipMemcpyHostToDevice));
  UC(uccl_dedup_reset((uint32_t*)d_bm, N, st));
  UC(uccl_chunk_reduce_gather(d_acc, NULL, d_recv, (const uccl_gather_desc*)d_g, N, (uint32_t*)d_bm, UCCL_F32, UCCL_SUM,
                              NULL, NULL, NULL, st));
  CK(hipStreamSynchronize(st));
  CK(hipMemcpy(g_acc, d_acc, bytes, hipMemcpyDeviceToHost));
  if (memcmp(g_acc, o_acc, bytes)) { fprintf(stderr, "multi-source fold differs\n"); return 8; }

  /* sender side: 1 000 003 bytes of the tensor from offset 4096 in 48 KiB chunks, slots 64 KiB apart */
  enum { SEG = 1000003, CHUNK = 49152, STRIDE = 65536, NCH = (SEG + CHUNK - 1) / CHUNK };
  orc_send_desc o_sd[NCH];
  uccl_send_desc g_sd[NCH];
  if (sizeof(orc_send_desc) != sizeof(uccl_send_desc)) return 9;
  memset(o_out, 0, bytes);
  if (orc_segment(o_out, bytes, h_acc, bytes, 4096, SEG, CHUNK, 128, STRIDE, o_sd, 9, 127, 250) != NCH) return 9;
  void* d_sd;
  CK(hipMalloc(&d_sd, sizeof(g_sd)));
  CK(hipMemcpy(d_acc, h_acc, bytes, hipMemcpyHostToDevice));
  CK(hipMemset(d_out, 0, bytes));
  UC(uccl_chunk_segment(d_out, d_acc, 4096, SEG, CHUNK, 128, STRIDE, (uccl_send_desc*)d_sd, 9, 127, 250, st));
  CK(hipStreamSynchronize(st));
  CK(hipMemcpy(g_out, d_out, bytes, hipMemcpyDeviceToHost));
  CK(hipMemcpy(g_sd, d_sd, sizeof(g_sd), hipMemcpyDeviceToHost));
  if (memcmp(g_out, o_out, bytes) || memcmp(g_sd, o_sd, sizeof(g_sd))) { fprintf(stderr, "segmentation differs\n"); return 9; }

  /* per-message status of 16 windows of 64 bits, with recycling */
  uint32_t h_bits[SLOTS * BPS / 32], o_bits[SLOTS * BPS / 32], h_cnt[SLOTS], o_st[SLOTS * 4], g_st[SLOTS * 4];
  for (uint32_t i = 0; i < SLOTS * BPS / 32; ++i) h_bits[i] = (i % 3 == 0) ? 0xFFFFFFFFu : (lcg(&seed) | (lcg(&seed) << 16));
  for (uint32_t i = 0; i < SLOTS; ++i) h_cnt[i] = (i % 4 == 0) ? 0u : 1u + lcg(&seed) % BPS;
  h_bits[2] = h_bits[3] = 0xFFFFFFFFu; h_cnt[1] = 40;   /* slot 1: complete */
  memcpy(o_bits, h_bits, sizeof(h_bits));
  orc_message_status(o_bits, h_cnt, SLOTS, BPS, o_st, 1);
  void *d_n, *d_st;
  CK(hipMalloc(&d_n, sizeof(h_cnt))); CK(hipMalloc(&d_st, sizeof(g_st)));
  CK(hipMemcpy(d_bm, h_bits, sizeof(h_bits), hipMemcpyHostToDevice));
  CK(hipMemcpy(d_n, h_cnt, sizeof(h_cnt), hipMemcpyHostToDevice));
  UC(uccl_message_status((uint32_t*)d_bm, (const uint32_t*)d_n, SLOTS, BPS, (uccl_msg_status*)d_st, 1, st));
  CK(hipStreamSynchronize(st));
  CK(hipMemcpy(g_st, d_st, sizeof(g_st), hipMemcpyDeviceToHost));
  CK(hipMemcpy(h_bits, d_bm, sizeof(h_bits), hipMemcpyDeviceToHost));
  if (memcmp(g_st, o_st, sizeof(g_st)) || memcmp(h_bits, o_bits, sizeof(h_bits))) { fprintf(stderr, "message status differs\n"); return 10; }
  if (o_st[1 * 4 + 2] != 1u || o_bits[2] != 0u) { fprintf(stderr, "slot 1 was to be complete and recycled\n"); return 10; }

  printf("MORE OK: no-alloc / cut / indirect apply, multi-source fold, segmentation (%d chunks), message status\n", (int)NCH);
  return 0;
}

int main(void) {
  enum { N = 300, C = 8192, DUP = 37 }; /* 300 logical chunks of 8 KiB, 37 retransmitted */
  const uint64_t n_arr = N + DUP, acc_bytes = (uint64_t)N * C, recv_bytes = n_arr * C;
  uint32_t seed = 12345u;

  /* arrival order: a shuffle of all chunks plus duplicates of the first DUP of them */
  uint32_t* order = (uint32_t*)malloc(sizeof(uint32_t) * n_arr);
  for (uint32_t i = 0; i < N; ++i) order[i] = i;
  for (uint32_t i = 0; i < DUP; ++i) order[N + i] = (i * 7u) % N;
  for (uint64_t i = n_arr - 1; i > 0; --i) {
    uint64_t j = lcg(&seed) % (i + 1);
    uint32_t t = order[i]; order[i] = order[j]; order[j] = t;
  }
  float* chunk_val = (float*)malloc(acc_bytes); /* payload of logical chunk s */
  for (uint64_t i = 0; i < acc_bytes / 4; ++i) chunk_val[i] = (float)(lcg(&seed) % 2001) / 1000.0f - 1.0f;
  float* h_recv = (float*)malloc(recv_bytes);
  float* h_acc = (float*)malloc(acc_bytes);
  for (uint64_t i = 0; i < acc_bytes / 4; ++i) h_acc[i] = (float)(lcg(&seed) % 2001) / 500.0f - 2.0f;
  uccl_chunk_desc* h_desc = (uccl_chunk_desc*)malloc(sizeof(uccl_chunk_desc) * n_arr);
  for (uint64_t k = 0; k < n_arr; ++k) {
    uint32_t s = order[k];
    memcpy((char*)h_recv + k * C, (char*)chunk_val + (uint64_t)s * C, C);
    h_desc[k].src_off = k * C;
    h_desc[k].dst_off = (uint64_t)(N - 1 - s) * C; /* placed in reverse */
    h_desc[k].out_off = (s % 3 == 0) ? UCCL_NO_FORWARD : (uint64_t)s * C;
    h_desc[k].len = (s % 5 == 0) ? C - 48 : C;      /* some short chunks */
    h_desc[k].seq = s;
  }

  /* oracle (its record layout is byte-compatible by construction of the interface) */
  float* o_acc = (float*)malloc(acc_bytes);
  unsigned char* o_out = (unsigned char*)calloc(acc_bytes, 1);
  uint8_t* seen = (uint8_t*)calloc(N, 1);
  memcpy(o_acc, h_acc, acc_bytes);
  if (sizeof(orc_desc) != sizeof(uccl_chunk_desc)) return 4;
  int64_t applied = orc_apply(o_acc, acc_bytes, o_out, acc_bytes, h_recv, recv_bytes, (const orc_desc*)h_desc,
                              n_arr, seen, N, ORC_F32, ORC_SUM);
  if (applied != N) { fprintf(stderr, "oracle applied %lld\n", (long long)applied); return 4; }
  uint32_t o_words[(N + 31) / 32];
  orc_pack_bitmap(seen, N, o_words);

  /* GPU */
  void *d_acc, *d_out, *d_recv, *d_desc, *d_bm, *d_rej, *d_rep;
  hipStream_t st;
  CK(hipStreamCreate(&st));
  CK(hipMalloc(&d_acc, acc_bytes)); CK(hipMalloc(&d_out, acc_bytes)); CK(hipMalloc(&d_recv, recv_bytes));
  CK(hipMalloc(&d_desc, sizeof(uccl_chunk_desc) * n_arr)); CK(hipMalloc(&d_bm, sizeof(o_words)));
  CK(hipMalloc(&d_rej, 4)); CK(hipMalloc(&d_rep, sizeof(uccl_ack_report) + 16 * 8));
  CK(hipMemcpy(d_acc, h_acc, acc_bytes, hipMemcpyHostToDevice));
  CK(hipMemcpy(d_recv, h_recv, recv_bytes, hipMemcpyHostToDevice));
  CK(hipMemcpy(d_desc, h_desc, sizeof(uccl_chunk_desc) * n_arr, hipMemcpyHostToDevice));
  CK(hipMemset(d_out, 0, acc_bytes)); CK(hipMemset(d_rej, 0, 4)); CK(hipMemset(d_bm, 0xFF, sizeof(o_words)));
  UC(uccl_dedup_reset((uint32_t*)d_bm, N, st));
  uccl_extents ext = {acc_bytes, acc_bytes, recv_bytes, N};
  /* first half through the checked entry point, second half through the plain one */
  UC(uccl_chunk_apply_checked(d_acc, d_out, d_recv, (const uccl_chunk_desc*)d_desc, (uint32_t)(n_arr / 2),
                              (uint32_t*)d_bm, UCCL_F32, UCCL_SUM, &ext, (uint32_t*)d_rej, st));
  UC(uccl_chunk_apply(d_acc, d_out, d_recv, (const uccl_chunk_desc*)d_desc + n_arr / 2,
                      (uint32_t)(n_arr - n_arr / 2), (uint32_t*)d_bm, UCCL_F32, UCCL_SUM, st));
  UC(uccl_dedup_report((const uint32_t*)d_bm, N, d_rep, 8, st));
  CK(hipStreamSynchronize(st));

  float* g_acc = (float*)malloc(acc_bytes);
  unsigned char* g_out = (unsigned char*)malloc(acc_bytes);
  uint32_t g_words[(N + 31) / 32], rejected = 99;
  uccl_ack_report rep;
  CK(hipMemcpy(g_acc, d_acc, acc_bytes, hipMemcpyDeviceToHost));
  CK(hipMemcpy(g_out, d_out, acc_bytes, hipMemcpyDeviceToHost));
  CK(hipMemcpy(g_words, d_bm, sizeof(g_words), hipMemcpyDeviceToHost));
  CK(hipMemcpy(&rejected, d_rej, 4, hipMemcpyDeviceToHost));
  CK(hipMemcpy(&rep, d_rep, sizeof(rep), hipMemcpyDeviceToHost));
  if (memcmp(g_acc, o_acc, acc_bytes)) { fprintf(stderr, "acc differs\n"); return 5; }
  if (memcmp(g_out, o_out, acc_bytes)) { fprintf(stderr, "out_stage differs\n"); return 5; }
  if (memcmp(g_words, o_words, sizeof(o_words))) { fprintf(stderr, "bitmap differs\n"); return 5; }
  if (rejected != 0) { fprintf(stderr, "rejected %u\n", rejected); return 5; }
  if (rep.cum_ack != N || rep.n_applied != N || rep.n_ranges != 0 || rep.complete != 1) {
    fprintf(stderr, "report: cum %llu applied %llu ranges %u complete %u\n", (unsigned long long)rep.cum_ack,
            (unsigned long long)rep.n_applied, rep.n_ranges, rep.complete);
    return 5;
  }

  /* all-to-all scatter of the same stream into a fresh destination */
  unsigned char* o_dst = (unsigned char*)calloc(acc_bytes, 1);
  memset(seen, 0, N);
  for (uint64_t k = 0; k < n_arr; ++k) h_desc[k].out_off = UCCL_NO_FORWARD;
  if (orc_scatter(o_dst, acc_bytes, h_recv, recv_bytes, (const orc_desc*)h_desc, n_arr, seen, N) != N) return 6;
  CK(hipMemcpy(d_desc, h_desc, sizeof(uccl_chunk_desc) * n_arr, hipMemcpyHostToDevice));
  CK(hipMemset(d_acc, 0, acc_bytes));
  UC(uccl_dedup_reset((uint32_t*)d_bm, N, st));
  UC(uccl_chunk_scatter(d_acc, d_recv, (const uccl_chunk_desc*)d_desc, (uint32_t)n_arr, (uint32_t*)d_bm, st));
  CK(hipStreamSynchronize(st));
  CK(hipMemcpy(g_out, d_acc, acc_bytes, hipMemcpyDeviceToHost));
  if (memcmp(g_out, o_dst, acc_bytes)) { fprintf(stderr, "scatter differs\n"); return 6; }

  printf("C ABI OK: %d chunks, %d duplicates, version %d\n", (int)N, (int)DUP, uccl_version());
  const int more = more_entry_points(st);
  if (more != 0) return more;
  return feed_check(st);
}
