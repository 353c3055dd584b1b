/*
 * CPU oracle for the receive-side chunk data path.  TEST INFRASTRUCTURE ONLY:
 * see chunk_oracle.h for scope, citations and parity status.  Plain C, one
 * thread, no blocking or fusion: one loop over arrivals, one loop over elements.
 * Build without fast-math and without fused contraction so that every add is a
 * single IEEE-754 binary32 operation with subnormals kept.
 */
#include "chunk_oracle.h"

#include <stdlib.h>
#include <string.h>

/* ---- element numerics ------------------------------------------------------ */

static uint32_t f32_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }
static float bits_f32(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }

/* bf16 is the upper half of a binary32: widening is exact. */
static float bf16_widen(uint16_t h) { return bits_f32((uint32_t)h << 16); }

/* binary32 -> bf16, round to nearest, ties to even; NaN stays a (quiet) NaN. */
uint16_t orc_f32_to_bf16(float f) {
  uint32_t u = f32_bits(f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u);
  uint32_t lsb = (u >> 16) & 1u;
  return (uint16_t)((u + 0x7FFFu + lsb) >> 16);
}

/* IEEE binary16 (1 sign, 5 exponent, 10 fraction bits) -> binary32, exact. */
float orc_f16_to_f32(uint16_t h) {
  uint32_t sign = (uint32_t)(h & 0x8000u) << 16, e = (h >> 10) & 31u, m = h & 0x3FFu;
  if (e == 31u) return bits_f32(sign | 0x7F800000u | (m << 13)); /* inf / NaN */
  if (e == 0u) {                                                  /* zero / subnormal: m * 2^-24 */
    float v = (float)m * 5.9604644775390625e-08f;                 /* exact: m < 2^10 */
    return sign ? -v : v;
  }
  return bits_f32(sign | ((e + 112u) << 23) | (m << 13));
}

/* binary32 -> binary16, round to nearest, ties to even, gradual underflow. */
uint16_t orc_f32_to_f16(float f) {
  uint32_t u = f32_bits(f);
  uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
  uint32_t mag = u & 0x7FFFFFFFu;
  if (mag > 0x7F800000u) return (uint16_t)(sign | 0x7E00u | ((mag >> 13) & 0x1FFu)); /* NaN, quieted */
  if (mag >= 0x47800000u) return (uint16_t)(sign | 0x7C00u);                         /* >= 2^16, and inf */
  int32_t e = (int32_t)(mag >> 23) - 127;
  uint32_t m = mag & 0x7FFFFFu;
  if (e >= -14) { /* normal range: drop 13 fraction bits; a carry may run into the exponent, up to inf */
    uint32_t h = ((uint32_t)(e + 15) << 10) | (m >> 13);
    uint32_t rem = m & 0x1FFFu;
    if (rem > 0x1000u || (rem == 0x1000u && (h & 1u))) ++h;
    return (uint16_t)(sign | h);
  }
  if (e < -25) return sign; /* below half of the smallest subnormal (2^-25 itself is a tie to even 0) */
  /* subnormal result: value = (2^23 + m) * 2^(e-23), unit 2^-24  =>  shift right by -(e+1) */
  uint32_t full = m | 0x800000u;
  uint32_t s = (uint32_t)(-(e + 1));
  uint32_t h = full >> s, rem = full & ((1u << s) - 1u), half = 1u << (s - 1u);
  if (rem > half || (rem == half && (h & 1u))) ++h;
  return (uint16_t)(sign | h);
}

/* The tensor-buffer value a is combined with the received value r.
 * SUM: one binary32 add.  MAX / MIN are defined here as a strict
 * comparison that keeps the local value on ties and whenever the comparison is
 * false, i.e. MAX(a,r) = r if r > a else a.  The paper names "sum, max" only
 * (Section 2.1); NaN and signed-zero behaviour is a choice made here. */
float orc_combine_f32(float a, float r, int op) {
  switch (op) {
    case ORC_SUM: return a + r;
    case ORC_PROD: return a * r;
    case ORC_MAX: return (r > a) ? r : a;
    case ORC_MIN: return (r < a) ? r : a;
    default: return r; /* COPY */
  }
}

/* bf16: widen both, combine in binary32, round once.  MAX/MIN/COPY select one of
 * the two 16-bit inputs unchanged. */
uint16_t orc_combine_bf16(uint16_t a, uint16_t r, int op) {
  float fa = bf16_widen(a), fr = bf16_widen(r);
  switch (op) {
    case ORC_SUM: return orc_f32_to_bf16(fa + fr);
    case ORC_PROD: return orc_f32_to_bf16(fa * fr);
    case ORC_MAX: return (fr > fa) ? r : a;
    case ORC_MIN: return (fr < fa) ? r : a;
    default: return r;
  }
}

/* binary16: the same scheme -- widen, combine in binary32, round once. */
uint16_t orc_combine_f16(uint16_t a, uint16_t r, int op) {
  float fa = orc_f16_to_f32(a), fr = orc_f16_to_f32(r);
  switch (op) {
    case ORC_SUM: return orc_f32_to_f16(fa + fr);
    case ORC_PROD: return orc_f32_to_f16(fa * fr);
    case ORC_MAX: return (fr > fa) ? r : a;
    case ORC_MIN: return (fr < fa) ? r : a;
    default: return r;
  }
}

/* int32: two's complement; SUM and PROD wrap modulo 2^32 (done in unsigned arithmetic). */
int32_t orc_combine_i32(int32_t a, int32_t r, int op) {
  switch (op) {
    case ORC_SUM: return (int32_t)((uint32_t)a + (uint32_t)r);
    case ORC_PROD: return (int32_t)((uint32_t)a * (uint32_t)r);
    case ORC_MAX: return (r > a) ? r : a;
    case ORC_MIN: return (r < a) ? r : a;
    default: return r;
  }
}

/* ---- per-record checks ------------------------------------------------------ */

static int range_ok(uint64_t off, uint64_t len, uint64_t size) {
  return off <= size && len <= size - off;
}

static int64_t check_record(const orc_desc* d, uint64_t acc_bytes, uint64_t out_bytes,
                            int have_out, uint64_t recv_bytes, uint64_t n_bits, uint32_t es) {
  if (d->seq >= n_bits) return ORC_E_SEQ;
  if ((d->src_off | d->dst_off) & 15u) return ORC_E_ALIGN;
  const uint64_t out_at = d->out_off & ~ORC_FORWARD_ONLY;
  if (d->out_off != ORC_NO_FORWARD && (out_at & 15u)) return ORC_E_ALIGN;
  if (d->len % es) return ORC_E_ALIGN;
  if (!range_ok(d->src_off, d->len, recv_bytes)) return ORC_E_BOUNDS;
  if (!range_ok(d->dst_off, d->len, acc_bytes)) return ORC_E_BOUNDS;
  if (d->out_off != ORC_NO_FORWARD) {
    if (!have_out || !range_ok(out_at, d->len, out_bytes)) return ORC_E_BOUNDS;
  }
  return 0;
}

/* ---- the definition --------------------------------------------------------- */

int64_t orc_apply(void* acc, uint64_t acc_bytes, void* out_stage, uint64_t out_bytes,
                  const void* recv_stage, uint64_t recv_bytes, const orc_desc* descs,
                  uint64_t n_descs, uint8_t* seen, uint64_t n_bits, int dtype, int op) {
  if (dtype < ORC_F32 || dtype > ORC_I32) return ORC_E_ARG;
  if (op < ORC_SUM || op > ORC_PROD) return ORC_E_ARG;
  if (n_descs == 0) return 0;
  if (!acc || !recv_stage || !descs || !seen) return ORC_E_ARG;
  const uint32_t es = (dtype == ORC_F32 || dtype == ORC_I32) ? 4u : 2u;
  int64_t applied = 0;
  for (uint64_t k = 0; k < n_descs; ++k) { /* array order = arrival order */
    const orc_desc* d = &descs[k];
    int64_t rc = check_record(d, acc_bytes, out_bytes, out_stage != NULL, recv_bytes, n_bits, es);
    if (rc) return rc;
    if (seen[d->seq]) continue; /* a retransmitted copy of a chunk already applied: drop */
    seen[d->seq] = 1;
    ++applied;
    const uint64_t n = d->len / es;
    const int fwd = d->out_off != ORC_NO_FORWARD;
    const int keep = !(fwd && (d->out_off & ORC_FORWARD_ONLY)); /* write the result back to acc */
    const uint64_t out_at = d->out_off & ~ORC_FORWARD_ONLY;
    if (dtype == ORC_F32) {
      const float* r = (const float*)((const char*)recv_stage + d->src_off);
      float* a = (float*)((char*)acc + d->dst_off);
      float* o = fwd ? (float*)((char*)out_stage + out_at) : NULL;
      for (uint64_t i = 0; i < n; ++i) {
        float t = orc_combine_f32(a[i], r[i], op);
        if (keep) a[i] = t;
        if (fwd) o[i] = t;
      }
    } else if (dtype == ORC_I32) {
      const int32_t* r = (const int32_t*)((const char*)recv_stage + d->src_off);
      int32_t* a = (int32_t*)((char*)acc + d->dst_off);
      int32_t* o = fwd ? (int32_t*)((char*)out_stage + out_at) : NULL;
      for (uint64_t i = 0; i < n; ++i) {
        int32_t t = orc_combine_i32(a[i], r[i], op);
        if (keep) a[i] = t;
        if (fwd) o[i] = t;
      }
    } else {
      const uint16_t* r = (const uint16_t*)((const char*)recv_stage + d->src_off);
      uint16_t* a = (uint16_t*)((char*)acc + d->dst_off);
      uint16_t* o = fwd ? (uint16_t*)((char*)out_stage + out_at) : NULL;
      for (uint64_t i = 0; i < n; ++i) {
        uint16_t t = dtype == ORC_BF16 ? orc_combine_bf16(a[i], r[i], op) : orc_combine_f16(a[i], r[i], op);
        if (keep) a[i] = t;
        if (fwd) o[i] = t;
      }
    }
  }
  return applied;
}

int64_t orc_reduce_gather(void* acc, uint64_t acc_bytes, void* out_stage, uint64_t out_bytes,
                          const void* recv_stage, uint64_t recv_bytes, const orc_gather_desc* descs,
                          uint64_t n_descs, uint8_t* seen, uint64_t n_bits, int dtype, int op) {
  if (dtype < ORC_F32 || dtype > ORC_I32) return ORC_E_ARG;
  if (op != ORC_SUM && op != ORC_MAX && op != ORC_MIN && op != ORC_PROD) return ORC_E_ARG;
  if (n_descs == 0) return 0;
  if (!acc || !recv_stage || !descs || !seen) return ORC_E_ARG;
  const uint32_t es = (dtype == ORC_F32 || dtype == ORC_I32) ? 4u : 2u;
  int64_t applied = 0;
  for (uint64_t k = 0; k < n_descs; ++k) {
    const orc_gather_desc* d = &descs[k];
    if (d->n_src < 1 || d->n_src > ORC_MAX_SOURCES) return ORC_E_ARG;
    for (uint32_t j = 0; j < d->n_src; ++j) { /* every source slot obeys the single-source rules */
      orc_desc one = {d->src_off[j], d->dst_off, d->out_off, d->len, d->seq};
      int64_t rc = check_record(&one, acc_bytes, out_bytes, out_stage != NULL, recv_bytes, n_bits, es);
      if (rc) return rc;
    }
    if (seen[d->seq]) continue;
    seen[d->seq] = 1;
    ++applied;
    const uint64_t n = d->len / es;
    const int fwd = d->out_off != ORC_NO_FORWARD;
    const int keep = !(fwd && (d->out_off & ORC_FORWARD_ONLY));
    const uint64_t out_at = d->out_off & ~ORC_FORWARD_ONLY;
    for (uint64_t i = 0; i < n; ++i) {
      if (dtype == ORC_F32) {
        float* a = (float*)((char*)acc + d->dst_off) + i;
        float t = *a;
        for (uint32_t j = 0; j < d->n_src; ++j)
          t = orc_combine_f32(t, ((const float*)((const char*)recv_stage + d->src_off[j]))[i], op);
        if (keep) *a = t;
        if (fwd) ((float*)((char*)out_stage + out_at))[i] = t;
      } else if (dtype == ORC_I32) {
        int32_t* a = (int32_t*)((char*)acc + d->dst_off) + i;
        int32_t t = *a;
        for (uint32_t j = 0; j < d->n_src; ++j)
          t = orc_combine_i32(t, ((const int32_t*)((const char*)recv_stage + d->src_off[j]))[i], op);
        if (keep) *a = t;
        if (fwd) ((int32_t*)((char*)out_stage + out_at))[i] = t;
      } else {
        uint16_t* a = (uint16_t*)((char*)acc + d->dst_off) + i;
        uint16_t t;
        if (op == ORC_SUM || op == ORC_PROD) { /* binary32 running value, one rounding at the end */
          float f = dtype == ORC_BF16 ? bf16_widen(*a) : orc_f16_to_f32(*a);
          for (uint32_t j = 0; j < d->n_src; ++j) {
            uint16_t r = ((const uint16_t*)((const char*)recv_stage + d->src_off[j]))[i];
            float fr = dtype == ORC_BF16 ? bf16_widen(r) : orc_f16_to_f32(r);
            f = op == ORC_SUM ? f + fr : f * fr;
          }
          t = dtype == ORC_BF16 ? orc_f32_to_bf16(f) : orc_f32_to_f16(f);
        } else {
          t = *a;
          for (uint32_t j = 0; j < d->n_src; ++j) {
            uint16_t r = ((const uint16_t*)((const char*)recv_stage + d->src_off[j]))[i];
            t = dtype == ORC_BF16 ? orc_combine_bf16(t, r, op) : orc_combine_f16(t, r, op);
          }
        }
        if (keep) *a = t;
        if (fwd) ((uint16_t*)((char*)out_stage + out_at))[i] = t;
      }
    }
  }
  return applied;
}

int64_t orc_scatter(void* dst, uint64_t dst_bytes, const void* recv_stage, uint64_t recv_bytes,
                    const orc_desc* descs, uint64_t n_descs, uint8_t* seen, uint64_t n_bits) {
  if (n_descs == 0) return 0;
  if (!dst || !recv_stage || !descs || !seen) return ORC_E_ARG;
  int64_t applied = 0;
  for (uint64_t k = 0; k < n_descs; ++k) {
    const orc_desc* d = &descs[k];
    if (d->out_off != ORC_NO_FORWARD) return ORC_E_ARG; /* a scatter never forwards */
    int64_t rc = check_record(d, dst_bytes, 0, 0, recv_bytes, n_bits, 1u);
    if (rc) return rc;
    if (seen[d->seq]) continue;
    seen[d->seq] = 1;
    ++applied;
    const unsigned char* r = (const unsigned char*)recv_stage + d->src_off;
    unsigned char* a = (unsigned char*)dst + d->dst_off;
    for (uint64_t i = 0; i < d->len; ++i) a[i] = r[i];
  }
  return applied;
}

void orc_pack_bitmap(const uint8_t* seen, uint64_t n_bits, uint32_t* words) {
  uint64_t nw = (n_bits + 31) / 32;
  for (uint64_t w = 0; w < nw; ++w) words[w] = 0;
  for (uint64_t s = 0; s < n_bits; ++s)
    if (seen[s]) words[s >> 5] |= (uint32_t)1 << (s & 31);
}

/* One pass over the bits, in order. */
void orc_ack_report(const uint32_t* words, uint64_t n_bits, uint64_t* cum_ack, uint64_t* n_applied,
                    uint32_t* n_ranges, uint64_t* ranges, uint32_t max_ranges) {
  uint64_t first_clear = n_bits, count = 0, run_start = 0;
  uint32_t runs = 0;
  int in_run = 0;
  for (uint64_t s = 0; s <= n_bits; ++s) {
    int bit = s < n_bits ? (int)((words[s >> 5] >> (s & 31)) & 1u) : 0; /* a clear bit past the end closes a run */
    if (bit) {
      ++count;
      if (!in_run) { in_run = 1; run_start = s; }
    } else {
      if (s < n_bits && first_clear == n_bits) first_clear = s;
      if (in_run) {
        in_run = 0;
        if (run_start > 0) { /* the run that begins at bit 0 is the cumulative part */
          if (runs < max_ranges) { ranges[2 * runs] = run_start; ranges[2 * runs + 1] = s; }
          ++runs;
        }
      }
    }
  }
  *cum_ack = first_clear;
  *n_applied = count;
  *n_ranges = runs;
}

void orc_message_status(uint32_t* words, const uint32_t* n_chunks, uint32_t n_slots,
                        uint32_t bits_per_slot, uint32_t* out4, int recycle) {
  for (uint32_t i = 0; i < n_slots; ++i) {
    const uint64_t base = (uint64_t)i * bits_per_slot;
    uint32_t limit = n_chunks[i] == 0 ? bits_per_slot : n_chunks[i];
    if (limit > bits_per_slot) limit = bits_per_slot;
    uint32_t first_clear = limit, count = 0;
    for (uint32_t b = 0; b < limit; ++b) {
      const uint64_t s = base + b;
      if ((words[s >> 5] >> (s & 31)) & 1u) ++count;
      else if (first_clear == limit) first_clear = b;
    }
    const uint32_t complete = (n_chunks[i] != 0 && count == limit) ? 1u : 0u;
    out4[4 * i + 0] = first_clear;
    out4[4 * i + 1] = count;
    out4[4 * i + 2] = complete;
    out4[4 * i + 3] = 0;
    if (recycle && complete)
      for (uint32_t b = 0; b < bits_per_slot; ++b) {
        const uint64_t s = base + b;
        words[s >> 5] &= ~(1u << (s & 31));
      }
  }
}

/* ---- sender side: tensor buffer -> staged chunks + send records ---------------- */

int64_t orc_segment(void* stage, uint64_t stage_bytes, const void* tensor, uint64_t tensor_bytes,
                    uint64_t tensor_off, uint64_t bytes, uint32_t chunk_bytes, uint64_t stage_off,
                    uint64_t slot_stride, orc_send_desc* descs, uint32_t conn_id, uint32_t msg_id,
                    uint32_t first_csn) {
  if (conn_id > 255u || msg_id > 127u) return ORC_E_ARG;
  if (chunk_bytes == 0u || (chunk_bytes & 15u) || (tensor_off & 15u) || (stage_off & 15u) || (slot_stride & 15u))
    return ORC_E_ALIGN;
  if (bytes == 0) return 0;
  if (!stage || !tensor) return ORC_E_ARG;
  if (slot_stride < chunk_bytes) return ORC_E_BOUNDS; /* slots would overlap */
  if (!range_ok(tensor_off, bytes, tensor_bytes)) return ORC_E_BOUNDS;
  const uint64_t n = (bytes + chunk_bytes - 1) / chunk_bytes;
  const uint64_t last_len = bytes - (n - 1) * chunk_bytes;
  if (stage_off > stage_bytes || (n - 1) > (stage_bytes - stage_off) / slot_stride ||
      !range_ok(stage_off + (n - 1) * slot_stride, last_len, stage_bytes))
    return ORC_E_BOUNDS;
  for (uint64_t i = 0; i < n; ++i) {
    const uint64_t len = i + 1 < n ? chunk_bytes : last_len;
    const unsigned char* from = (const unsigned char*)tensor + tensor_off + i * chunk_bytes;
    unsigned char* to = (unsigned char*)stage + stage_off + i * slot_stride;
    for (uint64_t b = 0; b < len; ++b) to[b] = from[b];
    if (descs) {
      const uint64_t number = (uint64_t)first_csn + i; /* position in the run of chunks of this connection */
      const uint32_t csn = (uint32_t)(number % 256u);
      const uint32_t msg = (uint32_t)((msg_id + number / 256u) % 128u);
      const uint32_t mark = (csn == 255u || i + 1 == n) ? 1u : 0u;
      descs[i].stage_off = stage_off + i * slot_stride;
      descs[i].len = (uint32_t)len;
      descs[i].header = csn | (mark << 8) | (msg << 9) | (conn_id << 16);
    }
  }
  return (int64_t)n;
}

/* ---- whole-call preconditions ---------------------------------------------- */

typedef struct { uint64_t key, end; uint64_t idx; } ivl;

static int cmp_ivl(const void* x, const void* y) {
  const ivl* a = (const ivl*)x; const ivl* b = (const ivl*)y;
  if (a->key != b->key) return a->key < b->key ? -1 : 1;
  if (a->idx != b->idx) return a->idx < b->idx ? -1 : 1;
  return 0;
}

int64_t orc_check_call(const void* recv_stage, uint64_t recv_bytes, const orc_desc* descs,
                       uint64_t n_descs) {
  if (n_descs == 0) return 0;
  ivl* v = (ivl*)malloc(sizeof(ivl) * n_descs);
  if (!v) return ORC_E_ARG;
  int64_t rc = 0;
  /* records of one seq must agree in every field and in payload bytes */
  for (uint64_t k = 0; k < n_descs; ++k) { v[k].key = descs[k].seq; v[k].end = 0; v[k].idx = k; }
  qsort(v, n_descs, sizeof(ivl), cmp_ivl);
  uint64_t n_rep = 0;
  for (uint64_t k = 0; k < n_descs && !rc; ++k) {
    const orc_desc* d = &descs[v[k].idx];
    if (!range_ok(d->src_off, d->len, recv_bytes)) { rc = ORC_E_BOUNDS; break; }
    if (k > 0 && v[k - 1].key == v[k].key) {
      const orc_desc* p = &descs[v[k - 1].idx];
      if (p->dst_off != d->dst_off || p->out_off != d->out_off || p->len != d->len ||
          memcmp((const char*)recv_stage + p->src_off, (const char*)recv_stage + d->src_off, d->len))
        rc = ORC_E_MISMATCH;
    } else {
      v[n_rep++].idx = v[k].idx; /* keep one representative per seq (k >= n_rep always) */
    }
  }
  /* representatives must not overlap in acc, nor in out_stage */
  for (int pass = 0; pass < 2 && !rc; ++pass) {
    ivl* w = (ivl*)malloc(sizeof(ivl) * (n_rep ? n_rep : 1));
    if (!w) { rc = ORC_E_ARG; break; }
    uint64_t m = 0;
    for (uint64_t k = 0; k < n_rep; ++k) {
      const orc_desc* d = &descs[v[k].idx];
      if (d->len == 0) continue;
      uint64_t off = pass == 0 ? d->dst_off : d->out_off;
      if (pass == 1 && off == ORC_NO_FORWARD) continue;
      if (pass == 1) off &= ~ORC_FORWARD_ONLY;
      w[m].key = off; w[m].end = off + d->len; w[m].idx = k; ++m;
    }
    qsort(w, m, sizeof(ivl), cmp_ivl);
    for (uint64_t k = 1; k < m; ++k)
      if (w[k].key < w[k - 1].end) { rc = ORC_E_OVERLAP; break; }
    free(w);
  }
  free(v);
  return rc;
}

/* ---- textbook ring allreduce ------------------------------------------------- */

/* R ranks in a ring, buffer of n elements cut into R equal segments.  In
 * reduce-scatter step s rank r combines into its own segment (r-s-1) mod R what
 * rank r-1 held for that segment before the step; after R-1 steps rank r holds
 * the complete result of segment (r+1) mod R.  In allgather step s rank r
 * overwrites segment (r-s) mod R with rank r-1's copy.  All ranks step together,
 * so each step reads a snapshot of the previous state. */
int orc_ring_allreduce(const void* x, uint32_t R, uint64_t n, int dtype, int op, void* result) {
  if (!x || !result || R == 0 || n % R) return ORC_E_ARG;
  if (dtype < ORC_F32 || dtype > ORC_I32) return ORC_E_ARG;
  if (op != ORC_SUM && op != ORC_MAX && op != ORC_MIN && op != ORC_PROD) return ORC_E_ARG;
  const uint32_t es = (dtype == ORC_F32 || dtype == ORC_I32) ? 4u : 2u;
  const uint64_t seg = n / R, total = (uint64_t)R * n * es;
  char* cur = (char*)result;
  memcpy(cur, x, total);
  if (R == 1) return 0;
  char* prev = (char*)malloc(total);
  if (!prev) return ORC_E_ARG;
  for (uint32_t phase = 0; phase < 2; ++phase) {
    for (uint32_t s = 0; s + 1 < R; ++s) {
      memcpy(prev, cur, total);
      for (uint32_t r = 0; r < R; ++r) {
        uint32_t left = (r + R - 1) % R;
        uint32_t j = phase == 0 ? (r + 2 * R - s - 1) % R : (r + R - s) % R;
        for (uint64_t i = j * seg; i < (j + 1) * seg; ++i) {
          if (dtype == ORC_F32) {
            float mine = ((float*)prev)[r * n + i], got = ((float*)prev)[left * n + i];
            ((float*)cur)[r * n + i] = phase == 0 ? orc_combine_f32(mine, got, op) : got;
          } else if (dtype == ORC_I32) {
            int32_t mine = ((int32_t*)prev)[r * n + i], got = ((int32_t*)prev)[left * n + i];
            ((int32_t*)cur)[r * n + i] = phase == 0 ? orc_combine_i32(mine, got, op) : got;
          } else {
            uint16_t mine = ((uint16_t*)prev)[r * n + i], got = ((uint16_t*)prev)[left * n + i];
            uint16_t t = dtype == ORC_BF16 ? orc_combine_bf16(mine, got, op) : orc_combine_f16(mine, got, op);
            ((uint16_t*)cur)[r * n + i] = phase == 0 ? t : got;
          }
        }
      }
    }
  }
  free(prev);
  return 0;
}
