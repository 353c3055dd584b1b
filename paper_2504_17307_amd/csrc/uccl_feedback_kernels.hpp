// Kernels that read the dedup bitmap back for the control path: acknowledgement report and
// per-message window status.  Internal to the library: included by uccl_chunk.hip only.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

// Receiver feedback from the dedup bitmap: cumulative acknowledgement (first clear bit),
// number of applied chunks, and the runs of set bits above the cumulative point in
// ascending order (what a selective-acknowledgement option would carry).  The bitmap is tiny
// next to the payload (one bit per chunk), so this is a latency problem, not a bandwidth one:
// one 1024-thread workgroup, one launch, no atomics in global memory.
//
// Each of the 16 wavefronts owns one contiguous sixteenth of the words and walks it 256 words at
// a time: lane l takes words 4l .. 4l+3 of the step with one 128-bit load (a compute unit issues
// a wavefront's load in the same time whether a lane asks for 4 or 16 bytes, so this is what
// bounds the walk).  A word's run starts (bit set, previous bit clear) and run ends (bit set,
// next bit clear) come from two word-wide shifts and the edge bits of the neighbouring words:
// the lane's own, the next lane's (shuffle), or, at the step's edges, the previous step's last
// word and one look-ahead word.  First walk: every wavefront counts its starts and set bits and
// finds its first clear bit; no barrier inside the walk.  One barrier; the counts of the
// wavefronts before it give each wavefront the ordinal of its first start, and of its first end
// (the same, less one if a run is open where the wavefront's words begin).
// Second walk (only if a range is to be written): a wavefront-wide prefix sum per step, by lane
// shuffles, gives every start and end its ordinal, so the k-th start and the k-th end land in
// the same output pair.
struct AckHeader {
  uint64_t cum_ack, n_applied;
  uint32_t n_ranges, complete;
  uint64_t reserved;
};

constexpr int kAckBatch = 12;         // steps whose loads are issued together (1.5 M bits in one go)
constexpr uint32_t kAckStep = 256;    // words per wavefront and step

// Words w .. w+3 (0 for words at and beyond n_words); `aligned`: the bitmap starts on a 16-byte
// boundary (w is always a multiple of 4), so a full group is one 128-bit load.
__device__ __forceinline__ uint4 ack_load4(const uint32_t* __restrict__ bitmap, uint64_t w, uint64_t n_words,
                                           bool aligned) {
  uint4 v = make_uint4(0u, 0u, 0u, 0u);
  if (aligned && w + 4 <= n_words) {
    v = *reinterpret_cast<const uint4*>(bitmap + w);
  } else {
    if (w < n_words) v.x = bitmap[w];
    if (w + 1 < n_words) v.y = bitmap[w + 1];
    if (w + 2 < n_words) v.z = bitmap[w + 2];
    if (w + 3 < n_words) v.w = bitmap[w + 3];
  }
  return v;
}

// Bits of word w that lie inside the bitmap.
__device__ __forceinline__ uint32_t ack_mask(uint64_t w, uint64_t n_bits) {
  const uint64_t lo = w * 32;
  return n_bits >= lo + 32 ? ~0u : (n_bits > lo ? (1u << (n_bits - lo)) - 1u : 0u);
}

// One lane's four words of a step, masked, with their run starts and run ends.
struct AckQuad {
  uint32_t word[4], starts[4], ends[4], mask[4];
};

// raw: the lane's words w4 .. w4+3; before: the word just below the step (0 if none); after: the
// word just above it (0 if none).  Neighbouring lanes exchange their edge words by shuffle.
// FULL: every word of the step lies wholly inside the bitmap (all steps but the last of a bitmap):
// no masks to compute.  The whole workgroup's arithmetic runs on one compute unit, so the walk is
// bound by instructions per word, not by memory.
// ENDS: also compute the run ends (the counting walk needs only the starts).
template <bool FULL, bool ENDS>
__device__ __forceinline__ AckQuad ack_quad(uint4 raw, uint64_t w4, uint64_t n_bits, uint32_t before,
                                            uint32_t after, uint32_t lane) {
  AckQuad q;
  const uint32_t in[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    q.mask[j] = FULL ? ~0u : ack_mask(w4 + j, n_bits);
    q.word[j] = in[j] & q.mask[j];
  }
  uint32_t below = __shfl_up(q.word[3], 1, 64);   // the word under this lane's first
  if (lane == 0) below = before;
  uint32_t above = 0u;
  if constexpr (ENDS) {
    above = __shfl_down(q.word[0], 1, 64);  // the word over this lane's last
    if (lane == 63) above = after;
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const uint32_t prev = j == 0 ? below : q.word[j - 1];
    q.starts[j] = q.word[j] & ~((q.word[j] << 1) | (prev >> 31));
    if constexpr (ENDS) {
      const uint32_t next = j == 3 ? above : q.word[j + 1];
      q.ends[j] = q.word[j] & ~((q.word[j] >> 1) | (next << 31));
    } else {
      q.ends[j] = 0u;
    }
  }
  return q;
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
#pragma unroll
  for (uint32_t d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
  return v;
}

__global__ void __launch_bounds__(1024) ack_report_kernel(const uint32_t* __restrict__ bitmap,
                                                          uint64_t n_bits, AckHeader* hdr,
                                                          uint64_t* ranges, uint32_t max_ranges) {
  __shared__ uint32_t s_starts[16];
  __shared__ unsigned long long s_applied[16], s_first_clear[16];
  const uint32_t tid = threadIdx.x, lane = tid & 63u;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint64_t n_words = (n_bits + 31) / 32;
  const uint64_t per_wave = (((n_words + 15) / 16) + kAckStep - 1) / kAckStep * kAckStep;  // whole steps
  const uint64_t w_lo = wave * per_wave;
  const uint64_t w_hi = w_lo + per_wave < n_words ? w_lo + per_wave : n_words;
  const bool aligned = (reinterpret_cast<uintptr_t>(bitmap) & 15u) == 0;
  // beyond the last word of the bitmap a masked word is 0, so the last run ends at n_bits by itself
  const uint32_t seg_before = (w_lo > 0 && w_lo < n_words) ? bitmap[w_lo - 1] : 0u;

  uint32_t my_starts = 0, my_applied = 0;
  unsigned long long my_first_clear = ~0ull;
  bool found = false;
  uint32_t before = seg_before;
  for (uint64_t wb = w_lo; wb < w_hi; wb += kAckStep * kAckBatch) {
    uint4 raw[kAckBatch];
#pragma unroll
    for (int i = 0; i < kAckBatch; ++i) {
      const uint64_t w0 = wb + static_cast<uint64_t>(i) * kAckStep;  // wavefront-uniform
      raw[i] = ack_load4(bitmap, w0 + 4 * lane, w0 < w_hi ? n_words : 0, aligned);
    }
#pragma unroll
    for (int i = 0; i < kAckBatch; ++i) {
      const uint64_t w0 = wb + static_cast<uint64_t>(i) * kAckStep;
      if (w0 < w_hi) {  // else the batch reaches past the wavefront's words (uniform)
        const uint64_t w4 = w0 + 4 * lane;
        const bool full = (w0 + kAckStep) * 32 <= n_bits;  // uniform
        const AckQuad q = full ? ack_quad<true, false>(raw[i], w4, n_bits, before, 0u, lane)
                               : ack_quad<false, false>(raw[i], w4, n_bits, before, 0u, lane);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          my_starts += __popc(q.starts[j]);
          my_applied += __popc(q.word[j]);
        }
        if (!found) {  // the lane's words ascend, so its first clear bit is the first it meets
#pragma unroll
          for (int j = 3; j >= 0; --j) {
            const uint32_t clear = ~q.word[j] & q.mask[j];
            if (clear != 0u) { my_first_clear = (w4 + j) * 32 + (__ffs(clear) - 1); found = true; }
          }
        }
        before = __shfl(q.word[3], 63, 64);  // the step's last word
      }
    }
  }
  my_starts = wave_sum(my_starts);
  const uint32_t app_lo = wave_sum(static_cast<uint32_t>(my_applied & 0xFFFFFu));   // per lane < 2^35 set bits:
  const uint32_t app_hi = wave_sum(static_cast<uint32_t>(my_applied >> 20));        // both halves fit 32-bit sums
#pragma unroll
  for (uint32_t d = 32; d >= 1; d >>= 1) {
    const uint32_t lo = __shfl_xor(static_cast<uint32_t>(my_first_clear), d, 64);
    const uint32_t hi = __shfl_xor(static_cast<uint32_t>(my_first_clear >> 32), d, 64);
    const unsigned long long other = lo | (static_cast<unsigned long long>(hi) << 32);
    if (other < my_first_clear) my_first_clear = other;
  }
  if (lane == 0) {
    s_starts[wave] = my_starts;
    s_applied[wave] = static_cast<unsigned long long>(app_lo) + (static_cast<unsigned long long>(app_hi) << 20);
    s_first_clear[wave] = my_first_clear;
  }
  __syncthreads();

  uint32_t s_at = 0, n_starts = 0;
  unsigned long long applied = 0, first_clear = ~0ull;
  for (uint32_t v = 0; v < 16; ++v) {
    if (v < wave) s_at += s_starts[v];
    n_starts += s_starts[v];
    applied += s_applied[v];
    if (s_first_clear[v] < first_clear) first_clear = s_first_clear[v];
  }
  // ordinal 0 is the run that begins at bit 0, if there is one: that is the cumulative part,
  // not a selective range; `skip` shifts the ordinals accordingly
  const uint32_t skip = n_bits > 0 ? (bitmap[0] & 1u) : 0u;
  if (tid == 0) {
    hdr->cum_ack = first_clear == ~0ull ? n_bits : first_clear;
    hdr->n_applied = applied;
    hdr->n_ranges = n_starts - skip;
    hdr->complete = applied == n_bits ? 1u : 0u;
    hdr->reserved = 0;
  }
  if (max_ranges == 0u || n_starts <= skip) return;  // nothing to list: uniform over the workgroup

  // Every run that starts below this wavefront's first bit also ends below it, except one that is
  // still open there (the bit below and the first bit both set): ends before = starts before - open.
  uint32_t e_at = s_at;
  if (w_lo > 0 && w_lo < n_words) e_at -= (seg_before >> 31) & bitmap[w_lo] & ack_mask(w_lo, n_bits) & 1u;
  // ordinals only grow along the walk: once the next start and the next end both lie beyond the
  // ranges that are to be written, nothing further has to be looked at (uniform over the wavefront)
  const uint64_t beyond = static_cast<uint64_t>(skip) + max_ranges;
  before = seg_before;
  for (uint64_t wb = w_lo; wb < w_hi && (s_at < beyond || e_at < beyond); wb += kAckStep * kAckBatch) {
    uint4 raw[kAckBatch];
    uint32_t after[kAckBatch];
#pragma unroll
    for (int i = 0; i < kAckBatch; ++i) {
      const uint64_t w0 = wb + static_cast<uint64_t>(i) * kAckStep;
      raw[i] = ack_load4(bitmap, w0 + 4 * lane, w0 < w_hi ? n_words : 0, aligned);
    }
#pragma unroll
    for (int i = 0; i < kAckBatch; ++i) {  // the word just above step i: the next step's first, if this batch holds it
      const uint64_t up = wb + static_cast<uint64_t>(i + 1) * kAckStep;
      if (i + 1 < kAckBatch && up < w_hi) after[i] = __shfl(raw[i + 1 < kAckBatch ? i + 1 : i].x, 0, 64);
      else after[i] = (up - kAckStep < w_hi && up < n_words) ? bitmap[up] : 0u;
    }
#pragma unroll
    for (int i = 0; i < kAckBatch; ++i) {
      const uint64_t w0 = wb + static_cast<uint64_t>(i) * kAckStep;
      if (w0 >= w_hi || (s_at >= beyond && e_at >= beyond)) continue;  // uniform
      const uint64_t w4 = w0 + 4 * lane;
      const AckQuad q = ack_quad<false, true>(raw[i], w4, n_bits, before, after[i], lane);
      before = __shfl(q.word[3], 63, 64);
      // starts in the low half, ends in the high half: at most 64 of each per lane, 4096 per step
      uint32_t mine = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) mine += __popc(q.starts[j]) | (static_cast<uint32_t>(__popc(q.ends[j])) << 16);
      uint32_t incl = mine;
#pragma unroll
      for (uint32_t d = 1; d < 64; d <<= 1) {
        const uint32_t below = __shfl_up(incl, d, 64);
        if (lane >= d) incl += below;
      }
      uint32_t ks = s_at + ((incl - mine) & 0xFFFFu), ke = e_at + ((incl - mine) >> 16);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        for (uint32_t m = q.starts[j]; m; m &= m - 1, ++ks)
          if (ks >= skip && ks - skip < max_ranges)
            ranges[2 * static_cast<uint64_t>(ks - skip)] = (w4 + j) * 32 + (__ffs(m) - 1);
        for (uint32_t m = q.ends[j]; m; m &= m - 1, ++ke)
          if (ke >= skip && ke - skip < max_ranges)
            ranges[2 * static_cast<uint64_t>(ke - skip) + 1] = (w4 + j) * 32 + (__ffs(m) - 1) + 1;
      }
      const uint32_t step_total = __shfl(incl, 63, 64);
      s_at += step_total & 0xFFFFu;
      e_at += step_total >> 16;
    }
  }
}

// Per-message window status (Section 3.1's message id / chunk sequence number / last-chunk
// mark): one wavefront per slot.  Lane l owns word l of the slot's window (a window is at
// most 64 words), masks it to the slot's limit, and the wavefront combines: a ballot of
// "has a clear bit below the limit" locates the first hole, a butterfly sum gives the
// applied count.  With `recycle`, the lanes of a complete slot store zeros over its window.
__global__ void __launch_bounds__(256) message_status_kernel(uint32_t* __restrict__ bitmap,
                                                             const uint32_t* __restrict__ n_chunks,
                                                             uint32_t n_slots, uint32_t words_per_slot,
                                                             uint4* __restrict__ status, uint32_t recycle) {
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t slot = blockIdx.x * 4u + (threadIdx.x >> 6);
  if (slot >= n_slots) return;  // whole wavefronts leave together; no barrier follows
  const uint32_t window = words_per_slot * 32u;
  const uint32_t known = n_chunks[slot];
  const uint32_t limit = known == 0u ? window : (known < window ? known : window);
  uint32_t* w = bitmap + static_cast<uint64_t>(slot) * words_per_slot + lane;
  uint32_t word = 0u, mask = 0u;
  if (lane < words_per_slot) {
    word = *w;
    const uint32_t lo = lane * 32u;
    mask = limit >= lo + 32u ? ~0u : (limit > lo ? (1u << (limit - lo)) - 1u : 0u);
  }
  const uint32_t clear = ~word & mask;
  const unsigned long long holes = __ballot(clear != 0u);
  uint32_t cum = limit;
  if (holes) {
    const int first = __ffsll(holes) - 1;
    cum = static_cast<uint32_t>(first) * 32u + static_cast<uint32_t>(__shfl(__ffs(clear) - 1, first, 64));
  }
  uint32_t count = __popc(word & mask);
#pragma unroll
  for (uint32_t d = 32; d >= 1; d >>= 1) count += __shfl_xor(count, d, 64);
  const uint32_t complete = (known != 0u && count == limit) ? 1u : 0u;
  if (lane == 0) status[slot] = make_uint4(cum, count, complete, 0u);
  if (recycle && complete && lane < words_per_slot) *w = 0u;
}

}  // namespace
