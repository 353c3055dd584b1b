// Kernels that read the dedup bitmap back for the control path: acknowledgement report and
// per-message window status.  Internal to the library: included by uccl_chunk.hip only.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

// Receiver feedback from the dedup bitmap: cumulative acknowledgement (first clear bit),
// number of applied chunks, and the runs of set bits above the cumulative point in
// ascending order (what a selective-acknowledgement option would carry).  One 1024-thread
// workgroup walks the words in order, 1024 words per round: thread i owns word i of the
// round, finds run starts (bit set, previous bit clear) and run ends (bit set, next bit
// clear) with two word-wide shifts, and a block-wide exclusive scan of the per-word counts
// gives every start and end its ordinal, so the k-th start and the k-th end land in the
// same output pair.  The bitmap is tiny next to the payload (one bit per chunk), so this is
// a latency problem, not a bandwidth one: one workgroup, no atomics, no second pass.
struct AckHeader {
  uint64_t cum_ack, n_applied;
  uint32_t n_ranges, complete;
  uint64_t reserved;
};

__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t tid, uint32_t* s_wave,
                                                         uint32_t* total) {
  uint32_t incl = v;
#pragma unroll
  for (uint32_t d = 1; d < 64; d <<= 1) {
    const uint32_t below = __shfl_up(incl, d, 64);
    if ((tid & 63u) >= d) incl += below;
  }
  if ((tid & 63u) == 63u) s_wave[tid >> 6] = incl;
  __syncthreads();
  uint32_t base = 0, sum = 0;
  for (uint32_t w = 0; w < 16; ++w) {
    const uint32_t x = s_wave[w];
    if (w < (tid >> 6)) base += x;
    sum += x;
  }
  __syncthreads();  // s_wave is reused by the next scan
  *total = sum;
  return base + incl - v;
}

__global__ void __launch_bounds__(1024) ack_report_kernel(const uint32_t* __restrict__ bitmap,
                                                          uint64_t n_bits, AckHeader* hdr,
                                                          uint64_t* ranges, uint32_t max_ranges) {
  __shared__ uint32_t s_wave[16];
  __shared__ unsigned long long s_first_clear;
  const uint32_t tid = threadIdx.x;
  const uint64_t n_words = (n_bits + 31) / 32;
  if (tid == 0) s_first_clear = ~0ull;
  __syncthreads();
  uint64_t applied = 0;      // per-thread partial popcount
  uint32_t starts_seen = 0;  // runs started / ended in earlier rounds (same in every thread)
  uint32_t ends_seen = 0;
  for (uint64_t w0 = 0; w0 < n_words; w0 += 1024) {
    const uint64_t w = w0 + tid;
    uint32_t word = 0, prev_msb = 0, next_lsb = 0;
    if (w < n_words) {
      word = bitmap[w];
      const uint64_t valid = n_bits - w * 32;  // bits of this word inside the bitmap
      if (valid < 32) word &= (1u << valid) - 1u;
      if (w > 0) prev_msb = bitmap[w - 1] >> 31;
      if (w + 1 < n_words) {
        uint32_t nx = bitmap[w + 1];
        const uint64_t nvalid = n_bits - (w + 1) * 32;
        if (nvalid < 32) nx &= (1u << nvalid) - 1u;
        next_lsb = nx & 1u;
      }
      applied += __popc(word);
      const uint32_t clear = ~word & (valid < 32 ? (1u << valid) - 1u : ~0u);
      if (clear) atomicMin(&s_first_clear, w * 32 + (__ffs(clear) - 1));  // LDS atomic
    }
    const uint32_t starts = word & ~((word << 1) | prev_msb);
    const uint32_t ends = word & ~((word >> 1) | (next_lsb << 31));
    uint32_t n_starts, n_ends;
    const uint32_t s_at = starts_seen + block_exclusive_scan(__popc(starts), tid, s_wave, &n_starts);
    const uint32_t e_at = ends_seen + block_exclusive_scan(__popc(ends), tid, s_wave, &n_ends);
    // ordinal 0 is the run that begins at bit 0, if there is one: that is the cumulative
    // part, not a selective range; `skip` shifts the ordinals accordingly
    const uint32_t skip = bitmap[0] & 1u;
    uint32_t k = s_at;
    for (uint32_t m = starts; m; m &= m - 1, ++k)
      if (k >= skip && k - skip < max_ranges) ranges[2 * (k - skip)] = w * 32 + (__ffs(m) - 1);
    k = e_at;
    for (uint32_t m = ends; m; m &= m - 1, ++k)
      if (k >= skip && k - skip < max_ranges) ranges[2 * (k - skip) + 1] = w * 32 + (__ffs(m) - 1) + 1;
    starts_seen += n_starts;
    ends_seen += n_ends;
  }
  // block-wide sum of the popcounts: 64-bit totals as two 32-bit scans would overflow only
  // beyond 2^32 set bits per thread-lane, impossible for n_bits < 2^42; keep it simple
  uint32_t tot_lo, tot_hi;
  block_exclusive_scan(static_cast<uint32_t>(applied & 0xFFFFFu), tid, s_wave, &tot_lo);
  block_exclusive_scan(static_cast<uint32_t>(applied >> 20), tid, s_wave, &tot_hi);
  if (tid == 0) {
    const uint64_t total = static_cast<uint64_t>(tot_lo) + (static_cast<uint64_t>(tot_hi) << 20);
    const uint64_t first_clear = s_first_clear == ~0ull ? n_bits : s_first_clear;
    const uint32_t skip = n_bits > 0 ? (bitmap[0] & 1u) : 0u;
    hdr->cum_ack = first_clear;
    hdr->n_applied = total;
    hdr->n_ranges = starts_seen - skip;
    hdr->complete = (total == n_bits) ? 1u : 0u;
    hdr->reserved = 0;
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
