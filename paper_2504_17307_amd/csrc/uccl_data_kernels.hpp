// Data-path kernels: dedup of a tile of records, the kernel that streams the winners (whole tiles
// per workgroup, or one record cut into parts over several workgroups), the multi-source fold,
// and the bitmap fill.  Internal to the library: included by uccl_chunk.hip only.
#pragma once

#include "uccl_chunk.h"
#include "uccl_elements.hpp"

// Tunable compile-time shape constants (defaults chosen by measurement on MI355X).
#ifndef UCCL_GATHER_UNROLL
#define UCCL_GATHER_UNROLL 2  // multi-sender reduce: vectors per lane per unit
#endif
#ifndef UCCL_GATHER_BATCH
#define UCCL_GATHER_BATCH 4   // and how many sources are loaded before the folds start
#endif
#ifndef UCCL_FLAT_THREADS
#define UCCL_FLAT_THREADS 1024  // workgroup size of chunk_flat_kernel
#endif
#ifndef UCCL_FLAT_UNROLL
#define UCCL_FLAT_UNROLL 2    // vectors per lane per unit: a unit is 64*U*16 bytes per stream
#endif
#ifndef UCCL_FLAT1_REDUCE_UNROLL
#define UCCL_FLAT1_REDUCE_UNROLL 1  // the same for one-record tiles of kernels that read the accumulator
#endif
#ifndef UCCL_FEW_THREADS
#define UCCL_FEW_THREADS 1024   // calls of few records: one workgroup per record
#endif
#ifndef UCCL_FEW_UNROLL
#define UCCL_FEW_UNROLL 4
#endif
#ifndef UCCL_PART_THREADS
#define UCCL_PART_THREADS 256   // workgroup size when one record is cut into parts
#endif
#ifndef UCCL_PART_UNROLL
#define UCCL_PART_UNROLL 2
#endif
#ifndef UCCL_XCD_CONTIGUOUS
#define UCCL_XCD_CONTIGUOUS 0   // 1: chunk_flat_kernel gives each of the 8 XCDs one contiguous eighth of the tiles
#endif
#ifndef UCCL_CLAIM_STRIDE
#define UCCL_CLAIM_STRIDE 16    // 64-bit words from one record's claim word to the next: one 128-byte line each
#endif
#ifndef UCCL_CLAIM_SPIN_LIMIT
#define UCCL_CLAIM_SPIN_LIMIT (1u << 16)  // polls of a claim word before a part gives up (see claim_await)
#endif
namespace {

struct Extents {
  uint64_t acc_bytes, out_bytes, recv_bytes, n_bits;
};

struct Args {
  char* acc;
  char* out;
  const char* recv;
  const uccl_chunk_desc* descs;
  uint32_t* bitmap;
  uint32_t* rejected;
  Extents ext;
  const uint32_t* n_ptr;  // optional: the record count is read from here (capped by n_descs)
  uint32_t n_descs;
  uint32_t allow_forward;
  // one record cut into `parts` workgroups (see claim_enter): claims[k] is record k's claim word,
  // tag is this call's own value, faults counts parts that gave up waiting for a decision
  unsigned long long* claims;
  uint32_t* faults;
  unsigned long long tag;
  uint32_t parts;
};

// ---- one record, several workgroups ------------------------------------------------------
//
// A call of few, large records (a 4 MiB message in 64 KiB chunks is 57 of them per phase) puts
// one workgroup per record on the machine, and a single compute unit moves its 4 x 64 KiB far
// below its share of the memory system's rate.  Such a call is launched with `parts` workgroups
// per record, and the record's units are dealt over the wavefronts of all of them.  The sequence
// number must still be decided exactly once, by one atomic OR on the bitmap, and every part that
// has units must learn the outcome.  Record k of the call has a 64-bit claim word in scratch
// memory, holding `tag * 4 + state`: the tag of the last call that used the word, and 0 = a part
// is deciding, 1 = applied, 2 = not applied.
//
//   enter    every part issues one atomic max of `tag * 4` on the word, after the payload loads of
//            its first unit (memory operations return in order, so entering earlier would hold up
//            the record itself).  Tags grow from call to call in the order the calls run (the host
//            draws the tag and enqueues the launch under one lock, and calls that share a word run
//            on one stream), so exactly one part of the call -- the first to get there -- finds an
//            older tag in the word: it decides.
//   decide   the deciding part issues the bitmap atomic (or rejects the record) and stores
//            `tag * 4 + outcome`.  It waits for nothing.
//   await    the other parts poll the word until it carries the call's tag and an outcome.
//
// A part only ever waits for a part that is already running and never waits itself, so the wait
// ends whatever order the hardware starts workgroups in.  It is bounded all the same: a part that
// gives up counts itself in `faults` and streams nothing.  Claim words are read and written with
// device-scope atomics only, so every part sees the one coherent copy whichever XCD it runs on;
// each record's word has a 128-byte line to itself (UCCL_CLAIM_STRIDE), because device-scope atomics
// on one line are served one after the other and a call's parts all arrive at about the same time
// (57 records x 8 parts: 6.2 us per call with the words packed, 5.4 us with a line each).
// Nothing is ever cleared between calls: a stale word is recognised by its older tag.
__device__ __forceinline__ unsigned long long claim_enter(unsigned long long* claim, unsigned long long tag) {
  return __hip_atomic_fetch_max(claim, tag << 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ bool claim_decides(unsigned long long entered, unsigned long long tag) {
  return (entered >> 2) < tag;
}

__device__ __forceinline__ void claim_publish(unsigned long long* claim, unsigned long long tag, bool win) {
  __hip_atomic_store(claim, (tag << 2) | (win ? 1ull : 2ull), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// `seen`: what this part's claim_enter returned (the outcome may already be in it).
__device__ __forceinline__ bool claim_await(unsigned long long* claim, unsigned long long seen,
                                            unsigned long long tag, uint32_t* faults) {
  for (uint32_t polls = 0; (seen >> 2) != tag || (seen & 3ull) == 0ull; ++polls) {
    if (polls >= UCCL_CLAIM_SPIN_LIMIT) {
      atomicAdd(faults, 1u);
      return false;
    }
    __builtin_amdgcn_s_sleep(1);
    seen = __hip_atomic_load(claim, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  return (seen & 3ull) == 1ull;
}

// The last len % 16 bytes of a chunk, element by element.
template <class Op, bool FWD, bool WB>
__device__ __forceinline__ void stream_tail(const char* r, char* a, char* o, uint32_t rem,
                                            uint32_t lane) {
  if constexpr (Op::kEs == 4) {
    if (lane < rem / 4) {
      uint32_t* ap = reinterpret_cast<uint32_t*>(a) + lane;
      const uint32_t t = Op::word(*ap, reinterpret_cast<const uint32_t*>(r)[lane]);
      if (WB) *ap = t;
      if (FWD) reinterpret_cast<uint32_t*>(o)[lane] = t;
    }
  } else if constexpr (Op::kEs == 2) {
    if (lane < rem / 2) {
      uint16_t* ap = reinterpret_cast<uint16_t*>(a) + lane;
      const uint32_t t = Op::half(*ap, reinterpret_cast<const uint16_t*>(r)[lane]);
      if (WB) *ap = static_cast<uint16_t>(t);
      if (FWD) reinterpret_cast<uint16_t*>(o)[lane] = static_cast<uint16_t>(t);
    }
  } else {
    if (lane < rem) {
      const char t = r[lane];
      if (WB) a[lane] = t;
      if (FWD) o[lane] = t;
    }
  }
}

// What a record must satisfy before its bit is touched (the unchecked entry points pass
// unbounded extents, which leaves alignment, granularity and the forward rules).
template <class Op>
__device__ __forceinline__ bool record_ok(const Args& g, uint64_t src, uint64_t dst, uint64_t out,
                                          uint32_t len, uint32_t seq) {
  const bool fwd = out != UCCL_NO_FORWARD;
  const uint64_t out_at = out & ~UCCL_FORWARD_ONLY;
  bool ok = seq < g.ext.n_bits && ((src | dst) & 15u) == 0 && len % Op::kEs == 0 &&
            src <= g.ext.recv_bytes && len <= g.ext.recv_bytes - src &&
            dst <= g.ext.acc_bytes && len <= g.ext.acc_bytes - dst;
  if (fwd)
    ok = ok && g.allow_forward && g.out != nullptr && (out_at & 15u) == 0 &&
         out_at <= g.ext.out_bytes && len <= g.ext.out_bytes - out_at;
  return ok;
}

// Winners of one tile of records, compacted; first[] is the exclusive prefix sum of
// their unit counts with the total in first[count].
template <int T>
struct Tile {
  uint64_t src[T], dst[T], out[T];
  uint32_t len[T];
  uint32_t first[T + 1];
  uint32_t count;
};

// Run by the first wavefront of a workgroup: lane i takes record tile*T + i, validates
// it, claims its sequence number, and the winners are compacted into LDS in record order.
// kUnitVecs > 0 also computes how many units of kUnitVecs 16-byte vectors each winner has.
template <int T, class Op, uint32_t kUnitVecs>
__device__ __forceinline__ void dedup_tile(const Args& g, Tile<T>& s, uint32_t tile, uint32_t tid) {
  static_assert(T >= 1 && T <= 64, "one wavefront dedups the tile");
  const uint64_t k = static_cast<uint64_t>(tile) * T + tid;
  bool win = false;
  uint64_t src = 0, dst = 0, out = 0;
  uint32_t len = 0;
  if (tid < T && k < g.n_descs) {  // inside the array's capacity: safe to load
    const u32x4* p = reinterpret_cast<const u32x4*>(g.descs + k);
    const u32x4 lo = p[0], hi = p[1];
    const uint32_t live = g.n_ptr != nullptr ? *g.n_ptr : g.n_descs;
    src = lo.x | (static_cast<uint64_t>(lo.y) << 32);
    dst = lo.z | (static_cast<uint64_t>(lo.w) << 32);
    out = hi.x | (static_cast<uint64_t>(hi.y) << 32);
    len = hi.z;
    const uint32_t seq = hi.w;
    const bool ok = record_ok<Op>(g, src, dst, out, len, seq);
    if (k >= live) {
      // beyond the published count: not a record at all, neither applied nor rejected
    } else if (ok) {
      const uint32_t bit = 1u << (seq & 31u);
      const uint32_t old = atomicOr(g.bitmap + (seq >> 5), bit);  // device scope, relaxed
      win = (old & bit) == 0;
    } else if (g.rejected != nullptr) {
      atomicAdd(g.rejected, 1u);
    }
  }
  const uint64_t winners = __ballot(win);
  const uint32_t pos = __popcll(winners & ((1ull << tid) - 1ull));
  const uint32_t count = __popcll(winners);
  if (win) {
    s.src[pos] = src;
    s.dst[pos] = dst;
    s.out[pos] = out;
    s.len[pos] = len;
  }
  if (tid == 0) s.count = count;
  if (kUnitVecs > 0) {
    // a partial last vector (len % 16 != 0) counts as a vector of its unit
    const uint32_t vecs = (len >> 4) + ((len & 15u) != 0u ? 1u : 0u);  // no overflow for len up to 2^32 - 1
    const uint32_t units = win ? (vecs + kUnitVecs - 1u) / kUnitVecs : 0u;
    uint32_t incl = units;
#pragma unroll
    for (uint32_t d = 1; d < 64; d <<= 1) {
      const uint32_t below = __shfl_up(incl, d, 64);
      if (tid >= d) incl += below;
    }
    if (win) s.first[pos] = incl - units;
    if (tid == 63) s.first[count] = incl;
  }
}

// One unit = 64*U consecutive 16-byte vectors of a chunk, streamed by one wavefront.
template <int U, class Op, bool FWD, bool WB>
__device__ __forceinline__ void stream_unit(const char* r, char* a, char* o, uint32_t len,
                                            uint32_t trip, uint32_t lane) {
  constexpr uint32_t kPolicy = cache_policy<Op, FWD, WB>();
  constexpr bool kNtRecv = (kPolicy & 8u) != 0, kNtOut = (kPolicy & 4u) != 0;
  constexpr bool kNtAccLoad = (kPolicy & 2u) != 0, kNtAccStore = (kPolicy & 1u) != 0;
  constexpr uint32_t kUnit = 64u * U;
  const uint32_t nvec = len >> 4;
  const uint32_t v0 = trip * kUnit;
  const u32x4* rp = reinterpret_cast<const u32x4*>(r) + v0 + lane;
  u32x4* ap = reinterpret_cast<u32x4*>(a) + v0 + lane;
  u32x4* op = reinterpret_cast<u32x4*>(o) + v0 + lane;
  if (v0 + kUnit <= nvec) {
    u32x4 rv[U], av[U];
#pragma unroll
    for (int u = 0; u < U; ++u) rv[u] = load16<kNtRecv>(rp + u * 64);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if constexpr (Op::kReadsAcc) av[u] = load16<kNtAccLoad>(ap + u * 64);
      else av[u] = rv[u];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const u32x4 t = combine<Op>(av[u], rv[u]);
      if (WB) store16<kNtAccStore>(ap + u * 64, t);
      if (FWD) store16<kNtOut>(op + u * 64, t);
    }
    return;
  }
  // last unit of the chunk: ragged
#pragma unroll
  for (int u = 0; u < U; ++u) {
    if (v0 + lane + u * 64 < nvec) {
      const u32x4 rv = load16<kNtRecv>(rp + u * 64);
      u32x4 av = rv;
      if constexpr (Op::kReadsAcc) av = load16<kNtAccLoad>(ap + u * 64);
      const u32x4 t = combine<Op>(av, rv);
      if (WB) store16<kNtAccStore>(ap + u * 64, t);
      if (FWD) store16<kNtOut>(op + u * 64, t);
    }
  }
  const uint32_t rem = len & 15u;
  if (rem) {  // nvec lies in this unit, or the chunk would have had one unit fewer
    const uint64_t off = static_cast<uint64_t>(nvec) << 4;
    stream_tail<Op, FWD, WB>(r + off, a + off, FWD ? o + off : o, rem, lane);
  }
}

// The winners' units are numbered consecutively across the tile and dealt round-robin to the
// wavefronts of the workgroup, so the machine sees the same stream whether a tile holds one
// 128 KiB chunk or thirty-two 4 KiB chunks.
template <int NT, int T, int U, class Op>
__global__ void __launch_bounds__(NT) chunk_flat_kernel(const Args g) {
  constexpr uint32_t kUnit = 64u * U;
  constexpr uint32_t kWaves = NT / 64;
  __shared__ Tile<T> s;
  const uint32_t tid = threadIdx.x;
  // Consecutive workgroups run on different XCDs (each with an L2 of its own) and take consecutive
  // tiles, so at any moment the whole chip works on one contiguous window of receive slots.  The
  // alternative, one contiguous eighth of the tiles per XCD, keeps records and bitmap words inside
  // one L2 but makes the chip work on eight distant windows at once: measured slower (build switch).
  uint32_t tile = blockIdx.x;
  if (UCCL_XCD_CONTIGUOUS) {
    const uint32_t per_xcd = (gridDim.x + 7u) / 8u;   // the launch has 8 * per_xcd workgroups
    tile = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
  }
  if (tid < 64) dedup_tile<T, Op, kUnit>(g, s, tile, tid);
  __syncthreads();

  const uint32_t count = s.count;
  const uint32_t total = s.first[count];
  const uint32_t wave = tid >> 6, lane = tid & 63u;
  for (uint32_t u = wave; u < total; u += kWaves) {
    uint32_t w = 0;
    if (T > 1) {
      const bool mine = lane < count && s.first[lane] <= u && u < s.first[lane + 1];
      w = __ffsll(static_cast<unsigned long long>(__ballot(mine))) - 1;  // exactly one lane
    }
    w = __builtin_amdgcn_readfirstlane(w);
    const uint32_t trip = u - __builtin_amdgcn_readfirstlane(s.first[w]);
    const uint64_t src = wave_uniform(s.src[w]);
    const uint64_t dst = wave_uniform(s.dst[w]);
    const uint64_t out = wave_uniform(s.out[w]);
    const uint32_t len = __builtin_amdgcn_readfirstlane(s.len[w]);
    if (out == UCCL_NO_FORWARD)
      stream_unit<U, Op, false, true>(g.recv + src, g.acc + dst, nullptr, len, trip, lane);
    else if (out & UCCL_FORWARD_ONLY)
      stream_unit<U, Op, true, false>(g.recv + src, g.acc + dst, g.out + (out & ~UCCL_FORWARD_ONLY), len, trip, lane);
    else
      stream_unit<U, Op, true, true>(g.recv + src, g.acc + dst, g.out + out, len, trip, lane);
  }
}

// ---- calls of few records --------------------------------------------------------------------
//
// A call of a few dozen records (a 4 MiB message in 64 KiB chunks is 57 of them per phase) cannot
// fill the machine; what it costs is one workgroup's chain of latencies: read the record, decide
// the sequence number (one atomic round trip), read the payload, write it.  This kernel shortens
// the chain instead of the stream: one record per workgroup (or per group of `parts` workgroups),
// every wavefront reads the record for itself and issues the loads of its first unit at once,
// while one lane decides the sequence number; after one barrier the winners combine and store
// what is already in registers.  A duplicate therefore costs its payload reads (never a write),
// which is why calls of many records, where duplicates are many and latency is hidden by the
// number of workgroups anyway, use chunk_flat_kernel.  PARTS: blockIdx.x = record * parts + part
// (see claim_enter).
template <int U, class Op, bool FWD, bool WB>
__device__ __forceinline__ void finish_unit(const u32x4 (&rv)[U], const u32x4 (&av)[U], u32x4* ap,
                                            u32x4* op, uint32_t first_vec, uint32_t nvec) {
  constexpr uint32_t kPolicy = cache_policy<Op, FWD, WB>();
  constexpr bool kNtOut = (kPolicy & 4u) != 0, kNtAccStore = (kPolicy & 1u) != 0;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    if (first_vec + u * 64 < nvec) {
      const u32x4 t = combine<Op>(Op::kReadsAcc ? av[u] : rv[u], rv[u]);
      if (WB) store16<kNtAccStore>(ap + u * 64, t);
      if (FWD) store16<kNtOut>(op + u * 64, t);
    }
  }
}

template <int NT, int U, class Op, bool PARTS>
__global__ void __launch_bounds__(NT) chunk_few_kernel(const Args g) {
  constexpr uint32_t kUnit = 64u * U;
  constexpr uint32_t kWaves = NT / 64;
  __shared__ uint32_t s_win;
  const uint32_t tid = threadIdx.x, wave = tid >> 6, lane = tid & 63u;
  const uint32_t k = PARTS ? blockIdx.x / g.parts : blockIdx.x;   // the launch has n_descs (* parts) workgroups
  const uint32_t part = PARTS ? blockIdx.x % g.parts : 0u;

  unsigned long long* const claim = PARTS ? g.claims + static_cast<size_t>(k) * UCCL_CLAIM_STRIDE : nullptr;

  // every lane reads the same 32 bytes: one request per wavefront
  const u32x4* p = reinterpret_cast<const u32x4*>(g.descs + k);
  const u32x4 lo = p[0], hi = p[1];
  const uint32_t live = g.n_ptr != nullptr ? *g.n_ptr : g.n_descs;
  const uint64_t src = wave_uniform(lo.x | (static_cast<uint64_t>(lo.y) << 32));
  const uint64_t dst = wave_uniform(lo.z | (static_cast<uint64_t>(lo.w) << 32));
  const uint64_t out = wave_uniform(hi.x | (static_cast<uint64_t>(hi.y) << 32));
  const uint32_t len = __builtin_amdgcn_readfirstlane(hi.z);
  const uint32_t seq = __builtin_amdgcn_readfirstlane(hi.w);
  const bool is_record = k < live;
  const bool ok = is_record && record_ok<Op>(g, src, dst, out, len, seq);

  const uint32_t nvec = len >> 4;
  const uint32_t vecs = nvec + ((len & 15u) != 0u ? 1u : 0u);
  const uint32_t total = (vecs + kUnit - 1u) / kUnit;
  const uint32_t stride = PARTS ? kWaves * g.parts : kWaves;
  const uint32_t u0 = part * kWaves + wave;
  const uint32_t first_vec = u0 * kUnit + lane;
  const bool have = ok && u0 < total;
  const bool part_has_units = ok && part * kWaves < total;  // uniform over the workgroup
  const u32x4* rp = reinterpret_cast<const u32x4*>(g.recv + src) + first_vec;
  u32x4* ap = reinterpret_cast<u32x4*>(g.acc + dst) + first_vec;
  u32x4 rv[U], av[U];
  if (have) {  // in bounds whether or not this record turns out to be the first arrival
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (first_vec + u * 64 < nvec) rv[u] = __builtin_nontemporal_load(rp + u * 64);
    if constexpr (Op::kReadsAcc) {
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (first_vec + u * 64 < nvec) av[u] = ap[u * 64];
    }
  }
  if (tid == 0) {
    uint32_t win = 0u;
    unsigned long long entered = 0ull;
    if constexpr (PARTS) entered = claim_enter(claim, g.tag);
    if (!PARTS || claim_decides(entered, g.tag)) {
      if (ok) {
        const uint32_t bit = 1u << (seq & 31u);
        win = (atomicOr(g.bitmap + (seq >> 5), bit) & bit) == 0u ? 1u : 0u;
      } else if (is_record && g.rejected != nullptr) {  // a rejected record is counted once: by the part that decides
        atomicAdd(g.rejected, 1u);
      }
      if constexpr (PARTS) claim_publish(claim, g.tag, win != 0u);
    } else if (part_has_units) {  // a part without units has nothing to wait for
      win = claim_await(claim, entered, g.tag, g.faults) ? 1u : 0u;
    }
    s_win = win;
  }
  __syncthreads();
  if (s_win != 0u) {
    const bool fwd = out != UCCL_NO_FORWARD;
    const bool relay = fwd && (out & UCCL_FORWARD_ONLY) != 0;
    char* o = g.out + (out & ~UCCL_FORWARD_ONLY);
    if (have) {
      u32x4* op = reinterpret_cast<u32x4*>(o) + first_vec;
      if (!fwd) finish_unit<U, Op, false, true>(rv, av, ap, op, first_vec, nvec);
      else if (relay) finish_unit<U, Op, true, false>(rv, av, ap, op, first_vec, nvec);
      else finish_unit<U, Op, true, true>(rv, av, ap, op, first_vec, nvec);
      const uint32_t rem = len & 15u;
      if (rem != 0u && nvec >= u0 * kUnit && nvec < (u0 + 1u) * kUnit) {  // the unit that holds the partial vector
        const uint64_t off = static_cast<uint64_t>(nvec) << 4;
        if (!fwd) stream_tail<Op, false, true>(g.recv + src + off, g.acc + dst + off, nullptr, rem, lane);
        else if (relay) stream_tail<Op, true, false>(g.recv + src + off, g.acc + dst + off, o + off, rem, lane);
        else stream_tail<Op, true, true>(g.recv + src + off, g.acc + dst + off, o + off, rem, lane);
      }
    }
    for (uint32_t u = u0 + stride; u < total; u += stride) {
      if (!fwd) stream_unit<U, Op, false, true>(g.recv + src, g.acc + dst, nullptr, len, u, lane);
      else if (relay) stream_unit<U, Op, true, false>(g.recv + src, g.acc + dst, o, len, u, lane);
      else stream_unit<U, Op, true, true>(g.recv + src, g.acc + dst, o, len, u, lane);
    }
  }
}

// ---- several sources per destination chunk ---------------------------------------------
//
// Section 2.1: the kernel reduces transport buffers "from multiple sender GPUs" into the
// tensor buffer.  A gather record names up to UCCL_MAX_SOURCES receive slots for one
// destination chunk; they are folded into the accumulator's value in the order listed, so
// the floating-point result is fixed by the record, not by arrival timing.  The accumulator
// is read and written once per chunk however many sources there are.  Same tile / unit
// dealing as chunk_flat_kernel; per unit a wavefront keeps the running value in registers
// (widened to binary32 for 16-bit types); sources are loaded in batches, all loads of a
// batch in flight before the folds, which then run in the listed order.
struct GatherArgs {
  char* acc;
  char* out;
  const char* recv;
  const uccl_gather_desc* descs;
  uint32_t* bitmap;
  uint32_t* rejected;
  Extents ext;
  uint32_t n_descs;
  // records cut into parts (chunk_gather_parts_kernel; see claim_enter)
  unsigned long long* claims;
  uint32_t* faults;
  unsigned long long tag;
  uint32_t parts;
};

// One unit (64 * U vectors from vector v0 on) of one destination chunk: the accumulator's value,
// the sources folded into it in the listed order (src[] in LDS), the result written back and / or
// forwarded.  Sources are loaded in batches, all loads of a batch issued before the folds.
template <int U, class Op>
__device__ __forceinline__ void gather_unit(const GatherArgs& g, uint64_t dst, uint64_t out, uint32_t len,
                                            uint32_t n_src, const uint64_t* src, uint32_t v0, uint32_t lane) {
  constexpr uint32_t kUnit = 64u * U;
  constexpr uint32_t kBatch = UCCL_GATHER_BATCH;
  const uint32_t nvec = len >> 4;
  const bool fwd = out != UCCL_NO_FORWARD;
  const bool keep = !(fwd && (out & UCCL_FORWARD_ONLY));
  u32x4* ap = reinterpret_cast<u32x4*>(g.acc + dst) + v0 + lane;
  u32x4* op = reinterpret_cast<u32x4*>(g.out + (out & ~UCCL_FORWARD_ONLY)) + v0 + lane;
  bool live[U];
  typename Op::State st[U][4];
#pragma unroll
  for (int i = 0; i < U; ++i) {
    live[i] = v0 + lane + i * 64 < nvec;
    u32x4 a = {0u, 0u, 0u, 0u};
    if (live[i]) a = ap[i * 64];
    st[i][0] = Op::open(a.x); st[i][1] = Op::open(a.y); st[i][2] = Op::open(a.z); st[i][3] = Op::open(a.w);
  }
  for (uint32_t j0 = 0; j0 < n_src; j0 += kBatch) {
    u32x4 rv[kBatch][U];
#pragma unroll
    for (uint32_t b = 0; b < kBatch; ++b) {
      if (j0 + b < n_src) {
        const u32x4* rp = reinterpret_cast<const u32x4*>(g.recv + wave_uniform(src[j0 + b])) + v0 + lane;
#pragma unroll
        for (int i = 0; i < U; ++i) {
          rv[b][i] = u32x4{0u, 0u, 0u, 0u};
          if (live[i]) rv[b][i] = __builtin_nontemporal_load(rp + i * 64);
        }
      }
    }
#pragma unroll
    for (uint32_t b = 0; b < kBatch; ++b) {
      if (j0 + b < n_src) {
#pragma unroll
        for (int i = 0; i < U; ++i) {
          Op::fold(st[i][0], rv[b][i].x); Op::fold(st[i][1], rv[b][i].y);
          Op::fold(st[i][2], rv[b][i].z); Op::fold(st[i][3], rv[b][i].w);
        }
      }
    }
  }
#pragma unroll
  for (int i = 0; i < U; ++i) {
    if (!live[i]) continue;
    u32x4 t;
    t.x = Op::close(st[i][0]); t.y = Op::close(st[i][1]); t.z = Op::close(st[i][2]); t.w = Op::close(st[i][3]);
    if (keep) ap[i * 64] = t;
    if (fwd) __builtin_nontemporal_store(t, op + i * 64);
  }
  // the last len % 16 bytes, element by element, by the unit that holds vector index nvec
  const uint32_t rem = len & 15u;
  if (rem && nvec >= v0 && nvec < v0 + kUnit && lane < rem / Op::kEs) {
    const uint64_t off = (static_cast<uint64_t>(nvec) << 4) + lane * Op::kEs;
    uint32_t a_el;
    if constexpr (Op::kEs == 4) a_el = *reinterpret_cast<const uint32_t*>(g.acc + dst + off);
    else a_el = *reinterpret_cast<const uint16_t*>(g.acc + dst + off);
    typename Op::State t = Op::open(a_el);
    for (uint32_t j = 0; j < n_src; ++j) {
      const char* rp = g.recv + wave_uniform(src[j]) + off;
      uint32_t r_el;
      if constexpr (Op::kEs == 4) r_el = *reinterpret_cast<const uint32_t*>(rp);
      else r_el = *reinterpret_cast<const uint16_t*>(rp);
      Op::fold(t, r_el);
    }
    const uint32_t res = Op::close(t);
    if constexpr (Op::kEs == 4) {
      if (keep) *reinterpret_cast<uint32_t*>(g.acc + dst + off) = res;
      if (fwd) *reinterpret_cast<uint32_t*>(g.out + (out & ~UCCL_FORWARD_ONLY) + off) = res;
    } else {
      if (keep) *reinterpret_cast<uint16_t*>(g.acc + dst + off) = static_cast<uint16_t>(res);
      if (fwd) *reinterpret_cast<uint16_t*>(g.out + (out & ~UCCL_FORWARD_ONLY) + off) = static_cast<uint16_t>(res);
    }
  }
}

template <int T>
struct GatherTile {
  uint64_t dst[T], out[T];
  uint64_t src[T][UCCL_MAX_SOURCES];
  uint32_t len[T], n_src[T];
  uint32_t first[T + 1];
  uint32_t count;
};

template <int NT, int T, int U, class Op>
__global__ void __launch_bounds__(NT) chunk_gather_kernel(const GatherArgs g) {
  static_assert(T >= 1 && T <= 64, "one wavefront dedups the tile");
  constexpr uint32_t kUnit = 64u * U;
  __shared__ GatherTile<T> s;
  const uint32_t tid = threadIdx.x;
  if (tid < 64) {
    const uint64_t k = static_cast<uint64_t>(blockIdx.x) * T + tid;
    bool win = false;
    uint64_t dst = 0, out = 0;
    uint32_t len = 0, n_src = 0;
    const uccl_gather_desc* d = g.descs + k;
    if (tid < T && k < g.n_descs) {
      const u32x4* p = reinterpret_cast<const u32x4*>(d);
      const u32x4 lo = p[0], hi = p[1];
      dst = lo.x | (static_cast<uint64_t>(lo.y) << 32);
      out = lo.z | (static_cast<uint64_t>(lo.w) << 32);
      len = hi.x;
      const uint32_t seq = hi.y;
      n_src = hi.z;
      const bool fwd = out != UCCL_NO_FORWARD;
      const uint64_t out_at = out & ~UCCL_FORWARD_ONLY;
      bool ok = seq < g.ext.n_bits && (dst & 15u) == 0 && len % Op::kEs == 0 && n_src >= 1 &&
                n_src <= UCCL_MAX_SOURCES && dst <= g.ext.acc_bytes && len <= g.ext.acc_bytes - dst;
      if (fwd)
        ok = ok && g.out != nullptr && (out_at & 15u) == 0 && out_at <= g.ext.out_bytes &&
             len <= g.ext.out_bytes - out_at;
      if (ok) {
        for (uint32_t j = 0; j < n_src; ++j) {
          const uint64_t so = d->src_off[j];
          ok = ok && (so & 15u) == 0 && so <= g.ext.recv_bytes && len <= g.ext.recv_bytes - so;
        }
      }
      if (ok) {
        const uint32_t bit = 1u << (seq & 31u);
        const uint32_t old = atomicOr(g.bitmap + (seq >> 5), bit);
        win = (old & bit) == 0;
      } else if (g.rejected != nullptr) {
        atomicAdd(g.rejected, 1u);
      }
    }
    const uint64_t winners = __ballot(win);
    const uint32_t pos = __popcll(winners & ((1ull << tid) - 1ull));
    const uint32_t count = __popcll(winners);
    if (win) {
      s.dst[pos] = dst;
      s.out[pos] = out;
      s.len[pos] = len;
      s.n_src[pos] = n_src;
      for (uint32_t j = 0; j < n_src; ++j) s.src[pos][j] = d->src_off[j];
    }
    if (tid == 0) s.count = count;
    const uint32_t vecs = (len >> 4) + ((len & 15u) != 0u ? 1u : 0u);  // no overflow for len up to 2^32 - 1
    const uint32_t units = win ? (vecs + kUnit - 1u) / kUnit : 0u;
    uint32_t incl = units;
#pragma unroll
    for (uint32_t dlt = 1; dlt < 64; dlt <<= 1) {
      const uint32_t below = __shfl_up(incl, dlt, 64);
      if (tid >= dlt) incl += below;
    }
    if (win) s.first[pos] = incl - units;
    if (tid == 63) s.first[count] = incl;
  }
  __syncthreads();

  const uint32_t count = s.count;
  const uint32_t total = s.first[count];
  const uint32_t wave = tid >> 6, lane = tid & 63u;
  for (uint32_t u = wave; u < total; u += NT / 64) {
    uint32_t w = 0;
    if (T > 1) {
      const bool mine = lane < count && s.first[lane] <= u && u < s.first[lane + 1];
      w = __ffsll(static_cast<unsigned long long>(__ballot(mine))) - 1;
    }
    w = __builtin_amdgcn_readfirstlane(w);
    const uint32_t v0 = (u - __builtin_amdgcn_readfirstlane(s.first[w])) * kUnit;
    gather_unit<U, Op>(g, wave_uniform(s.dst[w]), wave_uniform(s.out[w]), __builtin_amdgcn_readfirstlane(s.len[w]),
                       __builtin_amdgcn_readfirstlane(s.n_src[w]), s.src[w], v0, lane);
  }
}

// A call of few multi-source records: `parts` workgroups per record share its units (one compute
// unit reads a record's n + 1 streams far below its share of the memory system's rate: eight
// records of 128 KiB from seven senders take 25 us uncut).  The record's fate is decided once, by
// the first part to arrive (see claim_enter); blockIdx.x = record * parts + part.
template <int NT, int U, class Op>
__global__ void __launch_bounds__(NT) chunk_gather_parts_kernel(const GatherArgs g) {
  constexpr uint32_t kUnit = 64u * U;
  constexpr uint32_t kWaves = NT / 64;
  __shared__ uint64_t s_src[UCCL_MAX_SOURCES];
  __shared__ uint32_t s_win;
  const uint32_t tid = threadIdx.x, wave = tid >> 6, lane = tid & 63u;
  const uint32_t k = blockIdx.x / g.parts, part = blockIdx.x % g.parts;   // the launch has n_descs * parts workgroups
  const uccl_gather_desc* d = g.descs + k;
  const u32x4* p = reinterpret_cast<const u32x4*>(d);
  const u32x4 lo = p[0], hi = p[1];   // every lane reads the same 32 bytes
  const uint64_t dst = wave_uniform(lo.x | (static_cast<uint64_t>(lo.y) << 32));
  const uint64_t out = wave_uniform(lo.z | (static_cast<uint64_t>(lo.w) << 32));
  const uint32_t len = __builtin_amdgcn_readfirstlane(hi.x);
  const uint32_t seq = __builtin_amdgcn_readfirstlane(hi.y);
  const uint32_t n_src = __builtin_amdgcn_readfirstlane(hi.z);
  const uint32_t vecs = (len >> 4) + ((len & 15u) != 0u ? 1u : 0u);
  const uint32_t total = (vecs + kUnit - 1u) / kUnit;
  if (wave == 0) {
    const bool fwd = out != UCCL_NO_FORWARD;
    const uint64_t out_at = out & ~UCCL_FORWARD_ONLY;
    bool ok = seq < g.ext.n_bits && (dst & 15u) == 0 && len % Op::kEs == 0 && n_src >= 1 &&
              n_src <= UCCL_MAX_SOURCES && dst <= g.ext.acc_bytes && len <= g.ext.acc_bytes - dst;
    if (fwd)
      ok = ok && g.out != nullptr && (out_at & 15u) == 0 && out_at <= g.ext.out_bytes && len <= g.ext.out_bytes - out_at;
    bool src_ok = true;
    if (lane < UCCL_MAX_SOURCES && lane < n_src) {  // lane j checks and stages source j
      const uint64_t so = d->src_off[lane];
      s_src[lane] = so;
      src_ok = (so & 15u) == 0 && so <= g.ext.recv_bytes && len <= g.ext.recv_bytes - so;
    }
    ok = ok && __all(src_ok);
    if (lane == 0) {
      uint32_t win = 0u;
      unsigned long long* const claim = g.claims + static_cast<size_t>(k) * UCCL_CLAIM_STRIDE;
      const unsigned long long entered = claim_enter(claim, g.tag);
      if (claim_decides(entered, g.tag)) {
        if (ok) {
          const uint32_t bit = 1u << (seq & 31u);
          win = (atomicOr(g.bitmap + (seq >> 5), bit) & bit) == 0u ? 1u : 0u;
        } else if (g.rejected != nullptr) {
          atomicAdd(g.rejected, 1u);
        }
        claim_publish(claim, g.tag, win != 0u);
      } else if (ok && part * kWaves < total) {  // a part without units has nothing to wait for
        win = claim_await(claim, entered, g.tag, g.faults) ? 1u : 0u;
      }
      s_win = win;
    }
  }
  __syncthreads();
  if (s_win == 0u) return;   // uniform over the workgroup
  for (uint32_t u = part * kWaves + wave; u < total; u += kWaves * g.parts)
    gather_unit<U, Op>(g, dst, out, len, n_src, s_src, u * kUnit, lane);
}

// ---- sender side: tensor buffer -> staged chunks + send records --------------------------------
//
// Section 2.1: the kernel copies from the tensor buffer to the transport buffer the NIC sends
// from; Section 3.1: the sender CPU names each chunk's address and sends a 32-bit control header
// with it.  A dense copy: chunk i of the range goes to slot i of the staging buffer, cut into
// 2 KiB units (64 lanes x 2 x 16 bytes), one unit per wavefront, 16 per workgroup.  The wavefront
// that takes a chunk's first unit also writes the chunk's send record.  The tensor is read with
// default policy (it is the accumulator, read again by the next step), staging is written
// non-temporally (the NIC reads it, the GPU does not).
struct SegmentArgs {
  char* stage;
  const char* tensor;
  uccl_send_desc* descs;
  uint64_t bytes;        // length of the range (tensor already points at its start)
  uint64_t slot_stride;
  uint64_t stage_off;    // of slot 0, for the records (stage already points there)
  uint64_t n_chunks;
  uint32_t chunk_bytes;
  uint32_t units_per_chunk;
  uint32_t conn_id, msg_id, first_csn;
};

__global__ void __launch_bounds__(1024) segment_kernel(const SegmentArgs g) {
  constexpr uint32_t kUnit = 128u;  // 16-byte vectors per unit
  const uint32_t lane = threadIdx.x & 63u;
  const uint64_t unit = static_cast<uint64_t>(blockIdx.x) * 16u + (threadIdx.x >> 6);
  const uint64_t i = unit / g.units_per_chunk;           // chunk
  const uint32_t u = static_cast<uint32_t>(unit % g.units_per_chunk);
  if (i >= g.n_chunks) return;                            // whole wavefronts leave; no barrier follows
  const uint64_t from = i * g.chunk_bytes;
  const uint64_t left = g.bytes - from;
  const uint32_t len = left < g.chunk_bytes ? static_cast<uint32_t>(left) : g.chunk_bytes;
  if (u == 0 && lane == 0 && g.descs != nullptr) {
    const uint64_t number = static_cast<uint64_t>(g.first_csn) + i;
    const uint32_t csn = static_cast<uint32_t>(number & 255u);
    const uint32_t msg = static_cast<uint32_t>((g.msg_id + (number >> 8)) & 127u);
    const uint32_t mark = (csn == 255u || i + 1 == g.n_chunks) ? 1u : 0u;
    uccl_send_desc d;
    d.stage_off = g.stage_off + i * g.slot_stride;
    d.len = len;
    d.header = csn | (mark << 8) | (msg << 9) | (g.conn_id << 16);
    g.descs[i] = d;
  }
  const uint32_t nvec = len >> 4;
  const uint32_t v0 = u * kUnit;
  const u32x4* sp = reinterpret_cast<const u32x4*>(g.tensor + from) + v0 + lane;
  u32x4* dp = reinterpret_cast<u32x4*>(g.stage + i * g.slot_stride) + v0 + lane;
  u32x4 v[2];
#pragma unroll
  for (int k = 0; k < 2; ++k)
    if (v0 + lane + k * 64 < nvec) v[k] = sp[k * 64];
#pragma unroll
  for (int k = 0; k < 2; ++k)
    if (v0 + lane + k * 64 < nvec) __builtin_nontemporal_store(v[k], dp + k * 64);
  const uint32_t rem = len & 15u;  // the last, partial vector: byte by byte, by the unit that holds it
  if (rem != 0u && nvec >= v0 && nvec < v0 + kUnit && lane < rem) {
    const uint64_t at = (static_cast<uint64_t>(nvec) << 4) + lane;
    g.stage[i * g.slot_stride + at] = g.tensor[from + at];
  }
}

__global__ void __launch_bounds__(256) fill_words_kernel(uint32_t* p, uint64_t n, uint32_t v) {
  for (uint64_t i = static_cast<uint64_t>(blockIdx.x) * 256 + threadIdx.x; i < n;
       i += static_cast<uint64_t>(gridDim.x) * 256)
    p[i] = v;
}

}  // namespace
