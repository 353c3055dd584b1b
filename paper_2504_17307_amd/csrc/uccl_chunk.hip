// Receive-side chunk data path for multipath collectives, gfx950 (MI355X).
//
// One kernel does, per record of the arrival-ordered list the control path hands over
// (paper Section 3.1 "challenge of reassembly", Section 5): dedup by sequence number,
// place, combine with the tensor buffer (Section 2.1: "sum, max") or copy, write back,
// and forward to the outbound staging buffer.  The paper's own kernel first copies
// payloads into a transport buffer and then reduces; here the payload is read once,
// straight from its arrival slot, which gives the same result with 2x chunk size fewer
// bytes moved.
//
// Mapping onto the machine.  The work is a stream: at most one add per 4..8 bytes
// moved, so HBM bandwidth bounds it and no matrix core is involved.  A 1024-thread
// workgroup takes a tile of T consecutive records.  The lanes of its first wavefront each
// load one 32-byte record with two 128-bit loads, validate it, and test-and-set its bit
// with one device-scope atomic OR; the returned old word tells the lane whether it is the
// first arrival.  A wave ballot compacts the winners into LDS and a wave scan numbers
// their 2 KiB units.  After one barrier the 16 wavefronts take units round-robin and
// stream them with 128-bit loads and stores: every thread issues all its loads, then
// combines, then stores, and the workgroup retires.  Duplicates cost their record and one
// atomic, nothing else.  Two lanes holding the same seq each issue their own atomic, so
// the hardware serialises them and exactly one sees the bit clear.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include <atomic>
#include <new>
#include <tuple>
#include <utility>

#include "uccl_chunk.h"

// Tunable compile-time shape constants (defaults chosen by measurement on MI355X).
#ifndef UCCL_WAVE_TILE
#define UCCL_WAVE_TILE 4      // records per 256-thread workgroup, one wavefront per chunk
#endif
#ifndef UCCL_WAVE_UNROLL
#define UCCL_WAVE_UNROLL 4
#endif
#ifndef UCCL_WAVE_TILE_SMALL
#define UCCL_WAVE_TILE_SMALL 16  // same shape, used when a call carries very many records
#endif
#ifndef UCCL_GROUP_TILE
#define UCCL_GROUP_TILE 1     // records per workgroup, 256 threads per chunk
#endif
#ifndef UCCL_GROUP_UNROLL
#define UCCL_GROUP_UNROLL 4
#endif
#ifndef UCCL_GATHER_UNROLL
#define UCCL_GATHER_UNROLL 2  // multi-sender reduce: vectors per lane per unit
#endif
#ifndef UCCL_GATHER_BATCH
#define UCCL_GATHER_BATCH 4   // and how many sources are loaded before the folds start
#endif
#ifndef UCCL_FLAT_THREADS
#define UCCL_FLAT_THREADS 1024  // workgroup size of the flat shape
#endif
#ifndef UCCL_FLAT_UNROLL
#define UCCL_FLAT_UNROLL 2    // vectors per lane per unit: a unit is 64*U*16 bytes per stream
#endif
// Cache policy of the four streams, one 4-bit mask per kind of chunk (measured on
// MI355X with buffers too large to stay cache resident).  Bit 3: non-temporal load of the
// arrival slot; bit 2: non-temporal store of the staging copy; bit 1: non-temporal load
// of the accumulator; bit 0: non-temporal store of the accumulator.
#ifndef UCCL_POLICY_REDUCE_FWD
#define UCCL_POLICY_REDUCE_FWD 0xD   // slot read once, staging written once, acc line dropped after its write
#endif
#ifndef UCCL_POLICY_REDUCE_KEEP
#define UCCL_POLICY_REDUCE_KEEP 0x9
#endif
#ifndef UCCL_POLICY_COPY_FWD
#define UCCL_POLICY_COPY_FWD 0xC
#endif
#ifndef UCCL_POLICY_REDUCE_RELAY
#define UCCL_POLICY_REDUCE_RELAY 0xE  // forward-only: the accumulator is read once and not written
#endif
#ifndef UCCL_POLICY_COPY_RELAY
#define UCCL_POLICY_COPY_RELAY 0xC
#endif
#ifndef UCCL_POLICY_COPY_KEEP
#define UCCL_POLICY_COPY_KEEP 0x9
#endif

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <bool NT>
__device__ __forceinline__ u32x4 load16(const u32x4* p) {
  if constexpr (NT) return __builtin_nontemporal_load(p);
  else return *p;
}
template <bool NT>
__device__ __forceinline__ void store16(u32x4* p, u32x4 v) {
  if constexpr (NT) __builtin_nontemporal_store(v, p);
  else *p = v;
}

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
};

__device__ __forceinline__ float as_f32(uint32_t u) { return __uint_as_float(u); }
__device__ __forceinline__ uint32_t as_u32(float f) { return __float_as_uint(f); }

// binary32 -> bf16 bits, round to nearest even; a NaN keeps its top bits and is quieted.
__device__ __forceinline__ uint32_t round_bf16(float s) {
  const uint32_t u = as_u32(s);
  uint32_t h = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) h = (u >> 16) | 0x0040u;
  return h;
}

// Element operations.  word() combines one 32-bit word (one fp32 / int32, or two 16-bit
// elements side by side); half() one 16-bit element (tails).  a = tensor-buffer value,
// r = received value.  SUM and PROD compute in binary32 and round once to the storage
// type; MAX and MIN compare the (widened) values strictly and select one of the two
// inputs unchanged, the accumulator's on a tie or an unordered pair.
enum Kind { kSum = 0, kMax = 1, kMin = 2, kProd = 4 };

template <int K>
__device__ __forceinline__ float arith(float a, float r) {
  return K == kSum ? a + r : a * r;
}
template <int K>
__device__ __forceinline__ bool takes_received(float a, float r) {
  return K == kMax ? r > a : r < a;
}

struct WidenBF16 {
  static __device__ __forceinline__ float widen(uint32_t h) { return as_f32(h << 16); }
  static __device__ __forceinline__ uint32_t narrow(float f) { return round_bf16(f); }
};
// IEEE binary16 through the hardware converts (round to nearest even, subnormals kept).
struct WidenF16 {
  static __device__ __forceinline__ float widen(uint32_t h) {
    return static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(h)));
  }
  static __device__ __forceinline__ uint32_t narrow(float f) {
    return __builtin_bit_cast(uint16_t, static_cast<_Float16>(f));
  }
};

template <int K>
struct OpF32 {
  static constexpr bool kReadsAcc = true;
  static constexpr uint32_t kEs = 4;
  static __device__ __forceinline__ uint32_t word(uint32_t a, uint32_t r) {
    if constexpr (K == kSum || K == kProd) return as_u32(arith<K>(as_f32(a), as_f32(r)));
    else return takes_received<K>(as_f32(a), as_f32(r)) ? r : a;
  }
  // Folding several received words into one accumulator word, in the order given.
  struct State { uint32_t v; };
  static __device__ __forceinline__ State open(uint32_t a) { return State{a}; }
  static __device__ __forceinline__ void fold(State& t, uint32_t r) { t.v = word(t.v, r); }
  static __device__ __forceinline__ uint32_t close(const State& t) { return t.v; }
};

template <int K>
struct OpI32 {  // two's complement; SUM and PROD wrap modulo 2^32
  static constexpr bool kReadsAcc = true;
  static constexpr uint32_t kEs = 4;
  static __device__ __forceinline__ uint32_t word(uint32_t a, uint32_t r) {
    if constexpr (K == kSum) return a + r;
    else if constexpr (K == kProd) return a * r;
    else if constexpr (K == kMax) return static_cast<int32_t>(r) > static_cast<int32_t>(a) ? r : a;
    else return static_cast<int32_t>(r) < static_cast<int32_t>(a) ? r : a;
  }
  struct State { uint32_t v; };
  static __device__ __forceinline__ State open(uint32_t a) { return State{a}; }
  static __device__ __forceinline__ void fold(State& t, uint32_t r) { t.v = word(t.v, r); }
  static __device__ __forceinline__ uint32_t close(const State& t) { return t.v; }
};

template <int K, class W>
struct Op16 {
  static constexpr bool kReadsAcc = true;
  static constexpr uint32_t kEs = 2;
  static __device__ __forceinline__ uint32_t half(uint32_t a, uint32_t r) {  // low 16 bits
    if constexpr (K == kSum || K == kProd) return W::narrow(arith<K>(W::widen(a), W::widen(r)));
    else return takes_received<K>(W::widen(a), W::widen(r)) ? r : a;
  }
  static __device__ __forceinline__ uint32_t word(uint32_t a, uint32_t r) {
    const uint32_t lo = half(a & 0xFFFFu, r & 0xFFFFu);
    const uint32_t hi = half(a >> 16, r >> 16);
    return (lo & 0xFFFFu) | (hi << 16);
  }
  // Several sources: SUM / PROD stay in binary32 across the whole fold and round once at
  // the end; MAX / MIN carry the selected 16-bit pattern along with its widened value.
  struct State { float lo, hi; uint32_t bits; };
  static __device__ __forceinline__ State open(uint32_t a) {
    return State{W::widen(a & 0xFFFFu), W::widen(a >> 16), a};
  }
  static __device__ __forceinline__ void fold(State& t, uint32_t r) {
    const float rl = W::widen(r & 0xFFFFu), rh = W::widen(r >> 16);
    if constexpr (K == kSum || K == kProd) {
      t.lo = arith<K>(t.lo, rl);
      t.hi = arith<K>(t.hi, rh);
    } else {
      if (takes_received<K>(t.lo, rl)) { t.lo = rl; t.bits = (t.bits & 0xFFFF0000u) | (r & 0xFFFFu); }
      if (takes_received<K>(t.hi, rh)) { t.hi = rh; t.bits = (t.bits & 0x0000FFFFu) | (r & 0xFFFF0000u); }
    }
  }
  static __device__ __forceinline__ uint32_t close(const State& t) {
    if constexpr (K == kSum || K == kProd) return (W::narrow(t.lo) & 0xFFFFu) | (W::narrow(t.hi) << 16);
    else return t.bits;
  }
};

struct Copy {
  static constexpr bool kReadsAcc = false;
  static constexpr uint32_t kEs = 1;
  static __device__ __forceinline__ uint32_t word(uint32_t, uint32_t r) { return r; }
};

// Which streams of a chunk exist: FWD = the staging copy is written, WB = the accumulator
// is written back (a forward-only record relays the combined value without keeping it).
template <class Op, bool FWD, bool WB>
constexpr uint32_t cache_policy() {
  if (Op::kReadsAcc) return FWD ? (WB ? UCCL_POLICY_REDUCE_FWD : UCCL_POLICY_REDUCE_RELAY) : UCCL_POLICY_REDUCE_KEEP;
  return FWD ? (WB ? UCCL_POLICY_COPY_FWD : UCCL_POLICY_COPY_RELAY) : UCCL_POLICY_COPY_KEEP;
}

template <class Op>
__device__ __forceinline__ u32x4 combine(u32x4 a, u32x4 r) {
  u32x4 t;
  t.x = Op::word(a.x, r.x);
  t.y = Op::word(a.y, r.y);
  t.z = Op::word(a.z, r.z);
  t.w = Op::word(a.w, r.w);
  return t;
}

__device__ __forceinline__ uint64_t wave_uniform(uint64_t v) {
  const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(v));
  const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(v >> 32));
  return lo | (static_cast<uint64_t>(hi) << 32);
}

// Stream one chunk with SG cooperating threads: U independent 16-byte vectors per thread
// per trip, loads first, then combine and store.  Which streams carry a non-temporal
// hint depends on the kind of chunk (see the policy masks above).
template <int SG, int U, class Op, bool FWD, bool WB>
__device__ __forceinline__ void stream_vectors(const u32x4* __restrict__ r, u32x4* __restrict__ a,
                                               u32x4* __restrict__ o, uint32_t nvec,
                                               uint32_t lane) {
  constexpr uint32_t kPolicy = cache_policy<Op, FWD, WB>();
  constexpr bool kNtRecv = (kPolicy & 8u) != 0, kNtOut = (kPolicy & 4u) != 0;
  constexpr bool kNtAccLoad = (kPolicy & 2u) != 0, kNtAccStore = (kPolicy & 1u) != 0;
  constexpr uint32_t kTrip = SG * U;
  const uint32_t full = nvec - nvec % kTrip;
  for (uint32_t base = lane; base < full; base += kTrip) {
    u32x4 rv[U], av[U];
#pragma unroll
    for (int u = 0; u < U; ++u) rv[u] = load16<kNtRecv>(r + base + u * SG);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if constexpr (Op::kReadsAcc) av[u] = load16<kNtAccLoad>(a + base + u * SG);
      else av[u] = rv[u];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const u32x4 t = combine<Op>(av[u], rv[u]);
      if (WB) store16<kNtAccStore>(a + base + u * SG, t);
      if (FWD) store16<kNtOut>(o + base + u * SG, t);
    }
  }
  for (uint32_t i = full + lane; i < nvec; i += SG) {
    const u32x4 rv = load16<kNtRecv>(r + i);
    u32x4 av = rv;
    if constexpr (Op::kReadsAcc) av = load16<kNtAccLoad>(a + i);
    const u32x4 t = combine<Op>(av, rv);
    if (WB) store16<kNtAccStore>(a + i, t);
    if (FWD) store16<kNtOut>(o + i, t);
  }
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

template <int SG, int U, class Op, bool FWD, bool WB>
__device__ __forceinline__ void stream_chunk(const char* r, char* a, char* o, uint32_t len,
                                             uint32_t lane) {
  const uint32_t nvec = len >> 4;
  stream_vectors<SG, U, Op, FWD, WB>(reinterpret_cast<const u32x4*>(r), reinterpret_cast<u32x4*>(a),
                                 reinterpret_cast<u32x4*>(o), nvec, lane);
  const uint32_t rem = len & 15u;
  if (rem) {
    const uint64_t off = static_cast<uint64_t>(nvec) << 4;
    stream_tail<Op, FWD, WB>(r + off, a + off, FWD ? o + off : o, rem, lane);
  }
}

// Winners of one tile of records, compacted; first[] is the exclusive prefix sum of
// their unit counts (flat shape only) with the total in first[count].
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
__device__ __forceinline__ void dedup_tile(const Args& g, Tile<T>& s, uint32_t tid) {
  static_assert(T >= 1 && T <= 64, "one wavefront dedups the tile");
  const uint64_t k = static_cast<uint64_t>(blockIdx.x) * T + tid;
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
    const bool fwd = out != UCCL_NO_FORWARD;
    const uint64_t out_at = out & ~UCCL_FORWARD_ONLY;
    bool ok = seq < g.ext.n_bits && ((src | dst) & 15u) == 0 && len % Op::kEs == 0 &&
              src <= g.ext.recv_bytes && len <= g.ext.recv_bytes - src &&
              dst <= g.ext.acc_bytes && len <= g.ext.acc_bytes - dst;
    if (fwd)
      ok = ok && g.allow_forward && g.out != nullptr && (out_at & 15u) == 0 &&
           out_at <= g.ext.out_bytes && len <= g.ext.out_bytes - out_at;
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

// Shapes WAVE / GROUP: subgroups of SG threads take whole winners in turn.  Kept
// selectable because they are the obvious alternatives (one wavefront per chunk, one
// workgroup per chunk); both measure slower than the flat shape on MI355X.
template <int NT, int T, int SG, int U, class Op>
__global__ void __launch_bounds__(NT) chunk_apply_kernel(const Args g) {
  static_assert(NT % SG == 0 && SG % 64 == 0, "subgroups are whole wavefronts");
  constexpr uint32_t kSubgroups = NT / SG;
  __shared__ Tile<T> s;
  const uint32_t tid = threadIdx.x;
  if (tid < 64) dedup_tile<T, Op, 0>(g, s, tid);
  __syncthreads();

  const uint32_t count = s.count;
  const uint32_t sg = tid / SG, lane = tid % SG;
  for (uint32_t w = sg; w < count; w += kSubgroups) {
    const uint64_t src = wave_uniform(s.src[w]);
    const uint64_t dst = wave_uniform(s.dst[w]);
    const uint64_t out = wave_uniform(s.out[w]);
    const uint32_t len = __builtin_amdgcn_readfirstlane(s.len[w]);
    if (out == UCCL_NO_FORWARD)
      stream_chunk<SG, U, Op, false, true>(g.recv + src, g.acc + dst, nullptr, len, lane);
    else if (out & UCCL_FORWARD_ONLY)
      stream_chunk<SG, U, Op, true, false>(g.recv + src, g.acc + dst, g.out + (out & ~UCCL_FORWARD_ONLY), len, lane);
    else
      stream_chunk<SG, U, Op, true, true>(g.recv + src, g.acc + dst, g.out + out, len, lane);
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

// Shape FLAT: the winners' units are numbered consecutively across the tile and dealt
// round-robin to the 16 wavefronts of a 1024-thread workgroup, so the machine sees the
// same stream whether a tile holds one 128 KiB chunk or thirty-two 4 KiB chunks.
template <int NT, int T, int U, class Op>
__global__ void __launch_bounds__(NT) chunk_flat_kernel(const Args g) {
  constexpr uint32_t kUnit = 64u * U;
  constexpr uint32_t kWaves = NT / 64;
  __shared__ Tile<T> s;
  const uint32_t tid = threadIdx.x;
  if (tid < 64) dedup_tile<T, Op, kUnit>(g, s, tid);
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

// ---- several sources per destination chunk ---------------------------------------------
//
// Section 2.1: the kernel reduces transport buffers "from multiple sender GPUs" into the
// tensor buffer.  A gather record names up to UCCL_MAX_SOURCES receive slots for one
// destination chunk; they are folded into the accumulator's value in the order listed, so
// the floating-point result is fixed by the record, not by arrival timing.  The accumulator
// is read and written once per chunk however many sources there are.  Same tile / unit
// dealing as the flat shape; per unit a wavefront keeps the running value in registers
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
};

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
  constexpr uint32_t kBatch = UCCL_GATHER_BATCH;
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
    const uint64_t dst = wave_uniform(s.dst[w]);
    const uint64_t out = wave_uniform(s.out[w]);
    const uint32_t len = __builtin_amdgcn_readfirstlane(s.len[w]);
    const uint32_t n_src = __builtin_amdgcn_readfirstlane(s.n_src[w]);
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
    // sources in batches: all loads of a batch are issued before the first fold waits
    for (uint32_t j0 = 0; j0 < n_src; j0 += kBatch) {
      u32x4 rv[kBatch][U];
#pragma unroll
      for (uint32_t b = 0; b < kBatch; ++b) {
        if (j0 + b < n_src) {
          const u32x4* rp = reinterpret_cast<const u32x4*>(g.recv + wave_uniform(s.src[w][j0 + b])) + v0 + lane;
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
        const char* rp = g.recv + wave_uniform(s.src[w][j]) + off;
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
}

__global__ void __launch_bounds__(256) fill_words_kernel(uint32_t* p, uint64_t n, uint32_t v) {
  for (uint64_t i = static_cast<uint64_t>(blockIdx.x) * 256 + threadIdx.x; i < n;
       i += static_cast<uint64_t>(gridDim.x) * 256)
    p[i] = v;
}

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

// Per-message window status (Section 3.2's message id / chunk sequence number / last-chunk
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

// ---- host side ----------------------------------------------------------------------

thread_local char t_detail[256] = "";
thread_local hipEvent_t t_start = nullptr, t_stop = nullptr;  // one-shot, see uccl_time_next_launch
// process-wide tuning knobs; atomics so that a setter racing with a launch on another thread
// yields the old or the new value, never a torn one
std::atomic<int> g_shape{UCCL_SHAPE_AUTO};
std::atomic<uint32_t> g_chunk_hint{0};

int launch_failed(hipError_t e) {
  snprintf(t_detail, sizeof(t_detail), "%s: %s", hipGetErrorName(e), hipGetErrorString(e));
  return UCCL_ELAUNCH;
}

// Launch through the calls that RETURN the launch status (the <<<>>> form leaves it in the
// thread's last-error slot, where an earlier, unrelated error could be mistaken for ours and
// reading it would clear the caller's).  The one-shot timing events, if any, are attached to
// this very dispatch.
template <class... Params, size_t... I>
hipError_t launch_raw(void (*kernel)(Params...), dim3 grid, dim3 block, hipStream_t s,
                      std::tuple<Params...>& params, std::index_sequence<I...>) {
  void* ptrs[] = {static_cast<void*>(&std::get<I>(params))...};
  hipEvent_t t0 = t_start, t1 = t_stop;
  t_start = t_stop = nullptr;
  if (t0 != nullptr || t1 != nullptr)
    return hipExtLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, 0, s, t0, t1, 0);
  return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, 0, s);
}

template <class... Params, class... KernelArgs>
int launch_kernel(void (*kernel)(Params...), uint32_t tiles, uint32_t threads, hipStream_t s, KernelArgs... a) {
  static_assert(sizeof...(Params) == sizeof...(KernelArgs), "one argument per kernel parameter");
  std::tuple<Params...> params(static_cast<Params>(a)...);  // objects of the kernel's own parameter types
  const hipError_t e = launch_raw(kernel, dim3(tiles), dim3(threads), s, params, std::index_sequence_for<Params...>{});
  return e == hipSuccess ? UCCL_OK : launch_failed(e);
}

uint32_t tiles_for(uint32_t n_descs, uint32_t tile) {
  return static_cast<uint32_t>((static_cast<uint64_t>(n_descs) + tile - 1) / tile);
}

template <int NT, int T, int SG, int U, class Op>
int launch(const Args& a, hipStream_t s) {
  return launch_kernel(chunk_apply_kernel<NT, T, SG, U, Op>, tiles_for(a.n_descs, T), NT, s, a);
}

template <int T, int U, class Op>
int launch_flat(const Args& a, hipStream_t s) {
  return launch_kernel(chunk_flat_kernel<UCCL_FLAT_THREADS, T, U, Op>, tiles_for(a.n_descs, T),
                       UCCL_FLAT_THREADS, s, a);
}

// Records per workgroup for the flat shape: enough that a tile holds about 32 KiB of
// payload per stream when the chunk size is known, otherwise grown with the record count.
uint32_t flat_tile(uint32_t n_descs) {
  uint32_t t;
  const uint32_t hint = g_chunk_hint.load(std::memory_order_relaxed);
  if (hint) {
    t = (32768u + hint - 1) / hint;
  } else {
    // Unknown chunk size: a tile too large for big chunks costs a few percent, a tile too
    // small for 4 KiB chunks costs a factor of two, so grow the tile once the record count
    // leaves enough workgroups either way.
    t = n_descs < 8192u ? 1u : n_descs < 32768u ? 4u : n_descs < 131072u ? 8u : 16u;
  }
  return t < 1u ? 1u : t > 32u ? 32u : t;
}

template <class Op>
int launch_flat_tile(const Args& a, hipStream_t s) {
  const uint32_t t = flat_tile(a.n_descs);
  if (t >= 32) return launch_flat<32, UCCL_FLAT_UNROLL, Op>(a, s);
  if (t >= 16) return launch_flat<16, UCCL_FLAT_UNROLL, Op>(a, s);
  if (t >= 8) return launch_flat<8, UCCL_FLAT_UNROLL, Op>(a, s);
  if (t >= 4) return launch_flat<4, UCCL_FLAT_UNROLL, Op>(a, s);
  if (t >= 2) return launch_flat<2, UCCL_FLAT_UNROLL, Op>(a, s);
  return launch_flat<1, UCCL_FLAT_UNROLL, Op>(a, s);
}

template <class Op>
int launch_shape(const Args& a, hipStream_t s) {
  const int shape = g_shape.load(std::memory_order_relaxed);
  if (shape == UCCL_SHAPE_AUTO || shape == UCCL_SHAPE_FLAT) return launch_flat_tile<Op>(a, s);
  if (shape == UCCL_SHAPE_WAVE) {
    if (a.n_descs >= 65536u) return launch<256, UCCL_WAVE_TILE_SMALL, 64, UCCL_WAVE_UNROLL, Op>(a, s);
    return launch<256, UCCL_WAVE_TILE, 64, UCCL_WAVE_UNROLL, Op>(a, s);
  }
  if (shape == UCCL_SHAPE_GROUP) return launch<256, UCCL_GROUP_TILE, 256, UCCL_GROUP_UNROLL, Op>(a, s);
  return UCCL_EINVAL;
}


template <int T, class Op>
int launch_gather(const GatherArgs& a, hipStream_t s) {
  return launch_kernel(chunk_gather_kernel<1024, T, UCCL_GATHER_UNROLL, Op>, tiles_for(a.n_descs, T), 1024, s, a);
}

template <class Op>
int launch_gather_tile(const GatherArgs& a, hipStream_t s) {
  const uint32_t t = flat_tile(a.n_descs);
  if (t >= 16) return launch_gather<16, Op>(a, s);
  if (t >= 8) return launch_gather<8, Op>(a, s);
  if (t >= 4) return launch_gather<4, Op>(a, s);
  if (t >= 2) return launch_gather<2, Op>(a, s);
  return launch_gather<1, Op>(a, s);
}

bool misaligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

bool overlaps(const void* p, uint64_t pn, const void* q, uint64_t qn) {
  if (!p || !q || pn == 0 || qn == 0) return false;
  const uintptr_t a = reinterpret_cast<uintptr_t>(p), b = reinterpret_cast<uintptr_t>(q);
  return a < b + qn && b < a + pn;
}

int apply_common(void* acc, void* out_stage, const void* recv_stage, const uccl_chunk_desc* descs,
                 uint32_t n_descs, uint32_t* bitmap, int dtype, int op, bool allow_forward,
                 const uccl_extents* ext, uint32_t* n_rejected, void* stream,
                 const uint32_t* n_ptr = nullptr) {
  if (dtype < UCCL_F32 || dtype > UCCL_I32) return UCCL_EINVAL;
  if (op < UCCL_SUM || op > UCCL_PROD) return UCCL_EINVAL;
  if (n_descs == 0) return UCCL_OK;
  if (!acc || !recv_stage || !descs || !bitmap) return UCCL_EINVAL;
  if (misaligned(acc, 16) || misaligned(out_stage, 16) || misaligned(recv_stage, 16) ||
      misaligned(descs, 16) || misaligned(bitmap, 4) || misaligned(n_rejected, 4) ||
      misaligned(n_ptr, 4))
    return UCCL_EALIGN;
  Args a;
  a.acc = static_cast<char*>(acc);
  a.out = static_cast<char*>(out_stage);
  a.recv = static_cast<const char*>(recv_stage);
  a.descs = descs;
  a.bitmap = bitmap;
  a.rejected = n_rejected;
  a.n_ptr = n_ptr;
  a.n_descs = n_descs;
  a.allow_forward = allow_forward ? 1u : 0u;
  if (ext) {
    if (overlaps(recv_stage, ext->recv_bytes, acc, ext->acc_bytes) ||
        overlaps(recv_stage, ext->recv_bytes, out_stage, ext->out_bytes) ||
        overlaps(acc, ext->acc_bytes, out_stage, ext->out_bytes))
      return UCCL_EINVAL;
    a.ext = Extents{ext->acc_bytes, out_stage ? ext->out_bytes : 0, ext->recv_bytes, ext->n_bits};
  } else {
    a.ext = Extents{UINT64_MAX, UINT64_MAX, UINT64_MAX, UINT64_MAX};
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (op == UCCL_COPY) return launch_shape<Copy>(a, s);
  switch (dtype * 8 + op) {
    case UCCL_F32 * 8 + UCCL_SUM: return launch_shape<OpF32<kSum>>(a, s);
    case UCCL_F32 * 8 + UCCL_MAX: return launch_shape<OpF32<kMax>>(a, s);
    case UCCL_F32 * 8 + UCCL_MIN: return launch_shape<OpF32<kMin>>(a, s);
    case UCCL_F32 * 8 + UCCL_PROD: return launch_shape<OpF32<kProd>>(a, s);
    case UCCL_BF16 * 8 + UCCL_SUM: return launch_shape<Op16<kSum, WidenBF16>>(a, s);
    case UCCL_BF16 * 8 + UCCL_MAX: return launch_shape<Op16<kMax, WidenBF16>>(a, s);
    case UCCL_BF16 * 8 + UCCL_MIN: return launch_shape<Op16<kMin, WidenBF16>>(a, s);
    case UCCL_BF16 * 8 + UCCL_PROD: return launch_shape<Op16<kProd, WidenBF16>>(a, s);
    case UCCL_F16 * 8 + UCCL_SUM: return launch_shape<Op16<kSum, WidenF16>>(a, s);
    case UCCL_F16 * 8 + UCCL_MAX: return launch_shape<Op16<kMax, WidenF16>>(a, s);
    case UCCL_F16 * 8 + UCCL_MIN: return launch_shape<Op16<kMin, WidenF16>>(a, s);
    case UCCL_F16 * 8 + UCCL_PROD: return launch_shape<Op16<kProd, WidenF16>>(a, s);
    case UCCL_I32 * 8 + UCCL_SUM: return launch_shape<OpI32<kSum>>(a, s);
    case UCCL_I32 * 8 + UCCL_MAX: return launch_shape<OpI32<kMax>>(a, s);
    case UCCL_I32 * 8 + UCCL_MIN: return launch_shape<OpI32<kMin>>(a, s);
    case UCCL_I32 * 8 + UCCL_PROD: return launch_shape<OpI32<kProd>>(a, s);
    default: return UCCL_EINVAL;
  }
}

// ---- host-side batcher -------------------------------------------------------------------
//
// Appendix C.4: launching a kernel per batch is what hurts small messages, and batching
// adaptively is the remedy.  The feed collects records on the host in pinned slots and
// hands a slot to the GPU (one asynchronous copy of the records, one kernel per lane) when
// the slot is full, when the caller says so, or -- uccl_feed_poll -- as soon as the previous
// hand-over has finished, so that batches grow exactly as large as the GPU's backlog
// requires and a lone message is launched at once.  Lanes keep records of dependent phases
// apart: a flush issues lane 0 before lane 1, so a message whose reduce-scatter records go
// to lane 0 before its allgather records go to lane 1 is always applied in that order.
// Hand-overs of at most this many records per lane are read from pinned host memory directly.
#ifndef UCCL_FEED_DIRECT_RECORDS
#define UCCL_FEED_DIRECT_RECORDS 16384
#endif

struct FeedSlot {
  uccl_chunk_desc* host[2];
  uccl_chunk_desc* dev[2];
  uint32_t count[2];
  hipEvent_t done;
  bool in_flight;
};

}  // namespace

struct uccl_feed {
  void* acc;
  void* out_stage;
  const void* recv_stage;
  uint32_t* bitmap;
  int dtype;
  int op[2];
  uint32_t capacity, n_slots, cur;
  hipStream_t stream;
  FeedSlot* slots;
  uccl_feed_stats stats;
};

namespace {

void feed_free(uccl_feed* f) {
  if (!f) return;
  if (f->slots) {
    for (uint32_t i = 0; i < f->n_slots; ++i) {
      for (int l = 0; l < 2; ++l) {
        if (f->slots[i].host[l]) (void)hipHostFree(f->slots[i].host[l]);
        if (f->slots[i].dev[l]) (void)hipFree(f->slots[i].dev[l]);
      }
      if (f->slots[i].done) (void)hipEventDestroy(f->slots[i].done);
    }
    delete[] f->slots;
  }
  delete f;
}

int feed_flush(uccl_feed* f) {
  FeedSlot& sl = f->slots[f->cur];
  const uint32_t n = sl.count[0] + sl.count[1];
  if (n == 0) return UCCL_OK;
  for (int l = 0; l < 2; ++l) {
    if (sl.count[l] == 0) continue;
    // A small batch is read by the kernel straight from the pinned slot (one bus round trip per
    // workgroup, no copy to enqueue); a large one is copied to device memory first, so that
    // thousands of workgroups do not each wait on the host bus.
    const uccl_chunk_desc* records = sl.host[l];
    if (sl.count[l] > UCCL_FEED_DIRECT_RECORDS) {
      const hipError_t e = hipMemcpyAsync(sl.dev[l], sl.host[l], sizeof(uccl_chunk_desc) * sl.count[l],
                                          hipMemcpyHostToDevice, f->stream);
      if (e != hipSuccess) return launch_failed(e);
      records = sl.dev[l];
    }
    const int rc = apply_common(f->acc, f->out_stage, f->recv_stage, records, sl.count[l], f->bitmap,
                                f->dtype, f->op[l], true, nullptr, nullptr, f->stream);
    if (rc != UCCL_OK) return rc;
  }
  const hipError_t e = hipEventRecord(sl.done, f->stream);
  if (e != hipSuccess) return launch_failed(e);
  sl.in_flight = true;
  f->stats.flushes += 1;
  f->stats.records += n;
  if (n > f->stats.max_batch) f->stats.max_batch = n;
  sl.count[0] = sl.count[1] = 0;
  // move on to the next slot; it may still be read by the copy of an earlier flush
  f->cur = (f->cur + 1) % f->n_slots;
  FeedSlot& nx = f->slots[f->cur];
  if (nx.in_flight) {
    if (hipEventQuery(nx.done) != hipSuccess) {
      (void)hipGetLastError();  // hipErrorNotReady is not an error here
      const hipError_t w = hipEventSynchronize(nx.done);
      if (w != hipSuccess) return launch_failed(w);
      f->stats.slot_waits += 1;
    }
    nx.in_flight = false;
  }
  return UCCL_OK;
}

}  // namespace

extern "C" {

int uccl_feed_create(uccl_feed** feed, void* acc, void* out_stage, const void* recv_stage,
                     uint32_t* dedup_bitmap, uccl_dtype dtype, uccl_op lane0_op, uccl_op lane1_op,
                     uint32_t capacity_records, uint32_t n_slots, void* stream) {
  if (!feed) return UCCL_EINVAL;
  *feed = nullptr;
  if (!acc || !recv_stage || !dedup_bitmap || capacity_records == 0 || n_slots < 2 || n_slots > 1024)
    return UCCL_EINVAL;
  if (dtype < UCCL_F32 || dtype > UCCL_I32) return UCCL_EINVAL;
  if (lane0_op < UCCL_SUM || lane0_op > UCCL_PROD || lane1_op < UCCL_SUM || lane1_op > UCCL_PROD)
    return UCCL_EINVAL;
  if (misaligned(acc, 16) || misaligned(out_stage, 16) || misaligned(recv_stage, 16) ||
      misaligned(dedup_bitmap, 4))
    return UCCL_EALIGN;
  uccl_feed* f = new (std::nothrow) uccl_feed();
  if (!f) return UCCL_ENOMEM;
  f->acc = acc;
  f->out_stage = out_stage;
  f->recv_stage = recv_stage;
  f->bitmap = dedup_bitmap;
  f->dtype = dtype;
  f->op[0] = lane0_op;
  f->op[1] = lane1_op;
  f->capacity = capacity_records;
  f->n_slots = n_slots;
  f->cur = 0;
  f->stream = static_cast<hipStream_t>(stream);
  f->stats = uccl_feed_stats{0, 0, 0, 0};
  f->slots = new (std::nothrow) FeedSlot[n_slots]();
  if (!f->slots) { feed_free(f); return UCCL_ENOMEM; }
  const size_t bytes = sizeof(uccl_chunk_desc) * static_cast<size_t>(capacity_records);
  for (uint32_t i = 0; i < n_slots; ++i) {
    for (int l = 0; l < 2; ++l) {
      if (hipHostMalloc(reinterpret_cast<void**>(&f->slots[i].host[l]), bytes, hipHostMallocDefault) != hipSuccess ||
          hipMalloc(reinterpret_cast<void**>(&f->slots[i].dev[l]), bytes) != hipSuccess) {
        (void)hipGetLastError();
        feed_free(f);
        return UCCL_ENOMEM;
      }
    }
    if (hipEventCreateWithFlags(&f->slots[i].done, hipEventDisableTiming) != hipSuccess) {
      (void)hipGetLastError();
      feed_free(f);
      return UCCL_ENOMEM;
    }
  }
  *feed = f;
  return UCCL_OK;
}

int uccl_feed_push(uccl_feed* f, int lane, const uccl_chunk_desc* host_records, uint32_t n) {
  if (!f || (lane != 0 && lane != 1) || (n > 0 && !host_records)) return UCCL_EINVAL;
  while (n > 0) {
    FeedSlot& sl = f->slots[f->cur];
    const uint32_t room = f->capacity - sl.count[lane];
    const uint32_t take = n < room ? n : room;
    memcpy(sl.host[lane] + sl.count[lane], host_records, sizeof(uccl_chunk_desc) * take);
    sl.count[lane] += take;
    host_records += take;
    n -= take;
    if (sl.count[lane] == f->capacity) {
      const int rc = feed_flush(f);
      if (rc != UCCL_OK) return rc;
    }
  }
  return UCCL_OK;
}

int uccl_feed_poll(uccl_feed* f) {
  if (!f) return UCCL_EINVAL;
  const FeedSlot& sl = f->slots[f->cur];
  if (sl.count[0] + sl.count[1] == 0) return UCCL_OK;
  const FeedSlot& prev = f->slots[(f->cur + f->n_slots - 1) % f->n_slots];
  if (prev.in_flight && hipEventQuery(prev.done) == hipErrorNotReady) {
    (void)hipGetLastError();  // "not ready" is an answer, not an error to leave behind
    return UCCL_OK;           // GPU still busy: keep batching
  }
  return feed_flush(f);
}

int uccl_feed_flush(uccl_feed* f) { return f ? feed_flush(f) : UCCL_EINVAL; }

int uccl_feed_sync(uccl_feed* f) {
  if (!f) return UCCL_EINVAL;
  const int rc = feed_flush(f);
  if (rc != UCCL_OK) return rc;
  for (uint32_t i = 0; i < f->n_slots; ++i) {
    if (f->slots[i].in_flight) {
      const hipError_t e = hipEventSynchronize(f->slots[i].done);
      if (e != hipSuccess) return launch_failed(e);
      f->slots[i].in_flight = false;
    }
  }
  return UCCL_OK;
}

int uccl_feed_get_stats(const uccl_feed* f, uccl_feed_stats* stats) {
  if (!f || !stats) return UCCL_EINVAL;
  *stats = f->stats;
  return UCCL_OK;
}

int uccl_feed_destroy(uccl_feed* f) {
  if (!f) return UCCL_EINVAL;
  int rc = UCCL_OK;
  for (uint32_t i = 0; i < f->n_slots; ++i)
    if (f->slots[i].in_flight && hipEventSynchronize(f->slots[i].done) != hipSuccess) rc = UCCL_ELAUNCH;
  feed_free(f);
  return rc;
}

}  // extern "C"

extern "C" {

int uccl_chunk_apply(void* acc, void* out_stage, const void* recv_stage,
                     const uccl_chunk_desc* descs, uint32_t n_descs, uint32_t* dedup_bitmap,
                     uccl_dtype dtype, uccl_op op, void* stream) {
  return apply_common(acc, out_stage, recv_stage, descs, n_descs, dedup_bitmap, dtype, op, true,
                      nullptr, nullptr, stream);
}

int uccl_chunk_apply_checked(void* acc, void* out_stage, const void* recv_stage,
                             const uccl_chunk_desc* descs, uint32_t n_descs,
                             uint32_t* dedup_bitmap, uccl_dtype dtype, uccl_op op,
                             const uccl_extents* extents, uint32_t* n_rejected, void* stream) {
  if (!extents) return UCCL_EINVAL;
  return apply_common(acc, out_stage, recv_stage, descs, n_descs, dedup_bitmap, dtype, op, true,
                      extents, n_rejected, stream);
}

int uccl_chunk_apply_indirect(void* acc, void* out_stage, const void* recv_stage,
                              const uccl_chunk_desc* descs, const uint32_t* n_descs_ptr,
                              uint32_t max_descs, uint32_t* dedup_bitmap, uccl_dtype dtype,
                              uccl_op op, const uccl_extents* extents, uint32_t* n_rejected,
                              void* stream) {
  if (max_descs > 0 && !n_descs_ptr) return UCCL_EINVAL;
  return apply_common(acc, out_stage, recv_stage, descs, max_descs, dedup_bitmap, dtype, op, true,
                      extents, n_rejected, stream, n_descs_ptr);
}

int uccl_chunk_reduce_gather(void* acc, void* out_stage, const void* recv_stage,
                             const uccl_gather_desc* descs, uint32_t n_descs, uint32_t* dedup_bitmap,
                             uccl_dtype dtype, uccl_op op, const uccl_extents* extents,
                             uint32_t* n_rejected, void* stream) {
  if (dtype < UCCL_F32 || dtype > UCCL_I32) return UCCL_EINVAL;
  if (op != UCCL_SUM && op != UCCL_MAX && op != UCCL_MIN && op != UCCL_PROD) return UCCL_EINVAL;
  if (n_descs == 0) return UCCL_OK;
  if (!acc || !recv_stage || !descs || !dedup_bitmap) return UCCL_EINVAL;
  if (misaligned(acc, 16) || misaligned(out_stage, 16) || misaligned(recv_stage, 16) ||
      misaligned(descs, 16) || misaligned(dedup_bitmap, 4) || misaligned(n_rejected, 4))
    return UCCL_EALIGN;
  GatherArgs a;
  a.acc = static_cast<char*>(acc);
  a.out = static_cast<char*>(out_stage);
  a.recv = static_cast<const char*>(recv_stage);
  a.descs = descs;
  a.bitmap = dedup_bitmap;
  a.rejected = n_rejected;
  a.n_descs = n_descs;
  if (extents) {
    if (overlaps(recv_stage, extents->recv_bytes, acc, extents->acc_bytes) ||
        overlaps(recv_stage, extents->recv_bytes, out_stage, extents->out_bytes) ||
        overlaps(acc, extents->acc_bytes, out_stage, extents->out_bytes))
      return UCCL_EINVAL;
    a.ext = Extents{extents->acc_bytes, out_stage ? extents->out_bytes : 0, extents->recv_bytes, extents->n_bits};
  } else {
    a.ext = Extents{UINT64_MAX, UINT64_MAX, UINT64_MAX, UINT64_MAX};
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  switch (dtype * 8 + op) {
    case UCCL_F32 * 8 + UCCL_SUM: return launch_gather_tile<OpF32<kSum>>(a, s);
    case UCCL_F32 * 8 + UCCL_MAX: return launch_gather_tile<OpF32<kMax>>(a, s);
    case UCCL_F32 * 8 + UCCL_MIN: return launch_gather_tile<OpF32<kMin>>(a, s);
    case UCCL_F32 * 8 + UCCL_PROD: return launch_gather_tile<OpF32<kProd>>(a, s);
    case UCCL_BF16 * 8 + UCCL_SUM: return launch_gather_tile<Op16<kSum, WidenBF16>>(a, s);
    case UCCL_BF16 * 8 + UCCL_MAX: return launch_gather_tile<Op16<kMax, WidenBF16>>(a, s);
    case UCCL_BF16 * 8 + UCCL_MIN: return launch_gather_tile<Op16<kMin, WidenBF16>>(a, s);
    case UCCL_BF16 * 8 + UCCL_PROD: return launch_gather_tile<Op16<kProd, WidenBF16>>(a, s);
    case UCCL_F16 * 8 + UCCL_SUM: return launch_gather_tile<Op16<kSum, WidenF16>>(a, s);
    case UCCL_F16 * 8 + UCCL_MAX: return launch_gather_tile<Op16<kMax, WidenF16>>(a, s);
    case UCCL_F16 * 8 + UCCL_MIN: return launch_gather_tile<Op16<kMin, WidenF16>>(a, s);
    case UCCL_F16 * 8 + UCCL_PROD: return launch_gather_tile<Op16<kProd, WidenF16>>(a, s);
    case UCCL_I32 * 8 + UCCL_SUM: return launch_gather_tile<OpI32<kSum>>(a, s);
    case UCCL_I32 * 8 + UCCL_MAX: return launch_gather_tile<OpI32<kMax>>(a, s);
    case UCCL_I32 * 8 + UCCL_MIN: return launch_gather_tile<OpI32<kMin>>(a, s);
    case UCCL_I32 * 8 + UCCL_PROD: return launch_gather_tile<OpI32<kProd>>(a, s);
    default: return UCCL_EINVAL;
  }
}

int uccl_chunk_scatter(void* dst, const void* recv_stage, const uccl_chunk_desc* descs,
                       uint32_t n_descs, uint32_t* dedup_bitmap, void* stream) {
  return apply_common(dst, nullptr, recv_stage, descs, n_descs, dedup_bitmap, UCCL_BF16, UCCL_COPY,
                      false, nullptr, nullptr, stream);
}

int uccl_chunk_scatter_checked(void* dst, const void* recv_stage, const uccl_chunk_desc* descs,
                               uint32_t n_descs, uint32_t* dedup_bitmap,
                               const uccl_extents* extents, uint32_t* n_rejected, void* stream) {
  if (!extents) return UCCL_EINVAL;
  return apply_common(dst, nullptr, recv_stage, descs, n_descs, dedup_bitmap, UCCL_BF16, UCCL_COPY,
                      false, extents, n_rejected, stream);
}

int uccl_dedup_reset(uint32_t* dedup_bitmap, uint64_t n_bits, void* stream) {
  if (n_bits == 0) return UCCL_OK;
  if (!dedup_bitmap) return UCCL_EINVAL;
  if (misaligned(dedup_bitmap, 4)) return UCCL_EALIGN;
  const uint64_t words = (n_bits + 31) / 32;
  const uint64_t blocks = (words + 255) / 256;
  const uint32_t grid = static_cast<uint32_t>(blocks < 4096 ? blocks : 4096);
  return launch_kernel(fill_words_kernel, grid, 256, static_cast<hipStream_t>(stream), dedup_bitmap, words, 0u);
}

int uccl_dedup_report(const uint32_t* dedup_bitmap, uint64_t n_bits, void* report,
                      uint32_t max_ranges, void* stream) {
  if (!report || (n_bits > 0 && !dedup_bitmap)) return UCCL_EINVAL;
  if (n_bits >= (1ull << 40)) return UCCL_EINVAL;
  if (misaligned(dedup_bitmap, 4) || misaligned(report, 8)) return UCCL_EALIGN;
  AckHeader* hdr = static_cast<AckHeader*>(report);
  uint64_t* ranges = reinterpret_cast<uint64_t*>(hdr + 1);
  return launch_kernel(ack_report_kernel, 1, 1024, static_cast<hipStream_t>(stream), dedup_bitmap,
                       n_bits, hdr, ranges, max_ranges);
}

int uccl_message_status(uint32_t* dedup_bitmap, const uint32_t* n_chunks, uint32_t n_slots,
                        uint32_t bits_per_slot, uccl_msg_status* status, int recycle, void* stream) {
  if (bits_per_slot < 32 || bits_per_slot > 2048 || (bits_per_slot & 31u)) return UCCL_EINVAL;
  if (n_slots == 0) return UCCL_OK;
  if (n_slots > (1u << 24)) return UCCL_EINVAL;
  if (!dedup_bitmap || !n_chunks || !status) return UCCL_EINVAL;
  if (misaligned(dedup_bitmap, 4) || misaligned(n_chunks, 4) || misaligned(status, 16)) return UCCL_EALIGN;
  const uint32_t grid = (n_slots + 3) / 4;  // one wavefront per slot, four per workgroup
  return launch_kernel(message_status_kernel, grid, 256, static_cast<hipStream_t>(stream), dedup_bitmap,
                       n_chunks, n_slots, bits_per_slot / 32, reinterpret_cast<uint4*>(status),
                       recycle ? 1u : 0u);
}

int uccl_time_next_launch(void* start_event, void* stop_event) {
  t_start = static_cast<hipEvent_t>(start_event);
  t_stop = static_cast<hipEvent_t>(stop_event);
  return UCCL_OK;
}

int uccl_set_chunk_hint(uint32_t chunk_bytes) {
  g_chunk_hint.store(chunk_bytes, std::memory_order_relaxed);
  return UCCL_OK;
}

int uccl_set_launch_shape(int shape) {
  if (shape != UCCL_SHAPE_AUTO && shape != UCCL_SHAPE_WAVE && shape != UCCL_SHAPE_GROUP &&
      shape != UCCL_SHAPE_FLAT)
    return UCCL_EINVAL;
  g_shape.store(shape, std::memory_order_relaxed);
  return UCCL_OK;
}

const char* uccl_strerror(int code) {
  switch (code) {
    case UCCL_OK: return "ok";
    case UCCL_EINVAL: return "invalid argument";
    case UCCL_EALIGN: return "misaligned pointer";
    case UCCL_ELAUNCH: return "HIP launch failed";
    case UCCL_ENOMEM: return "out of memory";
    default: return "unknown error code";
  }
}

const char* uccl_last_error_detail(void) { return t_detail; }

int uccl_version(void) { return UCCL_CHUNK_VERSION; }

}  // extern "C"
