// Element arithmetic and cache-policy selection of the receive-side chunk data path (device code).
// Internal to the library: included by uccl_chunk.hip only, inside its translation unit.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

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

}  // namespace
