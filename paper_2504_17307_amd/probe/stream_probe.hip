// Dense streaming kernels of the data path's traffic shapes, with no records, no dedup and no
// scatter: what the memory system of the GPU at hand delivers for the same mix of read and
// written streams, the same footprint and the same per-workgroup block.  A measurement aid for the
// benchmark (its own shared library, not part of libuccl_chunk.so): the receive path's kernels are
// compared with these beside the published peak.
//
// Every workgroup of 1024 threads takes one contiguous block of `block_bytes` of every stream, in
// 2 KiB units dealt round-robin to its 16 wavefronts, all loads of a unit issued before its stores,
// with the cache policy the data path uses for that stream (slot reads and staging writes
// non-temporal; the accumulator read with default policy, written non-temporally by a reduce
// that forwards and with default policy otherwise).
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

enum Mode {
  kRead = 0,        // 1R:     slot stream only (values folded into a checksum nobody stores)
  kWrite = 1,       // 1W:     staging stream only
  kCopy = 2,        // 1R+1W:  slot -> staging
  kReduceFwd = 3,   // 2R+2W:  acc = acc + slot; staging = acc   (ring reduce-scatter step)
  kCopyFwd = 4,     // 1R+2W:  acc = slot; staging = slot        (ring allgather step)
  kReduceKeep = 5,  // 2R+1W:  acc = acc + slot                  (last reduce-scatter step)
  kGather = 6,      // (n+1)R+1W: acc = acc + slot_0 + ... + slot_{n-1}, sources n consecutive regions of `slot`
  kModes = 7
};

__device__ __forceinline__ u32x4 add_f32(u32x4 a, u32x4 r) {
  u32x4 t;
  t.x = __float_as_uint(__uint_as_float(a.x) + __uint_as_float(r.x));
  t.y = __float_as_uint(__uint_as_float(a.y) + __uint_as_float(r.y));
  t.z = __float_as_uint(__uint_as_float(a.z) + __uint_as_float(r.z));
  t.w = __float_as_uint(__uint_as_float(a.w) + __uint_as_float(r.w));
  return t;
}

// `perm` (may be null): block b of the slot stream goes to block perm[b] of the accumulator and
// staging streams, the way arrivals go to scattered destinations (whole blocks only).
template <int MODE>
__global__ void __launch_bounds__(1024) stream_probe_kernel(const u32x4* __restrict__ slot, u32x4* __restrict__ acc,
                                                            u32x4* __restrict__ stage, uint64_t total_vecs,
                                                            uint32_t block_vecs, uint32_t* sink,
                                                            const uint32_t* __restrict__ perm) {
  constexpr uint32_t kUnit = 128;  // vectors per unit: 64 lanes x 2
  const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63u;
  const uint64_t base = static_cast<uint64_t>(blockIdx.x) * block_vecs;
  if (perm != nullptr) {
    const int64_t shift = (static_cast<int64_t>(perm[blockIdx.x]) - static_cast<int64_t>(blockIdx.x)) * block_vecs;
    acc += shift;
    stage += shift;
  }
  uint32_t fold = 0;
  for (uint32_t u = wave * kUnit; u < block_vecs; u += 16 * kUnit) {
    const uint64_t v0 = base + u + lane, v1 = v0 + 64;
    const bool in0 = v0 < total_vecs, in1 = v1 < total_vecs;
    u32x4 r0 = {1u, 2u, 3u, 4u}, r1 = {5u, 6u, 7u, 8u}, a0 = r0, a1 = r1;
    if (MODE != kWrite) {
      if (in0) r0 = __builtin_nontemporal_load(slot + v0);
      if (in1) r1 = __builtin_nontemporal_load(slot + v1);
    }
    if (MODE == kReduceFwd || MODE == kReduceKeep) {
      if (in0) a0 = acc[v0];
      if (in1) a1 = acc[v1];
    }
    u32x4 t0 = r0, t1 = r1;
    if (MODE == kReduceFwd || MODE == kReduceKeep) { t0 = add_f32(a0, r0); t1 = add_f32(a1, r1); }
    if (MODE == kRead) fold ^= t0.x ^ t0.y ^ t0.z ^ t0.w ^ t1.x ^ t1.y ^ t1.z ^ t1.w;
    if (MODE == kReduceFwd) {
      if (in0) __builtin_nontemporal_store(t0, acc + v0);
      if (in1) __builtin_nontemporal_store(t1, acc + v1);
    }
    if (MODE == kCopyFwd || MODE == kReduceKeep) {
      if (in0) acc[v0] = t0;
      if (in1) acc[v1] = t1;
    }
    if (MODE == kWrite || MODE == kCopy || MODE == kReduceFwd || MODE == kCopyFwd) {
      if (in0) __builtin_nontemporal_store(t0, stage + v0);
      if (in1) __builtin_nontemporal_store(t1, stage + v1);
    }
  }
  if (MODE == kRead && fold == 0x9E3779B9u && sink != nullptr) *sink = fold;  // keeps the loads alive
}

// Several sources folded into the accumulator (the multi-sender reduce): per unit every source's
// vectors are loaded, then folded in order; the accumulator is read and written once.
__global__ void __launch_bounds__(1024) gather_probe_kernel(const u32x4* __restrict__ slot, u32x4* __restrict__ acc,
                                                            uint64_t total_vecs, uint32_t block_vecs, uint32_t n_src) {
  constexpr uint32_t kUnit = 128;
  const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63u;
  const uint64_t base = static_cast<uint64_t>(blockIdx.x) * block_vecs;
  for (uint32_t u = wave * kUnit; u < block_vecs; u += 16 * kUnit) {
    const uint64_t v0 = base + u + lane, v1 = v0 + 64;
    const bool in0 = v0 < total_vecs, in1 = v1 < total_vecs;
    u32x4 t0 = {0u, 0u, 0u, 0u}, t1 = t0;
    if (in0) t0 = acc[v0];
    if (in1) t1 = acc[v1];
    for (uint32_t j0 = 0; j0 < n_src; j0 += 4) {
      u32x4 r0[4], r1[4];
#pragma unroll
      for (uint32_t b = 0; b < 4; ++b) {
        r0[b] = u32x4{0u, 0u, 0u, 0u};
        r1[b] = r0[b];
        if (j0 + b < n_src) {
          const u32x4* src = slot + static_cast<uint64_t>(j0 + b) * total_vecs;
          if (in0) r0[b] = __builtin_nontemporal_load(src + v0);
          if (in1) r1[b] = __builtin_nontemporal_load(src + v1);
        }
      }
#pragma unroll
      for (uint32_t b = 0; b < 4; ++b) {
        if (j0 + b < n_src) { t0 = add_f32(t0, r0[b]); t1 = add_f32(t1, r1[b]); }
      }
    }
    if (in0) acc[v0] = t0;
    if (in1) acc[v1] = t1;
  }
}

template <int MODE>
hipError_t launch(const void* slot, void* acc, void* stage, uint64_t bytes, uint32_t block_bytes, uint32_t* sink,
                  hipStream_t s, const uint32_t* perm = nullptr) {
  const uint64_t total_vecs = bytes / 16;
  const uint32_t block_vecs = block_bytes / 16;
  const uint64_t blocks = (total_vecs + block_vecs - 1) / block_vecs;
  if (blocks == 0 || blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
  stream_probe_kernel<MODE><<<dim3(static_cast<uint32_t>(blocks)), dim3(1024), 0, s>>>(
      static_cast<const u32x4*>(slot), static_cast<u32x4*>(acc), static_cast<u32x4*>(stage), total_vecs, block_vecs, sink,
      perm);
  return hipGetLastError();
}

}  // namespace

// mode: see enum Mode.  slot / acc / stage: DEVICE buffers of at least `bytes` bytes each (slot:
// n_src * bytes for the gather mode; those the mode does not touch may be NULL), 16-byte aligned;
// bytes and block_bytes multiples of 2048; n_src 1..16 (gather mode only).
// Returns 0, or -1 for bad arguments / a refused launch.  Stream ordered, nothing is allocated.
extern "C" int uccl_probe_stream(int mode, const void* slot, void* acc, void* stage, uint64_t bytes,
                                 uint32_t block_bytes, uint32_t n_src, uint32_t* sink, void* stream) {
  if (mode < 0 || mode >= kModes || bytes == 0 || block_bytes == 0 || (bytes % 2048) || (block_bytes % 2048)) return -1;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = hipErrorInvalidValue;
  if (mode == kGather) {
    if (n_src < 1 || n_src > 16) return -1;
    const uint64_t total_vecs = bytes / 16;
    const uint32_t block_vecs = block_bytes / 16;
    const uint64_t blocks = (total_vecs + block_vecs - 1) / block_vecs;
    if (blocks > 0x7FFFFFFFull) return -1;
    gather_probe_kernel<<<dim3(static_cast<uint32_t>(blocks)), dim3(1024), 0, s>>>(
        static_cast<const u32x4*>(slot), static_cast<u32x4*>(acc), total_vecs, block_vecs, n_src);
    return hipGetLastError() == hipSuccess ? 0 : -1;
  }
  switch (mode) {
    case kRead: e = launch<kRead>(slot, acc, stage, bytes, block_bytes, sink, s); break;
    case kWrite: e = launch<kWrite>(slot, acc, stage, bytes, block_bytes, sink, s); break;
    case kCopy: e = launch<kCopy>(slot, acc, stage, bytes, block_bytes, sink, s); break;
    case kReduceFwd: e = launch<kReduceFwd>(slot, acc, stage, bytes, block_bytes, sink, s); break;
    case kCopyFwd: e = launch<kCopyFwd>(slot, acc, stage, bytes, block_bytes, sink, s); break;
    case kReduceKeep: e = launch<kReduceKeep>(slot, acc, stage, bytes, block_bytes, sink, s); break;
  }
  return e == hipSuccess ? 0 : -1;
}

// The reduce-and-forward (mode 3) and copy-and-forward (mode 4) shapes with scattered destinations:
// block b of the slot stream is combined into block perm[b] of acc and stage.  perm: DEVICE array of
// bytes / block_bytes entries, a permutation of 0 .. bytes / block_bytes - 1 (not checked); bytes
// must be a multiple of block_bytes.  Returns 0, or -1 for bad arguments / a refused launch.
extern "C" int uccl_probe_scattered(int mode, const void* slot, void* acc, void* stage, uint64_t bytes,
                                    uint32_t block_bytes, const uint32_t* perm, void* stream) {
  if ((mode != kReduceFwd && mode != kCopyFwd) || bytes == 0 || block_bytes == 0 || (block_bytes % 2048) ||
      (bytes % block_bytes) || perm == nullptr)
    return -1;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const hipError_t e = mode == kReduceFwd ? launch<kReduceFwd>(slot, acc, stage, bytes, block_bytes, nullptr, s, perm)
                                          : launch<kCopyFwd>(slot, acc, stage, bytes, block_bytes, nullptr, s, perm);
  return e == hipSuccess ? 0 : -1;
}
