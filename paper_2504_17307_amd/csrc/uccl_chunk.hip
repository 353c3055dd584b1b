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
// their units (2 KiB; 1 KiB where a workgroup reduces a single record).  After one barrier
// the 16 wavefronts take units round-robin and stream them with 128-bit loads and stores:
// every thread issues all loads of a unit, then combines, then stores, and the workgroup
// retires.  Duplicates cost their record and one atomic, nothing else.  Two lanes holding
// the same seq each issue their own atomic, so the hardware serialises them and exactly one
// sees the bit clear.
//
// Calls of few records (Appendix C.4: small messages are where fixed costs show) take another
// kernel, which shortens the chain of latencies instead: one record per workgroup, payload
// loads issued before the sequence number is decided, and, when the records alone would leave
// most compute units idle, each record cut into parts over several workgroups that agree on
// its fate through a claim word in scratch memory (uccl_data_kernels.hpp).  The sender side
// (tensor range -> staged chunks + send records) and the feedback kernels (acknowledgement
// report, per-message status) are dense, small kernels of their own.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include <atomic>
#include <mutex>
#include <new>
#include <tuple>
#include <utility>

#include "uccl_chunk.h"

#include "uccl_elements.hpp"
#include "uccl_data_kernels.hpp"
#include "uccl_feedback_kernels.hpp"

// Claim words for uccl_chunk_apply_noalloc (see claim_enter): one per record of a call, each on a
// 128-byte line of its own, UCCL_NOALLOC_MAX_DESCS of them, then the word that counts parts that
// gave up waiting: 256.25 KiB.  Every GPU the
// library runs on holds its own copy at its own address until the process ends.  In host code
// this name only stands for the symbol: the device address is looked up per device (static_claims).
static __device__ __align__(256) unsigned long long scratch[UCCL_NOALLOC_MAX_DESCS * UCCL_CLAIM_STRIDE + 32];

namespace {

// ---- host side ----------------------------------------------------------------------

thread_local char t_detail[256] = "";
thread_local hipEvent_t t_start = nullptr, t_stop = nullptr;  // one-shot, see uccl_time_next_launch

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

// ---- claim words for records cut into parts ---------------------------------------------------
//
// Scratch memory of the split launch (see claim_enter): one 64-bit word per record of the call,
// on a 128-byte line of its own.  The library owns one pool per device (16 MiB), made at the first
// call that needs it (or by uccl_init) and kept until the process ends: kRegions regions for
// kRegionRecords records each, one region per stream
// handle that has issued a split call.  Calls on one stream run in order, so they can share a
// region; calls on different streams may overlap, so they never do.  A call whose stream finds
// no free region, or that is being captured into a graph (a replay would carry the captured tag
// again, and could overlap with anything), is launched with one workgroup per record.
//
// Tags must grow in the order in which the calls that share a word run.  They come from one
// process-wide counter, and a split call draws its tag and enqueues its launch while holding the
// device's launch lock, so on any one stream the later launch always carries the larger tag, also
// when several host threads issue calls on that stream.
constexpr uint32_t kRegionRecords = 2048;  // most records a split call can have
constexpr uint32_t kRegionWords = kRegionRecords * UCCL_CLAIM_STRIDE;
constexpr uint32_t kRegions = 64;
constexpr int kMaxDevices = 64;
constexpr size_t kPoolBytes = sizeof(unsigned long long) * kRegions * kRegionWords + 8;  // + fault counter

struct ClaimPool {
  std::atomic<unsigned long long*> base{nullptr};
  std::mutex lock;                       // guards creation and the stream table's growth
  std::mutex launch_lock;                // held from drawing a tag until its launch is enqueued
  std::atomic<uint32_t> n_streams{0};
  std::atomic<uintptr_t> stream_of[kRegions];
};
ClaimPool g_pools[kMaxDevices];
std::atomic<unsigned long long> g_next_tag{1};  // tags are unique across streams, devices and threads

unsigned long long* pool_base(int dev, bool may_allocate) {
  ClaimPool& p = g_pools[dev];
  unsigned long long* b = p.base.load(std::memory_order_acquire);
  if (b != nullptr || !may_allocate) return b;
  std::lock_guard<std::mutex> hold(p.lock);
  b = p.base.load(std::memory_order_acquire);
  if (b != nullptr) return b;
  void* mem = nullptr;
  if (hipMalloc(&mem, kPoolBytes) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
  if (hipMemset(mem, 0, kPoolBytes) != hipSuccess || hipDeviceSynchronize() != hipSuccess) {
    (void)hipGetLastError();
    (void)hipFree(mem);
    return nullptr;
  }
  p.base.store(static_cast<unsigned long long*>(mem), std::memory_order_release);
  return static_cast<unsigned long long*>(mem);
}

uint32_t* pool_faults(unsigned long long* base) {
  return reinterpret_cast<uint32_t*>(base + static_cast<size_t>(kRegions) * kRegionWords);
}

// The claim region of `stream` on the current device, or nullptr (then the call is not split).
unsigned long long* claim_region(hipStream_t stream, uint32_t** faults, ClaimPool** pool) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) { (void)hipGetLastError(); return nullptr; }
  hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(stream, &cap) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
  if (cap != hipStreamCaptureStatusNone) return nullptr;
  unsigned long long* base = pool_base(dev, true);
  if (base == nullptr) return nullptr;
  ClaimPool& p = g_pools[dev];
  const uintptr_t key = reinterpret_cast<uintptr_t>(stream) + 1;  // 0 marks a free entry; the null stream is 1
  uint32_t n = p.n_streams.load(std::memory_order_acquire);
  uint32_t at = kRegions;
  for (uint32_t i = 0; i < n; ++i)
    if (p.stream_of[i].load(std::memory_order_relaxed) == key) { at = i; break; }
  if (at == kRegions) {
    std::lock_guard<std::mutex> hold(p.lock);
    n = p.n_streams.load(std::memory_order_acquire);
    for (uint32_t i = 0; i < n; ++i)
      if (p.stream_of[i].load(std::memory_order_relaxed) == key) { at = i; break; }
    if (at == kRegions) {
      if (n == kRegions) return nullptr;
      p.stream_of[n].store(key, std::memory_order_relaxed);
      p.n_streams.store(n + 1, std::memory_order_release);
      at = n;
    }
  }
  *faults = pool_faults(base);
  *pool = &p;
  return base + static_cast<size_t>(at) * kRegionWords;
}

// The current device's copy of `scratch`, looked up once per device with that device current.
std::atomic<unsigned long long*> g_static_claims[kMaxDevices];
std::mutex g_static_lock;

int static_claims(unsigned long long** out) {
  int dev = 0;
  const hipError_t d = hipGetDevice(&dev);
  if (d != hipSuccess) return launch_failed(d);
  if (dev < 0 || dev >= kMaxDevices) return UCCL_EINVAL;
  unsigned long long* p = g_static_claims[dev].load(std::memory_order_acquire);
  if (p == nullptr) {
    std::lock_guard<std::mutex> hold(g_static_lock);
    p = g_static_claims[dev].load(std::memory_order_acquire);
    if (p == nullptr) {
      void* at = nullptr;
      const hipError_t e = hipGetSymbolAddress(&at, HIP_SYMBOL(scratch));
      if (e != hipSuccess) return launch_failed(e);
      if (at == nullptr) return UCCL_ELAUNCH;
      p = static_cast<unsigned long long*>(at);
      g_static_claims[dev].store(p, std::memory_order_release);
    }
  }
  *out = p;
  return UCCL_OK;
}

// Per-call tuning (uccl_launch_opts); zero = let the library decide.  static_claims: the call
// must not allocate; records are cut into parts only with these claim words.
struct Tuning {
  uint32_t chunk_bytes;
  uint32_t parts;
  unsigned long long* static_claims = nullptr;
};

template <int T, int U, class Op>
int launch_flat(const Args& a, hipStream_t s) {
  uint32_t tiles = tiles_for(a.n_descs, T);
  if (UCCL_XCD_CONTIGUOUS) tiles = (tiles + 7u) / 8u * 8u;   // whole eighths; tiles past the records find none
  return launch_kernel(chunk_flat_kernel<UCCL_FLAT_THREADS, T, U, Op>, tiles, UCCL_FLAT_THREADS, s, a);
}

// Records per workgroup: enough that a tile holds about 32 KiB of payload per stream when the
// chunk size is known, otherwise grown with the record count.
uint32_t flat_tile(uint32_t n_descs, uint32_t chunk_bytes) {
  uint32_t t;
  if (chunk_bytes) {
    t = (32768u + chunk_bytes - 1) / chunk_bytes;
  } else {
    // Unknown chunk size: a tile too large for big chunks costs a few percent, a tile too
    // small for 4 KiB chunks costs a factor of two, so grow the tile once the record count
    // leaves enough workgroups either way.
    t = n_descs < 8192u ? 1u : n_descs < 32768u ? 4u : n_descs < 131072u ? 8u : 16u;
  }
  return t < 1u ? 1u : t > 32u ? 32u : t;
}

// Calls of fewer single-record tiles than this are launched with chunk_few_kernel (measured with
// 32 / 64 / 128 KiB chunks and no duplicates: 512 records 12-20 % faster than chunk_flat_kernel,
// 1024 records 1-9 %, 2048 records 1-3 %; a duplicate costs chunk_few_kernel its payload reads, so
// large calls, where the difference has gone, stay with chunk_flat_kernel).
#ifndef UCCL_FEW_RECORDS
#define UCCL_FEW_RECORDS 2048
#endif
constexpr uint32_t kFewRecords = UCCL_FEW_RECORDS;
// Payload bytes per stream that one part's wavefronts take in their first, eagerly loaded trip.
constexpr uint32_t kPartBytes = UCCL_PART_THREADS * UCCL_PART_UNROLL * 16u;

// Workgroups per record for a call of few single-record tiles.  One compute unit moves its record's
// 3-4 streams at a small fraction of the memory system's rate, so while the records alone leave
// compute units idle a record is spread over several of them.  Measured (kernel time, fp32 SUM with
// forward, records x chunk size: uncut -> cut): 57 x 64 KiB 6.4 -> 5.2 us in 8 parts; 256 x 64 KiB
// 14.6 -> 12.4 us in 8; 128 x 128 KiB 17.4 -> 12.3 us in 16; 256 x 128 KiB 25.8 -> 24.1 us in 8;
// 32 x 32 KiB 4.4 -> 4.1 us in 8; but 128 x 32 KiB 5.6 -> 5.9 us in 4 and 512 x 64 KiB 24.7 ->
// 25.4 us in 8.  Hence: chunks above 32 KiB are cut into parts of about 8 KiB (at most 16) while
// the call holds at most 16 MiB of payload and the launch stays within 2048 workgroups; chunks of
// up to 32 KiB only in calls of at most 32 records; with the chunk size unknown, by record count
// alone.  Parts that find no unit in a shorter record leave at once.
uint32_t auto_parts(uint32_t n_descs, uint32_t chunk_bytes) {
  if (chunk_bytes == 0u) return n_descs <= 64u ? 8u : n_descs <= 128u ? 4u : 1u;
  if (chunk_bytes <= 32768u) return n_descs <= 32u && chunk_bytes > kPartBytes ? 8u : 1u;
  if (static_cast<uint64_t>(n_descs) * chunk_bytes > (16ull << 20)) return 1u;
  uint32_t parts = 16u;
  while (parts > 1u && parts * kPartBytes > chunk_bytes) parts /= 2u;   // about kPartBytes per part
  while (parts > 1u && n_descs * parts > 2048u) parts /= 2u;
  return parts;
}

// Calls of few small chunks (a message of a few dozen 4 KiB packets) take chunk_few_kernel with one
// small workgroup per record instead of a tile of records per large workgroup: the call is far too
// small to fill the machine either way, and the shorter chain of latencies wins (kernel time, fp32
// SUM with forward, 57 records: 4 KiB 4.7 -> 3.1 us, 8 KiB 5.3 -> 3.3 us, 16 KiB 5.6 -> 3.7 us; 128
// records 15-30 % faster; 512 records of 4 or 8 KiB 15-45 % slower, hence the limit).  Chunks above
// 8 KiB fill a workgroup and keep an edge for much longer (16 KiB: 1024 records 15 % faster, 4096
// records 10 %, 8192 records 1 %); one 16-byte vector per lane of a 1024-thread workgroup covers a
// 16 KiB chunk in one trip and is 2-6 % faster than two vectors per lane of a 512-thread one
// (all-to-all of 3 600 records 21.2 against 21.6 us, 1 024 reduced records 14.3 against 15.3 us).
#ifndef UCCL_SMALL_CALL_RECORDS
#define UCCL_SMALL_CALL_RECORDS 128
#endif
#ifndef UCCL_HALF_TILE_RECORDS
#define UCCL_HALF_TILE_RECORDS 8192
#endif
constexpr uint32_t kSmallCallRecords = UCCL_SMALL_CALL_RECORDS;
constexpr uint32_t kHalfTileRecords = UCCL_HALF_TILE_RECORDS;

// Which launch a call gets: decided here, in one place, from the record count and the tuning alone
// (pure host arithmetic; uccl_launch_plan reports it).  `parts` > 1 is a wish: it needs claim words,
// and a call that finds none (no free region, stream being captured) takes the uncut route instead.
enum Route : uint32_t {
  kRouteTile,       // chunk_flat_kernel, `tile` >= 2 records per workgroup
  kRouteOne,        // chunk_flat_kernel, one record per workgroup
  kRouteFew,        // chunk_few_kernel, one UCCL_FEW_THREADS workgroup per record (calls of < kFewRecords large records)
  kRouteParts,      // chunk_few_kernel, `parts` workgroups of UCCL_PART_THREADS per record
  kRouteHalf,       // chunk_few_kernel<1024, 1>: chunks of 8-16 KiB, one workgroup per record
  kRouteSmall1,     // chunk_few_kernel<256, 1>: at most kSmallCallRecords chunks of up to 4 KiB
  kRouteSmall2,     // chunk_few_kernel<256, 2>: the same, chunks of up to 8 KiB
};
struct Plan {
  Route route;
  uint32_t tile, parts, threads, unroll;
};

Plan plan_apply(uint32_t n_descs, const Tuning& tune, bool reads_acc) {
  const uint32_t t = flat_tile(n_descs, tune.chunk_bytes);
  if (t >= 2 && tune.chunk_bytes > 8192u && n_descs < kHalfTileRecords) return {kRouteHalf, 1u, 1u, 1024u, 1u};
  if (t >= 2 && tune.chunk_bytes != 0u && n_descs <= kSmallCallRecords) {
    // workgroup sized to the chunk: one trip of 16 bytes x unroll per lane covers it
    if (tune.chunk_bytes <= 4096u) return {kRouteSmall1, 1u, 1u, 256u, 1u};
    return {kRouteSmall2, 1u, 1u, 256u, 2u};
  }
  if (t >= 2) return {kRouteTile, t >= 32 ? 32u : t >= 16 ? 16u : t >= 8 ? 8u : t >= 4 ? 4u : 2u, 1u, UCCL_FLAT_THREADS, UCCL_FLAT_UNROLL};
  const uint32_t parts = tune.parts ? tune.parts : (n_descs < kFewRecords ? auto_parts(n_descs, tune.chunk_bytes) : 1u);
  if (parts > 1u && n_descs <= kRegionRecords) return {kRouteParts, 1u, parts, UCCL_PART_THREADS, UCCL_PART_UNROLL};
  if (n_descs < kFewRecords) return {kRouteFew, 1u, 1u, UCCL_FEW_THREADS, UCCL_FEW_UNROLL};
  // One record per workgroup.  Kernels that read the accumulator take 1 KiB units here (a wavefront
  // makes two trips through a 32 KiB chunk, eight through a 128 KiB one, its stores of one trip
  // between the loads of two): measured 0.7 % faster on 32 KiB chunks and 1.9 % on 128 KiB ones
  // than 2 KiB units; copies are 5 % slower that way and keep 2 KiB units.
  const uint32_t unroll = reads_acc ? UCCL_FLAT1_REDUCE_UNROLL : UCCL_FLAT_UNROLL;
  return {kRouteOne, 1u, 1u, UCCL_FLAT_THREADS, unroll};
}

template <class Op>
int launch_flat_tile(Args& a, hipStream_t s, const Tuning& tune) {
  Plan p = plan_apply(a.n_descs, tune, Op::kReadsAcc);
  if (p.route == kRouteParts) {
    if (tune.static_claims != nullptr) {
      // Every call shares the device's one array, which keeps what the last call (or the last replay
      // of this very launch) left in it: clear this call's words first, with a fill kernel (no memset
      // node, so that the pair can be captured), then launch with a tag larger than a cleared word's.
      a.claims = tune.static_claims;
      a.faults = reinterpret_cast<uint32_t*>(tune.static_claims + UCCL_NOALLOC_MAX_DESCS * UCCL_CLAIM_STRIDE);
      a.tag = 1ull;
      a.parts = p.parts;
      const hipEvent_t keep0 = t_start, keep1 = t_stop;  // the timing events belong to the data kernel
      t_start = t_stop = nullptr;
      const uint64_t words = 2ull * a.n_descs * UCCL_CLAIM_STRIDE;
      const int rc = launch_kernel(fill_words_kernel, static_cast<uint32_t>((words + 255) / 256), 256, s,
                                   reinterpret_cast<uint32_t*>(a.claims), words, 0u);
      t_start = keep0;
      t_stop = keep1;
      if (rc != UCCL_OK) { t_start = t_stop = nullptr; return rc; }
      return launch_kernel(chunk_few_kernel<UCCL_PART_THREADS, UCCL_PART_UNROLL, Op, true>, a.n_descs * p.parts,
                           UCCL_PART_THREADS, s, a);
    }
    ClaimPool* pool = nullptr;
    a.claims = claim_region(s, &a.faults, &pool);
    if (a.claims != nullptr) {
      std::lock_guard<std::mutex> in_order(pool->launch_lock);
      a.tag = g_next_tag.fetch_add(1, std::memory_order_relaxed);
      a.parts = p.parts;
      return launch_kernel(chunk_few_kernel<UCCL_PART_THREADS, UCCL_PART_UNROLL, Op, true>, a.n_descs * p.parts,
                           UCCL_PART_THREADS, s, a);
    }
    p.route = a.n_descs < kFewRecords ? kRouteFew : kRouteOne;   // no claim words to be had: uncut
  }
  switch (p.route) {
    case kRouteHalf: return launch_kernel(chunk_few_kernel<1024, 1, Op, false>, a.n_descs, 1024, s, a);
    case kRouteSmall1: return launch_kernel(chunk_few_kernel<256, 1, Op, false>, a.n_descs, 256, s, a);
    case kRouteSmall2: return launch_kernel(chunk_few_kernel<256, 2, Op, false>, a.n_descs, 256, s, a);
    case kRouteFew:
      return launch_kernel(chunk_few_kernel<UCCL_FEW_THREADS, UCCL_FEW_UNROLL, Op, false>, a.n_descs,
                           UCCL_FEW_THREADS, s, a);
    case kRouteTile:
      if (p.tile >= 32) return launch_flat<32, UCCL_FLAT_UNROLL, Op>(a, s);
      if (p.tile >= 16) return launch_flat<16, UCCL_FLAT_UNROLL, Op>(a, s);
      if (p.tile >= 8) return launch_flat<8, UCCL_FLAT_UNROLL, Op>(a, s);
      if (p.tile >= 4) return launch_flat<4, UCCL_FLAT_UNROLL, Op>(a, s);
      return launch_flat<2, UCCL_FLAT_UNROLL, Op>(a, s);
    default: return launch_flat<1, Op::kReadsAcc ? UCCL_FLAT1_REDUCE_UNROLL : UCCL_FLAT_UNROLL, Op>(a, s);
  }
}

template <int T, class Op>
int launch_gather(const GatherArgs& a, hipStream_t s) {
  return launch_kernel(chunk_gather_kernel<1024, T, UCCL_GATHER_UNROLL, Op>, tiles_for(a.n_descs, T), 1024, s, a);
}

// Workgroups per multi-source record for a call of few of them.  A record moves n + 2 streams of its
// length through one compute unit, so cutting pays from 32 KiB chunks on (measured with seven
// sources, kernel time uncut -> cut: 8 x 128 KiB 24.9 -> 6.0 us in 16 parts; 32 x 64 KiB 16.1 ->
// 6.7 us in 8; 128 x 32 KiB 12.3 -> 10.1 us in 4; 128 x 128 KiB 35.4 -> 28.1 us in 16; 512 x 32 KiB
// 32.2 -> 32.0 us in 4): parts of about 8 KiB, at most 16, while the call has at most 16 MiB of
// destination payload and the launch stays within 2048 workgroups; with the chunk size unknown, by
// record count alone.
uint32_t gather_parts(uint32_t n_descs, uint32_t chunk_bytes) {
  if (chunk_bytes == 0u) return n_descs <= 64u ? 8u : n_descs <= 128u ? 4u : 1u;
  if (static_cast<uint64_t>(n_descs) * chunk_bytes > (16ull << 20)) return 1u;
  uint32_t parts = 16u;
  while (parts > 1u && parts * kPartBytes > chunk_bytes) parts /= 2u;
  while (parts > 1u && n_descs * parts > 2048u) parts /= 2u;
  return parts;
}

Plan plan_gather(uint32_t n_descs, const Tuning& tune) {
  const uint32_t t = flat_tile(n_descs, tune.chunk_bytes);
  if (t >= 2) return {kRouteTile, t >= 16 ? 16u : t >= 8 ? 8u : t >= 4 ? 4u : 2u, 1u, 1024u, UCCL_GATHER_UNROLL};
  const uint32_t parts = tune.parts ? tune.parts : gather_parts(n_descs, tune.chunk_bytes);
  if (parts > 1u && n_descs <= kRegionRecords) return {kRouteParts, 1u, parts, UCCL_PART_THREADS, UCCL_GATHER_UNROLL};
  return {kRouteOne, 1u, 1u, 1024u, UCCL_GATHER_UNROLL};
}

template <class Op>
int launch_gather_tile(GatherArgs& a, hipStream_t s, const Tuning& tune) {
  const Plan p = plan_gather(a.n_descs, tune);
  if (p.route == kRouteTile) {
    if (p.tile >= 16) return launch_gather<16, Op>(a, s);
    if (p.tile >= 8) return launch_gather<8, Op>(a, s);
    if (p.tile >= 4) return launch_gather<4, Op>(a, s);
    return launch_gather<2, Op>(a, s);
  }
  if (p.route == kRouteParts) {
    ClaimPool* pool = nullptr;
    a.claims = claim_region(s, &a.faults, &pool);
    if (a.claims != nullptr) {
      std::lock_guard<std::mutex> in_order(pool->launch_lock);
      a.tag = g_next_tag.fetch_add(1, std::memory_order_relaxed);
      a.parts = p.parts;
      return launch_kernel(chunk_gather_parts_kernel<UCCL_PART_THREADS, UCCL_GATHER_UNROLL, Op>, a.n_descs * p.parts,
                           UCCL_PART_THREADS, s, a);
    }
  }
  return launch_gather<1, Op>(a, s);
}

bool misaligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

bool overlaps(const void* p, uint64_t pn, const void* q, uint64_t qn) {
  if (!p || !q || pn == 0 || qn == 0) return false;
  const uintptr_t a = reinterpret_cast<uintptr_t>(p), b = reinterpret_cast<uintptr_t>(q);
  return a < b + qn && b < a + pn;
}

bool tuning_from(const uccl_launch_opts* opts, Tuning* t) {
  *t = Tuning{0u, 0u, nullptr};
  if (opts == nullptr) return true;
  if (opts->parts > 16u || opts->reserved[0] != 0u || opts->reserved[1] != 0u) return false;
  *t = Tuning{opts->chunk_bytes, opts->parts, nullptr};
  return true;
}

int apply_common(void* acc, void* out_stage, const void* recv_stage, const uccl_chunk_desc* descs,
                 uint32_t n_descs, uint32_t* bitmap, int dtype, int op, bool allow_forward,
                 const uccl_extents* ext, uint32_t* n_rejected, const Tuning& tune, void* stream,
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
  a.claims = nullptr;
  a.faults = nullptr;
  a.parts = 1u;
  a.tag = 0ull;
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
  if (op == UCCL_COPY) return launch_flat_tile<Copy>(a, s, tune);
  switch (dtype * 8 + op) {
    case UCCL_F32 * 8 + UCCL_SUM: return launch_flat_tile<OpF32<kSum>>(a, s, tune);
    case UCCL_F32 * 8 + UCCL_MAX: return launch_flat_tile<OpF32<kMax>>(a, s, tune);
    case UCCL_F32 * 8 + UCCL_MIN: return launch_flat_tile<OpF32<kMin>>(a, s, tune);
    case UCCL_F32 * 8 + UCCL_PROD: return launch_flat_tile<OpF32<kProd>>(a, s, tune);
    case UCCL_BF16 * 8 + UCCL_SUM: return launch_flat_tile<Op16<kSum, WidenBF16>>(a, s, tune);
    case UCCL_BF16 * 8 + UCCL_MAX: return launch_flat_tile<Op16<kMax, WidenBF16>>(a, s, tune);
    case UCCL_BF16 * 8 + UCCL_MIN: return launch_flat_tile<Op16<kMin, WidenBF16>>(a, s, tune);
    case UCCL_BF16 * 8 + UCCL_PROD: return launch_flat_tile<Op16<kProd, WidenBF16>>(a, s, tune);
    case UCCL_F16 * 8 + UCCL_SUM: return launch_flat_tile<Op16<kSum, WidenF16>>(a, s, tune);
    case UCCL_F16 * 8 + UCCL_MAX: return launch_flat_tile<Op16<kMax, WidenF16>>(a, s, tune);
    case UCCL_F16 * 8 + UCCL_MIN: return launch_flat_tile<Op16<kMin, WidenF16>>(a, s, tune);
    case UCCL_F16 * 8 + UCCL_PROD: return launch_flat_tile<Op16<kProd, WidenF16>>(a, s, tune);
    case UCCL_I32 * 8 + UCCL_SUM: return launch_flat_tile<OpI32<kSum>>(a, s, tune);
    case UCCL_I32 * 8 + UCCL_MAX: return launch_flat_tile<OpI32<kMax>>(a, s, tune);
    case UCCL_I32 * 8 + UCCL_MIN: return launch_flat_tile<OpI32<kMin>>(a, s, tune);
    case UCCL_I32 * 8 + UCCL_PROD: return launch_flat_tile<OpI32<kProd>>(a, s, tune);
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
  uint32_t max_len[2];  // largest payload length among the lane's records: the hand-over's chunk size
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
                                f->dtype, f->op[l], true, nullptr, nullptr, Tuning{sl.max_len[l], 0u, nullptr},
                                f->stream);
    if (rc != UCCL_OK) return rc;
  }
  const hipError_t e = hipEventRecord(sl.done, f->stream);
  if (e != hipSuccess) return launch_failed(e);
  sl.in_flight = true;
  f->stats.flushes += 1;
  f->stats.records += n;
  if (n > f->stats.max_batch) f->stats.max_batch = n;
  sl.count[0] = sl.count[1] = 0;
  sl.max_len[0] = sl.max_len[1] = 0;
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
    for (uint32_t i = 0; i < take; ++i)
      if (host_records[i].len > sl.max_len[lane]) sl.max_len[lane] = host_records[i].len;
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
                      nullptr, nullptr, Tuning{0u, 0u, nullptr}, stream);
}

int uccl_chunk_apply_opts(void* acc, void* out_stage, const void* recv_stage,
                          const uccl_chunk_desc* descs, uint32_t n_descs, uint32_t* dedup_bitmap,
                          uccl_dtype dtype, uccl_op op, const uccl_extents* extents,
                          uint32_t* n_rejected, const uccl_launch_opts* opts, void* stream) {
  Tuning tune;
  if (!tuning_from(opts, &tune)) return UCCL_EINVAL;
  return apply_common(acc, out_stage, recv_stage, descs, n_descs, dedup_bitmap, dtype, op, true,
                      extents, n_rejected, tune, stream);
}

int uccl_chunk_apply_checked(void* acc, void* out_stage, const void* recv_stage,
                             const uccl_chunk_desc* descs, uint32_t n_descs,
                             uint32_t* dedup_bitmap, uccl_dtype dtype, uccl_op op,
                             const uccl_extents* extents, uint32_t* n_rejected, void* stream) {
  if (!extents) return UCCL_EINVAL;
  return apply_common(acc, out_stage, recv_stage, descs, n_descs, dedup_bitmap, dtype, op, true,
                      extents, n_rejected, Tuning{0u, 0u, nullptr}, stream);
}

int uccl_chunk_apply_indirect(void* acc, void* out_stage, const void* recv_stage,
                              const uccl_chunk_desc* descs, const uint32_t* n_descs_ptr,
                              uint32_t max_descs, uint32_t* dedup_bitmap, uccl_dtype dtype,
                              uccl_op op, const uccl_extents* extents, uint32_t* n_rejected,
                              const uccl_launch_opts* opts, void* stream) {
  if (max_descs > 0 && !n_descs_ptr) return UCCL_EINVAL;
  Tuning tune;
  if (!tuning_from(opts, &tune)) return UCCL_EINVAL;
  return apply_common(acc, out_stage, recv_stage, descs, max_descs, dedup_bitmap, dtype, op, true,
                      extents, n_rejected, tune, stream, n_descs_ptr);
}

int uccl_chunk_reduce_gather(void* acc, void* out_stage, const void* recv_stage,
                             const uccl_gather_desc* descs, uint32_t n_descs, uint32_t* dedup_bitmap,
                             uccl_dtype dtype, uccl_op op, const uccl_extents* extents,
                             uint32_t* n_rejected, const uccl_launch_opts* opts, void* stream) {
  if (dtype < UCCL_F32 || dtype > UCCL_I32) return UCCL_EINVAL;
  if (op != UCCL_SUM && op != UCCL_MAX && op != UCCL_MIN && op != UCCL_PROD) return UCCL_EINVAL;
  Tuning tune;
  if (!tuning_from(opts, &tune)) return UCCL_EINVAL;
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
  a.claims = nullptr;
  a.faults = nullptr;
  a.tag = 0ull;
  a.parts = 1u;
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
    case UCCL_F32 * 8 + UCCL_SUM: return launch_gather_tile<OpF32<kSum>>(a, s, tune);
    case UCCL_F32 * 8 + UCCL_MAX: return launch_gather_tile<OpF32<kMax>>(a, s, tune);
    case UCCL_F32 * 8 + UCCL_MIN: return launch_gather_tile<OpF32<kMin>>(a, s, tune);
    case UCCL_F32 * 8 + UCCL_PROD: return launch_gather_tile<OpF32<kProd>>(a, s, tune);
    case UCCL_BF16 * 8 + UCCL_SUM: return launch_gather_tile<Op16<kSum, WidenBF16>>(a, s, tune);
    case UCCL_BF16 * 8 + UCCL_MAX: return launch_gather_tile<Op16<kMax, WidenBF16>>(a, s, tune);
    case UCCL_BF16 * 8 + UCCL_MIN: return launch_gather_tile<Op16<kMin, WidenBF16>>(a, s, tune);
    case UCCL_BF16 * 8 + UCCL_PROD: return launch_gather_tile<Op16<kProd, WidenBF16>>(a, s, tune);
    case UCCL_F16 * 8 + UCCL_SUM: return launch_gather_tile<Op16<kSum, WidenF16>>(a, s, tune);
    case UCCL_F16 * 8 + UCCL_MAX: return launch_gather_tile<Op16<kMax, WidenF16>>(a, s, tune);
    case UCCL_F16 * 8 + UCCL_MIN: return launch_gather_tile<Op16<kMin, WidenF16>>(a, s, tune);
    case UCCL_F16 * 8 + UCCL_PROD: return launch_gather_tile<Op16<kProd, WidenF16>>(a, s, tune);
    case UCCL_I32 * 8 + UCCL_SUM: return launch_gather_tile<OpI32<kSum>>(a, s, tune);
    case UCCL_I32 * 8 + UCCL_MAX: return launch_gather_tile<OpI32<kMax>>(a, s, tune);
    case UCCL_I32 * 8 + UCCL_MIN: return launch_gather_tile<OpI32<kMin>>(a, s, tune);
    case UCCL_I32 * 8 + UCCL_PROD: return launch_gather_tile<OpI32<kProd>>(a, s, tune);
    default: return UCCL_EINVAL;
  }
}

int uccl_chunk_scatter(void* dst, const void* recv_stage, const uccl_chunk_desc* descs,
                       uint32_t n_descs, uint32_t* dedup_bitmap, void* stream) {
  return apply_common(dst, nullptr, recv_stage, descs, n_descs, dedup_bitmap, UCCL_BF16, UCCL_COPY,
                      false, nullptr, nullptr, Tuning{0u, 0u, nullptr}, stream);
}

int uccl_chunk_scatter_checked(void* dst, const void* recv_stage, const uccl_chunk_desc* descs,
                               uint32_t n_descs, uint32_t* dedup_bitmap,
                               const uccl_extents* extents, uint32_t* n_rejected, void* stream) {
  if (!extents) return UCCL_EINVAL;
  return apply_common(dst, nullptr, recv_stage, descs, n_descs, dedup_bitmap, UCCL_BF16, UCCL_COPY,
                      false, extents, n_rejected, Tuning{0u, 0u, nullptr}, stream);
}

int uccl_chunk_scatter_opts(void* dst, const void* recv_stage, const uccl_chunk_desc* descs,
                            uint32_t n_descs, uint32_t* dedup_bitmap, const uccl_extents* extents,
                            uint32_t* n_rejected, const uccl_launch_opts* opts, void* stream) {
  Tuning tune;
  if (!tuning_from(opts, &tune)) return UCCL_EINVAL;
  return apply_common(dst, nullptr, recv_stage, descs, n_descs, dedup_bitmap, UCCL_BF16, UCCL_COPY,
                      false, extents, n_rejected, tune, stream);
}

int uccl_init(void) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return launch_failed(hipGetLastError());
  if (dev < 0 || dev >= kMaxDevices) return UCCL_EINVAL;
  unsigned long long* fixed = nullptr;
  const int rc = static_claims(&fixed);
  if (rc != UCCL_OK) return rc;
  return pool_base(dev, true) != nullptr ? UCCL_OK : UCCL_ENOMEM;
}

int uccl_chunk_apply_noalloc(void* acc, void* out_stage, const void* recv_stage,
                             const uccl_chunk_desc* descs, uint32_t n_descs, uint32_t* dedup_bitmap,
                             uccl_dtype dtype, uccl_op op, void* stream) {
  if (dtype < UCCL_F32 || dtype > UCCL_I32) return UCCL_EINVAL;
  if (op < UCCL_SUM || op > UCCL_PROD) return UCCL_EINVAL;
  if (n_descs > UCCL_NOALLOC_MAX_DESCS) return UCCL_ETOOBIG;
  if (n_descs == 0) return UCCL_OK;
  Tuning tune{0u, 0u, nullptr};
  const int rc = static_claims(&tune.static_claims);
  if (rc != UCCL_OK) return rc;
  return apply_common(acc, out_stage, recv_stage, descs, n_descs, dedup_bitmap, dtype, op, true,
                      nullptr, nullptr, tune, stream);
}

int uccl_claim_timeouts(uint64_t* count) {
  if (!count) return UCCL_EINVAL;
  *count = 0;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return launch_failed(hipGetLastError());
  if (dev < 0 || dev >= kMaxDevices) return UCCL_EINVAL;
  uint64_t total = 0;
  unsigned long long* base = pool_base(dev, false);
  if (base != nullptr) {  // no pool: no split call through it so far
    uint32_t n = 0;
    const hipError_t e = hipMemcpy(&n, pool_faults(base), sizeof(n), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return launch_failed(e);
    total += n;
  }
  unsigned long long* fixed = g_static_claims[dev].load(std::memory_order_acquire);
  if (fixed != nullptr) {
    uint32_t n = 0;
    const hipError_t e = hipMemcpy(&n, fixed + UCCL_NOALLOC_MAX_DESCS * UCCL_CLAIM_STRIDE, sizeof(n), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return launch_failed(e);
    total += n;
  }
  *count = total;
  return UCCL_OK;
}

int uccl_chunk_segment(void* out_stage, const void* tensor, uint64_t tensor_off, uint64_t bytes,
                       uint32_t chunk_bytes, uint64_t stage_off, uint64_t slot_stride,
                       uccl_send_desc* send_descs, uint32_t conn_id, uint32_t msg_id, uint32_t first_csn,
                       void* stream) {
  if (conn_id > 255u || msg_id > 127u || chunk_bytes == 0u) return UCCL_EINVAL;
  if ((chunk_bytes & 15u) || (tensor_off & 15u) || (stage_off & 15u) || (slot_stride & 15u)) return UCCL_EALIGN;
  if (slot_stride < chunk_bytes) return UCCL_EINVAL;
  if (bytes == 0) return UCCL_OK;
  if (!out_stage || !tensor) return UCCL_EINVAL;
  if (misaligned(out_stage, 16) || misaligned(tensor, 16) || misaligned(send_descs, 8)) return UCCL_EALIGN;
  const uint64_t n_chunks = (bytes + chunk_bytes - 1) / chunk_bytes;
  if (n_chunks > 0xFFFFFFFFull) return UCCL_EINVAL;
  SegmentArgs a;
  a.stage = static_cast<char*>(out_stage) + stage_off;
  a.tensor = static_cast<const char*>(tensor) + tensor_off;
  a.descs = send_descs;
  a.bytes = bytes;
  a.slot_stride = slot_stride;
  a.stage_off = stage_off;
  a.n_chunks = n_chunks;
  a.chunk_bytes = chunk_bytes;
  a.units_per_chunk = (chunk_bytes + 2047u) / 2048u;
  a.conn_id = conn_id;
  a.msg_id = msg_id;
  a.first_csn = first_csn;
  const uint64_t groups = (n_chunks * a.units_per_chunk + 15) / 16;  // 16 units per workgroup
  if (groups > 0x7FFFFFFFull) return UCCL_EINVAL;
  return launch_kernel(segment_kernel, static_cast<uint32_t>(groups), 1024, static_cast<hipStream_t>(stream), a);
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

int uccl_launch_plan(uint32_t n_descs, const uccl_launch_opts* opts, int gather, int reads_acc, uccl_plan* plan) {
  Tuning tune;
  if (!plan || !tuning_from(opts, &tune)) return UCCL_EINVAL;
  const Plan p = gather ? plan_gather(n_descs, tune) : plan_apply(n_descs, tune, reads_acc != 0);
  const bool few = !gather && p.route != kRouteTile && p.route != kRouteOne;
  plan->kernel = gather ? (p.route == kRouteParts ? UCCL_KERNEL_GATHER_PARTS : UCCL_KERNEL_GATHER)
                        : (few ? UCCL_KERNEL_FEW : UCCL_KERNEL_FLAT);
  plan->records_per_group = p.tile;
  plan->parts = p.parts;
  plan->threads = p.threads;
  plan->unit_bytes = 64u * 16u * p.unroll;
  const uint64_t groups = p.route == kRouteTile ? tiles_for(n_descs, p.tile) : static_cast<uint64_t>(n_descs) * p.parts;
  plan->groups = static_cast<uint32_t>(groups);
  plan->reserved[0] = plan->reserved[1] = 0u;
  return UCCL_OK;
}

int uccl_time_next_launch(void* start_event, void* stop_event) {
  t_start = static_cast<hipEvent_t>(start_event);
  t_stop = static_cast<hipEvent_t>(stop_event);
  return UCCL_OK;
}

const char* uccl_strerror(int code) {
  switch (code) {
    case UCCL_OK: return "ok";
    case UCCL_EINVAL: return "invalid argument";
    case UCCL_EALIGN: return "misaligned pointer";
    case UCCL_ELAUNCH: return "HIP launch failed";
    case UCCL_ENOMEM: return "out of memory";
    case UCCL_ETOOBIG: return "too many records for this entry point";
    default: return "unknown error code";
  }
}

const char* uccl_last_error_detail(void) { return t_detail; }

int uccl_version(void) { return UCCL_CHUNK_VERSION; }

}  // extern "C"
