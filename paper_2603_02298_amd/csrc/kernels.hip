// HIP kernels for gfx950 (CDNA4, wave64) that execute a planned COPY (Sec. 2.6.1 of "CuTe Layout
// Representation and Algebra"): dst(i) = src(i) with the iteration order permuted consistently on
// both sides (Sec. 3.4.2) so that global accesses are wide and coalesced.  No MFMA: the work is
// pure data movement and is bounded by HBM bandwidth.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <map>
#include <mutex>
#include <string>
#include <utility>

#include "kernel_params.hpp"
#include "plan.hpp"

namespace lc {

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int W> struct Word;
template <> struct Word<1> { typedef uint8_t type; };
template <> struct Word<2> { typedef uint16_t type; };
template <> struct Word<4> { typedef uint32_t type; };
template <> struct Word<8> { typedef u32x2 type; };
template <> struct Word<16> { typedef u32x4 type; };

// NT: bit 0 = nontemporal loads, bit 1 = nontemporal stores (streaming data is touched once)
template <int NT, typename T>
__device__ __forceinline__ T gload(const T* p) {
  if (NT & 1) return __builtin_nontemporal_load(p);
  return *p;
}
template <int NT, typename T>
__device__ __forceinline__ void gstore(T* p, T v) {
  if (NT & 2) __builtin_nontemporal_store(v, p);
  else *p = v;
}

// Reads one dword of every 64-byte line of the kernel-argument block, all at once.  The blocks here
// span up to a dozen lines and their fields are needed one group after the other; without this
// each group's first use pays its own scalar-cache miss, in series, before the first global load.
template <int BYTES>
__device__ __forceinline__ void touch_kernel_arguments() {
  typedef const uint32_t __attribute__((address_space(4))) * KernargPtr;
  KernargPtr ka = (KernargPtr)__builtin_amdgcn_kernarg_segment_ptr();
  constexpr int LINES = (BYTES + 63) / 64;
  static_assert(LINES <= 16, "one scalar register per line");
  uint32_t t[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) t[i] = ka[(i < LINES ? i : 0) * 16];
  // a use the compiler cannot move or split: all loads are issued together, and waited for, here
  asm volatile("" ::"s"(t[0]), "s"(t[1]), "s"(t[2]), "s"(t[3]), "s"(t[4]), "s"(t[5]), "s"(t[6]), "s"(t[7]), "s"(t[8]), "s"(t[9]),
               "s"(t[10]), "s"(t[11]), "s"(t[12]), "s"(t[13]), "s"(t[14]), "s"(t[15]));
}

// ---------------------------------------------------------------------------------------------
// Element-wise: both layouts evaluated per element (idx2crd + inner_product, Eq. idx2crd / Eq. innerprod).
// ---------------------------------------------------------------------------------------------
template <int ES>
__global__ __launch_bounds__(kBlock) void generic_kernel(GenericParams P, const typename Word<ES>::type* __restrict__ src,
                                                        typename Word<ES>::type* __restrict__ dst) {
  touch_kernel_arguments<(int)sizeof(GenericParams)>();
  const uint32_t step = gridDim.x * kBlock;
  for (uint32_t i = blockIdx.x * kBlock + threadIdx.x; i < P.n; i += step) dst[flat_eval(P.dst, i)] = src[flat_eval(P.src, i)];
}

// ---------------------------------------------------------------------------------------------
// Last writer: a destination that maps several integral coordinates to one offset keeps what Sec. 2.6.1's loop (i ascending)
// writes there last, the value of the largest such coordinate.  Pass 1 records that coordinate per offset (atomic maximum
// into a zeroed word per destination offset), pass 2 lets exactly the recorded coordinates write.  Coordinate 0 needs no
// record of its own: an offset only it reaches keeps the zero the scratch memory starts with.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void zero_words_kernel(uint32_t* __restrict__ words, uint64_t n) {
  const uint64_t step = (uint64_t)gridDim.x * kBlock;
  for (uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += step) words[i] = 0u;
}
// `last` points at the record of destination offset 0 (offsets below 0 exist with negative strides: the records start lower)
__global__ __launch_bounds__(kBlock) void last_writer_mark_kernel(GenericParams P, uint32_t* __restrict__ last) {
  touch_kernel_arguments<(int)sizeof(GenericParams)>();
  const uint32_t step = gridDim.x * kBlock;
  for (uint32_t i = blockIdx.x * kBlock + threadIdx.x; i < P.n; i += step) atomicMax(last + flat_eval(P.dst, i), i);
}
template <int ES>
__global__ __launch_bounds__(kBlock) void last_writer_move_kernel(GenericParams P, const typename Word<ES>::type* __restrict__ src,
                                                                 typename Word<ES>::type* __restrict__ dst, const uint32_t* __restrict__ last) {
  touch_kernel_arguments<(int)sizeof(GenericParams)>();
  const uint32_t step = gridDim.x * kBlock;
  for (uint32_t i = blockIdx.x * kBlock + threadIdx.x; i < P.n; i += step) {
    const int64_t off = flat_eval(P.dst, i);
    if (last[off] == i) dst[off] = src[flat_eval(P.src, i)];
  }
}

// Tile queues: blocks of counters in device memory that belongs to the library's code object: nothing is allocated.
// A block is kQueueLines lines of 128 bytes with one counter at the start of each, so that no two counters share a cache
// line: line 0 counts the workgroups that are done, lines 1.. count the tiles handed out (a launch spreads its requests
// over up to kQueueLines - 1 of them, workgroup w asking counter w mod n); the one-counter form of the transposing kernel
// uses the second word of line 0 instead.  Launches on one stream run one after the
// other, so a stream keeps one block for good; the host hands out kTileQueues blocks and launches on further streams, or
// under graph capture, use the fixed order.
constexpr int kTileQueues = 64;
constexpr int kQueueLines = 16;
constexpr int kQueueLineWords = 32;   // 128 bytes
constexpr int kQueueBlockWords = kQueueLines * kQueueLineWords;
__device__ __attribute__((aligned(256))) unsigned int g_tile_queues[kTileQueues * kQueueBlockWords];
__device__ __forceinline__ void leave_tile_queue(unsigned int* queue) {
  if (atomicAdd(&queue[0], 1u) == gridDim.x - 1u) {   // the last workgroup out: nobody asks any more
#pragma unroll
    for (int c = 0; c < kQueueLines; ++c) queue[c * kQueueLineWords] = 0u;
    queue[1] = 0u;   // the one-counter form of the transposing kernel counts its tiles here
    __threadfence();
  }
}

// ---------------------------------------------------------------------------------------------
// Direct: one W-byte access per item and side; lanes are consecutive along the destination order.
// U items are in flight per lane; an optional looped mode re-uses a loaded value when its source
// stride is zero (broadcast).
// ---------------------------------------------------------------------------------------------
// item -> offsets through `offsets(item, &so, &dof)`; everything else by value
template <int W, int U, int NT, class Offsets>
__device__ __forceinline__ void direct_body(const typename Word<W>::type* __restrict__ src, typename Word<W>::type* __restrict__ dst,
                                            uint32_t n_items, bool blocked, uint32_t loop_extent, int64_t loop_sa, int64_t loop_sb,
                                            Offsets offsets) {
  typedef typename Word<W>::type T;
  // strided: lane items are `step` apart and the whole grid sweeps memory together;
  // blocked: a workgroup owns the contiguous range [first, last) and sweeps it kBlock items at a time
  uint32_t step = gridDim.x * kBlock, first = blockIdx.x * kBlock, last = n_items;
  if (blocked) {
    uint32_t chunk = (n_items + gridDim.x - 1) / gridDim.x;
    chunk = (chunk + kBlock * U - 1) / (kBlock * U) * (kBlock * U);
    step = kBlock;
    first = blockIdx.x * chunk;
    last = min(n_items, first + chunk);
    if (blockIdx.x * (uint64_t)chunk >= n_items) return;
  }
  for (uint32_t base = first + threadIdx.x; base < last; base += step * U) {
    int64_t so[U], dof[U];
    bool ok[U];
    T v[U];
#pragma unroll
    for (int j = 0; j < U; ++j) {
      uint32_t it = base + (uint32_t)j * step;
      ok[j] = it < last;
      so[j] = dof[j] = 0;
      if (ok[j]) offsets(it, &so[j], &dof[j]);
    }
    if (loop_extent == 1) {
#pragma unroll
      for (int j = 0; j < U; ++j) if (ok[j]) v[j] = gload<NT>(src + so[j]);
#pragma unroll
      for (int j = 0; j < U; ++j) if (ok[j]) gstore<NT>(dst + dof[j], v[j]);
    } else if (loop_sa == 0) {
#pragma unroll
      for (int j = 0; j < U; ++j) if (ok[j]) v[j] = gload<NT>(src + so[j]);
      for (uint32_t r = 0; r < loop_extent; ++r) {
#pragma unroll
        for (int j = 0; j < U; ++j) if (ok[j]) gstore<NT>(dst + dof[j] + (int64_t)r * loop_sb, v[j]);
      }
    } else {
      for (uint32_t r = 0; r < loop_extent; ++r) {
#pragma unroll
        for (int j = 0; j < U; ++j) if (ok[j]) v[j] = gload<NT>(src + so[j] + (int64_t)r * loop_sa);
#pragma unroll
        for (int j = 0; j < U; ++j) if (ok[j]) gstore<NT>(dst + dof[j] + (int64_t)r * loop_sb, v[j]);
      }
    }
  }
}

// The same work handed out on request: the items are cut into chunks of chunk_items consecutive items (about 32 KiB of
// destination), wavefront w starts on chunk w and asks a counter for every further one -- lane 0 asks, one chunk ahead, and
// the answer reaches the other lanes by v_readfirstlane: no barrier, no LDS.  In a grid-stride loop over gigabytes the
// workgroups drift apart and what is in flight at any moment spreads over memory; chunks taken in the order of asking keep
// it one compact window (measured on MI355X, plain copy of 2 x 2 GiB: 72-75 -> 76-77 % of the HBM peak; at 2 x 1 GiB and below
// the fixed order is faster, so the planner asks for chunks from 2 GiB per side on).  Counter c of n_counters hands out the chunks waves + c, waves + c + n_counters, ...; queue[0] counts
// the wavefronts that are done and the last one puts the counters back to zero (see the tile queues above).
template <int W, int U, int NT, bool LINEAR, class Offsets>
__device__ __forceinline__ void direct_body_on_request(const typename Word<W>::type* __restrict__ src, typename Word<W>::type* __restrict__ dst,
                                                       uint32_t n_items, uint32_t loop_extent, int64_t loop_sa, int64_t loop_sb,
                                                       unsigned int* queue, uint32_t chunk_items, uint32_t n_counters,
                                                       int64_t lin_sa, int64_t lin_sb, Offsets offsets) {
  typedef typename Word<W>::type T;
  const uint32_t lane = threadIdx.x & 63u, wave = (blockIdx.x * kBlock + threadIdx.x) >> 6, waves = gridDim.x * (kBlock / 64u);
  const uint32_t n_chunks = (n_items + chunk_items - 1u) / chunk_items, c = wave % n_counters;
  unsigned int* counter = queue + (1u + c) * kQueueLineWords;
  uint32_t chunk = wave;
  while (chunk < n_chunks) {
    uint32_t asked = 0;
    if (lane == 0) asked = atomicAdd(counter, 1u);
    const uint32_t first = chunk * chunk_items;
    if (LINEAR && loop_extent == 1 && n_items - first >= chunk_items) {
      // one joint mode: the offsets are item * stride, so a lane steps two pointers through the chunk
      const T* sp = src + (int64_t)(first + lane) * lin_sa;
      T* dp = dst + (int64_t)(first + lane) * lin_sb;
      const int64_t s64 = 64 * lin_sa, d64 = 64 * lin_sb;
      for (uint32_t t = 0; t < chunk_items; t += 64u * U, sp += U * s64, dp += U * d64) {
        T v[U];
#pragma unroll
        for (int j = 0; j < U; ++j) v[j] = gload<NT>(sp + j * s64);
#pragma unroll
        for (int j = 0; j < U; ++j) gstore<NT>(dp + j * d64, v[j]);
      }
    } else if (n_items - first >= chunk_items) {
      // a whole chunk (chunk_items is a multiple of 64 U): no lane is ever idle, so nothing here is predicated and the U
      // loads of a trip go out together
      for (uint32_t base = first + lane; base < first + chunk_items; base += 64u * U) {
        int64_t so[U], dof[U];
        T v[U];
#pragma unroll
        for (int j = 0; j < U; ++j) offsets(base + (uint32_t)j * 64u, &so[j], &dof[j]);
        if (loop_extent == 1) {
#pragma unroll
          for (int j = 0; j < U; ++j) v[j] = gload<NT>(src + so[j]);
#pragma unroll
          for (int j = 0; j < U; ++j) gstore<NT>(dst + dof[j], v[j]);
        } else {
          for (uint32_t r = 0; r < loop_extent; ++r) {
            if (r == 0 || loop_sa != 0) {
#pragma unroll
              for (int j = 0; j < U; ++j) v[j] = gload<NT>(src + so[j] + (int64_t)r * loop_sa);
            }
#pragma unroll
            for (int j = 0; j < U; ++j) gstore<NT>(dst + dof[j] + (int64_t)r * loop_sb, v[j]);
          }
        }
      }
    } else {
      // the last, short chunk: item by item
      for (uint32_t it = first + lane; it < n_items; it += 64u) {
        int64_t so, dof;
        offsets(it, &so, &dof);
        T v = gload<NT>(src + so);
        for (uint32_t r = 0; r < loop_extent; ++r) {
          if (r != 0 && loop_sa != 0) v = gload<NT>(src + so + (int64_t)r * loop_sa);
          gstore<NT>(dst + dof + (int64_t)r * loop_sb, v);
        }
      }
    }
    asked = (uint32_t)__builtin_amdgcn_readfirstlane((int)asked);
    chunk = waves + c + asked * n_counters;
  }
  if (lane == 0 && atomicAdd(&queue[0], 1u) == waves - 1u) {   // the last wavefront out: nobody asks any more
#pragma unroll
    for (int k = 0; k < kQueueLines; ++k) queue[k * kQueueLineWords] = 0u;
    __threadfence();
  }
}

// The leading scalar arguments (fourteen dwords, preloaded into scalar registers where the hardware does it) describe a
// copy over ONE joint mode completely (a plain copy, a strided gather or scatter, a broadcast): with h_ctl's bit 0 set the
// kernel never reads the argument block and its first loads wait for no memory.  h_ctl: bit 0 valid, bit 1 blocked,
// bits 2.. the looped mode's extent.
template <int W, int U, int NT>
__global__ __launch_bounds__(kBlock) void direct_kernel(const typename Word<W>::type* __restrict__ src, typename Word<W>::type* __restrict__ dst,
                                                       uint32_t h_ctl, uint32_t h_items, int64_t h_sa, int64_t h_sb, int64_t h_loop_sa,
                                                       int64_t h_loop_sb, DirectParams P, unsigned int* queue, uint32_t chunk_items,
                                                       uint32_t n_counters) {
  if (queue != nullptr) {   // long copies: chunks on request
    if (h_ctl & 1u) {
      direct_body_on_request<W, U, NT, true>(src, dst, h_items, h_ctl >> 2, h_loop_sa, h_loop_sb, queue, chunk_items, n_counters, h_sa, h_sb,
                                             [&](uint32_t item, int64_t* so, int64_t* dof) { *so = (int64_t)item * h_sa; *dof = (int64_t)item * h_sb; });
      return;
    }
    touch_kernel_arguments<(int)sizeof(DirectParams) + 64>();
    direct_body_on_request<W, U, NT, false>(src, dst, P.n_items, P.loop_extent, P.loop_sa, P.loop_sb, queue, chunk_items, n_counters, 0, 0,
                                            [&](uint32_t item, int64_t* so, int64_t* dof) { direct_offsets(P, item, so, dof); });
    return;
  }
  if (h_ctl & 1u) {
    direct_body<W, U, NT>(src, dst, h_items, (h_ctl & 2u) != 0, h_ctl >> 2, h_loop_sa, h_loop_sb,
                          [&](uint32_t item, int64_t* so, int64_t* dof) { *so = (int64_t)item * h_sa; *dof = (int64_t)item * h_sb; });
    return;
  }
  touch_kernel_arguments<(int)sizeof(DirectParams) + 64>();
  direct_body<W, U, NT>(src, dst, P.n_items, P.blocked != 0, P.loop_extent, P.loop_sa, P.loop_sb,
                        [&](uint32_t item, int64_t* so, int64_t* dof) { direct_offsets(P, item, so, dof); });
}

// ---------------------------------------------------------------------------------------------
// Gather with a small source stride: the destination-contiguous mode is read with stride GS elements (GS * ES < 32 bytes:
// every 16-byte word of the source span holds an element that is wanted).  A work item is one 16-byte vector of the
// destination; the lane loads the GS consecutive 16-byte words that hold its 16 / ES source elements (word GS * o on for
// vector o: always aligned), keeps every GS-th element and stores one vector.  A wavefront so reads GS KiB of contiguous
// source and writes 1 KiB.  The last vector along the mode would read up to 16 / ES - 1 elements past the last element the
// layout reaches, which the caller has not promised to be addressable: it loads element by element.
// Offsets are in units of 16 bytes, from the direct class's argument block; mode 0 is the gathered mode.
// ---------------------------------------------------------------------------------------------
template <int ES, int GS>
__device__ __forceinline__ u32x4 keep_every(const u32x4 (&t)[GS]) {
  uint32_t f[4 * GS];
#pragma unroll
  for (int k = 0; k < GS; ++k)
#pragma unroll
    for (int d = 0; d < 4; ++d) f[4 * k + d] = t[k][d];
  u32x4 o;
  if constexpr (ES == 4) {
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = f[e * GS];
  } else if constexpr (ES == 8) {
#pragma unroll
    for (int e = 0; e < 2; ++e) { o[2 * e] = f[2 * e * GS]; o[2 * e + 1] = f[2 * e * GS + 1]; }
  } else {   // ES == 2: element h is half h % 2 of dword h / 2
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      constexpr int dummy = 0; (void)dummy;
      const int h0 = 2 * j * GS, h1 = (2 * j + 1) * GS;
      const uint32_t lo = (f[h0 / 2] >> (16 * (h0 % 2))) & 0xffffu, hi = (f[h1 / 2] >> (16 * (h1 % 2))) & 0xffffu;
      o[j] = lo | (hi << 16);
    }
  }
  return o;
}
template <int ES, int GS, int U>
__global__ __launch_bounds__(kBlock) void gather_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, DirectParams P) {
  typedef typename Word<ES>::type E;
  touch_kernel_arguments<(int)sizeof(DirectParams) + 16>();
  const uint32_t step = gridDim.x * kBlock;
  const uint32_t ext0 = P.n_modes > 1 ? P.div[0].div : P.n_items;   // vectors along the gathered mode
  for (uint32_t base = blockIdx.x * kBlock + threadIdx.x; base < P.n_items; base += step * U) {
    int64_t so[U], dof[U];
    bool ok[U], last[U];
    u32x4 v[U];
#pragma unroll
    for (int j = 0; j < U; ++j) {
      const uint32_t it = base + (uint32_t)j * step;
      ok[j] = it < P.n_items;
      so[j] = dof[j] = 0;
      last[j] = false;
      if (ok[j]) {
        direct_offsets(P, it, &so[j], &dof[j]);
        const uint32_t o = P.n_modes > 1 ? it - fd_div(it, P.div[0]) * ext0 : it;
        last[j] = o == ext0 - 1u;
      }
    }
#pragma unroll
    for (int j = 0; j < U; ++j)
      if (ok[j]) {
        if (!last[j]) {
          u32x4 t[GS];
#pragma unroll
          for (int k = 0; k < GS; ++k) t[k] = gload<1>(src + so[j] + k);
          v[j] = keep_every<ES, GS>(t);
        } else {
          const E* e = reinterpret_cast<const E*>(src + so[j]);
          E* w = reinterpret_cast<E*>(&v[j]);
#pragma unroll
          for (int k = 0; k < 16 / ES; ++k) w[k] = e[k * GS];
        }
      }
#pragma unroll
    for (int j = 0; j < U; ++j) if (ok[j]) gstore<2>(dst + dof[j], v[j]);
  }
}

// ---------------------------------------------------------------------------------------------
// Transpose through LDS.  Persistent workgroups walk the grid of tiles (the rest mode of
// zipped_divide, Sec. 3.5.2); per tile each lane owns MT micro-tiles of V x V elements.
//   load : V global loads of V*ES bytes along the source-contiguous mode p (one per step along q)
//   park : register transpose, V LDS writes of V*ES bytes (now contiguous along q), XOR-swizzled slots
//   store: V LDS reads and V global stores of V*ES bytes along the destination-contiguous mode q
// The loads of the next tile are issued before the stores of the current one.
// ---------------------------------------------------------------------------------------------
template <int ES, int V>
__device__ __forceinline__ void micro_transpose(const uint32_t (&r)[V][V * ES / 4], uint32_t (&o)[V][V * ES / 4]) {
  if constexpr (V == 1) {  // a single element (a 16-byte word): nothing to transpose
#pragma unroll
    for (int k = 0; k < V * ES / 4; ++k) o[0][k] = r[0][k];
  } else if constexpr (ES == 4) {
#pragma unroll
    for (int ip = 0; ip < V; ++ip)
#pragma unroll
      for (int iq = 0; iq < V; ++iq) o[ip][iq] = r[iq][ip];
  } else {  // ES == 2: two elements per dword
#pragma unroll
    for (int ip = 0; ip < V; ++ip)
#pragma unroll
      for (int j = 0; j < V / 2; ++j) {
        uint32_t lo = r[2 * j][ip / 2], hi = r[2 * j + 1][ip / 2];
        o[ip][j] = (ip % 2 == 0) ? ((lo & 0xffffu) | (hi << 16)) : ((lo >> 16) | (hi & 0xffff0000u));
      }
  }
}

// FULL: every lane owns MT micro-tiles and MT*V picks (n_micro == MT * kBlock), so the tile loop has
// no per-lane predicates.  Its body is straight-line code on purpose: the loads of the next tile are
// issued before the stores of the current one, and with no branch between them the wait before
// parking can count the stores out (memory operations retire in issue order) instead of draining them.
//
// The leading scalar arguments (the source pointer and the twelve dwords of a TransposeHead) are all the first loads need;
// they are the arguments the hardware may preload into scalar registers at wavefront start.  With h_ctl's valid bit set a
// workgroup issues the loads of its first tile (tile id = workgroup index) from them alone, before the argument block is
// touched; the lane state from the block is worked out while those loads are in flight.
// DYN: tiles past the first rounds come from the queue (FULL tiles only); 0: the queue's code is not in the kernel; 1: one
// counter, the first round of the grid by index (the planner's default: a loop without the general form's branches, which
// measured 2-3 % faster on the fp16 tiled-partition workload); 2: the general form (several rounds, several counters).
template <int ES, int V, int MT, int NT, bool FULL, int DYN>
__global__ __launch_bounds__(kBlock) void transpose_kernel(const unsigned char* __restrict__ src, uint32_t h_ctl, int32_t h_aq, int32_t h_sa0,
                                                          int32_t h_sa1, int32_t h_sa2, int32_t h_sa3, uint32_t h_mul, uint32_t h_div,
                                                          int64_t h_ra0, int64_t h_ra1, TransposeParams P,
                                                          unsigned char* __restrict__ dst, unsigned int* queue, uint32_t tile_bytes, uint32_t grab,
                                                          uint32_t static_rounds, uint32_t n_counters, uint32_t leftover_lead) {
  constexpr int DW = V * ES / 4;                 // dwords per vector
  constexpr int SLOT = V * ES;                   // bytes per vector
  typedef typename Word<SLOT>::type Vec;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  uint32_t r[MT][V][DW];
  bool early = false;
  if constexpr (MT == 1) {
    if (h_ctl & 1u) {
      early = true;
      const TransposeHead H{h_ctl, h_aq, {h_sa0, h_sa1, h_sa2, h_sa3}, h_mul, h_div, h_ra0, h_ra1};
      const int64_t in_tile = head_lane_offset(H, threadIdx.x);
      const unsigned char* base = src + (head_tile_origin(H, blockIdx.x) + in_tile) * ES;
      if (FULL || threadIdx.x < head_n_micro(H)) {
#pragma unroll
        for (int iq = 0; iq < V; ++iq) {
          Vec v = gload<NT>(reinterpret_cast<const Vec*>(base + (int64_t)iq * h_aq * ES));
          const uint32_t* w = reinterpret_cast<const uint32_t*>(&v);
#pragma unroll
          for (int k = 0; k < DW; ++k) r[0][iq][k] = w[k];
        }
      }
      asm volatile("" ::: "memory");   // counts as a possible store: the loads stay ahead of everything below
    }
  }
  touch_kernel_arguments<(int)sizeof(TransposeParams) + 64>();

  // tile-invariant lane state (wavefront-level index arithmetic done once):
  // per owned micro-tile its source offset and LDS base index; per picked vector its destination offset
  int32_t src_in[MT], dst_in[MT * V];
  uint32_t park_g[MT];
  bool act[MT];
#pragma unroll
  for (int m = 0; m < MT; ++m) {
    uint32_t u = threadIdx.x + (uint32_t)m * kBlock;
    act[m] = FULL || u < P.n_micro;
    src_in[m] = 0;
    park_g[m] = 0;
  }
  if (P.src_split > 0) {
    int32_t s0;
    uint32_t g0;
    micro_lane_part(P, threadIdx.x, &s0, &g0);
#pragma unroll
    for (int m = 0; m < MT; ++m) {
      src_in[m] = s0 + P.src_trip_off[m];
      park_g[m] = g0 + P.src_trip_g[m];
    }
  } else {
#pragma unroll
    for (int m = 0; m < MT; ++m)
      if (act[m]) micro_from_src_order(P, threadIdx.x + (uint32_t)m * kBlock, &src_in[m], &park_g[m]);
  }
  // global -> registers: V vectors along p per micro-tile, one per step along q
  auto load_tile = [&](int64_t so) {
    const unsigned char* base = src + so * ES;
#pragma unroll
    for (int m = 0; m < MT; ++m)
      if (FULL || act[m]) {
#pragma unroll
        for (int iq = 0; iq < V; ++iq) {
          Vec v = gload<NT>(reinterpret_cast<const Vec*>(base + ((int64_t)src_in[m] + (int64_t)iq * P.a_q) * ES));
          const uint32_t* w = reinterpret_cast<const uint32_t*>(&v);
#pragma unroll
          for (int k = 0; k < DW; ++k) r[m][iq][k] = w[k];
        }
      }
  };
  // registers -> LDS: transposed micro-tiles, V vectors along q each
  auto park_tile = [&]() {
#pragma unroll
    for (int m = 0; m < MT; ++m)
      if (FULL || act[m]) {
        uint32_t o[V][DW];
        micro_transpose<ES, V>(r[m], o);
#pragma unroll
        for (int ip = 0; ip < V; ++ip) {
          Vec v;
          uint32_t* w = reinterpret_cast<uint32_t*>(&v);
#pragma unroll
          for (int k = 0; k < DW; ++k) w[k] = o[ip][k];
          *reinterpret_cast<Vec*>(lds + lds_slot(P, park_g[m] + (uint32_t)ip * P.gpos_pv) * SLOT) = v;
        }
      }
  };
  // LDS -> global: the tile's vectors in destination address order, consecutive lanes on consecutive vectors
  auto store_tile = [&](int64_t dof) {
    unsigned char* base = dst + dof * ES;
    Vec v[MT * V];
#pragma unroll
    for (int j = 0; j < MT * V; ++j) {
      const uint32_t g = threadIdx.x + (uint32_t)j * kBlock;
      if (FULL || g < P.n_vec) v[j] = *reinterpret_cast<const Vec*>(lds + lds_slot(P, g) * SLOT);
    }
#pragma unroll
    for (int j = 0; j < MT * V; ++j) {
      const uint32_t g = threadIdx.x + (uint32_t)j * kBlock;
      if (FULL || g < P.n_vec) gstore<NT>(reinterpret_cast<Vec*>(base + (int64_t)dst_in[j] * ES), v[j]);
    }
  };

  uint32_t tile = blockIdx.x, tile_step = gridDim.x, tile_end = P.n_tiles;
  if (P.blocked) {
    const uint32_t per_wg = (P.n_tiles + gridDim.x - 1) / gridDim.x;
    tile = blockIdx.x * per_wg;
    tile_step = 1;
    tile_end = min(P.n_tiles, tile + per_wg);
  }
  // queue != nullptr (never with `blocked`): the first static_rounds * gridDim.x tiles go by workgroup index, the tiles
  // past them are handed out in the order the workgroups ask for them, `grab` consecutive tiles per request, by n_counters
  // counters (workgroup w asks counter w mod n_counters, which hands out every n_counters-th batch).  Lane 0 asks one tile
  // ahead: when the loads of a workgroup's last tile by index begin it asks for its first batch, and when the loads of a
  // batch's first tile begin it asks for the batch after.  The request is issued before those loads and so returns before
  // them; the answer reaches the other lanes through a word of LDS behind the tile, at a barrier the loop has anyway.
  // queue[0] counts the workgroups that are done; the last one puts every counter back to zero for the next launch that is
  // given this block.
  // leftover_lead > 0 (fixed order only): the tiles that are left after the last whole round of the grid go to the first
  // leftover_lead workgroups alone, round after round (the workgroups a CU is given first run ahead of the later ones).
  constexpr bool dynamic = DYN != 0;
  const uint32_t G = gridDim.x;
  volatile uint32_t* handed_out = reinterpret_cast<volatile uint32_t*>(lds + tile_bytes);
  uint32_t asked = 0;
  uint32_t static_end = tile_end, batch_base = 0, batch_stride = 1;
  unsigned int* counter = queue;
  if (dynamic) {
    const uint32_t c = blockIdx.x % n_counters;
    static_end = static_rounds * G;
    counter = queue + (1u + c) * kQueueLineWords;
    batch_base = static_end + c * grab;   // an answer a (a multiple of grab) stands for the batch that starts at tile
    batch_stride = n_counters;            // batch_base + a * batch_stride
  }
  const uint32_t whole_rounds_end = (!dynamic && !P.blocked && leftover_lead > 0) ? (tile_end / G) * G : tile_end;
  auto fixed_next = [&](uint32_t t) -> uint32_t {   // the tile after t in the fixed order
    if (t + tile_step < whole_rounds_end || whole_rounds_end == tile_end) return t + tile_step;
    if (t < whole_rounds_end) return blockIdx.x < leftover_lead ? whole_rounds_end + blockIdx.x : tile_end;
    return t + leftover_lead;
  };
  if (tile >= tile_end) {
    if (dynamic && threadIdx.x == 0) leave_tile_queue(queue);
    return;
  }
  // the destination side of the lane state
  auto destination_side = [&]() {
    if (P.dst_split > 0) {
      const int32_t d0 = vector_lane_part(P, threadIdx.x);
#pragma unroll
      for (int j = 0; j < MT * V; ++j) dst_in[j] = d0 + P.dst_trip_off[j];
    } else {
#pragma unroll
      for (int j = 0; j < MT * V; ++j) {
        const uint32_t g = threadIdx.x + (uint32_t)j * kBlock;
        dst_in[j] = (FULL || g < P.n_vec) ? vector_dst_offset(P, g) : 0;
      }
    }
  };
  if constexpr (DYN == 1) {
    // One counter, one round by index: workgroup w starts on tile w and asks, with the loads of every batch's first tile,
    // for the batch after it (batch k starts at tile G + k grab).
    // The counter is the word beside the count of the workgroups that are done, in the block's first line: measured on
    // MI355X, 2^30 fp16 elements in 32 KiB tiles, 0.677 ms with the counter on a line of its own and 0.663 ms here.
    unsigned int* tiles_out = queue + 1;
    if (threadIdx.x == 0) asked = atomicAdd(tiles_out, grab);
    int64_t so, dof;
    tile_origin(P, tile, &so, &dof);
    load_tile(so);
    asm volatile("" ::: "memory");
    destination_side();
    park_tile();
    if (threadIdx.x == 0) *handed_out = G + asked;
    __syncthreads();
    uint32_t left = 0, next_batch = *handed_out, next = next_batch;
    for (;;) {
      if (next >= tile_end) {
        store_tile(dof);
        break;
      }
      const bool new_batch = left == 0;   // `next` is the first tile of a batch: ask for the batch after it
      if (new_batch && threadIdx.x == 0) asked = atomicAdd(tiles_out, grab);
      int64_t dof_next;
      tile_origin(P, next, &so, &dof_next);
      load_tile(so);
      __builtin_amdgcn_sched_barrier(0);   // keep every load ahead of every store in program order
      store_tile(dof);
      __builtin_amdgcn_sched_barrier(0);
      __syncthreads();   // every pick is done: LDS may be overwritten (and every lane has read the word behind the tile)
      park_tile();
      if (new_batch && threadIdx.x == 0) *handed_out = G + asked;
      __syncthreads();
      tile = next;
      dof = dof_next;
      if (new_batch) {
        left = grab - 1u;
        next_batch = *handed_out;
        next = left > 0 ? tile + 1u : next_batch;
      } else {
        --left;
        next = left > 0 ? tile + 1u : next_batch;
      }
    }
    if (threadIdx.x == 0) leave_tile_queue(queue);
    return;
  }
  bool ask = dynamic && tile + G >= static_end;   // the first tile is this workgroup's last tile by index
  if (ask && threadIdx.x == 0) asked = atomicAdd(counter, grab);
  int64_t so, dof;
  tile_origin(P, tile, &so, &dof);
  if (!early) load_tile(so);
  // The destination side of the lane state is worked out while the first loads are in flight.  The
  // empty statement below counts as a possible store, so the compiler cannot sink the loads past it.
  asm volatile("" ::: "memory");
  destination_side();
  park_tile();
  if (ask && threadIdx.x == 0) *handed_out = batch_base + asked * batch_stride;
  __syncthreads();
  // dynamic: `left` tiles of the current batch follow the current tile; next_batch is where the batch after it starts
  uint32_t left = 0, next_batch = ask ? *handed_out : 0u;
  uint32_t next = !dynamic ? fixed_next(tile) : (ask ? next_batch : tile + G);
  // invariant at the top: the current tile is parked in LDS, no load is in flight
  for (;;) {
    if (next >= tile_end) {
      store_tile(dof);
      break;
    }
    // a request goes out with the loads of `next` when that is the last tile by index or the first tile of a batch
    const bool by_index = dynamic && next < static_end;
    ask = dynamic && (by_index ? next + G >= static_end : left == 0);
    if (ask && threadIdx.x == 0) asked = atomicAdd(counter, grab);
    int64_t dof_next;
    tile_origin(P, next, &so, &dof_next);
    load_tile(so);
    __builtin_amdgcn_sched_barrier(0);   // keep every load ahead of every store in program order
    store_tile(dof);
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();   // every pick is done: LDS may be overwritten (and every lane has read the word behind the tile)
    park_tile();
    if (ask && threadIdx.x == 0) *handed_out = batch_base + asked * batch_stride;
    __syncthreads();
    tile = next;
    dof = dof_next;
    if (!dynamic) {
      next = fixed_next(tile);
    } else if (by_index) {
      next = ask ? *handed_out : tile + G;
      left = 0;
    } else if (ask) {
      left = grab - 1u;
      next_batch = *handed_out;
      next = left > 0 ? tile + 1u : next_batch;
    } else {
      --left;
      next = left > 0 ? tile + 1u : next_batch;
    }
  }
  if (dynamic && threadIdx.x == 0) leave_tile_queue(queue);
}

// ---------------------------------------------------------------------------------------------
// Ragged tiles: the same staging through LDS for shapes the tile does not divide (odd extents, extents
// with large prime factors) and for element-wise transposes (V = 1, no vector on either side).  The
// grid has ceil(extent / tile) tiles along a ragged mode; every access first compares its coordinate
// with what is left of the mode (coordinate predication, Sec. 2.3.2).  Kept apart from the kernel above
// so that its predicates do not reach into that kernel's straight-line loop; no software pipeline here,
// several resident workgroups per CU overlap each other's phases.
// ---------------------------------------------------------------------------------------------
template <int ES, int V, int MT, int NT>
__global__ __launch_bounds__(kBlock) void ragged_transpose_kernel(TransposeParams P, const unsigned char* __restrict__ src,
                                                                 unsigned char* __restrict__ dst) {
  constexpr int SLOT = V * ES;
  typedef typename Word<SLOT>::type Vec;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  touch_kernel_arguments<(int)sizeof(TransposeParams)>();

  int32_t src_in[MT], dst_in[MT * V];
  uint32_t park_g[MT], crd_s[MT], crd_d[MT * V];
  bool act_s[MT], act_d[MT * V];
#pragma unroll
  for (int m = 0; m < MT; ++m) {
    const uint32_t u = threadIdx.x + (uint32_t)m * kBlock;
    act_s[m] = u < P.n_micro;
    src_in[m] = 0;
    park_g[m] = 0;
    crd_s[m] = 0;
    if (act_s[m]) micro_from_src_order_ragged(P, u, &src_in[m], &park_g[m], &crd_s[m]);
  }
#pragma unroll
  for (int j = 0; j < MT * V; ++j) {
    const uint32_t g = threadIdx.x + (uint32_t)j * kBlock;
    act_d[j] = g < P.n_vec;
    crd_d[j] = 0;
    dst_in[j] = act_d[j] ? vector_dst_offset_ragged(P, g, &crd_d[j]) : 0;
  }

  uint32_t tile = blockIdx.x, tile_step = gridDim.x, tile_end = P.n_tiles;
  if (P.blocked) {
    const uint32_t per_wg = (P.n_tiles + gridDim.x - 1) / gridDim.x;
    tile = blockIdx.x * per_wg;
    tile_step = 1;
    tile_end = min(P.n_tiles, tile + per_wg);
  }
  for (; tile < tile_end; tile += tile_step) {
    int64_t so, dof;
    uint32_t rem0, rem1;
    tile_origin_ragged(P, tile, &so, &dof, &rem0, &rem1);
    const unsigned char* sbase = src + so * ES;
    unsigned char* dbase = dst + dof * ES;
#pragma unroll
    for (int m = 0; m < MT; ++m)
      if (act_s[m] && inside_ragged(crd_s[m], rem0, rem1)) {
        if constexpr (V == 1) {
          const Vec v = gload<NT>(reinterpret_cast<const Vec*>(sbase + (int64_t)src_in[m] * ES));
          *reinterpret_cast<Vec*>(lds + lds_slot(P, park_g[m]) * SLOT) = v;
        } else {
          constexpr int DW = V * ES / 4;
          uint32_t r[V][DW], o[V][DW];
#pragma unroll
          for (int iq = 0; iq < V; ++iq) {
            const Vec v = gload<NT>(reinterpret_cast<const Vec*>(sbase + ((int64_t)src_in[m] + (int64_t)iq * P.a_q) * ES));
            const uint32_t* w = reinterpret_cast<const uint32_t*>(&v);
#pragma unroll
            for (int k = 0; k < DW; ++k) r[iq][k] = w[k];
          }
          micro_transpose<ES, V>(r, o);
#pragma unroll
          for (int ip = 0; ip < V; ++ip) {
            Vec v;
            uint32_t* w = reinterpret_cast<uint32_t*>(&v);
#pragma unroll
            for (int k = 0; k < DW; ++k) w[k] = o[ip][k];
            *reinterpret_cast<Vec*>(lds + lds_slot(P, park_g[m] + (uint32_t)ip * P.gpos_pv) * SLOT) = v;
          }
        }
      }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < MT * V; ++j)
      if (act_d[j] && inside_ragged(crd_d[j], rem0, rem1)) {
        const uint32_t g = threadIdx.x + (uint32_t)j * kBlock;
        const Vec v = *reinterpret_cast<const Vec*>(lds + lds_slot(P, g) * SLOT);
        *reinterpret_cast<Vec*>(dbase + (int64_t)dst_in[j] * ES) = v;
      }
    __syncthreads();
  }
}

// ---------------------------------------------------------------------------------------------
// Launchers
// ---------------------------------------------------------------------------------------------
static thread_local std::string g_last_hip_error;
const char* last_hip_error() { return g_last_hip_error.c_str(); }
void set_last_hip_error(const std::string& text) { g_last_hip_error = text; }
static bool hip_failed(hipError_t e, const char* what) {
  if (e == hipSuccess) return false;
  g_last_hip_error = std::string(what) + ": " + hipGetErrorName(e) + " (" + hipGetErrorString(e) + ")";
  return true;
}

static int device_cu_count() {
  static std::atomic<int> cus{0};
  if (cus.load() == 0) {
    int dev = 0;
    if (hip_failed(hipGetDevice(&dev), "hipGetDevice")) return -1;
    int n = 0;
    if (hip_failed(hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev), "hipDeviceGetAttribute") || n <= 0) return -1;
    cus.store(n);
  }
  return cus.load();
}

template <int ES>
static void launch_generic(const lc_plan& plan, const void* src, void* dst, unsigned grid, hipStream_t s) {
  typedef typename Word<ES>::type T;
  hipLaunchKernelGGL(generic_kernel<ES>, dim3(grid), dim3(kBlock), 0, s, plan.generic, static_cast<const T*>(src), static_cast<T*>(dst));
}

template <int W, int U>
static void launch_direct_u(const lc_plan& plan, const void* src, void* dst, unsigned grid, hipStream_t s, unsigned int* queue) {
  typedef typename Word<W>::type T;
  const T* sp = static_cast<const T*>(src);
  T* dp = static_cast<T*>(dst);
  // a copy over one joint mode travels whole in the leading arguments (see direct_kernel)
  const DirectParams& P = plan.direct;
  uint32_t ctl = 0;
  if (plan.early_loads && P.n_modes == 1 && P.loop_extent < (1u << 30)) ctl = 1u | (P.blocked ? 2u : 0u) | (P.loop_extent << 2);
  const uint32_t items = P.n_items;
  const int64_t sa = P.sa[0], sb = P.sb[0], lsa = P.loop_sa, lsb = P.loop_sb;
  const uint32_t chunk = (uint32_t)((std::max(1, plan.direct_queue_items) + 64 * U - 1) / (64 * U) * (64 * U)), counters = (uint32_t)std::max(1, std::min(plan.queue_counters, kQueueLines - 1));
  switch (plan.nontemporal) {
    case 0: hipLaunchKernelGGL((direct_kernel<W, U, 0>), dim3(grid), dim3(kBlock), 0, s, sp, dp, ctl, items, sa, sb, lsa, lsb, P, queue, chunk, counters); break;
    case 1: hipLaunchKernelGGL((direct_kernel<W, U, 1>), dim3(grid), dim3(kBlock), 0, s, sp, dp, ctl, items, sa, sb, lsa, lsb, P, queue, chunk, counters); break;
    case 2: hipLaunchKernelGGL((direct_kernel<W, U, 2>), dim3(grid), dim3(kBlock), 0, s, sp, dp, ctl, items, sa, sb, lsa, lsb, P, queue, chunk, counters); break;
    default: hipLaunchKernelGGL((direct_kernel<W, U, 3>), dim3(grid), dim3(kBlock), 0, s, sp, dp, ctl, items, sa, sb, lsa, lsb, P, queue, chunk, counters); break;
  }
}
template <int ES, int GS>
static void launch_gather_s(const lc_plan& plan, const void* src, void* dst, unsigned grid, hipStream_t s) {
  const u32x4* sp = static_cast<const u32x4*>(src);
  u32x4* dp = static_cast<u32x4*>(dst);
  if (plan.unroll >= 2) hipLaunchKernelGGL((gather_kernel<ES, GS, 2>), dim3(grid), dim3(kBlock), 0, s, sp, dp, plan.direct);
  else hipLaunchKernelGGL((gather_kernel<ES, GS, 1>), dim3(grid), dim3(kBlock), 0, s, sp, dp, plan.direct);
}
template <int ES>
static bool launch_gather(const lc_plan& plan, const void* src, void* dst, unsigned grid, hipStream_t s) {
  switch (plan.gather_stride) {
    case 2: launch_gather_s<ES, 2>(plan, src, dst, grid, s); return true;
    case 3: launch_gather_s<ES, 3>(plan, src, dst, grid, s); return true;
    case 4: if constexpr (ES < 8) { launch_gather_s<ES, 4>(plan, src, dst, grid, s); return true; } break;
    case 5: if constexpr (ES < 8) { launch_gather_s<ES, 5>(plan, src, dst, grid, s); return true; } break;
    case 6: if constexpr (ES < 8) { launch_gather_s<ES, 6>(plan, src, dst, grid, s); return true; } break;
    case 7: if constexpr (ES < 8) { launch_gather_s<ES, 7>(plan, src, dst, grid, s); return true; } break;
  }
  return false;
}
template <int W>
static void launch_direct(const lc_plan& plan, const void* src, void* dst, unsigned grid, hipStream_t s, unsigned int* queue) {
  switch (plan.unroll) {
    case 1: launch_direct_u<W, 1>(plan, src, dst, grid, s, queue); break;
    case 2: launch_direct_u<W, 2>(plan, src, dst, grid, s, queue); break;
    case 8: launch_direct_u<W, 8>(plan, src, dst, grid, s, queue); break;
    default: launch_direct_u<W, 4>(plan, src, dst, grid, s, queue); break;
  }
}

// The pair of queue counters a launch on stream `s` may use, or nullptr (fixed tile order) when no pair can be promised to
// this launch alone: the stream is being captured into a graph (a replay may run beside anything), the handle is
// hipStreamPerThread (one value, a different stream in every host thread), the stream belongs to another device than the
// current one, or all pairs belong to other streams already.  One pair per stream and device: launches on a stream do not
// overlap, which is what the counters' reset by the last workgroup relies on.  `failed` names the call behind an error.
static hipError_t tile_queue_of_stream(hipStream_t s, unsigned int** out, const char** failed) {
  *out = nullptr;
  if (s == hipStreamPerThread) return hipSuccess;
  hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
  *failed = "hipStreamIsCapturing";
  hipError_t e = hipStreamIsCapturing(s, &capturing);
  if (e != hipSuccess) return e;
  if (capturing != hipStreamCaptureStatusNone) return hipSuccess;
  int dev = 0;
  *failed = "hipGetDevice";
  if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
  if (s != nullptr) {   // the null stream is the current device's
    hipDevice_t owner = 0;
    *failed = "hipStreamGetDevice";
    if ((e = hipStreamGetDevice(s, &owner)) != hipSuccess) return e;
    if ((int)owner != dev) return hipSuccess;
  }
  static std::mutex lock;
  static std::map<std::pair<int, hipStream_t>, int> slot_of;      // (device, stream) -> pair
  static std::map<int, std::pair<unsigned int*, int>> per_device;   // device -> (address of the array, pairs handed out)
  std::lock_guard<std::mutex> hold(lock);
  auto dv = per_device.find(dev);
  if (dv == per_device.end()) {
    void* base = nullptr;
    *failed = "hipGetSymbolAddress";
    if ((e = hipGetSymbolAddress(&base, HIP_SYMBOL(g_tile_queues))) != hipSuccess) return e;
    dv = per_device.emplace(dev, std::make_pair(static_cast<unsigned int*>(base), 0)).first;
  }
  auto it = slot_of.find({dev, s});
  if (it == slot_of.end()) {
    if (dv->second.second >= kTileQueues) return hipSuccess;   // no pair left: fixed order
    it = slot_of.emplace(std::make_pair(dev, s), dv->second.second++).first;
  }
  *out = dv->second.first + (size_t)kQueueBlockWords * it->second;
  return hipSuccess;
}

// what a launcher reports back: the HIP status of whatever it called before the launch, and that call's name
struct PreLaunch {
  hipError_t status = hipSuccess;
  const char* call = "";
};

template <int ES, int V, int MT, int NT, bool FULL>
static PreLaunch launch_transpose_f(const lc_plan& plan, const void* src, void* dst, unsigned grid, hipStream_t s) {
  const unsigned char* sp = static_cast<const unsigned char*>(src);
  unsigned char* dp = static_cast<unsigned char*>(dst);
  PreLaunch pre;
  unsigned int* queue = nullptr;
  unsigned lds_bytes = plan.lds_bytes;
  if (FULL && plan.tile_queue && grid < plan.transpose.n_tiles) {
    pre.status = tile_queue_of_stream(s, &queue, &pre.call);
    if (pre.status != hipSuccess) return pre;
    if (queue) lds_bytes += 16;   // the word that carries the next tile to the other lanes
  }
  if (lds_bytes > 64 * 1024) {   // what this launch asks for, the queue's word included
    static std::atomic<bool> raised{false};   // one flag per instantiation: the attribute belongs to the kernel function
    if (!raised.load(std::memory_order_acquire)) {
      pre.call = "hipFuncSetAttribute";
      pre.status = hipFuncSetAttribute(reinterpret_cast<const void*>(&transpose_kernel<ES, V, MT, NT, FULL, 0>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
      if (pre.status == hipSuccess && FULL)
        pre.status = hipFuncSetAttribute(reinterpret_cast<const void*>(&transpose_kernel<ES, V, MT, NT, FULL, FULL ? 1 : 0>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
      if (pre.status == hipSuccess && FULL)
        pre.status = hipFuncSetAttribute(reinterpret_cast<const void*>(&transpose_kernel<ES, V, MT, NT, FULL, FULL ? 2 : 0>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
      if (pre.status != hipSuccess) return pre;
      raised.store(true, std::memory_order_release);
    }
  }
  const uint32_t counters = (uint32_t)std::max(1, std::min(plan.queue_counters, kQueueLines - 1));
  // whole rounds of the grid that go by index before the queue takes over (at least one, never past the last whole round)
  const uint32_t rounds = (uint32_t)std::max<int64_t>(1, std::min<int64_t>(plan.queue_static_rounds, plan.transpose.n_tiles / grid));
  // the head serves launches in the fixed tile order, where a workgroup's first tile is its index (a request to the queue
  // would have to go out ahead of the first loads), on grids whose first tiles the planner has checked
  TransposeHead h = plan.head;
  if (queue || MT != 1 || grid > (unsigned)kHeadMaxGrid || grid > plan.transpose.n_tiles) h.ctl = 0;
  const uint32_t grab = (uint32_t)std::max(1, plan.tile_queue), lead = (uint32_t)std::min<int64_t>(std::max(0, plan.leftover_lead), grid);
  if (FULL && queue && rounds == 1u && counters == 1u)
    hipLaunchKernelGGL((transpose_kernel<ES, V, MT, NT, FULL, FULL ? 1 : 0>), dim3(grid), dim3(kBlock), lds_bytes, s, sp, h.ctl, h.a_q, h.sa[0], h.sa[1],
                       h.sa[2], h.sa[3], h.r0_mul, h.r0_div, h.ra0, h.ra1, plan.transpose, dp, queue, plan.lds_bytes, grab, rounds, counters, lead);
  else if (FULL && queue)
    hipLaunchKernelGGL((transpose_kernel<ES, V, MT, NT, FULL, FULL ? 2 : 0>), dim3(grid), dim3(kBlock), lds_bytes, s, sp, h.ctl, h.a_q, h.sa[0], h.sa[1],
                       h.sa[2], h.sa[3], h.r0_mul, h.r0_div, h.ra0, h.ra1, plan.transpose, dp, queue, plan.lds_bytes, grab, rounds, counters, lead);
  else
    hipLaunchKernelGGL((transpose_kernel<ES, V, MT, NT, FULL, 0>), dim3(grid), dim3(kBlock), lds_bytes, s, sp, h.ctl, h.a_q, h.sa[0], h.sa[1],
                       h.sa[2], h.sa[3], h.r0_mul, h.r0_div, h.ra0, h.ra1, plan.transpose, dp, queue, plan.lds_bytes, grab, rounds, counters, lead);
  return pre;
}
template <int ES, int V, int MT, int NT>
static PreLaunch launch_transpose_n(const lc_plan& plan, const void* src, void* dst, unsigned grid, hipStream_t s) {
  if (plan.transpose.n_micro == (uint32_t)MT * kBlock) return launch_transpose_f<ES, V, MT, NT, true>(plan, src, dst, grid, s);
  return launch_transpose_f<ES, V, MT, NT, false>(plan, src, dst, grid, s);
}
template <int ES, int V, int MT>
static PreLaunch launch_transpose_m(const lc_plan& plan, const void* src, void* dst, unsigned grid, hipStream_t s) {
  switch (plan.nontemporal) {
    case 0: return launch_transpose_n<ES, V, MT, 0>(plan, src, dst, grid, s);
    case 1: return launch_transpose_n<ES, V, MT, 1>(plan, src, dst, grid, s);
    case 2: return launch_transpose_n<ES, V, MT, 2>(plan, src, dst, grid, s);
    default: return launch_transpose_n<ES, V, MT, 3>(plan, src, dst, grid, s);
  }
}
template <int ES, int V>
static PreLaunch launch_transpose(const lc_plan& plan, const void* src, void* dst, unsigned grid, hipStream_t s) {
  switch (plan.micro_per_thread) {
    case 1: return launch_transpose_m<ES, V, 1>(plan, src, dst, grid, s);
    case 2: return launch_transpose_m<ES, V, 2>(plan, src, dst, grid, s);
    case 4: return launch_transpose_m<ES, V, 4>(plan, src, dst, grid, s);
    case 8:
      if constexpr (V == 1) return launch_transpose_m<ES, V, 8>(plan, src, dst, grid, s);
      break;
  }
  return PreLaunch{hipErrorInvalidValue, "kernel selection (micro-tiles per lane)"};
}

template <int ES, int V, int MT>
static PreLaunch launch_ragged_m(const lc_plan& plan, const void* src, void* dst, unsigned grid, hipStream_t s) {
  const unsigned char* sp = static_cast<const unsigned char*>(src);
  unsigned char* dp = static_cast<unsigned char*>(dst);
  if (plan.nontemporal & 1)
    hipLaunchKernelGGL((ragged_transpose_kernel<ES, V, MT, 1>), dim3(grid), dim3(kBlock), plan.lds_bytes, s, plan.transpose, sp, dp);
  else
    hipLaunchKernelGGL((ragged_transpose_kernel<ES, V, MT, 0>), dim3(grid), dim3(kBlock), plan.lds_bytes, s, plan.transpose, sp, dp);
  return PreLaunch{};
}
template <int ES, int V>
static PreLaunch launch_ragged(const lc_plan& plan, const void* src, void* dst, unsigned grid, hipStream_t s) {
  if (plan.lds_bytes > 64 * 1024) return PreLaunch{hipErrorInvalidValue, "ragged tile larger than the default LDS limit"};   // the planner keeps them within it
  switch (plan.micro_per_thread) {
    case 1: return launch_ragged_m<ES, V, 1>(plan, src, dst, grid, s);
    case 2: return launch_ragged_m<ES, V, 2>(plan, src, dst, grid, s);
    case 4: return launch_ragged_m<ES, V, 4>(plan, src, dst, grid, s);
    case 8:
      if constexpr (V == 1) return launch_ragged_m<ES, V, 8>(plan, src, dst, grid, s);
      break;
  }
  return PreLaunch{hipErrorInvalidValue, "kernel selection (micro-tiles per lane)"};
}

template <int ES>
static void launch_last_writer_move(const lc_plan& plan, const void* src, void* dst, const uint32_t* last, unsigned grid, hipStream_t s) {
  typedef typename Word<ES>::type T;
  hipLaunchKernelGGL(last_writer_move_kernel<ES>, dim3(grid), dim3(kBlock), 0, s, plan.generic, static_cast<const T*>(src), static_cast<T*>(dst), last);
}

static lc_status_t execute_with(const lc_plan& plan, const void* src, void* dst, void* workspace, size_t workspace_bytes, void* stream);

lc_status_t execute_plan(const lc_plan& plan, const void* src, void* dst, void* stream) {
  if (plan.cls == KernelClass::LastWriter) return LC_ERR_NEEDS_WORKSPACE;
  return execute_with(plan, src, dst, nullptr, 0, stream);
}

lc_status_t execute_plan_workspace(const lc_plan& plan, const void* src, void* dst, void* workspace, size_t workspace_bytes, void* stream) {
  if (plan.workspace_bytes > 0 &&
      (!workspace || (int64_t)workspace_bytes < plan.workspace_bytes || reinterpret_cast<uintptr_t>(workspace) % 4 != 0))
    return LC_ERR_WORKSPACE_TOO_SMALL;
  return execute_with(plan, src, dst, workspace, workspace_bytes, stream);
}

// Scratch memory for callers that cannot allocate: one array per GPU in the device memory of this code object.  Its name is
// a host-side stand-in; the address on a device comes from hipGetSymbolAddress, asked once per device with that device
// current, and only that address is ever handed to a kernel.
static __device__ __align__(256) unsigned char scratch[LC_STATIC_SCRATCH_BYTES];
size_t static_scratch_bytes() { return LC_STATIC_SCRATCH_BYTES; }

lc_status_t execute_plan_static(const lc_plan& plan, const void* src, void* dst, void* stream) {
  if (plan.workspace_bytes == 0) return execute_with(plan, src, dst, nullptr, 0, stream);   // no scratch needed, nothing allocated either
  if (plan.workspace_bytes > (int64_t)LC_STATIC_SCRATCH_BYTES) {
    set_last_hip_error("the plan needs " + std::to_string(plan.workspace_bytes) + " bytes of scratch, the static array holds " +
                       std::to_string((size_t)LC_STATIC_SCRATCH_BYTES));
    return LC_ERR_SCRATCH_LIMIT;
  }
  int dev = 0;
  if (hip_failed(hipGetDevice(&dev), "hipGetDevice")) return LC_ERR_HIP;
  static std::mutex lock;
  static std::map<int, void*> address_on;   // device -> address of its copy of the array
  void* ptr = nullptr;
  {
    std::lock_guard<std::mutex> hold(lock);
    auto it = address_on.find(dev);
    if (it == address_on.end()) {
      void* found = nullptr;
      if (hip_failed(hipGetSymbolAddress(&found, HIP_SYMBOL(scratch)), "hipGetSymbolAddress") || !found) return LC_ERR_HIP;
      it = address_on.emplace(dev, found).first;
    }
    ptr = it->second;
  }
  return execute_with(plan, src, dst, ptr, LC_STATIC_SCRATCH_BYTES, stream);
}

static lc_status_t execute_with(const lc_plan& plan, const void* src, void* dst, void* workspace, size_t, void* stream) {
  if (!src || !dst) return LC_ERR_INVALID_ARG;
  // offsets the planner folded into the accessors: the slice that is written last, the last elements of modes walked backwards
  src = static_cast<const unsigned char*>(src) + plan.src_offset_elems * plan.elem_bytes;
  dst = static_cast<unsigned char*>(dst) + plan.dst_offset_elems * plan.elem_bytes;
  if ((reinterpret_cast<uintptr_t>(src) % plan.src_align) != 0 || (reinterpret_cast<uintptr_t>(dst) % plan.dst_align) != 0)
    return LC_ERR_MISALIGNED;
  const int cus = device_cu_count();
  if (cus <= 0) return LC_ERR_HIP;
  hipStream_t s = static_cast<hipStream_t>(stream);
  (void)hipGetLastError();
  PreLaunch pre;
  if (plan.cls == KernelClass::LastWriter) {
    // three launches in stream order: clear the records, record the last coordinate per offset, move
    uint32_t* records = static_cast<uint32_t*>(workspace);
    uint32_t* last = records + plan.workspace_bias;   // the record of destination offset 0
    const uint64_t words = (uint64_t)plan.workspace_bytes / 4;
    const unsigned zgrid = (unsigned)std::max<uint64_t>(1, std::min<uint64_t>((words + kBlock - 1) / kBlock, (uint64_t)cus * 16));
    const unsigned grid = (unsigned)std::max<uint64_t>(1, std::min<uint64_t>(((uint64_t)plan.generic.n + kBlock - 1) / kBlock, (uint64_t)cus * 16));
    hipLaunchKernelGGL(zero_words_kernel, dim3(zgrid), dim3(kBlock), 0, s, records, words);
    hipLaunchKernelGGL(last_writer_mark_kernel, dim3(grid), dim3(kBlock), 0, s, plan.generic, last);
    switch (plan.elem_bytes) {
      case 1: launch_last_writer_move<1>(plan, src, dst, last, grid, s); break;
      case 2: launch_last_writer_move<2>(plan, src, dst, last, grid, s); break;
      case 4: launch_last_writer_move<4>(plan, src, dst, last, grid, s); break;
      case 8: launch_last_writer_move<8>(plan, src, dst, last, grid, s); break;
      case 16: launch_last_writer_move<16>(plan, src, dst, last, grid, s); break;
      default: return LC_ERR_UNSUPPORTED_DTYPE;
    }
  } else if (plan.cls == KernelClass::Generic) {
    uint64_t want = ((uint64_t)plan.generic.n + kBlock - 1) / kBlock;
    unsigned grid = (unsigned)std::max<uint64_t>(1, std::min<uint64_t>(want, (uint64_t)cus * 16));
    switch (plan.elem_bytes) {
      case 1: launch_generic<1>(plan, src, dst, grid, s); break;
      case 2: launch_generic<2>(plan, src, dst, grid, s); break;
      case 4: launch_generic<4>(plan, src, dst, grid, s); break;
      case 8: launch_generic<8>(plan, src, dst, grid, s); break;
      case 16: launch_generic<16>(plan, src, dst, grid, s); break;
      default: return LC_ERR_UNSUPPORTED_DTYPE;
    }
  } else if (plan.cls == KernelClass::Direct) {
    uint64_t want = ((uint64_t)plan.direct.n_items + (uint64_t)kBlock * plan.unroll - 1) / ((uint64_t)kBlock * plan.unroll);
    unsigned grid = (unsigned)std::max<uint64_t>(1, std::min<uint64_t>(want, plan.grid_override > 0 ? (uint64_t)plan.grid_override : (uint64_t)cus * plan.wgs_per_cu));
    // long copies take their chunks on request, through the stream's block of counters (none to be had: the fixed order)
    unsigned int* dq = nullptr;
    if (plan.direct_queue_items > 0 && plan.gather_stride == 0) {
      pre.status = tile_queue_of_stream(s, &dq, &pre.call);
      if (hip_failed(pre.status, pre.call)) return LC_ERR_HIP;
    }
    for (int64_t j = 0; j < plan.n_launches; ++j) {
      const void* sj = static_cast<const unsigned char*>(src) + j * plan.launch_src_step * plan.elem_bytes;
      void* dj = static_cast<unsigned char*>(dst) + j * plan.launch_dst_step * plan.elem_bytes;
      if (plan.gather_stride > 0) {
        bool launched = false;
        switch (plan.elem_bytes) {
          case 2: launched = launch_gather<2>(plan, sj, dj, grid, s); break;
          case 4: launched = launch_gather<4>(plan, sj, dj, grid, s); break;
          case 8: launched = launch_gather<8>(plan, sj, dj, grid, s); break;
        }
        if (!launched) return LC_ERR_UNSUPPORTED_DTYPE;
        continue;
      }
      switch (plan.width_bytes) {
        case 1: launch_direct<1>(plan, sj, dj, grid, s, dq); break;
        case 2: launch_direct<2>(plan, sj, dj, grid, s, dq); break;
        case 4: launch_direct<4>(plan, sj, dj, grid, s, dq); break;
        case 8: launch_direct<8>(plan, sj, dj, grid, s, dq); break;
        case 16: launch_direct<16>(plan, sj, dj, grid, s, dq); break;
        default: return LC_ERR_UNSUPPORTED_DTYPE;
      }
    }
  } else {
    unsigned grid = (unsigned)std::max<uint64_t>(1, std::min<uint64_t>(plan.transpose.n_tiles, plan.grid_override > 0 ? (uint64_t)plan.grid_override : (uint64_t)cus * plan.wgs_per_cu));
    const int key = plan.tile_elem_bytes * 100 + plan.V;
    if (plan.transpose.n_ragged > 0 || (plan.V == 1 && plan.tile_elem_bytes != 16)) {
      switch (key) {
        case 1601: pre = launch_ragged<16, 1>(plan, src, dst, grid, s); break;
        case 801: pre = launch_ragged<8, 1>(plan, src, dst, grid, s); break;
        case 401: pre = launch_ragged<4, 1>(plan, src, dst, grid, s); break;
        case 201: pre = launch_ragged<2, 1>(plan, src, dst, grid, s); break;
        case 101: pre = launch_ragged<1, 1>(plan, src, dst, grid, s); break;
        case 404: pre = launch_ragged<4, 4>(plan, src, dst, grid, s); break;
        case 402: pre = launch_ragged<4, 2>(plan, src, dst, grid, s); break;
        case 208: pre = launch_ragged<2, 8>(plan, src, dst, grid, s); break;
        case 204: pre = launch_ragged<2, 4>(plan, src, dst, grid, s); break;
        case 202: pre = launch_ragged<2, 2>(plan, src, dst, grid, s); break;
        default: return LC_ERR_UNSUPPORTED_DTYPE;
      }
    } else
    switch (key) {
      case 1601: pre = launch_transpose<16, 1>(plan, src, dst, grid, s); break;
      case 404: pre = launch_transpose<4, 4>(plan, src, dst, grid, s); break;
      case 402: pre = launch_transpose<4, 2>(plan, src, dst, grid, s); break;
      case 208: pre = launch_transpose<2, 8>(plan, src, dst, grid, s); break;
      case 204: pre = launch_transpose<2, 4>(plan, src, dst, grid, s); break;
      case 202: pre = launch_transpose<2, 2>(plan, src, dst, grid, s); break;
      default: return LC_ERR_UNSUPPORTED_DTYPE;
    }
  }
  if (hip_failed(pre.status, pre.call) || hip_failed(hipGetLastError(), "kernel launch")) return LC_ERR_HIP;
  return LC_OK;
}

lc_status_t time_plan(const lc_plan& plan, const void* const* srcs, void* const* dsts, int n_buffers, int warmup,
                      int iters, void* stream, float* ms_per_iter) {
  if (!srcs || !dsts || n_buffers < 1 || iters < 1 || warmup < 0 || !ms_per_iter) return LC_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipEvent_t e0, e1;
  if (hip_failed(hipEventCreate(&e0), "hipEventCreate")) return LC_ERR_HIP;
  if (hip_failed(hipEventCreate(&e1), "hipEventCreate")) { (void)hipEventDestroy(e0); return LC_ERR_HIP; }
  lc_status_t st = LC_OK;
  int b = 0;
  for (int i = 0; i < warmup && st == LC_OK; ++i, b = (b + 1) % n_buffers) st = execute_plan(plan, srcs[b], dsts[b], stream);
  if (st == LC_OK && hip_failed(hipEventRecord(e0, s), "hipEventRecord")) st = LC_ERR_HIP;
  for (int i = 0; i < iters && st == LC_OK; ++i, b = (b + 1) % n_buffers) st = execute_plan(plan, srcs[b], dsts[b], stream);
  if (st == LC_OK && hip_failed(hipEventRecord(e1, s), "hipEventRecord")) st = LC_ERR_HIP;
  if (st == LC_OK && hip_failed(hipEventSynchronize(e1), "hipEventSynchronize")) st = LC_ERR_HIP;
  float ms = 0.f;
  if (st == LC_OK && hip_failed(hipEventElapsedTime(&ms, e0, e1), "hipEventElapsedTime")) st = LC_ERR_HIP;
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (st == LC_OK) *ms_per_iter = ms / (float)iters;
  return st;
}

// The same launches with an event between every two of them: ms_each[i] is the time from the event before execution i
// to the event after it (the kernel and whatever gap the stream leaves before the next event).
lc_status_t time_plan_each(const lc_plan& plan, const void* const* srcs, void* const* dsts, int n_buffers, int warmup,
                           int iters, void* stream, float* ms_each) {
  if (!srcs || !dsts || n_buffers < 1 || iters < 1 || iters > 4096 || warmup < 0 || !ms_each) return LC_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(stream);
  std::vector<hipEvent_t> ev((size_t)iters + 1, nullptr);
  lc_status_t st = LC_OK;
  for (hipEvent_t& e : ev)
    if (st == LC_OK && hip_failed(hipEventCreate(&e), "hipEventCreate")) { e = nullptr; st = LC_ERR_HIP; }
  int b = 0;
  for (int i = 0; i < warmup && st == LC_OK; ++i, b = (b + 1) % n_buffers) st = execute_plan(plan, srcs[b], dsts[b], stream);
  if (st == LC_OK && hip_failed(hipEventRecord(ev[0], s), "hipEventRecord")) st = LC_ERR_HIP;
  for (int i = 0; i < iters && st == LC_OK; ++i, b = (b + 1) % n_buffers) {
    st = execute_plan(plan, srcs[b], dsts[b], stream);
    if (st == LC_OK && hip_failed(hipEventRecord(ev[(size_t)i + 1], s), "hipEventRecord")) st = LC_ERR_HIP;
  }
  if (st == LC_OK && hip_failed(hipEventSynchronize(ev[(size_t)iters]), "hipEventSynchronize")) st = LC_ERR_HIP;
  for (int i = 0; i < iters && st == LC_OK; ++i)
    if (hip_failed(hipEventElapsedTime(&ms_each[i], ev[(size_t)i], ev[(size_t)i + 1]), "hipEventElapsedTime")) st = LC_ERR_HIP;
  for (hipEvent_t e : ev)
    if (e) (void)hipEventDestroy(e);
  return st;
}

}  // namespace lc
