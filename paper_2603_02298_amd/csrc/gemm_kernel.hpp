// Device code of the generic GEMM, included by the translation units that instantiate it (one per element type
// and tile size, so that they compile in parallel).
// Generic GEMM for gfx950 (CDNA4, wave64): C(m,n) += A(m,k) * B(n,k) (Sec. 2.6.2 of "CuTe Layout
// Representation and Algebra") for operands described by layouts, on the matrix cores
// (v_mfma_f32_32x32x16 bf16 / f16, fp32 accumulation).
//
// One workgroup of 4 wavefronts owns a BM x BN tile of C; wavefront (wm, wn) owns a (BM/2) x (BN/2)
// quarter as WMB x WNB fragments of 32 x 32.  Per k tile of 64 the operand tiles pass through LDS.  How a
// tile is loaded depends on which mode of the operand is contiguous (GemmLoad).  Pairs of operands that
// qualify go straight from global memory into a ring of five LDS tiles (one barrier per k tile, loads a
// quarter of a tile per k step); any other pair is loaded into registers before the MFMAs of k tile t and
// parked in the other of two LDS stages after them.
#pragma once
#include <hip/hip_runtime.h>

#include <atomic>
#include <string>
#include <type_traits>

#include "gemm_plan.hpp"
#include "plan.hpp"

namespace lc {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

template <bool BF16>
__device__ __forceinline__ f32x16 mfma_32x32x16(u32x4 a, u32x4 b, f32x16 c) {
  if constexpr (BF16)
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

// Row i of the transpose of an 8x8 block of 16-bit elements held as 8 vectors of 8 (in[j] = the 8 rows' elements
// at column j): element j of the result is element i of in[j].  `odd` says whether i is odd (it may be a run-time
// value: it only picks the halves of the dwords, never a register); half = i / 2 picks the dword.
__device__ __forceinline__ u32x4 transposed_row_b16(const u32x4 (&in)[8], int half, bool odd) {
  // v_perm_b32 picks 4 of the 8 bytes {in[2d+1] dword : in[2d] dword}: low halves of both, or high halves of both
  const uint32_t sel = odd ? 0x07060302u : 0x05040100u;
  u32x4 out;
#pragma unroll
  for (int d = 0; d < 4; ++d) out[d] = __builtin_amdgcn_perm(in[2 * d + 1][half], in[2 * d][half], sel);
  return out;
}

// compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>); the accumulators are
// only ever indexed with constants, so they stay in registers
template <int N, int I = 0, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<N, I + 1>(f);
  }
}

// One 32 x 16 fragment's share of a lane from a k-major tile (row k of the tile = BR elements, see gemm_rdirect_lds_offset):
// two LDS transpose loads (ds_read_b64_tr_b16) of k .. k + 3 and k + 4 .. k + 7; `at` is the lane's address for the
// tile's first 16 k, kk the k step.
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
// The restrict qualifier gives the load alias information once inlined; without any, the compiler makes every such load wait
// for all direct loads in flight (they write LDS too), although those go to the other stage.
__device__ __forceinline__ s16x4 lds_transpose_load(lds_s16x4* __restrict__ p) { return __builtin_amdgcn_ds_read_tr16_b64_v4i16(p); }
template <int BR, typename KK>
__device__ __forceinline__ u32x4 lds_read_tr_16x8(const unsigned char* at, KK kk) {
  const unsigned char* p = at + (uint32_t)kk * 16u * (BR * 2u);
  const s16x4 lo = lds_transpose_load((lds_s16x4*)(p));
  const s16x4 hi = lds_transpose_load((lds_s16x4*)(p + 4u * (BR * 2u)));
  typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
  const u32x2 l = __builtin_bit_cast(u32x2, lo), h = __builtin_bit_cast(u32x2, hi);
  return u32x4{l[0], l[1], h[0], h[1]};
}

__device__ __forceinline__ u32x4 select_or_zero(bool keep, u32x4 v) {
  return u32x4{keep ? v[0] : 0u, keep ? v[1] : 0u, keep ? v[2] : 0u, keep ? v[3] : 0u};
}

// One operand (A or B) of one workgroup: issues the global loads of a k tile into registers, parks them in LDS.
// Loads are unconditional from clamped coordinates (always inside the tensor); what lies past K is zeroed
// in registers afterwards, so the loop carries no divergent branch.
// KTAIL (direct loads): K is not a multiple of the k tile; the lanes whose piece of the last k tile lies at or past K
// present an offset outside the buffer there, which the memory pipeline answers with zeros (no access is made).
template <int BR, int LOAD, bool KTAIL = false>
struct OperandLoader {
  static constexpr int ROWS = BR / 32;                                    // rows per lane for k-vector / element loads
  static constexpr bool DIRECT = LOAD == kLoadKDirect || LOAD == kLoadRDirect;
  static constexpr int NREG = LOAD == kLoadRVec ? 8 : (DIRECT ? 1 : ROWS);
  const uint16_t* base;
  __amdgpu_buffer_rsrc_t rsrc;           // direct loads: the operand as a raw buffer (uniform base, 32-bit byte offsets)
  uint32_t K, kv, row_in_tile;           // row_in_tile: first row of the lane (block row for row-vector loads)
  uint32_t rowoff[LOAD == kLoadRVec ? 1 : ROWS];
  uint32_t tail_mask;                    // KTAIL: bit i = instruction i of this lane asks for k below K in the last k tile
  bool active, k_inside;
  u32x4 regs[NREG];

  __device__ __forceinline__ void init(const uint16_t* p, const GemmMode& rmode, const GemmMode& kmode, uint32_t row0, uint32_t extent,
                                       uint32_t Ktot, uint32_t tid) {
    base = p;
    // every offset the lanes present is inside the operand by construction (rows are clamped, k tiles whole), except the
    // offset 0xFFFFFFFF that stands for "past K" in a short last k tile: it is out of the buffer's range whatever the range
    if constexpr (DIRECT) rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p), 0, 0xFFFFFFFFu, 0x00020000);
    K = Ktot;
    tail_mask = 0u;
    const uint32_t k_rem = Ktot - (Ktot - 1u) / kGemmBK * kGemmBK;   // k present in the last k tile (1 .. 64)
    kv = gemm_lane_kvec(LOAD, tid);
    row_in_tile = gemm_lane_row(LOAD, tid, 0);
    active = LOAD != kLoadRVec || BR >= kBlock || tid < (uint32_t)BR;   // whole wavefronts: lanes 128.. of a 128-row tile
    if constexpr (LOAD == kLoadRVec) {
      rowoff[0] = gemm_mode_eval(rmode, gemm_clamp_row(LOAD, row0 + (active ? row_in_tile : 0u), extent));
    } else if constexpr (LOAD == kLoadKDirect) {
      // per instruction: offset of the row it fills plus the k vector its slot holds (k tiles are contiguous along k)
#pragma unroll
      for (int i = 0; i < ROWS; ++i) {
        const uint32_t row = gemm_direct_row(ROWS, tid, (uint32_t)i);
        rowoff[i] = 2u * (gemm_mode_eval(rmode, gemm_clamp_row(LOAD, row0 + row, extent)) + 8u * gemm_direct_kvec(row, tid));   // bytes
        tail_mask |= (8u * gemm_direct_kvec(row, tid) < k_rem ? 1u : 0u) << i;
      }
      row_in_tile = (uint32_t)__builtin_amdgcn_readfirstlane((int)(tid >> 6)) * ROWS;   // the wavefront's first KiB of the tile (uniform)
    } else if constexpr (LOAD == kLoadRDirect) {
      // per instruction: offset of the 8 rows its slot holds plus that of the slot's k row (an even step of the k mode's
      // first leaf from the tile's first k)
#pragma unroll
      for (int i = 0; i < ROWS; ++i) {
        uint32_t k, row;
        gemm_rdirect_unit(BR, ROWS, tid, (uint32_t)i, &k, &row);
        rowoff[i] = 2u * (gemm_mode_eval(rmode, gemm_clamp_row(LOAD, row0 + row, extent)) + k * kmode.lead_stride);   // bytes
        tail_mask |= (k < k_rem ? 1u : 0u) << i;
      }
      row_in_tile = (uint32_t)__builtin_amdgcn_readfirstlane((int)(tid >> 6)) * ROWS;   // the wavefront's first KiB of the tile (uniform)
    } else {
#pragma unroll
      for (int i = 0; i < ROWS; ++i) rowoff[i] = gemm_mode_eval(rmode, gemm_clamp_row(LOAD, row0 + gemm_lane_row(LOAD, tid, (uint32_t)i), extent));
    }
  }

  // Direct loads of one k tile: k_bytes is the tile's byte offset along the k mode (uniform), stage_tile the LDS byte offset
  // of this operand's tile in the stage the k tile goes to.  Lane l's 16 bytes land at byte 16 l of the instruction's KiB.
  // tail (uniform): the k tile is the short last one
  template <int FIRST = 0, int END = ROWS>
  __device__ __forceinline__ void fetch_direct(uint32_t k_bytes, uint32_t stage_tile, bool tail = false) {
    typedef __attribute__((address_space(3))) void lds_void;
    // The same dynamic LDS as the kernel's `lds`, under a name of its own on purpose: the compiler then sees no alias
    // between these writes and the fragment reads and adds no waits of its own (it would make every LDS read wait for
    // all loads in flight).  Ordering is stated by hand where it is needed: s_waitcnt vmcnt(n) before the k tile's
    // barrier, and the barrier itself.
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_bytes[];
    static_for<(END > FIRST ? END - FIRST : 0)>([&](auto d) {
      constexpr int i = FIRST + d;
      if constexpr (i >= 0 && i < ROWS) {
        uint32_t voff = rowoff[i];
        if constexpr (KTAIL) voff = (tail && ((tail_mask >> i) & 1u) == 0u) ? 0xFFFFFFFFu : voff;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void*)(lds_bytes + stage_tile + (row_in_tile + (uint32_t)i) * 1024u), 16,
                                                 (int)voff, (int)k_bytes, 0, 0);
      }
    });
  }

  __device__ __forceinline__ void fetch(uint32_t kt, const GemmMode& kmode) {
    const uint32_t k0 = kt * kGemmBK + kv * 8u;
    if constexpr (DIRECT) {
      (void)kmode;
    } else if constexpr (LOAD == kLoadKVec) {
      k_inside = k0 < K;
      const uint16_t* p = base + gemm_mode_eval(kmode, k_inside ? k0 : 0u);
#pragma unroll
      for (int i = 0; i < ROWS; ++i) regs[i] = *reinterpret_cast<const u32x4*>(p + rowoff[i]);
    } else if constexpr (LOAD == kLoadRVec) {
      k_inside = k0 < K;
      if (active) {
        const uint16_t* p = base + rowoff[0] + gemm_mode_eval(kmode, k_inside ? k0 : 0u);
        const uint32_t kstep = kmode.lead_stride;   // k0 .. k0 + 7 stay inside the leading leaf of the k mode
#pragma unroll
        for (int j = 0; j < 8; ++j) regs[j] = *reinterpret_cast<const u32x4*>(p + (uint32_t)j * kstep);
      }
    } else {
      uint32_t koff[8];
      bool in[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        in[j] = k0 + (uint32_t)j < K;
        koff[j] = gemm_mode_eval(kmode, in[j] ? k0 + (uint32_t)j : 0u);
      }
#pragma unroll
      for (int i = 0; i < ROWS; ++i) {
        uint32_t e[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          e[j] = (uint32_t)base[rowoff[i] + koff[j]];
          e[j] = in[j] ? e[j] : 0u;
        }
        regs[i] = u32x4{e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16)};
      }
    }
  }

  __device__ __forceinline__ void park(unsigned char* tile) {
    if constexpr (DIRECT) {
      (void)tile;   // already on its way into LDS
    } else if constexpr (LOAD == kLoadRVec) {
      if (active) {
        // the two k vectors of a quarter wavefront write rows of opposite parity (distinct LDS banks):
        // step ii of a lane with odd kv handles row ii ^ 1
        const bool flip = (kv & 1u) != 0;
        static_for<8>([&](auto ii) {
          const u32x4 v = transposed_row_b16(regs, ii / 2, ((ii & 1) != 0) != flip);
          const uint32_t i = (uint32_t)ii ^ (flip ? 1u : 0u);
          *reinterpret_cast<u32x4*>(tile + gemm_lds_offset(row_in_tile + i, kv)) = select_or_zero(k_inside, v);
        });
      }
    } else if constexpr (LOAD == kLoadKVec) {
#pragma unroll
      for (int i = 0; i < ROWS; ++i)
        *reinterpret_cast<u32x4*>(tile + gemm_lds_offset(row_in_tile + 32u * (uint32_t)i, kv)) = select_or_zero(k_inside, regs[i]);
    } else {
#pragma unroll
      for (int i = 0; i < ROWS; ++i) *reinterpret_cast<u32x4*>(tile + gemm_lds_offset(row_in_tile + 32u * (uint32_t)i, kv)) = regs[i];
    }
  }
};

// Workgroup barrier that orders LDS accesses only.  __syncthreads() would also wait for every load in flight (the direct
// loads count as global loads), which is exactly what the ring of tiles must not do; the caller states its own wait.
__device__ __forceinline__ void lds_barrier() {
  // the empty statements are compiler-only fences: no memory access is moved across the barrier, nothing is emitted
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// Byte offset of k tile t along an operand's k mode, for operands whose k tiles lie inside the mode's first leaf: stepping
// to the next tile adds 64 strides of that leaf until the leaf is exhausted; only then is the layout function evaluated again.
struct KTileOffset {
  uint32_t bytes, step, left;   // left: k tiles from the current one to the end of the first leaf's run
  __device__ __forceinline__ void seek(const GemmMode& k, uint32_t t) {
    bytes = 2u * gemm_mode_eval(k, t * kGemmBK);
    step = 2u * kGemmBK * k.lead_stride;
    if (k.n == 1) {
      left = 0xFFFFFFFFu;
    } else {
      uint32_t q, r;
      fd_divmod(t * kGemmBK, k.div[0], &q, &r);
      left = (k.div[0].div - r) / kGemmBK;
    }
  }
  __device__ __forceinline__ void next(const GemmMode& k, uint32_t t) {
    if (--left == 0) seek(k, t);
    else bytes += step;
  }
};

template <bool BF16, int WMB, int WNB, int A_LOAD, int B_LOAD, bool KTAIL = false>
__global__ __launch_bounds__(kBlock, (WMB <= 2 ? 2 : 1)) void gemm_kernel(GemmParams P, const uint16_t* __restrict__ A,
                                                                          const uint16_t* __restrict__ B, float* __restrict__ C) {
  constexpr int BM = 64 * WMB, BN = 64 * WNB;
  constexpr uint32_t A_BYTES = BM * 128u, STAGE = (BM + BN) * 128u;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

  const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
  const uint32_t wm = wave & 1u, wn = wave >> 1;
  uint32_t tm, tn;
  gemm_tile_of_order(P, gemm_tile_order_of_block(blockIdx.x, P.tiles_m * P.tiles_n), &tm, &tn);
  const uint32_t m0 = tm * BM, n0 = tn * BN;
  // batch entry (the third mode of the rank-3 form): slicing folds its offset into the three accessors (Sec. 2.5.1)
  A += gemm_mode_eval(P.a_l, blockIdx.y);
  B += gemm_mode_eval(P.b_l, blockIdx.y);
  C += gemm_mode_eval(P.c_l, blockIdx.y);

  OperandLoader<BM, A_LOAD, KTAIL> la;
  OperandLoader<BN, B_LOAD, KTAIL> lb;
  la.init(A, P.a_r, P.a_k, m0, P.M, P.K, tid);
  lb.init(B, P.b_r, P.b_k, n0, P.N, P.K, tid);

  f32x16 acc[WMB][WNB];
  static_for<WMB>([&](auto i) {
    static_for<WNB>([&](auto j) {
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    });
  });

  constexpr bool A_DIRECT = A_LOAD == kLoadKDirect || A_LOAD == kLoadRDirect, B_DIRECT = B_LOAD == kLoadKDirect || B_LOAD == kLoadRDirect;
  static_assert(A_DIRECT == B_DIRECT, "operands go straight into LDS as a pair");
  constexpr int KSTEPS = kGemmBK / 16;
  // LDS read instructions per k step: two transpose loads, or one 16-byte load, per fragment
  constexpr int DS_READS = WMB * (A_LOAD == kLoadRDirect ? 2 : 1) + WNB * (B_LOAD == kLoadRDirect ? 2 : 1);
  u32x4 af[2][WMB], bf[2][WNB];   // fragments, double-buffered in registers (one wavefront per SIMD: nothing else covers the LDS latency)
  auto multiply = [&](auto buf) {
    static_for<WMB>([&](auto i) {
      static_for<WNB>([&](auto j) { acc[i][j] = mfma_32x32x16<BF16>(af[buf][i], bf[buf][j], acc[i][j]); });
    });
  };

  if constexpr (A_DIRECT) {
    // Both tiles arrive by direct loads: no registers are held for them, so the loop is one basic block, software-pipelined
    // around a single barrier per k tile.  LDS is a ring of five slots of one operand tile each, filled in the order
    // A(0), B(0), A(1), B(1), A(2), ...: A(t) sits in slot 2t mod 5, B(t) in slot (2t + 1) mod 5.  While k tile t is
    // multiplied, two slots hold it, A(t + 1) is complete or landing, and B(t + 1) and A(t + 2) are being loaded: one
    // quarter of a tile's load instructions per k step, because the vector memory path moves about 64 bytes per clock and
    // CU and a tile issued at once stalls the wavefronts (and the matrix cores with them) at issue.
    // The barrier sits between k steps 2 and 3: by then every wavefront has read its last fragments of tile t (two slots
    // fall free: B(t + 2) and A(t + 3) go there), and tile t + 1 is complete: its first fragments are read while the MFMAs
    // of k step 3 run.  Past the last k tile the loads repeat it (in bounds, into slots nobody reads again).
    static_assert(BM == BN, "the ring's slots hold a tile of either operand");
    static_assert(KSTEPS == 4, "the loop below spells out the four k steps");
    constexpr uint32_t SLOT = A_BYTES;
    constexpr int RA = BM / 32, RB = BN / 32, MFMAS = WMB * WNB;   // load instructions per lane and operand tile
    // per fragment: the lane's LDS address for the tile's first k step in the slot being multiplied.  Row-major tiles: k step
    // kk flips slot bits (address ^ 32 kk); k-major tiles: k step kk is a constant offset.
    uint32_t a_fr[WMB], b_fr[WNB];
    static_for<WMB>([&](auto i) {
      const uint32_t row = wm * (WMB * 32u) + 32u * (uint32_t)i;
      a_fr[i] = A_LOAD == kLoadRDirect ? gemm_rdirect_frag_offset(BM, lane, row, 8u * mfma_ab_kvec(lane))
                                       : gemm_lds_offset(row + mfma_ab_row(lane), mfma_ab_kvec(lane));
    });
    static_for<WNB>([&](auto j) {
      const uint32_t row = wn * (WNB * 32u) + 32u * (uint32_t)j;
      b_fr[j] = SLOT + (B_LOAD == kLoadRDirect ? gemm_rdirect_frag_offset(BN, lane, row, 8u * mfma_ab_kvec(lane))
                                               : gemm_lds_offset(row + mfma_ab_row(lane), mfma_ab_kvec(lane)));
    });
    auto read_fragments = [&](auto kk, auto buf) {
      static_for<WMB>([&](auto i) {
        if constexpr (A_LOAD == kLoadRDirect) af[buf][i] = lds_read_tr_16x8<BM>(lds + a_fr[i], kk);
        else af[buf][i] = *reinterpret_cast<const u32x4*>(lds + (a_fr[i] ^ (32u * (uint32_t)kk)));
      });
      static_for<WNB>([&](auto j) {
        if constexpr (B_LOAD == kLoadRDirect) bf[buf][j] = lds_read_tr_16x8<BN>(lds + b_fr[j], kk);
        else bf[buf][j] = *reinterpret_cast<const u32x4*>(lds + (b_fr[j] ^ (32u * (uint32_t)kk)));
      });
    };
    // issue order inside a k step: its loads and LDS reads spread evenly between the MFMAs (the reads over the first
    // `span` of them)
    auto issue_order = [&](auto loads_c, auto span_c) {
      constexpr int LOADS = loads_c, SPAN = span_c;
      static_for<MFMAS>([&](auto g) {
        constexpr int loads = LOADS * (g + 1) / MFMAS - LOADS * g / MFMAS;
        constexpr int reads = g < SPAN ? DS_READS * (g + 1) / SPAN - DS_READS * g / SPAN : 0;
        if constexpr (loads > 0) __builtin_amdgcn_sched_group_barrier(0x010, loads, 0);
        if constexpr (reads > 0) __builtin_amdgcn_sched_group_barrier(0x100, reads, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      });
    };
    auto next_slot = [](uint32_t slot) { return slot + 2u >= 5u ? slot + 2u - 5u : slot + 2u; };
    // s_waitcnt vmcnt(n) lgkmcnt(0): all but the n youngest loads have landed, every LDS read has returned
    auto wait_loads_but = [](auto n) {
      constexpr int N = decltype(n)::value;
      static_assert(N >= 0 && N < 64, "vmcnt has six bits");
      __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0070);
    };

    const uint32_t last = P.k_tiles - 1u;
    KTileOffset ka, kb;   // of the newest k tile requested for A and for B
    ka.seek(P.a_k, 0u);
    kb.seek(P.b_k, 0u);
    // (the last argument of a fetch: the k tile it asks for is the last one, which KTAIL kernels load short)
    la.fetch_direct(ka.bytes, 0u * SLOT, last == 0u);
    lb.fetch_direct(kb.bytes, 1u * SLOT, last == 0u);
    __builtin_amdgcn_sched_barrier(0x038F);   // k tile 0's loads stay the oldest: the first wait below counts from the youngest
    ka.seek(P.a_k, last < 1u ? last : 1u);
    kb.seek(P.b_k, last < 1u ? last : 1u);
    la.fetch_direct(ka.bytes, 2u * SLOT, last <= 1u);
    lb.fetch_direct(kb.bytes, 3u * SLOT, last <= 1u);
    ka.seek(P.a_k, last < 2u ? last : 2u);
    la.fetch_direct(ka.bytes, 4u * SLOT, last <= 2u);
    wait_loads_but(std::integral_constant<int, 2 * RA + RB>{});   // k tile 0 has landed
    lds_barrier();
    read_fragments(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
    uint32_t sa = 0u, sb = 1u;   // slots of the k tile being multiplied
    for (uint32_t kt = 0; kt < P.k_tiles; ++kt) {
      const uint32_t s_b1 = next_slot(sb), s_a2 = next_slot(next_slot(sa));   // slots of B(kt + 1) and A(kt + 2)
      // k step 0: second half of B(kt + 1); k steps 1 and 2: A(kt + 2)
      const bool b1_last = kt + 1u >= last, a2_last = kt + 2u >= last;   // B(kt + 1) / A(kt + 2) and B(kt + 2) are the last k tile
      lb.template fetch_direct<RB / 2, RB>(kb.bytes, s_b1 * SLOT, b1_last);
      read_fragments(std::integral_constant<int, 1>{}, std::integral_constant<int, 1>{});
      multiply(std::integral_constant<int, 0>{});
      issue_order(std::integral_constant<int, RB - RB / 2>{}, std::integral_constant<int, MFMAS>{});
      // The wait before the barrier counts loads: all but the RA youngest must have landed, and those must be A(kt + 2)'s.
      // So no load of B may be scheduled behind a load of A: nothing but vector memory instructions is held back here
      // (mask: ALU, VALU, SALU, MFMA and LDS instructions may cross).
      __builtin_amdgcn_sched_barrier(0x038F);
      la.template fetch_direct<0, RA / 2>(ka.bytes, s_a2 * SLOT, a2_last);
      read_fragments(std::integral_constant<int, 2>{}, std::integral_constant<int, 0>{});
      multiply(std::integral_constant<int, 1>{});
      issue_order(std::integral_constant<int, RA / 2>{}, std::integral_constant<int, MFMAS>{});
      la.template fetch_direct<RA / 2, RA>(ka.bytes, s_a2 * SLOT, a2_last);
      read_fragments(std::integral_constant<int, 3>{}, std::integral_constant<int, 1>{});
      multiply(std::integral_constant<int, 0>{});
      // the reads before the barrier over the first half of the MFMAs, so that the last one has returned when the last MFMA is issued
      issue_order(std::integral_constant<int, RA - RA / 2>{}, std::integral_constant<int, (MFMAS + 1) / 2>{});
      wait_loads_but(std::integral_constant<int, RA>{});   // k tile kt + 1 has landed; A(kt + 2) may still be on its way
      lds_barrier();
      if (kt + 2u <= last) kb.next(P.b_k, kt + 2u);
      if (kt + 3u <= last) ka.next(P.a_k, kt + 3u);
      // k step 3: first half of B(kt + 2), into the slot A(kt) leaves
      lb.template fetch_direct<0, RB / 2>(kb.bytes, sa * SLOT, a2_last);
      const uint32_t sa_next = next_slot(sa), sb_next = next_slot(sb);
      const uint32_t da = (sa_next - sa) * SLOT, db = (sb_next - sb) * SLOT;
      static_for<WMB>([&](auto i) { a_fr[i] += da; });
      static_for<WNB>([&](auto j) { b_fr[j] += db; });
      sa = sa_next;
      sb = sb_next;
      read_fragments(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
      multiply(std::integral_constant<int, 1>{});
      issue_order(std::integral_constant<int, RB / 2>{}, std::integral_constant<int, MFMAS>{});
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);   // the repeated loads of the last k tile end before the wavefront does
  } else {
    la.fetch(0, P.a_k);
    lb.fetch(0, P.b_k);
    la.park(lds);
    lb.park(lds + A_BYTES);
    __syncthreads();

    // The loads of k tile kt + 1 are issued before the MFMAs of k tile kt and parked after them; the fragments of k step
    // kk + 1 are read from LDS while the MFMAs of step kk run.
    const uint32_t a_row = wm * (WMB * 32u) + mfma_ab_row(lane), b_row = wn * (WNB * 32u) + mfma_ab_row(lane);
    auto read_fragments = [&](const unsigned char* stage, auto kk, auto buf) {
      const uint32_t kvec = 2u * (uint32_t)kk + mfma_ab_kvec(lane);
      static_for<WMB>([&](auto i) { af[buf][i] = *reinterpret_cast<const u32x4*>(stage + gemm_lds_offset(a_row + 32u * (uint32_t)i, kvec)); });
      static_for<WNB>([&](auto j) { bf[buf][j] = *reinterpret_cast<const u32x4*>(stage + A_BYTES + gemm_lds_offset(b_row + 32u * (uint32_t)j, kvec)); });
    };
    read_fragments(lds, std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
    for (uint32_t kt = 0; kt < P.k_tiles; ++kt) {
      const unsigned char* cur = lds + (kt & 1u) * STAGE;
      unsigned char* nxt = lds + ((kt & 1u) ^ 1u) * STAGE;
      const bool more = kt + 1 < P.k_tiles;
      if (more) {
        la.fetch(kt + 1, P.a_k);
        lb.fetch(kt + 1, P.b_k);
      }
      static_for<KSTEPS>([&](auto kk) {
        constexpr int buf = kk % 2;
        if constexpr (kk + 1 < KSTEPS) read_fragments(cur, std::integral_constant<int, kk + 1>{}, std::integral_constant<int, buf ^ 1>{});
        multiply(std::integral_constant<int, buf>{});
        if constexpr (kk + 1 < KSTEPS) {
          // issue order: one LDS read, then two MFMAs, repeated
          static_for<WMB + WNB>([&](auto) {
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, (WMB * WNB) / (WMB + WNB), 0);
          });
        }
      });
      if (more) {
        la.park(nxt);
        lb.park(nxt + A_BYTES);
      }
      __syncthreads();
      if (more) read_fragments(nxt, std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
    }
  }

  // C(m,n) += acc: a lane holds column n = lane % 32 of each fragment and 4 groups of 4 consecutive rows
  static_for<WNB>([&](auto j) {
    const uint32_t n = n0 + wn * (WNB * 32u) + 32u * (uint32_t)j + mfma_c_col(lane);
    const bool n_in = n < P.N;
    const uint32_t noff = gemm_mode_eval(P.c_n, n_in ? n : 0u);
    if (P.c_vec) {
      // All 4 WMB vectors of this fragment column are loaded before the first is stored.  Written as one read-modify-write
      // after the other, every load waits behind the store before it (they may alias as far as the compiler knows) and a
      // lane pays 16 WMB memory round trips per tile instead of 4: measured 0.905 -> 0.873 ms on 8192^3.  Loading column
      // j + 1 before column j is stored (two columns of registers) measured slower again (0.885 ms).
      f32x4 cv[WMB][4];
      static_for<WMB>([&](auto i) {
        static_for<4>([&](auto g) {
          const uint32_t m = m0 + wm * (WMB * 32u) + 32u * (uint32_t)i + mfma_c_row(lane, 4u * (uint32_t)g);
          if (n_in && m < P.M) cv[i][g] = *reinterpret_cast<const f32x4*>(C + gemm_mode_eval(P.c_m, m) + noff);
        });
      });
      static_for<WMB>([&](auto i) {
        static_for<4>([&](auto g) {
          const uint32_t m = m0 + wm * (WMB * 32u) + 32u * (uint32_t)i + mfma_c_row(lane, 4u * (uint32_t)g);
          if (n_in && m < P.M) {
            f32x4 c = cv[i][g];
            static_for<4>([&](auto v) { c[(int)v] += acc[i][j][4 * g + v]; });
            *reinterpret_cast<f32x4*>(C + gemm_mode_eval(P.c_m, m) + noff) = c;
          }
        });
      });
    } else {
      // element by element, for the same reason a fragment (16 elements per lane) at a time
      static_for<WMB>([&](auto i) {
        float cs[4][4];
        static_for<4>([&](auto g) {
          const uint32_t m = m0 + wm * (WMB * 32u) + 32u * (uint32_t)i + mfma_c_row(lane, 4u * (uint32_t)g);
          static_for<4>([&](auto v) {
            if (n_in && m + (uint32_t)v < P.M) cs[g][v] = C[gemm_mode_eval(P.c_m, m + (uint32_t)v) + noff];
          });
        });
        static_for<4>([&](auto g) {
          const uint32_t m = m0 + wm * (WMB * 32u) + 32u * (uint32_t)i + mfma_c_row(lane, 4u * (uint32_t)g);
          static_for<4>([&](auto v) {
            if (n_in && m + (uint32_t)v < P.M) C[gemm_mode_eval(P.c_m, m + (uint32_t)v) + noff] = cs[g][v] + acc[i][j][4 * g + v];
          });
        });
      });
    }
  });
}

// ---------------------------------------------------------------------------------------------
// Launchers
// ---------------------------------------------------------------------------------------------

template <bool BF16, int WB, int A_LOAD, int B_LOAD, bool KTAIL>
static inline hipError_t launch_gemm_abk(const lc_gemm_plan& plan, const uint16_t* a, const uint16_t* b, float* c, hipStream_t s) {
  if (plan.lds_bytes > 64 * 1024) {
    static std::atomic<bool> raised{false};   // one flag per instantiation: the attribute belongs to the kernel function
    if (!raised.load(std::memory_order_acquire)) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_kernel<BF16, WB, WB, A_LOAD, B_LOAD, KTAIL>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
      if (e != hipSuccess) return e;
      raised.store(true, std::memory_order_release);
    }
  }
  const unsigned grid = plan.params.tiles_m * plan.params.tiles_n;
  hipLaunchKernelGGL((gemm_kernel<BF16, WB, WB, A_LOAD, B_LOAD, KTAIL>), dim3(grid, plan.params.L), dim3(kBlock), plan.lds_bytes, s, plan.params, a, b, c);
  return hipSuccess;
}
template <bool BF16, int WB, int A_LOAD, int B_LOAD>
static inline hipError_t launch_gemm_ab(const lc_gemm_plan& plan, const uint16_t* a, const uint16_t* b, float* c, hipStream_t s) {
  // a short last k tile: direct loads only (the staged loads zero what lies past K in registers)
  if constexpr (A_LOAD == kLoadKDirect || A_LOAD == kLoadRDirect)
    if (plan.params.K % kGemmBK != 0) return launch_gemm_abk<BF16, WB, A_LOAD, B_LOAD, true>(plan, a, b, c, s);
  return launch_gemm_abk<BF16, WB, A_LOAD, B_LOAD, false>(plan, a, b, c, s);
}
// vector loads are compiled per pair of modes; an operand that needs element loads takes the other one along.
// Operands that go straight into LDS do so as a pair (the planner marks both or neither).
template <bool BF16, int WB, int A_LOAD, int FIRST, int SECOND>
static inline hipError_t launch_gemm_a(const lc_gemm_plan& plan, int lb, const uint16_t* a, const uint16_t* b, float* c, hipStream_t s) {
  if (lb == FIRST) return launch_gemm_ab<BF16, WB, A_LOAD, FIRST>(plan, a, b, c, s);
  if (lb == SECOND) return launch_gemm_ab<BF16, WB, A_LOAD, SECOND>(plan, a, b, c, s);
  return hipErrorInvalidValue;
}
template <bool BF16, int WB>
static inline hipError_t launch_gemm(const lc_gemm_plan& plan, const uint16_t* a, const uint16_t* b, float* c, hipStream_t s) {
  const int la = gemm_effective_load(plan.params.a_load, plan.params.a_direct), lb = gemm_effective_load(plan.params.b_load, plan.params.b_direct);
  if (la == kLoadElem && lb == kLoadElem) return launch_gemm_ab<BF16, WB, kLoadElem, kLoadElem>(plan, a, b, c, s);
  if (la == kLoadKDirect) return launch_gemm_a<BF16, WB, kLoadKDirect, kLoadKDirect, kLoadRDirect>(plan, lb, a, b, c, s);
  if (la == kLoadRDirect) return launch_gemm_a<BF16, WB, kLoadRDirect, kLoadKDirect, kLoadRDirect>(plan, lb, a, b, c, s);
  if (la == kLoadKVec) return launch_gemm_a<BF16, WB, kLoadKVec, kLoadKVec, kLoadRVec>(plan, lb, a, b, c, s);
  if (la == kLoadRVec) return launch_gemm_a<BF16, WB, kLoadRVec, kLoadKVec, kLoadRVec>(plan, lb, a, b, c, s);
  return hipErrorInvalidValue;
}

}  // namespace lc
