// Device code of the generic GEMM, included by the translation units that instantiate it (one per element type
// and tile size, so that they compile in parallel).
// Generic GEMM for gfx950 (CDNA4, wave64): C(m,n) += A(m,k) * B(n,k) (Sec. 2.6.2 of "CuTe Layout
// Representation and Algebra") for operands described by layouts, on the matrix cores
// (v_mfma_f32_32x32x16 bf16 / f16, fp32 accumulation).
//
// One workgroup of 4 wavefronts owns a BM x BN tile of C; wavefront (wm, wn) owns a (BM/2) x (BN/2)
// quarter as WMB x WNB fragments of 32 x 32.  Per k tile of 64 the operand tiles pass through LDS,
// double-buffered: the loads of k tile t+1 are issued before the MFMAs of k tile t and parked after
// them.  How a tile is loaded depends on which mode of the operand is contiguous (GemmLoad).
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

__device__ __forceinline__ u32x4 select_or_zero(bool keep, u32x4 v) {
  return u32x4{keep ? v[0] : 0u, keep ? v[1] : 0u, keep ? v[2] : 0u, keep ? v[3] : 0u};
}

// One operand (A or B) of one workgroup: issues the global loads of a k tile into registers, parks them in LDS.
// Loads are unconditional from clamped coordinates (always inside the tensor); what lies past K is zeroed
// in registers afterwards, so the loop carries no divergent branch.
template <int BR, int LOAD>
struct OperandLoader {
  static constexpr int ROWS = BR / 32;                                    // rows per lane for k-vector / element loads
  static constexpr int NREG = LOAD == kLoadRVec ? 8 : (LOAD == kLoadKDirect ? 1 : ROWS);
  const uint16_t* base;
  uint32_t K, kv, row_in_tile;           // row_in_tile: first row of the lane (block row for row-vector loads)
  uint32_t rowoff[LOAD == kLoadRVec ? 1 : ROWS];
  bool active, k_inside;
  u32x4 regs[NREG];

  __device__ __forceinline__ void init(const uint16_t* p, const GemmMode& rmode, uint32_t row0, uint32_t extent, uint32_t Ktot,
                                       uint32_t tid) {
    base = p;
    K = Ktot;
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
        rowoff[i] = gemm_mode_eval(rmode, gemm_clamp_row(LOAD, row0 + row, extent)) + 8u * gemm_direct_kvec(row, tid);
      }
      row_in_tile = (tid >> 6) * ROWS * 8u;   // first row this wavefront fills
    } else {
#pragma unroll
      for (int i = 0; i < ROWS; ++i) rowoff[i] = gemm_mode_eval(rmode, gemm_clamp_row(LOAD, row0 + gemm_lane_row(LOAD, tid, (uint32_t)i), extent));
    }
  }

  // stage_tile: LDS byte offset of this operand's tile in the stage the k tile goes to (used by kLoadKDirect only)
  __device__ __forceinline__ void fetch(uint32_t kt, const GemmMode& kmode, uint32_t stage_tile) {
    const uint32_t k0 = kt * kGemmBK + kv * 8u;
    if constexpr (LOAD == kLoadKDirect) {
      extern __shared__ __attribute__((aligned(16))) unsigned char lds_bytes[];
      const uint16_t* p = base + gemm_mode_eval(kmode, kt * kGemmBK);
#pragma unroll
      for (int i = 0; i < ROWS; ++i)
        __builtin_amdgcn_global_load_lds(p + rowoff[i], reinterpret_cast<uint32_t*>(lds_bytes + stage_tile + (row_in_tile + 8u * (uint32_t)i) * 128u), 16, 0, 0);
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
    if constexpr (LOAD == kLoadKDirect) {
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

template <bool BF16, int WMB, int WNB, int A_LOAD, int B_LOAD>
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

  OperandLoader<BM, A_LOAD> la;
  OperandLoader<BN, B_LOAD> lb;
  la.init(A, P.a_r, m0, P.M, P.K, tid);
  lb.init(B, P.b_r, n0, P.N, P.K, tid);

  f32x16 acc[WMB][WNB];
  static_for<WMB>([&](auto i) {
    static_for<WNB>([&](auto j) {
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    });
  });

  constexpr bool ANY_DIRECT = A_LOAD == kLoadKDirect || B_LOAD == kLoadKDirect;
  la.fetch(0, P.a_k, 0u);
  lb.fetch(0, P.b_k, A_BYTES);
  la.park(lds);
  lb.park(lds + A_BYTES);
  if constexpr (ANY_DIRECT) __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wavefront's direct loads have landed in LDS
  __syncthreads();

  // Fragments are double-buffered in registers: those of k step kk + 1 are read from LDS while the MFMAs of
  // step kk run (one wavefront per SIMD: nothing else would cover the LDS latency).
  const uint32_t a_row = wm * (WMB * 32u) + mfma_ab_row(lane), b_row = wn * (WNB * 32u) + mfma_ab_row(lane);
  u32x4 af[2][WMB], bf[2][WNB];
  auto read_fragments = [&](const unsigned char* stage, auto kk, auto buf) {
    const uint32_t kvec = 2u * (uint32_t)kk + mfma_ab_kvec(lane);
    static_for<WMB>([&](auto i) { af[buf][i] = *reinterpret_cast<const u32x4*>(stage + gemm_lds_offset(a_row + 32u * (uint32_t)i, kvec)); });
    static_for<WNB>([&](auto j) { bf[buf][j] = *reinterpret_cast<const u32x4*>(stage + A_BYTES + gemm_lds_offset(b_row + 32u * (uint32_t)j, kvec)); });
  };
  constexpr int KSTEPS = kGemmBK / 16;
  read_fragments(lds, std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
  for (uint32_t kt = 0; kt < P.k_tiles; ++kt) {
    const unsigned char* cur = lds + (kt & 1u) * STAGE;
    unsigned char* nxt = lds + ((kt & 1u) ^ 1u) * STAGE;
    const bool more = kt + 1 < P.k_tiles;
    const uint32_t nxt_offset = ((kt & 1u) ^ 1u) * STAGE;
    if (more) {
      la.fetch(kt + 1, P.a_k, nxt_offset);
      lb.fetch(kt + 1, P.b_k, nxt_offset + A_BYTES);
    }
    static_for<KSTEPS>([&](auto kk) {
      constexpr int buf = kk % 2;
      if constexpr (kk + 1 < KSTEPS) read_fragments(cur, std::integral_constant<int, kk + 1>{}, std::integral_constant<int, buf ^ 1>{});
      static_for<WMB>([&](auto i) {
        static_for<WNB>([&](auto j) { acc[i][j] = mfma_32x32x16<BF16>(af[buf][i], bf[buf][j], acc[i][j]); });
      });
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
    if constexpr (ANY_DIRECT) __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0) before telling the others the stage is complete
    __syncthreads();
    if (more) read_fragments(nxt, std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
  }

  // C(m,n) += acc: a lane holds column n = lane % 32 of each fragment and 4 groups of 4 consecutive rows
  static_for<WNB>([&](auto j) {
    const uint32_t n = n0 + wn * (WNB * 32u) + 32u * (uint32_t)j + mfma_c_col(lane);
    const bool n_in = n < P.N;
    const uint32_t noff = gemm_mode_eval(P.c_n, n_in ? n : 0u);
    static_for<WMB>([&](auto i) {
      static_for<4>([&](auto g) {
        const uint32_t m = m0 + wm * (WMB * 32u) + 32u * (uint32_t)i + mfma_c_row(lane, 4u * (uint32_t)g);
        if (P.c_vec) {
          if (n_in && m < P.M) {
            f32x4* p = reinterpret_cast<f32x4*>(C + gemm_mode_eval(P.c_m, m) + noff);
            f32x4 c = *p;
            static_for<4>([&](auto v) { c[(int)v] += acc[i][j][4 * g + v]; });
            *p = c;
          }
        } else {
          static_for<4>([&](auto v) {
            if (n_in && m + (uint32_t)v < P.M) C[gemm_mode_eval(P.c_m, m + (uint32_t)v) + noff] += acc[i][j][4 * g + v];
          });
        }
      });
    });
  });
}

// ---------------------------------------------------------------------------------------------
// Launchers
// ---------------------------------------------------------------------------------------------

template <bool BF16, int WB, int A_LOAD, int B_LOAD>
static inline hipError_t launch_gemm_ab(const lc_gemm_plan& plan, const uint16_t* a, const uint16_t* b, float* c, hipStream_t s) {
  if (plan.lds_bytes > 64 * 1024) {
    static std::atomic<bool> raised{false};   // one flag per instantiation: the attribute belongs to the kernel function
    if (!raised.load(std::memory_order_acquire)) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_kernel<BF16, WB, WB, A_LOAD, B_LOAD>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
      if (e != hipSuccess) return e;
      raised.store(true, std::memory_order_release);
    }
  }
  const unsigned grid = plan.params.tiles_m * plan.params.tiles_n;
  hipLaunchKernelGGL((gemm_kernel<BF16, WB, WB, A_LOAD, B_LOAD>), dim3(grid, plan.params.L), dim3(kBlock), plan.lds_bytes, s, plan.params, a, b, c);
  return hipSuccess;
}
// vector loads are compiled per pair of modes; an operand that needs element loads takes the other one along.
// A k-vector operand goes straight into LDS (kLoadKDirect) when the plan says it qualifies.
template <bool BF16, int WB, int A_LOAD>
static inline hipError_t launch_gemm_a(const lc_gemm_plan& plan, int lb, const uint16_t* a, const uint16_t* b, float* c, hipStream_t s) {
  if (lb == kLoadKDirect) return launch_gemm_ab<BF16, WB, A_LOAD, kLoadKDirect>(plan, a, b, c, s);
  if (lb == kLoadKVec) return launch_gemm_ab<BF16, WB, A_LOAD, kLoadKVec>(plan, a, b, c, s);
  if (lb == kLoadRVec) return launch_gemm_ab<BF16, WB, A_LOAD, kLoadRVec>(plan, a, b, c, s);
  return hipErrorInvalidValue;
}
template <bool BF16, int WB>
static inline hipError_t launch_gemm(const lc_gemm_plan& plan, const uint16_t* a, const uint16_t* b, float* c, hipStream_t s) {
  int la = plan.params.a_load, lb = plan.params.b_load;
  if (la == kLoadElem && lb == kLoadElem) return launch_gemm_ab<BF16, WB, kLoadElem, kLoadElem>(plan, a, b, c, s);
  if (la == kLoadKVec && plan.params.a_direct) la = kLoadKDirect;
  if (lb == kLoadKVec && plan.params.b_direct) lb = kLoadKDirect;
  if (la == kLoadKDirect) return launch_gemm_a<BF16, WB, kLoadKDirect>(plan, lb, a, b, c, s);
  if (la == kLoadKVec) return launch_gemm_a<BF16, WB, kLoadKVec>(plan, lb, a, b, c, s);
  if (la == kLoadRVec) return launch_gemm_a<BF16, WB, kLoadRVec>(plan, lb, a, b, c, s);
  return hipErrorInvalidValue;
}

}  // namespace lc
