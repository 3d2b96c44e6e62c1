// Kernel arguments and index arithmetic of the generic GEMM (Sec. 2.6.2 of "CuTe Layout Representation
// and Algebra"): C(m,n) += A(m,k) * B(n,k) for tensors given by rank-2 layouts.  A rank-2 layout is
// the sum of the layout functions of its two modes, L(r,k) = L_0(r) + L_1(k) (Eq. innerprod over the
// concatenation, Eq. concat), so each operand travels as two coalesced modes.  The functions here are
// shared by the device kernel and by the host walk that checks a plan's addresses without a GPU.
#pragma once
#include "kernel_params.hpp"

namespace lc {

constexpr int kGemmMaxLeaves = 4;   // leaves of one coalesced top-level mode
constexpr int kGemmBK = 64;         // k extent of a tile: 8 vectors of 8 sixteen-bit elements = one 128-byte LDS row

// how an operand tile is brought from global memory into LDS
enum GemmLoad : int32_t {
  kLoadKVec = 0,   // 16-byte vectors along k (k-mode leads with a stride-1 leaf): straight into place
  kLoadRVec = 1,   // 16-byte vectors along the row mode (m or n): 8x8 blocks transposed in registers
  kLoadElem = 2,   // element by element: any layout, any extent
  // kLoadKVec without the registers: 16-byte vectors along k sent by the memory pipeline straight into LDS.  Needs k tiles
  // that are contiguous along k (whole tiles inside the k mode's first leaf; a k mode of one leaf may end in a short tile,
  // whose lanes past K are answered with zeros); chosen at launch, a plan still says kLoadKVec.
  kLoadKDirect = 3,
  // kLoadRVec without the registers: the tile goes into LDS as it lies in memory (k rows of BR contiguous elements) and the
  // fragments are read with the LDS transpose load (ds_read_b64_tr_b16).  Same conditions; a plan still says kLoadRVec.
  kLoadRDirect = 4
};

// One coalesced mode: integral coordinate -> offset in elements (all offsets of a GEMM operand fit 31 bits).
// The leaves but the last are reduced modulo their extents, the last one takes what is left (Eq. idx2crd).
// Storage is branch-free for the kernel: the reduced leaves sit in front, padded with extent-1 leaves
// (quotient passes through, remainder 0), and the last leaf's stride always sits in last_stride.
struct GemmMode {
  int32_t n;                              // leaves of the coalesced mode (1 .. kGemmMaxLeaves)
  FastDiv div[kGemmMaxLeaves - 1];
  uint32_t stride[kGemmMaxLeaves - 1];
  uint32_t last_stride;
  uint32_t lead_stride;                   // stride of the first leaf (one step of the coordinate while it stays inside that leaf)
};
LC_HD uint32_t gemm_mode_eval(const GemmMode& g, uint32_t i) {
  uint32_t off = 0;
#pragma unroll
  for (int k = 0; k < kGemmMaxLeaves - 1; ++k) {
    uint32_t q, r;
    fd_divmod(i, g.div[k], &q, &r);
    off += r * g.stride[k];
    i = q;
  }
  return off + i * g.last_stride;
}

struct GemmParams {
  GemmMode a_r, a_k, b_r, b_k, c_m, c_n;   // A over (M,K), B over (N,K), C over (M,N)
  GemmMode a_l, b_l, c_l;                  // batch modes of the rank-3 form (Sec. 1): "1:0" for plain matrices
  uint32_t M, N, K, L;
  uint32_t tiles_m, tiles_n, k_tiles;
  int32_t a_load, b_load;                  // GemmLoad
  int32_t a_direct, b_direct;              // 1: the operand goes straight into LDS (kLoadKVec -> kLoadKDirect, kLoadRVec -> kLoadRDirect)
  int32_t c_vec;                           // 1: four consecutive m are contiguous and 16-byte aligned in C
  uint32_t group_m;                        // tile rows walked together before moving on along n
};

// the load the kernel runs for an operand the plan classified as `load`
LC_HD int32_t gemm_effective_load(int32_t load, int32_t direct) {
  if (!direct) return load;
  return load == kLoadKVec ? (int32_t)kLoadKDirect : (load == kLoadRVec ? (int32_t)kLoadRDirect : load);
}

// ---------------------------------------------------------------------------------------------
// Workgroup -> tile.  Workgroups are handed to the 8 XCDs round-robin and every XCD has its own L2,
// so XCD x takes a contiguous stretch of the tile order; the order itself walks group_m tile rows
// together along n, which keeps the A rows and B rows of concurrently running tiles few.
// ---------------------------------------------------------------------------------------------
constexpr uint32_t kXcds = 8;
LC_HD uint32_t gemm_tile_order_of_block(uint32_t block, uint32_t n_tiles) {
  const uint32_t xcd = block % kXcds, slot = block / kXcds;
  const uint32_t base = n_tiles / kXcds, extra = n_tiles % kXcds;
  return xcd * base + (xcd < extra ? xcd : extra) + slot;
}
LC_HD void gemm_tile_of_order(const GemmParams& P, uint32_t t, uint32_t* tm, uint32_t* tn) {
  const uint32_t width = P.group_m * P.tiles_n;
  const uint32_t group = t / width, in = t % width;
  const uint32_t first = group * P.group_m;
  const uint32_t rows = (P.tiles_m - first) < P.group_m ? (P.tiles_m - first) : P.group_m;
  *tm = first + in % rows;
  *tn = in / rows;
}

// ---------------------------------------------------------------------------------------------
// Operand tile in LDS: BR rows (m or n) of kGemmBK elements, 128 bytes per row, eight 16-byte
// vectors per row.  Vector kv of row r sits at slot kv ^ r ^ (r >> 3) (low three bits): this is the
// XOR layout (Sec. 2.3.2) under which all three access patterns below touch 16 distinct 16-byte
// bank groups per 16 lanes: fragment reads (16 rows, one kv), k-vector writes (2 rows x 8 kv) and
// the writes of transposed 8x8 blocks (8 row groups x 2 kv, rows of opposite parity for odd kv).
// ---------------------------------------------------------------------------------------------
LC_HD uint32_t gemm_lds_offset(uint32_t row, uint32_t kv) { return row * 128u + (((kv ^ row ^ (row >> 3)) & 7u) << 4); }

// ---------------------------------------------------------------------------------------------
// Lane -> what it loads (256 lanes).
//   kLoadKVec / kLoadElem: k vector lane % 8 of rows lane / 8 + 32 i, i < BR / 32: a quarter wavefront
//                          (16 lanes, one pass of a 16-byte load) reads two rows of 128 contiguous bytes
//   kLoadRVec            : the 8x8 block of rows 8 b .. 8 b + 7, b = lane % 8 + 8 (lane / 64), and k vector
//                          (lane / 8) % 8 (lanes < BR only): a quarter wavefront reads, for each of its two k
//                          vectors, 128 contiguous bytes along the row mode
// Rows past the end of the mode are clamped to its last row (last 8-row group for kLoadRVec): the
// tile then holds a copy of valid data there, which only feeds entries of C that are never stored.
// k past K parks zeros.
// ---------------------------------------------------------------------------------------------
LC_HD uint32_t gemm_lane_kvec(int32_t load, uint32_t lane) { return load == kLoadRVec ? (lane >> 3) & 7u : lane & 7u; }
LC_HD uint32_t gemm_lane_row(int32_t load, uint32_t lane, uint32_t i) {
  return load == kLoadRVec ? ((lane & 7u) + 8u * (lane >> 6)) * 8u : (lane >> 3) + 32u * i;
}
// ---------------------------------------------------------------------------------------------
// kLoadRDirect: the operand tile in LDS is k-major: row k holds the BR elements (BR / 8 slots of 16 bytes) of that k,
// the 8-element group g of the row mode in slot g ^ 4 (k % 4).  A transpose load of 16 lanes reads 16 rows x 4 k
// (4 k rows x 32 bytes); with this XOR layout (Sec. 2.3.2) the two lane groups that share a pass (rows 0..15 and
// 16..31 of a fragment) and their 4 k rows touch 16 distinct 16-byte bank groups.
// ---------------------------------------------------------------------------------------------
LC_HD uint32_t gemm_rdirect_lds_offset(uint32_t BR, uint32_t k, uint32_t row) { return k * (BR * 2u) + ((((row >> 3) ^ (4u * (k & 3u)))) << 4) + (row & 7u) * 2u; }
// Instruction i of wavefront w fills 1 KiB = 64 slots; lane l's slot is unit (w R + i) 64 + l of the tile: its k row and
// the 8-row group it must ask memory for.
LC_HD void gemm_rdirect_unit(uint32_t BR, uint32_t rows_per_lane, uint32_t tid, uint32_t i, uint32_t* k, uint32_t* row) {
  const uint32_t unit = ((tid >> 6) * rows_per_lane + i) * 64u + (tid & 63u), slots = BR / 8u;
  *k = unit / slots;
  *row = ((unit % slots) ^ (4u * (*k & 3u))) * 8u;
}
// ds_read_b64_tr_b16 (checked on the GPU with an in-bounds probe): within each group of 16 lanes, result lane i element e
// is element i % 4 of the 8 bytes that lane 4 e + i / 4 of the group points at.  Lane j of a group therefore points at
// rows 4 (j % 4) .. + 3 of its group's 16 rows, at k step j / 4 of the 4: lane i then holds row i at k .. k + 3.
// Byte offset (inside the operand's tile) for fragment rows row_base .. row_base + 31, k = k_base .. k_base + 3:
LC_HD uint32_t gemm_rdirect_frag_offset(uint32_t BR, uint32_t lane, uint32_t row_base, uint32_t k_base) {
  const uint32_t j = lane & 15u;
  return gemm_rdirect_lds_offset(BR, k_base + (j >> 2), row_base + 16u * ((lane >> 4) & 1u) + 4u * (j & 3u));
}

// kLoadKDirect: instruction i of wavefront w fills the 1 KiB of LDS that holds rows 8 (w R + i) .. + 7 of the tile
// (R = BR / 32 instructions per lane); lane l lands at byte 16 l of it, i.e. row + l / 8, slot l % 8, and therefore
// asks for the k vector that lives in that slot: kv = slot ^ row ^ (row >> 3).
LC_HD uint32_t gemm_direct_row(uint32_t rows_per_lane, uint32_t tid, uint32_t i) { return ((tid >> 6) * rows_per_lane + i) * 8u + ((tid & 63u) >> 3); }
LC_HD uint32_t gemm_direct_kvec(uint32_t row, uint32_t tid) { return ((tid & 7u) ^ row ^ (row >> 3)) & 7u; }
LC_HD uint32_t gemm_clamp_row(int32_t load, uint32_t row, uint32_t extent) {
  const uint32_t last = load == kLoadRVec || load == kLoadRDirect ? extent - 8u : extent - 1u;
  return row < last ? row : last;
}

// ---------------------------------------------------------------------------------------------
// MFMA fragments of v_mfma_f32_32x32x16 (bf16 / f16), as thread-value layouts (Sec. 3.3.4):
//   A fragment (32 x 16): lane t holds A(t % 32, 8 (t / 32) + v), v < 8   -> ((32,2),8):((1,256),32) on m + 32 k
//   B fragment (32 x 16): lane t holds B(t % 32, 8 (t / 32) + v)          -> the same on n + 32 k
//   C fragment (32 x 32): lane t holds C(8 (v / 4) + 4 (t / 32) + v % 4, t % 32), v < 16
//                                                                          -> ((32,2),(4,4)):((32,4),(1,8)) on m + 32 n
// ---------------------------------------------------------------------------------------------
LC_HD uint32_t mfma_ab_row(uint32_t lane) { return lane & 31u; }
LC_HD uint32_t mfma_ab_kvec(uint32_t lane) { return lane >> 5; }            // which 8-element k vector of the 16
LC_HD uint32_t mfma_c_row(uint32_t lane, uint32_t v) { return 8u * (v >> 2) + 4u * (lane >> 5) + (v & 3u); }
LC_HD uint32_t mfma_c_col(uint32_t lane) { return lane & 31u; }

}  // namespace lc
