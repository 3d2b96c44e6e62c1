// Kernel argument blocks and the index arithmetic shared by the device kernels and the host-side
// plan checker.  Everything here is plain-old-data passed by value at launch: the planner does the
// layout algebra once on the host, the kernels only evaluate idx2crd / inner_product
// (Eq. idx2crd, Eq. innerprod of "CuTe Layout Representation and Algebra") on what is left.
#pragma once
#include <cstdint>

#if defined(__HIPCC__)
#include <hip/hip_runtime.h>
#define LC_HD __host__ __device__ inline
#else
#define LC_HD inline
#endif

namespace lc {

constexpr int kMaxModes = 8;          // joint / rest / micro modes per kernel
constexpr int kMaxGenericModes = 12;  // leaf modes per side in the element-wise kernel
constexpr int kBlock = 256;           // threads per workgroup = 4 wavefronts of 64
constexpr int kMaxMicroPerLane = 8;   // micro-tiles a lane owns per tile
constexpr int kMaxPicksPerLane = 32;  // vectors a lane stores per tile (micro-tiles per lane x longest vector)

// Division of a 31-bit unsigned value by a constant: q = (mulhi(n, mul) + n) >> shift
// (round-up multiplier of Granlund & Montgomery; exact for n < 2^31, any divisor in [1, 2^31)).
struct FastDiv {
  uint32_t mul, shift, div;
};

LC_HD uint32_t mulhi_u32(uint32_t a, uint32_t b) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __umulhi(a, b);
#else
  return (uint32_t)(((uint64_t)a * b) >> 32);
#endif
}
LC_HD uint32_t fd_div(uint32_t n, const FastDiv& f) { return (mulhi_u32(n, f.mul) + n) >> f.shift; }
// n -> (n / div, n % div)
LC_HD void fd_divmod(uint32_t n, const FastDiv& f, uint32_t* q, uint32_t* r) {
  *q = fd_div(n, f);
  *r = n - *q * f.div;
}
inline FastDiv make_fastdiv(uint32_t d) {
  FastDiv f;
  f.div = d;
  uint32_t l = 0;
  while ((1ull << l) < d) ++l;
  f.shift = l;
  f.mul = (uint32_t)((((1ull << l) - d) << 32) / d + 1);
  return f;
}

// ---------------------------------------------------------------------------------------------
// Element-wise kernel: dst[L_dst(i)] = src[L_src(i)] with both (coalesced) layouts evaluated per
// element.  Used when the two shapes have no common refinement.
// ---------------------------------------------------------------------------------------------
struct FlatLayoutArg {
  int32_t n_modes;
  FastDiv div[kMaxGenericModes];   // extents, leftmost mode first
  int64_t stride[kMaxGenericModes];
};
struct GenericParams {
  FlatLayoutArg src, dst;
  uint32_t n;                      // elements (< 2^31)
};
LC_HD int64_t flat_eval(const FlatLayoutArg& L, uint32_t i) {
  int64_t off = 0;
  for (int k = 0; k + 1 < L.n_modes; ++k) {
    uint32_t q, r;
    fd_divmod(i, L.div[k], &q, &r);
    off += (int64_t)r * L.stride[k];
    i = q;
  }
  return off + (int64_t)i * L.stride[L.n_modes - 1];
}

// ---------------------------------------------------------------------------------------------
// Direct kernel: joint modes (extent, src stride, dst stride) in destination order; consecutive
// lanes walk the destination-contiguous mode.  One work item = one access of W bytes on each side;
// all strides are in units of W bytes.  One more mode may be looped inside the thread (a stride-0
// source mode is then read once and written `loop_extent` times).
// ---------------------------------------------------------------------------------------------
struct DirectParams {
  int32_t n_modes;
  FastDiv div[kMaxModes];
  int64_t sa[kMaxModes], sb[kMaxModes];
  uint32_t loop_extent;
  int64_t loop_sa, loop_sb;
  uint32_t n_items;                // items excluding the looped mode (< 2^31)
  uint32_t blocked;                // 1: a workgroup owns one contiguous range of items; 0: grid-stride
};
LC_HD void direct_offsets(const DirectParams& P, uint32_t item, int64_t* so, int64_t* dof) {
  int64_t s = 0, d = 0;
  for (int k = 0; k + 1 < P.n_modes; ++k) {
    uint32_t q, r;
    fd_divmod(item, P.div[k], &q, &r);
    s += (int64_t)r * P.sa[k];
    d += (int64_t)r * P.sb[k];
    item = q;
  }
  *so = s + (int64_t)item * P.sa[P.n_modes - 1];
  *dof = d + (int64_t)item * P.sb[P.n_modes - 1];
}

// ---------------------------------------------------------------------------------------------
// Transpose kernel: the source-contiguous mode p and the destination-contiguous mode q differ.
// A tile is a box of the joint modes; it is cut into V x V micro-tiles (V elements along p times V
// along q).  A lane loads V vectors along p (one per q step), transposes them in registers, and
// parks V vectors along q in LDS; after a barrier the tile's vectors are picked up in destination
// address order, consecutive lanes taking consecutive vectors.
// Micro-tiles are enumerated in source order (index u) for the loads; vectors are enumerated in
// destination order (index g) for the stores and for their place in LDS.
// ---------------------------------------------------------------------------------------------
struct TransposeParams {
  int32_t n_micro_modes;
  // source-order decode of the micro-tile index u: extents, source stride (elements) and the
  // weight of the mode in the destination-order vector index g
  FastDiv ext_s[kMaxModes];
  int32_t sa_s[kMaxModes];
  uint32_t gpos_s[kMaxModes];
  uint32_t gpos_pv;                // weight in g of the position ip along p inside a micro-tile
  // destination-order decode of the vector index g: the micro modes plus the mode "ip" (extent V)
  int32_t n_dst_modes;
  FastDiv ext_d[kMaxModes + 1];
  int32_t sb_d[kMaxModes + 1];
  // When extents and kBlock nest (the leading modes of the source-order / destination-order decode
  // multiply up to a divisor of kBlock, and what is left of kBlock divides the next extent), the
  // index lane + i * kBlock decodes without a carry between its two terms: the lane reaches into
  // the first src_split (dst_split) modes only, and the offset is the lane's plus the trip's.  The
  // planner tabulates the trips' parts (the same for every lane), so a lane decodes once, over few
  // modes.  0 = no such nesting: every index is decoded in full.
  int32_t src_split, dst_split;
  int32_t src_trip_off[kMaxMicroPerLane];      // source offset contributed by trip i (micro-tile lane + i * kBlock)
  uint32_t src_trip_g[kMaxMicroPerLane];       // ... and its part of g
  int32_t dst_trip_off[kMaxPicksPerLane];      // destination offset contributed by trip i (vector lane + i * kBlock)
  uint32_t n_micro;                // micro-tiles per tile
  uint32_t n_vec;                  // vectors per tile = n_micro * V
  int32_t a_q;                     // source stride of one step along q (elements)
  // LDS holds the tile's vectors at slot(g) = g ^ ((g >> swz_shift) & swz_mask) ^ ((g >> swz_shift2) & swz_mask2),
  // g = destination-order index: an XOR layout over the bits of g (Sec. 2.3.2), bit b carrying f_(2^b), or
  // f_(2^b + 2^(b - shift)) when a term's mask picks it up.  An unused term has mask 0.
  uint32_t swz_shift, swz_mask, swz_shift2, swz_mask2;
  // tiles: the rest modes of zipped_divide; the tile id is their colexicographic index
  int32_t n_rest;
  FastDiv rdiv[kMaxModes];
  int64_t ra[kMaxModes], rb[kMaxModes];
  uint32_t n_tiles;
  uint32_t blocked;                // 1: a workgroup owns a contiguous range of tile ids; 0: tile ids strided by the grid
  // Ragged tiles: up to two joint modes whose extent the tile does not divide.  The grid then has
  // ceil(extent / tile) tiles along such a mode and the last of them hangs over the edge; an access
  // is made only if its coordinate along the mode is inside (the role the paper gives to coordinate
  // tensors, Sec. 2.3.2 / Fig. layouts2: a layout with strides e_i yields the coordinate to compare
  // with the shape).  Coordinates of the two modes travel packed, 16 bits each.
  int32_t n_ragged;                // 0: every tile is whole
  uint32_t rag_extent[2];          // extent of the mode (elements)
  uint32_t rag_tile[2];            // tile extent along it (elements, < 2^15)
  int32_t rag_rest[2];             // which rest mode counts the tiles along it (-1: the mode has a single tile)
  uint32_t cw_s[kMaxModes];        // coordinate step (packed) of one step of source-order micro mode k
  uint32_t cw_d[kMaxModes + 1];    // the same for the destination-order modes
};
LC_HD uint32_t lds_slot(const TransposeParams& P, uint32_t g) {
  return g ^ ((g >> P.swz_shift) & P.swz_mask) ^ ((g >> P.swz_shift2) & P.swz_mask2);
}
// A loop over modes with a run-time trip count reads its parameters with one dependent scalar load
// per trip, and every index decode costs three quarter-rate integer multiplies per mode and lane;
// a chain of those ahead of the first global load costs microseconds per launch.  Hence the lane /
// trip split below and the loops that run to a compile-time bound with the live count as a guard
// (their parameters sit at constant offsets and arrive in a few wide scalar loads).
// micro-tile u (source order) -> source offset inside the tile and the part of g the micro-tile fixes
LC_HD void micro_from_src_order(const TransposeParams& P, uint32_t u, int32_t* src_off, uint32_t* g0) {
  int32_t s = 0;
  uint32_t g = 0;
  for (int k = 0; k < P.n_micro_modes; ++k) {
    uint32_t q, r;
    fd_divmod(u, P.ext_s[k], &q, &r);
    u = q;
    s += (int32_t)r * P.sa_s[k];
    g += r * P.gpos_s[k];
  }
  *src_off = s;
  *g0 = g;
}
// the lane's digits only (P.src_split > 0): micro-tile lane + i * kBlock adds src_trip_off[i] / src_trip_g[i]
LC_HD void micro_lane_part(const TransposeParams& P, uint32_t lane, int32_t* src_off, uint32_t* g0) {
  int32_t s = 0;
  uint32_t g = 0;
#pragma unroll
  for (int k = 0; k < kMaxModes; ++k) {
    if (k < P.src_split) {
      uint32_t q, r;
      fd_divmod(lane, P.ext_s[k], &q, &r);
      lane = q;
      s += (int32_t)r * P.sa_s[k];
      g += r * P.gpos_s[k];
    }
  }
  *src_off = s;
  *g0 = g;
}
// the same with the micro-tile's packed coordinates along the ragged modes
LC_HD void micro_from_src_order_ragged(const TransposeParams& P, uint32_t u, int32_t* src_off, uint32_t* g0, uint32_t* crd) {
  int32_t s = 0;
  uint32_t g = 0, c = 0;
  for (int k = 0; k < P.n_micro_modes; ++k) {
    uint32_t q, r;
    fd_divmod(u, P.ext_s[k], &q, &r);
    u = q;
    s += (int32_t)r * P.sa_s[k];
    g += r * P.gpos_s[k];
    c += r * P.cw_s[k];
  }
  *src_off = s;
  *g0 = g;
  *crd = c;
}
LC_HD int32_t vector_dst_offset_ragged(const TransposeParams& P, uint32_t g, uint32_t* crd) {
  int32_t d = 0;
  uint32_t c = 0;
  for (int k = 0; k < P.n_dst_modes; ++k) {
    uint32_t q, r;
    fd_divmod(g, P.ext_d[k], &q, &r);
    g = q;
    d += (int32_t)r * P.sb_d[k];
    c += r * P.cw_d[k];
  }
  *crd = c;
  return d;
}
// packed coordinates inside the tile against what is left of the two ragged modes from this tile's origin on
LC_HD bool inside_ragged(uint32_t crd, uint32_t rem0, uint32_t rem1) { return (crd & 0xffffu) < rem0 && (crd >> 16) < rem1; }
// tile id -> origin offsets and the remaining extents along the ragged modes
LC_HD void tile_origin_ragged(const TransposeParams& P, uint32_t tile, int64_t* so, int64_t* dof, uint32_t* rem0, uint32_t* rem1) {
  int64_t s = 0, d = 0;
  uint32_t rem[2] = {P.n_ragged > 0 ? P.rag_extent[0] : 0x10000u, P.n_ragged > 1 ? P.rag_extent[1] : 0x10000u};
  for (int k = 0; k < P.n_rest; ++k) {
    uint32_t q, r;
    fd_divmod(tile, P.rdiv[k], &q, &r);
    s += (int64_t)r * P.ra[k];
    d += (int64_t)r * P.rb[k];
    tile = q;
    for (int j = 0; j < 2; ++j)
      if (j < P.n_ragged && P.rag_rest[j] == k) rem[j] = P.rag_extent[j] - r * P.rag_tile[j];
  }
  *so = s;
  *dof = d;
  *rem0 = rem[0];
  *rem1 = rem[1];
}
// vector g (destination order) -> destination offset inside the tile
LC_HD int32_t vector_dst_offset(const TransposeParams& P, uint32_t g) {
  int32_t d = 0;
  for (int k = 0; k < P.n_dst_modes; ++k) {
    uint32_t q, r;
    fd_divmod(g, P.ext_d[k], &q, &r);
    g = q;
    d += (int32_t)r * P.sb_d[k];
  }
  return d;
}
// the lane's digits only (P.dst_split > 0): vector lane + i * kBlock adds dst_trip_off[i]
LC_HD int32_t vector_lane_part(const TransposeParams& P, uint32_t lane) {
  int32_t d = 0;
#pragma unroll
  for (int k = 0; k < kMaxModes + 1; ++k) {
    if (k < P.dst_split) {
      uint32_t q, r;
      fd_divmod(lane, P.ext_d[k], &q, &r);
      lane = q;
      d += (int32_t)r * P.sb_d[k];
    }
  }
  return d;
}
// What the first loads of a launch need, in fourteen dwords.  They travel as the kernel's leading scalar arguments (the
// source pointer and the twelve dwords below), which the hardware can place in scalar registers when a wavefront starts
// (kernel-argument preload); a wavefront then issues the loads of its first tile before the rest of the argument block has
// arrived from memory, about half a microsecond earlier per launch.  Covers plans whose lanes own one micro-tile, whose
// lane index decodes by shifts (the lane / trip split above) over at most four modes, and whose grid of tiles has at most
// two modes; every other plan leaves `ctl` at 0 and starts through the argument block.
struct TransposeHead {
  uint32_t ctl;        // bit 0: valid; bits 1..16: four 4-bit counts, the bits of the lane index each source-order mode takes
                       // (the last mode in use takes 8: all that is left); bits 17..21: shift of the division below;
                       // bits 22..30: micro-tiles per tile (lanes at or past it load nothing)
  int32_t a_q;         // source stride of one step along q (elements)
  int32_t sa[4];       // source strides of the lane's modes (elements)
  uint32_t r0_mul, r0_div;   // the first rest mode's extent as a multiply-shift division
  int64_t ra0, ra1;    // source strides of the two rest modes (elements)
};
constexpr int kHeadMaxGrid = 8192;   // largest grid whose first tiles the planner has compared with the argument block's decode
LC_HD int32_t head_lane_offset(const TransposeHead& H, uint32_t lane) {
  int32_t s = 0;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const uint32_t bits = (H.ctl >> (1 + 4 * k)) & 15u;
    s += (int32_t)(lane & ((1u << bits) - 1u)) * H.sa[k];
    lane >>= bits;
  }
  return s;
}
LC_HD uint32_t head_n_micro(const TransposeHead& H) { return (H.ctl >> 22) & 511u; }
LC_HD int64_t head_tile_origin(const TransposeHead& H, uint32_t tile) {
  const uint32_t q = (mulhi_u32(tile, H.r0_mul) + tile) >> ((H.ctl >> 17) & 31u);
  return (int64_t)(tile - q * H.r0_div) * H.ra0 + (int64_t)q * H.ra1;
}
// tile id -> offsets of the tile's origin (slicing the rest mode: the coordinate is folded into the accessor, Sec. 2.5.1)
LC_HD void tile_origin(const TransposeParams& P, uint32_t tile, int64_t* so, int64_t* dof) {
  int64_t s = 0, d = 0;
  constexpr int kInline = 4;   // the first modes at constant offsets of the argument block, the others in a loop
#pragma unroll
  for (int k = 0; k < kInline; ++k) {
    if (k < P.n_rest) {
      uint32_t q, r;
      fd_divmod(tile, P.rdiv[k], &q, &r);
      s += (int64_t)r * P.ra[k];
      d += (int64_t)r * P.rb[k];
      tile = q;
    }
  }
  for (int k = kInline; k < P.n_rest; ++k) {
    uint32_t q, r;
    fd_divmod(tile, P.rdiv[k], &q, &r);
    s += (int64_t)r * P.ra[k];
    d += (int64_t)r * P.rb[k];
    tile = q;
  }
  *so = s;
  *dof = d;
}

}  // namespace lc
