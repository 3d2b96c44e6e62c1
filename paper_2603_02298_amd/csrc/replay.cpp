// Host replay of a plan: the same index arithmetic as the kernels (kernel_params.hpp), executed
// lane by lane on host memory, with every access checked against the buffer sizes.  A checking
// device for plans; never part of executing a copy.
#include <algorithm>
#include <cstring>
#include <vector>

#include "plan.hpp"

namespace lc {


namespace {
struct Buffers {
  const unsigned char* src;   // the plan's effective source / destination pointers (offsets folded in)
  unsigned char* dst;
  int64_t src_lo, src_hi, dst_lo, dst_hi;   // byte offsets around them that belong to the buffers
  bool ok = true;
  void move(int64_t so, int64_t dof, int bytes) {
    if (so < src_lo || dof < dst_lo || so + bytes > src_hi || dof + bytes > dst_hi) { ok = false; return; }
    std::memcpy(dst + dof, src + so, (size_t)bytes);
  }
};
}  // namespace

lc_status_t replay_on_host(const lc_plan& plan, const void* src, int64_t src_lo, int64_t src_hi, void* dst, int64_t dst_lo,
                           int64_t dst_hi, int64_t* lds_conflicts) {
  const int es = plan.cls == KernelClass::Transpose ? plan.tile_elem_bytes : plan.elem_bytes;
  const int eb = plan.elem_bytes;
  if (plan.src_offset_elems < src_lo || plan.src_offset_elems >= src_hi || plan.dst_offset_elems < dst_lo || plan.dst_offset_elems >= dst_hi)
    return LC_ERR_INVALID_ARG;
  Buffers B{static_cast<const unsigned char*>(src) + plan.src_offset_elems * eb, static_cast<unsigned char*>(dst) + plan.dst_offset_elems * eb,
            (src_lo - plan.src_offset_elems) * eb, (src_hi - plan.src_offset_elems) * eb,
            (dst_lo - plan.dst_offset_elems) * eb, (dst_hi - plan.dst_offset_elems) * eb};
  if (lds_conflicts) *lds_conflicts = 0;
  if (plan.cls == KernelClass::Generic) {
    const GenericParams& P = plan.generic;
    for (uint32_t i = 0; i < P.n; ++i) B.move(flat_eval(P.src, i) * es, flat_eval(P.dst, i) * es, es);
  } else if (plan.cls == KernelClass::LastWriter) {
    // the two passes of the device path, both walked BACKWARDS here: the result may not depend on the order
    const GenericParams& P = plan.generic;
    std::vector<uint32_t> winner((size_t)(plan.workspace_bytes / 4), 0u);
    for (uint32_t i = P.n; i-- > 0;) {
      const int64_t off = flat_eval(P.dst, i), word = off + plan.workspace_bias;
      if (word < 0 || word >= (int64_t)winner.size()) { B.ok = false; break; }
      if (winner[(size_t)word] < i) winner[(size_t)word] = i;
    }
    for (uint32_t i = P.n; B.ok && i-- > 0;) {
      const int64_t off = flat_eval(P.dst, i);
      if (winner[(size_t)(off + plan.workspace_bias)] == i) B.move(flat_eval(P.src, i) * es, off * es, es);
    }
  } else if (plan.cls == KernelClass::Direct) {
    const DirectParams& P = plan.direct;
    const int W = plan.width_bytes;
    if (plan.gather_stride > 0) {
      // gather_kernel: vector `item` of the destination keeps every S-th element of S consecutive source words; all but the
      // last vector along mode 0 load those words whole
      const int S = plan.gather_stride, VE = 16 / eb;
      const uint32_t ext0 = P.n_modes > 1 ? P.div[0].div : P.n_items;
      if (W != 16) return LC_ERR_INVALID_ARG;
      for (int64_t j = 0; j < plan.n_launches; ++j)
        for (uint32_t item = 0; item < P.n_items; ++item) {
          int64_t so, dof;
          direct_offsets(P, item, &so, &dof);
          const int64_t sbyte = so * 16 + j * plan.launch_src_step * eb, dbyte = dof * 16 + j * plan.launch_dst_step * eb;
          const uint32_t o = P.n_modes > 1 ? item % ext0 : item;
          if (o != ext0 - 1u && (sbyte < B.src_lo || sbyte + (int64_t)S * 16 > B.src_hi)) B.ok = false;
          for (int e = 0; e < VE; ++e) B.move(sbyte + (int64_t)e * S * eb, dbyte + (int64_t)e * eb, eb);
        }
    } else
    for (int64_t j = 0; j < plan.n_launches; ++j)
      for (uint32_t item = 0; item < P.n_items; ++item) {
        int64_t so, dof;
        direct_offsets(P, item, &so, &dof);
        for (uint32_t r = 0; r < P.loop_extent; ++r)
          B.move((so + r * P.loop_sa) * W + j * plan.launch_src_step * es, (dof + r * P.loop_sb) * W + j * plan.launch_dst_step * es, W);
      }
  } else {
    const TransposeParams& P = plan.transpose;
    const int V = plan.V, slot = V * es;
    std::vector<unsigned char> lds((size_t)plan.lds_bytes);
    const uint32_t lanes = (uint32_t)kBlock * (uint32_t)plan.micro_per_thread;
    if (plan.head.ctl & 1u) {
      // the first loads of a workgroup are addressed from the head alone: it has to agree with the argument block for every
      // lane and for every tile id a workgroup can start on
      if (plan.micro_per_thread != 1 || head_n_micro(plan.head) != P.n_micro || plan.head.a_q != P.a_q || P.src_split < 1) return LC_ERR_INVALID_ARG;
      for (uint32_t lane = 0; lane < P.n_micro; ++lane) {
        int32_t so;
        uint32_t g0;
        micro_lane_part(P, lane, &so, &g0);
        if (head_lane_offset(plan.head, lane) != so + P.src_trip_off[0]) return LC_ERR_INVALID_ARG;
      }
      for (uint32_t tile = 0; tile < std::min<uint32_t>(P.n_tiles, (uint32_t)kHeadMaxGrid); ++tile) {
        int64_t so, dof;
        tile_origin(P, tile, &so, &dof);
        if (head_tile_origin(plan.head, tile) != so) return LC_ERR_INVALID_ARG;
      }
    }
    for (uint32_t tile = 0; tile < P.n_tiles && B.ok; ++tile) {
      int64_t sbase, dbase;
      uint32_t rem0 = 0x10000u, rem1 = 0x10000u;
      if (P.n_ragged > 0) tile_origin_ragged(P, tile, &sbase, &dbase, &rem0, &rem1);
      else tile_origin(P, tile, &sbase, &dbase);
      // load phase: lane u reads V vectors along p (one per step along q), parks V vectors along q
      for (uint32_t u = 0; u < lanes; ++u) {
        if (u >= P.n_micro) continue;
        int32_t so;
        uint32_t g0;
        // the same choice of decode as the kernel's lanes make
        if (P.n_ragged > 0) {
          uint32_t crd;
          micro_from_src_order_ragged(P, u, &so, &g0, &crd);
          if (!inside_ragged(crd, rem0, rem1)) continue;
        } else if (P.src_split > 0) {
          micro_lane_part(P, u % (uint32_t)kBlock, &so, &g0);
          so += P.src_trip_off[u / (uint32_t)kBlock];
          g0 += P.src_trip_g[u / (uint32_t)kBlock];
        } else {
          micro_from_src_order(P, u, &so, &g0);
        }
        for (int iq = 0; iq < V; ++iq) {
          int64_t off = (sbase + so + (int64_t)iq * P.a_q) * es;
          if (off < B.src_lo || off + slot > B.src_hi) { B.ok = false; break; }
          for (int ip = 0; ip < V; ++ip) {
            size_t l = (size_t)lds_slot(P, g0 + (uint32_t)ip * P.gpos_pv) * (size_t)slot + (size_t)iq * (size_t)es;
            if (l + (size_t)es > lds.size()) { B.ok = false; break; }
            std::memcpy(&lds[l], B.src + off + (int64_t)ip * es, (size_t)es);
          }
        }
      }
      // store phase: the tile's vectors in destination order, consecutive lanes taking consecutive vectors
      for (uint32_t g = 0; g < lanes * (uint32_t)V && B.ok; ++g) {
        if (g >= P.n_vec) continue;
        int32_t din;
        if (P.n_ragged > 0) {
          uint32_t crd;
          din = vector_dst_offset_ragged(P, g, &crd);
          if (!inside_ragged(crd, rem0, rem1)) continue;
        } else {
          din = P.dst_split > 0 ? vector_lane_part(P, g % (uint32_t)kBlock) + P.dst_trip_off[g / (uint32_t)kBlock] : vector_dst_offset(P, g);
        }
        int64_t off = (dbase + din) * es;
        size_t l = (size_t)lds_slot(P, g) * (size_t)slot;
        if (off < B.dst_lo || off + slot > B.dst_hi || l + (size_t)slot > lds.size()) { B.ok = false; break; }
        std::memcpy(B.dst + off, &lds[l], (size_t)slot);
      }
      if (lds_conflicts && tile == 0) {
        for (uint32_t wave = 0; wave * 64 < lanes; ++wave) {
          uint32_t g0[64];
          bool act[64];
          for (int l = 0; l < 64; ++l) {
            uint32_t u = wave * 64 + (uint32_t)l;
            act[l] = u < P.n_micro;
            int32_t so;
            g0[l] = 0;
            if (act[l]) micro_from_src_order(P, u, &so, &g0[l]);
          }
          for (int ip = 0; ip < V; ++ip) {
            uint32_t wa[64];
            for (int l = 0; l < 64; ++l) wa[l] = lds_slot(P, g0[l] + (uint32_t)ip * P.gpos_pv) * (uint32_t)slot;
            *lds_conflicts += lds_pass_conflicts(wa, act, 64, slot, true);
          }
        }
        for (uint32_t wave = 0; wave * 64 < lanes * (uint32_t)V; ++wave) {
          uint32_t ra[64];
          bool act[64];
          for (int l = 0; l < 64; ++l) {
            uint32_t g = wave * 64 + (uint32_t)l;
            act[l] = g < P.n_vec;
            ra[l] = lds_slot(P, g) * (uint32_t)slot;
          }
          *lds_conflicts += lds_pass_conflicts(ra, act, 64, slot, false);
        }
      }
    }
  }
  return B.ok ? LC_OK : LC_ERR_INVALID_ARG;
}

}  // namespace lc
