// Host planner for COPY (Sec. 2.6.1 of "CuTe Layout Representation and Algebra"): turns a pair of
// layouts into kernel arguments using the layout algebra (Sec. 3).
#pragma once
#include <string>
#include <vector>

#include "algebra.hpp"
#include "kernel_params.hpp"

namespace lc {

struct JointMode {
  int64_t extent, a, b;   // extent, source stride, destination stride (elements)
};

enum class KernelClass { Generic, Direct, Transpose, LastWriter };

// Knobs the planner normally chooses itself; values < 0 mean "planner's choice".  Read from the
// environment (LC_TUNE_*) once per plan so that tile shapes can be swept without rebuilding.
struct Tuning {
  int micro_per_thread = -1;   // transpose: micro-tiles per lane (1, 2, 4; 8 with V = 1)
  int rest_order = -1;         // transpose: 0 = tiles ordered by destination stride, 1 = by source stride (default)
  int wgs_per_cu = -1;         // persistent grid size = CUs * wgs_per_cu
  int unroll = -1;             // direct: items per lane per loop trip (1, 2, 4, 8)
  int swizzle_shift = -2;      // transpose: -1 = no swizzle
  int nontemporal = -1;        // bit 0 = nontemporal loads, bit 1 = nontemporal stores
  int blocked = -1;            // 1 = contiguous range of tiles / items per workgroup, 0 = strided by the grid
  int64_t max_items = -1;      // direct: work items per launch before the copy is sliced (default 2^31 - 1; lowered in tests)
  std::vector<int64_t> tile;   // transpose: tile extents per joint mode (overrides the planner's choice)
  int force_class = -1;        // 0 generic, 1 direct, 2 transpose (falls back when not applicable)
  int max_vec_bytes = -1;      // cap on the access width
  int tile_queue = -1;         // transpose: n > 0 = hand tiles out through a device-side queue, n per request; 0 = in a fixed order
  int queue_rounds = -1;       // transpose: whole rounds of the grid handed out by index before the queue takes over (>= 1)
  int queue_counters = -1;     // transpose: counters the requests are spread over (1..15)
  int grid = -1;               // workgroups of the launch (overrides CUs * wgs_per_cu)
  int leftover_lead = -1;      // transpose, fixed order: the tiles left after the last whole round go to this many leading workgroups
  int direct_queue = -1;       // direct: KiB of destination per chunk handed out on request; 0 = grid-stride order
  int gather = -1;             // direct: 1 = a small source stride along the destination-contiguous mode is read in whole 16-byte words (gather_kernel)
  int early_loads = -1;        // transpose: 0 = the first loads wait for the whole argument block (no TransposeHead)
};
Tuning tuning_from_env();

}  // namespace lc

struct lc_plan {
  lc::KernelClass cls = lc::KernelClass::Generic;
  int elem_bytes = 0;
  int64_t n_elems = 0;
  int64_t distinct_reads = 0;              // source elements read when modes of stride 0 (re-reads of one element) count once
  // Destination modes of stride 0: the sequential loop's last write wins, so the copy is the slice at those modes'
  // last coordinates: the source is read from src + src_offset_elems, the modes are gone from the plan.
  int64_t src_offset_elems = 0;
  int overwritten_modes = 0;
  // Joint modes of negative destination stride are walked backwards (the same order on both sides, Sec. 3.4.2): their
  // last elements become the origins, folded into both pointers.
  int64_t dst_offset_elems = 0;
  int reflected_modes = 0;
  int64_t common_vector = 1;               // K of Sec. 3.4.2 before hardware clamps
  std::vector<lc::JointMode> joint;        // after common refinement, destination-order sort, joint coalesce
  unsigned src_align = 0, dst_align = 0;   // alignment the access widths rely on

  // Direct
  int width_bytes = 0;                     // bytes per access (element width x vector length)
  lc::DirectParams direct{};
  int unroll = 4;
  int direct_queue_items = 0;              // > 0: items per chunk; wavefronts take chunks on request (long copies)
  int gather_stride = 0;                   // > 0: the destination-contiguous mode is read with this stride; 16-byte words on both sides (gather_kernel)
  int64_t n_launches = 1;                  // slices along the outermost mode, one launch each
  int64_t launch_src_step = 0, launch_dst_step = 0;   // elements between consecutive slices

  // Transpose
  int tile_elem_bytes = 0;                 // width of what the tiled kernel treats as an element: elem_bytes, or 16 when whole
                                           // 16-byte words keep together on both sides and are only re-ordered (V = 1)
  int V = 0;                               // micro-tile edge (elements of tile_elem_bytes)
  int micro_per_thread = 1;
  std::vector<int64_t> tile_extent;        // per joint mode
  int p_mode = -1, q_mode = -1;
  lc::TransposeParams transpose{};
  lc::TransposeHead head{};                // what the first loads need, for the kernel's leading arguments (ctl = 0: not in use)
  unsigned lds_bytes = 0;
  bool swizzle_derived = false;            // the LDS slot layout came out of the park layout's bits (else: searched against the bank model)
  int64_t src_run_bytes = 0, dst_run_bytes = 0;

  // Generic and LastWriter (both evaluate the two coalesced layouts per element)
  lc::GenericParams generic{};
  // LastWriter: the destination maps several coordinates to one offset (or could not be shown not to).  Sec. 2.6.1's loop
  // leaves the value of the LARGEST integral coordinate that reaches an offset.  A first pass records that coordinate per
  // offset in scratch memory (one 32-bit word per element of the destination's span), a second pass lets only the recorded
  // coordinates write: the result does not depend on the order in which lanes run.
  int64_t workspace_bytes = 0;
  int64_t workspace_bias = 0;              // the record of destination offset o is word o + workspace_bias (negative strides reach below 0)

  int wgs_per_cu = 0;
  int grid_override = 0;                   // > 0: workgroups of the launch, whatever the CU count
  int tile_queue = 0;                      // transposing class: tiles past the first rounds of the grid are handed out on request, this many at a time
  int queue_static_rounds = 1;             // ... whole rounds of the grid that go by workgroup index first
  int queue_counters = 1;                  // ... counters (one cache line each) the requests are spread over
  int leftover_lead = 0;                   // fixed order: leading workgroups that share the tiles left after the last whole round (0: all)
  int nontemporal = 0;                     // bit 0: loads, bit 1: stores
  bool early_loads = true;                 // kernels may start from their leading scalar arguments alone (tuning can switch it off)
  std::string note;                        // why a faster class was not taken
};

namespace lc {

lc_status_t make_plan(const Layout& src, const Layout& dst, int elem_bytes, unsigned src_align,
                      unsigned dst_align, const Tuning& tune, lc_plan* out);
std::string describe(const lc_plan& plan);
// Do distinct coordinates of the (coalesced) layout of size n reach distinct offsets?  Nested strides prove it,
// small layouts are enumerated, large ones that cannot be proved cheaply count as aliasing.
bool layout_is_injective(const Modes& coalesced, int64_t n);

// Walks the plan on the host exactly along the kernels' index arithmetic and moves the bytes in
// host memory.  It exists to prove the routing of a plan (and that every access stays inside the
// two buffers) without a GPU; it is not a way to execute a copy and nothing in the copy path calls it.
// src / dst point at offset 0 of the layouts; [src_lo, src_hi) and [dst_lo, dst_hi) are the element offsets around them
// that belong to the buffers (lo <= 0 < hi).
lc_status_t replay_on_host(const lc_plan& plan, const void* src, int64_t src_lo, int64_t src_hi, void* dst, int64_t dst_lo,
                           int64_t dst_hi, int64_t* lds_conflicts);

// The LDS bank model (plan.cpp): extra cycles of one wavefront instruction whose active lane l accesses access_bytes at byte_addr[l].
int lds_pass_conflicts(const uint32_t* byte_addr, const bool* active, int lanes, int access_bytes, bool is_write);

// Defined with the kernels: enqueue the plan's kernel on a HIP stream / time repeated executions.
const char* last_hip_error();
void set_last_hip_error(const std::string& text);
lc_status_t execute_plan(const lc_plan& plan, const void* src, void* dst, void* stream);
// the same with scratch device memory for the plans that need it (workspace_bytes > 0); others ignore it
// the same with the library's static scratch array of the current device; allocates nothing
size_t static_scratch_bytes();
lc_status_t execute_plan_static(const lc_plan& plan, const void* src, void* dst, void* stream);
lc_status_t execute_plan_workspace(const lc_plan& plan, const void* src, void* dst, void* workspace, size_t workspace_bytes, void* stream);
lc_status_t time_plan(const lc_plan& plan, const void* const* srcs, void* const* dsts, int n_buffers, int warmup,
                      int iters, void* stream, float* ms_per_iter);
lc_status_t time_plan_each(const lc_plan& plan, const void* const* srcs, void* const* dsts, int n_buffers, int warmup,
                           int iters, void* stream, float* ms_each);

}  // namespace lc
