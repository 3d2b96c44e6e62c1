// Host planner of the generic GEMM (Sec. 2.6.2 of "CuTe Layout Representation and Algebra").
#pragma once
#include <string>

#include "algebra.hpp"
#include "gemm_params.hpp"

struct lc_gemm_plan {
  int ab_dtype = 0;                  // LC_BF16 or LC_F16 (A and B); C is fp32
  int64_t M = 0, N = 0, K = 0, L = 1; // of the caller's problem (L: batch entries of the rank-3 form)
  bool exchanged = false;            // the kernel computes C^T = B A^T: roles of A and B exchanged, C's modes exchanged
  int tile_m = 0, tile_n = 0;        // workgroup tile (kernel's m x n)
  lc::GemmParams params{};
  unsigned a_align = 2, b_align = 2, c_align = 4;   // pointer alignment the chosen access widths rely on (caller's A, B, C)
  unsigned lds_bytes = 0;
  int64_t a_cosize = 0, b_cosize = 0, c_cosize = 0; // elements addressable behind the caller's A, B, C
  std::string a_text, b_text, c_text;               // the three layouts coalesced by mode, as the kernel sees them
};

namespace lc {

// ab_dtype: LC_BF16 / LC_F16.  *_align: alignment in bytes the caller guarantees for the three pointers.
lc_status_t make_gemm_plan(const Layout& A, const Layout& B, const Layout& C, int ab_dtype, unsigned a_align, unsigned b_align,
                           unsigned c_align, lc_gemm_plan* out);
std::string describe(const lc_gemm_plan& plan);

// Thread-value layouts of the v_mfma_f32_32x32x16 fragments (which: 0 = A, 1 = B, 2 = C), (lane, value) ->
// integral coordinate of the fragment's (32,16) / (32,32) tile (Sec. 3.3.4).
lc_status_t mfma_fragment_layout(int which, Layout* out);

// Walks the plan on the host along the kernel's index arithmetic with HOST buffers: every global access is
// bounds- and alignment-checked, tiles pass through a model of the LDS arrangement and of the MFMA fragment
// layouts.  A checking device for tests (no GPU needed); nothing that executes a GEMM calls it.
// a / b hold 16-bit patterns (bf16 or f16 as the plan says), c holds fp32 and is updated in place.
lc_status_t gemm_replay_on_host(const lc_gemm_plan& plan, const uint16_t* a, int64_t a_elems, const uint16_t* b, int64_t b_elems,
                                float* c, int64_t c_elems);

// Defined with the kernel.
lc_status_t execute_gemm_plan(const lc_gemm_plan& plan, const void* a, const void* b, void* c, void* stream);
lc_status_t time_gemm_plan(const lc_gemm_plan& plan, const void* a, const void* b, void* c, int warmup, int iters, void* stream,
                           float* ms_per_iter);

}  // namespace lc
