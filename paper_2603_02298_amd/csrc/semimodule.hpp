// Layouts with strides from an integer-semimodule other than Z (Sec. 2.3.2 of "CuTe Layout
// Representation and Algebra"): scaled basis elements a*e_i, which make the layout yield a
// coordinate (Fig. layouts2, Table TVLayoutExamples row Coordinate), and XOR elements f_d
// (row Swizzled).  Host side only; the copy kernels use the coordinate idea for ragged tiles.
#pragma once
#include <cstdint>
#include <string>
#include <vector>

#include "layout.hpp"

namespace lc {

struct SemiStride {
  enum Kind : int32_t { Int = 0, Coord = 1, Xor = 2 };
  Kind kind = Int;
  int64_t a = 0;      // the integer, the coefficient of e_axis, or d of f_d
  int32_t axis = 0;   // Coord only
};

struct SemiLayout {
  std::vector<int32_t> profile;       // pre-order, as in Layout
  std::vector<int64_t> extent;        // per leaf
  std::vector<SemiStride> stride;     // per leaf
  SemiStride::Kind kind() const;      // Int when no stride is of another kind
  int codomain_rank() const;          // Coord: 1 + largest axis; otherwise 1
  int64_t size() const;
  std::string str() const;
  void eval(int64_t i, int64_t* out) const;   // writes codomain_rank() values (extended domain)
};

lc_status_t parse(const char* text, SemiLayout* out);
lc_status_t composition(const SemiLayout& a, const Layout& b, SemiLayout* out);   // Sec. 3.3, "Reductive case: Coordinate"
SemiLayout coalesce(const SemiLayout& a);                                        // Sec. 3.2 in the semimodule
lc_status_t right_inverse(const SemiLayout& a, Layout* out);                      // Table rinv, rows with e_i strides
// Table rinv, last row: a layout with XOR strides whose function is additive over XOR of integral coordinates (extents
// powers of two, no carry among a stride's multiples inside its mode) is a matrix over F2 from the coordinate's bits to the
// offset's bits.  R = (2,...,2):(f_x0, f_x1, ...) with x_b the smallest integral coordinate that A sends to 2^b, for
// b = 0, 1, ... up to the first power of two outside A's image; A(R(k)) = k for every k < |R|.  By elimination over F2;
// layouts that are not additive are refused (LC_ERR_INVALID_ARG).
lc_status_t xor_right_inverse(const SemiLayout& a, SemiLayout* out);

}  // namespace lc

struct lc_slayout {
  lc::SemiLayout L;
};
