// Host-side layout representation of the library: a shape/stride tree stored as a pre-order
// profile plus the list of its leaf modes (extent, stride).  The algebra works on the flat mode
// list and re-nests results with profiles.
// Follows "CuTe Layout Representation and Algebra": HTuple (Sec. 2.1), Shape (Sec. 2.2),
// Stride (Sec. 2.3), Layout (Sec. 2.4).
#pragma once
#include <cstdint>
#include <string>
#include <vector>

#include "layoutcopy.h"

namespace lc {

struct Mode {
  int64_t extent;
  int64_t stride;
};
using Modes = std::vector<Mode>;

// Pre-order profile entry: 0 = leaf, k >= 1 = tuple with k children.
struct Layout {
  std::vector<int32_t> profile;
  Modes leaves;

  static Layout leaf(int64_t extent, int64_t stride) { return Layout{{0}, {{extent, stride}}}; }
  // flat layout: one mode -> "s:d", several -> "(s0,s1,..):(d0,d1,..)"
  static Layout flat(const Modes& m);
  // (parts_0, parts_1, ...): concatenation (Eq. concat)
  static Layout tuple(const std::vector<Layout>& parts);

  bool is_leaf() const { return profile.size() == 1 && profile[0] == 0; }
  int rank() const { return profile[0] == 0 ? 1 : profile[0]; }
  int depth() const;
  int64_t size() const;
  int64_t cosize() const;                   // largest offset + 1
  int64_t min_offset() const;               // smallest offset: 0 unless a stride is negative
  bool has_negative_stride() const;
  Layout mode(int i) const;                 // L_i = S_i : D_i (a leaf is its own mode 0)
  std::string str() const;
  int64_t operator()(int64_t i) const;      // integral coordinate, extended domain
};

lc_status_t parse(const char* text, Layout* out);
lc_status_t validate(const Layout& L);

}  // namespace lc

struct lc_layout {
  lc::Layout L;
};
