#include "semimodule.hpp"

#include <algorithm>

#include "algebra.hpp"

namespace lc {

namespace {
struct Reader {
  const char* p;
  bool fail = false;
  void ws() { while (*p == ' ' || *p == '\t') ++p; }
  bool digits(int64_t* v) {
    int n = 0;
    int64_t x = 0;
    while (*p >= '0' && *p <= '9') { x = x * 10 + (*p - '0'); ++p; if (++n > 18) return false; }
    *v = x;
    return n > 0;
  }
  // a tree of leaves; `leaf` reads one leaf at the cursor and appends it to its own list
  template <typename LeafFn>
  void tree(std::vector<int32_t>* profile, LeafFn leaf) {
    ws();
    if (*p != '(') { profile->push_back(0); leaf(); return; }
    ++p;
    const size_t at = profile->size();
    profile->push_back(0);
    int32_t n = 0;
    for (;;) {
      tree(profile, leaf);
      if (fail) return;
      ++n;
      ws();
      if (*p == ',') { ++p; continue; }
      if (*p == ')') { ++p; break; }
      fail = true;
      return;
    }
    (*profile)[at] = n;
  }
};

std::string stride_str(const SemiStride& s) {
  if (s.kind == SemiStride::Xor) return "f" + std::to_string(s.a);
  if (s.kind == SemiStride::Coord) return (s.a == 1 ? "" : std::to_string(s.a)) + "e" + std::to_string(s.axis);
  return std::to_string(s.a);
}

template <typename Print>
std::string print_tree(const std::vector<int32_t>& profile, size_t* node, size_t* leaf, Print print) {
  const int32_t k = profile[(*node)++];
  if (k == 0) return print((*leaf)++);
  std::string r = "(";
  for (int32_t c = 0; c < k; ++c) {
    if (c) r += ",";
    r += print_tree(profile, node, leaf, print);
  }
  return r + ")";
}
}  // namespace

SemiStride::Kind SemiLayout::kind() const {
  for (const SemiStride& s : stride)
    if (s.a != 0 && s.kind != SemiStride::Int) return s.kind;
  return SemiStride::Int;
}
int SemiLayout::codomain_rank() const {
  int r = 1;
  for (const SemiStride& s : stride)
    if (s.kind == SemiStride::Coord && s.a != 0) r = std::max(r, s.axis + 1);
  return r;
}
int64_t SemiLayout::size() const {
  int64_t n = 1;
  for (int64_t e : extent) n *= e;
  return n;
}
std::string SemiLayout::str() const {
  size_t node = 0, leaf = 0;
  std::string s = print_tree(profile, &node, &leaf, [&](size_t k) { return std::to_string(extent[k]); });
  node = leaf = 0;
  return s + ":" + print_tree(profile, &node, &leaf, [&](size_t k) { return stride_str(stride[k]); });
}

// The leaves in left-to-right order are the digits of the integral coordinate, least significant
// first (Sec. 2.2.2); the last one is not reduced (extended domain, Sec. 2.4.1).
void SemiLayout::eval(int64_t i, int64_t* out) const {
  const SemiStride::Kind k = kind();
  const int r = k == SemiStride::Coord ? codomain_rank() : 1;
  for (int j = 0; j < r; ++j) out[j] = 0;
  for (size_t m = 0; m < extent.size(); ++m) {
    const bool last = m + 1 == extent.size();
    const int64_t digit = last ? i : i % extent[m];
    i = last ? 0 : i / extent[m];
    const SemiStride& s = stride[m];
    if (s.a == 0) continue;
    if (k == SemiStride::Coord) out[s.axis] += digit * s.a;
    else if (k == SemiStride::Xor) out[0] ^= digit * s.a;
    else out[0] += digit * s.a;
  }
}

lc_status_t parse(const char* text, SemiLayout* out) {
  SemiLayout L;
  Reader rd{text};
  rd.tree(&L.profile, [&]() {
    int64_t v;
    if (!rd.digits(&v)) rd.fail = true;
    L.extent.push_back(v);
  });
  rd.ws();
  if (rd.fail || *rd.p != ':') return LC_ERR_PARSE;
  ++rd.p;
  std::vector<int32_t> dprofile;
  rd.tree(&dprofile, [&]() {
    SemiStride s;
    if (*rd.p == 'f') {
      ++rd.p;
      s.kind = SemiStride::Xor;
      if (!rd.digits(&s.a)) rd.fail = true;
    } else {
      int64_t v = 1;
      const bool number = *rd.p >= '0' && *rd.p <= '9';
      if (number && !rd.digits(&v)) rd.fail = true;
      if (*rd.p == 'e') {
        ++rd.p;
        int64_t ax;
        if (!rd.digits(&ax) || ax > 15) rd.fail = true;
        s.kind = SemiStride::Coord;
        s.a = v;
        s.axis = (int32_t)ax;
      } else if (number) {
        s.a = v;
      } else {
        rd.fail = true;
      }
    }
    L.stride.push_back(s);
  });
  rd.ws();
  if (rd.fail || *rd.p != 0) return LC_ERR_PARSE;
  if (dprofile != L.profile) return LC_ERR_NOT_CONGRUENT;
  if (L.extent.size() > 64) return LC_ERR_INVALID_ARG;
  int64_t total = 1;
  for (int64_t e : L.extent) {
    if (e < 1) return LC_ERR_BAD_EXTENT;
    if (total > (int64_t)4e18 / e) return LC_ERR_INVALID_ARG;
    total *= e;
  }
  const SemiStride::Kind k = L.kind();
  for (const SemiStride& s : L.stride)
    if (s.a != 0 && s.kind != k) return LC_ERR_INVALID_ARG;   // one semimodule per layout
  *out = L;
  return LC_OK;
}

// A o B: B only addresses the integral coordinate of A's shape, so admissibility and the shape of
// the result are those of P o B for an integer layout P over A's shape.  P's strides are place
// values with a factor-2 gap after each leaf: a compact P would let composition merge modes across
// leaves, which semimodule strides do not allow.  A result mode with stride step * P_k walks leaf k
// and carries step * d_k.
lc_status_t composition(const SemiLayout& a, const Layout& b, SemiLayout* out) {
  Layout proxy;
  proxy.profile = a.profile;
  std::vector<int64_t> lo;             // proxy stride of each leaf
  int64_t place = 1;
  for (int64_t e : a.extent) {
    proxy.leaves.push_back({e, place});
    lo.push_back(place);
    if (place > (int64_t)2e18 / (2 * e)) return LC_ERR_INVALID_ARG;
    place *= 2 * e;
  }
  Layout pb;
  lc_status_t st = composition(proxy, b, &pb);
  if (st != LC_OK) return st;
  SemiLayout r;
  r.profile = pb.profile;
  // XOR strides: the bits that the modes walking leaf k can set so far.  A mode contributes c * (step * d_k) for c below its
  // extent; inside one leaf those contributions are added as integers before A scales them, and that equals their XOR
  // exactly when no two modes can set the same bit.  Otherwise no layout with XOR strides is A o B: refused.
  const bool is_xor = a.kind() == SemiStride::Xor;
  std::vector<uint64_t> bits_of_leaf(a.extent.size(), 0);
  for (const Mode& m : pb.leaves) {
    r.extent.push_back(m.extent);
    SemiStride s;
    if (m.stride != 0 && m.extent > 1) {
      size_t k = 0;
      while (k + 1 < lo.size() && m.stride >= lo[k + 1]) ++k;
      if (m.stride % lo[k] != 0) return LC_ERR_STRIDE_DIVISIBILITY;
      s = a.stride[k];
      s.a *= m.stride / lo[k];
      if (s.a == 0) s = SemiStride{};
      if (is_xor && s.a != 0) {
        if (s.a < 0 || m.extent > (int64_t(1) << 24) || (long double)s.a * (long double)(m.extent - 1) > 4.0e18L) return LC_ERR_TOO_LARGE;
        uint64_t mine = 0;
        for (int64_t c = 1; c < m.extent; ++c) mine |= (uint64_t)c * (uint64_t)s.a;
        if (mine & bits_of_leaf[k]) return LC_ERR_NOT_SEGREGATED;
        bits_of_leaf[k] |= mine;
      }
    }
    r.stride.push_back(s);
  }
  *out = r;
  return LC_OK;
}

SemiLayout coalesce(const SemiLayout& a) {
  const SemiStride::Kind kind = a.kind();
  SemiLayout r;
  for (size_t k = 0; k < a.extent.size(); ++k) {
    if (a.extent[k] == 1) continue;
    const SemiStride& s = a.stride[k];
    if (!r.extent.empty() && kind != SemiStride::Xor) {
      // XOR strides never merge: (i0 + s i1) d and (i0 d) xor (i1 s d) differ once bits meet
      const SemiStride& t = r.stride.back();
      const bool both_zero = s.a == 0 && t.a == 0;
      const bool continues = s.a != 0 && t.a != 0 && s.a == t.a * r.extent.back() && (kind != SemiStride::Coord || s.axis == t.axis);
      if (both_zero || continues) { r.extent.back() *= a.extent[k]; continue; }
    }
    r.extent.push_back(a.extent[k]);
    r.stride.push_back(s);
  }
  if (r.extent.empty()) { r.extent.push_back(1); r.stride.push_back(SemiStride{}); }
  if (r.extent.size() == 1) r.profile = {0};
  else { r.profile.assign(r.extent.size() + 1, 0); r.profile[0] = (int32_t)r.extent.size(); }
  return r;
}

lc_status_t right_inverse(const SemiLayout& a, Layout* out) {
  if (a.kind() != SemiStride::Coord) return LC_ERR_INVALID_ARG;
  std::vector<int64_t> lo;
  int64_t place = 1;
  for (int64_t e : a.extent) { lo.push_back(place); place *= e; }
  std::vector<Layout> axes;
  for (int axis = 0; axis < a.codomain_rank(); ++axis) {
    // the leaves of this axis by growing coefficient; each must start where the ones before end
    std::vector<std::pair<int64_t, size_t>> order;
    for (size_t k = 0; k < a.extent.size(); ++k)
      if (a.stride[k].kind == SemiStride::Coord && a.stride[k].a != 0 && a.stride[k].axis == axis && a.extent[k] > 1)
        order.push_back({a.stride[k].a, k});
    std::sort(order.begin(), order.end());
    Modes m;
    int64_t next = 1;
    for (const auto& [coef, k] : order) {
      if (coef != next) break;
      m.push_back({a.extent[k], lo[k]});
      next *= a.extent[k];
    }
    if (m.empty()) m.push_back({1, 0});
    axes.push_back(coalesce(Layout::flat(m)));
  }
  *out = axes.size() == 1 ? axes[0] : Layout::tuple(axes);
  return LC_OK;
}

lc_status_t xor_right_inverse(const SemiLayout& a, SemiLayout* out) {
  if (a.kind() != SemiStride::Xor) return LC_ERR_INVALID_ARG;
  // column t of the matrix: what bit t of the integral coordinate adds (by XOR) to the offset
  std::vector<uint64_t> col;
  for (size_t k = 0; k < a.extent.size(); ++k) {
    const int64_t e = a.extent[k];
    if (e < 1 || (e & (e - 1)) != 0) return LC_ERR_INVALID_ARG;
    int bits = 0;
    while ((int64_t(1) << bits) < e) ++bits;
    const uint64_t d = (uint64_t)a.stride[k].a;
    if (a.stride[k].a < 0 || (bits > 0 && d >= (uint64_t(1) << (62 - bits)))) return LC_ERR_INVALID_ARG;
    // c * d for c < 2^bits equals the XOR of d << u over the bits u of c exactly when those shifted copies share no bit
    uint64_t seen = 0;
    for (int u = 0; u < bits; ++u) {
      if (seen & (d << u)) return LC_ERR_INVALID_ARG;
      seen |= d << u;
      col.push_back(d << u);
    }
  }
  const int n = (int)col.size();
  if (n > 62) return LC_ERR_INVALID_ARG;
  // elimination: a basis of the image, each vector with the coordinate that produces it, and the coordinates that produce 0
  struct Row { uint64_t image, coord; };
  std::vector<Row> basis;          // distinct leading bits of `image`
  std::vector<uint64_t> kernel;    // coordinates A sends to 0, reduced to distinct leading bits below
  auto reduce = [&](Row r) {
    for (const Row& b : basis) {
      const uint64_t lead = uint64_t(1) << (63 - __builtin_clzll(b.image));
      if (r.image & lead) { r.image ^= b.image; r.coord ^= b.coord; }
    }
    return r;
  };
  for (int t = 0; t < n; ++t) {
    Row r = reduce(Row{col[(size_t)t], uint64_t(1) << t});
    if (r.image == 0) { kernel.push_back(r.coord); continue; }
    basis.push_back(r);
    std::sort(basis.begin(), basis.end(), [](const Row& x, const Row& y) { return x.image > y.image; });
  }
  // kernel vectors with distinct leading bits, highest first: subtracting them greedily gives the smallest member of a coset
  std::vector<uint64_t> kred;
  for (uint64_t v : kernel) {
    for (uint64_t w : kred) {
      const uint64_t lead = uint64_t(1) << (63 - __builtin_clzll(w));
      if (v & lead) v ^= w;
    }
    if (v) {
      kred.push_back(v);
      std::sort(kred.begin(), kred.end(), [](uint64_t x, uint64_t y) { return x > y; });
    }
  }
  // full reduction of kred so that a vector's leading bit appears in no other vector
  for (size_t i = 0; i < kred.size(); ++i) {
    const uint64_t lead = uint64_t(1) << (63 - __builtin_clzll(kred[i]));
    for (size_t j = 0; j < kred.size(); ++j)
      if (j != i && (kred[j] & lead)) kred[j] ^= kred[i];
  }
  std::sort(kred.begin(), kred.end(), [](uint64_t x, uint64_t y) { return x > y; });
  SemiLayout r;
  for (int b = 0; b < 62; ++b) {
    Row want = reduce(Row{uint64_t(1) << b, 0});
    if (want.image != 0) break;          // 2^b is not in the image
    uint64_t x = want.coord;            // A(x) = 2^b
    for (uint64_t v : kred) {
      const uint64_t lead = uint64_t(1) << (63 - __builtin_clzll(v));
      if (x & lead) x ^= v;
    }
    r.extent.push_back(2);
    SemiStride st;
    st.kind = SemiStride::Xor;
    st.a = (int64_t)x;
    r.stride.push_back(st);
  }
  if (r.extent.empty()) { r.extent.push_back(1); r.stride.push_back(SemiStride{}); }
  if (r.extent.size() == 1) r.profile = {0};
  else { r.profile.assign(r.extent.size() + 1, 0); r.profile[0] = (int32_t)r.extent.size(); }
  *out = r;
  return LC_OK;
}

}  // namespace lc
