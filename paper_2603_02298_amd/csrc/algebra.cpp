#include "algebra.hpp"

#include <algorithm>
#include <climits>

namespace lc {

// ---------------------------------------------------------------------------------------------
// Coalesce (Sec. 3.2): one pass over the leaves; a leaf joins the open mode when its stride
// continues it (stride == extent * stride of the open mode); unit extents vanish.
// ---------------------------------------------------------------------------------------------
Modes coalesce_modes(const Modes& in, bool keep_last_unit) {
  Modes out;
  for (size_t k = 0; k < in.size(); ++k) {
    const Mode& m = in[k];
    bool forced = keep_last_unit && k + 1 == in.size();
    if (m.extent == 1 && !forced) continue;
    if (!out.empty() && m.stride == out.back().extent * out.back().stride)
      out.back().extent *= m.extent;
    else
      out.push_back(m);
  }
  if (out.empty()) out.push_back({1, 0});
  return out;
}

Layout coalesce(const Layout& a) { return Layout::flat(coalesce_modes(a.leaves)); }

Layout coalesce_bymode(const Layout& a) {
  if (a.is_leaf()) return coalesce(a);
  std::vector<Layout> parts;
  for (int i = 0; i < a.rank(); ++i) parts.push_back(coalesce(a.mode(i)));
  return Layout::tuple(parts);
}

// ---------------------------------------------------------------------------------------------
// Composition (Sec. 3.3).  For one mode s:d of B the modes of the coalesced A are visited in
// order: first the leading d elements are "divided out" of A, then the first s elements of what
// remains are "kept" (Sec. 3.3.3).  A mode that the s*d reach never leaves ends the walk without
// any divisibility requirement (the truncation argument of Sec. 3.3.2).
// ---------------------------------------------------------------------------------------------
static lc_status_t compose_mode(const Modes& A, int64_t s, int64_t d, Modes* out) {
  out->clear();
  if (d == 0) { out->push_back({s, 0}); return LC_OK; }
  int64_t skip = d;   // elements of the current level between consecutive picks
  int64_t want = s;   // picks still to place
  for (size_t r = 0; r < A.size(); ++r) {
    const int64_t S = A[r].extent, D = A[r].stride;
    bool stays = (r + 1 == A.size()) || (want - 1) * skip < S;   // the picks never leave this mode
    if (stays) {
      out->push_back({want, D * skip});
      want = 1;
      break;
    }
    if (skip >= S) {                       // the whole mode is divided out
      if (skip % S != 0) return LC_ERR_STRIDE_DIVISIBILITY;          // Eq. divis_stride
      skip /= S;
      continue;
    }
    if (S % skip != 0) return LC_ERR_STRIDE_DIVISIBILITY;            // Eq. divis_stride
    int64_t kept = S / skip;               // this mode contributes `kept` picks at stride D*skip
    if (want % kept != 0) return LC_ERR_SHAPE_DIVISIBILITY;          // Eq. divis_shape
    out->push_back({kept, D * skip});
    want /= kept;
    skip = 1;
  }
  // unit modes carry no information, except when the result is the single mode 1:x
  Modes cleaned = coalesce_modes(*out);
  if (cleaned.size() == 1 && cleaned[0].extent == 1) cleaned[0].stride = A[0].stride * d;
  *out = cleaned;
  return LC_OK;
}

lc_status_t composition(const Layout& a, const Layout& b, Layout* out) {
  Modes A = coalesce_modes(a.leaves, true);
  // Conditions under which composition distributes over the modes of B (Sec. 3.3.2, distributive
  // case): needed only if B as a whole reaches beyond the first mode of A.
  int64_t reach = 0;
  std::vector<const Mode*> moving;
  for (const Mode& m : b.leaves)
    if (m.extent > 1 && m.stride > 0) { moving.push_back(&m); reach += (m.extent - 1) * m.stride; }
  size_t last_reached = 0;
  {
    int64_t below = 1;
    for (size_t r = 0; r < A.size(); ++r) {
      if (below <= reach) last_reached = r;
      below *= A[r].extent;
    }
  }
  if (last_reached >= 1 && moving.size() >= 2) {
    for (size_t i = 0; i < moving.size(); ++i)
      for (size_t j = i + 1; j < moving.size(); ++j) {
        const Mode &x = *moving[i], &y = *moving[j];
        if (x.extent * x.stride > y.stride && y.extent * y.stride > x.stride) return LC_ERR_NOT_SEGREGATED;
      }
    for (const Mode* m : moving) {
      int64_t below = 1;
      for (size_t r = 0; r <= last_reached; ++r) {
        if (below % m->stride != 0 && m->stride % below != 0) return LC_ERR_STRIDE_DIVISIBILITY;
        below *= A[r].extent;
      }
    }
  }
  // Eq. layout_distributivity: A o (B_0, B_1, ...) = (A o B_0, A o B_1, ...), keeping B's profile;
  // a mode of B that becomes several modes nests in place.
  Layout R;
  size_t leaf = 0;
  for (int32_t p : b.profile) {
    if (p != 0) { R.profile.push_back(p); continue; }
    Modes part;
    lc_status_t st = compose_mode(A, b.leaves[leaf].extent, b.leaves[leaf].stride, &part);
    if (st != LC_OK) return st;
    ++leaf;
    if (part.size() == 1) {
      R.profile.push_back(0);
    } else {
      R.profile.push_back((int32_t)part.size());
      R.profile.insert(R.profile.end(), part.size(), 0);
    }
    R.leaves.insert(R.leaves.end(), part.begin(), part.end());
  }
  *out = R;
  return LC_OK;
}

static int tiler_rank(const Layout& t) { return t.is_leaf() ? 1 : t.rank(); }

lc_status_t composition_bymode(const Layout& a, const Layout& tiler, Layout* out) {
  if (tiler.is_leaf()) return composition(a, tiler, out);
  if (tiler_rank(tiler) > a.rank()) return LC_ERR_INVALID_ARG;
  std::vector<Layout> parts;
  for (int i = 0; i < a.rank(); ++i) {
    if (i < tiler_rank(tiler)) {
      Layout part;
      lc_status_t st = composition(a.mode(i), tiler.mode(i), &part);
      if (st != LC_OK) return st;
      parts.push_back(part);
    } else {
      parts.push_back(a.mode(i));
    }
  }
  *out = Layout::tuple(parts);
  return LC_OK;
}

// ---------------------------------------------------------------------------------------------
// Complement (Sec. 3.5): the moving modes of A in stride order leave, below each of them, a hole
// of floor(stride / covered) multiples of what is already covered; the complement is the list of
// those holes followed by the mode that steps over all of A up to the cotarget.
// ---------------------------------------------------------------------------------------------
static Modes moving_modes_by_stride(const Modes& in) {
  Modes m;
  for (const Mode& x : in)
    if (x.extent > 1 && x.stride > 0) m.push_back(x);
  std::stable_sort(m.begin(), m.end(), [](const Mode& x, const Mode& y) { return x.stride < y.stride; });
  return m;
}

lc_status_t complement(const Layout& a, int64_t cotarget, Layout* out) {
  if (cotarget < 0) return LC_ERR_INVALID_ARG;
  if (cotarget == 0) cotarget = a.cosize();
  Modes result;
  int64_t covered = 1;
  for (const Mode& m : moving_modes_by_stride(a.leaves)) {
    if (m.stride < covered) return LC_ERR_NOT_INJECTIVE;
    int64_t hole = m.stride / covered;
    if (hole > 1) result.push_back({hole, covered});
    covered = m.extent * m.stride;
  }
  result.push_back({(cotarget + covered - 1) / covered, covered});
  *out = Layout::flat(result);
  return LC_OK;
}

// ---------------------------------------------------------------------------------------------
// Right-inverse (Sec. 3.4.1): offsets 0,1,2,... are produced by the mode of stride 1, then by the
// mode whose stride is the size of that one, and so on; each such mode sends offsets back to its
// own position (the product of the extents before it) in the coalesced layout.
// ---------------------------------------------------------------------------------------------
Layout right_inverse(const Layout& a) {
  Modes c = coalesce_modes(a.leaves);
  struct Link { int64_t extent, stride, position; };
  std::vector<Link> links;
  int64_t position = 1;
  for (const Mode& m : c) {
    if (m.stride > 0) links.push_back({m.extent, m.stride, position});
    position *= m.extent;
  }
  std::stable_sort(links.begin(), links.end(), [](const Link& x, const Link& y) { return x.stride < y.stride; });
  Modes inv;
  int64_t next = 1;
  for (const Link& l : links) {
    if (l.stride != next) break;
    inv.push_back({l.extent, l.position});
    next = l.extent * l.stride;
  }
  if (inv.empty()) inv.push_back({1, 0});
  return Layout::flat(coalesce_modes(inv));
}

// ---------------------------------------------------------------------------------------------
// Left-inverse (Sec. 3.4.3): offsets are decomposed digit by digit in the mixed radix given by the
// ratios of consecutive strides; digit k is sent to the position of the mode that produced it.
// ---------------------------------------------------------------------------------------------
lc_status_t left_inverse(const Layout& a, Layout* out) {
  Modes c = coalesce_modes(a.leaves);
  struct Link { int64_t extent, stride, position; };
  std::vector<Link> links;
  int64_t position = 1;
  for (const Mode& m : c) {
    if (m.stride > 0 && m.extent > 1) links.push_back({m.extent, m.stride, position});
    position *= m.extent;
  }
  std::stable_sort(links.begin(), links.end(), [](const Link& x, const Link& y) { return x.stride < y.stride; });
  if (links.empty()) { *out = Layout::leaf(1, 0); return LC_OK; }
  Modes inv;
  if (links.front().stride > 1) inv.push_back({links.front().stride, 0});   // offsets below the first stride
  for (size_t k = 0; k < links.size(); ++k) {
    int64_t radix = links[k].extent;
    if (k + 1 < links.size()) {
      if (links[k].extent * links[k].stride > links[k + 1].stride) return LC_ERR_NOT_INJECTIVE;
      if (links[k + 1].stride % links[k].stride != 0) return LC_ERR_STRIDE_DIVISIBILITY;
      radix = links[k + 1].stride / links[k].stride;
    }
    inv.push_back({radix, links[k].position});
  }
  *out = Layout::flat(coalesce_modes(inv));
  return LC_OK;
}

// ---------------------------------------------------------------------------------------------
// Application of the left-inverse (Sec. 3.4.3): which offsets of an instruction layout T exist in a data layout A, and
// where.  The left-inverse turns an offset into the only coordinate that could produce it; the offset exists in A exactly
// when that coordinate is inside A's domain and A maps it back to the offset.
// ---------------------------------------------------------------------------------------------
lc_status_t admissible(const Layout& a, const Layout& t, bool* yes, Layout* where, bool* has_where) {
  Layout inv;
  lc_status_t st = left_inverse(a, &inv);
  if (st != LC_OK) return st;
  const int64_t na = a.size(), nt = t.size();
  if (nt > (1ll << 26)) return LC_ERR_TOO_LARGE;
  *yes = true;
  for (int64_t i = 0; i < nt && *yes; ++i) {
    const int64_t off = t(i), c = inv(off);
    if (c < 0 || c >= na || a(c) != off) *yes = false;
  }
  *has_where = false;
  if (*yes && composition(inv, t, where) == LC_OK) *has_where = true;
  return LC_OK;
}

// ---------------------------------------------------------------------------------------------
// Products (Sec. 3.5.1): A (x) B = (A, A* o B); the blocked / raked products pair up like modes.
// ---------------------------------------------------------------------------------------------
lc_status_t logical_product(const Layout& a, const Layout& b, Layout* out) {
  Layout astar, grid;
  lc_status_t st = complement(a, 0, &astar);
  if (st != LC_OK) return st;
  st = composition(astar, b, &grid);
  if (st != LC_OK) return st;
  *out = Layout::tuple({a, grid});
  return LC_OK;
}

static lc_status_t paired_product(const Layout& a, const Layout& b, bool tile_first, Layout* out) {
  if (a.rank() != b.rank()) return LC_ERR_INVALID_ARG;
  Layout p;
  lc_status_t st = logical_product(a, b, &p);
  if (st != LC_OK) return st;
  const Layout tile = p.mode(0), grid = p.mode(1);
  std::vector<Layout> pairs;
  for (int i = 0; i < a.rank(); ++i) {
    Layout t = tile.mode(i), g = b.is_leaf() ? grid : grid.mode(i);
    pairs.push_back(tile_first ? Layout::tuple({t, g}) : Layout::tuple({g, t}));
  }
  *out = pairs.size() == 1 ? pairs[0] : Layout::tuple(pairs);
  return LC_OK;
}
lc_status_t blocked_product(const Layout& a, const Layout& b, Layout* out) { return paired_product(a, b, true, out); }
lc_status_t raked_product(const Layout& a, const Layout& b, Layout* out) { return paired_product(a, b, false, out); }

// ---------------------------------------------------------------------------------------------
// Divides (Sec. 3.5.2)
// ---------------------------------------------------------------------------------------------
static Layout without_unit_modes(const Layout& L) {
  if (L.is_leaf()) return L.leaves[0].extent == 1 ? Layout::leaf(1, 0) : L;
  std::vector<Layout> kept;
  for (int i = 0; i < L.rank(); ++i) {
    Layout sub = without_unit_modes(L.mode(i));
    if (sub.size() > 1) kept.push_back(sub);
  }
  if (kept.empty()) return Layout::leaf(1, 0);
  if (kept.size() == 1) return kept[0];
  return Layout::tuple(kept);
}

lc_status_t logical_divide(const Layout& a, const Layout& b, Layout* out) {
  Layout bstar;
  lc_status_t st = complement(b, a.size(), &bstar);
  if (st != LC_OK) return st;
  // (B, B*) has to reach every coordinate of A: the complement fills the space below a mode of B
  // only in whole multiples of what lies beneath it, so the first inexact step is the first miss.
  int64_t covered = 1;
  for (const Mode& m : moving_modes_by_stride(b.leaves)) {
    if (m.stride % covered != 0) {
      if (covered * (m.stride / covered) < a.size()) return LC_ERR_NOT_SURJECTIVE;
      break;
    }
    covered = m.extent * m.stride;
  }
  Layout both;
  st = composition(a, Layout::tuple({b, bstar}), &both);
  if (st != LC_OK) return st;
  *out = Layout::tuple({both.mode(0), without_unit_modes(both.mode(1))});
  return LC_OK;
}

lc_status_t logical_divide_bymode(const Layout& a, const Layout& tiler, Layout* out) {
  if (tiler_rank(tiler) > a.rank()) return LC_ERR_INVALID_ARG;
  std::vector<Layout> parts;
  for (int i = 0; i < a.rank(); ++i) {
    if (i < tiler_rank(tiler)) {
      Layout part;
      lc_status_t st = logical_divide(a.mode(i), tiler.mode(i), &part);
      if (st != LC_OK) return st;
      parts.push_back(part);
    } else {
      parts.push_back(a.mode(i));
    }
  }
  *out = parts.size() == 1 ? parts[0] : Layout::tuple(parts);
  return LC_OK;
}

lc_status_t zipped_divide(const Layout& a, const Layout& tiler, Layout* out) {
  if (tiler_rank(tiler) > a.rank()) return LC_ERR_INVALID_ARG;
  std::vector<Layout> tiles, rests;
  for (int i = 0; i < a.rank(); ++i) {
    if (i < tiler_rank(tiler)) {
      Layout part;
      lc_status_t st = logical_divide(a.mode(i), tiler.mode(i), &part);
      if (st != LC_OK) return st;
      tiles.push_back(part.mode(0));
      rests.push_back(part.mode(1));
    } else {
      rests.push_back(a.mode(i));
    }
  }
  Layout tile = tiles.size() == 1 ? tiles[0] : Layout::tuple(tiles);
  Layout rest = rests.size() == 1 ? rests[0] : Layout::tuple(rests);
  *out = Layout::tuple({tile, rest});
  return LC_OK;
}

// ---------------------------------------------------------------------------------------------
// Slicing (Sec. 2.5.1).  The coordinate text is walked together with the layout: an integer is
// evaluated by the sub-layout it addresses and added to the offset, "_" keeps that sub-layout.
// ---------------------------------------------------------------------------------------------
namespace {
struct SliceWalk {
  const char* p;
  int64_t offset = 0;
  lc_status_t status = LC_OK;
  void ws() { while (*p == ' ') ++p; }
  // returns the kept part of `L` under the coordinate at the cursor (nullptr-like: empty profile = nothing kept)
  bool walk(const Layout& L, Layout* kept) {
    ws();
    kept->profile.clear();
    kept->leaves.clear();
    if (*p == '_') { ++p; *kept = L; return true; }
    if (*p >= '0' && *p <= '9') {
      int64_t v = 0;
      int digits = 0;
      while (*p >= '0' && *p <= '9') { v = v * 10 + (*p++ - '0'); if (++digits > 18) { status = LC_ERR_PARSE; return false; } }
      offset += L(v);
      return true;
    }
    if (*p != '(') { status = LC_ERR_PARSE; return false; }
    ++p;
    if (L.is_leaf()) { status = LC_ERR_NOT_CONGRUENT; return false; }
    std::vector<Layout> mine;
    for (int i = 0; i < L.rank(); ++i) {
      Layout part;
      if (!walk(L.mode(i), &part)) return false;
      if (!part.profile.empty()) mine.push_back(part);
      ws();
      if (i + 1 < L.rank()) {
        if (*p != ',') { status = (*p == ')') ? LC_ERR_NOT_CONGRUENT : LC_ERR_PARSE; return false; }
        ++p;
      }
    }
    ws();
    if (*p != ')') { status = (*p == ',') ? LC_ERR_NOT_CONGRUENT : LC_ERR_PARSE; return false; }
    ++p;
    if (mine.size() == 1) *kept = mine[0];
    else if (mine.size() > 1) *kept = Layout::tuple(mine);
    return true;
  }
};
}  // namespace

lc_status_t slice(const Layout& a, const char* coord, int64_t* offset, Layout* out) {
  SliceWalk w{coord};
  Layout kept;
  if (!w.walk(a, &kept)) return w.status;
  w.ws();
  if (*w.p != 0) return LC_ERR_PARSE;
  *offset = w.offset;
  *out = kept.profile.empty() ? Layout::leaf(1, 0) : kept;
  return LC_OK;
}

// ---------------------------------------------------------------------------------------------
// Vectorisation (Sec. 3.4.2): K = extent of the stride-1 head of coalesce(A o B^).
// ---------------------------------------------------------------------------------------------
lc_status_t max_common_vector(const Layout& a, const Layout& b, int64_t* K) {
  if (a.size() != b.size()) return LC_ERR_SIZE_MISMATCH;
  Layout r;
  lc_status_t st = composition(a, right_inverse(b), &r);
  if (st != LC_OK) return st;
  Modes head = coalesce_modes(r.leaves);
  *K = head[0].stride == 1 ? head[0].extent : 1;
  return LC_OK;
}

}  // namespace lc
