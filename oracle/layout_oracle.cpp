// ORACLE — test infrastructure only (see layout_oracle.hpp).
// Plain recursive code over HTuple trees; no tuning of any kind.
#include "layout_oracle.hpp"

#include <algorithm>
#include <cctype>
#include <climits>
#include <cstring>

namespace oracle {

// ===========================================================================
// HTuple basics (Sec. 2.1)
// ===========================================================================
int rank(const HTuple& x) { return x.is_int ? 1 : (int)x.items.size(); }

int depth(const HTuple& x) {
  if (x.is_int) return 0;
  int m = 0;
  for (const HTuple& k : x.items) m = std::max(m, depth(k));
  return 1 + m;
}

const HTuple& mode(const HTuple& x, int i) { return x.is_int ? x : x.items[(size_t)i]; }

bool congruent(const HTuple& p, const HTuple& s) {
  if (p.is_int && s.is_int) return true;
  if (p.is_int || s.is_int) return false;
  if (p.items.size() != s.items.size()) return false;
  for (size_t i = 0; i < p.items.size(); ++i)
    if (!congruent(p.items[i], s.items[i])) return false;
  return true;
}

bool weakly_congruent(const HTuple& p, const HTuple& s) {
  if (p.is_int) return true;
  if (s.is_int) return false;
  if (p.items.size() != s.items.size()) return false;
  for (size_t i = 0; i < p.items.size(); ++i)
    if (!weakly_congruent(p.items[i], s.items[i])) return false;
  return true;
}

int64_t size(const HTuple& shape) {
  if (shape.is_int) return shape.value;
  int64_t n = 1;
  for (const HTuple& k : shape.items) n *= size(k);
  return n;
}

bool compatible(const HTuple& p, const HTuple& s) {
  if (p.is_int) return p.value == size(s);
  if (s.is_int) return false;
  if (p.items.size() != s.items.size()) return false;
  for (size_t i = 0; i < p.items.size(); ++i)
    if (!compatible(p.items[i], s.items[i])) return false;
  return true;
}

static void collect_leaves(const HTuple& x, std::vector<int64_t>* out) {
  if (x.is_int) { out->push_back(x.value); return; }
  for (const HTuple& k : x.items) collect_leaves(k, out);
}

std::vector<int64_t> leaves(const HTuple& x) {
  std::vector<int64_t> v;
  collect_leaves(x, &v);
  return v;
}

std::string to_string(const HTuple& x) {
  if (x.is_int) return std::to_string(x.value);
  std::string s = "(";
  for (size_t i = 0; i < x.items.size(); ++i) {
    if (i) s += ",";
    s += to_string(x.items[i]);
  }
  return s + ")";
}

bool equal(const HTuple& a, const HTuple& b) {
  if (a.is_int != b.is_int) return false;
  if (a.is_int) return a.value == b.value;
  if (a.items.size() != b.items.size()) return false;
  for (size_t i = 0; i < a.items.size(); ++i)
    if (!equal(a.items[i], b.items[i])) return false;
  return true;
}

// ===========================================================================
// Coordinates (Sec. 2.2.2)
// ===========================================================================
// Eq. idx2crd: (i mod |S_0|, floor(i/|S_0|) mod |S_1|, ..., floor(i / prod_{k<r-1}|S_k|)).
std::vector<int64_t> idx2crd(int64_t i, const HTuple& shape) {
  int r = rank(shape);
  std::vector<int64_t> c((size_t)r);
  int64_t prefix = 1;
  for (int k = 0; k < r; ++k) {
    int64_t sk = size(mode(shape, k));
    int64_t q = i / prefix;
    c[(size_t)k] = (k < r - 1) ? (q % sk) : q;  // the last entry is not reduced
    prefix *= sk;
  }
  return c;
}

// Eq. crd2idx: c_0 + c_1 |S_0| + ... + c_{r-1} prod_{k<r-1}|S_k|.
int64_t crd2idx(const std::vector<int64_t>& c, const HTuple& shape) {
  int64_t idx = 0, prefix = 1;
  for (int k = 0; k < rank(shape); ++k) {
    idx += c[(size_t)k] * prefix;
    prefix *= size(mode(shape, k));
  }
  return idx;
}

HTuple idx2crd_natural(int64_t i, const HTuple& shape) {
  if (shape.is_int) return HTuple::Int(i);
  std::vector<int64_t> c = idx2crd(i, shape);
  std::vector<HTuple> out;
  for (size_t k = 0; k < shape.items.size(); ++k) out.push_back(idx2crd_natural(c[k], shape.items[k]));
  return HTuple::Tup(out);
}

HTuple crd2natural(const HTuple& c, const HTuple& shape) {
  if (c.is_int) return idx2crd_natural(c.value, shape);
  std::vector<HTuple> out;  // c is a tuple of the same rank as shape (weak congruence)
  for (size_t k = 0; k < shape.items.size(); ++k) out.push_back(crd2natural(c.items[k], shape.items[k]));
  return HTuple::Tup(out);
}

int64_t crd2idx_h(const HTuple& c, const HTuple& shape) {
  if (c.is_int) return c.value;
  std::vector<int64_t> flat;
  for (size_t k = 0; k < shape.items.size(); ++k) flat.push_back(crd2idx_h(c.items[k], shape.items[k]));
  return crd2idx(flat, shape);
}

// Eq. innerprod.
int64_t inner_product(const HTuple& c, const HTuple& d) {
  if (c.is_int) return c.value * d.value;
  int64_t sum = 0;
  for (size_t k = 0; k < c.items.size(); ++k) sum += inner_product(c.items[k], d.items[k]);
  return sum;
}

// ===========================================================================
// Layout (Sec. 2.4)
// ===========================================================================
namespace {
struct Parser {
  const std::string& s;
  size_t pos = 0;
  bool ok = true;
  explicit Parser(const std::string& text) : s(text) {}
  void skip() { while (pos < s.size() && std::isspace((unsigned char)s[pos])) ++pos; }
  HTuple htuple() {
    skip();
    if (pos < s.size() && s[pos] == '(') {
      ++pos;
      std::vector<HTuple> items;
      for (;;) {
        items.push_back(htuple());
        if (!ok) return HTuple::Int(0);
        skip();
        if (pos < s.size() && s[pos] == ',') { ++pos; continue; }
        if (pos < s.size() && s[pos] == ')') { ++pos; break; }
        ok = false;
        return HTuple::Int(0);
      }
      return HTuple::Tup(items);
    }
    size_t start = pos;
    if (pos < s.size() && s[pos] == '-') ++pos;
    while (pos < s.size() && std::isdigit((unsigned char)s[pos])) ++pos;
    if (pos == start || (s[start] == '-' && pos == start + 1) || pos - start > 18) { ok = false; return HTuple::Int(0); }
    return HTuple::Int(std::stoll(s.substr(start, pos - start)));
  }
};
}  // namespace

Status parse_layout(const std::string& text, Layout* out) {
  Parser p(text);
  Layout L;
  L.shape = p.htuple();
  p.skip();
  if (!p.ok || p.pos >= text.size() || text[p.pos] != ':') return ERR_PARSE;
  ++p.pos;
  L.stride = p.htuple();
  p.skip();
  if (!p.ok || p.pos != text.size()) return ERR_PARSE;
  Status st = validate(L);
  if (st != OK) return st;
  *out = L;
  return OK;
}

Status validate(const Layout& L) {
  if (!congruent(L.shape, L.stride)) return ERR_NOT_CONGRUENT;  // Sec. 2.3: S ~ D
  for (int64_t s : leaves(L.shape)) if (s < 1) return ERR_BAD_EXTENT;          // shape is an HTuple(Z+)
  // strides are integers of either sign (Sec. 2.3.2: Z is an integer-semimodule).  The layout function, coalesce and
  // COPY take them as they are; the algebra whose statements are written for strides in N (composition's divisibility
  // conditions, complement's ordering, the inverses) refuses them: see has_negative_stride().
  return OK;
}

std::string to_string(const Layout& L) { return to_string(L.shape) + ":" + to_string(L.stride); }

Layout make_layout(const std::vector<int64_t>& s, const std::vector<int64_t>& d) {
  Layout L;
  if (s.size() == 1) {
    L.shape = HTuple::Int(s[0]);
    L.stride = HTuple::Int(d[0]);
    return L;
  }
  std::vector<HTuple> ss, dd;
  for (size_t i = 0; i < s.size(); ++i) { ss.push_back(HTuple::Int(s[i])); dd.push_back(HTuple::Int(d[i])); }
  L.shape = HTuple::Tup(ss);
  L.stride = HTuple::Tup(dd);
  return L;
}

Layout sublayout(const Layout& L, int i) {
  Layout R;
  R.shape = mode(L.shape, i);
  R.stride = mode(L.stride, i);
  return R;
}

Layout concat(const std::vector<Layout>& parts) {
  std::vector<HTuple> ss, dd;
  for (const Layout& p : parts) { ss.push_back(p.shape); dd.push_back(p.stride); }
  Layout L;
  L.shape = HTuple::Tup(ss);
  L.stride = HTuple::Tup(dd);
  return L;
}

int64_t size(const Layout& L) { return size(L.shape); }

int64_t cosize(const Layout& L) {
  // The largest offset is reached with every mode of positive stride at its last coordinate and every mode of negative
  // stride at coordinate 0.
  std::vector<int64_t> s = leaves(L.shape), d = leaves(L.stride);
  int64_t m = 0;
  for (size_t k = 0; k < s.size(); ++k) if (d[k] > 0) m += (s[k] - 1) * d[k];
  return m + 1;
}

int64_t min_offset(const Layout& L) {
  // The smallest offset: every mode of negative stride at its last coordinate (0 when no stride is negative).
  std::vector<int64_t> s = leaves(L.shape), d = leaves(L.stride);
  int64_t m = 0;
  for (size_t k = 0; k < s.size(); ++k) if (d[k] < 0) m += (s[k] - 1) * d[k];
  return m;
}

bool has_negative_stride(const Layout& L) {
  for (int64_t d : leaves(L.stride)) if (d < 0) return true;
  return false;
}

// L(i) = inner_product(idx2crd_S(i), D), idx2crd applied again inside every mode
// (Sec. 2.2.2 "repeated application", Sec. 2.4 Def. layout).
static int64_t eval_rec(const HTuple& S, const HTuple& D, int64_t i) {
  if (S.is_int) return i * D.value;
  int64_t sum = 0, q = i;   // q = floor(i / prod_{j<k} |S_j|)
  for (size_t k = 0; k < S.items.size(); ++k) {
    int64_t sk = size(S.items[k]);
    int64_t ck = (k + 1 < S.items.size()) ? (q % sk) : q;   // Eq. idx2crd, last entry not reduced
    q /= sk;
    sum += eval_rec(S.items[k], D.items[k], ck);            // Eq. innerprod, one term per mode
  }
  return sum;
}

int64_t eval(const Layout& L, int64_t i) { return eval_rec(L.shape, L.stride, i); }

int64_t eval_crd(const Layout& L, const HTuple& c) {
  return inner_product(crd2natural(c, L.shape), L.stride);
}

// ===========================================================================
// Slicing (Sec. 2.5.1): T(c' + c*) = (e + L(c')) o L(c*).  A hole keeps its whole sub-mode; a tuple
// that keeps exactly one piece is that piece, a tuple that keeps none disappears.
// ===========================================================================
static bool slice_rec(const Layout& L, const HTuple& c, int64_t* offset, std::vector<Layout>* kept, Status* st) {
  if (c.is_int) {
    if (c.value == -1) { kept->push_back(L); return true; }       // unspecified: stays
    *offset += eval(L, c.value);                                    // specified: L(c') goes into the accessor
    return true;
  }
  if (L.shape.is_int || rank(L.shape) != (int)c.items.size()) { *st = ERR_NOT_CONGRUENT; return false; }
  std::vector<Layout> mine;
  for (int i = 0; i < rank(L.shape); ++i)
    if (!slice_rec(sublayout(L, i), c.items[(size_t)i], offset, &mine, st)) return false;
  if (mine.size() == 1) kept->push_back(mine[0]);
  else if (mine.size() > 1) kept->push_back(concat(mine));
  return true;
}

Status slice(const Layout& L, const HTuple& coord_with_holes, Slice* out) {
  Status st = OK;
  int64_t offset = 0;
  std::vector<Layout> kept;
  if (!slice_rec(L, coord_with_holes, &offset, &kept, &st)) return st;
  out->offset = offset;
  out->rest = kept.empty() ? make_layout({1}, {0}) : kept[0];
  return OK;
}

// ===========================================================================
// Coalesce (Sec. 3.2).  Reading: walk the leaves left to right, skip extent-1
// leaves, merge a leaf into the previous kept mode when its stride equals
// extent*stride of that mode; never reorder.  All-ones collapses to 1:0.
// ===========================================================================
struct FlatModes { std::vector<int64_t> s, d; };

static FlatModes coalesce_flat(const Layout& A, bool keep_last_mode) {
  std::vector<int64_t> S = leaves(A.shape), D = leaves(A.stride);
  FlatModes r;
  for (size_t k = 0; k < S.size(); ++k) {
    bool last = (k + 1 == S.size());
    if (S[k] == 1 && !(keep_last_mode && last)) continue;
    if (!r.s.empty() && D[k] == r.s.back() * r.d.back()) { r.s.back() *= S[k]; continue; }
    r.s.push_back(S[k]);
    r.d.push_back(D[k]);
  }
  if (r.s.empty()) { r.s.push_back(1); r.d.push_back(0); }
  return r;
}

Layout coalesce(const Layout& A) {
  FlatModes f = coalesce_flat(A, false);
  return make_layout(f.s, f.d);
}

Layout coalesce_bymode(const Layout& A) {
  if (A.shape.is_int) return coalesce(A);
  std::vector<Layout> parts;
  for (int i = 0; i < rank(A.shape); ++i) parts.push_back(coalesce(sublayout(A, i)));
  return concat(parts);
}

// ===========================================================================
// Composition (Sec. 3.3).
// ===========================================================================
static int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

namespace {
struct ComposeCtx {
  std::vector<int64_t> S, D, Sbar;  // coalesced A and its exclusive prefix products
};
}

// Base case A o (s:d), Sec. 3.3.2 "Base Case".
static Status compose_leaf(const ComposeCtx& A, int64_t s, int64_t d, Layout* out) {
  if (d == 0) { *out = make_layout({s}, {0}); return OK; }   // B(i) = 0 for all i and A(0) = 0
  int R = (int)A.S.size() - 1;
  // Truncation: modes whose prefix product exceeds the reach (s-1)d never contribute,
  // and the last contributing mode needs no modulus.
  int64_t reach = (s - 1) * d;
  int Rp = 0;
  for (int r = 0; r <= R; ++r) if (A.Sbar[(size_t)r] <= reach) Rp = r;
  std::vector<int64_t> rs, rd;
  for (int r = 0; r <= Rp; ++r) {
    int64_t sb = A.Sbar[(size_t)r];
    if (sb % d != 0 && d % sb != 0) return ERR_STRIDE_DIVISIBILITY;      // Eq. divis_stride
    int64_t delta = ceil_div(d, sb), rho = ceil_div(sb, d);
    if (s % rho != 0) return ERR_SHAPE_DIVISIBILITY;                     // Eq. divis_shape
    int64_t extent;
    if (r < Rp) {
      if (delta < A.S[(size_t)r] && A.S[(size_t)r] % delta != 0) return ERR_STRIDE_DIVISIBILITY;  // delta_r | S_r
      extent = ceil_div(A.S[(size_t)r], delta);                          // S'_r = S_r / delta_r
    } else {
      extent = s / rho;                                                  // S'_R = s / rho_R
    }
    rs.push_back(extent);
    rd.push_back(A.D[(size_t)r] * delta);                                // D'_r = D_r delta_r
  }
  Layout raw = make_layout(rs, rd);
  if (size(raw) == 1) { *out = make_layout({1}, {A.D[0] * d}); return OK; }
  *out = coalesce(raw);
  return OK;
}

static Status compose_rec(const ComposeCtx& A, const Layout& B, Layout* out) {
  if (B.shape.is_int) return compose_leaf(A, B.shape.value, B.stride.value, out);
  std::vector<Layout> parts;   // distributes over the concatenation of B (Eq. layout_distributivity)
  for (int i = 0; i < rank(B.shape); ++i) {
    Layout part;
    Status st = compose_rec(A, sublayout(B, i), &part);
    if (st != OK) return st;
    parts.push_back(part);
  }
  *out = concat(parts);
  return OK;
}

Status composition(const Layout& A, const Layout& B, Layout* R) {
  // A may be coalesced first (Sec. 3.3.2); a trailing extent-1 mode is kept because its
  // stride defines A on the extended domain (needed by the products of Sec. 3.5.1).
  FlatModes f = coalesce_flat(A, true);
  ComposeCtx ctx;
  ctx.S = f.s;
  ctx.D = f.d;
  int64_t p = 1;
  for (size_t r = 0; r < f.s.size(); ++r) { ctx.Sbar.push_back(p); p *= f.s[r]; }

  // Distributivity conditions of Sec. 3.3.2 "Reductive Case: Distributive": over the leaves of
  // B that move (s > 1, d > 0), images are mutually segregated and every stride satisfies the
  // stride divisibility condition against every mode of A that B can reach in total.
  std::vector<int64_t> bs = leaves(B.shape), bd = leaves(B.stride);
  std::vector<size_t> moving;
  int64_t total_reach = 0;
  for (size_t i = 0; i < bs.size(); ++i)
    if (bs[i] > 1 && bd[i] > 0) { moving.push_back(i); total_reach += (bs[i] - 1) * bd[i]; }
  int Rtot = 0;
  for (size_t r = 0; r < ctx.Sbar.size(); ++r) if (ctx.Sbar[r] <= total_reach) Rtot = (int)r;
  if (Rtot >= 1 && moving.size() >= 2) {   // within reach A is not a single linear mode
    for (size_t a = 0; a < moving.size(); ++a)
      for (size_t b = a + 1; b < moving.size(); ++b) {
        size_t i = moving[a], j = moving[b];
        if (!(bs[i] * bd[i] <= bd[j] || bs[j] * bd[j] <= bd[i])) return ERR_NOT_SEGREGATED;
      }
    for (size_t a = 0; a < moving.size(); ++a)
      for (int r = 0; r <= Rtot; ++r) {
        int64_t d = bd[moving[a]], sb = ctx.Sbar[(size_t)r];
        if (sb % d != 0 && d % sb != 0) return ERR_STRIDE_DIVISIBILITY;
      }
  }
  return compose_rec(ctx, B, R);
}

Status composition_bymode(const Layout& A, const Layout& tiler, Layout* R) {
  // (A_0, A_1, ...) o <T_0, T_1, ...> = (A_0 o T_0, A_1 o T_1, ...); modes of A beyond the
  // tiler's rank are left whole.
  if (tiler.shape.is_int) return composition(A, tiler, R);
  if (rank(tiler.shape) > rank(A.shape)) return ERR_INVALID_ARG;
  std::vector<Layout> parts;
  for (int i = 0; i < rank(A.shape); ++i) {
    if (i < rank(tiler.shape)) {
      Layout part;
      Status st = composition(sublayout(A, i), sublayout(tiler, i), &part);
      if (st != OK) return st;
      parts.push_back(part);
    } else {
      parts.push_back(sublayout(A, i));
    }
  }
  *R = concat(parts);
  return OK;
}

// ===========================================================================
// Complement (Sec. 3.5).  Reading: drop stride-0 and extent-1 leaves, order the
// rest by stride, fill the hole below every mode, and always end with the mode
// that steps over everything ("1:32" in Table complements).
// ===========================================================================
Status complement(const Layout& A, int64_t cotarget, Layout* R) {
  if (cotarget < 0) return ERR_INVALID_ARG;
  if (cotarget == 0) cotarget = cosize(A);
  std::vector<int64_t> S = leaves(A.shape), D = leaves(A.stride);
  std::vector<std::pair<int64_t, int64_t>> modes;  // (stride, extent)
  for (size_t k = 0; k < S.size(); ++k)
    if (S[k] > 1 && D[k] > 0) modes.push_back({D[k], S[k]});
  std::stable_sort(modes.begin(), modes.end(),
                   [](const std::pair<int64_t, int64_t>& a, const std::pair<int64_t, int64_t>& b) { return a.first < b.first; });
  std::vector<int64_t> rs, rd;
  int64_t cur = 1;   // the offsets [0, cur) are covered by A together with the modes emitted so far
  for (const auto& m : modes) {
    int64_t d = m.first, s = m.second;
    if (d < cur) return ERR_NOT_INJECTIVE;   // this mode of A lands inside the span of the smaller ones
    int64_t hole = d / cur;
    if (hole > 1) { rs.push_back(hole); rd.push_back(cur); }
    cur = s * d;
  }
  rs.push_back(ceil_div(cotarget, cur));
  rd.push_back(cur);
  *R = make_layout(rs, rd);
  return OK;
}

// ===========================================================================
// Right-inverse (Sec. 3.4.1).  Reading: of the coalesced modes, follow the chain
// stride 1, then stride = extent*stride of the previous link, ...; each link maps
// offsets back to the position (prefix product) of its mode.  Ties keep the
// earlier mode.
// ===========================================================================
Layout right_inverse(const Layout& A) {
  FlatModes f = coalesce_flat(A, false);
  struct M { int64_t s, d, pos; };
  std::vector<M> modes;
  int64_t pos = 1;
  for (size_t k = 0; k < f.s.size(); ++k) {
    if (f.d[k] != 0) modes.push_back({f.s[k], f.d[k], pos});
    pos *= f.s[k];
  }
  std::stable_sort(modes.begin(), modes.end(), [](const M& a, const M& b) { return a.d < b.d; });
  std::vector<int64_t> rs, rd;
  int64_t cur = 1;
  for (const M& m : modes) {
    if (m.d != cur) break;
    rs.push_back(m.s);
    rd.push_back(m.pos);
    cur = m.s * m.d;
  }
  if (rs.empty()) return make_layout({1}, {0});
  return coalesce(make_layout(rs, rd));
}

// ===========================================================================
// Left-inverse (Sec. 3.4.3).  Reading: take the coalesced modes that move (stride > 0) in
// stride order; an offset o splits as o = sum_k c_k d_k with c_k = floor(o / d_k) mod (d_{k+1}/d_k),
// so the inverse has, per mode, extent d_{k+1}/d_k (the last keeps its own extent) and stride
// "position of that mode in A".  Offsets below the first stride map to coordinate 0 (a leading
// stride-0 mode; Table linv notes that any stride would do there).  Needs every stride to divide
// the next and the moving modes not to overlap (stride-0 modes are simply not inverted).
// ===========================================================================
Status left_inverse(const Layout& A, Layout* R) {
  FlatModes f = coalesce_flat(A, false);
  struct M { int64_t s, d, pos; };
  std::vector<M> modes;
  int64_t pos = 1;
  for (size_t k = 0; k < f.s.size(); ++k) {
    if (f.d[k] != 0 && f.s[k] > 1) modes.push_back({f.s[k], f.d[k], pos});
    pos *= f.s[k];
  }
  std::stable_sort(modes.begin(), modes.end(), [](const M& a, const M& b) { return a.d < b.d; });
  std::vector<int64_t> rs, rd;
  if (modes.empty()) { *R = make_layout({1}, {0}); return OK; }
  if (modes[0].d > 1) { rs.push_back(modes[0].d); rd.push_back(0); }
  for (size_t k = 0; k < modes.size(); ++k) {
    if (k + 1 < modes.size()) {
      if (modes[k].s * modes[k].d > modes[k + 1].d) return ERR_NOT_INJECTIVE;   // modes overlap: no layout inverts them
      if (modes[k + 1].d % modes[k].d != 0) return ERR_STRIDE_DIVISIBILITY;
      rs.push_back(modes[k + 1].d / modes[k].d);
    } else {
      rs.push_back(modes[k].s);
    }
    rd.push_back(modes[k].pos);
  }
  *R = coalesce(make_layout(rs, rd));
  return OK;
}

// ===========================================================================
// Application of the left-inverse (Sec. 3.4.3): every offset T(i) of an instruction layout exists in the
// image of the data layout A.  Written out as the statement reads: the image of A is enumerated, then
// every T(i) is looked up in it.
// ===========================================================================
bool admissible(const Layout& A, const Layout& T) {
  std::vector<int64_t> image;
  for (int64_t c = 0; c < size(A); ++c) image.push_back(eval(A, c));
  std::sort(image.begin(), image.end());
  for (int64_t i = 0; i < size(T); ++i)
    if (!std::binary_search(image.begin(), image.end(), eval(T, i))) return false;
  return true;
}

// ===========================================================================
// Logical product and its rearrangements (Sec. 3.5.1)
// ===========================================================================
Status logical_product(const Layout& A, const Layout& B, Layout* R) {
  Layout Astar;
  Status st = complement(A, 0, &Astar);
  if (st != OK) return st;
  Layout grid;
  st = composition(Astar, B, &grid);            // B orders and shapes the complement
  if (st != OK) return st;
  *R = concat({A, grid});
  return OK;
}

static Status zipped_product(const Layout& A, const Layout& B, bool tile_first, Layout* R) {
  int ra = A.shape.is_int ? 1 : rank(A.shape), rb = B.shape.is_int ? 1 : rank(B.shape);
  if (ra != rb) return ERR_INVALID_ARG;         // requires rank(A) == rank(B)
  Layout P;
  Status st = logical_product(A, B, &P);
  if (st != OK) return st;
  Layout tile = sublayout(P, 0), grid = sublayout(P, 1);
  std::vector<Layout> modes;
  for (int i = 0; i < ra; ++i) {
    Layout t = tile.shape.is_int ? tile : sublayout(tile, i);
    Layout g = grid.shape.is_int || B.shape.is_int ? grid : sublayout(grid, i);
    modes.push_back(tile_first ? concat({t, g}) : concat({g, t}));
  }
  *R = modes.size() == 1 ? modes[0] : concat(modes);
  return OK;
}

Status blocked_product(const Layout& A, const Layout& B, Layout* R) { return zipped_product(A, B, true, R); }
Status raked_product(const Layout& A, const Layout& B, Layout* R) { return zipped_product(A, B, false, R); }

// ===========================================================================
// Logical divide and zipped divide (Sec. 3.5.2)
// ===========================================================================
// Removes extent-1 leaves from a "rest" layout; nothing left -> 1:0; one mode left -> unwrapped.
static Layout drop_unit_modes(const Layout& L) {
  if (L.shape.is_int) return L.shape.value == 1 ? make_layout({1}, {0}) : L;
  std::vector<Layout> kept;
  for (int i = 0; i < rank(L.shape); ++i) {
    Layout sub = drop_unit_modes(sublayout(L, i));
    if (size(sub) > 1) kept.push_back(sub);
  }
  if (kept.empty()) return make_layout({1}, {0});
  if (kept.size() == 1) return kept[0];
  return concat(kept);
}

// First offset that neither B nor its complement produces (the complement fills the hole below
// each mode of B only in whole multiples of what lies beneath it); "none" is reported as INT64_MAX.
static int64_t first_offset_missed(const Layout& B) {
  std::vector<int64_t> S = leaves(B.shape), D = leaves(B.stride);
  std::vector<std::pair<int64_t, int64_t>> modes;  // (stride, extent)
  for (size_t k = 0; k < S.size(); ++k)
    if (S[k] > 1 && D[k] > 0) modes.push_back({D[k], S[k]});
  std::stable_sort(modes.begin(), modes.end(),
                   [](const std::pair<int64_t, int64_t>& a, const std::pair<int64_t, int64_t>& b) { return a.first < b.first; });
  int64_t cur = 1;
  for (const auto& m : modes) {
    if (m.first % cur != 0) return cur * (m.first / cur);
    cur = m.first * m.second;
  }
  return INT64_MAX;
}

Status logical_divide(const Layout& A, const Layout& B, Layout* R) {
  Layout Bstar;
  Status st = complement(B, size(A), &Bstar);     // complement of B with respect to |A|
  if (st != OK) return st;
  // (B, B*) must be surjective onto Z_|A| so that every element of A is kept (Sec. 3.5.2)
  if (first_offset_missed(B) < size(A)) return ERR_NOT_SURJECTIVE;
  Layout both;
  st = composition(A, concat({B, Bstar}), &both); // A o (B, B*)
  if (st != OK) return st;
  *R = concat({sublayout(both, 0), drop_unit_modes(sublayout(both, 1))});
  return OK;
}

static int tiler_rank(const Layout& tiler) { return tiler.shape.is_int ? 1 : rank(tiler.shape); }
static Layout tiler_mode(const Layout& tiler, int i) { return tiler.shape.is_int ? tiler : sublayout(tiler, i); }
static int layout_rank(const Layout& A) { return A.shape.is_int ? 1 : rank(A.shape); }
static Layout layout_mode(const Layout& A, int i) { return A.shape.is_int ? A : sublayout(A, i); }

Status logical_divide_bymode(const Layout& A, const Layout& tiler, Layout* R) {
  if (tiler_rank(tiler) > layout_rank(A)) return ERR_INVALID_ARG;
  std::vector<Layout> parts;
  for (int i = 0; i < layout_rank(A); ++i) {
    if (i < tiler_rank(tiler)) {
      Layout part;
      Status st = logical_divide(layout_mode(A, i), tiler_mode(tiler, i), &part);
      if (st != OK) return st;
      parts.push_back(part);
    } else {
      parts.push_back(layout_mode(A, i));
    }
  }
  *R = parts.size() == 1 ? parts[0] : concat(parts);
  return OK;
}

Status zipped_divide(const Layout& A, const Layout& tiler, Layout* R) {
  if (tiler_rank(tiler) > layout_rank(A)) return ERR_INVALID_ARG;
  std::vector<Layout> tiles, rests;
  for (int i = 0; i < layout_rank(A); ++i) {
    if (i < tiler_rank(tiler)) {
      Layout part;
      Status st = logical_divide(layout_mode(A, i), tiler_mode(tiler, i), &part);
      if (st != OK) return st;
      tiles.push_back(sublayout(part, 0));
      rests.push_back(sublayout(part, 1));
    } else {
      rests.push_back(layout_mode(A, i));   // untouched modes go whole into the rest
    }
  }
  Layout tile = tiles.size() == 1 ? tiles[0] : concat(tiles);
  Layout rest = rests.size() == 1 ? rests[0] : concat(rests);
  *R = concat({tile, rest});
  return OK;
}

// ===========================================================================
// Vectorisation (Sec. 3.4.2)
// ===========================================================================
int64_t max_common_vector_def(const Layout& A, const Layout& B) {
  Layout Ai = right_inverse(A), Bi = right_inverse(B);
  int64_t limit = std::min(size(Ai), size(Bi)), K = 0;
  while (K < limit && eval(Ai, K) == eval(Bi, K)) ++K;
  return K;
}

Status max_common_vector_alg(const Layout& A, const Layout& B, int64_t* K) {
  if (size(A) != size(B)) return ERR_SIZE_MISMATCH;   // stated for |A| = |B| (Sec. 3.4.2)
  Layout R;
  Status st = composition(A, right_inverse(B), &R);
  if (st != OK) return st;
  FlatModes f = coalesce_flat(R, false);
  *K = (f.d[0] == 1) ? f.s[0] : 1;
  return OK;
}

// ===========================================================================
// COPY (Sec. 2.6.1): dst(i) = src(i) for i = 0 .. size(dst)-1, in that order.
// ===========================================================================
Status copy_range(const void* src, const Layout& src_layout, void* dst, const Layout& dst_layout,
                  int elem_bytes, int64_t begin, int64_t end) {
  if (size(src_layout) != size(dst_layout)) return ERR_SIZE_MISMATCH;   // @pre size(src) == size(dst)
  if (elem_bytes < 1 || begin < 0 || end > size(dst_layout)) return ERR_INVALID_ARG;
  const unsigned char* s = static_cast<const unsigned char*>(src);
  unsigned char* d = static_cast<unsigned char*>(dst);
  for (int64_t i = begin; i < end; ++i) {
    int64_t so = eval(src_layout, i), dof = eval(dst_layout, i);   // T(i) = *(e + L(i)), Eq. tensor
    std::memcpy(d + dof * elem_bytes, s + so * elem_bytes, (size_t)elem_bytes);
  }
  return OK;
}

Status copy(const void* src, const Layout& src_layout, void* dst, const Layout& dst_layout, int elem_bytes) {
  if (size(src_layout) != size(dst_layout)) return ERR_SIZE_MISMATCH;
  return copy_range(src, src_layout, dst, dst_layout, elem_bytes, 0, size(dst_layout));
}

}  // namespace oracle
