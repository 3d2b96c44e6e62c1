#include "layout.hpp"

#include <cctype>

namespace lc {

Layout Layout::flat(const Modes& m) {
  Layout L;
  if (m.size() == 1) {
    L.profile = {0};
  } else {
    L.profile.assign(m.size() + 1, 0);
    L.profile[0] = (int32_t)m.size();
  }
  L.leaves = m;
  return L;
}

Layout Layout::tuple(const std::vector<Layout>& parts) {
  Layout L;
  L.profile.push_back((int32_t)parts.size());
  for (const Layout& p : parts) {
    L.profile.insert(L.profile.end(), p.profile.begin(), p.profile.end());
    L.leaves.insert(L.leaves.end(), p.leaves.begin(), p.leaves.end());
  }
  return L;
}

// Walks the sub-tree rooted at profile[pos]; returns the position after it and counts its leaves.
static size_t skip_subtree(const std::vector<int32_t>& prof, size_t pos, size_t* n_leaves) {
  int32_t k = prof[pos++];
  if (k == 0) { ++*n_leaves; return pos; }
  for (int32_t c = 0; c < k; ++c) pos = skip_subtree(prof, pos, n_leaves);
  return pos;
}

static int depth_at(const std::vector<int32_t>& prof, size_t* pos) {
  int32_t k = prof[(*pos)++];
  if (k == 0) return 0;
  int d = 0;
  for (int32_t c = 0; c < k; ++c) { int dc = depth_at(prof, pos); if (dc > d) d = dc; }
  return d + 1;
}

int Layout::depth() const {
  size_t pos = 0;
  return depth_at(profile, &pos);
}

int64_t Layout::size() const {
  int64_t n = 1;
  for (const Mode& m : leaves) n *= m.extent;
  return n;
}

int64_t Layout::cosize() const {
  int64_t top = 0;
  for (const Mode& m : leaves) if (m.stride > 0) top += (m.extent - 1) * m.stride;
  return top + 1;
}

int64_t Layout::min_offset() const {
  int64_t low = 0;
  for (const Mode& m : leaves) if (m.stride < 0) low += (m.extent - 1) * m.stride;
  return low;
}

bool Layout::has_negative_stride() const {
  for (const Mode& m : leaves) if (m.stride < 0) return true;
  return false;
}

Layout Layout::mode(int i) const {
  if (is_leaf()) return *this;
  size_t pos = 1, leaf0 = 0;
  for (int c = 0; c < i; ++c) pos = skip_subtree(profile, pos, &leaf0);
  size_t nl = 0;
  size_t end = skip_subtree(profile, pos, &nl);
  Layout R;
  R.profile.assign(profile.begin() + (long)pos, profile.begin() + (long)end);
  R.leaves.assign(leaves.begin() + (long)leaf0, leaves.begin() + (long)(leaf0 + nl));
  return R;
}

static void print_at(const Layout& L, size_t* pos, size_t* leaf, bool strides, std::string* out) {
  int32_t k = L.profile[(*pos)++];
  if (k == 0) {
    const Mode& m = L.leaves[(*leaf)++];
    *out += std::to_string(strides ? m.stride : m.extent);
    return;
  }
  *out += '(';
  for (int32_t c = 0; c < k; ++c) {
    if (c) *out += ',';
    print_at(L, pos, leaf, strides, out);
  }
  *out += ')';
}

std::string Layout::str() const {
  std::string s;
  size_t pos = 0, leaf = 0;
  print_at(*this, &pos, &leaf, false, &s);
  s += ':';
  pos = leaf = 0;
  print_at(*this, &pos, &leaf, true, &s);
  return s;
}

// L(i): the integral coordinate is split colexicographically over the leaves (Eq. idx2crd applied
// at every level is the same as splitting over the leaves left to right, Sec. 2.2.2); only the very
// last leaf keeps an unreduced coordinate, which is what defines L beyond |L| (Sec. 2.4.1).
int64_t Layout::operator()(int64_t i) const {
  int64_t off = 0;
  size_t n = leaves.size();
  for (size_t k = 0; k + 1 < n; ++k) {
    off += (i % leaves[k].extent) * leaves[k].stride;
    i /= leaves[k].extent;
  }
  return off + i * leaves[n - 1].stride;
}

namespace {
struct Cursor {
  const char* p;
  bool ok = true;
  void ws() { while (*p && std::isspace((unsigned char)*p)) ++p; }
};

// Parses one HTuple into a pre-order profile and the list of its integers.
void parse_tuple(Cursor* c, std::vector<int32_t>* prof, std::vector<int64_t>* vals) {
  c->ws();
  if (*c->p == '(') {
    ++c->p;
    size_t slot = prof->size();
    prof->push_back(0);
    int32_t k = 0;
    for (;;) {
      parse_tuple(c, prof, vals);
      if (!c->ok) return;
      ++k;
      c->ws();
      if (*c->p == ',') { ++c->p; continue; }
      if (*c->p == ')') { ++c->p; break; }
      c->ok = false;
      return;
    }
    (*prof)[slot] = k;
    return;
  }
  bool neg = false;
  if (*c->p == '-') { neg = true; ++c->p; }
  if (!std::isdigit((unsigned char)*c->p)) { c->ok = false; return; }
  int64_t v = 0;
  int digits = 0;
  while (std::isdigit((unsigned char)*c->p)) {
    v = v * 10 + (*c->p - '0');
    ++c->p;
    if (++digits > 18) { c->ok = false; return; }
  }
  prof->push_back(0);
  vals->push_back(neg ? -v : v);
}
}  // namespace

lc_status_t parse(const char* text, Layout* out) {
  Cursor c{text};
  std::vector<int32_t> sp, dp;
  std::vector<int64_t> sv, dv;
  parse_tuple(&c, &sp, &sv);
  c.ws();
  if (!c.ok || *c.p != ':') return LC_ERR_PARSE;
  ++c.p;
  parse_tuple(&c, &dp, &dv);
  c.ws();
  if (!c.ok || *c.p != 0) return LC_ERR_PARSE;
  if (sp != dp) return LC_ERR_NOT_CONGRUENT;
  Layout L;
  L.profile = sp;
  for (size_t k = 0; k < sv.size(); ++k) L.leaves.push_back({sv[k], dv[k]});
  lc_status_t st = validate(L);
  if (st != LC_OK) return st;
  *out = L;
  return LC_OK;
}

lc_status_t validate(const Layout& L) {
  if (L.profile.empty() || L.leaves.empty()) return LC_ERR_INVALID_ARG;
  size_t nl = 0;
  if (skip_subtree(L.profile, 0, &nl) != L.profile.size() || nl != L.leaves.size()) return LC_ERR_NOT_CONGRUENT;
  // sizes and offsets are computed in int64: keep size and cosize below 2^62
  const long double limit = 4.0e18L;
  long double size = 1.0L, top = 0.0L;
  for (const Mode& m : L.leaves) {
    if (m.extent < 1) return LC_ERR_BAD_EXTENT;
    // strides of either sign (Sec. 2.3.2: Z is an integer-semimodule); the operations stated for strides in N refuse them
    size *= (long double)m.extent;
    top += (long double)(m.extent - 1) * (long double)(m.stride < 0 ? -m.stride : m.stride);
    if (size > limit || top > limit) return LC_ERR_TOO_LARGE;
  }
  if (L.leaves.size() > 64 || L.profile.size() > 256) return LC_ERR_TOO_LARGE;
  return LC_OK;
}

}  // namespace lc
