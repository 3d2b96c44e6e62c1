// ORACLE — test infrastructure only (see semimodule_oracle.hpp).
#include "semimodule_oracle.hpp"

#include <algorithm>
#include <cctype>

namespace oracle {

namespace {
struct SParser {
  const std::string& s;
  size_t pos = 0;
  bool ok = true;
  explicit SParser(const std::string& t) : s(t) {}
  void skip() { while (pos < s.size() && std::isspace((unsigned char)s[pos])) ++pos; }
  bool number(int64_t* v) {
    size_t st = pos;
    while (pos < s.size() && std::isdigit((unsigned char)s[pos])) ++pos;
    if (pos == st || pos - st > 18) return false;
    *v = std::stoll(s.substr(st, pos - st));
    return true;
  }
  HTuple shape() {
    skip();
    if (pos < s.size() && s[pos] == '(') {
      ++pos;
      std::vector<HTuple> items;
      for (;;) {
        items.push_back(shape());
        if (!ok) return HTuple::Int(0);
        skip();
        if (pos < s.size() && s[pos] == ',') { ++pos; continue; }
        if (pos < s.size() && s[pos] == ')') { ++pos; break; }
        ok = false;
        return HTuple::Int(0);
      }
      return HTuple::Tup(items);
    }
    int64_t v;
    if (!number(&v)) { ok = false; return HTuple::Int(0); }
    return HTuple::Int(v);
  }
  // strides: same tree as the shape; leaves "12", "e1", "6e1", "f5"; the tree itself is returned as
  // an HTuple of leaf indices so that congruence with the shape can be checked
  HTuple strides(std::vector<Elem>* out) {
    skip();
    if (pos < s.size() && s[pos] == '(') {
      ++pos;
      std::vector<HTuple> items;
      for (;;) {
        items.push_back(strides(out));
        if (!ok) return HTuple::Int(0);
        skip();
        if (pos < s.size() && s[pos] == ',') { ++pos; continue; }
        if (pos < s.size() && s[pos] == ')') { ++pos; break; }
        ok = false;
        return HTuple::Int(0);
      }
      return HTuple::Tup(items);
    }
    Elem e;
    if (pos < s.size() && s[pos] == 'f') {
      ++pos;
      e.kind = Elem::XOR;
      if (!number(&e.a)) ok = false;
    } else {
      int64_t v = 1;
      const bool had_number = pos < s.size() && std::isdigit((unsigned char)s[pos]);
      if (had_number && !number(&v)) ok = false;
      if (pos < s.size() && s[pos] == 'e') {
        ++pos;
        int64_t b;
        e.kind = Elem::COORD;
        e.a = v;
        if (!number(&b) || b > 15) ok = false; else e.basis = (int)b;
      } else if (had_number) {
        e.kind = Elem::INT;
        e.a = v;
      } else {
        ok = false;
      }
    }
    out->push_back(e);
    return HTuple::Int((int64_t)out->size() - 1);
  }
};

std::string elem_text(const Elem& e) {
  if (e.kind == Elem::XOR) return "f" + std::to_string(e.a);
  if (e.kind == Elem::COORD) return (e.a == 1 ? std::string() : std::to_string(e.a)) + "e" + std::to_string(e.basis);
  return std::to_string(e.a);
}
std::string stride_text(const HTuple& shape, const std::vector<Elem>& d, size_t* next) {
  if (shape.is_int) return elem_text(d[(*next)++]);
  std::string r = "(";
  for (size_t k = 0; k < shape.items.size(); ++k) {
    if (k) r += ",";
    r += stride_text(shape.items[k], d, next);
  }
  return r + ")";
}
bool is_zero(const Elem& e) { return e.a == 0; }
}  // namespace

Elem::Kind kind_of(const SLayout& L) {
  for (const Elem& e : L.stride)
    if (!is_zero(e) && e.kind != Elem::INT) return e.kind;
  return Elem::INT;
}

Status parse_slayout(const std::string& text, SLayout* out) {
  SParser p(text);
  SLayout L;
  L.shape = p.shape();
  p.skip();
  if (!p.ok || p.pos >= text.size() || text[p.pos] != ':') return ERR_PARSE;
  ++p.pos;
  HTuple tree = p.strides(&L.stride);
  p.skip();
  if (!p.ok || p.pos != text.size()) return ERR_PARSE;
  if (!congruent(L.shape, tree)) return ERR_NOT_CONGRUENT;          // Sec. 2.3: S ~ D
  for (int64_t s : leaves(L.shape)) if (s < 1) return ERR_BAD_EXTENT;
  const Elem::Kind k = kind_of(L);
  for (const Elem& e : L.stride)
    if (!is_zero(e) && e.kind != k) return ERR_INVALID_ARG;         // one semimodule per layout
  *out = L;
  return OK;
}

std::string to_string(const SLayout& L) {
  size_t next = 0;
  return to_string(L.shape) + ":" + stride_text(L.shape, L.stride, &next);
}

int codomain_rank(const SLayout& L) {
  int r = 1;
  for (const Elem& e : L.stride)
    if (e.kind == Elem::COORD && !is_zero(e)) r = std::max(r, e.basis + 1);
  return r;
}

// Eq. innerprod in the semimodule: the natural coordinate of i (Sec. 2.2.2) against the strides.
std::vector<int64_t> eval(const SLayout& L, int64_t i) {
  const HTuple natural = idx2crd_natural(i, L.shape);
  const std::vector<int64_t> c = leaves(natural);
  const Elem::Kind k = kind_of(L);
  std::vector<int64_t> out((size_t)(k == Elem::COORD ? codomain_rank(L) : 1), 0);
  for (size_t j = 0; j < c.size(); ++j) {
    const Elem& e = L.stride[j];
    if (is_zero(e)) continue;
    if (k == Elem::COORD) out[(size_t)e.basis] += c[j] * e.a;       // c * (a e_i) = (c a) e_i, added component-wise
    else if (k == Elem::XOR) out[0] ^= c[j] * e.a;                  // c * f_d = f_{c d}, added by XOR
    else out[0] += c[j] * e.a;
  }
  return out;
}

Status composition(const SLayout& A, const Layout& B, SLayout* R) {
  // A = D_A o S_A, and B only addresses the integral coordinate of S_A.  Compose the integer layouts
  // P o B, where P has the shape of A and "place value" strides with a gap of 2 after every leaf
  // (P_0 = 1, P_{k+1} = 2 s_k P_k), so that neither P nor the result can merge modes across leaves of
  // A the way a compact layout would (the semimodule strides of two leaves do not continue each other).
  // Every mode of P o B then steps through one leaf k in units of P_k and carries (step / P_k) * d_k.
  const std::vector<int64_t> ext = leaves(A.shape);
  std::vector<int64_t> place(ext.size());
  int64_t run = 1;
  for (size_t k = 0; k < ext.size(); ++k) {
    place[k] = run;
    if (run > (int64_t)2e18 / (2 * ext[k])) return ERR_INVALID_ARG;
    run *= 2 * ext[k];
  }
  Layout P;
  P.shape = A.shape;
  {
    size_t next = 0;
    struct Fill {
      static HTuple go(const HTuple& s, const std::vector<int64_t>& pv, size_t* n) {
        if (s.is_int) return HTuple::Int(pv[(*n)++]);
        std::vector<HTuple> xs;
        for (const HTuple& x : s.items) xs.push_back(go(x, pv, n));
        return HTuple::Tup(xs);
      }
    };
    P.stride = Fill::go(A.shape, place, &next);
  }
  Layout PB;
  Status st = composition(P, B, &PB);
  if (st != OK) return st;
  SLayout out;
  out.shape = PB.shape;
  const std::vector<int64_t> rs = leaves(PB.shape), rd = leaves(PB.stride);
  for (size_t j = 0; j < rd.size(); ++j) {
    Elem e;
    if (rd[j] == 0 || rs[j] == 1) {
      out.stride.push_back(e);                                      // a mode that does not move: stride 0
      continue;
    }
    size_t k = ext.size() - 1;
    while (k > 0 && rd[j] < place[k]) --k;                          // the leaf of A this mode walks in
    if (rd[j] % place[k] != 0) return ERR_STRIDE_DIVISIBILITY;
    e = A.stride[k];
    e.a *= rd[j] / place[k];
    if (e.a == 0) e = Elem();
    out.stride.push_back(e);
  }
  if (kind_of(A) == Elem::XOR) {
    // With XOR strides the modes found above describe A o B only while, inside one leaf of A, the modes of B add up
    // without a carry: (c0 a0 + c1 a1) d and (c0 a0 d) xor (c1 a1 d) differ as soon as two terms meet in a bit.  Composition
    // is functional composition (Sec. 3.3), so the definition decides: R(c) = A(B(c)) on every coordinate of B, or no result.
    const int64_t n = size(B);
    if (n > (int64_t(1) << 24)) return ERR_INVALID_ARG;             // too large to enumerate here
    for (int64_t c = 0; c < n; ++c)
      if (eval(out, c) != eval(A, eval(B, c))) return ERR_NOT_SEGREGATED;
  }
  *R = out;
  return OK;
}

SLayout coalesce(const SLayout& A) {
  const std::vector<int64_t> ext = leaves(A.shape);
  const Elem::Kind kind = kind_of(A);
  std::vector<int64_t> s;
  std::vector<Elem> d;
  for (size_t k = 0; k < ext.size(); ++k) {
    if (ext[k] == 1) continue;                                      // a unit mode contributes nothing
    const Elem& e = A.stride[k];
    if (!s.empty() && kind != Elem::XOR) {
      const Elem& last = d.back();
      const bool same_axis = kind != Elem::COORD || is_zero(e) || is_zero(last) || e.basis == last.basis;
      if (same_axis && e.a == last.a * s.back() && (is_zero(e) == is_zero(last))) { s.back() *= ext[k]; continue; }
    }
    s.push_back(ext[k]);
    d.push_back(e);
  }
  SLayout R;
  if (s.empty()) { s.push_back(1); Elem z; d.push_back(z); }
  if (s.size() == 1) R.shape = HTuple::Int(s[0]);
  else { std::vector<HTuple> xs; for (int64_t v : s) xs.push_back(HTuple::Int(v)); R.shape = HTuple::Tup(xs); }
  R.stride = d;
  return R;
}

Status right_inverse(const SLayout& A, Layout* R) {
  if (kind_of(A) != Elem::COORD) return ERR_INVALID_ARG;
  const std::vector<int64_t> ext = leaves(A.shape);
  std::vector<int64_t> place(ext.size());
  int64_t run = 1;
  for (size_t k = 0; k < ext.size(); ++k) { place[k] = run; run *= ext[k]; }
  // per axis: chain the modes a e_i by growing coefficient while each continues the previous one
  // (coefficient = number of coordinates already covered); the chain's modes keep their place values
  std::vector<Layout> axes;
  const int rank = codomain_rank(A);
  for (int axis = 0; axis < rank; ++axis) {
    std::vector<size_t> ms;
    for (size_t k = 0; k < ext.size(); ++k)
      if (A.stride[k].kind == Elem::COORD && A.stride[k].a != 0 && A.stride[k].basis == axis && ext[k] > 1) ms.push_back(k);
    std::sort(ms.begin(), ms.end(), [&](size_t x, size_t y) { return A.stride[x].a < A.stride[y].a; });
    std::vector<int64_t> s, d;
    int64_t covered = 1;
    for (size_t k : ms) {
      if (A.stride[k].a != covered) break;
      s.push_back(ext[k]);
      d.push_back(place[k]);
      covered *= ext[k];
    }
    if (s.empty()) { s.push_back(1); d.push_back(0); }
    axes.push_back(coalesce(make_layout(s, d)));
  }
  *R = rank == 1 ? axes[0] : concat(axes);
  return OK;
}

Status xor_right_inverse(const SLayout& A, SLayout* R) {
  if (kind_of(A) != Elem::XOR) return ERR_INVALID_ARG;
  const int64_t n = size(A.shape);
  if (n > (int64_t(1) << 24)) return ERR_INVALID_ARG;   // the definition is applied by enumeration
  std::vector<int64_t> x;   // x[b]: smallest integral coordinate whose offset is 2^b
  for (int b = 0; b < 62; ++b) {
    int64_t found = -1;
    for (int64_t i = 0; i < n && found < 0; ++i)
      if (eval(A, i)[0] == (int64_t(1) << b)) found = i;
    if (found < 0) break;
    x.push_back(found);
  }
  // the longest prefix of them for which the defining property holds, coordinate by coordinate
  for (size_t j = x.size();; --j) {
    SLayout out;
    std::vector<HTuple> leaves_;
    if (j == 0) {
      out.shape = HTuple::Int(1);
      out.stride.push_back(Elem{});
    } else {
      for (size_t b = 0; b < j; ++b) {
        leaves_.push_back(HTuple::Int(2));
        Elem e;
        e.kind = Elem::XOR;
        e.a = x[b];
        out.stride.push_back(e);
      }
      out.shape = j == 1 ? leaves_[0] : HTuple::Tup(leaves_);
    }
    bool holds = true;
    for (int64_t k = 0; k < (int64_t(1) << j) && holds; ++k) {
      const int64_t c = eval(out, k)[0];
      holds = c >= 0 && c < n && eval(A, c)[0] == k;
    }
    if (holds) {
      *R = out;
      return OK;
    }
  }
}

}  // namespace oracle
