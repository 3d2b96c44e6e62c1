// ORACLE — test infrastructure only (see layout_oracle.hpp).
// C entry points (prefix oracle_) so that tests can reach the oracle through ctypes.
#include <cstring>
#include <string>

#include "layout_oracle.hpp"
#include "semimodule_oracle.hpp"
#include "gemm_oracle.hpp"

using oracle::Layout;

namespace {
int put_string(const std::string& s, char* buf, size_t cap, size_t* needed) {
  if (needed) *needed = s.size() + 1;
  if (buf && cap > 0) {
    size_t n = s.size() < cap - 1 ? s.size() : cap - 1;
    std::memcpy(buf, s.data(), n);
    buf[n] = 0;
  }
  return oracle::OK;
}
// Coordinates and bare shapes are written as HTuples of non-negative integers, e.g. "((0,1),(1,1))".
bool parse_htuple(const char* text, oracle::HTuple* out) {
  struct P {
    const char* s; size_t pos = 0; bool ok = true;
    void skip() { while (s[pos] == ' ') ++pos; }
    oracle::HTuple go() {
      skip();
      if (s[pos] == '(') {
        ++pos;
        std::vector<oracle::HTuple> items;
        for (;;) {
          items.push_back(go());
          if (!ok) return oracle::HTuple::Int(0);
          skip();
          if (s[pos] == ',') { ++pos; continue; }
          if (s[pos] == ')') { ++pos; break; }
          ok = false; return oracle::HTuple::Int(0);
        }
        return oracle::HTuple::Tup(items);
      }
      if (s[pos] == '_') { ++pos; return oracle::HTuple::Int(-1); }   // an unspecified position of a slice
      size_t st = pos;
      while (s[pos] >= '0' && s[pos] <= '9') ++pos;
      if (pos == st) { ok = false; return oracle::HTuple::Int(0); }
      return oracle::HTuple::Int(std::stoll(std::string(s + st, pos - st)));
    }
  } p{text};
  *out = p.go();
  p.skip();
  return p.ok && p.s[p.pos] == 0;
}
}  // namespace

extern "C" {

int oracle_layout_parse(const char* text, Layout** out) {
  if (!text || !out) return oracle::ERR_INVALID_ARG;
  Layout L;
  oracle::Status st = oracle::parse_layout(text, &L);
  if (st != oracle::OK) return st;
  *out = new Layout(L);
  return oracle::OK;
}
void oracle_layout_destroy(Layout* L) { delete L; }
int oracle_layout_to_string(const Layout* L, char* buf, size_t cap, size_t* needed) {
  return put_string(oracle::to_string(*L), buf, cap, needed);
}
int64_t oracle_layout_size(const Layout* L) { return oracle::size(*L); }
int64_t oracle_layout_cosize(const Layout* L) { return oracle::cosize(*L); }
int64_t oracle_layout_min_offset(const Layout* L) { return oracle::min_offset(*L); }
int oracle_layout_rank(const Layout* L) { return oracle::rank(L->shape); }
int oracle_layout_depth(const Layout* L) { return oracle::depth(L->shape); }
int64_t oracle_layout_eval(const Layout* L, int64_t i) { return oracle::eval(*L, i); }
void oracle_layout_eval_range(const Layout* L, int64_t begin, int64_t end, int64_t* out) {
  for (int64_t i = begin; i < end; ++i) out[i - begin] = oracle::eval(*L, i);
}
void oracle_layout_eval_many(const Layout* L, const int64_t* coords, int64_t n, int64_t* out) {
  for (int64_t k = 0; k < n; ++k) out[k] = oracle::eval(*L, coords[k]);
}
int oracle_layout_eval_crd(const Layout* L, const char* coord, int64_t* out) {
  oracle::HTuple c;
  if (!parse_htuple(coord, &c)) return oracle::ERR_PARSE;
  if (!oracle::weakly_congruent(c, L->shape)) return oracle::ERR_NOT_CONGRUENT;
  *out = oracle::eval_crd(*L, c);
  return oracle::OK;
}
int oracle_idx2crd_natural(const Layout* L, int64_t i, char* buf, size_t cap, size_t* needed) {
  return put_string(oracle::to_string(oracle::idx2crd_natural(i, L->shape)), buf, cap, needed);
}
// Coordinate of coordinate-set profile `coarse` (a shape that coarsens L's shape) for integral coordinate i.
int oracle_idx2crd_in(const char* coarse_shape, int64_t i, char* buf, size_t cap, size_t* needed) {
  oracle::HTuple s;
  if (!parse_htuple(coarse_shape, &s)) return oracle::ERR_PARSE;
  return put_string(oracle::to_string(oracle::idx2crd_natural(i, s)), buf, cap, needed);
}
int oracle_crd2idx(const Layout* L, const char* coord, int64_t* out) {
  oracle::HTuple c;
  if (!parse_htuple(coord, &c)) return oracle::ERR_PARSE;
  if (!oracle::weakly_congruent(c, L->shape)) return oracle::ERR_NOT_CONGRUENT;
  *out = oracle::crd2idx_h(oracle::crd2natural(c, L->shape), L->shape);
  return oracle::OK;
}
int oracle_shape_compatible(const char* p, const char* s) {
  oracle::HTuple a, b;
  if (!parse_htuple(p, &a) || !parse_htuple(s, &b)) return -1;
  return oracle::compatible(a, b) ? 1 : 0;
}
int oracle_congruent(const char* p, const char* s) {
  oracle::HTuple a, b;
  if (!parse_htuple(p, &a) || !parse_htuple(s, &b)) return -1;
  return oracle::congruent(a, b) ? 1 : 0;
}
int oracle_weakly_congruent(const char* p, const char* s) {
  oracle::HTuple a, b;
  if (!parse_htuple(p, &a) || !parse_htuple(s, &b)) return -1;
  return oracle::weakly_congruent(a, b) ? 1 : 0;
}

int oracle_layout_slice(const Layout* L, const char* coord, int64_t* offset, Layout** out) {
  oracle::HTuple c;
  if (!parse_htuple(coord, &c)) return oracle::ERR_PARSE;
  oracle::Slice sl;
  oracle::Status st = oracle::slice(*L, c, &sl);
  if (st != oracle::OK) return st;
  *offset = sl.offset;
  *out = new Layout(sl.rest);
  return oracle::OK;
}
int oracle_coalesce(const Layout* a, Layout** out) { *out = new Layout(oracle::coalesce(*a)); return oracle::OK; }
int oracle_coalesce_bymode(const Layout* a, Layout** out) { *out = new Layout(oracle::coalesce_bymode(*a)); return oracle::OK; }
// The statements of these operations are written for strides in N: negative strides are refused here, at the boundary.
#define REFUSE_NEGATIVE(L) do { if (oracle::has_negative_stride(*(L))) return oracle::ERR_NEGATIVE_STRIDE; } while (0)
int oracle_right_inverse(const Layout* a, Layout** out) {
  REFUSE_NEGATIVE(a);
  *out = new Layout(oracle::right_inverse(*a));
  return oracle::OK;
}

#define ORACLE_BINARY(name)                                             \
  int oracle_##name(const Layout* a, const Layout* b, Layout** out) {   \
    REFUSE_NEGATIVE(a);                                                 \
    REFUSE_NEGATIVE(b);                                                 \
    Layout r;                                                           \
    oracle::Status st = oracle::name(*a, *b, &r);                       \
    if (st != oracle::OK) return st;                                    \
    *out = new Layout(r);                                               \
    return oracle::OK;                                                  \
  }
ORACLE_BINARY(logical_product)
ORACLE_BINARY(blocked_product)
ORACLE_BINARY(raked_product)
ORACLE_BINARY(composition)
ORACLE_BINARY(composition_bymode)
ORACLE_BINARY(logical_divide)
ORACLE_BINARY(logical_divide_bymode)
ORACLE_BINARY(zipped_divide)
#undef ORACLE_BINARY

int oracle_left_inverse(const Layout* a, Layout** out) {
  REFUSE_NEGATIVE(a);
  Layout r;
  oracle::Status st = oracle::left_inverse(*a, &r);
  if (st != oracle::OK) return st;
  *out = new Layout(r);
  return oracle::OK;
}
int oracle_admissible(const Layout* a, const Layout* t) { return oracle::admissible(*a, *t) ? 1 : 0; }   // the statement holds for any integers
int oracle_complement(const Layout* a, int64_t cotarget, Layout** out) {
  REFUSE_NEGATIVE(a);
  Layout r;
  oracle::Status st = oracle::complement(*a, cotarget, &r);
  if (st != oracle::OK) return st;
  *out = new Layout(r);
  return oracle::OK;
}
int oracle_max_common_vector_def(const Layout* a, const Layout* b, int64_t* K) {
  REFUSE_NEGATIVE(a);
  REFUSE_NEGATIVE(b);
  *K = oracle::max_common_vector_def(*a, *b);
  return oracle::OK;
}
int oracle_max_common_vector(const Layout* a, const Layout* b, int64_t* K) {
  REFUSE_NEGATIVE(a);
  REFUSE_NEGATIVE(b);
  return oracle::max_common_vector_alg(*a, *b, K);
}

int oracle_copy(const void* src, const Layout* sl, void* dst, const Layout* dl, int elem_bytes) {
  return oracle::copy(src, *sl, dst, *dl, elem_bytes);
}
int oracle_copy_range(const void* src, const Layout* sl, void* dst, const Layout* dl, int elem_bytes,
                      int64_t begin, int64_t end) {
  return oracle::copy_range(src, *sl, dst, *dl, elem_bytes, begin, end);
}


// ---- semimodule strides (Sec. 2.3.2) ----
int oracle_slayout_parse(const char* text, oracle::SLayout** out) {
  if (!text || !out) return oracle::ERR_INVALID_ARG;
  oracle::SLayout L;
  oracle::Status st = oracle::parse_slayout(text, &L);
  if (st != oracle::OK) return st;
  *out = new oracle::SLayout(L);
  return oracle::OK;
}
void oracle_slayout_destroy(oracle::SLayout* L) { delete L; }
int oracle_slayout_to_string(const oracle::SLayout* L, char* buf, size_t cap, size_t* needed) { return put_string(oracle::to_string(*L), buf, cap, needed); }
int oracle_slayout_kind(const oracle::SLayout* L) { return (int)oracle::kind_of(*L); }
int oracle_slayout_codomain_rank(const oracle::SLayout* L) { return oracle::codomain_rank(*L); }
int64_t oracle_slayout_size(const oracle::SLayout* L) { return oracle::size(L->shape); }
int oracle_slayout_eval(const oracle::SLayout* L, int64_t i, int64_t* out, int cap) {
  std::vector<int64_t> v = oracle::eval(*L, i);
  if ((int)v.size() > cap) return oracle::ERR_INVALID_ARG;
  for (size_t k = 0; k < v.size(); ++k) out[k] = v[k];
  return oracle::OK;
}
int oracle_slayout_composition(const oracle::SLayout* a, const Layout* b, oracle::SLayout** out) {
  oracle::SLayout r;
  oracle::Status st = oracle::composition(*a, *b, &r);
  if (st != oracle::OK) return st;
  *out = new oracle::SLayout(r);
  return oracle::OK;
}
int oracle_slayout_coalesce(const oracle::SLayout* a, oracle::SLayout** out) { *out = new oracle::SLayout(oracle::coalesce(*a)); return oracle::OK; }
int oracle_slayout_right_inverse(const oracle::SLayout* a, Layout** out) {
  Layout r;
  oracle::Status st = oracle::right_inverse(*a, &r);
  if (st != oracle::OK) return st;
  *out = new Layout(r);
  return oracle::OK;
}
int oracle_slayout_xor_right_inverse(const oracle::SLayout* a, oracle::SLayout** out) {
  oracle::SLayout r;
  oracle::Status st = oracle::xor_right_inverse(*a, &r);
  if (st != oracle::OK) return st;
  *out = new oracle::SLayout(r);
  return oracle::OK;
}

// ---- GEMM (Sec. 2.6.2) ----
int oracle_gemm_check(const Layout* a, const Layout* b, const Layout* c, int64_t* M, int64_t* N, int64_t* K, int64_t* L) {
  return oracle::gemm_check(*a, *b, *c, M, N, K, L);
}
int oracle_gemm(const double* A, const Layout* la, const double* B, const Layout* lb, double* C, const Layout* lc) {
  return oracle::gemm(A, *la, B, *lb, C, *lc);
}
int oracle_gemm_at(const double* A, const Layout* la, const double* B, const Layout* lb, const double* C, const Layout* lc,
                   const int64_t* ms, const int64_t* ns, const int64_t* ls, int64_t count, double* out) {
  return oracle::gemm_at(A, *la, B, *lb, C, *lc, ms, ns, ls, count, out);
}

}  // extern "C"
