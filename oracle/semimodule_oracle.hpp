// ORACLE — test infrastructure only (see layout_oracle.hpp).
//
// Layouts whose strides come from an integer-semimodule other than Z (Sec. 2.3.2 of "CuTe Layout
// Representation and Algebra"): scaled basis elements a*e_i of Z^(*,...,*) (the layout then yields a
// coordinate) and elements f_d of (Z, XOR, *) (a "swizzled" offset).  The inner product of Eq. innerprod
// is taken in the semimodule: scalar multiplication c * (a e_i) = (c a) e_i, c * f_d = f_{c d};
// addition component-wise, respectively bitwise XOR.  A layout uses one kind of stride throughout
// (zero strides aside), as every layout the paper prints does.
#pragma once
#include "layout_oracle.hpp"

namespace oracle {

struct Elem {
  enum Kind { INT = 0, COORD = 1, XOR = 2 } kind = INT;
  int64_t a = 0;     // integer, coefficient of e_basis, or the index d of f_d
  int basis = 0;     // COORD only
};

struct SLayout {
  HTuple shape;
  std::vector<Elem> stride;   // one element per leaf of the shape, left to right (S ~ D)
};

Status parse_slayout(const std::string& text, SLayout* out);   // "(4,(4,2)):(e1,(e0,6e1))", "(8,8):(f1,f9)", integers as usual
std::string to_string(const SLayout& L);
Elem::Kind kind_of(const SLayout& L);                          // INT when every stride is an integer
int codomain_rank(const SLayout& L);                           // COORD: 1 + largest basis index; otherwise 1
// L(i) on the extended domain; a COORD layout fills codomain_rank(L) components, the others one.
std::vector<int64_t> eval(const SLayout& L, int64_t i);
// A o B for an integer layout B (Sec. 3.3; Table TVLayoutExamples rows Swizzled and Coordinate).
// Admissibility depends on the shape of A and on B only; each mode of the result lies in one leaf of
// A and takes that leaf's stride scaled by its step inside the leaf ("Reductive case: Coordinate").
// With XOR strides that construction is A o B only while the modes of B that walk one leaf of A never meet in a bit;
// the result is compared with A(B(c)) on every coordinate of B and refused (ERR_NOT_SEGREGATED) when it differs.
Status composition(const SLayout& A, const Layout& B, SLayout* R);
// Sec. 3.2 for semimodule strides: unit modes go; neighbours merge when the second stride is the first
// scaled by the first extent AND the merged mode is the same function (always for e_i, never for f_d,
// where (i0 + s i1) d and i0 d XOR i1 s d differ as soon as bits meet).
SLayout coalesce(const SLayout& A);
// Right-inverse of a coordinate layout (Table rinv, rows with e_i strides): an integer layout on the
// largest box of coordinates starting at 0, axis by axis, with L(R(c)) = c.
Status right_inverse(const SLayout& A, Layout* R);
// Right-inverse of a layout with XOR strides (Table rinv, last row: "possible to define"; this reading).  Offsets add by XOR,
// so the inverse is sought among layouts that add by XOR too: R = (2,...,2):(f_x0, f_x1, ...) over the bits of k, where x_b is the
// SMALLEST integral coordinate of A with A(x_b) = 2^b, for b = 0, 1, ... up to the first power of two A does not reach.
// R(k) is then the XOR of the x_b of k's set bits.  Of these modes the longest prefix is kept for which R(k) is an integral
// coordinate of A and A(R(k)) = k for every k < |R| (XOR of coordinates need not be additive under A: an extent that is no
// power of two, a stride whose multiples inside a mode meet a carry); nothing left: 1:0.
Status xor_right_inverse(const SLayout& A, SLayout* R);

}  // namespace oracle
