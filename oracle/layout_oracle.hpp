// ORACLE — test infrastructure only.
//
// A plain, slow, obviously-correct CPU statement of what the layout method of
// "CuTe Layout Representation and Algebra" computes: hierarchical tuples, the
// layout function, the layout algebra and the element-by-element COPY.
// Nothing here is tuned, blocked, fused or reordered beyond what the paper's
// definitions state.  Only tests, the smoke check and the benchmark's CPU
// baseline may use it; the GPU library shares no code with it.
//
// Every function cites the section / equation / table of the paper it follows.
// Where the paper leaves a choice open, the reading taken is stated at the
// function and its *printed form* for inputs the paper never prints is
// "parity unpinned" (the functional behaviour is pinned by the invariants).
#pragma once
#include <cstdint>
#include <string>
#include <vector>

namespace oracle {

// ---- HTuple (Sec. 2.1): an integer or a tuple of HTuples ------------------
struct HTuple {
  bool is_int = true;
  int64_t value = 0;              // when is_int
  std::vector<HTuple> items;      // when !is_int
  static HTuple Int(int64_t v) { HTuple t; t.is_int = true; t.value = v; return t; }
  static HTuple Tup(std::vector<HTuple> xs) { HTuple t; t.is_int = false; t.items = std::move(xs); return t; }
};

int rank(const HTuple& x);                       // Sec. 2.1, Def. HTuple: tuple length, else 1
int depth(const HTuple& x);                      // Sec. 2.1, Def. HTuple
const HTuple& mode(const HTuple& x, int i);      // access X_i (an int is its own mode 0)
bool congruent(const HTuple& p, const HTuple& s);        // Sec. 2.1, Def. congruence
bool weakly_congruent(const HTuple& p, const HTuple& s); // Sec. 2.1, Def. weak congruence
bool compatible(const HTuple& p, const HTuple& s);       // Sec. 2.2.1, Def. compatibility (shapes)
int64_t size(const HTuple& shape);               // Sec. 2.2, Def. shape: product of leaves
std::vector<int64_t> leaves(const HTuple& x);    // left-to-right leaves (colexicographic order, Sec. 2.2.2)
std::string to_string(const HTuple& x);
bool equal(const HTuple& a, const HTuple& b);

// idx2crd / crd2idx over the top-level modes of a shape (Eq. idx2crd, Eq. crd2idx).
// idx2crd is defined for every integer: the last entry is not reduced.
std::vector<int64_t> idx2crd(int64_t i, const HTuple& shape);
int64_t crd2idx(const std::vector<int64_t>& c, const HTuple& shape);
// Repeated application down the hierarchy (Sec. 2.2.2): integral coordinate ->
// natural coordinate congruent with the shape.
HTuple idx2crd_natural(int64_t i, const HTuple& shape);
// Any coordinate weakly congruent with the shape -> natural coordinate.
HTuple crd2natural(const HTuple& c, const HTuple& shape);
// Natural (or any weakly congruent) coordinate -> integral coordinate.
int64_t crd2idx_h(const HTuple& c, const HTuple& shape);
// inner_product of a coordinate with a congruent stride (Eq. innerprod).
int64_t inner_product(const HTuple& c, const HTuple& d);

// ---- Layout (Sec. 2.4): L = D o S with S ~ D ------------------------------
struct Layout {
  HTuple shape, stride;
};

enum Status {                 // numeric values mirror the GPU library's status codes on purpose
  OK = 0,
  ERR_INVALID_ARG = 1,
  ERR_PARSE = 2,
  ERR_NOT_CONGRUENT = 3,
  ERR_BAD_EXTENT = 4,
  ERR_NEGATIVE_STRIDE = 5,
  ERR_SIZE_MISMATCH = 6,
  ERR_STRIDE_DIVISIBILITY = 7,
  ERR_SHAPE_DIVISIBILITY = 8,
  ERR_NOT_SEGREGATED = 9,
  ERR_NOT_INJECTIVE = 10,
  ERR_NOT_SURJECTIVE = 11,
};

Status parse_layout(const std::string& text, Layout* out);  // "S:D" as the paper prints layouts (Sec. 2.4.1)
Status validate(const Layout& L);                           // S ~ D, extents >= 1, strides >= 0
std::string to_string(const Layout& L);
Layout make_layout(const std::vector<int64_t>& s, const std::vector<int64_t>& d); // flat; rank 1 -> "s:d"
Layout sublayout(const Layout& L, int i);                   // L_i = S_i : D_i (Sec. 2.4.1)
Layout concat(const std::vector<Layout>& parts);            // (L_0, L_1, ...) (Eq. concat)
int64_t size(const Layout& L);
int64_t cosize(const Layout& L);                            // max of the image + 1 (Sec. 2.4.1, image)
int64_t min_offset(const Layout& L);                        // min of the image: 0 unless a stride is negative
bool has_negative_stride(const Layout& L);

// L(c) for an integral coordinate; every integer is accepted (extended domain,
// Sec. 2.4.1): only the last mode at each level stays unreduced.
int64_t eval(const Layout& L, int64_t i);
// L(c) for any coordinate weakly congruent with the shape.
int64_t eval_crd(const Layout& L, const HTuple& c);

// Slicing (Sec. 2.5.1): a coordinate with unspecified positions (here: value -1 leaves, "_" in text)
// evaluates the specified part into an offset and leaves the sublayout of the unspecified modes.
struct Slice { int64_t offset; Layout rest; };
Status slice(const Layout& L, const HTuple& coord_with_holes, Slice* out);

// ---- Algebra (Sec. 3) ------------------------------------------------------
Layout coalesce(const Layout& A);                           // Sec. 3.2
Layout coalesce_bymode(const Layout& A);                    // Sec. 3.2 with the combinator of Eq. layout_combinator
Status composition(const Layout& A, const Layout& B, Layout* R);        // Sec. 3.3
Status composition_bymode(const Layout& A, const Layout& tiler, Layout* R); // Sec. 3.3.5
Status complement(const Layout& A, int64_t cotarget, Layout* R);        // Sec. 3.5; cotarget 0 = cosize(A)
Layout right_inverse(const Layout& A);                      // Sec. 3.4.1
Status left_inverse(const Layout& A, Layout* R);            // Sec. 3.4.3: A(R(A(k))) = A(k)
// Sec. 3.4.3, application: does the image of the data layout A hold every offset the instruction layout T produces?
// The statement itself, "for all i in Z_|T| there is c in Z(A) with T(i) = A(c)", by enumeration of both.
bool admissible(const Layout& A, const Layout& T);
Status logical_product(const Layout& A, const Layout& B, Layout* R);    // Sec. 3.5.1: (A, A* o B)
Status blocked_product(const Layout& A, const Layout& B, Layout* R);    // Sec. 3.5.1 "Related products": ((A_0,B'_0),(A_1,B'_1),...)
Status raked_product(const Layout& A, const Layout& B, Layout* R);      // Sec. 3.5.1 "Related products": ((B'_0,A_0),(B'_1,A_1),...)
Status logical_divide(const Layout& A, const Layout& B, Layout* R);     // Sec. 3.5.2: A o (B, B*_{|A|})
Status logical_divide_bymode(const Layout& A, const Layout& tiler, Layout* R); // Sec. 3.5.2 "Related divides"
Status zipped_divide(const Layout& A, const Layout& tiler, Layout* R);  // Sec. 3.5.2 "Related divides"
// Largest K with A^(k) == B^(k) for all k < K, by the literal definition (Sec. 3.4.2).
int64_t max_common_vector_def(const Layout& A, const Layout& B);
// The same K by the paper's algebraic route: stride-1 head of coalesce(A o B^) (Sec. 3.4.2).
Status max_common_vector_alg(const Layout& A, const Layout& B, int64_t* K);

// ---- COPY (Sec. 2.6.1) -----------------------------------------------------
// for i in [0, size(dst)): dst(i) = src(i), elements moved as opaque
// elem_bytes-wide bit patterns through pointer accessors (Sec. 2.5).
Status copy(const void* src, const Layout& src_layout, void* dst, const Layout& dst_layout, int elem_bytes);
// The same loop restricted to i in [begin, end): used to time a bounded sample.
Status copy_range(const void* src, const Layout& src_layout, void* dst, const Layout& dst_layout,
                  int elem_bytes, int64_t begin, int64_t end);

}  // namespace oracle
