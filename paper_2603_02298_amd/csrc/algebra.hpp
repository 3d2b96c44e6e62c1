// Layout algebra of the library (host): coalesce, composition, complement, right-inverse,
// logical / zipped divide, common vector width.  "CuTe Layout Representation and Algebra", Sec. 3.
#pragma once
#include "layout.hpp"

namespace lc {

// Sec. 3.2.  keep_last_unit: do not drop a trailing extent-1 mode (its stride still defines the
// layout on the extended domain; composition needs that for complements such as "(2,1):(1,80)").
Modes coalesce_modes(const Modes& in, bool keep_last_unit = false);
Layout coalesce(const Layout& a);
Layout coalesce_bymode(const Layout& a);

lc_status_t composition(const Layout& a, const Layout& b, Layout* out);                 // Sec. 3.3
lc_status_t composition_bymode(const Layout& a, const Layout& tiler, Layout* out);      // Sec. 3.3.5
lc_status_t complement(const Layout& a, int64_t cotarget, Layout* out);                 // Sec. 3.5
Layout right_inverse(const Layout& a);                                                  // Sec. 3.4.1
lc_status_t left_inverse(const Layout& a, Layout* out);                                 // Sec. 3.4.3
// Sec. 3.4.3, application: is every offset T(i) in the image of A?  Decided the paper's way, A(A^†(T(i))) = T(i) with
// A^†(T(i)) inside A's domain; *where = A^† o T (instruction coordinate -> data coordinate) when that composition exists,
// else a layout of size 0 modes ("1:0") and *has_where = false.
lc_status_t admissible(const Layout& a, const Layout& t, bool* yes, Layout* where, bool* has_where);
lc_status_t logical_product(const Layout& a, const Layout& b, Layout* out);             // Sec. 3.5.1
lc_status_t blocked_product(const Layout& a, const Layout& b, Layout* out);             // Sec. 3.5.1
lc_status_t raked_product(const Layout& a, const Layout& b, Layout* out);               // Sec. 3.5.1
lc_status_t logical_divide(const Layout& a, const Layout& b, Layout* out);              // Sec. 3.5.2
lc_status_t logical_divide_bymode(const Layout& a, const Layout& tiler, Layout* out);   // Sec. 3.5.2
lc_status_t zipped_divide(const Layout& a, const Layout& tiler, Layout* out);           // Sec. 3.5.2
// Sec. 2.5.1: coordinate text with "_" at the unspecified positions -> offset of the specified part
// and the sublayout of the unspecified modes.
lc_status_t slice(const Layout& a, const char* coord, int64_t* offset, Layout* out);
lc_status_t max_common_vector(const Layout& a, const Layout& b, int64_t* K);            // Sec. 3.4.2

}  // namespace lc
