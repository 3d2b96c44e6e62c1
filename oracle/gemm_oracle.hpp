// ORACLE — test infrastructure only.
//
// The generic GEMM of "CuTe Layout Representation and Algebra", Sec. 2.6.2: three tensors given as a
// pointer and a rank-2 layout each — A over (M,K), B over (N,K), C over (M,N), every mode possibly a
// multi-mode — and the triple loop C(m,n) += A(m,k) * B(n,k) with k outermost, then n, then m.
// Arithmetic is fp64 (the paper leaves the element types open); nothing is blocked, fused or
// reordered.  Shares no code with the GPU library.
#pragma once
#include <cstdint>

#include "layout_oracle.hpp"

namespace oracle {

// Preconditions of Sec. 2.6.2 (sizes of the top-level modes): size<0>(A) == size<0>(C),
// size<0>(B) == size<1>(C), size<1>(A) == size<1>(B); each layout must have rank 2 — or all three rank 3 for
// the batched form of Sec. 1 (canonical contraction C_mnl = A_mkl B_nkl), whose third modes must agree in size.
// *L is 1 for rank 2.
Status gemm_check(const Layout& A, const Layout& B, const Layout& C, int64_t* M, int64_t* N, int64_t* K, int64_t* L);

// The loop nest of Sec. 2.6.2 over buffers of doubles; T(m,k) = *(e + L(m,k)) with the 2-D coordinate
// evaluated through the hierarchy (Eq. tensor, Sec. 2.4).  C is read and written in place.
// Rank-3 layouts run the batched loop nest of Sec. 1 instead: l outermost, then m, n, and k innermost.
Status gemm(const double* A, const Layout& LA, const double* B, const Layout& LB, double* C, const Layout& LC);

// The same sum for chosen entries of C only: out[j] = C(m_j, n_j, l_j) + sum_k A(m_j,k,l_j) * B(n_j,k,l_j), k ascending.
// C is not modified.  Used where the whole loop nest is out of reach (sampled checks at full size).  ls may be
// null (all zero); it must be for rank-2 layouts.
Status gemm_at(const double* A, const Layout& LA, const double* B, const Layout& LB, const double* C, const Layout& LC,
               const int64_t* ms, const int64_t* ns, const int64_t* ls, int64_t count, double* out);

}  // namespace oracle
