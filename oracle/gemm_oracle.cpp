// ORACLE — test infrastructure only.  See gemm_oracle.hpp.
#include "gemm_oracle.hpp"

#include <vector>

namespace oracle {

static int64_t top_rank(const Layout& L) { return L.shape.is_int ? 1 : (int64_t)L.shape.items.size(); }

Status gemm_check(const Layout& A, const Layout& B, const Layout& C, int64_t* M, int64_t* N, int64_t* K, int64_t* L) {
  for (const Layout* X : {&A, &B, &C}) {
    Status st = validate(*X);
    if (st != OK) return st;
  }
  const int64_t r = top_rank(A);
  if ((r != 2 && r != 3) || top_rank(B) != r || top_rank(C) != r) return ERR_INVALID_ARG;   // matrices, or all three batched
  const int64_t m = size(mode(A.shape, 0)), ka = size(mode(A.shape, 1));
  const int64_t n = size(mode(B.shape, 0)), kb = size(mode(B.shape, 1));
  if (m != size(mode(C.shape, 0))) return ERR_SIZE_MISMATCH;   // @pre M
  if (n != size(mode(C.shape, 1))) return ERR_SIZE_MISMATCH;   // @pre N
  if (ka != kb) return ERR_SIZE_MISMATCH;                      // @pre K
  int64_t l = 1;
  if (r == 3) {
    l = size(mode(A.shape, 2));
    if (l != size(mode(B.shape, 2)) || l != size(mode(C.shape, 2))) return ERR_SIZE_MISMATCH;   // the batch mode is shared
  }
  *M = m;
  *N = n;
  *K = ka;
  *L = l;
  return OK;
}

// offset of the coordinate (i, j) or (i, j, l): each entry is an integral coordinate of its (multi-)mode
static int64_t at(const Layout& X, int64_t i, int64_t j, int64_t l) {
  if (top_rank(X) == 2) return eval_crd(X, HTuple::Tup({HTuple::Int(i), HTuple::Int(j)}));
  return eval_crd(X, HTuple::Tup({HTuple::Int(i), HTuple::Int(j), HTuple::Int(l)}));
}

Status gemm(const double* A, const Layout& LA, const double* B, const Layout& LB, double* C, const Layout& LC) {
  int64_t M, N, K, L;
  Status st = gemm_check(LA, LB, LC, &M, &N, &K, &L);
  if (st != OK) return st;
  const bool batched = top_rank(LA) == 3;
  // the three layout functions tabulated over the domain of one batch entry (each table entry is one evaluation of L)
  std::vector<int64_t> oa((size_t)(M * K)), ob((size_t)(N * K)), oc((size_t)(M * N));
  for (int64_t l = 0; l < L; ++l) {
    for (int64_t k = 0; k < K; ++k)
      for (int64_t m = 0; m < M; ++m) oa[(size_t)(k * M + m)] = at(LA, m, k, l);
    for (int64_t k = 0; k < K; ++k)
      for (int64_t n = 0; n < N; ++n) ob[(size_t)(k * N + n)] = at(LB, n, k, l);
    for (int64_t n = 0; n < N; ++n)
      for (int64_t m = 0; m < M; ++m) oc[(size_t)(n * M + m)] = at(LC, m, n, l);
    if (!batched) {
      // Sec. 2.6.2: k outermost, then n, then m
      for (int64_t k = 0; k < K; ++k)
        for (int64_t n = 0; n < N; ++n)
          for (int64_t m = 0; m < M; ++m)
            C[oc[(size_t)(n * M + m)]] += A[oa[(size_t)(k * M + m)]] * B[ob[(size_t)(k * N + n)]];
    } else {
      // Sec. 1 (this l of the outermost loop): m, then n, then k innermost
      for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n)
          for (int64_t k = 0; k < K; ++k)
            C[oc[(size_t)(n * M + m)]] += A[oa[(size_t)(k * M + m)]] * B[ob[(size_t)(k * N + n)]];
    }
  }
  return OK;
}

Status gemm_at(const double* A, const Layout& LA, const double* B, const Layout& LB, const double* C, const Layout& LC,
               const int64_t* ms, const int64_t* ns, const int64_t* ls, int64_t count, double* out) {
  int64_t M, N, K, L;
  Status st = gemm_check(LA, LB, LC, &M, &N, &K, &L);
  if (st != OK) return st;
  for (int64_t j = 0; j < count; ++j) {
    const int64_t m = ms[j], n = ns[j], l = ls ? ls[j] : 0;
    if (m < 0 || m >= M || n < 0 || n >= N || l < 0 || l >= L) return ERR_INVALID_ARG;
    double acc = C[at(LC, m, n, l)];
    for (int64_t k = 0; k < K; ++k) acc += A[at(LA, m, k, l)] * B[at(LB, n, k, l)];
    out[j] = acc;
  }
  return OK;
}

}  // namespace oracle
