// ORACLE — test infrastructure only.  See gemm_oracle.hpp.
#include "gemm_oracle.hpp"

#include <vector>

namespace oracle {

static int64_t top_rank(const Layout& L) { return L.shape.is_int ? 1 : (int64_t)L.shape.items.size(); }

Status gemm_check(const Layout& A, const Layout& B, const Layout& C, int64_t* M, int64_t* N, int64_t* K) {
  for (const Layout* L : {&A, &B, &C}) {
    Status st = validate(*L);
    if (st != OK) return st;
    if (top_rank(*L) != 2) return ERR_INVALID_ARG;   // matrices: 2-D shapes (Sec. 2.6.2, Sec. 2.2.1)
  }
  const int64_t m = size(mode(A.shape, 0)), ka = size(mode(A.shape, 1));
  const int64_t n = size(mode(B.shape, 0)), kb = size(mode(B.shape, 1));
  if (m != size(mode(C.shape, 0))) return ERR_SIZE_MISMATCH;   // @pre M
  if (n != size(mode(C.shape, 1))) return ERR_SIZE_MISMATCH;   // @pre N
  if (ka != kb) return ERR_SIZE_MISMATCH;                      // @pre K
  *M = m;
  *N = n;
  *K = ka;
  return OK;
}

// offset of the 2-D coordinate (i, j): each entry is an integral coordinate of its (multi-)mode
static int64_t at(const Layout& L, int64_t i, int64_t j) {
  return eval_crd(L, HTuple::Tup({HTuple::Int(i), HTuple::Int(j)}));
}

Status gemm(const double* A, const Layout& LA, const double* B, const Layout& LB, double* C, const Layout& LC) {
  int64_t M, N, K;
  Status st = gemm_check(LA, LB, LC, &M, &N, &K);
  if (st != OK) return st;
  // the three layout functions tabulated over their whole domains (each entry is one evaluation of L)
  std::vector<int64_t> oa((size_t)(M * K)), ob((size_t)(N * K)), oc((size_t)(M * N));
  for (int64_t k = 0; k < K; ++k)
    for (int64_t m = 0; m < M; ++m) oa[(size_t)(k * M + m)] = at(LA, m, k);
  for (int64_t k = 0; k < K; ++k)
    for (int64_t n = 0; n < N; ++n) ob[(size_t)(k * N + n)] = at(LB, n, k);
  for (int64_t n = 0; n < N; ++n)
    for (int64_t m = 0; m < M; ++m) oc[(size_t)(n * M + m)] = at(LC, m, n);
  for (int64_t k = 0; k < K; ++k)
    for (int64_t n = 0; n < N; ++n)
      for (int64_t m = 0; m < M; ++m)
        C[oc[(size_t)(n * M + m)]] += A[oa[(size_t)(k * M + m)]] * B[ob[(size_t)(k * N + n)]];
  return OK;
}

Status gemm_at(const double* A, const Layout& LA, const double* B, const Layout& LB, const double* C, const Layout& LC,
               const int64_t* ms, const int64_t* ns, int64_t count, double* out) {
  int64_t M, N, K;
  Status st = gemm_check(LA, LB, LC, &M, &N, &K);
  if (st != OK) return st;
  for (int64_t j = 0; j < count; ++j) {
    const int64_t m = ms[j], n = ns[j];
    if (m < 0 || m >= M || n < 0 || n >= N) return ERR_INVALID_ARG;
    double acc = C[at(LC, m, n)];
    for (int64_t k = 0; k < K; ++k) acc += A[at(LA, m, k)] * B[at(LB, n, k)];
    out[j] = acc;
  }
  return OK;
}

}  // namespace oracle
