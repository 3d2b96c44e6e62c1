"""The oracle's generic GEMM (Sec. 2.6.2) against what fixes it from outside: the rows of the paper's
table of GEMM applications reduce to numpy matmul / einsum / a directly written convolution, closed
forms, the order of the k loop, the `+=`, and the preconditions."""
import numpy as np
import pytest

from oracle.pyoracle import OracleError


def _ints(n, seed, lo=-4, hi=5):
    # integer-valued doubles: every product and partial sum is exact, so equality is exact
    return np.random.default_rng(seed).integers(lo, hi, size=n).astype(np.float64)


def _strided(buf, shape, strides):
    return np.lib.stride_tricks.as_strided(buf, shape=shape, strides=[s * buf.itemsize for s in strides], writeable=False)


def test_blas_nt_tn_ntt_and_blis_rows_are_matmul(oracle):
    M, N, K = 7, 5, 6
    lda, ldb, ldc = 9, 8, 11      # leading dimensions larger than the extents: padding must be skipped
    # NT: A (M,K):(1,lda)  B (N,K):(1,ldb)  C (M,N):(1,ldc)
    A, B, C = _ints(lda * K, 1), _ints(ldb * K, 2), _ints(ldc * N, 3)
    C0 = C.copy()
    oracle.gemm(A, "(%d,%d):(1,%d)" % (M, K, lda), B, "(%d,%d):(1,%d)" % (N, K, ldb), C, "(%d,%d):(1,%d)" % (M, N, ldc))
    a, b = _strided(A, (M, K), (1, lda)), _strided(B, (N, K), (1, ldb))
    want = _strided(C0, (M, N), (1, ldc)) + a @ b.T
    assert (_strided(C, (M, N), (1, ldc)) == want).all()
    pad = np.ones(ldc * N, bool)
    pad[(np.arange(M)[:, None] + ldc * np.arange(N)[None, :]).ravel()] = False
    assert (C[pad] == C0[pad]).all()          # nothing outside the image of C's layout is touched
    # TN: A (M,K):(lda,1)  B (N,K):(ldb,1)
    lda, ldb = 8, 7
    A, B, C = _ints(lda * M, 4), _ints(ldb * N, 5), np.zeros(ldc * N)
    oracle.gemm(A, "(%d,%d):(%d,1)" % (M, K, lda), B, "(%d,%d):(%d,1)" % (N, K, ldb), C, "(%d,%d):(1,%d)" % (M, N, ldc))
    a, b = _strided(A, (M, K), (lda, 1)), _strided(B, (N, K), (ldb, 1))
    assert (_strided(C, (M, N), (1, ldc)) == a @ b.T).all()
    # NTT: the roles of the operands exchanged, C is (N,M):(1,ldc): the transposed product
    ldc = 6
    C = np.zeros(ldc * M)
    oracle.gemm(B, "(%d,%d):(%d,1)" % (N, K, ldb), A, "(%d,%d):(%d,1)" % (M, K, lda), C, "(%d,%d):(1,%d)" % (N, M, ldc))
    assert (_strided(C, (N, M), (1, ldc)) == b @ a.T).all()
    # BLIS: general strides in both modes of all three matrices
    dma, dka, dnb, dkb, dmc, dnc = 3, 23, 19, 2, 2, 15
    A, B, C = _ints(dma * M + dka * K, 6), _ints(dnb * N + dkb * K, 7), np.zeros(dmc * M + dnc * N)
    oracle.gemm(A, "(%d,%d):(%d,%d)" % (M, K, dma, dka), B, "(%d,%d):(%d,%d)" % (N, K, dnb, dkb), C,
                "(%d,%d):(%d,%d)" % (M, N, dmc, dnc))
    a, b = _strided(A, (M, K), (dma, dka)), _strided(B, (N, K), (dnb, dkb))
    assert (_strided(C, (M, N), (dmc, dnc)) == a @ b.T).all()


def test_gett_rows_are_einsum(oracle):
    # GETT row 1: A ((M1,M2),K):((1,W),X), B (N,K):(K,1), C ((M1,M2),N):((1,Y),Z)
    M1, M2, N, K = 3, 4, 5, 6
    W, X, Y, Z = 4, 17, 3, 13
    A, B = _ints(M1 + W * M2 + X * K, 1), _ints(N * K, 2)
    C = np.zeros(M1 + Y * M2 + Z * N)
    oracle.gemm(A, "((%d,%d),%d):((1,%d),%d)" % (M1, M2, K, W, X), B, "(%d,%d):(%d,1)" % (N, K, K), C,
                "((%d,%d),%d):((1,%d),%d)" % (M1, M2, N, Y, Z))
    a = _strided(A, (M1, M2, K), (1, W, X))
    b = B.reshape(N, K)
    want = np.einsum("abk,nk->abn", a, b)
    assert (_strided(C, (M1, M2, N), (1, Y, Z)) == want).all()
    # GETT row 2: A (M,(K1,K2)):(1,(W,X)), B (N,(K1,K2)):(Y,(1,Z)), C (M,N):(1,M)
    M, N, K1, K2 = 4, 3, 2, 5
    W, X, Y, Z = 4, 9, 2, 7
    A, B = _ints(M + W * K1 + X * K2, 3), _ints(Y * N + K1 + Z * K2, 4)
    C = np.zeros(M * N)
    oracle.gemm(A, "(%d,(%d,%d)):(1,(%d,%d))" % (M, K1, K2, W, X), B, "(%d,(%d,%d)):(%d,(1,%d))" % (N, K1, K2, Y, Z), C,
                "(%d,%d):(1,%d)" % (M, N, M))
    a = _strided(A, (M, K1, K2), (1, W, X))
    b = _strided(B, (N, K1, K2), (Y, 1, Z))
    assert (C.reshape(N, M).T == np.einsum("mkl,nkl->mn", a, b)).all()


def test_conv_row_is_a_directly_written_convolution(oracle):
    # CONV row: A (K,(C,R,S)) filters, B ((N,P,Q),(C,R,S)) the im2col view of an NHWC activation,
    # C (K,(N,P,Q)).  B's layout repeats strides (P and R both step by a row of the image).
    Nb, H, Wd, Cc, Kf, R, S = 2, 6, 5, 3, 4, 3, 2
    P, Q = H - R + 1, Wd - S + 1
    act = _ints(Nb * H * Wd * Cc, 1)                       # NHWC, compact row-major
    flt = _ints(Kf * Cc * R * S, 2)                        # K,C,R,S compact row-major
    sN, sH, sW, sC = H * Wd * Cc, Wd * Cc, Cc, 1
    la = "(%d,(%d,%d,%d)):(%d,(%d,%d,1))" % (Kf, Cc, R, S, Cc * R * S, R * S, S)
    lb = "((%d,%d,%d),(%d,%d,%d)):((%d,%d,%d),(%d,%d,%d))" % (Nb, P, Q, Cc, R, S, sN, sH, sW, sC, sH, sW)
    lc = "(%d,(%d,%d,%d)):(1,(%d,%d,%d))" % (Kf, Nb, P, Q, Kf * P * Q, Kf * Q, Kf)   # N,P,Q,K row-major
    out = np.zeros(Nb * P * Q * Kf)
    oracle.gemm(flt, la, act, lb, out, lc)
    x = act.reshape(Nb, H, Wd, Cc)
    w = flt.reshape(Kf, Cc, R, S)
    want = np.zeros((Nb, P, Q, Kf))
    for n in range(Nb):
        for p in range(P):
            for q in range(Q):
                patch = x[n, p:p + R, q:q + S, :]                      # R,S,C
                want[n, p, q, :] = np.einsum("rsc,kcrs->k", patch, w)
    assert (out.reshape(Nb, P, Q, Kf) == want).all()


def test_closed_forms(oracle):
    M, N, K = 6, 4, 9
    la, lb, lc = "(%d,%d):(1,%d)" % (M, K, M), "(%d,%d):(%d,1)" % (N, K, K), "(%d,%d):(%d,1)" % (M, N, N)
    ones_a, ones_b = np.ones(M * K), np.ones(N * K)
    C = np.full(M * N, 2.0)
    oracle.gemm(ones_a, la, ones_b, lb, C, lc)
    assert (C == 2.0 + K).all()
    # A(m,k) = m + 1, B(n,k) = k + 1  =>  C(m,n) = (m + 1) K (K + 1) / 2 for every n
    A = np.tile(np.arange(1, M + 1, dtype=np.float64), K)
    B = np.tile(np.arange(1, K + 1, dtype=np.float64), N)
    C = np.zeros(M * N)
    oracle.gemm(A, la, B, lb, C, lc)
    assert (C.reshape(M, N) == (np.arange(1, M + 1) * K * (K + 1) / 2)[:, None]).all()
    # B = rows of the identity (N = K): C = A
    I = np.eye(K).ravel()
    C = np.zeros(M * K)
    A = _ints(M * K, 3)
    oracle.gemm(A, la, I, "(%d,%d):(%d,1)" % (K, K, K), C, "(%d,%d):(1,%d)" % (M, K, M))
    assert (C == A).all()
    # a stride-0 mode of A broadcasts one column over k: C(m,n) = a(m) * sum_k B(n,k)
    a = _ints(M, 4)
    B = _ints(N * K, 5)
    C = np.zeros(M * N)
    oracle.gemm(a, "(%d,%d):(1,0)" % (M, K), B, lb, C, "(%d,%d):(1,%d)" % (M, N, M))
    assert (C.reshape(N, M) == np.outer(B.reshape(N, K).sum(1), a)).all()


def test_k_is_the_outermost_loop_and_updates_accumulate_in_order(oracle):
    # in fp64, ((0 + 1e16) + 1) - 1e16 = 0 while any order that adds 1 last (or first to -1e16 + 1e16) gives 1
    A = np.array([1e16, 1.0, -1e16])
    B = np.ones(3)
    C = np.zeros(1)
    oracle.gemm(A, "(1,3):(0,1)", B, "(1,3):(0,1)", C, "(1,1):(0,0)")
    assert C[0] == 0.0
    C = np.zeros(1)
    oracle.gemm(A[::-1].copy(), "(1,3):(0,1)", B, "(1,3):(0,1)", C, "(1,1):(0,0)")
    assert C[0] == 0.0      # ((0 - 1e16) + 1) + 1e16: the 1 is absorbed again
    C = np.zeros(1)
    oracle.gemm(np.array([1e16, -1e16, 1.0]), "(1,3):(0,1)", B, "(1,3):(0,1)", C, "(1,1):(0,0)")
    assert C[0] == 1.0
    # an aliasing C (stride 0 along m) receives every update of the loop nest: sum over m as well
    M, N, K = 3, 2, 4
    A, Bm = _ints(M * K, 1), _ints(N * K, 2)
    C = np.zeros(N)
    oracle.gemm(A, "(%d,%d):(1,%d)" % (M, K, M), Bm, "(%d,%d):(%d,1)" % (N, K, K), C, "(%d,%d):(0,1)" % (M, N))
    assert (C == (A.reshape(K, M).T @ Bm.reshape(N, K).T).sum(0)).all()


def test_plus_equals(oracle):
    M, N, K = 5, 4, 3
    la, lb, lc = "(%d,%d):(%d,1)" % (M, K, K), "(%d,%d):(1,%d)" % (N, K, N), "(%d,%d):(1,%d)" % (M, N, M)
    A, B, C0 = _ints(M * K, 1), _ints(N * K, 2), _ints(M * N, 3)
    prod = (A.reshape(M, K) @ B.reshape(K, N)).T.ravel()
    C = C0.copy()
    oracle.gemm(A, la, B, lb, C, lc)
    assert (C == C0 + prod).all()
    oracle.gemm(A, la, B, lb, C, lc)
    assert (C == C0 + 2 * prod).all()


def test_sampled_entries_equal_the_loop_nest(oracle):
    M, N, K = 9, 7, 11
    la = "((3,3),%d):((1,40),3)" % K
    lb = "(%d,(%d,1)):(%d,(1,0))" % (N, K, K + 2)
    lc = "(%d,%d):(%d,1)" % (M, N, N + 1)
    rng = np.random.default_rng(5)
    A, B, C0 = rng.standard_normal(200), rng.standard_normal(100), rng.standard_normal(M * (N + 1))
    C = C0.copy()
    oracle.gemm(A, la, B, lb, C, lc)
    ms, ns = np.meshgrid(np.arange(M), np.arange(N), indexing="ij")
    got = oracle.gemm_at(A, la, B, lb, C0, lc, ms.ravel(), ns.ravel())
    assert (got == C[(ms * (N + 1) + ns).ravel()]).all()           # same sums in the same order: bit-equal
    a = np.array([[A[(m % 3) + 40 * (m // 3) + 3 * k] for k in range(K)] for m in range(M)])
    b = np.array([[B[n * (K + 2) + k] for k in range(K)] for n in range(N)])
    np.testing.assert_allclose(got.reshape(M, N), C0.reshape(M, N + 1)[:, :N] + a @ b.T, rtol=1e-12, atol=1e-12)


def test_preconditions(oracle):
    a = np.zeros(64)
    with pytest.raises(OracleError) as e:
        oracle.gemm(a, "(4,3):(1,4)", a, "(5,3):(1,5)", a, "(3,5):(1,3)")      # M differs
    assert e.value.status_name == "SIZE_MISMATCH"
    with pytest.raises(OracleError) as e:
        oracle.gemm(a, "(4,3):(1,4)", a, "(5,3):(1,5)", a, "(4,6):(1,4)")      # N differs
    assert e.value.status_name == "SIZE_MISMATCH"
    with pytest.raises(OracleError) as e:
        oracle.gemm(a, "(4,3):(1,4)", a, "(5,2):(1,5)", a, "(4,5):(1,4)")      # K differs
    assert e.value.status_name == "SIZE_MISMATCH"
    with pytest.raises(OracleError) as e:
        oracle.gemm(a, "12:1", a, "(5,3):(1,5)", a, "(4,5):(1,4)")             # A is not a matrix
    assert e.value.status_name == "INVALID_ARG"
    assert oracle.gemm_sizes("((2,2),3):((1,2),4)", "(5,(3,1)):(1,(5,0))", "(4,5):(1,4)") == (4, 5, 3)


def test_batched_contraction_is_einsum(oracle):
    # Sec. 1: C(m,n,l) += A(m,k,l) B(n,k,l) with every mode possibly a multi-mode; compared with einsum on strided views
    M, N, K, L = 5, 4, 6, 3
    A, B = _ints(M * K * L + 7, 1), _ints(N * K * L, 2)
    C0 = _ints(M * N * L, 3)
    la = "(%d,%d,%d):(1,%d,%d)" % (M, K, L, M, M * K)              # column-major matrices, batch outermost
    lb = "(%d,%d,%d):(%d,1,%d)" % (N, K, L, K * L, K)              # batch interleaved between n and k
    lc = "(%d,%d,%d):(%d,%d,1)" % (M, N, L, L, M * L)              # batch innermost
    C = C0.copy()
    oracle.gemm(A, la, B, lb, C, lc)
    a, b = _strided(A, (M, K, L), (1, M, M * K)), _strided(B, (N, K, L), (K * L, 1, K))
    want = _strided(C0, (M, N, L), (L, M * L, 1)) + np.einsum("mkl,nkl->mnl", a, b)
    assert (_strided(C, (M, N, L), (L, M * L, 1)) == want).all()
    assert oracle.gemm_sizes(la, lb, lc) == (M, N, K, L)
    # a folded batch mode (L1,L2) and a stride-0 batch mode of B (one B for every l): a GETT with two batch indices
    L1, L2 = 2, 3
    A = _ints(M * K * L1 * L2, 4)
    Bm = _ints(N * K, 5)
    la = "(%d,%d,(%d,%d)):(%d,1,(%d,%d))" % (M, K, L1, L2, K, M * K * L2, M * K)
    lb = "(%d,%d,(%d,%d)):(%d,1,(0,0))" % (N, K, L1, L2, K)
    lc = "(%d,%d,(%d,%d)):(1,%d,(%d,%d))" % (M, N, L1, L2, M, M * N, M * N * L1)
    C = np.zeros(M * N * L1 * L2)
    oracle.gemm(A, la, Bm, lb, C, lc)
    a = _strided(A, (M, K, L1, L2), (K, 1, M * K * L2, M * K))
    want = np.einsum("mkab,nk->mnab", a, Bm.reshape(N, K))
    assert (_strided(C, (M, N, L1, L2), (1, M, M * N, M * N * L1)) == want).all()
    # sampled entries agree with the loop nest (same sums, same order)
    rng = np.random.default_rng(3)
    A, Bm, C0 = rng.standard_normal(A.size), rng.standard_normal(Bm.size), rng.standard_normal(C.size)
    C = C0.copy()
    oracle.gemm(A, la, Bm, lb, C, lc)
    ms, ns, ls = rng.integers(0, M, 40), rng.integers(0, N, 40), rng.integers(0, L1 * L2, 40)
    got = oracle.gemm_at(A, la, Bm, lb, C0, lc, ms, ns, ls)
    assert (got == C[ms + M * ns + M * N * ((ls % L1) + L1 * (ls // L1))]).all()


def test_batched_preconditions(oracle):
    a = np.zeros(256)
    with pytest.raises(OracleError) as e:
        oracle.gemm(a, "(4,3,2):(1,4,12)", a, "(5,3,3):(1,5,15)", a, "(4,5,2):(1,4,20)")      # L differs in B
    assert e.value.status_name == "SIZE_MISMATCH"
    with pytest.raises(OracleError) as e:
        oracle.gemm(a, "(4,3,2):(1,4,12)", a, "(5,3):(1,5)", a, "(4,5,2):(1,4,20)")            # ranks differ
    assert e.value.status_name == "INVALID_ARG"
    with pytest.raises(OracleError) as e:
        oracle.gemm(a, "(4,3,2,2):(1,4,12,24)", a, "(5,3,2,2):(1,5,15,30)", a, "(4,5,2,2):(1,4,20,40)")   # rank 4
    assert e.value.status_name == "INVALID_ARG"
