"""The oracle's COPY against library routines it reduces to in special cases (numpy), the
counting-iterator routing check, and the paper's table of COPY applications."""
import numpy as np
import pytest

from conftest import golden_lines


def _rand(n, dtype, seed):
    rng = np.random.default_rng(seed)
    if np.dtype(dtype).itemsize == 2:
        return rng.integers(0, 2 ** 16, size=n, dtype=np.uint16)
    return rng.integers(0, 2 ** 32, size=n, dtype=np.uint32)


def test_identical_layouts_is_memcpy(oracle):
    src = _rand(96, np.uint32, 1)
    for text in ["96:1", "(8,12):(1,8)", "((2,4),(3,4)):((1,2),(8,24))"]:
        dst = np.zeros(96, np.uint32)
        oracle.copy(src, text, dst, text)
        assert (dst == src).all()


def test_transpose_is_numpy_transpose(oracle):
    # (M,N):(1,M) -> (M,N):(N,1): column-major source, row-major destination of the same logical matrix
    for M, N, dt in [(8, 3, np.uint32), (33, 17, np.uint16), (64, 64, np.uint32)]:
        src = _rand(M * N, dt, M)
        dst = np.zeros(M * N, dt)
        oracle.copy(src, "(%d,%d):(1,%d)" % (M, N, M), dst, "(%d,%d):(%d,1)" % (M, N, N))
        logical = src.reshape(N, M).T            # logical[m, n] = src[m + M n]
        assert (dst.reshape(M, N) == logical).all()


def test_nchw_to_nhwc_is_numpy_transpose(oracle):
    N, C, H, W = 2, 3, 4, 5
    src = _rand(N * C * H * W, np.uint32, 3)
    dst = np.zeros_like(src)
    # the fifth workload's layouts at a small size: logical shape (N,C,H,W)
    sl = "(%d,%d,%d,%d):(%d,%d,%d,1)" % (N, C, H, W, C * H * W, H * W, W)
    dl = "(%d,%d,%d,%d):(%d,1,%d,%d)" % (N, C, H, W, H * W * C, W * C, C)
    oracle.copy(src, sl, dst, dl)
    expect = src.reshape(N, C, H, W).transpose(0, 2, 3, 1)
    assert (dst.reshape(N, H, W, C) == expect).all()


def test_gather_and_broadcast_are_numpy_slicing(oracle):
    src = _rand(1000, np.uint32, 5)
    dst = np.zeros(300, np.uint32)
    oracle.copy(src, "300:3", dst, "300:1")
    assert (dst == src[::3][:300]).all()
    b = np.zeros(64 * 5, np.uint32)
    oracle.copy(src, "(64,5):(1,0)", b, "(64,5):(1,64)")
    assert (b.reshape(5, 64) == np.broadcast_to(src[:64], (5, 64))).all()


def test_counting_iterator_routing(oracle):
    # Sec. 2.5: with the source holding its own offsets, dst[L_dst(i)] == L_src(i) for every i
    cases = [("((2,2),(4,2)):((1,8),(2,16))", "(4,8):(8,1)"), ("(8,(3,5)):(1,(57,8))", "(8,15):(1,8)"),
             ("(2,3,2):(42,1,128)", "12:1"), ("12:1", "(2,3,2):(42,1,128)")]
    for s, d in cases:
        sl, dl = oracle.Layout(s), oracle.Layout(d)
        src = np.arange(sl.cosize, dtype=np.uint32)
        dst = np.full(dl.cosize, 0xFFFFFFFF, np.uint32)
        oracle.copy(src, sl, dst, dl)
        so, do = sl.offsets(), dl.offsets()
        assert (dst[do] == so).all()
        untouched = np.ones(dl.cosize, bool)
        untouched[do] = False
        assert (dst[untouched] == 0xFFFFFFFF).all()


def test_copy_applications_table(oracle):
    # Table copy: each row against an independent numpy statement of the same data movement
    rows = {}
    for ln in golden_lines("copy_applications.txt"):
        name, s, d = [x.strip() for x in ln.split("|")]
        rows[name] = (s, d)
    assert len(rows) == 8
    src = _rand(256, np.uint32, 9)

    def run(name):
        s, d = rows[name]
        dst = np.full(256, 7, np.uint32)
        oracle.copy(src, s, dst, d)
        return dst

    assert (run("1D Arrays")[:8] == src[:8]).all()
    nd = run("ND Arrays")
    idx = [i + 16 * j + 32 * k for k in range(3) for j in range(2) for i in range(8)]
    assert (nd[idx] == src[idx]).all() and (np.delete(nd, idx) == 7).all()
    g = run("Gather")
    assert list(g[:12]) == [src[42 * a + b + 128 * c] for c in range(2) for b in range(3) for a in range(2)]
    sc = run("Scatter")
    k = 0
    for c in range(2):
        for b in range(3):
            for a in range(2):
                assert sc[42 * a + b + 128 * c] == src[k]
                k += 1
    assert (run("Broadcast")[:7] == src[0]).all()
    assert run("Constant")[0] == src[0] and (run("Constant")[1:] == 7).all()
    t = run("Transpose")
    assert (t[:24].reshape(8, 3) == src[:24].reshape(3, 8).T).all()
    tt = run("Tensor Transpose")
    expect = np.array([src[i + 57 * j + 8 * k] for k in range(5) for j in range(3) for i in range(8)])
    assert (tt[:120] == expect).all()


def test_size_mismatch_is_rejected(oracle):
    with pytest.raises(oracle.OracleError) as e:
        oracle.copy(np.zeros(16, np.uint32), "8:1", np.zeros(16, np.uint32), "9:1")
    assert e.value.status_name == "SIZE_MISMATCH"


def test_aliasing_destination_last_write_wins(oracle):
    # sequential loop semantics for a non-injective destination (Table copy, "Constant" generalised)
    src = np.arange(6, dtype=np.uint32) + 10
    dst = np.zeros(3, np.uint32)
    oracle.copy(src, "6:1", dst, "(3,2):(1,0)")
    assert list(dst) == [13, 14, 15]


def test_ranges_on_host_threads_equal_the_single_loop(oracle):
    """The loop cut into ranges (one per host thread) against the loop as Sec. 2.6.1 writes it and against numpy:
    for an injective destination the order of the coordinates cannot matter."""
    N, C, H, W = 3, 5, 7, 11
    sl = "(%d,%d,%d,%d):(%d,%d,%d,1)" % (N, C, H, W, C * H * W, H * W, W)
    dl = "(%d,%d,%d,%d):(%d,1,%d,%d)" % (N, C, H, W, H * W * C, W * C, C)
    src = _rand(N * C * H * W, np.uint32, 21)
    whole = oracle.copy(src, sl, np.zeros_like(src), dl)
    for threads in (1, 2, 3, 8, 5000):
        cut = oracle.copy_parallel(src, sl, np.zeros_like(src), dl, threads)
        assert (cut == whole).all()
    assert (whole.reshape(N, H, W, C) == src.reshape(N, C, H, W).transpose(0, 2, 3, 1)).all()


def test_negative_strides_are_numpy_negative_steps(oracle):
    """Sec. 2.3.2 allows strides from Z; the accessor's pointer (Sec. 2.5) then sits inside the buffer.  The loop against
    numpy's negative-step slicing and flips: reversal, reversed gather, flipped matrix, flipped transpose."""
    src = _rand(40, np.uint32, 31)
    # reversed copy: dst[i] = src[39 - i]
    dst = np.zeros(40, np.uint32)
    oracle.copy(src, "40:-1", dst, "40:1", src_origin=39)
    assert (dst == src[::-1]).all()
    # the destination runs backwards instead
    dst = np.zeros(40, np.uint32)
    oracle.copy(src, "40:1", dst, "40:-1", dst_origin=39)
    assert (dst == src[::-1]).all()
    # both backwards: a plain copy again
    dst = np.zeros(40, np.uint32)
    oracle.copy(src, "40:-1", dst, "40:-1", src_origin=39, dst_origin=39)
    assert (dst == src).all()
    # gather every third element from the top down
    dst = np.zeros(13, np.uint32)
    oracle.copy(src, "13:-3", dst, "13:1", src_origin=38)
    assert (dst == src[38::-3]).all()
    # a 5 x 8 row-major matrix flipped upside down, left-right, and both, into a column-major destination
    M, N = 5, 8
    a = src.reshape(M, N)
    for flip_rows, flip_cols in [(True, False), (False, True), (True, True)]:
        sl = "(%d,%d):(%d,%d)" % (M, N, -N if flip_rows else N, -1 if flip_cols else 1)
        origin = (M - 1) * N * flip_rows + (N - 1) * flip_cols
        dst = np.zeros(M * N, np.uint32)
        oracle.copy(src, sl, dst, "(%d,%d):(1,%d)" % (M, N, M), src_origin=origin)
        want = a[::-1] if flip_rows else a
        want = want[:, ::-1] if flip_cols else want
        assert (dst.reshape(N, M).T == want).all(), sl
    # numpy's own strided view with a negative stride as the destination
    dst = np.zeros(40, np.uint32)
    oracle.copy(src, "(5,8):(8,1)", dst, "(5,8):(-1,5)", dst_origin=4)
    view = np.lib.stride_tricks.as_strided(dst[4:], shape=(5, 8), strides=(-4, 20))
    assert (view == a).all()
    lo = oracle.Layout("(5,8):(-1,5)")
    assert (lo.min_offset, lo.cosize) == (-4, 36)
