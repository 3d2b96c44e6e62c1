"""ORACLE — test infrastructure only.

ctypes access to the CPU oracle (``oracle/layout_oracle.cpp``).  Only tests, the smoke
check and the benchmark's CPU-baseline leg import this module; the GPU package never does.
Argument marshalling only: all arithmetic is in the C++ oracle.
"""
import ctypes
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboracle.so")
_SOURCES = ["layout_oracle.cpp", "semimodule_oracle.cpp", "gemm_oracle.cpp", "oracle_capi.cpp"]

STATUS_NAMES = {
    0: "OK", 1: "INVALID_ARG", 2: "PARSE", 3: "NOT_CONGRUENT", 4: "BAD_EXTENT", 5: "NEGATIVE_STRIDE",
    6: "SIZE_MISMATCH", 7: "STRIDE_DIVISIBILITY", 8: "SHAPE_DIVISIBILITY", 9: "NOT_SEGREGATED",
    10: "NOT_INJECTIVE", 11: "NOT_SURJECTIVE",
}


class OracleError(Exception):
    def __init__(self, status, what):
        super().__init__("%s: %s" % (what, STATUS_NAMES.get(status, status)))
        self.status = status
        self.status_name = STATUS_NAMES.get(status, str(status))


def build(force=False):
    """Compile the oracle (g++, host only)."""
    srcs = [os.path.join(_HERE, s) for s in _SOURCES]
    hdrs = [os.path.join(_HERE, h) for h in ("layout_oracle.hpp", "semimodule_oracle.hpp", "gemm_oracle.hpp")]
    if not force and os.path.exists(_LIB_PATH):
        newest = max(os.path.getmtime(p) for p in srcs + hdrs)
        if os.path.getmtime(_LIB_PATH) >= newest:
            return _LIB_PATH
    cmd = ["g++", "-std=c++17", "-O2", "-Wall", "-Wextra", "-fPIC", "-shared", "-o", _LIB_PATH] + srcs
    subprocess.check_call(cmd)
    return _LIB_PATH


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB_PATH)
        P = ctypes.c_void_p
        PP = ctypes.POINTER(ctypes.c_void_p)
        i64 = ctypes.c_int64
        L.oracle_layout_parse.argtypes = [ctypes.c_char_p, PP]
        L.oracle_layout_destroy.argtypes = [P]
        L.oracle_layout_destroy.restype = None
        L.oracle_layout_to_string.argtypes = [P, ctypes.c_char_p, ctypes.c_size_t, ctypes.POINTER(ctypes.c_size_t)]
        for name in ("size", "cosize", "min_offset"):
            f = getattr(L, "oracle_layout_" + name)
            f.argtypes = [P]
            f.restype = i64
        L.oracle_layout_rank.argtypes = [P]
        L.oracle_layout_depth.argtypes = [P]
        L.oracle_layout_eval.argtypes = [P, i64]
        L.oracle_layout_eval.restype = i64
        L.oracle_layout_eval_range.argtypes = [P, i64, i64, P]
        L.oracle_layout_eval_range.restype = None
        L.oracle_layout_eval_many.argtypes = [P, P, i64, P]
        L.oracle_layout_eval_many.restype = None
        L.oracle_layout_eval_crd.argtypes = [P, ctypes.c_char_p, ctypes.POINTER(i64)]
        L.oracle_idx2crd_natural.argtypes = [P, i64, ctypes.c_char_p, ctypes.c_size_t, ctypes.POINTER(ctypes.c_size_t)]
        L.oracle_idx2crd_in.argtypes = [ctypes.c_char_p, i64, ctypes.c_char_p, ctypes.c_size_t, ctypes.POINTER(ctypes.c_size_t)]
        L.oracle_crd2idx.argtypes = [P, ctypes.c_char_p, ctypes.POINTER(i64)]
        for name in ("shape_compatible", "congruent", "weakly_congruent"):
            getattr(L, "oracle_" + name).argtypes = [ctypes.c_char_p, ctypes.c_char_p]
        for name in ("coalesce", "coalesce_bymode", "right_inverse", "left_inverse"):
            getattr(L, "oracle_" + name).argtypes = [P, PP]
        for name in ("composition", "composition_bymode", "logical_divide", "logical_divide_bymode", "zipped_divide",
                     "logical_product", "blocked_product", "raked_product"):
            getattr(L, "oracle_" + name).argtypes = [P, P, PP]
        L.oracle_complement.argtypes = [P, i64, PP]
        L.oracle_admissible.argtypes = [P, P]
        L.oracle_layout_slice.argtypes = [P, ctypes.c_char_p, ctypes.POINTER(i64), PP]
        L.oracle_max_common_vector.argtypes = [P, P, ctypes.POINTER(i64)]
        L.oracle_max_common_vector_def.argtypes = [P, P, ctypes.POINTER(i64)]
        L.oracle_slayout_parse.argtypes = [ctypes.c_char_p, PP]
        L.oracle_slayout_destroy.argtypes = [P]
        L.oracle_slayout_destroy.restype = None
        L.oracle_slayout_to_string.argtypes = [P, ctypes.c_char_p, ctypes.c_size_t, ctypes.POINTER(ctypes.c_size_t)]
        L.oracle_slayout_kind.argtypes = [P]
        L.oracle_slayout_codomain_rank.argtypes = [P]
        L.oracle_slayout_size.argtypes = [P]
        L.oracle_slayout_size.restype = i64
        L.oracle_slayout_eval.argtypes = [P, i64, ctypes.POINTER(i64), ctypes.c_int]
        L.oracle_slayout_composition.argtypes = [P, P, PP]
        L.oracle_slayout_coalesce.argtypes = [P, PP]
        L.oracle_slayout_right_inverse.argtypes = [P, PP]
        L.oracle_slayout_xor_right_inverse.argtypes = [P, PP]
        L.oracle_copy.argtypes = [P, P, P, P, ctypes.c_int]
        L.oracle_copy_range.argtypes = [P, P, P, P, ctypes.c_int, i64, i64]
        L.oracle_gemm_check.argtypes = [P, P, P, ctypes.POINTER(i64), ctypes.POINTER(i64), ctypes.POINTER(i64), ctypes.POINTER(i64)]
        L.oracle_gemm.argtypes = [P, P, P, P, P, P]
        L.oracle_gemm_at.argtypes = [P, P, P, P, P, P, P, P, P, i64, P]
        _lib = L
    return _lib


def _check(status, what):
    if status != 0:
        raise OracleError(status, what)


class Layout:
    """A layout S:D held by the oracle."""

    def __init__(self, text=None, _handle=None):
        self._h = ctypes.c_void_p()
        if _handle is not None:
            self._h = _handle
        else:
            _check(lib().oracle_layout_parse(text.encode(), ctypes.byref(self._h)), "parse %r" % text)

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.oracle_layout_destroy(self._h)
            self._h = None

    def __str__(self):
        buf = ctypes.create_string_buffer(4096)
        lib().oracle_layout_to_string(self._h, buf, 4096, None)
        return buf.value.decode()

    __repr__ = __str__

    @property
    def size(self):
        return lib().oracle_layout_size(self._h)

    @property
    def cosize(self):
        return lib().oracle_layout_cosize(self._h)

    @property
    def min_offset(self):
        """Smallest offset of the image: 0 unless a stride is negative."""
        return lib().oracle_layout_min_offset(self._h)

    @property
    def rank(self):
        return lib().oracle_layout_rank(self._h)

    @property
    def depth(self):
        return lib().oracle_layout_depth(self._h)

    def __call__(self, c):
        """L(c): c is an int (integral coordinate, extended domain) or a coordinate string/tuple."""
        if isinstance(c, int):
            return lib().oracle_layout_eval(self._h, c)
        out = ctypes.c_int64()
        text = c if isinstance(c, str) else _tuple_text(c)
        _check(lib().oracle_layout_eval_crd(self._h, text.encode(), ctypes.byref(out)), "eval %s" % text)
        return out.value

    def offsets(self, begin=0, end=None):
        """numpy int64 array of L(i) for i in [begin, end)."""
        import numpy as np
        end = self.size if end is None else end
        out = np.empty(max(end - begin, 0), dtype=np.int64)
        lib().oracle_layout_eval_range(self._h, begin, end, out.ctypes.data_as(ctypes.c_void_p))
        return out

    def offsets_at(self, coords):
        """numpy int64 array of L(i) for the given integral coordinates."""
        import numpy as np
        coords = np.ascontiguousarray(coords, dtype=np.int64)
        out = np.empty(coords.size, dtype=np.int64)
        lib().oracle_layout_eval_many(self._h, coords.ctypes.data_as(ctypes.c_void_p), coords.size,
                                      out.ctypes.data_as(ctypes.c_void_p))
        return out

    def natural(self, i):
        buf = ctypes.create_string_buffer(1024)
        lib().oracle_idx2crd_natural(self._h, i, buf, 1024, None)
        return buf.value.decode()

    def crd2idx(self, c):
        out = ctypes.c_int64()
        text = c if isinstance(c, str) else _tuple_text(c)
        _check(lib().oracle_crd2idx(self._h, text.encode(), ctypes.byref(out)), "crd2idx %s" % text)
        return out.value


class SLayout:
    """A layout whose strides are integers, scaled basis elements a*e_i (it yields coordinates) or
    XOR elements f_d (Sec. 2.3.2), e.g. "(4,(4,2)):(e1,(e0,6e1))" or "(8,8):(f1,f9)"."""

    KINDS = {0: "int", 1: "coord", 2: "xor"}

    def __init__(self, text=None, _handle=None):
        self._h = ctypes.c_void_p()
        if _handle is not None:
            self._h = _handle
        else:
            _check(lib().oracle_slayout_parse(text.encode(), ctypes.byref(self._h)), "parse %r" % text)

    def __del__(self):
        if getattr(self, "_h", None) and self._h.value:
            lib().oracle_slayout_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __str__(self):
        buf = ctypes.create_string_buffer(4096)
        lib().oracle_slayout_to_string(self._h, buf, 4096, None)
        return buf.value.decode()

    @property
    def kind(self):
        return self.KINDS[lib().oracle_slayout_kind(self._h)]

    @property
    def size(self):
        return lib().oracle_slayout_size(self._h)

    def __call__(self, i):
        """L(i): a tuple of coordinates for e_i strides, an int otherwise."""
        out = (ctypes.c_int64 * 16)()
        _check(lib().oracle_slayout_eval(self._h, int(i), out, 16), "eval")
        r = lib().oracle_slayout_codomain_rank(self._h)
        return tuple(out[k] for k in range(r)) if self.kind == "coord" else out[0]


def _as_slayout(x):
    return x if isinstance(x, SLayout) else SLayout(str(x))


def slayout_composition(a, b):
    a, b = _as_slayout(a), _as_layout(b)
    h = ctypes.c_void_p()
    _check(lib().oracle_slayout_composition(a._h, b._h, ctypes.byref(h)), "composition(%s, %s)" % (a, b))
    return SLayout(_handle=h)


def slayout_coalesce(a):
    a = _as_slayout(a)
    h = ctypes.c_void_p()
    _check(lib().oracle_slayout_coalesce(a._h, ctypes.byref(h)), "coalesce(%s)" % a)
    return SLayout(_handle=h)


def slayout_right_inverse(a):
    a = _as_slayout(a)
    h = ctypes.c_void_p()
    _check(lib().oracle_slayout_right_inverse(a._h, ctypes.byref(h)), "right_inverse(%s)" % a)
    return Layout(_handle=h)


def slayout_xor_right_inverse(a):
    """Table rinv, last row: R = (2,...,2):(f_x0, f_x1, ...) with A(R(k)) = k; raises when A is not additive over XOR."""
    a = _as_slayout(a)
    h = ctypes.c_void_p()
    _check(lib().oracle_slayout_xor_right_inverse(a._h, ctypes.byref(h)), "xor_right_inverse(%s)" % a)
    return SLayout(_handle=h)


def _tuple_text(c):
    if isinstance(c, int):
        return str(c)
    return "(" + ",".join(_tuple_text(x) for x in c) + ")"


def _as_layout(x):
    return x if isinstance(x, Layout) else Layout(x)


def _unary(name, a):
    a = _as_layout(a)   # keep the temporary alive across the call
    h = ctypes.c_void_p()
    _check(getattr(lib(), "oracle_" + name)(a._h, ctypes.byref(h)), name)
    return Layout(_handle=h)


def _binary(name, a, b):
    a, b = _as_layout(a), _as_layout(b)
    h = ctypes.c_void_p()
    _check(getattr(lib(), "oracle_" + name)(a._h, b._h, ctypes.byref(h)), "%s(%s, %s)" % (name, a, b))
    return Layout(_handle=h)


def coalesce(a): return _unary("coalesce", a)
def coalesce_bymode(a): return _unary("coalesce_bymode", a)
def right_inverse(a): return _unary("right_inverse", a)
def left_inverse(a): return _unary("left_inverse", a)
def admissible(a, t):
    """Sec. 3.4.3, application: every offset of the instruction layout t is in the image of the data layout a."""
    a, t = _as_layout(a), _as_layout(t)
    return lib().oracle_admissible(a._h, t._h) == 1


def logical_product(a, b): return _binary("logical_product", a, b)
def blocked_product(a, b): return _binary("blocked_product", a, b)
def raked_product(a, b): return _binary("raked_product", a, b)
def composition(a, b): return _binary("composition", a, b)
def composition_bymode(a, t): return _binary("composition_bymode", a, t)
def logical_divide(a, b): return _binary("logical_divide", a, b)
def logical_divide_bymode(a, t): return _binary("logical_divide_bymode", a, t)
def zipped_divide(a, t): return _binary("zipped_divide", a, t)


def slice_layout(a, coord):
    """(offset, remaining layout) for a coordinate text with "_" at the unspecified positions."""
    a = _as_layout(a)
    h, off = ctypes.c_void_p(), ctypes.c_int64()
    _check(lib().oracle_layout_slice(a._h, coord.encode(), ctypes.byref(off), ctypes.byref(h)), "slice(%s, %s)" % (a, coord))
    return off.value, Layout(_handle=h)


def complement(a, cotarget=0):
    a = _as_layout(a)
    h = ctypes.c_void_p()
    _check(lib().oracle_complement(a._h, cotarget, ctypes.byref(h)), "complement(%s, %d)" % (a, cotarget))
    return Layout(_handle=h)


def max_common_vector(a, b):
    a, b = _as_layout(a), _as_layout(b)
    k = ctypes.c_int64()
    _check(lib().oracle_max_common_vector(a._h, b._h, ctypes.byref(k)), "max_common_vector")
    return k.value


def max_common_vector_def(a, b):
    a, b = _as_layout(a), _as_layout(b)
    k = ctypes.c_int64()
    _check(lib().oracle_max_common_vector_def(a._h, b._h, ctypes.byref(k)), "max_common_vector_def")
    return k.value


def idx2crd(shape_text, i):
    """The i-th coordinate of the coordinate set Z_shape (Fig. coordlists)."""
    buf = ctypes.create_string_buffer(1024)
    _check(lib().oracle_idx2crd_in(shape_text.encode(), i, buf, 1024, None), "idx2crd")
    return buf.value.decode()


def shape_compatible(p, s): return lib().oracle_shape_compatible(p.encode(), s.encode()) == 1
def congruent(p, s): return lib().oracle_congruent(p.encode(), s.encode()) == 1
def weakly_congruent(p, s): return lib().oracle_weakly_congruent(p.encode(), s.encode()) == 1


def copy(src, src_layout, dst, dst_layout, begin=0, end=None, spans_checked=False, src_origin=0, dst_origin=0):
    """dst(i) = src(i) over numpy arrays (1-D, same itemsize), element by element, in order.
    With a range [begin, end) the caller may pass buffers that only cover the offsets that range
    reaches and vouch for it with spans_checked=True.  src_origin / dst_origin: the element of the array that offset 0
    of the layout refers to (the accessor's pointer, Sec. 2.5); needed when strides are negative."""
    sl, dl = _as_layout(src_layout), _as_layout(dst_layout)
    assert src.dtype.itemsize == dst.dtype.itemsize and src.flags.c_contiguous and dst.flags.c_contiguous
    if not spans_checked:
        assert src_origin + sl.min_offset >= 0 and src_origin + sl.cosize <= src.size, "source buffer does not cover the layout's image"
        assert dst_origin + dl.min_offset >= 0 and dst_origin + dl.cosize <= dst.size, "destination buffer does not cover the layout's image"
    sp = ctypes.c_void_p(src.ctypes.data + src_origin * src.dtype.itemsize)
    dp = ctypes.c_void_p(dst.ctypes.data + dst_origin * dst.dtype.itemsize)
    if end is None:
        st = lib().oracle_copy(sp, sl._h, dp, dl._h, src.dtype.itemsize)
    else:
        st = lib().oracle_copy_range(sp, sl._h, dp, dl._h, src.dtype.itemsize, begin, end)
    _check(st, "copy")
    return dst


def copy_parallel(src, src_layout, dst, dst_layout, threads, begin=0, end=None, spans_checked=False):
    """The same element loop with the integral coordinates [begin, end) cut into `threads` consecutive ranges, one host
    thread per range (ctypes releases the interpreter lock during the call).  Every range runs the oracle's own
    copy_range.  Only for an injective destination: then no two coordinates write the same offset and the order of
    Sec. 2.6.1's loop cannot matter; the caller vouches for that (the five benchmark workloads are injective)."""
    from concurrent.futures import ThreadPoolExecutor
    sl, dl = _as_layout(src_layout), _as_layout(dst_layout)
    end = dl.size if end is None else end
    n = end - begin
    threads = max(1, min(int(threads), n))
    if not spans_checked:
        assert sl.cosize <= src.size and dl.cosize <= dst.size, "buffer smaller than the layout's cosize"
    cuts = [begin + n * k // threads for k in range(threads + 1)]
    with ThreadPoolExecutor(max_workers=threads) as pool:
        list(pool.map(lambda k: copy(src, sl, dst, dl, cuts[k], cuts[k + 1], spans_checked=True), range(threads)))
    return dst


def host_threads(limit=16):
    """Host cores this process may use (its affinity mask), at most `limit`."""
    try:
        return max(1, min(limit, len(os.sched_getaffinity(0))))
    except AttributeError:
        return max(1, min(limit, os.cpu_count() or 1))


def gemm_sizes(a_layout, b_layout, c_layout):
    """(M, N, K) — (M, N, K, L) for rank-3 layouts — when the three layouts meet the preconditions of the generic
    (batched) GEMM, else OracleError."""
    la, lb, lc = _as_layout(a_layout), _as_layout(b_layout), _as_layout(c_layout)
    M, N, K, L = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
    _check(lib().oracle_gemm_check(la._h, lb._h, lc._h, ctypes.byref(M), ctypes.byref(N), ctypes.byref(K), ctypes.byref(L)), "gemm_check")
    return (M.value, N.value, K.value) if la.rank == 2 else (M.value, N.value, K.value, L.value)


def _f64(x, layout, what):
    import numpy as np
    assert x.dtype == np.float64 and x.flags.c_contiguous and x.ndim == 1, what + ": 1-D float64 buffer expected"
    assert layout.cosize <= x.size, what + ": buffer smaller than the layout's cosize"
    return x.ctypes.data_as(ctypes.c_void_p)


def gemm(A, a_layout, B, b_layout, C, c_layout):
    """C(m,n) += A(m,k) * B(n,k) over float64 numpy buffers, k outermost, in place; returns C."""
    la, lb, lc = _as_layout(a_layout), _as_layout(b_layout), _as_layout(c_layout)
    st = lib().oracle_gemm(_f64(A, la, "A"), la._h, _f64(B, lb, "B"), lb._h, _f64(C, lc, "C"), lc._h)
    _check(st, "gemm")
    return C


def gemm_at(A, a_layout, B, b_layout, C, c_layout, ms, ns, ls=None):
    """The value the generic GEMM leaves in C(m_j, n_j) — C(m_j, n_j, l_j) for rank-3 layouts — for the listed
    coordinates (C itself untouched)."""
    import numpy as np
    la, lb, lc = _as_layout(a_layout), _as_layout(b_layout), _as_layout(c_layout)
    ms = np.ascontiguousarray(ms, dtype=np.int64)
    ns = np.ascontiguousarray(ns, dtype=np.int64)
    assert ms.shape == ns.shape and ms.ndim == 1
    if ls is not None:
        ls = np.ascontiguousarray(ls, dtype=np.int64)
        assert ls.shape == ms.shape
    out = np.zeros(ms.size, dtype=np.float64)
    st = lib().oracle_gemm_at(_f64(A, la, "A"), la._h, _f64(B, lb, "B"), lb._h, _f64(C, lc, "C"), lc._h,
                              ms.ctypes.data_as(ctypes.c_void_p), ns.ctypes.data_as(ctypes.c_void_p),
                              ls.ctypes.data_as(ctypes.c_void_p) if ls is not None else None, ms.size,
                              out.ctypes.data_as(ctypes.c_void_p))
    _check(st, "gemm_at")
    return out
