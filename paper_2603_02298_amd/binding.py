"""ctypes binding of liblayoutcopy.so: the same entry points as include/layoutcopy.h, with
argument marshalling only.  Every step of a copy runs in the library's HIP kernels; there is no
Python or CPU fallback, and a missing library is an error."""
import ctypes
import os

from . import build as _build

_lib = None

DTYPES = {"f32": 0, "f16": 1, "bf16": 2, "b8": 3, "b16": 4, "b32": 5, "b64": 6, "b128": 7}
DTYPE_BYTES = {"f32": 4, "f16": 2, "bf16": 2, "b8": 1, "b16": 2, "b32": 4, "b64": 8, "b128": 16}


class LayoutCopyError(RuntimeError):
    def __init__(self, status, what):
        name = lib().lc_status_string(status).decode()
        detail = lib().lc_last_hip_error().decode() if name == "HIP" else ""
        super().__init__("%s: %s%s" % (what, name, " [" + detail + "]" if detail else ""))
        self.status = status
        self.status_name = name


def lib():
    """Loads the in-tree library (built by paper_2603_02298_amd.build / __graft_entry__.build)."""
    global _lib
    if _lib is not None:
        return _lib
    path = _build.LIB_PATH
    if not os.path.exists(path):
        raise RuntimeError("liblayoutcopy.so is not built: run `python -m paper_2603_02298_amd.build` "
                           "(there is no fallback path)")
    # Streams and device pointers handed to the library come from PyTorch, so both must talk to the
    # same HIP runtime: PyTorch's wheel carries its own libamdhip64 and the loader keeps whichever
    # copy it sees first.  Importing torch first makes that copy the one this library binds to.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    L = ctypes.CDLL(path)
    P, PP = ctypes.c_void_p, ctypes.POINTER(ctypes.c_void_p)
    i64, sz = ctypes.c_int64, ctypes.c_size_t
    L.lc_status_string.argtypes = [ctypes.c_int]
    L.lc_status_string.restype = ctypes.c_char_p
    L.lc_last_hip_error.argtypes = []
    L.lc_last_hip_error.restype = ctypes.c_char_p
    L.lc_dtype_bytes.argtypes = [ctypes.c_int]
    L.lc_layout_parse.argtypes = [ctypes.c_char_p, PP]
    L.lc_layout_from_tree.argtypes = [ctypes.POINTER(i64), ctypes.c_int, ctypes.POINTER(i64), ctypes.c_int, PP]
    L.lc_layout_destroy.argtypes = [P]
    L.lc_layout_destroy.restype = None
    L.lc_layout_to_string.argtypes = [P, ctypes.c_char_p, sz, ctypes.POINTER(sz)]
    for n in ("size", "cosize"):
        f = getattr(L, "lc_layout_" + n)
        f.argtypes, f.restype = [P], i64
    L.lc_layout_rank.argtypes = [P]
    L.lc_layout_depth.argtypes = [P]
    L.lc_layout_eval.argtypes = [P, i64]
    L.lc_layout_eval.restype = i64
    for n in ("coalesce", "coalesce_bymode", "right_inverse", "left_inverse"):
        getattr(L, "lc_" + n).argtypes = [P, PP]
    for n in ("composition", "composition_bymode", "logical_divide", "logical_divide_bymode", "zipped_divide",
              "logical_product", "blocked_product", "raked_product"):
        getattr(L, "lc_" + n).argtypes = [P, P, PP]
    L.lc_complement.argtypes = [P, i64, PP]
    L.lc_layout_slice.argtypes = [P, ctypes.c_char_p, ctypes.POINTER(i64), PP]
    L.lc_slayout_parse.argtypes = [ctypes.c_char_p, PP]
    L.lc_slayout_destroy.argtypes = [P]
    L.lc_slayout_destroy.restype = None
    L.lc_slayout_to_string.argtypes = [P, ctypes.c_char_p, ctypes.c_size_t, ctypes.POINTER(ctypes.c_size_t)]
    L.lc_slayout_kind.argtypes = [P]
    L.lc_slayout_codomain_rank.argtypes = [P]
    L.lc_slayout_size.argtypes = [P]
    L.lc_slayout_size.restype = i64
    L.lc_slayout_eval.argtypes = [P, i64, ctypes.POINTER(i64), ctypes.c_int]
    L.lc_slayout_composition.argtypes = [P, P, PP]
    L.lc_slayout_coalesce.argtypes = [P, PP]
    L.lc_slayout_right_inverse.argtypes = [P, PP]
    L.lc_slayout_xor_right_inverse.argtypes = [P, PP]
    L.lc_layout_min_offset.argtypes = [P]
    L.lc_layout_min_offset.restype = i64
    L.lc_max_common_vector.argtypes = [P, P, ctypes.POINTER(i64)]
    L.lc_admissible.argtypes = [P, P, ctypes.POINTER(ctypes.c_int), PP]
    L.lc_plan_create.argtypes = [P, P, ctypes.c_int, ctypes.c_uint, ctypes.c_uint, PP]
    L.lc_plan_describe.argtypes = [P, ctypes.c_char_p, sz, ctypes.POINTER(sz)]
    L.lc_plan_execute.argtypes = [P, P, P, P]
    L.lc_plan_workspace_bytes.argtypes = [P]
    L.lc_plan_workspace_bytes.restype = i64
    L.lc_plan_execute_workspace.argtypes = [P, P, P, P, sz, P]
    L.lc_plan_execute_static.argtypes = [P, P, P, P]
    L.lc_static_scratch_bytes.restype = sz
    L.lc_plan_destroy.argtypes = [P]
    L.lc_plan_destroy.restype = None
    L.lc_copy.argtypes = [P, P, P, P, ctypes.c_int, P]
    L.lc_plan_algorithmic_bytes.argtypes = [P]
    L.lc_plan_algorithmic_bytes.restype = i64
    L.lc_plan_time.argtypes = [P, PP, PP, ctypes.c_int, ctypes.c_int, ctypes.c_int, P, ctypes.POINTER(ctypes.c_float)]
    L.lc_plan_time_each.argtypes = [P, PP, PP, ctypes.c_int, ctypes.c_int, ctypes.c_int, P, ctypes.POINTER(ctypes.c_float)]
    L.lc_debug_replay_on_host.argtypes = [P, P, i64, P, i64, ctypes.POINTER(i64)]
    L.lc_debug_replay_on_host_at.argtypes = [P, P, i64, i64, P, i64, i64, ctypes.POINTER(i64)]
    u = ctypes.c_uint
    L.lc_gemm_plan_create.argtypes = [P, P, P, ctypes.c_int, u, u, u, PP]
    L.lc_gemm_plan_describe.argtypes = [P, ctypes.c_char_p, sz, ctypes.POINTER(sz)]
    L.lc_gemm_plan_execute.argtypes = [P, P, P, P, P]
    L.lc_gemm_plan_destroy.argtypes = [P]
    L.lc_gemm_plan_destroy.restype = None
    L.lc_gemm.argtypes = [P, P, P, P, P, P, ctypes.c_int, P]
    L.lc_gemm_plan_flops.argtypes = [P]
    L.lc_gemm_plan_flops.restype = i64
    L.lc_gemm_plan_time.argtypes = [P, P, P, P, ctypes.c_int, ctypes.c_int, P, ctypes.POINTER(ctypes.c_float)]
    L.lc_mfma_fragment_layout.argtypes = [ctypes.c_int, PP]
    L.lc_debug_gemm_replay_on_host.argtypes = [P, P, i64, P, i64, P, i64]
    L.lc_debug_gemm_lds_address.argtypes = [ctypes.c_int, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_uint32]
    L.lc_debug_gemm_lds_address.restype = i64
    _lib = L
    return L


def _check(status, what):
    if status != 0:
        raise LayoutCopyError(status, what)


class Layout:
    """lc_layout_t handle."""

    def __init__(self, text=None, _handle=None):
        self._h = _handle if _handle is not None else ctypes.c_void_p()
        if _handle is None:
            _check(lib().lc_layout_parse(text.encode(), ctypes.byref(self._h)), "lc_layout_parse(%r)" % text)

    @classmethod
    def from_tree(cls, shape_preorder, leaf_strides):
        a = (ctypes.c_int64 * len(shape_preorder))(*shape_preorder)
        b = (ctypes.c_int64 * len(leaf_strides))(*leaf_strides)
        h = ctypes.c_void_p()
        _check(lib().lc_layout_from_tree(a, len(shape_preorder), b, len(leaf_strides), ctypes.byref(h)), "lc_layout_from_tree")
        return cls(_handle=h)

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.lc_layout_destroy(self._h)
            self._h = None

    def __str__(self):
        need = ctypes.c_size_t()
        lib().lc_layout_to_string(self._h, None, 0, ctypes.byref(need))
        buf = ctypes.create_string_buffer(need.value)
        lib().lc_layout_to_string(self._h, buf, need.value, None)
        return buf.value.decode()

    __repr__ = __str__
    size = property(lambda self: lib().lc_layout_size(self._h))
    cosize = property(lambda self: lib().lc_layout_cosize(self._h))
    min_offset = property(lambda self: lib().lc_layout_min_offset(self._h))
    rank = property(lambda self: lib().lc_layout_rank(self._h))
    depth = property(lambda self: lib().lc_layout_depth(self._h))

    def __call__(self, i):
        return lib().lc_layout_eval(self._h, i)


def _as_layout(x):
    return x if isinstance(x, Layout) else Layout(x)


def _unary(name, a):
    a = _as_layout(a)
    h = ctypes.c_void_p()
    _check(getattr(lib(), name)(a._h, ctypes.byref(h)), "%s(%s)" % (name, a))
    return Layout(_handle=h)


def _binary(name, a, b):
    a, b = _as_layout(a), _as_layout(b)
    h = ctypes.c_void_p()
    _check(getattr(lib(), name)(a._h, b._h, ctypes.byref(h)), "%s(%s, %s)" % (name, a, b))
    return Layout(_handle=h)


def lc_coalesce(a): return _unary("lc_coalesce", a)
def lc_coalesce_bymode(a): return _unary("lc_coalesce_bymode", a)
def lc_right_inverse(a): return _unary("lc_right_inverse", a)
def lc_left_inverse(a): return _unary("lc_left_inverse", a)
def lc_logical_product(a, b): return _binary("lc_logical_product", a, b)
def lc_blocked_product(a, b): return _binary("lc_blocked_product", a, b)
def lc_raked_product(a, b): return _binary("lc_raked_product", a, b)
def lc_composition(a, b): return _binary("lc_composition", a, b)
def lc_composition_bymode(a, t): return _binary("lc_composition_bymode", a, t)
def lc_logical_divide(a, b): return _binary("lc_logical_divide", a, b)
def lc_logical_divide_bymode(a, t): return _binary("lc_logical_divide_bymode", a, t)
def lc_zipped_divide(a, t): return _binary("lc_zipped_divide", a, t)


def lc_layout_slice(a, coord):
    """(offset, remaining layout) for a coordinate text with "_" at the unspecified positions."""
    a = _as_layout(a)
    h, off = ctypes.c_void_p(), ctypes.c_int64()
    _check(lib().lc_layout_slice(a._h, coord.encode(), ctypes.byref(off), ctypes.byref(h)), "lc_layout_slice(%s, %s)" % (a, coord))
    return off.value, Layout(_handle=h)


class SLayout:
    """A layout with integer-semimodule strides (Sec. 2.3.2): "(4,(4,2)):(e1,(e0,6e1))", "(8,8):(f1,f9)"."""

    KINDS = {0: "int", 1: "coord", 2: "xor"}

    def __init__(self, text=None, _handle=None):
        self._h = ctypes.c_void_p()
        if _handle is not None:
            self._h = _handle
        else:
            _check(lib().lc_slayout_parse(str(text).encode(), ctypes.byref(self._h)), "lc_slayout_parse(%r)" % (text,))

    def __del__(self):
        if getattr(self, "_h", None) and self._h.value:
            lib().lc_slayout_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __str__(self):
        buf = ctypes.create_string_buffer(4096)
        _check(lib().lc_slayout_to_string(self._h, buf, 4096, None), "lc_slayout_to_string")
        return buf.value.decode()

    @property
    def kind(self):
        return self.KINDS[lib().lc_slayout_kind(self._h)]

    @property
    def size(self):
        return lib().lc_slayout_size(self._h)

    def __call__(self, i):
        out = (ctypes.c_int64 * 16)()
        _check(lib().lc_slayout_eval(self._h, int(i), out, 16), "lc_slayout_eval")
        r = lib().lc_slayout_codomain_rank(self._h)
        return tuple(out[k] for k in range(r)) if self.kind == "coord" else out[0]


def _as_slayout(x):
    return x if isinstance(x, SLayout) else SLayout(x)


def lc_slayout_composition(a, b):
    a, b = _as_slayout(a), _as_layout(b)
    h = ctypes.c_void_p()
    _check(lib().lc_slayout_composition(a._h, b._h, ctypes.byref(h)), "lc_slayout_composition(%s, %s)" % (a, b))
    return SLayout(_handle=h)


def lc_slayout_coalesce(a):
    a = _as_slayout(a)
    h = ctypes.c_void_p()
    _check(lib().lc_slayout_coalesce(a._h, ctypes.byref(h)), "lc_slayout_coalesce(%s)" % a)
    return SLayout(_handle=h)


def lc_slayout_right_inverse(a):
    a = _as_slayout(a)
    h = ctypes.c_void_p()
    _check(lib().lc_slayout_right_inverse(a._h, ctypes.byref(h)), "lc_slayout_right_inverse(%s)" % a)
    return Layout(_handle=h)


def lc_slayout_xor_right_inverse(a):
    a = _as_slayout(a)
    h = ctypes.c_void_p()
    _check(lib().lc_slayout_xor_right_inverse(a._h, ctypes.byref(h)), "lc_slayout_xor_right_inverse(%s)" % a)
    return SLayout(_handle=h)


def lc_complement(a, cotarget=0):
    a = _as_layout(a)
    h = ctypes.c_void_p()
    _check(lib().lc_complement(a._h, cotarget, ctypes.byref(h)), "lc_complement(%s, %d)" % (a, cotarget))
    return Layout(_handle=h)


def lc_admissible(a, t):
    """(yes, where): Sec. 3.4.3's check that the data layout a holds every offset of the instruction layout t, and the
    layout a^† o t of their locations (None when not admissible, or when that composition does not exist)."""
    a, t = _as_layout(a), _as_layout(t)
    yes = ctypes.c_int()
    h = ctypes.c_void_p()
    _check(lib().lc_admissible(a._h, t._h, ctypes.byref(yes), ctypes.byref(h)), "lc_admissible(%s, %s)" % (a, t))
    return bool(yes.value), (Layout(_handle=h) if h.value else None)


def lc_max_common_vector(a, b):
    a, b = _as_layout(a), _as_layout(b)
    k = ctypes.c_int64()
    _check(lib().lc_max_common_vector(a._h, b._h, ctypes.byref(k)), "lc_max_common_vector(%s, %s)" % (a, b))
    return k.value


class Plan:
    """lc_plan_t handle."""

    def __init__(self, src_layout, dst_layout, dtype, src_align=256, dst_align=256):
        self.src_layout, self.dst_layout = _as_layout(src_layout), _as_layout(dst_layout)
        self.dtype = dtype
        self._h = ctypes.c_void_p()
        _check(lib().lc_plan_create(self.src_layout._h, self.dst_layout._h, DTYPES[dtype], src_align, dst_align,
                                    ctypes.byref(self._h)),
               "lc_plan_create(%s -> %s, %s)" % (self.src_layout, self.dst_layout, dtype))

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.lc_plan_destroy(self._h)
            self._h = None

    def describe(self):
        need = ctypes.c_size_t()
        lib().lc_plan_describe(self._h, None, 0, ctypes.byref(need))
        buf = ctypes.create_string_buffer(need.value)
        lib().lc_plan_describe(self._h, buf, need.value, None)
        return buf.value.decode()

    @property
    def algorithmic_bytes(self):
        return lib().lc_plan_algorithmic_bytes(self._h)

    def execute(self, src_ptr, dst_ptr, stream=0):
        """src_ptr / dst_ptr: device addresses (e.g. tensor.data_ptr()); stream: hipStream_t as int."""
        _check(lib().lc_plan_execute(self._h, src_ptr, dst_ptr, stream), "lc_plan_execute")

    def execute_static(self, src_ptr, dst_ptr, stream=0):
        """The same with the library's static scratch array on the current GPU: allocates nothing."""
        _check(lib().lc_plan_execute_static(self._h, src_ptr, dst_ptr, stream), "lc_plan_execute_static")

    @property
    def workspace_bytes(self):
        return lib().lc_plan_workspace_bytes(self._h)

    def execute_workspace(self, src_ptr, dst_ptr, workspace_ptr, workspace_bytes, stream=0):
        """The same with scratch device memory (a device address and its size) for plans of class last-writer."""
        _check(lib().lc_plan_execute_workspace(self._h, src_ptr, dst_ptr, workspace_ptr, workspace_bytes, stream),
               "lc_plan_execute_workspace")

    def time(self, src_ptrs, dst_ptrs, warmup, iters, stream=0):
        n = len(src_ptrs)
        a = (ctypes.c_void_p * n)(*src_ptrs)
        b = (ctypes.c_void_p * n)(*dst_ptrs)
        ms = ctypes.c_float()
        _check(lib().lc_plan_time(self._h, a, b, n, warmup, iters, stream, ctypes.byref(ms)), "lc_plan_time")
        return ms.value

    def time_each(self, src_ptrs, dst_ptrs, warmup, iters, stream=0):
        """Milliseconds of each of `iters` executions (an event between every two of them)."""
        n = len(src_ptrs)
        a = (ctypes.c_void_p * n)(*src_ptrs)
        b = (ctypes.c_void_p * n)(*dst_ptrs)
        ms = (ctypes.c_float * iters)()
        _check(lib().lc_plan_time_each(self._h, a, b, n, warmup, iters, stream, ms), "lc_plan_time_each")
        return list(ms)

    def debug_replay_on_host(self, src, dst, src_origin=0, dst_origin=0):
        """Test instrumentation: walk the plan's index arithmetic over numpy arrays on the host
        (bounds-checked); returns the modelled LDS bank-conflict cycles of one tile.  src_origin / dst_origin: the
        element of each array that offset 0 of its layout refers to (layouts with negative strides reach below it)."""
        c = ctypes.c_int64()
        _check(lib().lc_debug_replay_on_host_at(self._h, src.ctypes.data_as(ctypes.c_void_p), src.size, src_origin,
                                                dst.ctypes.data_as(ctypes.c_void_p), dst.size, dst_origin, ctypes.byref(c)),
               "lc_debug_replay_on_host")
        return c.value


def lc_copy(src_ptr, src_layout, dst_ptr, dst_layout, dtype, stream=0):
    """COPY on the GPU: dst(i) = src(i) for device pointers src_ptr / dst_ptr."""
    sl, dl = _as_layout(src_layout), _as_layout(dst_layout)
    _check(lib().lc_copy(src_ptr, sl._h, dst_ptr, dl._h, DTYPES[dtype], stream), "lc_copy(%s -> %s)" % (sl, dl))


def copy_tensor(src, src_layout, dst, dst_layout, dtype=None, src_origin=0, dst_origin=0):
    """Convenience for torch tensors on the GPU: takes data pointers and torch's current stream.  src_origin / dst_origin:
    the element of each tensor that offset 0 of its layout refers to (layouts with negative strides reach below it)."""
    import torch
    if not (src.is_cuda and dst.is_cuda):
        raise RuntimeError("copy_tensor needs GPU tensors: the copy only runs in the HIP kernels")
    if dtype is None:
        dtype = {4: "b32", 2: "b16", 1: "b8", 8: "b64"}[src.element_size()]
    sl, dl = _as_layout(src_layout), _as_layout(dst_layout)
    if src_origin + sl.min_offset < 0 or src_origin + sl.cosize > src.numel() or dst_origin + dl.min_offset < 0 or dst_origin + dl.cosize > dst.numel():
        raise ValueError("tensor does not cover the offsets the layout reaches")
    lc_copy(src.data_ptr() + src_origin * src.element_size(), sl, dst.data_ptr() + dst_origin * dst.element_size(), dl, dtype,
            torch.cuda.current_stream().cuda_stream)


class GemmPlan:
    """lc_gemm_plan_t handle: C(m,n) += A(m,k) * B(n,k) over three rank-2 layouts."""

    def __init__(self, a_layout, b_layout, c_layout, ab_dtype="bf16", a_align=256, b_align=256, c_align=256):
        self.a_layout, self.b_layout, self.c_layout = _as_layout(a_layout), _as_layout(b_layout), _as_layout(c_layout)
        self.ab_dtype = ab_dtype
        self._h = ctypes.c_void_p()
        _check(lib().lc_gemm_plan_create(self.a_layout._h, self.b_layout._h, self.c_layout._h, DTYPES[ab_dtype], a_align, b_align,
                                         c_align, ctypes.byref(self._h)),
               "lc_gemm_plan_create(%s, %s, %s, %s)" % (self.a_layout, self.b_layout, self.c_layout, ab_dtype))

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.lc_gemm_plan_destroy(self._h)
            self._h = None

    def describe(self):
        need = ctypes.c_size_t()
        lib().lc_gemm_plan_describe(self._h, None, 0, ctypes.byref(need))
        buf = ctypes.create_string_buffer(need.value)
        lib().lc_gemm_plan_describe(self._h, buf, need.value, None)
        return buf.value.decode()

    @property
    def flops(self):
        return lib().lc_gemm_plan_flops(self._h)

    def execute(self, a_ptr, b_ptr, c_ptr, stream=0):
        """a_ptr / b_ptr / c_ptr: device addresses; stream: hipStream_t as int."""
        _check(lib().lc_gemm_plan_execute(self._h, a_ptr, b_ptr, c_ptr, stream), "lc_gemm_plan_execute")

    def time(self, a_ptr, b_ptr, c_ptr, warmup, iters, stream=0):
        ms = ctypes.c_float()
        _check(lib().lc_gemm_plan_time(self._h, a_ptr, b_ptr, c_ptr, warmup, iters, stream, ctypes.byref(ms)), "lc_gemm_plan_time")
        return ms.value

    def debug_replay_on_host(self, a, b, c):
        """Test instrumentation: walk the plan's index arithmetic over numpy arrays on the host (uint16 bit
        patterns for a and b, float32 c updated in place), every access bounds-checked."""
        vp = ctypes.c_void_p
        _check(lib().lc_debug_gemm_replay_on_host(self._h, a.ctypes.data_as(vp), a.size, b.ctypes.data_as(vp), b.size,
                                                  c.ctypes.data_as(vp), c.size), "lc_debug_gemm_replay_on_host")
        return c


def lc_gemm(a_ptr, a_layout, b_ptr, b_layout, c_ptr, c_layout, ab_dtype="bf16", stream=0):
    """GEMM on the GPU for device pointers: C(m,n) += A(m,k) * B(n,k)."""
    la, lb, lc_ = _as_layout(a_layout), _as_layout(b_layout), _as_layout(c_layout)
    _check(lib().lc_gemm(a_ptr, la._h, b_ptr, lb._h, c_ptr, lc_._h, DTYPES[ab_dtype], stream),
           "lc_gemm(%s, %s, %s)" % (la, lb, lc_))


def lc_mfma_fragment_layout(which):
    h = ctypes.c_void_p()
    _check(lib().lc_mfma_fragment_layout(which, ctypes.byref(h)), "lc_mfma_fragment_layout(%d)" % which)
    return Layout(_handle=h)


def gemm_tensor(a, a_layout, b, b_layout, c, c_layout):
    """Convenience for torch tensors on the GPU (a, b: bfloat16 or float16; c: float32)."""
    import torch
    if not (a.is_cuda and b.is_cuda and c.is_cuda):
        raise RuntimeError("gemm_tensor needs GPU tensors: the GEMM only runs in the HIP kernel")
    if a.dtype != b.dtype or a.dtype not in (torch.bfloat16, torch.float16) or c.dtype != torch.float32:
        raise ValueError("a, b: both bfloat16 or both float16; c: float32")
    la, lb, lc_ = _as_layout(a_layout), _as_layout(b_layout), _as_layout(c_layout)
    if la.cosize > a.numel() or lb.cosize > b.numel() or lc_.cosize > c.numel():
        raise ValueError("tensor smaller than the layout's cosize")
    lc_gemm(a.data_ptr(), la, b.data_ptr(), lb, c.data_ptr(), lc_, "bf16" if a.dtype == torch.bfloat16 else "f16",
            torch.cuda.current_stream().cuda_stream)
