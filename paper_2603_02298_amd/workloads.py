"""Seeded synthetic inputs and the five benchmark workloads.

This module holds no layout arithmetic: layouts are given as text, buffer sizes as plain numbers
(checked against cosize in the tests), values come from numpy's seeded generators.  It serves the
CPU oracle and the GPU path alike so that both see the same bits.

The paper names no dataset; the workloads are stand-ins shaped like its tiling / partitioning
examples (tile-then-slice of Sec. 3.5.2, the COPY applications table of Sec. 2.6.1), at the sizes
the benchmark spec lists.  `scale` shrinks a workload for parity tests by shortening its outer modes.
"""
import numpy as np

SEED_BASE = 2603022980


class Workload:
    def __init__(self, name, dtype, src_layout, dst_layout, src_elems, dst_elems, n, values, note="", distinct_reads=None,
                 dram_read_elems=None):
        self.name, self.dtype = name, dtype
        self.src_layout, self.dst_layout = src_layout, dst_layout
        self.src_elems, self.dst_elems, self.n = src_elems, dst_elems, n
        self.values, self.note = values, note
        # plain numbers stated per workload (no layout arithmetic here; the tests check them against the oracle):
        # distinct source elements the copy reads (a stride-0 mode re-reads the same ones), and source elements whose
        # 32-byte sectors DRAM has to deliver (a strided gather drags its neighbours along)
        self.distinct_reads = n if distinct_reads is None else distinct_reads
        self.dram_read_elems = self.distinct_reads if dram_read_elems is None else dram_read_elems

    @property
    def elem_bytes(self):
        return 2 if self.dtype in ("bf16", "f16") else 4

    @property
    def algorithmic_bytes(self):
        """Element reads + element writes the method performs, re-reads through a stride-0 mode counted once."""
        return (self.distinct_reads + self.n) * self.elem_bytes

    @property
    def dram_minimum_bytes(self):
        """Bytes HBM cannot avoid moving: every 32-byte sector of the source that holds a read element, every written byte."""
        return (self.dram_read_elems + self.n) * self.elem_bytes


def _c1(scale=1):
    m = 1024 // scale
    return Workload("c1_transpose_f32", "f32", "(%d,%d):(1,%d)" % (m, m, m), "(%d,%d):(%d,1)" % (m, m, m),
                    m * m, m * m, m * m, "uniform", "2-D fp32 transpose, column-major to row-major")


def _c2(scale=1):
    # shape ((8,512),(8,1024)); source compact column-major; destination compact with mode order (2,0,3,1)
    a, b = 512 // scale, 1024 // scale
    src = "((8,%d),(8,%d)):((1,8),(%d,%d))" % (a, b, 8 * a, 64 * a)
    dst = "((8,%d),(8,%d)):((8,%d),(1,64))" % (a, b, 64 * b)
    n = 64 * a * b
    return Workload("c2_hier_relayout_bf16", "bf16", src, dst, n, n, n, "normal",
                    "hierarchical bf16 relayout, compact reading of the destination")


def _c2_literal():
    # the strides exactly as the benchmark spec prints them: not compact, cosize 2^32 - 1016 elements
    src = "((8,512),(8,1024)):((1,8),(4096,32768))"
    dst = "((8,512),(8,1024)):((1024,8388608),(1,8192))"
    n = 1 << 25
    return Workload("c2_literal_bf16", "bf16", src, dst, n, 4294966280, n, "normal",
                    "destination strides as printed; 16-byte runs over an 8.6 GB span")


def _c3(scale=1):
    # (S,D,H,B) column-major over (D,S,H,B), zipped_divide by <128,64>, into the compact layout of that shape
    S, D, H, B = 4096, 128, max(32 // scale, 1), max(64 // scale, 1)
    so, do = S // 128, D // 64
    src = "((128,64),(%d,%d,%d,%d)):((%d,1),(%d,64,%d,%d))" % (so, do, H, B, D, 128 * D, S * D, S * D * H)
    t = 128 * 64
    dst = "((128,64),(%d,%d,%d,%d)):((1,128),(%d,%d,%d,%d))" % (so, do, H, B, t, t * so, t * so * do, t * so * do * H)
    n = S * D * H * B
    return Workload("c3_tiled_partition_f16", "f16", src, dst, n, n, n, "normal",
                    "fp16 (B,H,S,D) tensor partitioned into 128x64 tiles")


def _c4a(scale=1):
    n = (1 << 26) // scale
    return Workload("c4a_strided_gather_f32", "f32", "%d:3" % n, "%d:1" % n, (1 << 28) // scale, n, n, "int_valued",
                    "gather with stride 3 into a contiguous destination",
                    dram_read_elems=3 * n)   # every 32-byte sector of the 3n-element span holds a read element


def _c4b(scale=1):
    m = (1 << 20) // scale
    return Workload("c4b_broadcast_f32", "f32", "(%d,16):(1,0)" % m, "(%d,16):(1,%d)" % (m, m), m, 16 * m, 16 * m,
                    "int_valued", "stride-0 broadcast of a vector into 16 rows", distinct_reads=m)


def _c5(scale=1):
    N, C, H, W = max(64 // scale, 1), 256, 256, 256
    if scale > 64:
        C = H = W = 256 // (scale // 64)
    src = "(%d,%d,%d,%d):(%d,%d,%d,1)" % (N, C, H, W, C * H * W, H * W, W)
    dst = "(%d,%d,%d,%d):(%d,1,%d,%d)" % (N, C, H, W, H * W * C, W * C, C)
    n = N * C * H * W
    return Workload("c5_nchw_to_nhwc_f32", "f32", src, dst, n, n, n, "uniform", "rank-4 fp32 permutation NCHW -> NHWC")


def _copy(scale=1):
    # not one of the BASELINE configs: a plain contiguous copy, used to calibrate the profiler's byte
    # counters and as the practical ceiling of any copy on this chip
    n = (1 << 28) // scale
    return Workload("c0_plain_copy_f32", "f32", "%d:1" % n, "%d:1" % n, n, n, n, "uniform", "contiguous copy (calibration)")


_MAKERS = {"c1": _c1, "c2": _c2, "c3": _c3, "c4a": _c4a, "c4b": _c4b, "c5": _c5, "copy": _copy}


def workload(name, scale=1):
    if name == "c2_literal":
        return _c2_literal()
    return _MAKERS[name](scale)


WORKLOAD_NAMES = ["c1", "c2", "c3", "c4a", "c4b", "c5"]


def _bf16_bits(x32):
    """float32 array -> bfloat16 bit patterns (round to nearest even), as uint16."""
    u = x32.view(np.uint32).astype(np.uint64)
    rounded = u + 0x7FFF + ((u >> 16) & 1)
    return (rounded >> 16).astype(np.uint16)


def source_bits(w, elems=None, chunk=1 << 24):
    """Seeded source buffer of the workload as raw bit patterns (uint16 / uint32 numpy array)."""
    elems = w.src_elems if elems is None else elems
    rng = np.random.default_rng(SEED_BASE + int(w.name[1]))   # one seed per BASELINE config (c1..c5)
    out = np.empty(elems, dtype=np.uint16 if w.elem_bytes == 2 else np.uint32)
    for lo in range(0, elems, chunk):
        hi = min(lo + chunk, elems)
        if w.values == "uniform":
            x = rng.uniform(-1.0, 1.0, hi - lo).astype(np.float32)
        elif w.values == "normal":
            x = rng.standard_normal(hi - lo, dtype=np.float32)
        else:  # integer-valued fp32 in [0, 2^20)
            x = rng.integers(0, 1 << 20, hi - lo).astype(np.float32)
        if w.dtype == "f32":
            out[lo:hi] = x.view(np.uint32)
        elif w.dtype == "f16":
            out[lo:hi] = x.astype(np.float16).view(np.uint16)
        else:
            out[lo:hi] = _bf16_bits(x)
    return out


# ---------------------------------------------------------------------------------------------
# GEMM workloads: stand-ins shaped like the rows of the paper's table of GEMM applications
# (Sec. 2.6.2): layouts as text, buffer sizes as plain numbers, seeded values.
# ---------------------------------------------------------------------------------------------
class GemmWorkload:
    def __init__(self, name, ab_dtype, a_layout, b_layout, c_layout, a_elems, b_elems, c_elems, M, N, K, values="normal", note="", L=1):
        self.name, self.ab_dtype = name, ab_dtype
        self.a_layout, self.b_layout, self.c_layout = a_layout, b_layout, c_layout
        self.a_elems, self.b_elems, self.c_elems = a_elems, b_elems, c_elems
        self.M, self.N, self.K, self.L = M, N, K, L
        self.values, self.note = values, note

    @property
    def flops(self):
        return 2 * self.M * self.N * self.K * self.L


def gemm_workload(name, M=8192, N=8192, K=8192, ab_dtype="bf16", values="normal"):
    if name == "tn":      # BLAS TN: both operands contiguous along k; C column-major
        return GemmWorkload("gemm_tn_" + ab_dtype, ab_dtype, "(%d,%d):(%d,1)" % (M, K, K), "(%d,%d):(%d,1)" % (N, K, K),
                            "(%d,%d):(1,%d)" % (M, N, M), M * K, N * K, M * N, M, N, K, values, "TN GEMM")
    if name == "nt":      # BLAS NT: both operands contiguous along m / n
        return GemmWorkload("gemm_nt_" + ab_dtype, ab_dtype, "(%d,%d):(1,%d)" % (M, K, M), "(%d,%d):(1,%d)" % (N, K, N),
                            "(%d,%d):(1,%d)" % (M, N, M), M * K, N * K, M * N, M, N, K, values, "NT GEMM")
    if name == "nn_rowmajor_c":   # A contiguous along m, B along k, C row-major (contiguous along n)
        return GemmWorkload("gemm_nn_rowc_" + ab_dtype, ab_dtype, "(%d,%d):(1,%d)" % (M, K, M), "(%d,%d):(%d,1)" % (N, K, K),
                            "(%d,%d):(%d,1)" % (M, N, N), M * K, N * K, M * N, M, N, K, values, "mixed operands, row-major C")
    if name == "gett":    # GETT: the row mode of A and C is the multi-mode (M1,M2) with a padded second stride
        M1 = 64
        M2 = M // M1
        W, Y = M1 + 8, M1 + 4
        X, Z = W * M2, Y * M2
        return GemmWorkload("gemm_gett_" + ab_dtype, ab_dtype, "((%d,%d),%d):((1,%d),%d)" % (M1, M2, K, W, X),
                            "(%d,%d):(%d,1)" % (N, K, K), "((%d,%d),%d):((1,%d),%d)" % (M1, M2, N, Y, Z),
                            X * K, N * K, Z * N, M1 * M2, N, K, values, "GETT with a folded, padded row mode")
    if name == "blis":    # general strides in every mode: no vector on any side
        dma, dka, dnb, dkb, dmc, dnc = 3, 3 * M + 1, 2 * K + 3, 2, 2, 2 * M + 1
        return GemmWorkload("gemm_blis_" + ab_dtype, ab_dtype, "(%d,%d):(%d,%d)" % (M, K, dma, dka), "(%d,%d):(%d,%d)" % (N, K, dnb, dkb),
                            "(%d,%d):(%d,%d)" % (M, N, dmc, dnc), dma * M + dka * K, dnb * N + dkb * K, dmc * M + dnc * N, M, N, K,
                            values, "BLIS-style general strides")
    raise KeyError(name)


def batched_gemm_workload(name, M, N, K, L, ab_dtype="bf16", values="normal"):
    """Rank-3 layouts of the batched form C(m,n,l) += A(m,k,l) B(n,k,l)."""
    if name == "strided_batch":   # the strided-batched BLAS extension: TN matrices one after the other, padded batch stride
        sa, sb, sc = M * K + 8, N * K + 16, M * N + 4
        return GemmWorkload("bgemm_strided_" + ab_dtype, ab_dtype, "(%d,%d,%d):(%d,1,%d)" % (M, K, L, K, sa),
                            "(%d,%d,%d):(%d,1,%d)" % (N, K, L, K, sb), "(%d,%d,%d):(1,%d,%d)" % (M, N, L, M, sc),
                            sa * L, sb * L, sc * L, M, N, K, values, "strided-batched TN GEMM", L)
    if name == "shared_b":        # one B for every batch entry (stride-0 batch mode), A and C with the batch innermost of the rows
        return GemmWorkload("bgemm_shared_b_" + ab_dtype, ab_dtype, "(%d,%d,%d):(1,%d,%d)" % (M, K, L, M * L, M),
                            "(%d,%d,%d):(%d,1,0)" % (N, K, L, K), "(%d,%d,%d):(1,%d,%d)" % (M, N, L, M * L, M),
                            M * K * L, N * K, M * N * L, M, N, K, values, "batch interleaved along the rows, B shared", L)
    if name == "folded_batch":    # a GETT with two batch indices folded into one mode, general strides (element loads)
        L1 = 2
        L2 = L // L1
        return GemmWorkload("bgemm_folded_" + ab_dtype, ab_dtype, "(%d,%d,(%d,%d)):(%d,1,(%d,%d))" % (M, K, L1, L2, K + 1, (K + 1) * M * L2, (K + 1) * M),
                            "(%d,%d,(%d,%d)):(1,%d,(%d,%d))" % (N, K, L1, L2, N + 3, (N + 3) * K, (N + 3) * K * L1),
                            "(%d,%d,(%d,%d)):(%d,1,(%d,%d))" % (M, N, L1, L2, N, M * N, M * N * L1),
                            (K + 1) * M * L1 * L2, (N + 3) * K * L1 * L2, M * N * L1 * L2, M, N, K, values, "folded batch mode", L1 * L2)
    raise KeyError(name)


def conv_gemm_workload(Nb, H, Wd, C, Kf, R, S, filters="kcrs", ab_dtype="bf16", values="normal"):
    """The CONV row of Table gemm (Sec. 2.6.2): a convolution of an NHWC activation as one GEMM.  A (Kf,(C,R,S)) are
    the filters, B ((Nb,P,Q),(C,R,S)) is the im2col view of the activation (no copy: P and R both step by an image row,
    Q and S by a pixel, so the layout repeats strides and is not injective), C (Kf,(Nb,P,Q)) is the N,P,Q,K output.
    filters: "kcrs" stores them K,C,R,S row-major (general strides along k: element loads), "krsc" K,R,S,C (channels
    contiguous on both sides: vector loads)."""
    P, Q = H - R + 1, Wd - S + 1
    sN, sH, sW = H * Wd * C, Wd * C, C
    if filters == "kcrs":
        a = "(%d,(%d,%d,%d)):(%d,(%d,%d,1))" % (Kf, C, R, S, C * R * S, R * S, S)
    else:
        a = "(%d,(%d,%d,%d)):(%d,(1,%d,%d))" % (Kf, C, R, S, C * R * S, S * C, C)
    b = "((%d,%d,%d),(%d,%d,%d)):((%d,%d,%d),(1,%d,%d))" % (Nb, P, Q, C, R, S, sN, sH, sW, sH, sW)
    c = "(%d,(%d,%d,%d)):(1,(%d,%d,%d))" % (Kf, Nb, P, Q, Kf * P * Q, Kf * Q, Kf)
    return GemmWorkload("gemm_conv_%s_%s" % (filters, ab_dtype), ab_dtype, a, b, c, Kf * C * R * S, Nb * H * Wd * C, Nb * P * Q * Kf,
                        Kf, Nb * P * Q, C * R * S, values, "convolution as a GEMM over an im2col view")


def _f16_bits(x32):
    return x32.astype(np.float16).view(np.uint16)


def gemm_operand_bits(w, which, elems=None):
    """Seeded bit patterns (uint16) of operand 'a' or 'b'; values N(0,1) or small integers."""
    elems = (w.a_elems if which == "a" else w.b_elems) if elems is None else elems
    rng = np.random.default_rng(SEED_BASE + 100 + (0 if which == "a" else 1))
    if w.values == "normal":
        x = rng.standard_normal(elems, dtype=np.float32)
    else:   # integers in [-4, 4]: every product and every partial sum is exact in fp32
        x = rng.integers(-4, 5, elems).astype(np.float32)
    return _bf16_bits(x) if w.ab_dtype == "bf16" else _f16_bits(x)


def gemm_c_values(w, elems=None):
    """Seeded initial contents of C (float32)."""
    elems = w.c_elems if elems is None else elems
    rng = np.random.default_rng(SEED_BASE + 102)
    if w.values == "normal":
        return rng.standard_normal(elems, dtype=np.float32)
    return rng.integers(-8, 9, elems).astype(np.float32)


def bits_to_float64(bits, ab_dtype):
    """Decode bf16 / f16 bit patterns exactly (both are subsets of float64)."""
    if ab_dtype == "bf16":
        return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return bits.view(np.float16).astype(np.float64)
