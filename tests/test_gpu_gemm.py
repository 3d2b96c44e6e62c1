"""GPU parity of the generic GEMM: the MFMA kernel (through the C ABI) against the CPU oracle on the same
seeded inputs.  Integer-valued inputs must agree exactly (every product and partial sum is exact in
fp32 whatever the order); N(0,1) inputs within K * 2^-23 * (|C0| + sum_k |A B|), the bound on fp32
accumulation of exact products in any order and rounding mode.  Run on the MI355X machine with `-m gpu`."""
import os

import numpy as np
import pytest

import paper_2603_02298_amd as lc
from paper_2603_02298_amd import workloads as W

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _plan_env(env):
    class Ctx:
        def __enter__(self):
            self.old = {k: os.environ.get(k) for k in env}
            os.environ.update({k: str(v) for k, v in env.items()})

        def __exit__(self, *a):
            for k, v in self.old.items():
                if v is None:
                    del os.environ[k]
                else:
                    os.environ[k] = v
    return Ctx()


def _gpu_gemm(w, a_bits, b_bits, c0, env=None):
    dev = torch.device("cuda:0")
    tdt = torch.bfloat16 if w.ab_dtype == "bf16" else torch.float16
    a_t = torch.from_numpy(a_bits.view(np.int16)).to(dev).view(tdt)
    b_t = torch.from_numpy(b_bits.view(np.int16)).to(dev).view(tdt)
    c_t = torch.from_numpy(c0.copy()).to(dev)
    with _plan_env(env or {}):
        desc = lc.GemmPlan(w.a_layout, w.b_layout, w.c_layout, w.ab_dtype).describe()
        print("case", w.name, (w.M, w.N, w.K), desc, flush=True)
        lc.gemm_tensor(a_t, w.a_layout, b_t, w.b_layout, c_t, w.c_layout)
    torch.cuda.synchronize()
    return c_t.cpu().numpy(), desc


def _parity(oracle, w, env=None):
    a, b, c0 = W.gemm_operand_bits(w, "a"), W.gemm_operand_bits(w, "b"), W.gemm_c_values(w)
    got, desc = _gpu_gemm(w, a, b, c0, env)
    a64, b64 = W.bits_to_float64(a, w.ab_dtype), W.bits_to_float64(b, w.ab_dtype)
    want = oracle.gemm(a64, w.a_layout, b64, w.b_layout, c0.astype(np.float64), w.c_layout)
    if w.values == "ints":
        assert (got.astype(np.float64) == want).all(), desc
    else:
        bound = oracle.gemm(np.abs(a64), w.a_layout, np.abs(b64), w.b_layout, np.abs(c0).astype(np.float64), w.c_layout)
        err = np.abs(got.astype(np.float64) - want)
        assert (err <= w.K * 2.0 ** -23 * bound).all(), (desc, float(err.max()))
        # entries outside the image of C's layout keep their bits
        touched = bound != np.abs(c0).astype(np.float64)
        assert (got[~touched] == c0[~touched]).all(), desc
    return desc


# sizes the oracle finishes in seconds; each spans several tiles of the chosen size and has ragged edges
CASES = [
    ("tn", (520, 392, 200)),
    ("nt", (392, 520, 136)),
    ("nn_rowmajor_c", (264, 300, 96)),
    ("gett", (320, 200, 72)),
    ("blis", (150, 133, 77)),
]


@pytest.mark.parametrize("values", ["ints", "normal"])
@pytest.mark.parametrize("tile", [128, 256])
@pytest.mark.parametrize("ktail", [0, 1])
@pytest.mark.parametrize("name,mnk", CASES)
def test_gemm_table_rows(oracle, name, mnk, tile, values, ktail):
    # K is no multiple of the k tile in any of these: ktail = 0 takes the tiles through registers (what lies past K is zeroed
    # there), ktail = 1 (the default) sends vector operands straight into LDS with zeros for the lanes past K
    w = W.gemm_workload(name, *mnk, ab_dtype="bf16", values=values)
    desc = _parity(oracle, w, {"LC_TUNE_GEMM_TILE": tile, "LC_TUNE_GEMM_KTAIL": ktail})
    assert "tile=%dx%d" % (tile, tile) in desc
    assert ("direct-to-LDS" in desc) == (ktail == 1 and name != "blis"), desc


@pytest.mark.parametrize("name,Ks", [("tn", (8, 24, 72, 200, 1000)), ("nt", (8, 40, 72, 136, 200, 1000)), ("nn_rowmajor_c", (40, 136)), ("gett", (16, 88))])
def test_gemm_short_last_k_tiles_on_the_direct_path(oracle, name, Ks):
    # the ring of LDS tiles with a last k tile that is short (from a single k on): the lanes past K present an offset out
    # of the buffer's range and zeros arrive in their slots
    for K in Ks:
        for tile in (128, 256):
            for values in ("ints", "normal"):
                w = W.gemm_workload(name, 304, 264, K, ab_dtype="bf16", values=values)
                desc = _parity(oracle, w, {"LC_TUNE_GEMM_TILE": tile})
                assert desc.count("direct-to-LDS") == 2 and "k_tiles=%d " % ((K + 63) // 64) in desc, desc
    w = W.gemm_workload(name, 136, 200, Ks[-1], ab_dtype="f16", values="ints")
    assert "direct-to-LDS" in _parity(oracle, w)


@pytest.mark.parametrize("values", ["ints", "normal"])
def test_gemm_direct_to_lds_loads(oracle, values):
    # K a multiple of 64 and k tiles inside one leaf of the k mode: vector operands bypass the registers on their way into
    # LDS (row-vector tiles are stored k-major and read back with the LDS transpose load)
    for name, mnk in (("tn", (520, 392, 256)), ("nt", (392, 520, 192)), ("nn_rowmajor_c", (264, 300, 128)), ("gett", (320, 200, 64))):
        for tile in (128, 256):
            w = W.gemm_workload(name, *mnk, ab_dtype="bf16", values=values)
            assert "direct-to-LDS" in _parity(oracle, w, {"LC_TUNE_GEMM_TILE": tile})
    w = W.gemm_workload("tn", 200, 136, 192, ab_dtype="f16", values=values)
    assert "direct-to-LDS" in _parity(oracle, w)
    assert "direct-to-LDS" not in _parity(oracle, w, {"LC_TUNE_GEMM_DIRECT": 0})
    w = W.gemm_workload("nt", 136, 200, 128, ab_dtype="f16", values=values)
    assert "direct-to-LDS" in _parity(oracle, w)
    for name in ("tn", "nt", "nn_rowmajor_c"):   # fp16 on the 256-tile kernels
        w = W.gemm_workload(name, 392, 520, 192, ab_dtype="f16", values=values)
        desc = _parity(oracle, w, {"LC_TUNE_GEMM_TILE": 256})
        assert desc.count("direct-to-LDS") == 2 and "tile=256x256" in desc
    # k modes of several leaves whose first leaf holds whole k tiles: the tile offset steps inside the leaf and is
    # evaluated afresh at its end (A: two tiles per run, B: one)
    M, N = 200, 136
    w = W.GemmWorkload("folded_k_direct", "bf16", "(%d,(128,3)):(408,(1,136))" % M, "(%d,(64,6)):(1,(%d,%d))" % (N, N, 64 * N + 8),
                       "(%d,%d):(1,%d)" % (M, N, M), (M - 1) * 408 + 127 + 2 * 136 + 1, N + 63 * N + 5 * (64 * N + 8), M * N, M, N, 384, values)
    for tile in (128, 256):
        assert _parity(oracle, w, {"LC_TUNE_GEMM_TILE": tile}).count("direct-to-LDS") == 2
    assert "direct-to-LDS" not in _parity(oracle, w, {"LC_TUNE_GEMM_DIRECT": 1})


@pytest.mark.parametrize("K", [64, 128, 192, 256, 320])
@pytest.mark.parametrize("name", ["tn", "nt", "nn_rowmajor_c"])
def test_gemm_ring_of_tiles_with_few_k_tiles(oracle, name, K):
    # 1 to 5 k tiles through the ring of five LDS slots: the prologue requests k tiles 0, 1 and A(2) whatever K is (past
    # the last tile it repeats it), the loop's first passes run on slots the prologue filled, and with 5 tiles the
    # slots come round once.  Both tile sizes, integer values (exact) and N(0,1).
    for tile in (128, 256):
        for values in ("ints", "normal"):
            w = W.gemm_workload(name, 304, 264, K, ab_dtype="bf16", values=values)
            desc = _parity(oracle, w, {"LC_TUNE_GEMM_TILE": tile})
            assert desc.count("direct-to-LDS") == 2 and "k_tiles=%d " % (K // 64) in desc, desc


def test_gemm_f16_and_element_loads(oracle):
    for values in ("ints", "normal"):
        w = W.gemm_workload("tn", 200, 136, 104, ab_dtype="f16", values=values)
        _parity(oracle, w)
        _parity(oracle, w, {"LC_TUNE_GEMM_LOAD": 2, "LC_TUNE_GEMM_CVEC": 0})
        w = W.gemm_workload("nt", 136, 200, 64, ab_dtype="f16", values=values)
        _parity(oracle, w)


@pytest.mark.parametrize("values", ["ints", "normal"])
def test_gemm_conv_row(oracle, values):
    # the CONV row of Table gemm: a convolution as one GEMM over the im2col view of the activation
    for args in ((2, 12, 10, 3, 20, 3, 2, "kcrs"), (2, 11, 9, 8, 40, 3, 2, "krsc"), (2, 14, 12, 64, 136, 3, 3, "krsc")):
        w = W.conv_gemm_workload(*args, values=values)
        desc = _parity(oracle, w)
        assert ("direct-to-LDS" in desc) == (args[3] == 64), desc


def test_gemm_degenerate_shapes(oracle):
    # a single row / column / k, and extents below one fragment
    for M, N, K in [(1, 1, 1), (1, 40, 8), (33, 1, 5), (8, 8, 8), (31, 33, 17)]:
        w = W.gemm_workload("blis", M, N, K, values="ints")
        _parity(oracle, w)
    w = W.gemm_workload("tn", 8, 16, 8, values="ints")
    _parity(oracle, w)
    w = W.gemm_workload("nt", 8, 16, 8, values="ints")
    _parity(oracle, w)


def test_gemm_hierarchical_k_broadcast_and_accumulate(oracle):
    M, N, K1, K2 = 64, 24, 16, 3
    w = W.GemmWorkload("gett2", "bf16", "(%d,(%d,%d)):(1,(%d,%d))" % (M, K1, K2, M, M * K1 + 8),
                       "(%d,(%d,%d)):(%d,(1,%d))" % (N, K1, K2, K1, K1 * N + 16), "(%d,%d):(1,%d)" % (M, N, M),
                       (M * K1 + 8) * K2, (K1 * N + 16) * K2, M * N, M, N, K1 * K2, "ints")
    _parity(oracle, w)
    w = W.GemmWorkload("bcast", "bf16", "(40,24):(24,1)", "(16,24):(0,1)", "(40,16):(16,1)", 960, 24, 640, 40, 16, 24, "ints")
    _parity(oracle, w)
    # two executions accumulate twice (the `+=` of the loop nest)
    w = W.gemm_workload("tn", 136, 72, 40, values="ints")
    a, b, c0 = W.gemm_operand_bits(w, "a"), W.gemm_operand_bits(w, "b"), W.gemm_c_values(w)
    dev = torch.device("cuda:0")
    a_t = torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)
    b_t = torch.from_numpy(b.view(np.int16)).to(dev).view(torch.bfloat16)
    c_t = torch.from_numpy(c0.copy()).to(dev)
    lc.gemm_tensor(a_t, w.a_layout, b_t, w.b_layout, c_t, w.c_layout)
    lc.gemm_tensor(a_t, w.a_layout, b_t, w.b_layout, c_t, w.c_layout)
    torch.cuda.synchronize()
    a64, b64 = W.bits_to_float64(a, "bf16"), W.bits_to_float64(b, "bf16")
    want = oracle.gemm(a64, w.a_layout, b64, w.b_layout, c0.astype(np.float64), w.c_layout)
    want = oracle.gemm(a64, w.a_layout, b64, w.b_layout, want, w.c_layout)
    assert (c_t.cpu().numpy().astype(np.float64) == want).all()


@pytest.mark.parametrize("values", ["ints", "normal"])
@pytest.mark.parametrize("name,mnkl", [("strided_batch", (264, 136, 72, 5)), ("shared_b", (128, 300, 40, 4)),
                                       ("folded_batch", (70, 45, 33, 6)),
                                       ("strided_batch", (264, 136, 192, 3)), ("shared_b", (128, 300, 64, 4))])   # direct loads
def test_batched_gemm(oracle, name, mnkl, values):
    # the batched form of Sec. 1 (rank-3 layouts): strided batch, a shared (stride-0) operand, a folded batch mode
    w = W.batched_gemm_workload(name, *mnkl, values=values)
    desc = _parity(oracle, w)
    assert "L=%d" % w.L in desc


@pytest.mark.parametrize("name", ["tn", "nt"])
def test_gemm_full_size_sampled(oracle, name):
    # the benchmark's problem (8192^3 bf16) in the launch configuration the bench times; the oracle
    # computes sampled entries of C one by one
    M = N = K = 8192
    for values in ("ints", "normal"):
        w = W.gemm_workload(name, M, N, K, values=values)
        a, b = W.gemm_operand_bits(w, "a"), W.gemm_operand_bits(w, "b")
        c0 = W.gemm_c_values(w)
        got, desc = _gpu_gemm(w, a, b, c0)
        assert "tile=256x256" in desc
        rng = np.random.default_rng(7)
        ms = np.concatenate([rng.integers(0, M, 300), [0, M - 1, 255, 256, 4095]])
        ns = np.concatenate([rng.integers(0, N, 300), [0, N - 1, 256, 255, 4096]])
        a64, b64, c64 = W.bits_to_float64(a, "bf16"), W.bits_to_float64(b, "bf16"), c0.astype(np.float64)
        want = oracle.gemm_at(a64, w.a_layout, b64, w.b_layout, c64, w.c_layout, ms, ns)
        have = got[ms + M * ns].astype(np.float64)       # C is (M,N):(1,M)
        if values == "ints":
            assert (have == want).all(), desc
        else:
            bound = oracle.gemm_at(np.abs(a64), w.a_layout, np.abs(b64), w.b_layout, np.abs(c64), w.c_layout, ms, ns)
            assert (np.abs(have - want) <= K * 2.0 ** -23 * bound).all(), desc
