"""The GEMM planner and the kernel's index arithmetic, checked on the host (no GPU): plans are walked
with the library's checking device (every global access bounds-checked, tiles through a model of the
LDS arrangement and of the MFMA fragment layouts) and the result is compared with the oracle."""
import os

import numpy as np
import pytest

import paper_2603_02298_amd as lc
from paper_2603_02298_amd import workloads as W


def _walk_and_compare(oracle, w, env=None, expect=None):
    env = env or {}
    old = {k: os.environ.get(k) for k in env}
    os.environ.update({k: str(v) for k, v in env.items()})
    try:
        plan = lc.GemmPlan(w.a_layout, w.b_layout, w.c_layout, w.ab_dtype)
    finally:
        for k, v in old.items():
            if v is None:
                del os.environ[k]
            else:
                os.environ[k] = v
    text = plan.describe()
    for piece in (expect or []):
        assert piece in text, (piece, text)
    a, b, c0 = W.gemm_operand_bits(w, "a"), W.gemm_operand_bits(w, "b"), W.gemm_c_values(w)
    got = plan.debug_replay_on_host(a, b, c0.copy())
    want = oracle.gemm(W.bits_to_float64(a, w.ab_dtype), w.a_layout, W.bits_to_float64(b, w.ab_dtype), w.b_layout,
                       c0.astype(np.float64), w.c_layout)
    assert (got.astype(np.float64) == want).all(), text     # integer-valued inputs: every sum is exact
    return text


CASES = [
    # name, (M, N, K), pieces the plan's description must contain
    ("tn", (200, 136, 96), ["a_load=k-vectors", "b_load=k-vectors", "c_vec=1", "exchanged=0"]),
    ("nt", (136, 264, 72), ["a_load=row-vectors+transpose", "b_load=row-vectors+transpose", "c_vec=1"]),
    ("nn_rowmajor_c", (72, 140, 40), ["exchanged=1", "c_vec=1", "a_load=k-vectors", "b_load=row-vectors+transpose"]),
    ("gett", (192, 100, 48), ["a_load=row-vectors+transpose", "b_load=k-vectors", "c_vec=1"]),
    ("blis", (70, 45, 37), ["a_load=elements", "b_load=elements", "c_vec=0"]),
]


@pytest.mark.parametrize("name,mnk,expect", CASES)
@pytest.mark.parametrize("tile", [128, 256])
@pytest.mark.parametrize("ktail", [0, 1])
def test_walk_matches_oracle(oracle, name, mnk, expect, tile, ktail):
    # K is no multiple of the k tile in any of these.  ktail = 0: tiles pass through registers, what lies past K is zeroed
    # there; ktail = 1 (the default): vector operands still go straight into LDS, the lanes past K are answered with zeros
    w = W.gemm_workload(name, *mnk, ab_dtype="bf16", values="ints")
    text = _walk_and_compare(oracle, w, {"LC_TUNE_GEMM_TILE": tile, "LC_TUNE_GEMM_KTAIL": ktail}, expect + ["tile=%dx%d" % (tile, tile)])
    assert ("direct-to-LDS" in text) == (ktail == 1 and name != "blis"), text


def test_walk_short_last_k_tiles_on_the_direct_path(oracle):
    # K from a single vector to several tiles plus a remainder; K a multiple of 8 (no k vector may straddle K; row vectors
    # come in blocks of 8 k)
    for name, Ks in (("tn", (8, 24, 72, 200)), ("nt", (8, 40, 72, 136, 200)), ("nn_rowmajor_c", (40, 136)), ("gett", (16, 88))):
        for K in Ks:
            for tile in (128, 256):
                w = W.gemm_workload(name, 200, 136, K, ab_dtype="bf16", values="ints")
                text = _walk_and_compare(oracle, w, {"LC_TUNE_GEMM_TILE": tile})
                assert text.count("direct-to-LDS") == 2 and "k_tiles=%d " % ((K + 63) // 64) in text, text
    w = W.gemm_workload("tn", 200, 136, 100, ab_dtype="bf16", values="ints")     # 100 = 8 * 12 + 4: a k vector would straddle K
    assert "direct" not in _walk_and_compare(oracle, w, None)


def test_walk_direct_to_lds_loads(oracle):
    # whole k tiles (K a multiple of 64, k tiles one leaf of the k mode): vector operands go straight into LDS, k-vector
    # tiles row-major, row-vector tiles k-major and read back with the LDS transpose load; the walk checks that every
    # lane's 16 bytes land in the slot the fragment reads expect, and applies the transpose load's definition
    kd, rd = "k-vectors(direct-to-LDS)", "row-vectors+transpose(direct-to-LDS)"
    for name, mnk, pieces in (("tn", (200, 136, 128), ["a_load=" + kd, "b_load=" + kd]),
                              ("nt", (136, 264, 128), ["a_load=" + rd, "b_load=" + rd]),
                              ("nn_rowmajor_c", (72, 140, 64), ["a_load=" + kd, "b_load=" + rd]),
                              ("gett", (192, 100, 64), ["a_load=" + rd, "b_load=" + kd])):
        for tile in (128, 256):
            w = W.gemm_workload(name, *mnk, ab_dtype="bf16", values="ints")
            _walk_and_compare(oracle, w, {"LC_TUNE_GEMM_TILE": tile}, pieces)
    w = W.gemm_workload("tn", 200, 136, 128, ab_dtype="bf16", values="ints")
    assert "direct" not in _walk_and_compare(oracle, w, {"LC_TUNE_GEMM_DIRECT": 0})
    # k modes of several leaves whose first leaf holds whole k tiles: the tile offset steps inside the leaf and is
    # evaluated afresh at its end (A: two tiles per run, B: one)
    M, N = 200, 136
    w = W.GemmWorkload("folded_k_direct", "bf16", "(%d,(128,3)):(408,(1,136))" % M, "(%d,(64,6)):(1,(%d,%d))" % (N, N, 64 * N + 8),
                       "(%d,%d):(1,%d)" % (M, N, M), (M - 1) * 408 + 127 + 2 * 136 + 1, N + 63 * N + 5 * (64 * N + 8), M * N, M, N, 384, "ints")
    _walk_and_compare(oracle, w, None, ["a_load=" + kd, "b_load=" + rd])
    # the two kinds can be switched off separately (bit 0: k vectors, bit 1: row vectors); a pair goes direct together or not at all
    w = W.gemm_workload("nt", 136, 264, 64, ab_dtype="f16", values="ints")
    assert "direct" not in _walk_and_compare(oracle, w, {"LC_TUNE_GEMM_DIRECT": 1})
    assert "direct" in _walk_and_compare(oracle, w, {"LC_TUNE_GEMM_DIRECT": 2})
    w = W.gemm_workload("nn_rowmajor_c", 72, 140, 64, ab_dtype="bf16", values="ints")
    assert "direct" not in _walk_and_compare(oracle, w, {"LC_TUNE_GEMM_DIRECT": 1})


def test_walk_batched_direct_loads(oracle):
    # rank-3 layouts on the direct path: the batch offset is folded into the base the buffer loads start from
    for name, mnkl in (("strided_batch", (136, 72, 128, 3)), ("shared_b", (128, 140, 64, 2))):
        w = W.batched_gemm_workload(name, *mnkl, values="ints")
        text = _walk_and_compare(oracle, w)
        assert text.count("direct-to-LDS") == 2 and "L=%d" % w.L in text, text


def test_walk_conv_row(oracle):
    # the CONV row of Table gemm: B is the im2col view of the activation (repeated strides, not injective: fine for an
    # operand that is only read).  Filters K,C,R,S: general strides along k, element loads; filters K,R,S,C with 64
    # channels: both operands lead with whole k tiles of contiguous channels and go straight into LDS
    w = W.conv_gemm_workload(2, 6, 5, 3, 4, 3, 2, "kcrs", values="ints")
    _walk_and_compare(oracle, w, None, ["a_load=elements", "b_load=elements", "M=4 N=32 K=18"])
    w = W.conv_gemm_workload(2, 7, 6, 8, 40, 3, 2, "krsc", values="ints")
    _walk_and_compare(oracle, w, None, ["a_load=k-vectors", "b_load=k-vectors", "c_vec=1"])
    w = W.conv_gemm_workload(1, 5, 9, 64, 72, 2, 3, "krsc", values="ints")
    text = _walk_and_compare(oracle, w, None, ["a_load=k-vectors(direct-to-LDS)", "b_load=k-vectors(direct-to-LDS)"])
    assert "K=384" in text


def test_walk_f16_and_forced_element_loads(oracle):
    w = W.gemm_workload("tn", 130, 70, 40, ab_dtype="f16", values="ints")
    _walk_and_compare(oracle, w, {"LC_TUNE_GEMM_TILE": 128}, ["ab=f16"])
    _walk_and_compare(oracle, w, {"LC_TUNE_GEMM_TILE": 128, "LC_TUNE_GEMM_LOAD": 2, "LC_TUNE_GEMM_CVEC": 0},
                      ["a_load=elements", "b_load=elements", "c_vec=0"])


def test_walk_group_and_xcd_mapping_cover_every_tile_once(oracle):
    # 3 x 5 tiles of 128: neither a multiple of the group height nor of the 8 XCDs
    w = W.gemm_workload("tn", 300, 600, 16, ab_dtype="bf16", values="ints")
    for g in (1, 2, 4):
        _walk_and_compare(oracle, w, {"LC_TUNE_GEMM_TILE": 128, "LC_TUNE_GEMM_GROUP_M": g}, ["tiles=3x5"])


def test_hierarchical_k_and_broadcast_operand(oracle):
    # GETT row 2 of the table: K folded as (K1,K2) with different leading leaves in A and B; and a
    # stride-0 row mode in B (every n reads the same row)
    M, N, K1, K2 = 64, 24, 16, 3
    w = W.GemmWorkload("gett2", "bf16", "(%d,(%d,%d)):(1,(%d,%d))" % (M, K1, K2, M, M * K1 + 8),
                       "(%d,(%d,%d)):(%d,(1,%d))" % (N, K1, K2, K1, K1 * N + 16), "(%d,%d):(1,%d)" % (M, N, M),
                       (M * K1 + 8) * K2, (K1 * N + 16) * K2, M * N, M, N, K1 * K2, "ints")
    _walk_and_compare(oracle, w, {"LC_TUNE_GEMM_TILE": 128}, ["a_load=row-vectors+transpose", "b_load=k-vectors"])
    w = W.GemmWorkload("bcast", "bf16", "(40,24):(24,1)", "(16,24):(0,1)", "(40,16):(16,1)", 960, 24, 640, 40, 16, 24, "ints")
    _walk_and_compare(oracle, w, {"LC_TUNE_GEMM_TILE": 128}, ["exchanged=1"])


@pytest.mark.parametrize("name,mnkl,expect", [
    ("strided_batch", (136, 72, 40, 3), ["L=3", "a_load=k-vectors", "b_load=k-vectors", "c_vec=1"]),
    ("shared_b", (64, 40, 24, 4), ["L=4", "a_load=row-vectors+transpose", "b_load=k-vectors", "c_vec=1"]),
    ("folded_batch", (33, 20, 9, 6), ["L=6", "a_load=elements", "exchanged=1"]),
])
def test_walk_batched_matches_oracle(oracle, name, mnkl, expect):
    # the batched form of Sec. 1: rank-3 layouts, the batch index is the second grid dimension
    w = W.batched_gemm_workload(name, *mnkl, values="ints")
    assert oracle.gemm_sizes(w.a_layout, w.b_layout, w.c_layout) == (w.M, w.N, w.K, w.L)
    _walk_and_compare(oracle, w, {"LC_TUNE_GEMM_TILE": 128}, expect)


def test_fragment_layouts_are_the_thread_value_layouts():
    a, b, c = (lc.lc_mfma_fragment_layout(i) for i in range(3))
    assert str(a) == "((32,2),8):((1,256),32)" and str(b) == str(a) and str(c) == "((32,2),(4,4)):((32,4),(1,8))"
    # each is a bijection of (lane, value) onto the fragment's tile
    assert sorted(a(i) for i in range(512)) == list(range(512))
    assert sorted(c(i) for i in range(1024)) == list(range(1024))
    # a lane's values of A are 8 consecutive k of one row; of C, four runs of 4 consecutive rows of one column
    for lane in (0, 5, 31, 32, 63):
        ks = [a(lane + 64 * v) // 32 for v in range(8)]
        assert ks == list(range(8 * (lane // 32), 8 * (lane // 32) + 8)) and {a(lane + 64 * v) % 32 for v in range(8)} == {lane % 32}
        rows = [c(lane + 64 * v) % 32 for v in range(16)]
        assert rows == [8 * (v // 4) + 4 * (lane // 32) + v % 4 for v in range(16)]
        assert {c(lane + 64 * v) // 32 for v in range(16)} == {lane % 32}


def test_preconditions_and_refusals():
    def status(*args, **kw):
        with pytest.raises(lc.LayoutCopyError) as e:
            lc.GemmPlan(*args, **kw)
        return e.value.status_name
    assert status("(4,3):(1,4)", "(5,3):(1,5)", "(3,5):(1,3)") == "SIZE_MISMATCH"
    assert status("(4,3):(1,4)", "(5,3):(1,5)", "(4,6):(1,4)") == "SIZE_MISMATCH"
    assert status("(4,3):(1,4)", "(5,2):(1,5)", "(4,5):(1,4)") == "SIZE_MISMATCH"
    assert status("12:1", "(5,3):(1,5)", "(4,5):(1,4)") == "INVALID_ARG"
    assert status("(4,3,2):(1,4,12)", "(5,3):(1,5)", "(4,5,2):(1,4,20)") == "INVALID_ARG"            # ranks differ
    assert status("(4,3,2):(1,4,12)", "(5,3,3):(1,5,15)", "(4,5,2):(1,4,20)") == "SIZE_MISMATCH"     # batch sizes differ
    assert status("(4,3,2):(1,4,12)", "(5,3,2):(1,5,15)", "(4,5,2):(1,4,0)") == "DST_ALIASES"        # every batch entry into one C
    assert status("(4,3):(1,4)", "(5,3):(1,5)", "(4,5):(0,1)") == "DST_ALIASES"
    assert status("(4,3):(1,4)", "(5,3):(1,5)", "(4,5):(1,4)", "f32") == "UNSUPPORTED_DTYPE"
    assert status("(4,3):(1,%d)" % (1 << 30), "(5,3):(1,5)", "(4,5):(1,4)") == "TOO_LARGE"
    # less aligned pointers than vectors need: the planner falls back to element loads (for both operands
    # together) and scalar updates of C instead of refusing
    p = lc.GemmPlan("(64,64):(64,1)", "(64,64):(64,1)", "(64,64):(1,64)", "bf16", a_align=2, b_align=16, c_align=4)
    assert "a_load=elements" in p.describe() and "b_load=elements" in p.describe() and "c_vec=0" in p.describe()
    p = lc.GemmPlan("(64,64):(64,1)", "(64,64):(64,1)", "(64,64):(1,64)", "bf16", a_align=16, b_align=16, c_align=4)
    assert "a_load=k-vectors" in p.describe() and "b_load=k-vectors" in p.describe() and "c_vec=0" in p.describe()
    assert p.flops == 2 * 64 ** 3
    # execution checks the pointers against what the plan relies on before anything is launched (the addresses below
    # are never dereferenced: both calls return at the check)
    p = lc.GemmPlan("(64,64):(64,1)", "(64,64):(64,1)", "(64,64):(1,64)", "bf16")
    for ptrs in ((0x10000 + 2, 0x20000, 0x30000), (0x10000, 0x20000 + 8, 0x30000), (0x10000, 0x20000, 0x30000 + 4)):
        with pytest.raises(lc.LayoutCopyError) as e:
            p.execute(*ptrs)
        assert e.value.status_name == "MISALIGNED"
    with pytest.raises(lc.LayoutCopyError) as e:
        p.execute(0, 0x20000, 0x30000)
    assert e.value.status_name == "INVALID_ARG"


def test_lds_arrangements_are_xor_layouts_without_bank_conflicts(oracle):
    # Both LDS tile arrangements of the GEMM kernels are layouts with XOR strides (Sec. 2.3.2) over the bits of their
    # coordinates, in units of 16 bytes; and under the bank model (64 banks of 4 bytes, 256 bytes per pass) the fragment
    # reads of either arrangement touch every bank once per pass.
    from paper_2603_02298_amd.binding import lib
    addr = lib().lc_debug_gemm_lds_address
    # row-major tile: unit = 8 row + ((kv ^ row ^ (row >> 3)) & 7), coordinate (kv, row), 256 rows
    text = "((2,2,2),(2,2,2,2,2,2,2,2)):((f1,f2,f4),(f9,f18,f36,f65,f130,f260,f512,f1024))"
    for S in (oracle.SLayout, lc.SLayout):
        L = S(text)
        for row in range(256):
            for kv in range(8):
                assert 16 * L(kv + 8 * row) == addr(0, 256, 0, row, kv), (row, kv)
    # k-major tile of 256 rows (32 groups of 8 rows per k): unit = 32 k + (group ^ 4 (k mod 4)), coordinate (group, k)
    text = "((2,2,2,2,2),(2,2,2,2,2,2)):((f1,f2,f4,f8,f16),(f36,f72,f128,f256,f512,f1024))"
    for S in (oracle.SLayout, lc.SLayout):
        L = S(text)
        for k in range(64):
            for group in range(32):
                assert 16 * L(group + 32 * k) == addr(1, 256, 0, k, 8 * group), (k, group)
    # ... and of 128 rows (16 groups): the XOR reaches the top two bits of the group
    L = lc.SLayout("((2,2,2,2),(2,2,2,2,2,2)):((f1,f2,f4,f8),(f20,f40,f64,f128,f256,f512))")
    for k in range(64):
        for group in range(16):
            assert 16 * L(group + 16 * k) == addr(1, 128, 0, k, 8 * group), (k, group)

    def banks(byte_ranges):
        hit = []
        for lo, n in byte_ranges:
            assert lo % 4 == 0
            hit += [(lo // 4 + d) % 64 for d in range(n // 4)]
        return hit

    # one 16-byte read per lane, 16 lanes per pass: 16 consecutive fragment rows, one k vector
    for row0 in range(0, 256, 16):
        for kv in range(8):
            assert sorted(banks([(addr(0, 256, 0, row0 + r, kv), 16) for r in range(16)])) == list(range(64))
    # the direct loads fill 1 KiB contiguously: nothing to check.  Staged k-vector parks: lanes 0..15 = 2 rows x 8 vectors
    for row0 in range(0, 256, 2):
        assert sorted(banks([(addr(0, 256, 0, row0 + l // 8, l % 8), 16) for l in range(16)])) == list(range(64))
    # transpose loads: 8 bytes per lane, 32 lanes per pass (either half of the wavefront)
    for rows in (128, 256):
        for row_base in range(0, rows, 32):
            for k_base in range(0, 64, 4):
                for half in (0, 32):
                    got = banks([(addr(2, rows, half + l, row_base, k_base), 8) for l in range(32)])
                    assert sorted(got) == list(range(64)), (rows, row_base, k_base, half)
