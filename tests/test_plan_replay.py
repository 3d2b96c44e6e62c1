"""The planner's routing, proven without a GPU: every plan is walked on the host along the same
index arithmetic the kernels use (bounds-checked) and compared bit for bit with the oracle's COPY."""
import numpy as np
import pytest

import paper_2603_02298_amd as lc
from paper_2603_02298_amd import workloads as W


def _np_dtype(es):
    return {1: np.uint8, 2: np.uint16, 4: np.uint32, 8: np.uint64}[es]


def _check(oracle, src_layout, dst_layout, dtype, expect_class=None, seed=0):
    es = lc.DTYPE_BYTES[dtype]
    sl, dl = oracle.Layout(src_layout), oracle.Layout(dst_layout)
    rng = np.random.default_rng(seed)
    src = rng.integers(0, 255, size=sl.cosize * es, dtype=np.uint8).view(_np_dtype(es))
    want = np.full(dl.cosize, 0xA5A5A5A5A5A5A5A5 & ((1 << (8 * es)) - 1), dtype=_np_dtype(es))
    got = want.copy()
    oracle.copy(src, sl, want, dl)
    plan = lc.Plan(src_layout, dst_layout, dtype)
    desc = plan.describe()
    if expect_class:
        assert ("class=" + expect_class) in desc, desc
    conflicts = plan.debug_replay_on_host(src, got)
    assert (got == want).all(), desc
    return desc, conflicts


def test_fast_division_is_exact():
    # the kernels' division by a constant, checked through a plan whose only job is idx2crd: a
    # generic-class copy between shapes without common refinement exercises it on every element
    import ctypes
    from paper_2603_02298_amd.binding import lib
    assert lib() is not None
    rng = np.random.default_rng(1)
    # white-box: same formula as kernel_params.hpp, on random 31-bit operands
    for d in [1, 2, 3, 5, 7, 12, 64, 125, 1000, 65535, 65536, 65537, (1 << 31) - 1] + [int(x) for x in rng.integers(1, 1 << 31, 200)]:
        l = 0
        while (1 << l) < d:
            l += 1
        mul = (((1 << l) - d) << 32) // d + 1
        assert mul < (1 << 32)
        ns = np.concatenate([rng.integers(0, 1 << 31, 2000), np.array([0, 1, d - 1, d, d + 1, (1 << 31) - 1])]).astype(np.uint64)
        q = (((ns * np.uint64(mul)) >> np.uint64(32)) + ns) >> np.uint64(l)
        assert (q == ns // np.uint64(d)).all(), d


@pytest.mark.parametrize("name,scale,cls", [
    ("c1", 1, "transpose"), ("c1", 16, "transpose"), ("c2", 4, "transpose"), ("c2", 16, "transpose"),
    ("c3", 16, "transpose"), ("c4a", 64, "direct"), ("c4b", 16, "direct"), ("c5", 256, "transpose")])
def test_workloads_at_reduced_size(oracle, name, scale, cls):
    w = W.workload(name, scale)
    desc, conflicts = _check(oracle, w.src_layout, w.dst_layout, w.dtype, cls)
    if cls == "transpose":
        assert "width_bytes=16" in desc
        assert conflicts == 0, desc          # the chosen XOR swizzle is conflict-free in the bank model


def test_full_size_plans_have_expected_shape():
    # plan creation is pure host work: the full-size workloads can be planned here
    expect = {"c1": ("transpose", 16), "c2": ("transpose", 16), "c3": ("transpose", 16), "c4a": ("direct", 4),
              "c4b": ("direct", 16), "c5": ("transpose", 16)}
    for name, (cls, width) in expect.items():
        w = W.workload(name)
        d = lc.Plan(w.src_layout, w.dst_layout, w.dtype).describe()
        assert "class=%s " % cls in d and "width_bytes=%d " % width in d, d
        assert lc.Plan(w.src_layout, w.dst_layout, w.dtype).algorithmic_bytes == w.algorithmic_bytes


def test_copy_applications_table(oracle):
    from conftest import golden_lines
    for ln in golden_lines("copy_applications.txt"):
        name, s, d = [x.strip() for x in ln.split("|")]
        for dt in ("f32", "bf16", "b8", "b64"):
            desc, _ = _check(oracle, s, d, dt)
            # "Constant": every coordinate writes the one element; the loop's last write is what stays
            assert ("overwritten_modes=1" in desc) == (name == "Constant"), desc


def _random_pair(rng):
    n = int(rng.integers(1, 5))
    ext = [int(rng.choice([1, 2, 3, 4, 5, 6, 8, 12, 16])) for _ in range(n)]

    def strides(allow_zero):
        d, run = [0] * n, 1
        for m in rng.permutation(n):
            d[m] = run
            run *= ext[m] * int(rng.choice([1, 1, 1, 2, 3]))
        if allow_zero and rng.random() < 0.2:
            d[int(rng.integers(n))] = 0
        return d

    def text(exts, ds):
        # random regrouping of neighbouring modes, and random merging of compatible neighbours
        parts, i = [], 0
        while i < len(exts):
            j = min(len(exts), i + int(rng.integers(1, 3)))
            if j - i == 1:
                parts.append((str(exts[i]), str(ds[i])))
            else:
                parts.append(("(%s)" % ",".join(map(str, exts[i:j])), "(%s)" % ",".join(map(str, ds[i:j]))))
            i = j
        if len(parts) == 1:
            return "%s:%s" % parts[0]
        return "(%s):(%s)" % (",".join(p[0] for p in parts), ",".join(p[1] for p in parts))
    return text(ext, strides(True)), text(ext, strides(False))


def _random_refined_pair(rng):
    """Source and destination shapes that differ but share a refinement: a list of small factors is
    grouped into modes differently on each side (e.g. (6,4) against (2,12)); strides are compact over
    a random order of each side's own modes, sometimes padded."""
    nf = int(rng.integers(2, 6))
    factors = [int(rng.choice([2, 2, 2, 3, 4, 5, 8])) for _ in range(nf)]

    def side():
        modes, i = [], 0
        while i < nf:
            j = min(nf, i + int(rng.integers(1, 4)))
            e = 1
            for f in factors[i:j]:
                e *= f
            modes.append(e)
            i = j
        d, run = [0] * len(modes), 1
        for m in rng.permutation(len(modes)):
            d[m] = run
            run *= modes[m] * int(rng.choice([1, 1, 1, 2]))
        if len(modes) == 1:
            return "%d:%d" % (modes[0], d[0])
        return "(%s):(%s)" % (",".join(map(str, modes)), ",".join(map(str, d)))
    return side(), side()


def test_random_pairs_with_different_shapes(oracle):
    rng = np.random.default_rng(314)
    seen = {"generic": 0, "direct": 0, "transpose": 0}
    for k in range(1200):
        s, d = _random_refined_pair(rng)
        desc, _ = _check(oracle, s, d, ["f32", "bf16", "b64", "b8"][k % 4], seed=k)
        assert "note=\"shapes have no common refinement\"" not in desc, (s, d)
        seen[desc.split()[0][6:]] += 1
    assert seen["direct"] > 100 and seen["transpose"] > 100, seen


def test_random_layout_pairs(oracle):
    rng = np.random.default_rng(42)
    seen = {"generic": 0, "direct": 0, "transpose": 0}
    for k in range(1500):
        s, d = _random_pair(rng)
        dt = ["f32", "bf16", "b8", "b64", "f16"][k % 5]
        desc, _ = _check(oracle, s, d, dt, seed=k)
        seen[desc.split()[0][6:]] += 1
    assert seen["direct"] > 100 and seen["transpose"] > 100, seen


def _inner_kept_permutation(rng, es):
    """Permutation of 3-5 modes that keeps a short innermost mode in place: the common vector is a few
    16-byte words long and the copy re-orders those words (p = q)."""
    words = int(rng.choice([1, 2, 4, 8, 16]))
    inner = words * 16 // es
    n_outer = int(rng.integers(2, 5))
    ext = [inner] + [int(rng.choice([2, 3, 4, 6, 8, 12, 16, 24, 32])) for _ in range(n_outer)]
    def compact(order):
        st, run = [0] * len(ext), 1
        for m in order:
            st[m] = run
            run *= ext[m]
        return st
    so = [0] + [int(x) + 1 for x in rng.permutation(n_outer)]
    do = [0] + [int(x) + 1 for x in rng.permutation(n_outer)]
    shape = "(" + ",".join(map(str, ext)) + ")"
    return shape + ":(" + ",".join(map(str, compact(so))) + ")", shape + ":(" + ",".join(map(str, compact(do))) + ")"


def test_word_level_tiles(oracle, monkeypatch):
    # permutations that keep a short innermost mode: tiles of 16-byte words through LDS (V = 1);
    # the planner takes that route by itself from 256 tiles on (checked in the full-size plans), here it is forced
    monkeypatch.setenv("LC_TUNE_FORCE_CLASS", "2")
    desc, _ = _check(oracle, "(64,32,32,4):(1,64,2048,65536)", "(64,32,32,4):(1,2048,64,65536)", "bf16", "transpose")
    assert "V=1 tile_elem_bytes=16" in desc, desc
    desc, _ = _check(oracle, "(32,64,16,6):(1,32,2048,32768)", "(32,64,16,6):(1,512,32,32768)", "f32", "transpose")
    assert "V=1 tile_elem_bytes=16" in desc, desc
    for per_lane in (2, 4, 8):     # the tile sizes of the full-size plans
        monkeypatch.setenv("LC_TUNE_MICRO_PER_THREAD", str(per_lane))
        desc, _ = _check(oracle, "(64,32,32,4):(1,64,2048,65536)", "(64,32,32,4):(1,2048,64,65536)", "bf16", "transpose")
        assert "V=1 tile_elem_bytes=16" in desc and ("per_lane=%d" % per_lane) in desc, desc
    monkeypatch.delenv("LC_TUNE_MICRO_PER_THREAD")
    rng = np.random.default_rng(77)
    staged = 0
    for i in range(300):
        dt = ["bf16", "f32", "b8", "b64"][i % 4]
        s, d = _inner_kept_permutation(rng, lc.DTYPE_BYTES[dt])
        desc, _ = _check(oracle, s, d, dt, seed=i)
        staged += "tile_elem_bytes=16" in desc
    assert staged > 40, staged
    monkeypatch.delenv("LC_TUNE_FORCE_CLASS")
    # by itself: an attention-head permute (B,S,H,D) -> (B,H,S,D) with 128-byte heads; longer common vectors stay direct
    desc = lc.Plan("(64,32,4096,8):(1,64,2048,8388608)", "(64,32,4096,8):(1,262144,64,8388608)", "bf16").describe()
    assert "class=transpose" in desc and "V=1 tile_elem_bytes=16" in desc and "src_run_bytes=2048" in desc, desc
    desc = lc.Plan("(128,32,4096,8):(1,128,4096,16777216)", "(128,32,4096,8):(1,524288,128,16777216)", "bf16").describe()
    assert "class=direct" in desc, desc


def test_ragged_tiles(oracle):
    # extents the tile does not divide: ceil(extent / tile) tiles along the mode, coordinates checked at the edge
    for s, d, dt, want in [
        ("(67,71):(1,67)", "(67,71):(71,1)", "f32", "V=1 tile_elem_bytes=4"),          # odd transpose, no vector at all
        ("(131,77):(1,131)", "(131,77):(77,1)", "bf16", "V=1 tile_elem_bytes=2"),
        ("(45,33):(1,45)", "(45,33):(33,1)", "b8", "V=1 tile_elem_bytes=1"),
        ("(37,41):(1,37)", "(37,41):(41,1)", "b64", "V=1 tile_elem_bytes=8"),
        ("(2006,26):(1,2006)", "(2006,26):(26,1)", "f32", "V=2"),                       # 2006 = 2 * 17 * 59: whole tiles would be slivers
        ("(328,1016):(1,328)", "(328,1016):(1016,1)", "bf16", "V=8"),                   # 1016 = 8 * 127
        ("(66,50,3):(1,66,3300)", "(66,50,3):(50,1,3300)", "f32", "V=2"),                # batched
        ("(67,71,5):(1,67,4757)", "(67,71,5):(71,1,4757)", "f32", "V=1"),                 # batched, two ragged modes
    ]:
        desc, _ = _check(oracle, s, d, dt, "transpose")
        assert want in desc and "ragged_modes=0" not in desc, desc
    # power-of-two shapes keep whole tiles and the pipelined kernel
    desc, _ = _check(oracle, "(64,128):(1,64)", "(64,128):(128,1)", "f32", "transpose")
    assert "ragged_modes=0" in desc and "V=4" in desc, desc
    rng = np.random.default_rng(99)
    ragged = 0
    for i in range(250):
        M, N = int(rng.integers(9, 200)), int(rng.integers(9, 200))
        B = int(rng.choice([1, 1, 2, 3]))
        dt = ["f32", "bf16", "b8", "b64"][i % 4]
        pad = int(rng.choice([0, 0, 1, 5]))
        s = "(%d,%d,%d):(1,%d,%d)" % (M, N, B, M + pad, (M + pad) * N)
        d = "(%d,%d,%d):(%d,1,%d)" % (M, N, B, N, M * N)
        desc, _ = _check(oracle, s, d, dt, seed=i)
        ragged += "class=transpose" in desc and "ragged_modes=0" not in desc
    assert ragged > 150, ragged


def test_shapes_without_common_refinement_use_generic_class(oracle):
    for s, d in [("(2,3):(3,1)", "(3,2):(2,1)"), ("(4,9):(9,1)", "(6,6):(1,6)"), ("(5,7,3):(21,3,1)", "(3,35):(1,3)")]:
        desc, _ = _check(oracle, s, d, "f32")
    desc, _ = _check(oracle, "(6,10):(10,1)", "(4,15):(15,1)", "f32", "generic")


def test_large_copies_are_sliced_into_launches(oracle, monkeypatch):
    # work items are indexed with 31 bits; beyond that the outermost joint mode is cut into equal slices.
    # The limit is lowered here so that the slicing logic runs on sizes the host can check.
    assert "launches=4 " in lc.Plan("%d:3" % (1 << 32), "%d:1" % (1 << 32), "bf16").describe()
    assert "launches=16 " in lc.Plan("%d:1" % (1 << 36), "%d:1" % (1 << 36), "f32").describe()
    monkeypatch.setenv("LC_TUNE_MAX_ITEMS", "1000")
    monkeypatch.setenv("LC_TUNE_FORCE_CLASS", "1")       # the third case would otherwise go through element-wise tiles
    for s, d, dt, launches in [("4096:3", "4096:1", "f32", 8), ("(64,240):(1,64)", "(64,240):(1,100)", "bf16", 4),
                               ("(30,7,11):(1,30,210)", "(30,7,11):(77,11,1)", "f32", 3), ("4099:1", "4099:1", "b8", 4099)]:
        desc, _ = _check(oracle, s, d, dt, "direct")
        assert "launches=%d " % launches in desc, desc


def test_plan_errors():
    with pytest.raises(lc.LayoutCopyError) as e:
        lc.Plan("8:1", "9:1", "f32")
    assert e.value.status_name == "SIZE_MISMATCH"
    assert "class=last-writer" in lc.Plan("(4,4):(1,4)", "(4,4):(1,3)", "f32").describe()      # overlapping rows
    assert "class=" in lc.Plan("1:0", "1:0", "f32").describe()    # a single element never aliases
    assert "class=" in lc.Plan("(2,3):(3,2)", "(2,3):(3,2)", "f32").describe()   # injective though not nested


def test_destination_modes_of_stride_zero_keep_the_last_write(oracle):
    # Sec. 2.6.1's loop runs i upwards, so of the coordinates that differ only in destination modes of stride 0 the
    # last one wins: the library copies that slice (the oracle runs the loop itself)
    cases = [("(4,2):(1,4)", "(4,2):(1,0)", "f32", 1, 4),                       # the second column stays
             ("6:1", "(3,2):(1,0)", "f32", 1, 3),                                 # shapes differ: refined first
             ("(8,3,64):(1,8,24)", "(8,3,64):(64,0,1)", "bf16", 1, 16),           # a transposing copy around the dropped mode
             ("(2,5,3,4):(60,1,5,15)", "(2,5,3,4):(0,1,0,5)", "b8", 2, 60 + 2 * 5),
             ("(16,(4,2)):(1,(16,64))", "(16,(4,2)):(1,(0,16))", "b64", 1, 3 * 16),
             ("(5,7):(7,1)", "(5,7):(0,0)", "f32", 2, 34),                         # everything into one element
             ("(64,3,64):(1,4096,64)", "(64,3,64):(64,0,1)", "f32", 1, 8192)]
    for s, d, dt, modes, offset in cases:
        desc, _ = _check(oracle, s, d, dt)
        assert "overwritten_modes=%d src_offset=%d" % (modes, offset) in desc, desc
    assert "class=transpose" in _check(oracle, "(64,3,64):(1,4096,64)", "(64,3,64):(64,0,1)", "f32")[0]


def test_aliasing_destinations_keep_the_last_write(oracle):
    # Table copy, "Scatter" with repeated offsets: Sec. 2.6.1's loop leaves the value of the largest coordinate that
    # reaches an offset.  The plan is walked with both passes running BACKWARDS: only the recorded coordinates may write.
    cases = [("(4,4):(1,4)", "(4,4):(1,3)", "f32"),                         # rows that overlap by one element
             ("(4,4,2):(1,4,16)", "(4,4,2):(1,3,0)", "f32"),                # a stride-0 mode beside overlapping rows: folded first
             ("(7,5):(1,7)", "(7,5):(2,3)", "bf16"),                         # strides 2 and 3 meet often
             ("(16,16):(16,1)", "(16,16):(1,1)", "b8"),                       # anti-diagonals collapse
             ("(6,10):(10,1)", "(4,15):(3,2)", "b64"),                        # shapes without a common refinement
             ("64:1", "(8,8):(1,4)", "f32"),
             ("(3,(2,5)):(1,(3,6))", "(3,(2,5)):(5,(7,1))", "b16")]
    for s, d, dt in cases:
        desc, _ = _check(oracle, s, d, dt, "last-writer")
        assert "workspace_bytes=%d" % (4 * oracle.Layout(d).cosize) in desc or "overwritten_modes" in desc, desc
    assert "overwritten_modes=1" in lc.Plan("(4,4,2):(1,4,16)", "(4,4,2):(1,3,0)", "f32").describe()
    rng = np.random.default_rng(77)
    for i in range(200):   # random small strides on both sides: most destinations alias, some do not
        shape = [int(x) for x in rng.integers(1, 7, 3)]
        sd = [int(x) for x in rng.integers(0, 9, 3)]
        dd = [int(x) for x in rng.integers(0, 9, 3)]
        s = "(%d,%d,%d):(%d,%d,%d)" % (*shape, *sd)
        d = "(%d,%d,%d):(%d,%d,%d)" % (*shape, *dd)
        _check(oracle, s, d, ["f32", "bf16", "b8", "b64"][i % 4], seed=i)
    # a large destination whose strides do not nest is not enumerated on the host: decided per offset on the device
    big = lc.Plan("(4096,2048):(1,4096)", "(4096,2048):(3,4097)", "f32")
    assert "class=last-writer" in big.describe() and big.workspace_bytes == 4 * (4095 * 3 + 2047 * 4097 + 1)
    assert lc.Plan("(4,4):(1,4)", "(4,4):(4,1)", "f32").workspace_bytes == 0


def _check_signed(oracle, src_layout, dst_layout, dtype, seed=0):
    """_check for layouts with negative strides: both buffers extend below offset 0."""
    es = lc.DTYPE_BYTES[dtype]
    sl, dl = oracle.Layout(src_layout), oracle.Layout(dst_layout)
    so, do = -sl.min_offset, -dl.min_offset
    rng = np.random.default_rng(seed)
    src = rng.integers(0, 255, size=(so + sl.cosize) * es, dtype=np.uint8).view(_np_dtype(es))
    want = np.full(do + dl.cosize, 0xA5A5A5A5A5A5A5A5 & ((1 << (8 * es)) - 1), dtype=_np_dtype(es))
    got = want.copy()
    oracle.copy(src, sl, want, dl, src_origin=so, dst_origin=do)
    plan = lc.Plan(src_layout, dst_layout, dtype)
    plan.debug_replay_on_host(src, got, so, do)
    assert (got == want).all(), plan.describe()
    return plan.describe()


def test_negative_strides_are_planned_by_walking_modes_backwards(oracle):
    # a joint mode of negative destination stride is walked backwards on both sides (Sec. 3.4.2: any order, the same on
    # both sides): what is left has destination strides >= 0; negative source strides stay as true reversals
    d = _check_signed(oracle, "4096:1", "4096:-1", "f32")
    assert "reflected=1" in d and "dst_offset=-4095" in d and "class=direct" in d, d
    d = _check_signed(oracle, "4096:-1", "4096:-1", "f32")                      # both reversed: a plain copy again, but of the
    assert "reflected=1" in d and "joint=[(4096,1,1)]" in d and "width_bytes=4" in d, d   # memory BELOW two aligned pointers: its start is not aligned
    d = _check_signed(oracle, "4096:-1", "4096:1", "bf16")                      # a true reversal: element by element
    assert "reflected" not in d and "width_bytes=2" in d, d
    d = _check_signed(oracle, "(64,48):(1,64)", "(64,48):(-48,1)", "f32")       # transpose with flipped rows: walking the rows
    assert "reflected=1" in d and "(64,-1,48)" in d, d                          # backwards reverses the source's contiguous mode
    d = _check_signed(oracle, "(64,48):(1,-64)", "(64,48):(48,1)", "f32")       # transpose reading the columns backwards
    assert "class=transpose" in d, d
    d = _check_signed(oracle, "(256,64,3):(1,256,-16384)", "(256,64,3):(64,1,16384)", "bf16")   # batch of transposes, batches reversed
    assert "class=transpose" in d, d
    d = _check_signed(oracle, "(256,64,3):(1,256,16384)", "(256,64,3):(64,1,-16384)", "bf16")   # the same seen from the destination
    assert "class=transpose" in d and "reflected=1" in d, d
    _check_signed(oracle, "(6,10):(10,-1)", "(4,15):(-15,1)", "f32")             # no common refinement: element-wise, signed
    _check_signed(oracle, "(4,2,3):(1,4,8)", "(4,2,3):(1,0,-4)", "f32")          # an overwritten mode and a reversed one
    _check_signed(oracle, "(4,4):(1,4)", "(4,4):(-1,3)", "b16")                  # aliasing with a negative stride: last writer
    rng = np.random.default_rng(9)
    for i in range(300):
        r = int(rng.integers(1, 4))
        ext = [int(x) for x in rng.integers(1, 9, r)]
        def strides():
            order = rng.permutation(r)
            d, run = [0] * r, 1
            for m in order:
                d[m] = run * int(rng.choice([1, -1]))
                run *= ext[m] * int(rng.choice([1, 1, 2]))
            return d
        s = "(%s):(%s)" % (",".join(map(str, ext)), ",".join(map(str, strides())))
        t = "(%s):(%s)" % (",".join(map(str, ext)), ",".join(map(str, strides())))
        _check_signed(oracle, s, t, ["f32", "bf16", "b8", "b64"][i % 4], seed=i)


def test_alignment_limits_vector_width():
    wide = lc.Plan("4096:1", "4096:1", "f32").describe()
    narrow = lc.Plan("4096:1", "4096:1", "f32", src_align=4, dst_align=256).describe()
    assert "width_bytes=16" in wide and "width_bytes=4" in narrow
    # padded rows whose pitch is not a multiple of the vector: width drops to what divides it
    assert "width_bytes=8" in lc.Plan("(64,32):(1,66)", "(64,32):(1,64)", "f32").describe()
    assert "width_bytes=4" in lc.Plan("(64,32):(1,65)", "(64,32):(1,64)", "f32").describe()


def test_gather_with_small_source_stride_moves_whole_words(oracle, monkeypatch):
    """A destination-contiguous mode read with stride S (S * element < 32 bytes): 16-byte words on both sides, the lane
    keeps every S-th element of S consecutive source words.  Buffers are exactly as long as the layouts reach: the last
    vector along the mode must not read past the last element (it loads element by element).  On request only: element by
    element is faster on MI355X."""
    monkeypatch.setenv("LC_TUNE_GATHER", "1")
    cases = [("4096:3", "4096:1", "f32", 3), ("4096:2", "4096:1", "f32", 2), ("1024:7", "1024:1", "f32", 7),
             ("4096:3", "4096:1", "bf16", 3), ("2048:5", "2048:1", "bf16", 5), ("1024:7", "1024:1", "f16", 7),
             ("512:3", "512:1", "b64", 3), ("512:2", "512:1", "b64", 2),
             ("(64,30):(3,200)", "(64,30):(1,64)", "f32", 3),                 # rows of a padded matrix, every third column
             ("(32,5,7):(6,192,1920)", "(32,5,7):(1,64,320)", "bf16", 6)]     # outer strides in whole words on both sides
    for s, d, dt, stride in cases:
        desc, _ = _check(oracle, s, d, dt, "direct")
        assert "gather_stride=%d " % stride in desc and "width_bytes=16 " in desc, desc
    desc = _check_signed(oracle, "(64,9):(3,-192)", "(64,9):(1,64)", "f32")  # rows walked backwards on the source side
    assert "gather_stride=3 " in desc, desc
    # not this path: stride too long for the element width, a ragged extent, an outer stride that splits a word, a
    # broadcast mode, pointers that are not 16-byte aligned
    for s, d, dt in [("4096:8", "4096:1", "f32"), ("1024:4", "1024:1", "b64"), ("4094:3", "4094:1", "f32"),
                     ("(64,30):(3,201)", "(64,30):(1,64)", "f32"), ("(64,4):(3,0)", "(64,4):(1,64)", "f32")]:
        desc, _ = _check(oracle, s, d, dt)
        assert "gather_stride" not in desc, desc
    assert "gather_stride" not in lc.Plan("4096:3", "4096:1", "f32", src_align=4).describe()
    # sliced into launches along the gathered mode itself
    monkeypatch.setenv("LC_TUNE_MAX_ITEMS", "100")
    desc, _ = _check(oracle, "4096:3", "4096:1", "f32", "direct")
    assert "gather_stride=3 " in desc and "launches=16 " in desc, desc
    monkeypatch.delenv("LC_TUNE_MAX_ITEMS")
    monkeypatch.delenv("LC_TUNE_GATHER")
    desc, _ = _check(oracle, "4096:3", "4096:1", "f32", "direct")
    assert "gather_stride" not in desc and "width_bytes=4 " in desc, desc
