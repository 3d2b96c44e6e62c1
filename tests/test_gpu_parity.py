"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, bit for bit, on the same
seeded inputs.  Run on the MI355X machine with `-m gpu`."""
import os

import numpy as np
import pytest

import paper_2603_02298_amd as lc
from paper_2603_02298_amd import workloads as W
from conftest import golden_lines

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _torch_int(es):
    return {1: torch.uint8, 2: torch.int16, 4: torch.int32, 8: torch.int64}[es]


def _np_int(es):
    return {1: np.uint8, 2: np.int16, 4: np.int32, 8: np.int64}[es]


def _gpu_copy(src_bits, src_layout, dst_layout, dtype, dst_elems, fill=0x5A):
    es = lc.DTYPE_BYTES[dtype]
    dev = torch.device("cuda:0")
    src_t = torch.from_numpy(src_bits.view(_np_int(es))).to(dev)
    dst_t = torch.from_numpy(np.full(dst_elems * es, fill, np.uint8).view(_np_int(es))).to(dev)
    lc.copy_tensor(src_t, src_layout, dst_t, dst_layout, dtype)
    torch.cuda.synchronize()
    return dst_t.cpu().numpy()


def _parity(oracle, src_layout, dst_layout, dtype, seed=0, src_bits=None, tag=""):
    es = lc.DTYPE_BYTES[dtype]
    sl, dl = oracle.Layout(src_layout), oracle.Layout(dst_layout)
    print("case", tag, src_layout, "->", dst_layout, dtype, flush=True)
    if src_bits is None:
        rng = np.random.default_rng(seed)
        src_bits = rng.integers(0, 255, size=max(sl.cosize, 1) * es, dtype=np.uint8).view(_np_int(es))
    want = np.full(dl.cosize * es, 0x5A, np.uint8).view(_np_int(es))
    oracle.copy(src_bits.view(want.dtype), sl, want, dl)
    got = _gpu_copy(src_bits, src_layout, dst_layout, dtype, dl.cosize)
    desc = lc.Plan(src_layout, dst_layout, dtype).describe()
    assert (got == want).all(), desc
    return desc


@pytest.mark.parametrize("name,scale", [("c1", 1), ("c1", 16), ("c2", 4), ("c2", 16), ("c3", 16), ("c4a", 16),
                                        ("c4b", 4), ("c5", 256), ("c5", 64)])
def test_workloads_elementwise(oracle, name, scale):
    # sizes the oracle finishes in seconds; every one spans many tiles
    w = W.workload(name, scale)
    _parity(oracle, w.src_layout, w.dst_layout, w.dtype, src_bits=W.source_bits(w), tag=w.name)


def test_copy_applications_table(oracle):
    for ln in golden_lines("copy_applications.txt"):
        name, s, d = [x.strip() for x in ln.split("|")]
        for dt in ("f32", "bf16", "b8", "b64"):
            _parity(oracle, s, d, dt, tag=name)


def test_destination_modes_of_stride_zero_keep_the_last_write(oracle):
    # the sequential loop's last write wins; the library copies the slice that is written last
    for s, d, dt in [("(4,2):(1,4)", "(4,2):(1,0)", "f32"), ("6:1", "(3,2):(1,0)", "f32"),
                     ("(2,5,3,4):(60,1,5,15)", "(2,5,3,4):(0,1,0,5)", "b8"), ("(5,7):(7,1)", "(5,7):(0,0)", "f32"),
                     ("(256,3,512):(1,131072,256)", "(256,3,512):(512,0,1)", "f32"),          # transposing class, several tiles
                     ("(4096,5,64):(1,262144,4096)", "(4096,5,64):(1,0,4096)", "bf16"),       # direct class
                     ("(1000,3,7):(21,7,1)", "(1000,3,7):(1,0,1000)", "b64")]:                # strided gather, offset of 14 elements
        assert "overwritten_modes=" in _parity(oracle, s, d, dt, tag="stride-0 destination")


def test_random_layout_pairs(oracle):
    import sys
    sys.path.insert(0, os.path.dirname(__file__))
    from test_plan_replay import _random_pair
    rng = np.random.default_rng(4242)
    for k in range(400):
        s, d = _random_pair(rng)
        _parity(oracle, s, d, ["f32", "bf16", "b8", "b64", "f16"][k % 5], seed=k, tag="random%d" % k)


def test_random_pairs_with_different_shapes(oracle):
    import sys
    sys.path.insert(0, os.path.dirname(__file__))
    from test_plan_replay import _random_refined_pair
    rng = np.random.default_rng(2718)
    for k in range(400):
        s, d = _random_refined_pair(rng)
        _parity(oracle, s, d, ["f32", "bf16", "b64", "b8"][k % 4], seed=k, tag="refined%d" % k)


@pytest.mark.parametrize("s,d,dt", [
    ("1:0", "1:0", "f32"),                                   # single element
    ("1:5", "1:7", "bf16"),
    ("(1,1,1):(3,4,5)", "1:0", "f32"),
    ("7:1", "7:1", "f32"),                                   # shorter than one vector
    ("1000003:1", "1000003:1", "f32"),                       # prime length: ragged tail, width 4
    ("(1000,3):(3,3001)", "(1000,3):(1,1000)", "f32"),       # ragged rows
    ("(68,36):(1,68)", "(68,36):(36,1)", "f32"),             # transpose, 4 | extents but not tile multiples
    ("(70,34):(1,70)", "(70,34):(34,1)", "f32"),             # transpose with V=2
    ("(71,33):(1,71)", "(71,33):(33,1)", "f32"),             # odd extents: no vector on either side
    ("(136,72):(1,136)", "(136,72):(72,1)", "bf16"),         # V=8 with ragged tile counts
    ("(132,68):(1,132)", "(132,68):(68,1)", "f16"),          # V=4
    ("(8,3,8):(1,64,8)", "(8,3,8):(24,8,1)", "f16"),         # tiny transposed tiles, batch of 3
    ("(6,10):(10,1)", "(4,15):(15,1)", "f32"),               # no common refinement: element-wise kernel
    ("(5,7,3):(21,3,1)", "(3,35):(1,3)", "bf16"),
    ("(256,16):(1,0)", "(256,16):(1,256)", "f32"),           # broadcast
    ("(3,16,5):(1,0,3)", "(3,16,5):(80,1,16)", "f32"),       # broadcast in the middle
    ("4096:7", "4096:1", "bf16"),                            # 2-byte gather
    ("4096:1", "4096:5", "f32"),                             # scatter
    ("(64,64,4):(1,64,4096)", "(64,64,4):(64,1,8192)", "b64"),
])
def test_edge_cases(oracle, s, d, dt):
    _parity(oracle, s, d, dt, seed=3, tag="edge")


def test_large_lds_tiles(oracle, monkeypatch):
    # 4 micro-tiles per lane: 64 KiB (fp32) and 128 KiB (bf16) of LDS per workgroup
    monkeypatch.setenv("LC_TUNE_MICRO_PER_THREAD", "4")
    w = W.workload("c2", 8)
    assert "lds_bytes=131072" in lc.Plan(w.src_layout, w.dst_layout, w.dtype).describe()
    _parity(oracle, w.src_layout, w.dst_layout, w.dtype, src_bits=W.source_bits(w), tag="c2 mt4")
    w = W.workload("c1", 2)
    _parity(oracle, w.src_layout, w.dst_layout, w.dtype, src_bits=W.source_bits(w), tag="c1 mt4")
    monkeypatch.setenv("LC_TUNE_MICRO_PER_THREAD", "2")
    _parity(oracle, w.src_layout, w.dst_layout, w.dtype, src_bits=W.source_bits(w), tag="c1 mt2")


def test_tuning_variants_stay_exact(oracle, monkeypatch):
    w = W.workload("c5", 256)
    bits = W.source_bits(w)
    for env in [{"LC_TUNE_NONTEMPORAL": "1"}, {"LC_TUNE_REST_ORDER": "1"}, {"LC_TUNE_SWIZZLE_SHIFT": "-1"},
                {"LC_TUNE_FORCE_CLASS": "1"}, {"LC_TUNE_FORCE_CLASS": "0"}, {"LC_TUNE_MAX_VEC_BYTES": "8"}]:
        for k, v in env.items():
            monkeypatch.setenv(k, v)
        _parity(oracle, w.src_layout, w.dst_layout, w.dtype, src_bits=bits, tag=str(env))
        for k in env:
            monkeypatch.delenv(k)
    w = W.workload("c4a", 64)
    for u in ("1", "2", "8"):
        monkeypatch.setenv("LC_TUNE_UNROLL", u)
        _parity(oracle, w.src_layout, w.dst_layout, w.dtype, src_bits=W.source_bits(w), tag="unroll" + u)


def test_gathers_with_small_source_stride(oracle, monkeypatch):
    """16-byte words on both sides of a gather whose source stride is a few elements (gather_kernel): every stride the
    kernel is built for, the three element widths, outer modes, a single vector per row, sizes that span many
    workgroups with a ragged last trip; buffers exactly as long as the layouts reach."""
    monkeypatch.setenv("LC_TUNE_GATHER", "1")
    cases = [("%d:%d" % (n, s), "%d:1" % n, dt) for dt, strides in (("f32", (2, 3, 4, 5, 6, 7)), ("bf16", (2, 3, 4, 5, 6, 7)), ("b64", (2, 3)))
             for s in strides for n in (16, 1000 * 8, (1 << 20) + 136)]
    cases += [("(64,30):(3,200)", "(64,30):(1,64)", "f32"), ("(32,5,7):(6,192,1920)", "(32,5,7):(1,64,320)", "bf16"),
              ("(8,3001):(5,40)", "(8,3001):(1,8)", "bf16")]
    for s, d, dt in cases:
        desc = _parity(oracle, s, d, dt, seed=21, tag="gather")
        assert "gather_stride=" in desc, desc
    monkeypatch.setenv("LC_TUNE_MAX_ITEMS", "1000")
    desc = _parity(oracle, "%d:3" % (1 << 16), "%d:1" % (1 << 16), "f32", seed=22, tag="gather sliced")
    assert "gather_stride=3 " in desc and "launches=1 " not in desc, desc
    monkeypatch.setenv("LC_TUNE_UNROLL", "1")
    _parity(oracle, "%d:3" % (1 << 16), "%d:1" % (1 << 16), "bf16", seed=23, tag="gather one item per lane")


def test_sliced_launches(oracle, monkeypatch):
    # the slicing used beyond 2^31 work items, forced at a small size
    monkeypatch.setenv("LC_TUNE_MAX_ITEMS", "1000")
    for s, d, dt in [("4096:3", "4096:1", "f32"), ("(64,240):(1,64)", "(64,240):(1,100)", "bf16"),
                     ("(30,7,11):(1,30,210)", "(30,7,11):(77,11,1)", "f32"), ("(8192,16):(1,0)", "(8192,16):(1,8192)", "f32")]:
        assert "launches=1 " not in lc.Plan(s, d, dt).describe()
        _parity(oracle, s, d, dt, seed=9, tag="sliced")


def test_literal_strides_pattern_small(oracle):
    # the shape of BASELINE config 2 with its printed (non-compact) destination strides, scaled down:
    # 16-byte destination runs at a large pitch, transposing class
    s = "((8,16),(8,32)):((1,8),(128,1024))"
    d = "((8,16),(8,32)):((32,8192),(1,256))"
    assert "class=transpose" in lc.Plan(s, d, "bf16").describe()
    _parity(oracle, s, d, "bf16", seed=4, tag="literal-small")


def test_misaligned_pointers(oracle):
    dev = torch.device("cuda:0")
    n = 4096
    src = torch.arange(n + 8, dtype=torch.int32, device=dev)
    dst = torch.zeros(n + 8, dtype=torch.int32, device=dev)
    plan = lc.Plan("%d:1" % n, "%d:1" % n, "f32")            # created for 256-byte aligned pointers
    with pytest.raises(lc.LayoutCopyError) as e:
        plan.execute(src.data_ptr() + 4, dst.data_ptr(), torch.cuda.current_stream().cuda_stream)
    assert e.value.status_name == "MISALIGNED"
    # lc_copy derives the alignment from the pointers and narrows the accesses instead
    lc.lc_copy(src.data_ptr() + 4, "%d:1" % n, dst.data_ptr() + 8, "%d:1" % n, "f32", torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert torch.equal(dst[2:n + 2], src[1:n + 1])
    assert int(dst[:2].abs().sum()) == 0 and int(dst[n + 2:].abs().sum()) == 0


def test_plan_reuse_and_streams(oracle):
    w = W.workload("c2", 16)
    bits = W.source_bits(w)
    dev = torch.device("cuda:0")
    src = torch.from_numpy(bits.view(np.int16)).to(dev)
    plan = lc.Plan(w.src_layout, w.dst_layout, w.dtype)
    want = np.zeros(w.dst_elems, np.int16)
    oracle.copy(bits.view(np.int16), w.src_layout, want, w.dst_layout)
    side = torch.cuda.Stream()
    outs = []
    for k in range(4):
        dst = torch.zeros(w.dst_elems, dtype=torch.int16, device=dev)
        st = side if k % 2 else torch.cuda.current_stream()
        st.wait_stream(torch.cuda.current_stream())
        plan.execute(src.data_ptr(), dst.data_ptr(), st.cuda_stream)
        outs.append(dst)
    torch.cuda.synchronize()
    for dst in outs:
        assert (dst.cpu().numpy() == want).all()


def test_tile_queue(oracle, monkeypatch):
    # tiles handed out on request (a pair of counters in device memory, reset by the last workgroup): forced on for
    # sizes the oracle can check in full; twice in a row on one stream (the second launch finds the counters at zero)
    monkeypatch.setenv("LC_TUNE_TILE_QUEUE", "1")
    for name, scale in (("c5", 64), ("c2", 4), ("c3", 16), ("c1", 1)):
        w = W.workload(name, scale)
        for rep in range(2):
            desc = _parity(oracle, w.src_layout, w.dst_layout, w.dtype, src_bits=W.source_bits(w), tag=w.name + " queue")
        assert "tile_queue=1" in desc, desc
    # one workgroup per CU, so that the grid is shorter than the list of tiles and every workgroup asks several times;
    # one, three and eight tiles per request (the last batch straddles the end of the list)
    monkeypatch.setenv("LC_TUNE_WGS_PER_CU", "1")
    for grab in (1, 3, 8):
        monkeypatch.setenv("LC_TUNE_TILE_QUEUE", str(grab))
        for name, scale in (("c5", 64), ("c2", 4), ("c3", 16), ("c1", 1)):
            w = W.workload(name, scale)
            desc = _parity(oracle, w.src_layout, w.dst_layout, w.dtype, src_bits=W.source_bits(w), tag="%s queue %d, 1 per CU" % (w.name, grab))
            assert "tile_queue=%d" % grab in desc, desc


def test_plan_time_each_reports_every_launch(oracle):
    # per-launch timing: as many figures as launches, all positive, their mean close to the batch mean of lc_plan_time
    w = W.workload("c5", 64)
    dev = torch.device("cuda:0")
    src = torch.from_numpy(W.source_bits(w).view(np.int32)).to(dev)
    dsts = [torch.zeros(w.dst_elems, dtype=torch.int32, device=dev) for _ in range(2)]
    plan = lc.Plan(w.src_layout, w.dst_layout, w.dtype)
    sp, dp = [src.data_ptr()] * 2, [d.data_ptr() for d in dsts]
    each = plan.time_each(sp, dp, 2, 12)
    mean = plan.time(sp, dp, 2, 12)
    assert len(each) == 12 and min(each) > 0
    assert 0.5 * mean < sum(each) / len(each) < 3.0 * mean + 0.01, (each, mean)
    want = np.zeros(w.dst_elems, np.uint32)
    oracle.copy(W.source_bits(w).view(np.uint32), oracle.Layout(w.src_layout), want, oracle.Layout(w.dst_layout))
    for d in dsts:
        assert (d.cpu().numpy().view(np.uint32) == want).all()
    with pytest.raises(lc.LayoutCopyError):
        plan.time_each(sp, dp, 0, 0)


def test_direct_class_chunks_on_request(oracle, monkeypatch):
    # the direct class with its items handed out to the wavefronts in chunks (counters of the stream's block, put back to zero
    # by the last wavefront): forced on at sizes the oracle walks in full.  Plain copies, a strided gather, a broadcast
    # (looped mode), several joint modes, every element width; chunks of 1, 4 and 32 KiB, 1, 8 and 15 counters, grids from
    # one workgroup to more wavefronts than chunks; each case twice in a row (the second launch finds the counters at zero)
    cases = [("%d:1" % n, "%d:1" % n, dt) for n in (1 << 20, (1 << 20) + 77, 5000) for dt in ("f32", "bf16", "b8", "b64")]
    cases += [("%d:3" % (1 << 18), "%d:1" % (1 << 18), "f32"), ("(%d,16):(1,0)" % (1 << 14), "(%d,16):(1,%d)" % (1 << 14, 1 << 14), "f32"),
              ("(256,240):(1,256)", "(256,240):(1,300)", "bf16"), ("(30,7,111):(1,30,210)", "(30,7,111):(777,111,1)", "f32")]
    for kib, counters, grid in ((1, 8, 0), (4, 1, 7), (32, 15, 0), (1, 3, 1), (4, 8, 2000)):
        monkeypatch.setenv("LC_TUNE_DIRECT_QUEUE", str(kib))
        monkeypatch.setenv("LC_TUNE_QUEUE_COUNTERS", str(counters))
        monkeypatch.setenv("LC_TUNE_FORCE_CLASS", "1")
        if grid:
            monkeypatch.setenv("LC_TUNE_GRID", str(grid))
        for s_, d_, dt in cases:
            for rep in range(2):
                desc = _parity(oracle, s_, d_, dt, seed=31 + rep, tag="chunks %d KiB, %d counters, grid %d" % (kib, counters, grid))
            assert "class=direct" in desc and "chunk_items=" in desc, desc
        if grid:
            monkeypatch.delenv("LC_TUNE_GRID")
    # sliced into launches as well: every launch takes the counters afresh
    monkeypatch.setenv("LC_TUNE_DIRECT_QUEUE", "1")
    monkeypatch.setenv("LC_TUNE_MAX_ITEMS", "1000")
    desc = _parity(oracle, "%d:3" % (1 << 14), "%d:1" % (1 << 14), "f32", seed=33, tag="chunks, sliced")
    assert "chunk_items=" in desc and "launches=1 " not in desc, desc


def test_direct_class_chunks_on_several_streams(oracle, monkeypatch):
    monkeypatch.setenv("LC_TUNE_DIRECT_QUEUE", "4")
    n = (1 << 22) + 40
    src_layout = dst_layout = "%d:1" % n
    dev = torch.device("cuda:0")
    plan = lc.Plan(src_layout, dst_layout, "f32")
    assert "chunk_items=" in plan.describe()
    streams = [torch.cuda.Stream() for _ in range(4)]
    srcs = [torch.randint(-2 ** 31, 2 ** 31 - 1, (n,), dtype=torch.int32, device=dev) for _ in streams]
    dsts = [torch.zeros(n, dtype=torch.int32, device=dev) for _ in streams]
    torch.cuda.synchronize()
    for rep in range(5):
        for st, a, d in zip(streams, srcs, dsts):
            plan.execute(a.data_ptr(), d.data_ptr(), st.cuda_stream)
    torch.cuda.synchronize()
    for a, d in zip(srcs, dsts):
        assert torch.equal(a, d)


def test_tile_queue_after_whole_rounds_and_over_several_counters(oracle, monkeypatch):
    # the queue taking over after two (or, capped, all) whole rounds of the grid, requests spread over 8 and 15 counters;
    # and, in the fixed order, the tiles left after the last whole round going to the leading workgroups only
    for name, scale in (("c2", 4), ("c5", 64), ("c3", 16)):
        w = W.workload(name, scale)
        bits = W.source_bits(w)
        for env in ({"LC_TUNE_TILE_QUEUE": "1", "LC_TUNE_QUEUE_ROUNDS": "2", "LC_TUNE_QUEUE_COUNTERS": "8", "LC_TUNE_GRID": "100"},
                    {"LC_TUNE_TILE_QUEUE": "2", "LC_TUNE_QUEUE_ROUNDS": "1", "LC_TUNE_QUEUE_COUNTERS": "15", "LC_TUNE_GRID": "37"},
                    {"LC_TUNE_TILE_QUEUE": "1", "LC_TUNE_QUEUE_ROUNDS": "1000", "LC_TUNE_QUEUE_COUNTERS": "3", "LC_TUNE_GRID": "48"},
                    {"LC_TUNE_TILE_QUEUE": "3", "LC_TUNE_QUEUE_ROUNDS": "2", "LC_TUNE_QUEUE_COUNTERS": "8"},
                    {"LC_TUNE_TILE_QUEUE": "0", "LC_TUNE_LEFTOVER_LEAD": "7", "LC_TUNE_GRID": "100"},
                    {"LC_TUNE_TILE_QUEUE": "0", "LC_TUNE_LEFTOVER_LEAD": "1", "LC_TUNE_GRID": "61"},
                    {"LC_TUNE_TILE_QUEUE": "0", "LC_TUNE_LEFTOVER_LEAD": "5000", "LC_TUNE_GRID": "96"}):
            for k, v in env.items():
                monkeypatch.setenv(k, v)
            for rep in range(2):   # twice: the second launch must find every counter at zero
                _parity(oracle, w.src_layout, w.dst_layout, w.dtype, src_bits=bits, tag="%s %s" % (w.name, env))
            for k in env:
                monkeypatch.delenv(k)


def test_aliasing_destinations_keep_the_last_write(oracle):
    # Scatter with repeated offsets (Table copy): the loop's last write to an offset stays.  Class last-writer, with a
    # workspace of one word per destination offset; the same workspace is used again without clearing (the plan clears it)
    dev = torch.device("cuda:0")
    cases = [("(4,4):(1,4)", "(4,4):(1,3)", "f32"), ("(4,4,2):(1,4,16)", "(4,4,2):(1,3,0)", "f32"),
             ("(7,5):(1,7)", "(7,5):(2,3)", "bf16"), ("(16,16):(16,1)", "(16,16):(1,1)", "b8"),
             ("(6,10):(10,1)", "(4,15):(3,2)", "b64"), ("(3,(2,5)):(1,(3,6))", "(3,(2,5)):(5,(7,1))", "b16"),
             ("(1000,300):(1,1000)", "(1000,300):(3,7)", "f32"),                    # 300000 coordinates onto 5097 offsets
             ("(4096,2048):(1,4096)", "(4096,2048):(3,4097)", "f32"),               # injective, but too large to show on the host
             ("(512,512,8):(1,512,262144)", "(512,512,8):(512,1,1000)", "bf16")]    # 2^21 coordinates, overlapping slabs
    ws = torch.full((64 << 20,), -1, dtype=torch.int32, device=dev)                 # stale contents on purpose
    for s, d, dt in cases:
        es = lc.DTYPE_BYTES[dt]
        sl, dl = oracle.Layout(s), oracle.Layout(d)
        print("case last-writer", s, "->", d, dt, flush=True)
        rng = np.random.default_rng(len(s))
        src_bits = rng.integers(0, 255, size=sl.cosize * es, dtype=np.uint8).view(_np_int(es))
        want = np.full(dl.cosize * es, 0x5A, np.uint8).view(_np_int(es))
        oracle.copy(src_bits, sl, want, dl)
        plan = lc.Plan(s, d, dt)
        assert "class=last-writer" in plan.describe() and 0 < plan.workspace_bytes <= ws.numel() * 4, plan.describe()
        src_t = torch.from_numpy(src_bits).to(dev)
        for rep in range(2):
            dst_t = torch.from_numpy(np.full(dl.cosize * es, 0x5A, np.uint8).view(_np_int(es))).to(dev)
            plan.execute_workspace(src_t.data_ptr(), dst_t.data_ptr(), ws.data_ptr(), ws.numel() * 4, torch.cuda.current_stream().cuda_stream)
            torch.cuda.synchronize()
            assert (dst_t.cpu().numpy() == want).all(), plan.describe()
        with pytest.raises(lc.LayoutCopyError) as e:
            plan.execute(src_t.data_ptr(), dst_t.data_ptr(), torch.cuda.current_stream().cuda_stream)
        assert e.value.status_name == "NEEDS_WORKSPACE"
        with pytest.raises(lc.LayoutCopyError) as e:
            plan.execute_workspace(src_t.data_ptr(), dst_t.data_ptr(), ws.data_ptr(), plan.workspace_bytes - 4, 0)
        assert e.value.status_name == "WORKSPACE_TOO_SMALL"
    # a plan that needs no workspace runs through the same call
    w = W.workload("c1", 16)
    bits = W.source_bits(w)
    want = np.zeros(w.dst_elems, dtype=bits.dtype)
    oracle.copy(bits, w.src_layout, want, w.dst_layout)
    plan = lc.Plan(w.src_layout, w.dst_layout, w.dtype)
    src_t = torch.from_numpy(bits.view(np.int32)).to(dev)
    dst_t = torch.zeros(w.dst_elems, dtype=torch.int32, device=dev)
    plan.execute_workspace(src_t.data_ptr(), dst_t.data_ptr(), 0, 0, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert (dst_t.cpu().numpy().view(bits.dtype) == want).all()


def test_negative_strides(oracle):
    # modes of negative destination stride are walked backwards on both sides; negative source strides stay as reversals
    dev = torch.device("cuda:0")
    cases = [("4096:1", "4096:-1", "f32"), ("4096:-1", "4096:-1", "f32"), ("100000:-1", "100000:1", "bf16"), ("13:-3", "13:1", "b8"),
             ("(64,48):(1,64)", "(64,48):(-48,1)", "f32"), ("(64,48):(1,-64)", "(64,48):(48,1)", "f32"),
             ("(256,64,3):(1,256,-16384)", "(256,64,3):(64,1,16384)", "bf16"), ("(256,64,3):(1,256,16384)", "(256,64,3):(64,1,-16384)", "bf16"),
             ("(512,512,4):(1,512,-262144)", "(512,512,4):(512,1,262144)", "f32"),        # several tiles, batches reversed
             ("(1024,1024):(1,1024)", "(1024,1024):(1024,-1)", "f32"),                    # transpose onto flipped columns
             ("(6,10):(10,-1)", "(4,15):(-15,1)", "b64"), ("(4,2,3):(1,4,8)", "(4,2,3):(1,0,-4)", "f32"),
             ("(64,9):(3,-192)", "(64,9):(1,64)", "f32")]                                  # a gather with its rows backwards
    rng = np.random.default_rng(9)
    for i in range(60):
        r = int(rng.integers(1, 4))
        ext = [int(x) for x in rng.integers(1, 40, r)]
        def strides():
            order = rng.permutation(r)
            d, run = [0] * r, 1
            for m in order:
                d[m] = run * int(rng.choice([1, -1]))
                run *= ext[m] * int(rng.choice([1, 1, 2]))
            return d
        cases.append(("(%s):(%s)" % (",".join(map(str, ext)), ",".join(map(str, strides()))),
                      "(%s):(%s)" % (",".join(map(str, ext)), ",".join(map(str, strides()))), ["f32", "bf16", "b8", "b64"][i % 4]))
    for s, d, dt in cases:
        es = lc.DTYPE_BYTES[dt]
        sl, dl = oracle.Layout(s), oracle.Layout(d)
        so, do = -sl.min_offset, -dl.min_offset
        print("case signed", s, "->", d, dt, flush=True)
        src_bits = np.random.default_rng(len(s) + len(d)).integers(0, 255, size=(so + sl.cosize) * es, dtype=np.uint8).view(_np_int(es))
        want = np.full((do + dl.cosize) * es, 0x5A, np.uint8).view(_np_int(es))
        oracle.copy(src_bits, sl, want, dl, src_origin=so, dst_origin=do)
        src_t = torch.from_numpy(src_bits).to(dev)
        dst_t = torch.from_numpy(np.full((do + dl.cosize) * es, 0x5A, np.uint8).view(_np_int(es))).to(dev)
        lc.copy_tensor(src_t, s, dst_t, d, dt, src_origin=so, dst_origin=do)
        torch.cuda.synchronize()
        assert (dst_t.cpu().numpy() == want).all(), lc.Plan(s, d, dt).describe()


def test_tile_queue_on_several_streams(oracle, monkeypatch):
    # every stream keeps a pair of counters of its own: copies that run side by side do not share one
    monkeypatch.setenv("LC_TUNE_TILE_QUEUE", "1")
    monkeypatch.setenv("LC_TUNE_WGS_PER_CU", "1")
    w = W.workload("c5", 64)
    src_bits = W.source_bits(w)
    want = np.zeros(w.dst_elems, dtype=src_bits.dtype)
    oracle.copy(src_bits, oracle.Layout(w.src_layout), want, oracle.Layout(w.dst_layout))
    dev = torch.device("cuda:0")
    plan = lc.Plan(w.src_layout, w.dst_layout, w.dtype)
    assert "tile_queue=1" in plan.describe()
    streams = [torch.cuda.Stream() for _ in range(4)]
    src_t = torch.from_numpy(src_bits.view(np.int32)).to(dev)
    dsts = [torch.zeros(w.dst_elems, dtype=torch.int32, device=dev) for _ in streams]
    torch.cuda.synchronize()
    for rep in range(5):
        for st, d in zip(streams, dsts):
            plan.execute(src_t.data_ptr(), d.data_ptr(), st.cuda_stream)
    torch.cuda.synchronize()
    for d in dsts:
        assert (d.cpu().numpy().view(src_bits.dtype) == want).all()
