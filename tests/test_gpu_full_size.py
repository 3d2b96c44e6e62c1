"""Full-size workloads (the benchmark spec sizes) in the launch configuration bench.py times (tile queue on, byte
offsets past 2^32 in workload 5).  Every destination element of every workload is compared with the oracle's COPY
(Sec. 2.6.1) on the same source bits: the oracle's own loop runs over [0, size) cut into one range per host thread
(legal because the five destinations are injective).  torch's permute / slicing of the same device buffer is kept
as a second, independent witness."""
import numpy as np
import pytest

import paper_2603_02298_amd as lc
from paper_2603_02298_amd import workloads as W

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _device_source(w, dev):
    """Seeded device-side stand-in for the numpy generator (same distribution family, torch's generator):
    generating 2^30 values on the host would dominate the test."""
    g = torch.Generator(device=dev)
    g.manual_seed(W.SEED_BASE + int(w.name[1]))
    if w.elem_bytes == 2:
        x = torch.randn(w.src_elems, device=dev, generator=g, dtype=torch.float32)
        x = x.to(torch.bfloat16 if w.dtype == "bf16" else torch.float16)
        return x.view(torch.int16)
    if w.values == "uniform":
        return (torch.rand(w.src_elems, device=dev, generator=g, dtype=torch.float32) * 2 - 1).view(torch.int32)
    return torch.randint(0, 1 << 20, (w.src_elems,), device=dev, generator=g).to(torch.float32).view(torch.int32)


def _reference(name, src):
    if name == "c1":
        return src.view(1024, 1024).t()                       # src[m + 1024 n] -> dst[1024 m + n]
    if name == "c2":
        # src offset = i0 + 8 i1 + 4096 j0 + 32768 j1 ; dst offset = j0 + 8 i0 + 64 j1 + 65536 i1
        return src.view(1024, 8, 512, 8).permute(2, 0, 3, 1)  # dims (j1,j0,i1,i0) -> (i1,j1,i0,j0)
    if name == "c3":
        # src (b,h,s_out,s_in,d_out,d_in) row-major ; dst (b,h,d_out,s_out,d_in,s_in) row-major
        return src.view(64, 32, 32, 128, 2, 64).permute(0, 1, 4, 2, 5, 3)
    if name == "c4a":
        return src[::3][:1 << 26]
    if name == "c4b":
        return src[:1 << 20].unsqueeze(0).expand(16, 1 << 20)
    if name == "c5":
        return src.view(64, 256, 256, 256).permute(0, 2, 3, 1)
    raise KeyError(name)


@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c4a", "c4b", "c5"])
def test_full_size(oracle, name):
    dev = torch.device("cuda:0")
    w = W.workload(name)
    print("full-size", w.name, w.src_layout, "->", w.dst_layout, flush=True)
    npdt = np.uint16 if w.elem_bytes == 2 else np.uint32
    tdt = torch.int16 if w.elem_bytes == 2 else torch.int32
    if w.src_elems <= (1 << 28):
        src_host = W.source_bits(w)                                       # the seeded numpy generator, as in the small cases
        src = torch.from_numpy(src_host.view(np.int16 if w.elem_bytes == 2 else np.int32)).to(dev)
    else:                                                                 # 2^30 elements: seeded device generator, downloaded
        src = _device_source(w, dev)
        src_host = src.cpu().numpy().view(npdt)
    fill = 0x5A5A if w.elem_bytes == 2 else 0x5A5A5A5A
    dst = torch.full((w.dst_elems,), fill, dtype=tdt, device=dev)
    plan = lc.Plan(w.src_layout, w.dst_layout, w.dtype)
    print(plan.describe(), flush=True)
    lc.copy_tensor(src, w.src_layout, dst, w.dst_layout, w.dtype)       # same call bench.py times
    torch.cuda.synchronize()
    # (a) every element against the oracle's loop on the same bits
    want = np.full(w.dst_elems, fill, dtype=npdt)
    threads = oracle.host_threads(16)
    oracle.copy_parallel(src_host, w.src_layout, want, w.dst_layout, threads)
    print("oracle walked %d integral coordinates on %d host threads" % (w.n, threads), flush=True)
    got = dst.cpu().numpy().view(npdt)
    assert np.array_equal(got, want), "GPU result differs from the oracle at offsets %s" % np.flatnonzero(got != want)[:8]
    del want, got
    # (b) second witness: torch's own permute / slicing of the same buffer
    ref = _reference(name, src)
    assert torch.equal(dst.view(ref.shape), ref)


def test_long_plain_copy_hands_chunks_out_on_request(oracle):
    """A contiguous copy of 2 GiB per side (and a ragged tail): the size from which the planner hands the items out to
    the wavefronts in chunks by itself.  Every element against the oracle's loop, two calls in a row."""
    dev = torch.device("cuda:0")
    n = (1 << 29) + 4 * 777
    layout = "%d:1" % n
    plan = lc.Plan(layout, layout, "f32")
    desc = plan.describe()
    print(desc, flush=True)
    assert "class=direct" in desc and "chunk_items=2048" in desc, desc
    g = torch.Generator(device=dev)
    g.manual_seed(W.SEED_BASE + 9)
    src = torch.randint(-2 ** 31, 2 ** 31 - 1, (n,), device=dev, generator=g, dtype=torch.int32)
    src_host = src.cpu().numpy().view(np.uint32)
    want = np.full(n, 0x5A5A5A5A, dtype=np.uint32)
    threads = oracle.host_threads(16)
    oracle.copy_parallel(src_host, layout, want, layout, threads)
    print("oracle walked %d integral coordinates on %d host threads" % (n, threads), flush=True)
    for rep in range(2):
        dst = torch.full((n,), 0x5A5A5A5A, dtype=torch.int32, device=dev)
        lc.copy_tensor(src, layout, dst, layout, "f32")
        torch.cuda.synchronize()
        got = dst.cpu().numpy().view(np.uint32)
        assert np.array_equal(got, want), "call %d differs from the oracle at offsets %s" % (rep, np.flatnonzero(got != want)[:8])
        del dst, got


def test_head_permute_through_word_tiles(oracle):
    """(B,S,H,D) -> (B,H,S,D) with 128-byte heads, 2^26 bf16 elements: the common vector is 8 words
    long, so the planner re-orders 16-byte words through LDS tiles instead of reading 128-byte pieces."""
    dev = torch.device("cuda:0")
    D, H, S, B = 64, 32, 4096, 8
    n = D * H * S * B
    src_layout = "(%d,%d,%d,%d):(1,%d,%d,%d)" % (D, H, S, B, D, D * H, D * H * S)
    dst_layout = "(%d,%d,%d,%d):(1,%d,%d,%d)" % (D, H, S, B, D * S, D, D * H * S)
    desc = lc.Plan(src_layout, dst_layout, "bf16").describe()
    print(desc, flush=True)
    assert "class=transpose" in desc and "V=1 tile_elem_bytes=16" in desc, desc
    g = torch.Generator(device=dev)
    g.manual_seed(W.SEED_BASE + 7)
    src = torch.randint(-32768, 32767, (n,), device=dev, generator=g, dtype=torch.int16)
    dst = torch.full((n,), 0x5A5A, dtype=torch.int16, device=dev)
    lc.copy_tensor(src, src_layout, dst, dst_layout, "bf16")
    torch.cuda.synchronize()
    sl, dl = oracle.Layout(src_layout), oracle.Layout(dst_layout)
    rng = np.random.default_rng(13)
    idx = np.unique(np.concatenate([rng.integers(0, n, 400000), np.arange(0, 4096), np.arange(n - 4096, n)]))
    so = torch.from_numpy(sl.offsets_at(idx)).to(dev)
    do = torch.from_numpy(dl.offsets_at(idx)).to(dev)
    assert torch.equal(dst[do], src[so])
    assert torch.equal(dst.view(B, H, S, D), src.view(B, S, H, D).permute(0, 2, 1, 3))


@pytest.mark.parametrize("M,N,dt", [(4001, 4003, "f32"), (8008, 8000, "bf16"), (8001, 8003, "bf16")])
def test_odd_transposes_through_ragged_tiles(oracle, M, N, dt):
    """Transposes whose extents the tiles do not divide (4001 and 4003 are primes, 8008 = 8 * 7 * 11 * 13)."""
    dev = torch.device("cuda:0")
    n = M * N
    src_layout, dst_layout = "(%d,%d):(1,%d)" % (M, N, M), "(%d,%d):(%d,1)" % (M, N, N)
    desc = lc.Plan(src_layout, dst_layout, dt).describe()
    print(desc, flush=True)
    assert "class=transpose" in desc and "ragged_modes=0" not in desc, desc
    tdt = torch.int32 if dt == "f32" else torch.int16
    g = torch.Generator(device=dev)
    g.manual_seed(W.SEED_BASE + 8)
    src = torch.randint(-32768, 32767, (n,), device=dev, generator=g, dtype=tdt)
    dst = torch.full((n,), 0x5A5A, dtype=tdt, device=dev)
    lc.copy_tensor(src, src_layout, dst, dst_layout, dt)
    torch.cuda.synchronize()
    sl, dl = oracle.Layout(src_layout), oracle.Layout(dst_layout)
    rng = np.random.default_rng(14)
    idx = np.unique(np.concatenate([rng.integers(0, n, 400000), np.arange(0, 4096), np.arange(n - 4096, n)]))
    so = torch.from_numpy(sl.offsets_at(idx)).to(dev)
    do = torch.from_numpy(dl.offsets_at(idx)).to(dev)
    assert torch.equal(dst[do], src[so])
    assert torch.equal(dst.view(M, N), src.view(N, M).t())


def test_c2_literal_strides(oracle):
    """Destination strides exactly as the benchmark spec prints them (not compact: 8.6 GB span, 16-byte runs)."""
    dev = torch.device("cuda:0")
    w = W.workload("c2_literal")
    src = _device_source(w, dev)
    dst = torch.zeros(w.dst_elems, dtype=torch.int16, device=dev)
    print(lc.Plan(w.src_layout, w.dst_layout, w.dtype).describe(), flush=True)
    lc.copy_tensor(src, w.src_layout, dst, w.dst_layout, w.dtype)
    torch.cuda.synchronize()
    sl, dl = oracle.Layout(w.src_layout), oracle.Layout(w.dst_layout)
    rng = np.random.default_rng(12)
    idx = np.unique(np.concatenate([rng.integers(0, w.n, 400000), np.arange(0, 4096), np.arange(w.n - 4096, w.n)]))
    so = torch.from_numpy(sl.offsets_at(idx)).to(dev)
    do = torch.from_numpy(dl.offsets_at(idx)).to(dev)
    assert torch.equal(dst[do], src[so])
    # every written element is accounted for: the number of non-zero destinations equals the non-zero sources
    assert int((dst != 0).sum()) == int((src != 0).sum())


def test_more_than_2_31_work_items(oracle):
    """A 2^32-element gather: the work items no longer fit 31 bits, so the copy runs as four launches over
    slices of the outermost mode (24 GiB source span, 8 GiB destination)."""
    dev = torch.device("cuda:0")
    n = 1 << 32
    src_layout, dst_layout = "%d:3" % n, "%d:1" % n
    plan = lc.Plan(src_layout, dst_layout, "bf16")
    print(plan.describe(), flush=True)
    assert "launches=4 " in plan.describe()
    g = torch.Generator(device=dev)
    g.manual_seed(W.SEED_BASE)
    src = torch.randint(-32768, 32767, (3 * n,), device=dev, generator=g, dtype=torch.int16)
    dst = torch.zeros(n, dtype=torch.int16, device=dev)
    lc.copy_tensor(src, src_layout, dst, dst_layout, "bf16")
    torch.cuda.synchronize()
    assert torch.equal(dst, src[::3])
    sl, dl = oracle.Layout(src_layout), oracle.Layout(dst_layout)
    idx = np.concatenate([np.arange(0, 1024), np.arange(n - 1024, n), np.arange((1 << 31) - 512, (1 << 31) + 512),
                          np.random.default_rng(5).integers(0, n, 100000)])
    so = torch.from_numpy(sl.offsets_at(idx)).to(dev)
    do = torch.from_numpy(dl.offsets_at(idx)).to(dev)
    assert torch.equal(dst[do], src[so])
