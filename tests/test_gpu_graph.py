"""HIP graph capture of the library's launches: a plan's execute call makes no allocation, copy or synchronisation, so a
caller may record it into a graph (launch-bound callers: the 1024^2 transpose takes 4 us of kernel time per 16 us step
when launched eagerly).  Each graph is replayed several times with eager work and synchronisations in between, on
changed inputs, and every replay is compared with the oracle.  Run on the MI355X machine with `-m gpu`."""
import numpy as np
import pytest

import paper_2603_02298_amd as lc
from paper_2603_02298_amd import workloads as W

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _capture(launch):
    """Runs launch(stream_handle) once eagerly (first-use set-up happens outside the capture), then records it."""
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        launch(side.cuda_stream)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        launch(torch.cuda.current_stream().cuda_stream)
    return graph


@pytest.mark.parametrize("src_layout,dst_layout,dtype", [
    ("(1024,1024):(1,1024)", "(1024,1024):(1024,1)", "f32"),          # transposing class
    ("(4096,64):(1,4096)", "(4096,64):(1,8192)", "bf16"),              # direct class, padded destination
    ("(1000,3):(3,3001)", "(1000,3):(1,1000)", "f32"),                 # ragged gather
])
def test_copy_plan_in_a_graph(oracle, src_layout, dst_layout, dtype, monkeypatch):
    monkeypatch.setenv("LC_TUNE_TILE_QUEUE", "1")   # a captured launch never uses the tile queue: replays may overlap anything
    es = lc.DTYPE_BYTES[dtype]
    npdt = {2: np.int16, 4: np.int32}[es]
    sl, dl = oracle.Layout(src_layout), oracle.Layout(dst_layout)
    dev = torch.device("cuda:0")
    src_t = torch.zeros(sl.cosize, dtype={2: torch.int16, 4: torch.int32}[es], device=dev)
    dst_t = torch.zeros(dl.cosize, dtype=src_t.dtype, device=dev)
    plan = lc.Plan(src_layout, dst_layout, dtype)
    print("case", plan.describe(), flush=True)
    graph = _capture(lambda stream: plan.execute(src_t.data_ptr(), dst_t.data_ptr(), stream))
    for rep in range(4):
        rng = np.random.default_rng(rep)
        src = rng.integers(-30000, 30000, sl.cosize).astype(npdt)
        src_t.copy_(torch.from_numpy(src))          # eager work between the replays
        dst_t.fill_(-1 - rep)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        want = np.full(dl.cosize, -1 - rep, npdt)
        oracle.copy(src, sl, want, dl)
        assert (dst_t.cpu().numpy() == want).all(), (rep, plan.describe())


@pytest.mark.parametrize("name,mnk,env_direct", [("tn", (264, 136, 128), True), ("nt", (136, 264, 128), True), ("gett", (192, 100, 72), True), ("gett", (192, 100, 76), False)])   # a short last k tile on the direct path; staged loads
def test_gemm_plan_in_a_graph(oracle, name, mnk, env_direct):
    w = W.gemm_workload(name, *mnk, ab_dtype="bf16", values="ints")
    plan = lc.GemmPlan(w.a_layout, w.b_layout, w.c_layout, "bf16")
    desc = plan.describe()
    print("case", desc, flush=True)
    assert ("direct-to-LDS" in desc) == env_direct
    dev = torch.device("cuda:0")
    a_t = torch.zeros(w.a_elems, dtype=torch.bfloat16, device=dev)
    b_t = torch.zeros(w.b_elems, dtype=torch.bfloat16, device=dev)
    c_t = torch.zeros(w.c_elems, dtype=torch.float32, device=dev)
    graph = _capture(lambda stream: plan.execute(a_t.data_ptr(), b_t.data_ptr(), c_t.data_ptr(), stream))
    for rep in range(3):
        rng = np.random.default_rng(10 + rep)
        a = rng.integers(-4, 5, w.a_elems).astype(np.float32)
        b = rng.integers(-4, 5, w.b_elems).astype(np.float32)
        c0 = rng.integers(-8, 9, w.c_elems).astype(np.float32)
        a_t.copy_(torch.from_numpy(a).to(torch.bfloat16))
        b_t.copy_(torch.from_numpy(b).to(torch.bfloat16))
        c_t.copy_(torch.from_numpy(c0))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        want = oracle.gemm(a.astype(np.float64), w.a_layout, b.astype(np.float64), w.b_layout, c0.astype(np.float64), w.c_layout)
        assert (c_t.cpu().numpy().astype(np.float64) == want).all(), (rep, desc)   # integer-valued inputs: exact
