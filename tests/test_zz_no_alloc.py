"""The entry point that allocates nothing, lc_plan_execute_static (scratch memory in a static array of the library's code
object), against lc_plan_execute_workspace (scratch memory from the caller) through the C ABI: same bits, on two calls in
a row of which the second is the smaller one and finds the first one's records still in the array; the oracle as the
third witness; the refusal beyond the array's size."""
import ctypes

import numpy as np
import pytest

import paper_2603_02298_amd as lc

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _np_int(es):
    return {1: np.uint8, 2: np.int16, 4: np.int32, 8: np.int64}[es]


def _run(L, plan, entry, src_t, dl_cosize, es, dev, ws=None):
    dst_t = torch.from_numpy(np.full(dl_cosize * es, 0x5A, np.uint8).view(_np_int(es))).to(dev)
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    if entry == "static":
        st = L.lc_plan_execute_static(plan._h, ctypes.c_void_p(src_t.data_ptr()), ctypes.c_void_p(dst_t.data_ptr()), stream)
    else:
        st = L.lc_plan_execute_workspace(plan._h, ctypes.c_void_p(src_t.data_ptr()), ctypes.c_void_p(dst_t.data_ptr()),
                                         ctypes.c_void_p(ws.data_ptr()), ctypes.c_size_t(ws.numel() * 4), stream)
    assert st == 0, L.lc_status_string(st).decode()
    torch.cuda.synchronize()
    return dst_t.cpu().numpy()


def test_static_scratch_entry_point_matches_the_workspace_one(oracle):
    dev = torch.device("cuda:0")
    L = lc.lib()
    assert L.lc_static_scratch_bytes() == 8 << 20
    ws = torch.full((4 << 20,), -1, dtype=torch.int32, device=dev)
    # the first call is the larger one (2^21 coordinates, 1 MiB of records), the second a smaller one (20 KiB of records)
    # that runs over the same bytes of the array, then the large one again
    cases = [("(512,512,8):(1,512,262144)", "(512,512,8):(512,1,1000)", "bf16"),
             ("(1000,300):(1,1000)", "(1000,300):(3,7)", "f32"),
             ("(512,512,8):(1,512,262144)", "(512,512,8):(512,1,1000)", "bf16"),
             ("(7,5):(1,7)", "(7,5):(2,3)", "b8")]
    for s, d, dt in cases:
        print("case static scratch", s, "->", d, dt, flush=True)
        es = lc.DTYPE_BYTES[dt]
        sl, dl = oracle.Layout(s), oracle.Layout(d)
        rng = np.random.default_rng(len(d))
        src_bits = rng.integers(0, 255, size=sl.cosize * es, dtype=np.uint8).view(_np_int(es))
        want = np.full(dl.cosize * es, 0x5A, np.uint8).view(_np_int(es))
        oracle.copy(src_bits, sl, want, dl)
        plan = lc.Plan(s, d, dt)
        assert "class=last-writer" in plan.describe()
        src_t = torch.from_numpy(src_bits).to(dev)
        got_static = _run(L, plan, "static", src_t, dl.cosize, es, dev)
        got_ws = _run(L, plan, "workspace", src_t, dl.cosize, es, dev, ws)
        assert (got_static == got_ws).all(), plan.describe()
        assert (got_static == want).all(), plan.describe()
    # more scratch than the array holds: refused, nothing launched
    big = lc.Plan("(4096,2048):(1,4096)", "(4096,2048):(3,4097)", "f32")
    assert big.workspace_bytes > L.lc_static_scratch_bytes()
    x = torch.zeros(16, dtype=torch.int32, device=dev)
    st = L.lc_plan_execute_static(big._h, ctypes.c_void_p(x.data_ptr()), ctypes.c_void_p(x.data_ptr()), None)
    assert L.lc_status_string(st).decode() == "SCRATCH_LIMIT"
    assert "8388608" in L.lc_last_hip_error().decode()
    # a plan without scratch runs through the same entry point
    plain = lc.Plan("(64,48):(1,64)", "(64,48):(48,1)", "f32")
    src_bits = np.random.default_rng(3).integers(0, 1 << 31, 64 * 48, dtype=np.int64).astype(np.int32)
    want = np.zeros(64 * 48, np.int32)
    oracle.copy(src_bits, "(64,48):(1,64)", want, "(64,48):(48,1)")
    got = _run(L, plain, "static", torch.from_numpy(src_bits).to(dev), 64 * 48, 4, dev)
    assert (got == want).all()
