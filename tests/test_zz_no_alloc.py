"""The entry point that allocates nothing (softmax2p_f32_static) against softmax2p_f32.

Both run the same kernels with the same launch plan, so the outputs must agree bit for bit
(and therefore meet the same 4e-6 bound against the oracle, which is checked as well).  The
static scratch array keeps what the previous call left in it: every case is run as two calls
in a row, the second on a smaller input, and the second result is checked too."""
import ctypes

import numpy as np
import pytest

from paper_2001_04438_amd import workloads

pytestmark = pytest.mark.gpu

TOL_2P = 4e-6


@pytest.fixture(scope="module")
def gpu():
    import torch
    from paper_2001_04438_amd import binding
    assert torch.cuda.is_available(), "these tests need the MI355X"
    binding.lib()
    binding.softmax_tp_tune_reset()
    yield binding
    binding.softmax_tp_tune_reset()
    binding.softmax_tp_release()


def _pair(gpu, x):
    """(static-scratch result, softmax2p_f32 result) for one input, through the C ABI."""
    import torch
    rows, n = x.shape
    xd = torch.from_numpy(np.ascontiguousarray(x).reshape(-1)).cuda()
    ya = torch.full_like(xd, -7.0)
    yb = torch.full_like(xd, -7.0)
    gpu.softmax2p_f32_static(xd, ya, rows, n)
    torch.cuda.synchronize()
    gpu.softmax2p_f32(xd, yb, rows, n)
    torch.cuda.synchronize()
    return ya.cpu().numpy().reshape(rows, n), yb.cpu().numpy().reshape(rows, n)


# first call, then a smaller second call that reuses the front of the same scratch array
CASES = [
    # several hundred partials + merge launch, then 8 rows of 64 partials folded by pass 2 itself
    ((1, 17_000_003), (8, 300_001)),
    # 64 rows x 8 partials, then one row whose partials land on the slots of rows 0..7
    ((64, 200_003), (1, 1_000_001)),
    # merge launch over two rows, then one row of 128 partials that pass 2 folds itself (stale
    # partials and a stale merged pair behind the live ones)
    ((2, 9_000_001), (1, (1 << 23) + 3)),
    # rows path (no scratch), then chunk path
    ((300, 5000), (3, 70_001)),
]


@pytest.mark.parametrize("first,second", CASES)
def test_static_scratch_matches_the_allocating_entry_point(gpu, oracle_mod, first, second):
    if first[1] > 8_000_000:
        assert gpu.softmax_tp_plan(*first).merge_kernel == 1 and gpu.softmax_tp_plan(*second).merge_kernel == 0
    for rows, n in (first, second):
        x = workloads.cfg3(rows=rows, n=n)
        print(f"softmax2p_f32_static {rows} x {n}", flush=True)
        ya, yb = _pair(gpu, x)
        assert np.array_equal(ya.view(np.uint32), yb.view(np.uint32)), (rows, n)
        c = oracle_mod.compare(x, ya, TOL_2P)
        assert c.n_total == x.size and c.ok(), c.as_dict()


def test_static_scratch_unaligned_and_in_place(gpu, oracle_mod):
    import torch
    x = workloads.cfg3(rows=2, n=200_003)
    flat = torch.from_numpy(x.reshape(-1))
    for x_off, y_off in ((1, 1), (1, 3)):          # 16-byte vectors with edges; element-wise kernels
        xb = torch.empty(flat.numel() + 8, dtype=torch.float32, device="cuda")
        yb = torch.full((flat.numel() + 8,), -7.0, dtype=torch.float32, device="cuda")
        xd, yd = xb[x_off:x_off + flat.numel()], yb[y_off:y_off + flat.numel()]
        xd.copy_(flat)
        gpu.softmax2p_f32_static(xd, yd, 2, 200_003)
        torch.cuda.synchronize()
        assert (yb[:y_off] == -7).all() and (yb[y_off + flat.numel():] == -7).all()
        c = oracle_mod.compare(x, yd.cpu().numpy().reshape(2, 200_003), TOL_2P)
        assert c.ok(), c.as_dict()
    xd = flat.cuda()
    gpu.softmax2p_f32_static(xd, xd, 2, 200_003)
    torch.cuda.synchronize()
    assert oracle_mod.compare(x, xd.cpu().numpy().reshape(2, 200_003), TOL_2P).ok()


def test_static_scratch_rejects_what_does_not_fit(gpu):
    """More partial results than the array holds: refused before anything is launched."""
    import torch
    n = 1 << 26
    x = torch.zeros(n, dtype=torch.float32, device="cuda")
    y = torch.full_like(x, -7.0)
    try:
        gpu.softmax_tp_tune("unroll_reduce", 2)       # 512-vector tiles ...
        gpu.softmax_tp_tune("target_reduce", 1 << 20)  # ... and as many chunks as the row allows
        plan = gpu.softmax_tp_plan(1, n)
        assert (plan.reduce.chunks + 1) * 8 > gpu.TP_STATIC_SCRATCH_BYTES
        with pytest.raises(gpu.SoftmaxTpError) as e:
            gpu.softmax2p_f32_static(x, y, 1, n)
        assert e.value.code == gpu.TP_ERR_SCRATCH
        torch.cuda.synchronize()
        assert bool((y == -7.0).all())
        gpu.softmax_tp_tune("target_reduce", 30000)   # fits: 30000 pairs + 1
        plan = gpu.softmax_tp_plan(1, n)
        assert plan.merge_kernel == 1 and (plan.reduce.chunks + 1) * 8 <= gpu.TP_STATIC_SCRATCH_BYTES
        gpu.softmax2p_f32_static(x, y, 1, n)
        torch.cuda.synchronize()
        assert abs(float(y.double().sum()) - 1.0) < 1e-6 and float(y.max()) == float(y.min())
    finally:
        gpu.softmax_tp_tune_reset()
    # the usual argument checks still come first
    with pytest.raises(gpu.SoftmaxTpError) as e:
        gpu.softmax2p_f32_static(x, None, 1, 5)
    assert e.value.code == gpu.TP_ERR_NULL
    gpu.softmax2p_f32_static(None, None, 0, 0)


def test_static_scratch_call_makes_no_allocation(gpu):
    """Captured into a graph with no reserve, on a shape the library has never seen (an
    allocation during capture would fail the capture); replays agree with the eager
    softmax2p_f32; and the device's free memory does not move over a call."""
    import torch
    rows, n = 3, 700_001
    x = torch.randn(rows * n, dtype=torch.float32, device="cuda")
    y = torch.empty_like(x)
    want = torch.empty_like(x)
    gpu.softmax_tp_release()
    gpu.softmax2p_f32_static(x, y, 2, 70_001)      # first use on this device: address lookup
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        gpu.softmax2p_f32_static(x, y, rows, n)
    for trial in range(3):
        x.copy_(torch.randn_like(x) * 5)
        y.fill_(-7.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        gpu.softmax2p_f32(x, want, rows, n)
        torch.cuda.synchronize()
        assert torch.equal(y, want), trial
    del graph
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    gpu.softmax2p_f32_static(x, y, 1, 2_000_003)   # another new shape, with the merge launch
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    assert free1 == free0
    assert torch.equal(y[:2_000_003].double().sum().round(decimals=5), torch.tensor(1.0, dtype=torch.float64, device="cuda"))
