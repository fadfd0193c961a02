"""The measurement modules on the GPU: results on CU-masked streams against the oracle (the
streams the CU-count scaling study of Section 6.6's analogue runs on), and the size sweep's
measuring function (Sections 6.4 and 6.5's analogue) at two small shapes."""
import numpy as np
import pytest

from paper_2001_04438_amd import workloads

pytestmark = pytest.mark.gpu

TOL = 4e-6
SLOPE_3P = 2.0 ** -24     # the Three-Pass algorithms round x - mu to fp32 before Exp sees it


@pytest.fixture(scope="module")
def gpu():
    import torch
    from paper_2001_04438_amd import binding
    assert torch.cuda.is_available(), "these tests need the MI355X"
    binding.lib()
    binding.softmax_tp_tune_reset()
    yield binding
    binding.softmax_tp_release()


ALGOS = [("softmax2p_f32", 0.0), ("softmax3p_recompute_f32", SLOPE_3P), ("softmax3p_reload_f32", SLOPE_3P)]


@pytest.mark.parametrize("k", [8, 64, 0])          # 0: every compute unit of the device
def test_all_algorithms_on_cu_masked_streams(gpu, oracle_mod, k):
    import torch
    from paper_2001_04438_amd import cu_scaling
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    k = k or cus
    shapes = [workloads.cfg3(rows=3, n=700_001),       # chunk path: partial results cross workgroups
              workloads.cfg4(n=(1 << 22) + 5),         # chunk path with the merge launch
              workloads.cfg2(rows=300, n=5000),        # one workgroup per row
              workloads.cfg2(rows=2000, n=200)]        # one wave per row
    for x in shapes:
        rows, n = x.shape
        xd = torch.from_numpy(x.reshape(-1)).cuda()
        torch.cuda.synchronize()
        for name, slope in ALGOS:
            yd = torch.full_like(xd, -7.0)
            torch.cuda.synchronize()
            print(f"{name} {rows} x {n} on {k} of {cus} compute units", flush=True)
            with cu_scaling.masked_stream(k, cus) as st:
                getattr(gpu, name)(xd, yd, rows, n, stream=st)
            # leaving the block has synchronised the stream
            c = oracle_mod.compare(x, yd.cpu().numpy().reshape(rows, n), TOL, slope=slope)
            assert c.n_total == x.size and c.ok(), (name, k, rows, n, c.as_dict())
    with pytest.raises(ValueError):
        with cu_scaling.masked_stream(cus + 1, cus):
            pass


def test_timing_on_a_masked_stream_scales_with_the_compute_units(gpu):
    """Fewer compute units, longer calls: the mask is really in force, and the timing helper works."""
    import torch
    from paper_2001_04438_amd import cu_scaling
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    n = 1 << 24
    x = torch.randn(n, device="cuda") * 4
    y = torch.empty_like(x)
    torch.cuda.synchronize()
    ms = {}
    for k in (8, cus):
        with cu_scaling.masked_stream(k, cus) as st:
            ms[k] = cu_scaling.time_on_stream(lambda s: gpu.softmax2p_f32(x, y, 1, n, stream=s), st, 5)
    print(ms, flush=True)
    assert ms[8] > 3 * ms[cus] > 0


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_sweep_point(gpu, dtype):
    import torch
    from paper_2001_04438_amd import sweep
    s = 4 if dtype == "f32" else 2
    for rows, n, path in ((512, 4096, "rows"), (2, 1 << 19, "chunk")):
        p = sweep.point(torch, gpu, rows, n, iters=5, dtype=dtype)
        assert p["path"] == path
        expect = {"2p", "3p_recompute", "3p_reload"} | ({"2p_onchip"} if n <= 32768 else set())
        assert set(p) - {"path"} == expect
        for key, _, per_elem in sweep.VARIANTS:
            if key not in p:
                continue
            ms, gbs = p[key]
            assert 0 < ms < 50
            assert gbs == pytest.approx(per_elem * rows * n * s / ms / 1e6)
    # what the sweep times is what the library computes: same call, checked once against torch
    x = torch.randn(64 * 4096, device="cuda") * 4
    y = torch.empty_like(x)
    gpu.softmax2p_f32(x, y, 64, 4096)
    ref = torch.softmax(x.view(64, 4096).double(), dim=1).float().view(-1)
    torch.cuda.synchronize()
    assert float(((y - ref).abs() / ref.clamp_min(1e-30)).max()) < 1e-5
