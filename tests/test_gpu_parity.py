"""GPU parity: every C-ABI softmax entry point against the long-double oracle.

All tests call through the ctypes binding of libsoftmax_tp.so (no fallback) and
compare element by element with the oracle's streaming comparator:

  fp32 I/O, Two-Pass     |y - p| <= 4e-6 p      where p >= FLT_MIN
  bf16 I/O, Two-Pass     |y - p| <= 1e-2 p      (p is the unrounded long-double value)
  fp32 I/O, Three-Pass   |y - p| <= (4e-6 + 2^-24 |x - mu|) p, element by element: the fp32
                                                 subtraction x - mu alone costs up to 2^-24 |x - mu|
                                                 (<= 5.2e-6 while p >= FLT_MIN) before Exp is even called
  fp16 I/O               |y - p| <= 5e-4 p      where p >= 2^-14: one rounding to 11 bits (2^-11 =
                                                 4.883e-4) on top of the fp32 result; 1.1e-3 for
                                                 the reloading variant, which rounds twice
  p < FLT_MIN            |y - p| <= FLT_MIN     (flushed zero or denormal both pass; for fp16 I/O
                                                 the threshold is the format's 2^-14)
  every y finite, >= 0;  |sum_i y_i - 1| <= tol + n 2^-126   (fp16: + n 2^-25, the rounding of
                                                 results in the subnormal range)
"""
import math

import numpy as np
import pytest

from paper_2001_04438_amd import workloads

pytestmark = pytest.mark.gpu

class Bound(float):
    """A relative tolerance that may grow with |x_i - mu| (slope > 0: the Three-Pass rule)."""
    slope = 0.0

    def __new__(cls, tol, slope=0.0):
        b = super().__new__(cls, tol)
        b.slope = slope
        return b


TOL_2P = 4e-6
TOL_3P = Bound(4e-6, slope=2.0 ** -24)
TOL_BF16 = 1e-2
TOL_F16 = 5e-4
TOL_F16_RELOAD = 1.1e-3


@pytest.fixture(scope="module")
def gpu():
    import torch
    from paper_2001_04438_amd import binding
    assert torch.cuda.is_available(), "these tests need the MI355X"
    binding.lib()  # raises if the HIP library has not been built
    yield binding
    binding.softmax_tp_tune_reset()
    binding.softmax_tp_release()


def _run(fn, x, inplace=False, x_off=0, y_off=0):
    """Runs a softmax entry point on a numpy array (fp32, or uint16 holding bf16 bits).

    x_off / y_off shift the device buffers by that many elements to exercise
    unaligned base pointers."""
    import torch
    rows, n = x.shape
    flat = np.ascontiguousarray(x).reshape(-1)
    host = torch.from_numpy(flat.view(np.int16) if flat.dtype == np.uint16 else flat)
    xbuf = torch.empty(flat.size + 16, dtype=host.dtype, device="cuda")
    xd = xbuf[x_off:x_off + flat.size]
    xd.copy_(host)
    if inplace:
        yd = xd
    else:
        ybuf = torch.full((flat.size + 16,), -7, dtype=host.dtype, device="cuda")
        yd = ybuf[y_off:y_off + flat.size]
    fn(xd, yd, rows, n)
    torch.cuda.synchronize()
    if not inplace:
        # nothing outside the output range may be touched
        assert (ybuf[:y_off] == -7).all() and (ybuf[y_off + flat.size:] == -7).all()
    y = yd.cpu().numpy()
    if flat.dtype == np.uint16:
        y = y.view(np.uint16)
    return y.reshape(rows, n)


def _check(oracle_mod, x, y, tol, bf16=False, f16=False):
    slope = getattr(tol, "slope", 0.0)
    c = oracle_mod.compare(x, y, float(tol), bf16=bf16, f16=f16, slope=slope)
    n = x.shape[1]
    assert c.n_total == x.size
    assert c.ok(), c.as_dict()
    if f16:
        assert c.max_row_sum_dev <= 2 * tol + n * 2.0 ** -25, c.as_dict()
    elif slope:   # the allowance weighs in with sum_i p_i |x_i - mu| 2^-24, and p e^-|d| |d| <= 1 / e
        assert c.max_row_sum_dev <= 1e-5 + n * 2.0 ** -126, c.as_dict()
    else:
        assert c.max_row_sum_dev <= (tol if not bf16 else 2 * tol) + n * 2.0 ** -126, c.as_dict()
    return c


ALGOS_F32 = [("softmax2p_f32", TOL_2P), ("softmax3p_recompute_f32", TOL_3P),
             ("softmax3p_reload_f32", TOL_3P)]
ALGOS_F16 = [("softmax2p_f16io", TOL_F16), ("softmax3p_recompute_f16io", TOL_F16),
             ("softmax3p_reload_f16io", TOL_F16_RELOAD)]
ONCHIP_F16 = [("softmax2p_onchip_f16io", TOL_F16), ("softmax3p_onchip_f16io", TOL_F16)]


def _f16(rng, rows, n, scale, shift=0.0):
    x = rng.standard_normal((rows, n)) * scale + shift
    return workloads.f32_to_f16_bits(x.astype(np.float32)).reshape(rows, n)


# ---------------------------------------------------------------------------
# the benchmark configurations (small one in full, large ones at reduced row
# counts here and at full size in test_gpu_full_configs.py)
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("name,tol", ALGOS_F32)
@pytest.mark.parametrize("probes", [False, True])
def test_cfg1_single_vector(gpu, oracle_mod, name, tol, probes):
    x = workloads.cfg1(probes=probes)
    y = _run(getattr(gpu, name), x)
    _check(oracle_mod, x, y, tol)
    if probes:  # e^(1e4) overflows any fp32 exp; the result must be the one-hot limit
        assert y[0, 0] == 1.0 and y[0, 1] == 0.0 and y[0, 2:].max() == 0.0


@pytest.mark.parametrize("name,tol", ALGOS_F32)
def test_cfg2_rows_path(gpu, oracle_mod, name, tol):
    x = workloads.cfg2(rows=37, n=32768)
    assert gpu.softmax_tp_plan(37, 32768).path == 1
    _check(oracle_mod, x, _run(getattr(gpu, name), x), tol)


@pytest.mark.parametrize("name,tol", ALGOS_F32)
def test_cfg3_chunk_path(gpu, oracle_mod, name, tol):
    x = workloads.cfg3(rows=3, n=1_000_000)
    plan = gpu.softmax_tp_plan(3, 1_000_000)
    assert plan.path == 2 and plan.reduce.chunks > 1 and plan.map.chunks > 1
    _check(oracle_mod, x, _run(getattr(gpu, name), x), tol)


@pytest.mark.parametrize("name,tol", ALGOS_F32)
def test_cfg4_single_long_vector(gpu, oracle_mod, name, tol):
    n = (1 << 23) + 3  # thousands of chunks, ragged tail
    x = workloads.cfg4(n=n)
    plan = gpu.softmax_tp_plan(1, n)
    # 32 MiB: 128 chunks of 1024 threads for the read-only passes, no merge launch
    assert plan.path == 2 and plan.merge_kernel == 0 and plan.map.chunks >= 1024
    assert plan.reduce.block == 1024 and 64 < plan.reduce.chunks <= 128
    c = _check(oracle_mod, x, _run(getattr(gpu, name), x), tol)
    assert c.n_normal < x.size // 100  # almost everything underflows next to the outliers
    try:
        # the arrangement of vectors beyond 64 MiB: 512 chunks and a merge launch
        gpu.softmax_tp_tune("target_reduce", 512)
        plan = gpu.softmax_tp_plan(1, n)
        assert plan.merge_kernel == 1 and plan.reduce.block == 256 and plan.reduce.chunks > 128
        _check(oracle_mod, x, _run(getattr(gpu, name), x), tol)
    finally:
        gpu.softmax_tp_tune_reset()


def test_cfg5_bf16(gpu, oracle_mod):
    x = workloads.cfg5(rows=61, n=21846)  # row pitch 43692 B: rows start 0/12/8/4 bytes past 16
    y = _run(gpu.softmax2p_bf16io, x)
    _check(oracle_mod, x, y, TOL_BF16, bf16=True)


def test_bf16_chunk_path(gpu, oracle_mod):
    x = workloads.cfg5(rows=2, n=300_001)
    assert gpu.softmax_tp_plan(2, 300_001, 2).path == 2
    _check(oracle_mod, x, _run(gpu.softmax2p_bf16io, x), TOL_BF16, bf16=True)


@pytest.mark.parametrize("name", ["softmax3p_recompute_bf16io", "softmax3p_reload_bf16io"])
def test_three_pass_bf16_baselines(gpu, oracle_mod, name):
    for x in (workloads.cfg5(rows=61, n=21846), workloads.cfg5(rows=2, n=300_001),
              workloads.cfg5(rows=3, n=1003)):
        _check(oracle_mod, x, _run(getattr(gpu, name), x), TOL_BF16, bf16=True)
    x = workloads.cfg5(rows=5, n=4001)
    _check(oracle_mod, x, _run(getattr(gpu, name), x, x_off=3, y_off=3), TOL_BF16, bf16=True)
    _check(oracle_mod, x, _run(getattr(gpu, name), x, x_off=1, y_off=2), TOL_BF16, bf16=True)
    _check(oracle_mod, x, _run(getattr(gpu, name), x, inplace=True), TOL_BF16, bf16=True)


# ---------------------------------------------------------------------------
# edge shapes, alignment, aliasing
# ---------------------------------------------------------------------------

EDGE_N = [1, 2, 3, 4, 5, 7, 8, 9, 15, 16, 17, 63, 64, 65, 255, 256, 257, 1023, 1024, 1025, 4095,
          4099, 16385]


@pytest.mark.parametrize("name,tol", ALGOS_F32)
def test_edge_lengths_f32(gpu, oracle_mod, name, tol):
    rng = np.random.default_rng(77)
    for n in EDGE_N:
        for rows in (1, 3):
            x = rng.normal(0, 6, size=(rows, n)).astype(np.float32)
            y = _run(getattr(gpu, name), x)
            _check(oracle_mod, x, y, tol)
            if n == 1:  # m * fl(1 / m) may be one rounding below 1 (Algorithm 3 multiplies by lambda)
                assert np.all(np.abs(y - 1.0) <= 2.0 ** -23)


def test_edge_lengths_bf16(gpu, oracle_mod):
    rng = np.random.default_rng(78)
    for n in EDGE_N:
        for rows in (1, 5):
            x = workloads.f32_to_bf16_bits(rng.normal(0, 6, size=(rows, n)).astype(np.float32))
            x = x.reshape(rows, n)
            _check(oracle_mod, x, _run(gpu.softmax2p_bf16io, x), TOL_BF16, bf16=True)


@pytest.mark.parametrize("name,tol", ALGOS_F32)
def test_short_rows_one_lane_group_each(gpu, oracle_mod, name, tol):
    """Rows of at most 12 vectors (16-bit: 16) get a quad of lanes each (64 rows per workgroup), up to
    64 vectors (16-bit: 128) 16 lanes each (16 rows per workgroup), up to 256 vectors a wave each (4 rows
    per workgroup): every unroll of each, row counts that leave groups idle."""
    rng = np.random.default_rng(83)
    for rows, n, lanes in ((1001, 100, 16), (4097, 256, 16), (3000, 33, 4), (50, 1, 1), (17, 64, 16),
                           (1, 129, 16), (33, 7, 1), (260, 255, 16), (5000, 16, 4), (777, 61, 16), (65, 65, 16),
                           (70001, 4, 1), (9999, 8, 1), (257, 9, 1), (300, 2, 1), (1025, 5, 1), (4000, 10, 4),
                           (901, 48, 4), (333, 45, 4), (444, 92, 16), (555, 380, 64), (99, 190, 16),
                           (6, 1024, 64), (513, 1021, 64), (1003, 257, 64), (5, 600, 64), (1234, 768, 64),
                           (700, 1300, 64), (301, 1405, 64), (299, 1409, 256)):   # a second round of the wave
        assert gpu.softmax_tp_plan(rows, n).rows.block == lanes
        x = rng.normal(0, 5, size=(rows, n)).astype(np.float32)
        _check(oracle_mod, x, _run(getattr(gpu, name), x), tol)
    for n in (3, 4, 8, 9, 50, 255, 1001):   # unaligned rows: a lane per row element by element; up to six edge elements
        x = rng.normal(0, 5, size=(333, n)).astype(np.float32)
        _check(oracle_mod, x, _run(getattr(gpu, name), x, x_off=1, y_off=1), tol)
        _check(oracle_mod, x, _run(getattr(gpu, name), x, x_off=1, y_off=2), tol)   # element-wise format
        _check(oracle_mod, x, _run(getattr(gpu, name), x, inplace=True), tol)
    # rows far apart in magnitude side by side in one wave: the 16-lane reductions do not mix them
    for n in (200, 40):           # 16 lanes per row, 4 lanes per row
        x = rng.normal(0, 2, size=(64, n)).astype(np.float32) + (np.arange(64, dtype=np.float32) * 900 - 30000)[:, None]
        _check(oracle_mod, x, _run(getattr(gpu, name), x), tol)
    x[5, 17] = np.nan
    y = _run(getattr(gpu, name), x)
    assert np.isnan(y[5]).all() and np.isfinite(np.delete(y, 5, axis=0)).all()


def test_short_rows_with_and_without_the_store_hint(gpu, oracle_mod):
    """Rows on 4 or 16 lanes store y with or without the non-temporal hint depending on how they
    share cache lines; both variants of every kernel, forced through the tuning key, and the default."""
    rng = np.random.default_rng(98)
    try:
        for setting in (1, 2, 0):
            gpu.softmax_tp_tune("nt_store", setting)
            for rows, n in ((3001, 25), (2000, 100), (999, 64), (700, 250), (300, 1000)):
                x = rng.normal(0, 5, size=(rows, n)).astype(np.float32)
                for name, tol in ALGOS_F32 + ONCHIP_F32:
                    _check(oracle_mod, x, _run(getattr(gpu, name), x), tol)
                    _check(oracle_mod, x, _run(getattr(gpu, name), x, inplace=True), tol)
                xb = workloads.f32_to_bf16_bits(x).reshape(x.shape)
                for name in ("softmax2p_bf16io", "softmax3p_recompute_bf16io", "softmax3p_reload_bf16io") + tuple(ONCHIP_BF16):
                    _check(oracle_mod, xb, _run(getattr(gpu, name), xb, x_off=3, y_off=3), TOL_BF16, bf16=True)
    finally:
        gpu.softmax_tp_tune_reset()


@pytest.mark.parametrize("name,tol", ALGOS_F32)
def test_very_many_rows(gpu, oracle_mod, name, tol):
    """Grids of hundreds of thousands of workgroups: one wave per row and one workgroup per row."""
    rng = np.random.default_rng(85)
    for rows, n in (((1 << 20) + 3, 7), (300_001, 64), (70_001, 1500)):
        x = rng.normal(0, 3, size=(rows, n)).astype(np.float32)
        c = _check(oracle_mod, x, _run(getattr(gpu, name), x), tol)
        assert c.n_total == rows * n


def test_short_rows_one_wave_each_bf16(gpu, oracle_mod):
    rng = np.random.default_rng(84)
    for name in ("softmax2p_bf16io", "softmax3p_recompute_bf16io", "softmax3p_reload_bf16io"):
        for rows, n in ((1001, 100), (4097, 512), (7, 2048), (513, 2041), (300, 513), (9, 8), (2000, 37),
                        (1500, 96), (700, 192), (600, 768), (450, 1000), (350, 1536), (3333, 48),
                        (500, 3000), (257, 4090), (255, 4100), (30001, 4), (777, 16), (555, 11), (444, 15), (3, 1)):
            assert gpu.softmax_tp_plan(rows, n, 2).rows.block == (1 if n <= 16 else 4 if n <= 128 else 16 if n <= 1024
                                                                  else 64 if n <= 4096 else 256)
            x = workloads.f32_to_bf16_bits(rng.normal(0, 5, size=(rows, n)).astype(np.float32)).reshape(rows, n)
            _check(oracle_mod, x, _run(getattr(gpu, name), x), TOL_BF16, bf16=True)
        x = workloads.cfg5(rows=77, n=1003)
        _check(oracle_mod, x, _run(getattr(gpu, name), x, x_off=3, y_off=3), TOL_BF16, bf16=True)
        for n in (4, 8, 13, 16):     # a lane per row: vectors only when every row starts on 16 bytes
            x = workloads.f32_to_bf16_bits(rng.normal(0, 5, size=(2001, n)).astype(np.float32)).reshape(2001, n)
            for off, yoff in ((1, 1), (8, 8), (4, 4), (0, 3)):
                _check(oracle_mod, x, _run(getattr(gpu, name), x, x_off=off, y_off=yoff), TOL_BF16, bf16=True)
            _check(oracle_mod, x, _run(getattr(gpu, name), x, inplace=True), TOL_BF16, bf16=True)


@pytest.mark.parametrize("name,tol", ALGOS_F32)
def test_unaligned_and_incongruent_pointers_f32(gpu, oracle_mod, name, tol):
    rng = np.random.default_rng(79)
    x = rng.normal(0, 5, size=(4, 1001)).astype(np.float32)
    for x_off, y_off in ((1, 1), (3, 3), (2, 2), (0, 1), (3, 0), (1, 2)):
        _check(oracle_mod, x, _run(getattr(gpu, name), x, x_off=x_off, y_off=y_off), tol)
    big = workloads.cfg3(rows=2, n=200_003)  # chunk path, rows not 16-byte aligned
    for x_off, y_off in ((0, 0), (1, 1), (1, 3)):
        _check(oracle_mod, big, _run(getattr(gpu, name), big, x_off=x_off, y_off=y_off), tol)


def test_unaligned_and_incongruent_pointers_bf16(gpu, oracle_mod):
    x = workloads.cfg5(rows=5, n=1003)
    for x_off, y_off in ((0, 0), (1, 1), (7, 7), (0, 1), (5, 2)):
        y = _run(gpu.softmax2p_bf16io, x, x_off=x_off, y_off=y_off)
        _check(oracle_mod, x, y, TOL_BF16, bf16=True)


@pytest.mark.parametrize("name,tol", ALGOS_F32)
def test_in_place(gpu, oracle_mod, name, tol):
    for x in (workloads.cfg2(rows=33, n=5000), workloads.cfg3(rows=2, n=150_001)):
        _check(oracle_mod, x, _run(getattr(gpu, name), x, inplace=True), tol)


def test_in_place_bf16(gpu, oracle_mod):
    x = workloads.cfg5(rows=9, n=3001)
    _check(oracle_mod, x, _run(gpu.softmax2p_bf16io, x, inplace=True), TOL_BF16, bf16=True)


# ---------------------------------------------------------------------------
# fp16 storage
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("name,tol", ALGOS_F16 + ONCHIP_F16)
def test_f16_all_paths(gpu, oracle_mod, name, tol):
    rng = np.random.default_rng(1616)
    fn = getattr(gpu, name)
    onchip = "onchip" in name
    shapes = [(1000, 300, 2.0), (257, 1000, 1.0), (64, 4096, 2.0), (5, 21846, 4.0), (3, 32768, 6.0)]
    if not onchip:
        shapes += [(40, 65536, 6.0), (2, 300_001, 8.0), (1, 1 << 21, 10.0)]
    normal = 0
    for rows, n, scale in shapes:
        x = _f16(rng, rows, n, scale, shift=rng.uniform(-30, 30, size=(rows, 1)))
        c = _check(oracle_mod, x, _run(fn, x), tol, f16=True)
        normal += c.n_normal
    assert normal > 400_000          # enough results in the normal range for the relative bound to bite
    x = _f16(rng, 7, 5003, 3.0)
    _check(oracle_mod, x, _run(fn, x, x_off=3, y_off=3), tol, f16=True)
    _check(oracle_mod, x, _run(fn, x, inplace=True), tol, f16=True)
    if not onchip:                   # x and y not congruent modulo 16 bytes: element-wise kernels
        _check(oracle_mod, x, _run(fn, x, x_off=1, y_off=2), tol, f16=True)
        x = _f16(rng, 2, 200_003, 8.0)
        _check(oracle_mod, x, _run(fn, x, x_off=1, y_off=4), tol, f16=True)


@pytest.mark.parametrize("name,tol", ALGOS_F16)
def test_f16_edge_lengths_and_range(gpu, oracle_mod, name, tol):
    rng = np.random.default_rng(1617)
    fn = getattr(gpu, name)
    for rows in (1, 3):
        for n in (1, 2, 7, 8, 9, 63, 64, 65, 511, 513, 2047, 2049, 8191, 8193):
            x = _f16(rng, rows, n, 5.0)
            _check(oracle_mod, x, _run(fn, x), tol, f16=True)
    # the whole range of the format in one row: +-65504 next to subnormals and zeros
    x = np.array([[0x7BFF, 0xFBFF, 0x0001, 0x8001, 0x03FF, 0x0000, 0x8000, 0x7BFE, 0x7BFF, 0x3C00]],
                 dtype=np.uint16)
    y = _run(fn, x)
    c = _check(oracle_mod, x, y, tol, f16=True)
    assert c.n_normal == 2           # the two maxima share the mass; their neighbour is 32 below
    # rows made of fp16 subnormals and zeros only: a uniform distribution to within 6e-5
    x = rng.integers(0, 0x0400, size=(4, 1000)).astype(np.uint16)
    x[:, ::3] |= 0x8000
    _check(oracle_mod, x, _run(fn, x), tol, f16=True)
    # a long flat row: every result is an fp16 subnormal, held to 2^-25 absolute
    x = _f16(rng, 1, 1 << 20, 0.01)
    c = _check(oracle_mod, x, _run(fn, x), tol, f16=True)
    assert c.n_normal == 0 and c.max_sub_abs_err <= 2.0 ** -25 * 1.01


def test_empty_and_invalid_arguments(gpu):
    import torch
    t = torch.zeros(64, dtype=torch.float32, device="cuda")
    for fn in (gpu.softmax2p_f32, gpu.softmax3p_recompute_f32, gpu.softmax3p_reload_f32):
        fn(t, t, 0, 5)
        fn(t, t, 5, 0)
        fn(None, None, 0, 0)
        for args, code in (((t, t, -1, 4), gpu.TP_ERR_NEGATIVE), ((None, t, 1, 4), gpu.TP_ERR_NULL),
                           ((t, None, 1, 4), gpu.TP_ERR_NULL),
                           ((t, t, 1 << 40, 1 << 40), gpu.TP_ERR_TOO_LARGE),
                           ((t.data_ptr() + 2, t, 1, 4), gpu.TP_ERR_ALIGN)):
            with pytest.raises(gpu.SoftmaxTpError) as e:
                fn(*args)
            assert e.value.code == code
    torch.cuda.synchronize()
    assert float(t.abs().sum()) == 0.0


def test_nan_poisons_only_its_row(gpu):
    x = workloads.cfg2(rows=34, n=3000)
    x[5, 17] = np.nan
    for name, _ in ALGOS_F32:
        y = _run(getattr(gpu, name), x)
        assert np.isnan(y[5]).all()
        assert np.isfinite(np.delete(y, 5, axis=0)).all()


def test_infinity_poisons_only_its_row(gpu):
    """Infinite inputs are outside the contract (the header says so); what happens is pinned
    all the same: the range reduction turns an infinity into NaN, so the row that holds it comes
    out NaN, as with a NaN input, and no other row is touched."""
    base = workloads.cfg2(rows=34, n=3000)
    for bad in (-np.inf, np.inf):
        x = base.copy()
        x[7, 1234] = bad
        for name in ("softmax2p_f32", "softmax3p_recompute_f32", "softmax3p_reload_f32",
                     "softmax2p_onchip_f32", "softmax3p_onchip_f32"):
            y = _run(getattr(gpu, name), x)
            assert np.isnan(y[7]).all(), (name, bad)
            assert np.isfinite(np.delete(y, 7, axis=0)).all(), (name, bad)
        xb = workloads.f32_to_bf16_bits(x).reshape(x.shape)
        xh = workloads.f32_to_f16_bits(x).reshape(x.shape)
        for name, xs, conv in (("softmax2p_bf16io", xb, workloads.bf16_bits_to_f32),
                               ("softmax2p_onchip_bf16io", xb, workloads.bf16_bits_to_f32),
                               ("softmax2p_f16io", xh, workloads.f16_bits_to_f32),
                               ("softmax2p_onchip_f16io", xh, workloads.f16_bits_to_f32)):
            y = conv(_run(getattr(gpu, name), xs)).reshape(x.shape)
            assert np.isnan(y[7]).all(), (name, bad)
            assert np.isfinite(np.delete(y, 7, axis=0)).all(), (name, bad)


def test_a_stale_hip_error_of_the_callers_is_not_reported_as_ours(gpu, oracle_mod):
    """An earlier failed HIP call of the caller's leaves an error behind in the thread.  The
    library reports what its own launches return, so the call succeeds and every pass runs."""
    import ctypes
    import torch
    hip = ctypes.CDLL("libamdhip64.so")
    hip.hipMalloc.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_size_t]
    x = workloads.cfg3(rows=2, n=1_500_000)
    rows, n = x.shape
    xd = torch.from_numpy(x.reshape(-1)).cuda()
    for name, tol in ALGOS_F32:                       # three to five launches each
        yd = torch.full_like(xd, -7.0)
        torch.cuda.synchronize()
        p = ctypes.c_void_p()
        assert hip.hipMalloc(ctypes.byref(p), 1 << 60) != 0     # refused: far beyond the device
        rc = getattr(gpu.lib(), name)(xd.data_ptr(), yd.data_ptr(), rows, n, None)
        hip.hipGetLastError()                          # leave no error behind for torch to find
        assert rc == 0, (name, rc)
        torch.cuda.synchronize()
        _check(oracle_mod, x, yd.cpu().numpy().reshape(rows, n), tol)


# ---------------------------------------------------------------------------
# on-chip variant (row kept in registers between the passes)
# ---------------------------------------------------------------------------

ONCHIP_F32 = [("softmax2p_onchip_f32", TOL_2P), ("softmax3p_onchip_f32", TOL_3P)]
ONCHIP_BF16 = ["softmax2p_onchip_bf16io", "softmax3p_onchip_bf16io"]


@pytest.mark.parametrize("name,tol", ONCHIP_F32)
def test_onchip_f32(gpu, oracle_mod, name, tol):
    fn = getattr(gpu, name)
    rng = np.random.default_rng(90)
    cases = [workloads.cfg1(), workloads.cfg1(probes=True), workloads.cfg2(rows=37, n=32768),
             workloads.cfg2(rows=700, n=8192),          # more rows than resident workgroups
             workloads.cfg2(rows=2100, n=1000)]
    # (1026, 2050, 4100, 8197: a vector or two more than a power of two, which no tile fills slot by slot)
    for n in EDGE_N + [1026, 2050, 4100, 8191, 8193, 8197, 20000, 28001, 32767]:
        cases.append(rng.normal(0, 6, size=(3, n)).astype(np.float32))
    for x in cases:
        _check(oracle_mod, x, _run(fn, x), tol)
    x = workloads.cfg2(rows=9, n=5003)
    for off in (1, 2, 3):                                # rows start anywhere relative to 16 bytes
        _check(oracle_mod, x, _run(fn, x, x_off=off, y_off=off), tol)
    _check(oracle_mod, x, _run(fn, x, inplace=True), tol)
    # same arithmetic as the entry point that traverses memory for every pass
    x = workloads.cfg2(rows=40, n=32768)
    a = _run(fn, x)
    b = _run(gpu.softmax2p_f32 if name.startswith("softmax2p") else gpu.softmax3p_reload_f32, x)
    nz = b > 1e-30
    assert np.max(np.abs(a[nz] - b[nz]) / b[nz]) < 1e-6


@pytest.mark.parametrize("name", ONCHIP_BF16)
def test_onchip_bf16(gpu, oracle_mod, name):
    fn = getattr(gpu, name)
    rng = np.random.default_rng(91)
    cases = [workloads.cfg5(rows=61, n=21846), workloads.cfg5(rows=1500, n=3000),
             workloads.cfg5(rows=5, n=32768)]
    for n in EDGE_N + [2052, 4100, 8200, 16383, 16390, 21841, 32767]:
        cases.append(workloads.f32_to_bf16_bits(rng.normal(0, 6, size=(3, n)).astype(np.float32)).reshape(3, n))
    for x in cases:
        _check(oracle_mod, x, _run(fn, x), TOL_BF16, bf16=True)
    x = workloads.cfg5(rows=7, n=3001)
    for off in (1, 5, 7):
        _check(oracle_mod, x, _run(fn, x, x_off=off, y_off=off), TOL_BF16, bf16=True)
    _check(oracle_mod, x, _run(fn, x, inplace=True), TOL_BF16, bf16=True)


@pytest.mark.parametrize("fmt", ["f32", "bf16", "f16"])
def test_onchip_short_rows_every_lane_group(gpu, oracle_mod, fmt):
    """Rows of at most 256 vectors are held by a quad, a row of 16 lanes or a wave: every group with
    one to four vectors per lane, many rows per wave, bases that leave up to 2 (V - 1) edge elements
    (more than a quad has lanes) and row counts that leave groups idle."""
    rng = np.random.default_rng(92)
    V = 4 if fmt == "f32" else 8
    names = {"f32": ONCHIP_F32, "bf16": [(n, TOL_BF16) for n in ONCHIP_BF16], "f16": ONCHIP_F16}[fmt]
    for nvec in (1, 2, 3, 4, 5, 7, 8, 9, 12, 16, 17, 31, 33, 48, 64, 65, 100, 129, 190, 255, 256):
        for n in {nvec * V, max(1, nvec * V - V // 2 - 1)}:
            rows = 1000 // nvec + 7
            x = (rng.normal(0, 5, size=(rows, n)) + rng.uniform(-40, 40, size=(rows, 1))).astype(np.float32)
            if fmt == "bf16":
                x = workloads.f32_to_bf16_bits(x).reshape(rows, n)
            elif fmt == "f16":
                x = workloads.f32_to_f16_bits(x).reshape(rows, n)
            for name, tol in names:
                for off in (0, 1, V - 1):
                    y = _run(getattr(gpu, name), x, x_off=off, y_off=off)
                    _check(oracle_mod, x, y, tol, bf16=fmt == "bf16", f16=fmt == "f16")


def test_onchip_limits(gpu):
    import torch
    t = torch.zeros(40000, dtype=torch.float32, device="cuda")
    for fn in (gpu.softmax2p_onchip_f32, gpu.softmax3p_onchip_f32):
        with pytest.raises(gpu.SoftmaxTpError) as e:        # row longer than the register tile
            fn(t, t, 1, 32769)
        assert e.value.code == gpu.TP_ERR_TOO_LARGE
        with pytest.raises(gpu.SoftmaxTpError) as e:        # x and y not congruent modulo 16 bytes
            fn(t, t.data_ptr() + 4, 1, 100)
        assert e.value.code == gpu.TP_ERR_ALIGN
        fn(t, t, 0, 100)
    torch.cuda.synchronize()
    assert float(t.abs().sum()) == 0.0


# ---------------------------------------------------------------------------
# wide dynamic range: nothing overflows, shift invariance
# ---------------------------------------------------------------------------

def test_extreme_magnitudes_two_pass(gpu, oracle_mod):
    rng = np.random.default_rng(80)
    base = rng.normal(0, 3, size=(6, 2000)).astype(np.float32)
    for c in (0.0, 88.0, -104.0, 1e4, -1e4, 9e4, -9e4):
        x = (base + np.float32(c)).astype(np.float32)
        y = _run(gpu.softmax2p_f32, x)
        _check(oracle_mod, x, y, TOL_2P)
    # rows mixing huge positive and negative entries
    x = base.copy()
    x[:, ::7] += np.float32(5e3)
    x[:, 1::7] -= np.float32(7e4)
    _check(oracle_mod, x, _run(gpu.softmax2p_f32, x), TOL_2P)
    xb = workloads.f32_to_bf16_bits(x).reshape(x.shape)
    _check(oracle_mod, xb, _run(gpu.softmax2p_bf16io, xb), TOL_BF16, bf16=True)


def test_bf16_up_to_the_edge_of_its_exponent_trick(gpu, oracle_mod):
    """The 16-bit entry points read the exponent from the bit pattern of x log2e + 1.5 * 2^23, valid
    for |x| < 2.9e6.  bf16 values of that size are 8192 or 16384 apart, so rows there are ties at the
    maximum sharing the mass; rows a few thousand in size still have structure."""
    rng = np.random.default_rng(86)
    for centre, spread in ((2.0e6, 3e4), (-2.7e6, 5e4), (3.0e4, 40.0), (-1.0e5, 300.0)):
        x = (rng.normal(0, spread, size=(7, 3001)) + centre).astype(np.float32)
        xb = workloads.f32_to_bf16_bits(x).reshape(x.shape)
        for name in ("softmax2p_bf16io", "softmax2p_onchip_bf16io", "softmax3p_recompute_bf16io"):
            y = _run(getattr(gpu, name), xb)
            c = _check(oracle_mod, xb, y, TOL_BF16, bf16=True)
            assert c.n_normal >= 7            # at least the maximum of every row


def test_shift_invariance_on_gpu(gpu):
    rng = np.random.default_rng(81)
    x = (rng.integers(-3000, 3000, size=(4, 777)) / 256.0).astype(np.float32)
    y0 = _run(gpu.softmax2p_f32, x)
    for c in (64.0, -512.0, 8192.0):
        yc = _run(gpu.softmax2p_f32, (x + np.float32(c)).astype(np.float32))
        nz = y0 > 1e-30
        assert np.max(np.abs(yc[nz] - y0[nz]) / y0[nz]) < 2 * TOL_2P


# ---------------------------------------------------------------------------
# pieces of the path: ExtExp, pass 1 pairs, pass 2
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("name", ["softmax_tp_extexp_f32", "softmax_tp_extexp_hw_f32"])
def test_extexp_pairs(gpu, oracle_mod, name):
    import torch
    rng = np.random.default_rng(82)
    xs = np.concatenate([
        np.linspace(-104, 89, 200_001), rng.uniform(-1e5, 1e5, 100_000),
        rng.normal(0, 1e-3, 1000), [0.0, -0.0, 1e4, -1e4, 88.72, -103.97, 0.34657359, -0.34657359],
    ]).astype(np.float32)
    xd = torch.from_numpy(xs).cuda()
    md = torch.empty_like(xd)
    ed = torch.empty_like(xd)
    getattr(gpu, name)(xd, md, ed, xs.size)
    torch.cuda.synchronize()
    m, e = md.cpu().numpy(), ed.cpu().numpy()
    if name.endswith("hw_f32"):            # both evaluators split x at the same n
        m0, e0 = torch.empty_like(xd), torch.empty_like(xd)
        gpu.softmax_tp_extexp_f32(xd, m0, e0, xs.size)
        assert torch.equal(e0, ed)
        assert float(((m0 - md).abs() / m0).max()) < 4e-7
    assert np.all(e == np.rint(e))                                   # n is an integer
    assert np.all(np.abs(e - xs.astype(np.float64) * 1.4426950408889634) <= 0.5 + 1e-2)
    inner = np.abs(xs) <= 1e4
    # Section 4: m = e^t in [sqrt(2)/2, sqrt(2)] (up to the slop of rounding x log2 e)
    assert m[inner].min() >= math.sqrt(2) / 2 * (1 - 2e-3) and m[inner].max() <= math.sqrt(2) * (1 + 2e-3)
    rel, worst = oracle_mod.pair_rel_err(xs, m, e)
    assert rel[inner].max() < 2.5e-7       # 2 ULP of a value just below a power of two
    assert worst < 4e-7                    # |x| up to 1e5: reduced argument slightly outside the fit


def test_pass1_pairs_and_pass2(gpu, oracle_mod):
    import torch
    for x in (workloads.cfg1(probes=True), workloads.cfg3(rows=5, n=70_001), workloads.cfg4(n=3_000_000)):
        rows, n = x.shape
        xd = torch.from_numpy(x.reshape(-1)).cuda()
        pairs = torch.empty(2 * rows, dtype=torch.float32, device="cuda")
        gpu.softmax2p_f32_pass1(xd, pairs, rows, n)
        yd = torch.empty_like(xd)
        gpu.softmax2p_f32_pass2(xd, pairs, yd, rows, n)
        torch.cuda.synchronize()
        p = pairs.cpu().numpy().reshape(rows, 2)
        for r in range(rows):
            m_sum, n_sum = float(p[r, 0]), float(p[r, 1])
            assert n_sum == round(n_sum) and m_sum >= 0.7
            # n_sum is the largest exponent in the row
            assert abs(n_sum - float(x[r].max()) * 1.4426950408889634) <= 0.51
            lse = float(oracle_mod.logsumexp(x[r]))
            assert abs(math.log(m_sum) + n_sum * math.log(2.0) - lse) < 3e-6
        _check(oracle_mod, x, yd.cpu().numpy().reshape(rows, n), TOL_2P)


def test_two_pass_and_three_pass_agree(gpu):
    x = workloads.cfg2(rows=35, n=8192)
    y2 = _run(gpu.softmax2p_f32, x)
    for name in ("softmax3p_recompute_f32", "softmax3p_reload_f32"):
        y3 = _run(getattr(gpu, name), x)
        nz = y2 > 1e-30
        assert np.max(np.abs(y3[nz] - y2[nz]) / y2[nz]) < 1e-5


# ---------------------------------------------------------------------------
# every launch shape gives the same answer; runs are reproducible
# ---------------------------------------------------------------------------

def test_launch_shapes(gpu, oracle_mod):
    x = workloads.cfg3(rows=4, n=50_003)
    xb = workloads.cfg5(rows=4, n=50_003)
    try:
        for path in (1, 2):
            gpu.softmax_tp_tune("path", path)
            for block in (256, 512, 1024):
                for unroll in (2, 4, 8):
                    for key in ("block_rows", "block_reduce", "block_map", "block_mapsum"):
                        gpu.softmax_tp_tune(key, block)
                    for key in ("unroll_rows", "unroll_reduce", "unroll_map", "unroll_mapsum"):
                        gpu.softmax_tp_tune(key, unroll)
                    for name, tol in ALGOS_F32:
                        _check(oracle_mod, x, _run(getattr(gpu, name), x), tol)
                    if unroll < 8:
                        _check(oracle_mod, xb, _run(gpu.softmax2p_bf16io, xb), TOL_BF16, bf16=True)
                    else:  # bf16 keeps at most four 16-byte loads in flight
                        with pytest.raises(gpu.SoftmaxTpError):
                            _run(gpu.softmax2p_bf16io, xb)
        # chunk path: many small chunks vs few large ones, every direction / hint setting
        gpu.softmax_tp_tune_reset()
        gpu.softmax_tp_tune("path", 2)
        for direction in (1, 2):
            for nt_first in (1, 2):
                for target, tiles in ((64, 1), (100_000, 3)):
                    gpu.softmax_tp_tune("direction", direction)
                    gpu.softmax_tp_tune("nt_first", nt_first)
                    gpu.softmax_tp_tune("target_reduce", target)
                    gpu.softmax_tp_tune("tiles_map", tiles)
                    gpu.softmax_tp_tune("tiles_mapsum", tiles)
                    for name, tol in ALGOS_F32:
                        _check(oracle_mod, x, _run(getattr(gpu, name), x), tol)
                    _check(oracle_mod, xb, _run(gpu.softmax2p_bf16io, xb), TOL_BF16, bf16=True)
        # the read-write shape used for arrays beyond the caches: 128 threads, one access each
        gpu.softmax_tp_tune_reset()
        gpu.softmax_tp_tune("path", 2)
        gpu.softmax_tp_tune("block_map", 128)
        gpu.softmax_tp_tune("unroll_map", 1)
        xh = workloads.f32_to_f16_bits(x).reshape(x.shape)
        for tiles in (1, 2, 5):
            gpu.softmax_tp_tune("tiles_map", tiles)
            for name, tol in ALGOS_F32:
                _check(oracle_mod, x, _run(getattr(gpu, name), x, x_off=1, y_off=1), tol)
            _check(oracle_mod, xb, _run(gpu.softmax2p_bf16io, xb), TOL_BF16, bf16=True)
            _check(oracle_mod, xh, _run(gpu.softmax3p_recompute_f16io, xh), TOL_F16, f16=True)
        gpu.softmax_tp_tune("unroll_map", 2)               # 128 threads come with one access only
        with pytest.raises(gpu.SoftmaxTpError):
            _run(gpu.softmax2p_f32, x)
    finally:
        gpu.softmax_tp_tune_reset()


def test_every_default_shape_of_the_rows_path(gpu, oracle_mod):
    """The planner gives every algorithm its own workgroup shape by row length; one row length inside
    every step of every table, each algorithm in each format, all of them ragged."""
    seen = set()
    rng = np.random.default_rng(97)
    for s, lengths in ((4, (2901, 3503, 5001, 9003, 14001, 19999, 30001, 50003)),
                       (2, (5001, 9003, 15001, 24999, 40001, 59999, 90001, 120003))):
        for n in lengths:
            rows = 37
            x = (rng.normal(0, 6, size=(rows, n)) + rng.uniform(-30, 30, size=(rows, 1))).astype(np.float32)
            plan = gpu.softmax_tp_plan(rows, n, s)
            assert plan.path == 1
            for sh in (plan.rows, plan.rows_recompute, plan.rows_reload):
                seen.add((s, sh.block, sh.unroll))
            if s == 4:
                for name, tol in ALGOS_F32:
                    _check(oracle_mod, x, _run(getattr(gpu, name), x), tol)
            else:
                xb = workloads.f32_to_bf16_bits(x).reshape(x.shape)
                xh = workloads.f32_to_f16_bits(x).reshape(x.shape)
                for name in ("softmax2p_bf16io", "softmax3p_recompute_bf16io", "softmax3p_reload_bf16io"):
                    _check(oracle_mod, xb, _run(getattr(gpu, name), xb), TOL_BF16, bf16=True)
                for name, tol in ALGOS_F16:
                    _check(oracle_mod, xh, _run(getattr(gpu, name), xh), tol, f16=True)
    assert {(4, 256, 2), (4, 512, 2), (4, 1024, 2), (4, 1024, 4), (4, 1024, 8),
            (2, 256, 2), (2, 512, 2), (2, 512, 4), (2, 1024, 2), (2, 1024, 4)} <= seen, seen


@pytest.mark.parametrize("name,tol", ALGOS_F32)
def test_partials_folded_by_the_consuming_pass(gpu, oracle_mod, name, tol):
    """65..128 partials per row: lanes fold two each; the fold_max key moves the hand-over
    to the merge kernel either way."""
    fn = getattr(gpu, name)
    for rows, n in ((4, 1_200_001), (4, 1_500_001)):
        plan = gpu.softmax_tp_plan(rows, n)
        assert plan.path == 2 and 64 < plan.reduce.chunks <= 128 and plan.merge_kernel == 0
        x = workloads.cfg3(rows=rows, n=n)
        want = _run(fn, x)
        _check(oracle_mod, x, want, tol)
        try:
            gpu.softmax_tp_tune("fold_max", 64)
            assert gpu.softmax_tp_plan(rows, n).reduce.chunks <= 64   # inputs this short follow the limit
            gpu.softmax_tp_tune("target_reduce", 512)                  # ... unless the sweep insists
            assert gpu.softmax_tp_plan(rows, n).merge_kernel == 1
            _check(oracle_mod, x, _run(fn, x), tol)
            gpu.softmax_tp_tune("fold_max", 512)
            x1 = workloads.cfg3(rows=1, n=3_000_017)
            plan = gpu.softmax_tp_plan(1, 3_000_017)
            assert plan.merge_kernel == 0 and plan.reduce.chunks > 128
            _check(oracle_mod, x1, _run(fn, x1), tol)
        finally:
            gpu.softmax_tp_tune_reset()


def test_bitwise_reproducible(gpu):
    x = workloads.cfg3(rows=2, n=400_000)
    for name, _ in ALGOS_F32:
        a = _run(getattr(gpu, name), x)
        b = _run(getattr(gpu, name), x)
        assert np.array_equal(a, b)


def test_random_shapes_all_entry_points(gpu, oracle_mod):
    """Seeded random (rows, n, pointer offset) across every path boundary."""
    rng = np.random.default_rng(20010443)
    f32 = [("softmax2p_f32", TOL_2P), ("softmax3p_recompute_f32", TOL_3P), ("softmax3p_reload_f32", TOL_3P),
           ("softmax2p_onchip_f32", TOL_2P), ("softmax3p_onchip_f32", TOL_3P)]
    bf16 = ["softmax2p_bf16io", "softmax3p_recompute_bf16io", "softmax3p_reload_bf16io",
            "softmax2p_onchip_bf16io", "softmax3p_onchip_bf16io"]
    f16 = ALGOS_F16 + ONCHIP_F16
    for trial in range(40):
        kind = trial % 4
        if kind == 0:      # short rows, many of them
            rows, n = int(rng.integers(1, 3000)), int(rng.integers(1, 1100))
        elif kind == 1:    # rows-path sizes
            rows, n = int(rng.integers(1, 200)), int(rng.integers(1000, 66000))
        elif kind == 2:    # chunk path, few long rows
            rows, n = int(rng.integers(1, 6)), int(rng.integers(70_000, 900_000))
        else:              # around the register-tile limits of the on-chip kernels
            rows, n = int(rng.integers(1, 600)), int(rng.choice([4095, 4096, 4097, 8191, 8192, 12289,
                                                                 16384, 20481, 24577, 32767, 32768]))
        off = int(rng.integers(0, 4))
        scale = float(rng.choice([0.5, 4.0, 30.0]))
        x = (rng.standard_normal((rows, n)) * scale + rng.uniform(-50, 50, size=(rows, 1))).astype(np.float32)
        xb = workloads.f32_to_bf16_bits(x).reshape(rows, n)
        xh = workloads.f32_to_f16_bits(x).reshape(rows, n)
        print(f"trial {trial}: rows={rows} n={n} off={off} scale={scale}", flush=True)
        for name, tol in f32:
            if "onchip" in name and n > 32768:
                continue
            _check(oracle_mod, x, _run(getattr(gpu, name), x, x_off=off, y_off=off), tol)
        for name in bf16:
            if "onchip" in name and n > 32768:
                continue
            _check(oracle_mod, xb, _run(getattr(gpu, name), xb, x_off=2 * off, y_off=2 * off), TOL_BF16, bf16=True)
        for name, tol in f16:
            if "onchip" in name and n > 32768:
                continue
            _check(oracle_mod, xh, _run(getattr(gpu, name), xh, x_off=2 * off, y_off=2 * off), tol, f16=True)


def test_reserve_and_release(gpu, oracle_mod):
    gpu.softmax_tp_release()
    gpu.softmax_tp_reserve(3, 500_000)            # chunk path: workspace allocated up front
    gpu.softmax_tp_reserve(100, 1000)             # rows path: nothing to allocate
    x = workloads.cfg3(rows=3, n=500_000)
    _check(oracle_mod, x, _run(gpu.softmax2p_f32, x), TOL_2P)
    gpu.softmax_tp_release()
    _check(oracle_mod, x, _run(gpu.softmax3p_reload_f32, x), TOL_3P)   # allocates again on demand
    with pytest.raises(gpu.SoftmaxTpError):
        gpu.softmax_tp_reserve(-1, 5)


def test_capture_into_a_graph_and_replay(gpu, oracle_mod):
    """A serving loop captures the call once and replays it: no allocation, no host
    synchronisation and no memset may hide in the call once its workspace is reserved."""
    import torch
    side = torch.cuda.Stream()
    cases = [("softmax2p_f32", 3, 700_001, TOL_2P),            # chunk path, pass 2 folds the partials
             ("softmax2p_f32", 1, 3_000_017, TOL_2P),          # chunk path with the merge launch
             ("softmax3p_reload_f32", 2, 1_500_000, TOL_3P),   # five launches
             ("softmax2p_f32", 300, 5000, TOL_2P),             # rows path
             ("softmax2p_onchip_f32", 300, 5000, TOL_2P)]
    for name, rows, n, tol in cases:
        fn = getattr(gpu, name)
        x = torch.empty(rows * n, dtype=torch.float32, device="cuda")
        y = torch.full_like(x, -7.0)
        want = torch.empty_like(x)
        gpu.softmax_tp_reserve(rows, n, 4, stream=side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            fn(x, y, rows, n)                                  # launched on the capturing stream
        for trial in range(3):
            host = workloads.cfg3(rows=rows, n=n) + np.float32(trial)
            x.copy_(torch.from_numpy(host.reshape(-1)))
            y.fill_(-7.0)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            fn(x, want, rows, n)                               # eager, default stream
            torch.cuda.synchronize()
            assert torch.equal(y, want), (name, rows, n, trial)
            if trial == 2:
                _check(oracle_mod, host, y.cpu().numpy().reshape(rows, n), tol)
        del graph


def test_reserve_covers_incongruent_pointers_and_pass_level_calls(gpu, oracle_mod):
    """x and y one element apart modulo 16 bytes: the element-wise kernels cut the storing pass
    into more chunks and need a larger workspace; the pass-level entry points use the chunk
    kernels for shapes whose full call needs no workspace.  One reserve must cover all of it,
    or the call would allocate under capture and the capture would fail."""
    import torch
    side = torch.cuda.Stream()
    rows, n = 1000, 100_000
    # beyond the smallest buffer the library ever allocates (64 KiB), and only when incongruent
    assert (gpu.softmax_tp_plan(rows, n, 4, False).workspace_bytes > 65536
            > gpu.softmax_tp_plan(rows, n, 4, True).workspace_bytes)
    host = workloads.cfg2(rows=rows, n=n)
    xbuf = torch.empty(rows * n + 8, dtype=torch.float32, device="cuda")
    ybuf = torch.full((rows * n + 8,), -7.0, dtype=torch.float32, device="cuda")
    x, y = xbuf[1:1 + rows * n], ybuf[2:2 + rows * n]
    x.copy_(torch.from_numpy(host.reshape(-1)))
    gpu.softmax_tp_release()
    gpu.softmax_tp_reserve(rows, n, 4, stream=side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        gpu.softmax3p_reload_f32(x, y, rows, n)
    graph.replay()
    torch.cuda.synchronize()
    _check(oracle_mod, host, y.cpu().numpy().reshape(rows, n), TOL_3P)
    del graph
    # a rows-path shape through the pass-level entry point
    rows, n = 300, 5000
    assert gpu.softmax_tp_plan(rows, n).path == 1
    host = workloads.cfg2(rows=rows, n=n)
    x = torch.from_numpy(host.reshape(-1)).cuda()
    y = torch.empty_like(x)
    pairs = torch.empty(2 * rows, dtype=torch.float32, device="cuda")
    gpu.softmax_tp_release()
    gpu.softmax_tp_reserve(rows, n, 4, stream=side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        gpu.softmax2p_f32_pass1(x, pairs, rows, n)
        gpu.softmax2p_f32_pass2(x, pairs, y, rows, n)
    graph.replay()
    torch.cuda.synchronize()
    _check(oracle_mod, host, y.cpu().numpy().reshape(rows, n), TOL_2P)
    del graph


def test_calibration_streams(gpu):
    import torch
    n = (1 << 22) + 5
    x = torch.arange(n, dtype=torch.float32, device="cuda") % 7
    y = torch.empty_like(x)
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    gpu.softmax_tp_stream_copy_f32(x, y, n)
    assert torch.equal(x, y)
    gpu.softmax_tp_stream_scale_f32(x, y, 2.5, n)
    assert torch.equal(x * 2.5, y)
    for off in (0, 1, 3):                               # 16-byte aligned or not: nothing outside is touched
        buf = torch.full((n + 8,), -7.0, dtype=torch.float32, device="cuda")
        gpu.softmax_tp_stream_fill_f32(buf[off:off + n], 1.25, n)
        assert bool((buf[off:off + n] == 1.25).all()) and bool((buf[:off] == -7).all()) \
            and bool((buf[off + n:] == -7).all())
    gpu.softmax_tp_stream_read_f32(x, sink, n)
    assert abs(float(sink[0]) - float(x.double().sum())) <= 1e-6 * float(x.double().sum())
