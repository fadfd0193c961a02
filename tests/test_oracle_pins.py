"""Pins for the long-double oracle: everything here runs on the CPU.

The oracle is checked against what the paper and the mathematics fix, never
against itself: closed forms, the unshifted definition evaluated by an
independent arbitrary-precision library (mpmath), invariants from Section 1,
the shift identity of Section 3, a float64 library softmax, and the fp32
thresholds the paper prints (tests/golden/paper_constants.json).  The same pin
suite is then run on deliberately wrong softmaxes to show each mistake is caught.
"""
import json
import math
import os

import mpmath
import numpy as np
import pytest
import scipy.special

from paper_2001_04438_amd import workloads

GOLDEN = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_constants.json")))

mpmath.mp.prec = 200
LD_EPS = float(np.finfo(np.longdouble).eps)  # 2^-63 on x86-64


def mp_softmax(row):
    """The literal, unshifted formula of Section 1 in 200-bit arithmetic."""
    e = [mpmath.exp(mpmath.mpf(float(v))) for v in row]
    s = mpmath.fsum(e)
    return [v / s for v in e]


def _ld_to_mp(v):
    """Exact conversion of a numpy longdouble to mpf (significand split into two doubles)."""
    frac, exp = np.frexp(np.longdouble(v))
    hi = np.float64(frac)
    lo = np.float64(frac - np.longdouble(hi))
    return mpmath.ldexp(mpmath.mpf(float(hi)) + mpmath.mpf(float(lo)), int(exp))


# --------------------------------------------------------------------------
# the pin suite, written against an arbitrary row-wise softmax callable
# --------------------------------------------------------------------------

def pin_closed_forms(sm):
    # all-equal row -> exactly 1/N
    for N in (1, 2, 7, 64, 1000):
        p = sm(np.full((1, N), 3.25, dtype=np.float32))[0]
        assert np.all(np.abs(np.asarray(p, dtype=np.float64) * N - 1.0) < 1e-15)
    # N = 2 -> logistic function
    for a, b in ((0.0, 0.0), (1.5, -2.25), (-30.0, 40.0), (88.0, -88.0)):
        p = sm(np.array([[a, b]], dtype=np.float32))[0]
        want = 1 / (1 + mpmath.exp(mpmath.mpf(b) - mpmath.mpf(a)))
        assert abs(_ld_to_mp(p[0]) - want) / want < 1e-17
        want1 = 1 / (1 + mpmath.exp(mpmath.mpf(a) - mpmath.mpf(b)))
        assert abs(_ld_to_mp(p[1]) - want1) / want1 < 1e-17
    # arithmetic progression -> geometric series p_i = r^i (1 - r) / (1 - r^N)
    a, d, N = -3.0, 0.375, 40
    x = (a + d * np.arange(N)).astype(np.float32)  # exact in fp32
    p = sm(x.reshape(1, N))[0]
    r = mpmath.exp(mpmath.mpf(d))
    for i in (0, 1, 17, N - 1):
        want = r ** i * (1 - r) / (1 - r ** N)
        assert abs(_ld_to_mp(p[i]) - want) / want < 1e-17


def pin_bruteforce(sm):
    rng = np.random.default_rng(11)
    rows = [
        rng.uniform(-10, 10, 9),
        rng.normal(0, 30, 16),
        np.array([1e4, -1e4, 9990.5, 3.0]),       # the config-1 probes: 80-bit exp would still cope,
        np.array([-1e4, -1.0001e4, -9999.25]),    # fp32/fp64 exp would not
        np.array([700.0, 710.0, 0.0, -745.0]),
        np.array([0.0]),
    ]
    for row in rows:
        row32 = row.astype(np.float32)
        p = sm(row32.reshape(1, -1))[0]
        want = mp_softmax(row32)
        for a, b in zip(p, want):
            a = _ld_to_mp(a)
            if b < mpmath.mpf(2) ** -16000:
                assert a == 0 or abs(a - b) / b < 1e-15
            else:
                assert abs(a - b) / b < 2e-17, (row, float(a), float(b))


def pin_invariants(sm):
    for x in (workloads.cfg1(), workloads.cfg1(probes=True), workloads.cfg2(rows=3, n=1111),
              workloads.cfg3(rows=2, n=5000), workloads.cfg4(n=20000)):
        p = sm(x)
        assert p.shape == x.shape
        assert np.all(p >= 0)
        assert np.all(np.isfinite(p.astype(np.float64)))
        s = p.sum(axis=1, dtype=np.longdouble)
        assert np.all(np.abs(s - 1) <= x.shape[1] * LD_EPS)
        # order preservation, row by row
        for r in range(x.shape[0]):
            order = np.argsort(x[r], kind="stable")
            assert np.all(np.diff(p[r][order]) >= 0)


def pin_shift_invariance(sm):
    rng = np.random.default_rng(5)
    x = (rng.integers(-4000, 4000, size=(3, 257)) / 256.0).astype(np.float32)  # multiples of 2^-8
    p0 = sm(x)
    for c in (1.0, -17.0, 1000.0, 16384.0, -30000.0):
        xc = (x + np.float32(c)).astype(np.float32)
        assert np.array_equal(xc.astype(np.float64), x.astype(np.float64) + c)  # shift is exact
        pc = sm(xc)
        denom = np.maximum(p0, np.longdouble(1e-300))
        assert np.max(np.abs(pc - p0) / denom) < 64 * LD_EPS


def pin_ratio_and_permutation(sm):
    rng = np.random.default_rng(8)
    x = rng.normal(0, 5, size=(1, 50)).astype(np.float32)
    p = sm(x)[0]
    for i, j in ((0, 1), (3, 40), (49, 7)):
        want = mpmath.exp(mpmath.mpf(float(x[0, i])) - mpmath.mpf(float(x[0, j])))
        got = _ld_to_mp(p[i]) / _ld_to_mp(p[j])
        assert abs(got - want) / want < 1e-17
    perm = rng.permutation(50)
    pp = sm(x[:, perm])[0]
    assert np.max(np.abs(pp - p[perm]) / p[perm]) < 64 * LD_EPS


def pin_rows_are_independent(sm):
    rng = np.random.default_rng(9)
    x = rng.normal(0, 3, size=(5, 33)).astype(np.float32)
    p = sm(x)
    for r in range(5):
        pr = sm(x[r:r + 1])[0]
        assert np.array_equal(p[r], pr)
    # and a library softmax in float64 agrees along the last axis
    lib = scipy.special.softmax(x.astype(np.float64), axis=1)
    assert np.max(np.abs(p.astype(np.float64) - lib) / lib) < 1e-13


def pin_overflow_probe(sm):
    x = workloads.cfg1(probes=True)
    p = sm(x)[0]
    assert np.all(np.isfinite(p.astype(np.float64)))
    assert abs(float(p[0]) - 1.0) < 1e-15          # e^(1e4) dwarfs everything else
    assert float(p[1]) == 0.0 and float(p[2:].max()) < 1e-300


PINS = [pin_closed_forms, pin_bruteforce, pin_invariants, pin_shift_invariance,
        pin_ratio_and_permutation, pin_rows_are_independent, pin_overflow_probe]


# --------------------------------------------------------------------------
# the oracle passes every pin
# --------------------------------------------------------------------------

@pytest.mark.parametrize("pin", PINS, ids=lambda f: f.__name__)
def test_oracle_pins(oracle_mod, pin):
    pin(lambda x: oracle_mod.softmax(x))


@pytest.mark.parametrize("pin", PINS, ids=lambda f: f.__name__)
def test_oracle_pins_single_thread(oracle_mod, pin):
    pin(lambda x: oracle_mod.softmax(x, threads=1))


# --------------------------------------------------------------------------
# planted mistakes (on the CPU, in numpy long double): each must fail a pin
# --------------------------------------------------------------------------

def _ld(x):
    return np.asarray(x, dtype=np.float32).astype(np.longdouble)


def mutant_wrong_sign(x):
    x = _ld(x)
    e = np.exp(x.max(axis=1, keepdims=True) - x)
    return e / e.sum(axis=1, keepdims=True)


def mutant_no_shift(x):  # naive formula: overflows on the probes
    e = np.exp(_ld(x).astype(np.float64)).astype(np.longdouble)
    with np.errstate(invalid="ignore", over="ignore"):
        return e / e.sum(axis=1, keepdims=True)


def mutant_wrong_axis(x):
    x = _ld(x)
    e = np.exp(x - x.max())
    return e / e.sum()


def mutant_dropped_term(x):  # sum skips the last element
    x = _ld(x)
    e = np.exp(x - x.max(axis=1, keepdims=True))
    return e / np.maximum(e[:, :-1].sum(axis=1, keepdims=True), np.longdouble(1e-4000))


def mutant_base_two(x):
    x = _ld(x)
    e = np.exp2(x - x.max(axis=1, keepdims=True))
    return e / e.sum(axis=1, keepdims=True)


def mutant_double_precision(x):  # right formula, float64 arithmetic: too coarse for the pins
    x = np.asarray(x, dtype=np.float64)
    e = np.exp(x - x.max(axis=1, keepdims=True))
    return (e / e.sum(axis=1, keepdims=True)).astype(np.longdouble)


def mutant_min_instead_of_max(x):
    x = _ld(x)
    with np.errstate(over="ignore", invalid="ignore"):
        e = np.exp(x - x.min(axis=1, keepdims=True))
        return e / e.sum(axis=1, keepdims=True)


@pytest.mark.parametrize("mutant", [mutant_wrong_sign, mutant_no_shift, mutant_wrong_axis,
                                    mutant_dropped_term, mutant_base_two, mutant_double_precision,
                                    mutant_min_instead_of_max], ids=lambda f: f.__name__)
@pytest.mark.filterwarnings("ignore::RuntimeWarning")
def test_pins_catch_planted_mistakes(mutant):
    failed = []
    for pin in PINS:
        try:
            pin(mutant)
        except (AssertionError, FloatingPointError, ZeroDivisionError):
            failed.append(pin.__name__)
    assert failed, f"{mutant.__name__} slipped through every pin"


# --------------------------------------------------------------------------
# mu, S, threading, bf16 decoding
# --------------------------------------------------------------------------

def test_stats_against_mpmath(oracle_mod):
    rng = np.random.default_rng(21)
    x = rng.normal(0, 20, size=(2, 300)).astype(np.float32)
    mu, S = oracle_mod.stats(x)
    for r in range(2):
        assert float(mu[r]) == float(x[r].max())
        want = mpmath.fsum(mpmath.exp(mpmath.mpf(float(v)) - mpmath.mpf(float(x[r].max())))
                           for v in x[r])
        assert abs(_ld_to_mp(S[r]) - want) / want < 300 * 2.0 ** -64


def test_thread_split_changes_nothing_material(oracle_mod):
    x = workloads.cfg4(n=300_001)
    mu1, S1 = oracle_mod.stats(x, threads=1)
    for t in (2, 3, 8):
        mu, S = oracle_mod.stats(x, threads=t)
        assert mu[0] == mu1[0]
        assert abs(S[0] - S1[0]) / S1[0] < 300_001 * LD_EPS
    p1 = oracle_mod.softmax(x, threads=1)
    p8 = oracle_mod.softmax(x, threads=8)
    nz = p1 > 0
    assert np.array_equal(nz, p8 > 0)
    assert np.max(np.abs(p8[nz] - p1[nz]) / p1[nz]) < 1e-15
    lse = oracle_mod.logsumexp(x)
    assert abs(lse - (mu1[0] + np.log(S1[0]))) < 1e-12   # returned through a C double


def test_bf16_bit_patterns(oracle_mod):
    # sign | 8 exponent bits | 7 fraction bits: the top half of a binary32
    bits = np.array([[0x3F80, 0xC000, 0x0000, 0x4049, 0x7F7F, 0xFF7F]], dtype=np.uint16)
    vals = workloads.bf16_bits_to_f32(bits)
    assert vals[0, 0] == 1.0 and vals[0, 1] == -2.0 and vals[0, 2] == 0.0
    assert vals[0, 3] == 3.140625
    assert vals[0, 4] == np.float32((2 - 2.0 ** -7) * 2.0 ** 127)
    p_bits = oracle_mod.softmax(bits[:, :4], bf16=True)
    p_vals = oracle_mod.softmax(vals[:, :4])
    assert np.array_equal(p_bits, p_vals)
    # round-to-nearest-even on the way in
    f = np.array([1.0, 1.00390625, 1.01171875, 1.0 + 2.0 ** -8 + 2.0 ** -20], dtype=np.float32)
    assert list(workloads.f32_to_bf16_bits(f)) == [0x3F80, 0x3F80, 0x3F82, 0x3F81]
    x5 = workloads.cfg5(rows=2, n=777)
    p5 = oracle_mod.softmax(x5, bf16=True)
    assert np.array_equal(p5, oracle_mod.softmax(workloads.bf16_bits_to_f32(x5)))


def test_f16_decoding_exhaustive(oracle_mod):
    # IEEE binary16: sign | 5 exponent bits (bias 15) | 10 fraction bits.  Values written out by hand
    bits = np.array([0x3C00, 0xC000, 0x0000, 0x7BFF, 0x0001, 0x03FF, 0x0400, 0x3555, 0xFBFF],
                    dtype=np.uint16)
    want = [1.0, -2.0, 0.0, 65504.0, 2.0 ** -24, 1023 * 2.0 ** -24, 2.0 ** -14,
            (1024 + 0x155) * 2.0 ** -12, -65504.0]
    mu, S = oracle_mod.stats(bits.reshape(-1, 1), f16=True)   # a row of one element: mu is the element
    assert [float(v) for v in mu] == want and np.all(S == 1)
    # every finite pattern against numpy's half type (an independent implementation of the format)
    allbits = np.arange(1 << 16, dtype=np.uint16)
    finite = allbits[(allbits & 0x7C00) != 0x7C00]
    mu, _ = oracle_mod.stats(finite.reshape(-1, 1), f16=True)
    assert np.array_equal(mu.astype(np.float64), finite.view(np.float16).astype(np.float64))
    assert finite.size == 2 * 31 * 1024
    # the generators' rounding on the way in: nearest even at 11 significand bits
    f = np.array([1.0, 1 + 2.0 ** -11, 1 + 3 * 2.0 ** -11, 1 + 2.0 ** -11 + 2.0 ** -20, 65519.0, 3e-8],
                 dtype=np.float32)
    assert list(workloads.f32_to_f16_bits(f)) == [0x3C00, 0x3C00, 0x3C02, 0x3C01, 0x7BFF, 0x0001]
    assert np.array_equal(workloads.f16_bits_to_f32(bits), np.array(want, dtype=np.float32))
    # a softmax over fp16 bit patterns is the softmax of the values they denote
    x = workloads.f32_to_f16_bits(np.random.default_rng(5).normal(0, 3, (2, 777)).astype(np.float32))
    assert np.array_equal(oracle_mod.softmax(x, f16=True),
                          oracle_mod.softmax(workloads.f16_bits_to_f32(x)))


# --------------------------------------------------------------------------
# fp32 thresholds printed in the paper (negative control for the probes)
# --------------------------------------------------------------------------

@pytest.mark.filterwarnings("ignore::RuntimeWarning")
def test_paper_fp32_exp_thresholds():
    hi = GOLDEN["exp_f32_overflow_above"]["value"]
    lo = GOLDEN["exp_f32_underflow_below"]["value"]
    with np.errstate(over="ignore", under="ignore"):
        assert np.isinf(np.float32(np.exp(np.float64(hi))))          # e^89 > FLT_MAX
        assert np.isfinite(np.float32(np.exp(np.float64(hi - 1))))
        assert np.float32(np.exp(np.float64(lo))) == 0               # e^-104 rounds to zero
        assert np.float32(np.exp(np.float64(lo + 1))) > 0
        # naive fp32 softmax on the probes gives NaN; the oracle does not
        x = workloads.cfg1(probes=True)[0]
        e = np.exp(x.astype(np.float32))
        naive = e / e.sum(dtype=np.float32)
    assert np.isnan(naive).any()


def test_table2_byte_model():
    t = GOLDEN["table2_bytes_per_element_units_of_N"]
    for k in ("three_pass_recompute", "three_pass_reload", "two_pass"):
        assert t[k]["reads"] + t[k]["writes"] == t[k]["cost"]
    adv = GOLDEN["bandwidth_advantage_percent"]
    assert round(100 * (t["three_pass_recompute"]["cost"] / t["two_pass"]["cost"] - 1)) == adv["vs_recompute"]
    assert round(100 * (t["three_pass_reload"]["cost"] / t["two_pass"]["cost"] - 1)) == adv["vs_reload"]


# --------------------------------------------------------------------------
# the comparator
# --------------------------------------------------------------------------

def test_comparator_accepts_correct_and_flags_wrong(oracle_mod):
    x = workloads.cfg3(rows=3, n=4099)
    p = oracle_mod.softmax(x)
    y = p.astype(np.float32)
    c = oracle_mod.compare(x, y, 4e-6)
    assert c.ok() and c.n_total == x.size
    assert c.max_rel_err <= 2.0 ** -24 * 1.0001
    assert c.max_row_sum_dev < 4099 * 2.0 ** -24
    # a 1e-5 relative error on one element is reported, at the right place
    y2 = y.copy()
    k = int(np.argmax(p[1]))
    y2[1, k] *= np.float32(1 + 1e-5)
    c2 = oracle_mod.compare(x, y2, 4e-6)
    assert c2.n_rel_viol == 1 and c2.worst_index == 4099 + k
    assert abs(c2.max_rel_err - 1e-5) < 2e-7
    # NaN, Inf and negative outputs are counted
    y3 = y.copy()
    y3[0, 0] = np.nan
    y3[0, 1] = np.inf
    y3[2, 5] = -abs(y3[2, 5]) - np.float32(1e-30)
    c3 = oracle_mod.compare(x, y3, 4e-6)
    assert c3.n_nonfinite == 2 and c3.n_negative == 1 and not c3.ok()


def test_comparator_per_element_bound_for_three_pass(oracle_mod):
    """Optional mode: element i is held to tol + slope |x_i - mu| (the Three-Pass algorithms'
    fl32(x_i - mu) costs up to 2^-24 |x_i - mu| relative whatever the evaluator does).  Pinned on
    planted errors placed just inside and just outside the bound of an element far below the
    maximum, and on what the subtraction itself does to an otherwise exact result."""
    slope = oracle_mod.THREE_PASS_SLOPE
    assert slope == 2.0 ** -24
    x = np.array([[0.0, -3.0, -40.0, -80.0, -86.5]], dtype=np.float32)
    p = oracle_mod.softmax(x)[0]
    assert p[4] > np.finfo(np.float32).tiny
    y = p.astype(np.float64)
    inside = y.copy()
    inside[3] *= 1 + 4e-6 + 0.5 * slope * 80.0          # within 4e-6 + 2^-24 * 80 = 8.77e-6
    outside = y.copy()
    outside[3] *= 1 + 4e-6 + 1.5 * slope * 80.0
    f = lambda v: v.astype(np.float32).reshape(1, -1)
    assert 4e-6 + slope * 80.0 == pytest.approx(8.768e-6, rel=1e-3)
    c_in = oracle_mod.compare(x, f(inside), 4e-6, slope=slope)
    assert c_in.ok() and 0.6 < c_in.max_bound_ratio < 1.0
    assert oracle_mod.compare(x, f(inside), 4e-6).n_rel_viol == 1           # flat rule: too far
    c_out = oracle_mod.compare(x, f(outside), 4e-6, slope=slope)
    assert c_out.n_rel_viol == 1 and c_out.worst_index == 3 and c_out.max_bound_ratio > 1.0
    # the allowance scales with |x_i - mu|: the same relative error next to the maximum is refused
    near = y.copy()
    near[1] *= 1 + 4e-6 + 0.5 * slope * 80.0
    assert oracle_mod.compare(x, f(near), 4e-6, slope=slope).n_rel_viol == 1
    # where the allowance comes from: exp of the ROUNDED difference, otherwise exact
    rng = np.random.default_rng(24)
    xs = rng.uniform(-86, 0, (1, 4000)).astype(np.float32)
    xs[0, 0] = np.float32(0.3337)        # the maximum: fine-grained, so x - mu needs more than 24 bits
    mu = xs.max()
    d32 = (xs - mu).astype(np.float32)                                       # one fp32 rounding
    e = np.exp(d32.astype(np.longdouble))
    y3 = (e / e.sum()).astype(np.float32)
    c = oracle_mod.compare(xs, y3, 4e-6, slope=slope)
    assert c.ok() and c.max_bound_ratio < 1.0
    assert c.max_rel_err > 1e-6          # the subtraction alone costs more than the 2 ULP of Exp
    assert c.max_rel_err <= 2.0 ** -24 * 86 + 2.0 ** -23


def test_comparator_subnormal_rule(oracle_mod):
    # p of the small entries lies below FLT_MIN: 0 or the denormal both pass, garbage does not
    x = np.array([[0.0, -88.0, -95.0, -120.0]], dtype=np.float32)
    p = oracle_mod.softmax(x)[0]
    assert p[1] < np.finfo(np.float32).tiny and p[2] > 0
    y_den = p.astype(np.float32).reshape(1, -1)
    y_ftz = y_den.copy()
    y_ftz[0, 1:] = 0
    assert oracle_mod.compare(x, y_den, 4e-6).ok()
    assert oracle_mod.compare(x, y_ftz, 4e-6).ok()
    y_bad = y_ftz.copy()
    y_bad[0, 3] = np.float32(1e-30)
    assert oracle_mod.compare(x, y_bad, 4e-6).n_sub_viol == 1


def test_comparator_bf16(oracle_mod):
    x = workloads.cfg5(rows=4, n=1001)
    p = oracle_mod.softmax(x, bf16=True)
    y = workloads.f32_to_bf16_bits(p.astype(np.float32))
    c = oracle_mod.compare(x, y, 1e-2, bf16=True)
    assert c.ok()
    assert 0 < c.max_rel_err <= 2.0 ** -8 * 1.0001   # bf16 rounding alone is up to 2^-9 relative... of the ulp
    # single-row, many threads path gives the same verdict as one thread
    c1 = oracle_mod.compare(x[:1], y[:1], 1e-2, bf16=True, threads=1)
    c8 = oracle_mod.compare(x[:1], y[:1], 1e-2, bf16=True, threads=8)
    assert c1.max_rel_err == c8.max_rel_err and c1.n_total == c8.n_total == 1001
    assert abs(c1.max_row_sum_dev - c8.max_row_sum_dev) < 1e-15


def test_comparator_f16(oracle_mod):
    rng = np.random.default_rng(16)
    x = workloads.f32_to_f16_bits(rng.normal(0, 2, (4, 1001)).astype(np.float32))
    p = oracle_mod.softmax(x, f16=True)
    y = workloads.f32_to_f16_bits(p.astype(np.float32))
    c = oracle_mod.compare(x, y, 5e-4, f16=True)
    assert c.ok() and c.n_total == x.size
    assert 2.0 ** -13 < c.max_rel_err <= 2.0 ** -11 * 1.0001        # one rounding to 11 bits
    assert 0 < c.n_normal < c.n_total                                # some results are fp16 subnormals
    assert c.max_sub_abs_err <= 2.0 ** -25 * 1.0001
    # two ulps off on a normal result is a violation at 5e-4
    k = int(np.argmax(p[2]))
    y2 = y.copy()
    y2[2, k] += 2
    c2 = oracle_mod.compare(x, y2, 5e-4, f16=True)
    assert c2.n_rel_viol == 1 and c2.worst_index == 2 * 1001 + k
    # the flush-to-zero allowance starts at the format's own smallest normal, 2^-14, not at fp32's
    for a, normal in ((9.625, True), (9.75, False)):
        xa = workloads.f32_to_f16_bits(np.array([[0.0, -a]], dtype=np.float32))
        pa = oracle_mod.softmax(xa, f16=True)[0]
        assert (pa[1] >= 2.0 ** -14) == normal
        y0 = np.array([[0x3C00, 0x0000]], dtype=np.uint16)           # [1.0, flushed to zero]
        ca = oracle_mod.compare(xa, y0, 5e-4, f16=True)
        assert (ca.n_rel_viol == 1) == normal and ca.n_sub_viol == 0
    # infinities and NaNs of the format are counted
    y3 = y.copy()
    y3[0, 0] = 0x7C00
    y3[0, 1] = 0x7E00
    y3[1, 0] |= 0x8000
    c3 = oracle_mod.compare(x, y3, 5e-4, f16=True)
    assert c3.n_nonfinite == 2 and c3.n_negative == 1


# --------------------------------------------------------------------------
# the oracle's C code under the address and undefined-behaviour sanitizers
# --------------------------------------------------------------------------

def test_oracle_under_sanitizers(tmp_path):
    import subprocess
    import sys
    here = os.path.dirname(os.path.abspath(__file__))
    root = os.path.dirname(here)
    lib = tmp_path / "liboracle_san.so"
    srcs = [os.path.join(root, "oracle", f) for f in ("softmax_oracle.c", "twopass_model.c")]
    subprocess.run(["gcc", "-std=c11", "-O1", "-g", "-fPIC", "-shared", "-fno-fast-math",
                    "-ffp-contract=off", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                    "-o", str(lib), *srcs, "-lm", "-lpthread"], check=True)
    script = f"""
import ctypes, numpy as np
L = ctypes.CDLL({str(lib)!r})
vp, i64 = ctypes.c_void_p, ctypes.c_int64
rng = np.random.default_rng(0)
for rows, n, threads in ((1, 1, 1), (3, 17, 2), (2, 4099, 8), (1, 100003, 5), (7, 33, 16)):
    x = rng.normal(0, 30, size=(rows, n)).astype(np.float32)
    p = np.zeros((rows, n), dtype=np.longdouble)
    L.oracle_softmax_f32(x.ctypes.data_as(vp), i64(rows), i64(n), p.ctypes.data_as(vp), threads)
    assert abs(float(p.sum()) - rows) < 1e-9
    y = p.astype(np.float32)
    buf = (ctypes.c_char * 256)()
    L.oracle_compare_f32(x.ctypes.data_as(vp), y.ctypes.data_as(vp), i64(rows), i64(n),
                         ctypes.c_double(4e-6), buf, threads)
    h = (x.view(np.uint32) >> 16).astype(np.uint16)
    L.oracle_softmax_bf16(h.ctypes.data_as(vp), i64(rows), i64(n), p.ctypes.data_as(vp), threads)
    assert abs(float(p.sum()) - rows) < 1e-9
    g = x.astype(np.float16).view(np.uint16)
    L.oracle_softmax_f16(g.ctypes.data_as(vp), i64(rows), i64(n), p.ctypes.data_as(vp), threads)
    assert abs(float(p.sum()) - rows) < 1e-9
    L.oracle_compare_f16(g.ctypes.data_as(vp), g.ctypes.data_as(vp), i64(rows), i64(n),
                         ctypes.c_double(5e-4), buf, threads)
d = np.linspace(-50, 50, 1001)
yd = np.zeros_like(d)
L.model_twopass(d.ctypes.data_as(vp), yd.ctypes.data_as(vp), i64(d.size))
assert abs(yd.sum() - 1) < 1e-12
print("sanitized run ok")
"""
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    preload = asan + (":" + os.environ["LD_PRELOAD"] if os.environ.get("LD_PRELOAD") else "")
    env = dict(os.environ, LD_PRELOAD=preload, ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0")
    res = subprocess.run([sys.executable, "-c", script], env=env, capture_output=True, text=True)
    assert res.returncode == 0 and "sanitized run ok" in res.stdout, res.stderr[-2000:]
