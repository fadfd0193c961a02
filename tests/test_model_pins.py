"""Pins for the double-precision scalar model of Algorithms 1-3 (CPU only).

The model states the (m, n) pair algebra of Section 4 (make a pair, add two pairs) and
builds the row sum and the outputs from those two operations alone; these tests show
that the algebra reproduces the softmax definition (the oracle, itself pinned in
test_oracle_pins.py), that pair addition is order-independent, and that nothing
overflows where a plain exp would.
"""
import json
import math
import os

import numpy as np
import pytest

from paper_2001_04438_amd import workloads

GOLDEN = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_constants.json")))


def test_extexp_ranges(oracle_mod):
    # Section 4: m = e^t in [sqrt(2)/2, sqrt(2)], n an integer, e^x = m 2^n
    assert GOLDEN["reduced_exp_range"]["lo"] == "sqrt(2)/2"
    rng = np.random.default_rng(1)
    for x in list(rng.uniform(-2000, 2000, 500)) + [0.0, 1e4, -1e4, 88.7, -103.9]:
        m, n = oracle_mod.model_extexp(x)
        assert n == round(n)
        assert math.sqrt(2) / 2 * (1 - 1e-12) <= m <= math.sqrt(2) * (1 + 1e-12)
        if abs(x) < 700:
            assert abs(m * 2.0 ** n / math.exp(x) - 1) < 1e-13
    # with the reconstruction removed nothing overflows where e^x itself would
    m, n = oracle_mod.model_extexp(1e4)
    assert math.isfinite(m) and n == 14427.0


def test_model_twopass_equals_definition(oracle_mod):
    for x in (workloads.cfg1()[0], workloads.cfg1(probes=True)[0], workloads.cfg4(n=30000)[0],
              workloads.cfg3(rows=1, n=10000)[0], np.array([5.0], dtype=np.float32)):
        p = oracle_mod.softmax(x.reshape(1, -1))[0].astype(np.float64)
        y = oracle_mod.model_twopass(x)
        nz = p > 1e-290
        assert np.max(np.abs(y[nz] - p[nz]) / p[nz]) < 1e-11
        assert np.all(y[~nz] < 1e-289)
        assert np.all(np.isfinite(y))


def test_model_threepass_equals_definition(oracle_mod):
    x = workloads.cfg3(rows=1, n=8000)[0]
    p = oracle_mod.softmax(x.reshape(1, -1))[0].astype(np.float64)
    for fn in (oracle_mod.model_threepass_recompute, oracle_mod.model_threepass_reload):
        y = fn(x)
        nz = p > 1e-290
        assert np.max(np.abs(y[nz] - p[nz]) / p[nz]) < 1e-11


def test_pass1_pair_is_logsumexp(oracle_mod):
    # ln(m_sum) + n_sum ln 2 must equal mu + ln S of the definition
    for x in (workloads.cfg1(probes=True)[0], workloads.cfg4(n=50000)[0], workloads.cfg2(rows=1, n=3000)[0]):
        m, n = oracle_mod.model_pass1(x)
        assert n == round(n) and m >= math.sqrt(2) / 2 * (1 - 1e-12)
        lse = float(oracle_mod.logsumexp(x))
        assert abs(math.log(m) + n * math.log(2) - lse) < 1e-9 * max(1.0, abs(lse))
    # n_sum is the largest exponent seen: for the probes that is round(1e4 log2 e)
    m, n = oracle_mod.model_pass1(workloads.cfg1(probes=True)[0])
    assert n == 14427.0


def test_pair_addition_any_order(oracle_mod):
    rng = np.random.default_rng(3)
    x = np.concatenate([rng.normal(0, 40, 200), [900.0, -900.0]])
    pairs = [oracle_mod.model_extexp(v) for v in x]
    seq = (0.0, -math.inf)
    for pr in pairs:
        seq = oracle_mod.model_pair_add(seq, pr)
    for trial in range(5):
        work = [pairs[i] for i in rng.permutation(len(pairs))]
        while len(work) > 1:  # random binary tree
            i = int(rng.integers(0, len(work) - 1))
            merged = oracle_mod.model_pair_add(work[i], work[i + 1])
            work[i:i + 2] = [merged]
        m, n = work[0]
        assert n == seq[1]
        assert abs(m - seq[0]) / seq[0] < 1e-13
    # the identity element leaves a pair unchanged, from either side
    a = oracle_mod.model_extexp(2.5)
    assert oracle_mod.model_pair_add((0.0, -math.inf), a) == a
    assert oracle_mod.model_pair_add(a, (0.0, -math.inf)) == a


def test_pair_rel_err_helper(oracle_mod):
    xs = np.array([0.0, 1.0, -50.0, 1e4, -1e4, 88.0], dtype=np.float32)
    ms, ns = zip(*(oracle_mod.model_extexp(float(v)) for v in xs))
    rel, worst = oracle_mod.pair_rel_err(xs, np.array(ms), np.array(ns))
    assert worst < 2.0 ** -23          # only the fp32 rounding of m is left
    bad = np.array(ms, dtype=np.float32) * np.float32(1.001)
    _, worst_bad = oracle_mod.pair_rel_err(xs, bad, np.array(ns))
    assert 0.9e-3 < worst_bad < 1.1e-3
