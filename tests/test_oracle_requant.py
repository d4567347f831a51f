"""Pins for the oracle's requantize rule: int32 -> (fp32) * scale -> round half to
even -> ReLU -> clamp -> int8."""
import os
from fractions import Fraction

import numpy as np

import oracle
from paper_2101_08458_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_requant_fixture_table():
    n = 0
    for line in open(os.path.join(GOLDEN, "requant_rule.txt")):
        if not line.strip() or line.startswith("#"):
            continue
        t, scale, relu, exp = line.split()
        assert oracle.requant_one(int(t), float(scale), int(relu)) == int(exp), line
        n += 1
    assert n >= 20


def exact_rule(t, scale32, relu):
    """The rule in exact arithmetic: RNE int->fp32, one RNE fp32 product, half-even
    rounding -- each rounding done by an independent mechanism (float64 -> float32
    narrowing of an exactly representable value; Python's round on an exact Fraction)."""
    f = np.float32(np.float64(t))                       # |t| < 2^53: exact in double, one RNE narrowing
    prod = Fraction(float(f)) * Fraction(float(scale32))
    g = np.float32(float(prod))                         # 24x24-bit product is exact in double
    i = round(Fraction(float(g)))                       # Fraction.__round__ is half-even
    if relu:
        i = max(i, 0)
    return min(max(i, -128), 127)


def test_requant_exhaustive_int16_range():
    scales = np.array([0.5, 0.0078125, 0.003, 1.0 / 49.0, 0.12345678, 1.5], np.float32)
    ts = np.arange(-2 ** 15, 2 ** 15, dtype=np.int32)
    for sc in scales:
        acc = ts.reshape(1, 1, -1).copy()
        for relu in (False, True):
            got = oracle.requant(acc, np.array([sc], np.float32), relu=relu).reshape(-1)
            exp = np.array([exact_rule(int(t), sc, relu) for t in ts[::7]])
            assert np.array_equal(got[::7].astype(np.int64), exp)
    # the ties (scale 0.5, odd t) over the whole clamp range, every one of them
    odd = np.arange(-255, 256, 2, dtype=np.int32).reshape(1, 1, -1)
    got = oracle.requant(odd, np.array([0.5], np.float32)).reshape(-1).astype(np.int64)
    exp = np.array([2 * round(Fraction(int(t), 4)) for t in odd.reshape(-1)])   # nearest even
    assert np.array_equal(got, np.clip(exp, -128, 127))


def test_requant_large_magnitudes_inexact_conversion():
    g = wl.rng(70)
    ts = np.concatenate([g.integers(-2 ** 31, 2 ** 31, size=4000),
                         2 ** 24 + np.arange(-8, 9), -(2 ** 24) + np.arange(-8, 9),
                         [2 ** 31 - 1, -2 ** 31, 75497472, -75497472]]).astype(np.int32)
    for sc in np.array([1e-6, 3.3e-7, 2.0 ** -20, 127.0 / 7.5e7], np.float32):
        got = oracle.requant(ts.reshape(1, 1, -1).copy(), np.array([sc], np.float32)).reshape(-1)
        exp = np.array([exact_rule(int(t), sc, False) for t in ts])
        assert np.array_equal(got.astype(np.int64), exp)


def test_requant_bias_residual_per_channel():
    g = wl.rng(71)
    acc = g.integers(-50000, 50000, size=(2, 3, 4, 5)).astype(np.int32)
    res = g.integers(-50000, 50000, size=(2, 3, 4, 5)).astype(np.int32)
    bias = np.array([100, -2000, 7], np.int32)
    scale = np.array([0.001, 0.002, 0.0005], np.float32)
    got = oracle.requant(acc, scale, bias=bias, residual=res, relu=True)
    for n in range(2):
        for k in range(3):
            for p in range(4):
                for q in range(5):
                    t = int(acc[n, k, p, q]) + int(bias[k]) + int(res[n, k, p, q])
                    assert got[n, k, p, q] == exact_rule(t, scale[k], True)
    # bias only / residual only / neither reduce to the same rule
    assert np.array_equal(oracle.requant(acc, scale),
                          oracle.requant(acc, scale, bias=np.zeros(3, np.int32),
                                         residual=np.zeros_like(acc)))
