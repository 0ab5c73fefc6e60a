"""Pins for the oracle's sampler and uniform generator (CPU only)."""
import math
from fractions import Fraction

import numpy as np
import pytest

from oracle.sampler import (uniform_u32, sample_token, integer_weights, scale_constant,
                            EXP2_POLY)


def test_splitmix64_published_vector():
    # first outputs of SplitMix64 seeded with 1234567 (reference implementation's
    # test vector; see tests/golden/splitmix64.txt)
    with open(__file__.rsplit("/", 1)[0] + "/golden/splitmix64.txt") as f:
        vals = [int(l) for l in f if l.strip() and not l.startswith("#")]
    assert len(vals) == 5
    for k, v in enumerate(vals):
        assert uniform_u32(1234567, 0, k) == v >> 32
    # the trajectory id occupies the high half of the counter
    assert uniform_u32(99, 3, 5) != uniform_u32(99, 5, 3)
    draws = [uniform_u32(3, t, p) for t in range(64) for p in range(256)]
    assert len(set(draws)) > 0.999 * len(draws)
    assert abs(np.mean(draws) / 2**32 - 0.5) < 0.01


def test_exp2_polynomial_and_weights_track_softmax():
    assert float(EXP2_POLY[0]) == 1.0
    rng = np.random.default_rng(0)
    for T in (1.0, 0.7, 2.5):
        z = (rng.standard_normal(5000) * 3).astype(np.float32)
        w = integer_weights(z, T).astype(np.float64)
        p = np.exp((z.astype(np.float64) - z.max()) / T)
        # floor() to a multiple of 2^-32 plus the polynomial's ~1e-7 relative error
        assert np.all(np.abs(w / 2**32 - p) <= 2.0**-32 + 1e-6 * p)
        assert w[np.argmax(z)] == 2**32
    # far tail is cut to exactly zero weight
    z = np.array([0.0, -20.0, -30.0, -100.0], np.float32)
    w = integer_weights(z, 1.0)
    assert w[3] == 0 and w[1] > 0 and w[0] == 2**32


def test_inverse_cdf_against_exact_rationals():
    # tiny vocabulary: enumerate a grid of u32 and compare with brute force in exact
    # integer / rational arithmetic
    rng = np.random.default_rng(1)
    z = (rng.standard_normal(8) * 2).astype(np.float32)
    w = [int(x) for x in integer_weights(z, 1.0)]
    W = sum(w)
    grid = list(range(0, 2**32, 2**32 // 4096)) + [2**32 - 1, 1, 2**31]
    counts = np.zeros(8)
    for u in grid:
        tok, _ = sample_token(z, 1.0, u)
        r = Fraction(u * W, 2**32).__floor__()
        acc, ref = 0, None
        for k in range(8):
            acc += w[k]
            if acc > r:
                ref = k
                break
        assert tok == ref
        # equivalently: id is the bucket of u / 2^32 in the exact CDF
        lo = Fraction(sum(w[:tok]), W)
        hi = Fraction(sum(w[:tok + 1]), W)
        x = Fraction(r, W)
        assert lo <= x < hi
        counts[tok] += 1
    p = np.exp(z.astype(np.float64)); p /= p.sum()
    assert np.abs(counts / len(grid) - p).max() < 2e-3


def test_zero_weight_tokens_are_never_chosen_and_extremes():
    z = np.array([-200.0, 0.0, -200.0, 0.0], np.float32)
    assert sample_token(z, 1.0, 0)[0] == 1
    assert sample_token(z, 1.0, 2**31 - 1)[0] == 1
    assert sample_token(z, 1.0, 2**31)[0] == 3
    assert sample_token(z, 1.0, 2**32 - 1)[0] == 3


def test_logprobs_logsumexp_to_zero():
    rng = np.random.default_rng(2)
    V = 64
    z = (rng.standard_normal(V) * 2).astype(np.float32)
    for T in (1.0, 0.5):
        # force each id in turn through its own CDF bucket and collect its log-prob
        w = integer_weights(z, T).astype(object)
        W = int(sum(w))
        lps, acc = [], 0
        for k in range(V):
            u = -(-(acc << 32) // W)             # smallest u32 with floor(u*W/2^32) >= acc
            tok, lp = sample_token(z, T, u)
            assert tok == k
            lps.append(lp)
            acc += int(w[k])
        assert abs(math.log(sum(math.exp(x) for x in lps))) < 1e-9
        ref = z.astype(np.float64) / T
        ref = ref - (ref.max() + math.log(np.exp(ref - ref.max()).sum()))
        assert np.abs(np.array(lps) - ref).max() < 1e-12


def test_uniform_logits_closed_form():
    for V in (4096, 151936):
        z = np.zeros(V, np.float32)
        for u in (0, 1, 123456789, 2**32 - 1):
            tok, lp = sample_token(z, 1.0, u)
            assert tok == (u * V) >> 32
            assert abs(lp + math.log(V)) < 1e-12
    assert abs(-math.log(4096) + 8.3178) < 1e-4 and abs(-math.log(151936) + 11.9312) < 1e-4


def test_greedy_and_low_temperature_limit():
    rng = np.random.default_rng(3)
    z = rng.standard_normal(1000).astype(np.float32)
    z[[100, 900]] = 5.0                               # tie: lowest index wins
    tok, lp = sample_token(z, 0.0, 12345)
    assert tok == 100
    z64 = z.astype(np.float64)
    assert abs(lp - (5.0 - math.log(np.exp(z64).sum()))) < 1e-12
    z[100] = 5.5
    for u in (0, 2**31, 2**32 - 1):
        assert sample_token(z, 1e-3, u)[0] == 100     # T -> 0 picks the arg-max


def test_chi_square_frequencies():
    rng = np.random.default_rng(4)
    V = 16
    z = rng.standard_normal(V).astype(np.float32)
    p = np.exp(z.astype(np.float64)); p /= p.sum()
    n = 40000
    counts = np.zeros(V)
    for i in range(n):
        counts[sample_token(z, 1.0, uniform_u32(7, i // 200, i % 200))[0]] += 1
    chi2 = ((counts - n * p) ** 2 / (n * p)).sum()
    assert chi2 < 45.0          # 15 dof: P(chi2 > 45) < 1e-4


def test_scale_constant():
    assert scale_constant(1.0) == np.float32(1.4426950408889634)
    assert scale_constant(0.5) == np.float32(2.8853900817779268)
