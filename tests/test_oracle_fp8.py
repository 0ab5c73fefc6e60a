"""Pins of the E4M3 oracle: values the format's specification fixes, exhaustive round trips,
brute force against exact rational arithmetic, and torch's float8_e4m3fn cast (an independent
library implementation) inside the finite range."""
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle.fp8 import e4m3_decode, e4m3_encode, e4m3_round, E4M3_MAX


def test_values_fixed_by_the_specification():
    assert E4M3_MAX == 448.0
    assert e4m3_decode(0x00) == 0.0 and e4m3_decode(0x80) == 0.0
    assert e4m3_decode(0x01) == 2.0 ** -9                 # smallest subnormal
    assert e4m3_decode(0x07) == 7 * 2.0 ** -9             # largest subnormal
    assert e4m3_decode(0x08) == 2.0 ** -6                 # smallest normal
    assert e4m3_decode(0x38) == 1.0 and e4m3_decode(0x39) == 1.125 and e4m3_decode(0xB8) == -1.0
    assert e4m3_decode(0x7E) == 448.0 and e4m3_decode(0xFE) == -448.0
    assert np.isnan(e4m3_decode(0x7F)) and np.isnan(e4m3_decode(0xFF))
    vals = [e4m3_decode(c) for c in range(0x7F)]
    assert all(b > a for a, b in zip(vals, vals[1:]))


def test_every_code_survives_a_round_trip():
    for c in range(256):
        if c & 0x7F == 0x7F:
            continue
        v = e4m3_decode(c)
        got = int(e4m3_encode(np.array([v]))[0])
        assert got == c or (v == 0.0 and got & 0x7F == 0), hex(c)
    assert e4m3_encode(np.array([-0.0]))[0] == 0x80


def test_ties_go_to_the_even_code_and_large_values_saturate():
    enc = lambda v: int(e4m3_encode(np.array([v]))[0])
    assert enc(1.0625) == 0x38          # halfway 1.0 (even) / 1.125
    assert enc(1.1875) == 0x3A          # halfway 1.125 / 1.25 (even)
    assert enc(1.0625 + 1e-9) == 0x39 and enc(1.0625 - 1e-9) == 0x38
    assert enc(2.0 ** -10) == 0x00      # halfway 0 (even) / 2^-9
    assert enc(3 * 2.0 ** -10) == 0x02  # halfway 2^-9 / 2^-8 (even)
    assert enc(15 * 2.0 ** -10) == 0x08  # halfway largest subnormal / smallest normal (even)
    assert enc(-1.1875) == 0xBA
    assert enc(448.0) == 0x7E and enc(449.0) == 0x7E and enc(1e30) == 0x7E and enc(-1e30) == 0xFE
    assert enc(432.0) == 0x7E           # halfway 416 (0x7d, odd) / 448 (even)
    with pytest.raises(ValueError):
        e4m3_encode(np.array([np.nan]))


def test_nearest_by_exact_rational_arithmetic():
    rng = np.random.default_rng(0)
    xs = np.concatenate([rng.normal(0, 1, 300), rng.normal(0, 60, 200), rng.normal(0, 0.01, 200)])
    finite = [(c, Fraction(e4m3_decode(c))) for c in range(0x7F)]
    for x in xs:
        fx = min(abs(Fraction(float(x))), Fraction(448))
        best = min(finite, key=lambda cv: (abs(cv[1] - fx), cv[0] % 2))     # nearest, then even code
        want = best[0] | (0x80 if x < 0 else 0)
        assert int(e4m3_encode(np.array([x]))[0]) == want


def test_against_torch_float8_cast_inside_the_finite_range():
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.normal(0, 1, 20000), rng.normal(0, 100, 20000), rng.normal(0, 1e-2, 20000),
                        np.array([e4m3_decode(c) for c in range(0x7F)]),
                        np.array([(e4m3_decode(c) + e4m3_decode(c + 1)) / 2 for c in range(0x7E)])])
    x = x[np.abs(x) <= 448.0].astype(np.float32)
    t = torch.from_numpy(x).to(torch.float8_e4m3fn)
    assert np.array_equal(t.view(torch.uint8).numpy(), e4m3_encode(x))
    assert np.array_equal(t.to(torch.float32).numpy().astype(np.float64), e4m3_round(x))


def test_relative_error_bound():
    rng = np.random.default_rng(2)
    x = rng.normal(0, 3, 50000)
    x = x[np.abs(x) >= 2.0 ** -6]
    assert (np.abs(e4m3_round(x) - x) / np.abs(x)).max() <= 2.0 ** -4


def test_cache_rule_in_the_decoder_is_consistent_and_moderate():
    # with the 8-bit cache rule the incremental decoder still equals the full forward (both see the
    # same stored keys / values), appends in chunks equal one append, and the logits move by about
    # the format's step relative to the unquantised model, not more
    from oracle import OracleEngine
    from oracle.decoder import OracleModel, forward_full
    from synthetic import SHAPES
    from synthetic.weights import make_weight_blob
    shape = SHAPES["tiny"]
    blob = make_weight_blob(shape, seed=4, weight_std=0.05, gain_std=0.1)
    toks = np.random.default_rng(0).integers(0, shape.vocab, 41)
    e1 = OracleEngine(blob, max_context=64, max_trajectories=2, kv_pool_pages=16, kv_cache_dtype="fp8_e4m3")
    e1.append_observation([0], toks, [41])
    e2 = OracleEngine(blob, max_context=64, max_trajectories=2, kv_pool_pages=16, kv_cache_dtype="fp8_e4m3")
    e2.append_observation([0], toks[:17], [17])
    e2.append_observation([0], toks[17:], [24])
    z1, z2 = e1.debug_logits(0), e2.debug_logits(0)
    assert np.abs(z1 - z2).max() < 1e-12
    full = forward_full(e1.model, toks)[-1]
    assert np.abs(full - z1).max() < 1e-12
    plain = forward_full(OracleModel(blob), toks)[-1]
    d = np.abs(plain - z1).max()
    assert 1e-5 < d < 0.25 * plain.std()
    with pytest.raises(ValueError):
        OracleEngine(blob, kv_cache_dtype="int4")
