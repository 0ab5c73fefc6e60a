"""The bf16 rounding-error model (CPU): exact when nothing is rounded; error level it predicts."""
import numpy as np

from oracle.bf16_error_model import forward_bf16_model, round_bf16, ALL_POINTS
from oracle.decoder import OracleModel, forward_full
from synthetic import SHAPES, make_weight_blob


def test_round_bf16_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.14159], np.float64)
    # 1 + 2^-8 is a tie between 1 and 1 + 2^-7 -> even (1.0); 1 + 3*2^-8 ties up to 1 + 2^-6
    assert list(round_bf16(x)[:3]) == [1.0, 1.0, 1.015625]
    assert abs(round_bf16(x)[4] - 3.14159) < 2 ** -7


def test_model_without_rounding_is_the_oracle_and_error_scale():
    shape = SHAPES["small-d128"].replace(n_layers=6)
    m = OracleModel(make_weight_blob(shape, seed=1, weight_std=0.0442))     # logit std ~ 1
    toks = np.random.default_rng(0).integers(0, shape.vocab, 40)
    z = forward_full(m, toks)
    assert np.abs(forward_bf16_model(m, toks, points=frozenset()) - z).max() < 1e-10
    err = forward_bf16_model(m, toks, ALL_POINTS) - z
    rms = float(np.sqrt((err ** 2).mean()))
    # bf16 keeps 8 significant bits: the logits of a unit-scale model move by a few 1e-3 rms and by
    # several times that at the worst of ~3e5 entries
    assert 2e-3 < rms < 2e-2 and np.abs(err).max() > 3 * rms
