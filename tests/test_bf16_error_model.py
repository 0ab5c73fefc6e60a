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


# ---- quantitative pins of the error model ---------------------------------------------------
# Relative error of rounding to bf16 (8 significant bits, nearest): uniform in +-2^-8 / mantissa;
# with log-uniform mantissas E[mantissa^-2] = 3 / (8 ln 2), so the rms relative error is
# 2^-8 * sqrt(1 / (8 ln 2)) = 1.659e-3.
BF16_RMS_REL = 2.0 ** -8 * np.sqrt(1.0 / (8.0 * np.log(2.0)))


def _rms(x):
    return float(np.sqrt(np.mean(np.square(x))))


def _model(layers=4, tokens=48):
    shape = SHAPES["small-d128"].replace(n_layers=layers)
    m = OracleModel(make_weight_blob(shape, seed=3, weight_std=0.0442))
    toks = np.random.default_rng(1).integers(0, shape.vocab, tokens)
    return m, toks, forward_full(m, toks)


def test_rounding_law_of_bf16():
    x = np.random.default_rng(0).standard_normal(1 << 18)
    rel = (round_bf16(x) - x) / x
    assert np.abs(rel).max() <= 2.0 ** -8
    assert abs(_rms(rel) / BF16_RMS_REL - 1.0) < 0.05


def test_final_norm_point_is_linear_and_follows_the_rounding_law():
    from oracle.decoder import hidden_full, rmsnorm
    m, toks, z = _model()
    f = rmsnorm(hidden_full(m, toks), m.w("g_final"), m.rms_eps)
    dz = forward_bf16_model(m, toks, frozenset("f")) - z
    # rounding only the final normed state perturbs the logits by exactly W_lm (round(f) - f)
    assert np.abs(dz - (round_bf16(f) - f) @ m.w("lm_head").T).max() < 1e-10
    # independent per-element errors of rms 1.659e-3 |f_i| through a random matrix: the logits move
    # by 1.659e-3 of their own standard deviation (gains are 1, so |f|^2 = H)
    assert abs(_rms(dz) / (BF16_RMS_REL * z.std()) - 1.0) < 0.1


def test_every_point_counts_once_and_energies_add():
    m, toks, z = _model()
    e_all = _rms(forward_bf16_model(m, toks, ALL_POINTS) - z) ** 2
    single = {}
    for pt in sorted(ALL_POINTS):
        single[pt] = _rms(forward_bf16_model(m, toks, frozenset(pt)) - z) ** 2
        # no point is a no-op, none dominates: each carries 0.5 % - 50 % of the total energy
        assert 0.005 * e_all < single[pt] < 0.5 * e_all, (pt, single[pt], e_all)
    # the nine roundings are independent first-order perturbations: their energies add
    assert abs(sum(single.values()) / e_all - 1.0) < 0.15, (single, e_all)
    # leaving out one of the four heaviest points lowers the predicted energy by about that point's
    # own energy (the other roundings fall differently once their inputs move, hence the wide band)
    for pt in "abov":
        e_wo = _rms(forward_bf16_model(m, toks, ALL_POINTS - {pt}) - z) ** 2
        assert 0.5 < (e_all - e_wo) / single[pt] < 1.5, (pt, e_all, e_wo, single[pt])
    # a rounding applied twice changes nothing (idempotent), so a doubled point cannot hide
    assert np.array_equal(round_bf16(round_bf16(z)), round_bf16(z))
