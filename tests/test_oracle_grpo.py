"""Pins of the GRPO-objective oracle against what the published definition fixes: hand-worked
values of every branch of the clipped surrogate, closed forms, and identities that hold for any
distributions (checked by brute force over small categorical distributions)."""
import math

import numpy as np
import pytest

from oracle.grpo import group_advantages, trajectory_objective, grpo_objective

LN2 = 0.6931471805599453


def test_advantages_hand_values():
    assert np.allclose(group_advantages([1, 0], 2, eps_std=0.0), [1, -1], atol=1e-15)
    assert np.allclose(group_advantages([3, 1, 1, 3], 4, eps_std=0.0), [1, -1, -1, 1], atol=1e-15)
    # sample standard deviation of (1, 0) is sqrt(1/2)
    assert np.allclose(group_advantages([1, 0], 2, eps_std=0.0, std_ddof=1), [0.7071067811865476, -0.7071067811865476])
    # two groups are normalised separately
    a = group_advantages([1, 0, 10, 30], 2, eps_std=0.0)
    assert np.allclose(a, [1, -1, -1, 1])
    # eps enters the denominator: (1 - 0.5) / (0.5 + 0.5)
    assert np.allclose(group_advantages([1, 0], 2, eps_std=0.5), [0.5, -0.5])


def test_advantages_invariants():
    rng = np.random.default_rng(0)
    r = rng.normal(size=24)
    a = group_advantages(r, 8, eps_std=0.0)
    for g in range(3):
        assert abs(a[g * 8:(g + 1) * 8].sum()) < 1e-12
        assert abs((a[g * 8:(g + 1) * 8] ** 2).sum() - 8) < 1e-12        # unit population variance
    assert np.allclose(group_advantages(5.0 * r + 3.0, 8, eps_std=0.0), a)  # shift and scale invariant
    a1 = group_advantages(r, 8, eps_std=0.0, std_ddof=1)
    assert np.allclose(a1, a * math.sqrt(7 / 8))
    assert np.all(group_advantages([2.0] * 4, 4) == 0.0)                 # all rewards equal
    with pytest.raises(ValueError):
        group_advantages([1, 2, 3], 2)
    with pytest.raises(ValueError):
        group_advantages([1.0], 1, std_ddof=1)


@pytest.mark.parametrize("adv,rho,expect", [(1.0, 1.5, 1.2), (1.0, 0.5, 0.5), (-1.0, 1.5, -1.5),
                                            (-1.0, 0.5, -0.8), (2.0, 1.1, 2.2), (-2.0, 0.9, -1.8)])
def test_clipped_surrogate_branches(adv, rho, expect):
    # positive advantage: the gain is capped at (1 + e) A; negative advantage: the penalty is at
    # least (1 - e) |A| and grows without bound with the ratio
    lp_new = [0.0, math.log(rho) - 1.0]
    lp_old = [0.0, -1.0]
    j, kl, n = trajectory_objective(lp_new, lp_old, None, [1, 0], adv, 0.2, 0.0)
    assert n == 1 and kl == 0.0 and abs(j - expect) < 1e-12


def test_on_policy_value_is_the_advantage():
    rng = np.random.default_rng(1)
    lp = -rng.random(40)
    mask = rng.integers(0, 2, 40)
    mask[5] = 0
    j, _, n = trajectory_objective(lp, lp, None, mask, -0.37, 0.2, 0.0)
    assert abs(j - (-0.37)) < 1e-15 and n == int((mask[1:] == 0).sum())
    # whole batch: group-normalised advantages average to zero
    lps = [lp[:10], lp[10:25], lp[25:33], lp[33:]]
    ms = [mask[:10], mask[10:25], mask[25:33], mask[33:]]
    for m in ms:
        m[1] = 0
    out = grpo_objective(lps, lps, None, ms, [0.3, 1.0, 0.0, 0.2], 4, eps_std=0.0)
    assert abs(out["objective"]) < 1e-15


def test_mask_and_first_position_are_excluded():
    lp_new = np.array([-0.3, -1.0, -2.0, -0.5, -0.1])
    lp_old = np.array([-0.9, -1.1, -2.5, -0.4, -0.7])
    mask = np.array([0, 0, 1, 0, 1])
    base = trajectory_objective(lp_new, lp_old, lp_old, mask, 0.8, 0.2, 0.05)
    assert base[2] == 2
    lp2 = lp_new.copy()
    lp2[[0, 2, 4]] += 3.0
    assert trajectory_objective(lp2, lp_old, lp_old, mask, 0.8, 0.2, 0.05) == base
    lp3 = lp_new.copy()
    lp3[3] += 0.01
    assert trajectory_objective(lp3, lp_old, lp_old, mask, 0.8, 0.2, 0.05) != base
    assert trajectory_objective(lp_new, lp_old, None, [1, 1, 1, 1, 1], 0.8, 0.2, 0.0) == (0.0, 0.0, 0)


def test_kl_estimator_values():
    # ref = 2 x new probability: k3 = 2 - ln 2 - 1; the KL term lowers the objective
    j, kl, _ = trajectory_objective([0.0, -1.0], [0.0, -1.0], [0.0, -1.0 + LN2], [1, 0], 1.0, 0.2, 0.1)
    assert abs(kl - (1.0 - LN2)) < 1e-15 and abs(j - (1.0 - 0.1 * (1.0 - LN2))) < 1e-15
    # ref = new: zero; small difference: d^2 / 2 to second order; never negative
    assert trajectory_objective([0, -1.0], [0, -1.0], [0, -1.0], [1, 0], 1.0, 0.2, 0.1)[1] == 0.0
    d = 1e-3
    kl = trajectory_objective([0, -1.0], [0, -1.0], [0, -1.0 + d], [1, 0], 1.0, 0.2, 0.1)[1]
    assert abs(kl - d * d / 2) < d ** 3
    rng = np.random.default_rng(2)
    for _ in range(100):
        a, b = -rng.random() * 5, -rng.random() * 5
        assert trajectory_objective([0, a], [0, a], [0, b], [1, 0], 1.0, 0.2, 1.0)[1] >= 0.0


def test_expectations_by_brute_force_over_a_categorical():
    # for x ~ pi_new: E[k3] = KL(pi_new || pi_ref); for x ~ pi_old: E[rho] = 1 (no clipping, A = 1)
    rng = np.random.default_rng(3)
    V = 7
    def dist():
        p = rng.random(V) + 0.05
        return p / p.sum()
    p_new, p_old, p_ref = dist(), dist(), dist()
    e_k3, e_rho = 0.0, 0.0
    for x in range(V):
        lpn, lpo, lpr = math.log(p_new[x]), math.log(p_old[x]), math.log(p_ref[x])
        _, k3, _ = trajectory_objective([0, lpn], [0, lpn], [0, lpr], [1, 0], 0.0, 0.2, 1.0)
        e_k3 += p_new[x] * k3
        rho, _, _ = trajectory_objective([0, lpn], [0, lpo], None, [1, 0], 1.0, 1e9, 0.0)
        e_rho += p_old[x] * rho
    kl_exact = float((p_new * np.log(p_new / p_ref)).sum())
    assert abs(e_k3 - kl_exact) < 1e-12
    assert abs(e_rho - 1.0) < 1e-12


def test_aggregation_is_per_trajectory_then_over_trajectories():
    # trajectory 0 (A = +1): one token at ratio 1.5 -> 1.2; trajectory 1 (A = -1): three tokens at
    # ratio 0.5 -> -0.8 each.  Mean of trajectory means = 0.2 (a mean over all four tokens would be -0.3)
    l15, l05 = math.log(1.5), math.log(0.5)
    out = grpo_objective([[0, l15], [0, l05, l05, l05]], [[0, 0], [0, 0, 0, 0]], None,
                         [[1, 0], [1, 0, 0, 0]], [1, 0], 2, clip_eps=0.2, eps_std=0.0)
    assert abs(out["objective"] - 0.2) < 1e-12 and out["n_tokens"] == 4
    # a trajectory without sampled tokens contributes zero and still counts in the mean
    out = grpo_objective([[0, l15], [0, l05]], [[0, 0], [0, 0]], None, [[1, 0], [1, 1]], [1, 0], 2,
                         clip_eps=0.2, eps_std=0.0)
    assert abs(out["objective"] - 0.6) < 1e-12 and out["n_tokens"] == 1


def test_engine_objective_uses_recomputed_logprobs():
    from oracle import OracleEngine
    from synthetic import SHAPES
    from synthetic.weights import make_weight_blob
    shape = SHAPES["tiny"]
    blob = make_weight_blob(shape, seed=3)
    e = OracleEngine(blob, max_context=64, max_trajectories=4, kv_pool_pages=32)
    rng = np.random.default_rng(5)
    e.append_observation([0], rng.integers(0, shape.vocab, 6), [6])
    e.fork(0, [1, 2, 3])
    for _ in range(5):
        e.decode_step([0, 1, 2, 3], 1.0, 11)
    e.append_observation([1, 2], rng.integers(0, shape.vocab, 6), [3, 3])
    for _ in range(3):
        e.decode_step([1, 2], 1.0, 11)
    # old = log-probs recorded at sampling time = the recomputed ones: on-policy, objective = mean advantage = 0
    out = e.grpo_objective([0, 1, 2, 3], 4, [1.0, 0.0, 0.5, 0.0], 1.0, 0.2, 0.0)
    assert abs(out["objective"]) < 1e-5 and out["n_tokens"] == 5 * 4 + 3 * 2
    # shifting the old log-probs of one trajectory down by ln 2 doubles its ratios: clipped at 1.2 for A > 0
    new = e.recompute_logprobs([0, 1, 2, 3], 1.0).astype(np.float64)
    old = new.copy()
    old[:11] -= LN2
    adv = out["advantages"]
    out2 = e.grpo_objective([0, 1, 2, 3], 4, [1.0, 0.0, 0.5, 0.0], 1.0, 0.2, 0.0, old_logprobs=old)
    assert adv[0] > 0 and abs(out2["objective"] - (1.2 * adv[0] + adv[1] + adv[2] + adv[3]) / 4) < 1e-5
