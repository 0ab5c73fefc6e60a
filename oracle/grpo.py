"""Oracle for the token-level masked GRPO objective (forward value only).

TEST INFRASTRUCTURE ONLY (see the package docstring).

The paper trains with GRPO on groups of trajectories that continue one prompt
(Section 2.3, the multi-turn interaction example) and excludes tool results from
the loss through the loss mask (Section 2.2, last paragraph; Section 2.3.2).  It
prints no objective.  What is written out here is the published GRPO objective
(Shao et al. 2024, "DeepSeekMath", the outcome-supervision form: group-normalised
reward as the advantage of every token of a trajectory, clipped importance ratio,
the unbiased non-negative KL estimator), with the sums running over the tokens the
policy sampled (mask 0) only:

    A_i   = (r_i - mean_group(r)) / (std_group(r) + eps_std)
    rho_t = exp(lp_new[t] - lp_old[t])
    k3_t  = exp(lp_ref[t] - lp_new[t]) - (lp_ref[t] - lp_new[t]) - 1
    J_i   = 1/|S_i| * sum_{t in S_i} ( min(rho_t A_i, clip(rho_t, 1-e, 1+e) A_i) - beta k3_t )
    J     = 1/n * sum_i J_i            (S_i = positions of trajectory i with mask 0)

A trajectory without sampled tokens contributes J_i = 0 and still counts in n.
Everything is float64, one token at a time.

parity unpinned against the paper (it states no formula and no value); pinned to
the published definition through closed forms and hand-worked cases in
tests/test_oracle_grpo.py.
"""
import math

import numpy as np


def group_advantages(rewards, group_size, eps_std=1e-6, std_ddof=0):
    """A_i for consecutive groups of group_size rewards."""
    r = np.asarray(rewards, np.float64)
    G = int(group_size)
    if G <= 0 or r.size % G != 0:
        raise ValueError("rewards must be whole groups")
    if std_ddof not in (0, 1) or (std_ddof == 1 and G < 2):
        raise ValueError("std_ddof must be 0, or 1 with groups of at least two")
    adv = np.zeros(r.size, np.float64)
    for g0 in range(0, r.size, G):
        mean = 0.0
        for i in range(g0, g0 + G):
            mean += r[i]
        mean /= G
        var = 0.0
        for i in range(g0, g0 + G):
            var += (r[i] - mean) ** 2
        std = math.sqrt(var / (G - std_ddof))
        for i in range(g0, g0 + G):
            adv[i] = (r[i] - mean) / (std + eps_std)
    return adv


def trajectory_objective(lp_new, lp_old, lp_ref, mask, advantage, clip_eps, beta):
    """(J_i, mean k3 over S_i, |S_i|) of one trajectory."""
    total, kl_total, cnt = 0.0, 0.0, 0
    for t in range(len(mask)):
        if t == 0 or mask[t] != 0:
            continue
        rho = math.exp(float(lp_new[t]) - float(lp_old[t]))
        clipped = min(max(rho, 1.0 - clip_eps), 1.0 + clip_eps)
        term = min(rho * advantage, clipped * advantage)
        if lp_ref is not None:
            d = float(lp_ref[t]) - float(lp_new[t])
            k3 = math.exp(d) - d - 1.0
            term -= beta * k3
            kl_total += k3
        total += term
        cnt += 1
    if cnt == 0:
        return 0.0, 0.0, 0
    return total / cnt, kl_total / cnt, cnt


def grpo_objective(lp_new, lp_old, lp_ref, masks, rewards, group_size, clip_eps=0.2, beta=0.0,
                   eps_std=1e-6, std_ddof=0):
    """lp_* and masks: one array per trajectory (lp_ref may be None).  Returns
    dict(objective, kl, n_tokens, advantages)."""
    n = len(masks)
    adv = group_advantages(rewards, group_size, eps_std, std_ddof)
    if adv.size != n:
        raise ValueError("one reward per trajectory")
    J, KL, N = 0.0, 0.0, 0
    for i in range(n):
        ji, kli, ci = trajectory_objective(lp_new[i], lp_old[i], None if lp_ref is None else lp_ref[i],
                                           masks[i], adv[i], clip_eps, beta)
        J += ji
        KL += kli
        N += ci
    return dict(objective=J / n if n else 0.0, kl=KL / n if n else 0.0, n_tokens=N, advantages=adv)
