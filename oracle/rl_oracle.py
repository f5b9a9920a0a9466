"""CPU oracle for the advantage estimators and the clipped policy objective that consume the
recomputed log-probabilities (fp64 numpy).  TEST INFRASTRUCTURE ONLY, like the rest of ``oracle/``.

Followed passages: generalized advantage estimation and the PPO clipped objective (appendix I-B);
the group-relative advantage and the GRPO objective with its 1/|tau| normalisation (appendix I-C); the
valid-action mask and the 1/T_succ normalisation (section IV-C.3, appendix II-C.2); the asymmetric clip
ratio (0.2, 0.28), gamma = 0.99 and GAE lambda = 0.95 of the hyper-parameter table; the token / action
/ chunk factorisation of the log-probability (section IV-C.1).

Readings where the paper is silent: (1) with partial reset a rollout row holds several episodes, so a
termination flag done_t cuts both the bootstrap term and the recursion at t (the paper's sum runs to
the episode horizon T); (2) the group standard deviation is the population one (no Bessel correction),
and a group whose returns are all equal gets zero advantages and is flagged for the success-rate
filter, which drops exactly those groups; (3) the expectation E_t of the PPO objective is the mean over
all valid steps of the batch."""
from __future__ import annotations

import numpy as np


def ogae(rewards, values, dones, gamma, lam):
    """A_t = sum_{k>=0} (gamma*lam)^k delta_{t+k}, delta_t = r_t + gamma V_{t+1} - V_t, cut at dones.
    rewards [n, T], values [n, T+1] (last column bootstraps), dones [n, T] or None.
    Returns (advantages [n, T], returns = advantages + values[:, :T])."""
    r = np.asarray(rewards, dtype=np.float64)
    v = np.asarray(values, dtype=np.float64)
    n, T = r.shape
    cont = np.ones((n, T)) if dones is None else 1.0 - np.asarray(dones, dtype=np.float64)
    adv = np.zeros((n, T))
    nxt = np.zeros(n)
    for t in range(T - 1, -1, -1):
        delta = r[:, t] + gamma * v[:, t + 1] * cont[:, t] - v[:, t]
        nxt = delta + gamma * lam * cont[:, t] * nxt
        adv[:, t] = nxt
    return adv, adv + v[:, :T]


def ogrpo_advantage(total_reward, G):
    """A_i = (R_i - mean_group) / std_group over groups of G consecutive trajectories.
    Returns (advantages [n], keep [n_groups] bool: False where the group's returns are all equal)."""
    R = np.asarray(total_reward, dtype=np.float64).reshape(-1, G)
    mean = R.mean(axis=1, keepdims=True)
    std = np.sqrt(((R - mean) ** 2).mean(axis=1, keepdims=True))
    keep = std[:, 0] > 0
    adv = np.where(std > 0, (R - mean) / np.where(std > 0, std, 1.0), 0.0)
    return adv.reshape(-1), keep


def opolicy_objective(logp_new, logp_old, adv, mask, clip_low, clip_high, per_trajectory):
    """Clipped surrogate min(rho A, clip(rho, 1 - clip_low, 1 + clip_high) A), rho = exp(new - old).
    logp_* [n, T]; adv [n, T] or [n] (one advantage per trajectory); mask [n, T] (1 = valid) or None.
    per_trajectory False: mean over all valid steps (PPO).  True: (1/n) sum_i (1/T_i) sum_t (GRPO with
    T_i the number of valid steps; trajectories without a valid step contribute zero).
    Returns (objective, per-step surrogate [n, T], fraction of valid steps where the clip is active)."""
    ln = np.asarray(logp_new, dtype=np.float64)
    lo = np.asarray(logp_old, dtype=np.float64)
    a = np.asarray(adv, dtype=np.float64)
    if a.ndim == 1:
        a = a[:, None] * np.ones_like(ln)
    m = np.ones_like(ln) if mask is None else np.asarray(mask, dtype=np.float64)
    rho = np.exp(ln - lo)
    unclipped = rho * a
    clipped = np.clip(rho, 1.0 - clip_low, 1.0 + clip_high) * a
    s = np.minimum(unclipped, clipped) * m
    n_valid = m.sum()
    if per_trajectory:
        Ti = m.sum(axis=1)
        obj = np.where(Ti > 0, s.sum(axis=1) / np.where(Ti > 0, Ti, 1.0), 0.0).mean()
    else:
        obj = s.sum() / n_valid if n_valid > 0 else 0.0
    frac = ((clipped < unclipped) * m).sum() / n_valid if n_valid > 0 else 0.0
    return float(obj), s, float(frac)


def ologp_aggregate(logp, inner):
    """Token -> action (inner = tokens per action) or action -> chunk (inner = actions per chunk):
    log of a product of probabilities = sum of the log-probabilities over the last `inner` entries."""
    x = np.asarray(logp, dtype=np.float64)
    return x.reshape(-1, inner).sum(axis=1)
