"""Pins for oracle/rl_oracle.py: closed forms, the paper's explicit sums written as scalar loops,
special cases."""
import math

import numpy as np

from oracle import rl_oracle as ro


def test_gae_matches_the_explicit_double_sum():
    rng = np.random.default_rng(0)
    n, T, g, lam = 3, 9, 0.99, 0.95
    r, v = rng.standard_normal((n, T)), rng.standard_normal((n, T + 1))
    adv, ret = ro.ogae(r, v, None, g, lam)
    for i in range(n):
        for t in range(T):
            s = 0.0
            for k in range(T - t):          # A_t = sum_{k=0}^{T-t-1} (gamma lambda)^k delta_{t+k}
                s += (g * lam) ** k * (r[i, t + k] + g * v[i, t + k + 1] - v[i, t + k])
            assert abs(adv[i, t] - s) < 1e-12
    assert np.allclose(ret, adv + v[:, :T])


def test_gae_closed_forms():
    T = 12
    r, v = np.ones((1, T)), np.zeros((1, T + 1))
    q = 0.99 * 0.95
    adv, _ = ro.ogae(r, v, None, 0.99, 0.95)        # geometric series
    assert np.allclose(adv[0], [(1 - q ** (T - t)) / (1 - q) for t in range(T)])
    rng = np.random.default_rng(1)
    r, v = rng.standard_normal((2, T)), rng.standard_normal((2, T + 1))
    adv0, _ = ro.ogae(r, v, None, 0.9, 0.0)          # lambda = 0: the TD error
    assert np.allclose(adv0, r + 0.9 * v[:, 1:] - v[:, :-1])
    adv1, ret1 = ro.ogae(r, v, None, 0.9, 1.0)       # lambda = 1: discounted return + bootstrap - V
    for t in range(T):
        disc = sum(0.9 ** k * r[:, t + k] for k in range(T - t)) + 0.9 ** (T - t) * v[:, T]
        assert np.allclose(adv1[:, t], disc - v[:, t]) and np.allclose(ret1[:, t], disc)


def test_gae_done_flag_splits_episodes():
    rng = np.random.default_rng(2)
    r, v = rng.standard_normal((1, 10)), rng.standard_normal((1, 11))
    d = np.zeros((1, 10)); d[0, 3] = 1
    adv, _ = ro.ogae(r, v, d, 0.99, 0.95)
    first, _ = ro.ogae(r[:, :4], np.concatenate([v[:, :4], np.zeros((1, 1))], 1), None, 0.99, 0.95)
    second, _ = ro.ogae(r[:, 4:], v[:, 4:], None, 0.99, 0.95)
    assert np.allclose(adv[0, :4], first[0]) and np.allclose(adv[0, 4:], second[0])


def test_grpo_advantage_properties_and_example():
    adv, keep = ro.ogrpo_advantage([1, 0, 0, 1, 1, 1, 1, 1, 3, 1, 1, 1], 4)
    assert keep.tolist() == [True, False, True]
    assert np.allclose(adv[:4], [1, -1, -1, 1]) and np.allclose(adv[4:8], 0)
    assert np.allclose(adv[8:], np.array([1.5, -0.5, -0.5, -0.5]) / math.sqrt(0.75))
    rng = np.random.default_rng(3)
    R = rng.standard_normal(64)
    a, k = ro.ogrpo_advantage(R, 8)
    a = a.reshape(8, 8)
    assert np.allclose(a.mean(1), 0) and np.allclose((a ** 2).mean(1), 1) and k.all()
    a2, _ = ro.ogrpo_advantage(5.0 * R + 3.0, 8)       # invariant to positive affine maps of the return
    assert np.allclose(a2.reshape(8, 8), a)


def test_objective_special_cases():
    lo = np.zeros((1, 4))
    A = np.array([[2.0, 2.0, -2.0, -2.0]])
    ln = np.log(np.array([[1.5, 0.5, 1.5, 0.5]]))
    obj, s, frac = ro.opolicy_objective(ln, lo, A, None, 0.2, 0.28, False)
    # A > 0: rho above 1.28 is clipped, rho below stays; A < 0: rho below 0.8 is clipped, above stays
    assert np.allclose(s, [[1.28 * 2, 0.5 * 2, 1.5 * -2, 0.8 * -2]])
    assert abs(obj - s.mean()) < 1e-15 and abs(frac - 0.5) < 1e-15
    obj1, _, f1 = ro.opolicy_objective(lo, lo, A, None, 0.2, 0.28, False)   # rho = 1: mean advantage
    assert abs(obj1 - A.mean()) < 1e-15 and f1 == 0


def test_objective_normalisations_match_scalar_loops():
    rng = np.random.default_rng(4)
    n, T = 6, 7
    ln, lo = rng.standard_normal((n, T)) * 0.3, rng.standard_normal((n, T)) * 0.3
    A = rng.standard_normal(n)
    mask = (np.arange(T)[None, :] < rng.integers(0, T + 1, n)[:, None]).astype(np.int32)
    mask[0] = 0                                          # one trajectory with no valid step
    obj, _, _ = ro.opolicy_objective(ln, lo, A, mask, 0.2, 0.28, True)
    tot = 0.0
    for i in range(n):
        Ti = int(mask[i].sum())
        acc = 0.0
        for t in range(Ti):                              # the first T_i steps are the valid ones
            rho = math.exp(ln[i, t] - lo[i, t])
            acc += min(rho * A[i], min(max(rho, 0.8), 1.28) * A[i])
        tot += acc / Ti if Ti else 0.0
    assert abs(obj - tot / n) < 1e-12
    objp, _, _ = ro.opolicy_objective(ln, lo, A, mask, 0.2, 0.28, False)
    tot, cnt = 0.0, 0
    for i in range(n):
        for t in range(T):
            if mask[i, t]:
                rho = math.exp(ln[i, t] - lo[i, t])
                tot += min(rho * A[i], min(max(rho, 0.8), 1.28) * A[i]); cnt += 1
    assert abs(objp - tot / cnt) < 1e-12


def test_logp_aggregate_is_the_log_of_the_product():
    rng = np.random.default_rng(5)
    p = rng.uniform(0.05, 1.0, (4, 8, 7))                # [env, action of the chunk, token]
    action = ro.ologp_aggregate(np.log(p), 7)
    assert np.allclose(action, np.log(p.prod(-1)).reshape(-1))
    chunk = ro.ologp_aggregate(action, 8)
    assert np.allclose(chunk, np.log(p.reshape(4, -1).prod(-1)))
