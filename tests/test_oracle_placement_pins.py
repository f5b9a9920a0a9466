"""Pins of the placement oracle (section IV-A) against things other than itself: a schedule worked
out by hand, the closed forms the schedule must reduce to, bounds that any schedule obeys, and an
independent brute-force search over placements."""
import itertools
import math
import random

import pytest

from oracle.placement_oracle import (oauto_placement, opipeline_time, oplacement_candidates,
                                     oprofile_lookup)


def test_hand_worked_pipeline():
    # g = 3, s = 1, two chunk steps, two sub-batches:
    #   G: A[0,3] B[3,6] A[6,9] B[9,12];  S: A[3,4] B[6,7] A[9,10] B[12,13]  -> 13
    assert opipeline_time(3.0, 1.0, 2, 2) == 13.0
    # g = 1, s = 3: G: A[0,1] B[1,2] A[4,5] B[7,8]; S: A[1,4] B[4,7] A[7,10] B[10,13] -> 13
    assert opipeline_time(1.0, 3.0, 2, 2) == 13.0
    # balanced g = s = 2, m = 3: G: A0-2 B2-4 A4-6 B6-8 A8-10 B10-12; S one slot behind -> 14
    assert opipeline_time(2.0, 2.0, 2, 3) == 14.0


@pytest.mark.parametrize("seed", range(5))
def test_closed_forms(seed):
    rng = random.Random(seed)
    for _ in range(50):
        g, s, m = rng.uniform(0.1, 9), rng.uniform(0.1, 9), rng.randint(1, 40)
        assert opipeline_time(g, s, 1, m) == pytest.approx(m * (g + s), rel=1e-12)     # the section's t_1
        # two sub-batches: the slower component never idles after its first start
        assert opipeline_time(g, s, 2, m) == pytest.approx(2 * m * max(g, s) + min(g, s), rel=1e-12)


def test_bounds_any_schedule_obeys():
    rng = random.Random(7)
    for _ in range(200):
        g, s, m, k = rng.uniform(0.1, 5), rng.uniform(0.1, 5), rng.randint(1, 20), rng.randint(1, 4)
        t = opipeline_time(g, s, k, m)
        assert t >= k * m * max(g, s) - 1e-9          # each partition does k m steps one after another
        assert t >= m * (g + s) - 1e-9                # a sub-batch's own chain of dependent steps
        assert t <= k * m * (g + s) + 1e-9            # no worse than running everything back to back


def test_pipelining_halves_when_balanced_and_batch_time_linear():
    # t(b) proportional to b and g = s: two half batches overlap perfectly, t_2 -> t_1 / 2 for large m
    m = 1000
    t1 = opipeline_time(2.0, 2.0, 1, m)
    t2 = opipeline_time(1.0, 1.0, 2, m)
    assert t2 / t1 == pytest.approx(0.5, rel=2e-3)


def test_profile_lookup():
    prof = [1.0, 1.5, 4.0, 5.0]                        # batch 1, 2, 4, 8
    assert oprofile_lookup(prof, 1) == 1.0 and oprofile_lookup(prof, 8) == 5.0
    assert oprofile_lookup(prof, 3) == pytest.approx(2.75)
    assert oprofile_lookup(prof, 6) == pytest.approx(4.5)
    with pytest.raises(ValueError):
        oprofile_lookup(prof, 9)
    with pytest.raises(ValueError):
        oprofile_lookup(prof, 0)


def test_search_against_independent_enumeration():
    rng = random.Random(3)
    for _ in range(30):
        n_prof = rng.randint(4, 9)
        tg = sorted(rng.uniform(1, 50) for _ in range(n_prof))
        ts = sorted(rng.uniform(1, 50) for _ in range(n_prof))
        n_gpus = rng.choice([2, 4, 8])
        n_envs = 2 ** (n_prof - 1)
        m = rng.randint(1, 30)
        best = oauto_placement(tg, ts, n_envs, n_gpus, m)
        # independent enumeration with the closed forms, exact power-of-two batches only
        cands = []
        if n_envs % n_gpus == 0:
            i = int(math.log2(n_envs // n_gpus))
            cands.append((1, n_gpus, n_gpus, m * (tg[i] + ts[i])))
        for n_g in range(1, n_gpus):
            n_s = n_gpus - n_g
            bg, bs = n_envs / (2 * n_g), n_envs / (2 * n_s)
            if bg != int(bg) or bs != int(bs) or bg < 1 or bs < 1:
                continue
            if math.log2(bg) != int(math.log2(bg)) or math.log2(bs) != int(math.log2(bs)):
                continue
            g, s = tg[int(math.log2(bg))], ts[int(math.log2(bs))]
            cands.append((2, n_g, n_s, 2 * m * max(g, s) + min(g, s)))
        ref = min(cands, key=lambda c: c[3])
        mine = {c[:3]: c[3] for c in oplacement_candidates(tg, ts, n_envs, n_gpus, m)}
        for c in cands:
            assert mine[c[:3]] == pytest.approx(c[3], rel=1e-12)
        assert best[3] <= ref[3] * (1 + 1e-12)             # the full search also has the uneven splits
        assert best[3] == pytest.approx(min(mine.values()), rel=1e-12)


def test_latency_bound_generator_heavy_simulator():
    # generator nearly flat in the batch (weight streaming), simulator linear and heavier per environment:
    # worked by hand with t_G(b) = 30 + 0.05 b, t_S(b) = 1.5 b, 256 environments, 8 GPUs, 10 chunk steps
    #   collocated b = 32: 10 (31.6 + 48) = 796
    #   (N_G, N_S) = (2, 6): b_G = 64, b_S = ceil(256 / 12) = 22: 2 * 10 * max(33.2, 33) + 33 = 697  <- best
    #   (1, 7): b_G = 128, b_S = 19: 20 * 36.4 + 28.5 = 756.5;  (3, 5): b_G = 43, b_S = 26: 20 * 39 + 32.15 = 812.15
    tg = [30 + 0.05 * 2 ** i for i in range(9)]
    ts = [1.5 * 2 ** i for i in range(9)]
    cands = {c[:3]: c[3] for c in oplacement_candidates(tg, ts, 256, 8, 10)}
    assert cands[(1, 8, 8)] == pytest.approx(796.0)
    assert cands[(2, 2, 6)] == pytest.approx(697.0)
    assert cands[(2, 1, 7)] == pytest.approx(756.5)
    assert cands[(2, 3, 5)] == pytest.approx(812.15)
    assert oauto_placement(tg, ts, 256, 8, 10)[:3] == (2, 2, 6)


def test_linear_times_make_collocation_optimal():
    # if both components scale linearly with the batch no GPU ever idles in the collocated mode, so no
    # disjoint split can beat it
    tg = [float(2 ** i) for i in range(9)]
    ts = [15.0 * 2 ** i for i in range(9)]
    assert oauto_placement(tg, ts, 256, 8, 10)[:3] == (1, 8, 8)
