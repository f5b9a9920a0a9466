"""The library's host-side placement arithmetic (closed forms) against the oracle's event-by-event
simulation and exhaustive search (section IV-A).  Host only: no device is touched."""
import random

import pytest

from oracle.placement_oracle import (oauto_placement, opipeline_time, oplacement_candidates,
                                     oprofile_lookup)
from paper_2510_06710_amd import binding as vb


@pytest.mark.parametrize("seed", range(4))
def test_pipeline_time_matches_simulation(seed):
    rng = random.Random(seed)
    for _ in range(200):
        g, s, m = rng.uniform(0.0, 20.0), rng.uniform(0.0, 20.0), rng.randint(0, 60)
        for k in (1, 2):
            assert vb.vla_pipeline_time(g, s, k, m) == pytest.approx(opipeline_time(g, s, k, m), rel=1e-12, abs=1e-12)


def test_pipeline_time_rejects_bad_arguments():
    for args in ((1.0, 1.0, 3, 5), (1.0, 1.0, 0, 5), (-1.0, 1.0, 1, 5), (float("nan"), 1.0, 2, 5), (1.0, 1.0, 2, -1)):
        with pytest.raises(vb.VlaError) as e:
            vb.vla_pipeline_time(*args)
        assert e.value.code == vb.VLA_EINVAL


def test_profile_lookup_matches_oracle():
    rng = random.Random(11)
    prof = sorted(rng.uniform(1, 100) for _ in range(9))
    for b in [1, 2, 3, 5, 8, 100, 255, 256, 1.5, 77.25]:
        assert vb.vla_profile_lookup(prof, b) == pytest.approx(oprofile_lookup(prof, b), rel=1e-12)
    for b in (0, 0.5, 257, 1e9):
        with pytest.raises(vb.VlaError) as e:
            vb.vla_profile_lookup(prof, b)
        assert e.value.code == vb.VLA_ESHAPE


@pytest.mark.parametrize("seed", range(6))
def test_auto_placement_matches_exhaustive_search(seed):
    rng = random.Random(100 + seed)
    for _ in range(40):
        n_prof = rng.randint(3, 10)
        tg = [rng.uniform(1, 30)]
        ts = [rng.uniform(1, 30)]
        for _ in range(n_prof - 1):                       # non-decreasing, sub- or super-linear at random
            tg.append(tg[-1] * rng.uniform(1.0, 2.3))
            ts.append(ts[-1] * rng.uniform(1.0, 2.3))
        n_gpus = rng.randint(1, 9)
        n_envs = rng.randint(1, 2 ** (n_prof - 1))
        m = rng.randint(1, 50)
        ref_all = oplacement_candidates(tg, ts, n_envs, n_gpus, m)
        if not ref_all:
            with pytest.raises(vb.VlaError):
                vb.vla_auto_placement(tg, ts, n_envs, n_gpus, m)
            continue
        best, cands = vb.vla_auto_placement(tg, ts, n_envs, n_gpus, m)
        assert len(cands) == len(ref_all)
        for c, r in zip(cands, ref_all):
            assert c[:3] == r[:3] and c[3] == pytest.approx(r[3], rel=1e-12)
        ref = oauto_placement(tg, ts, n_envs, n_gpus, m)
        assert best[:3] == ref[:3] and best[3] == pytest.approx(ref[3], rel=1e-12)


def test_worked_example():
    # t_G(b) = 30 + 0.05 b, t_S(b) = 1.5 b, 256 environments on 8 GPUs, 10 chunk steps: by hand the
    # collocated mode takes 796, the (2, 6) split 697 and wins
    tg = [30 + 0.05 * 2 ** i for i in range(9)]
    ts = [1.5 * 2 ** i for i in range(9)]
    best, cands = vb.vla_auto_placement(tg, ts, 256, 8, 10)
    assert best[:3] == (2, 2, 6) and best[3] == pytest.approx(697.0)
    assert cands[0][:3] == (1, 8, 8) and cands[0][3] == pytest.approx(796.0)
