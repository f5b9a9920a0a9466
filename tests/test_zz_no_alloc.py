"""The entry point that allocates nothing, vla_policy_objective_noalloc, against vla_policy_objective (same
kernels, partial sums in the library's built-in array instead of a workspace): identical bits, on two calls in a
row of which the second is smaller, so that what the first call left in the shared array would show if it were read."""
import numpy as np
import pytest
import torch

from paper_2510_06710_amd import binding as vb

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _case(n, T, seed):
    rng = np.random.default_rng(seed)
    lo = -np.abs(rng.standard_normal((n, T))).astype(np.float32) * 2
    ln = (lo + 0.25 * rng.standard_normal((n, T))).astype(np.float32)
    adv = rng.standard_normal(n).astype(np.float32)
    m = (np.arange(T)[None, :] < rng.integers(0, T + 1, n)[:, None]).astype(np.int32)
    t = lambda a, dt=torch.float32: torch.from_numpy(a).to(dt).to(DEV)
    return t(ln), t(lo), t(adv), t(m, torch.int32)


def _run_both(n, T, seed, per_traj):
    ln, lo, adv, m = _case(n, T, seed)
    outs = []
    for noalloc in (False, True):
        obj, frac = torch.full((1,), -7.0, device=DEV), torch.full((1,), -7.0, device=DEV)
        per = torch.full((n, T), -7.0, device=DEV)
        if noalloc:
            vb.vla_policy_objective_noalloc(ln, lo, adv, False, m, n, T, 0.2, 0.28, per_traj, obj, per, frac)
        else:
            ws = torch.empty(vb.vla_policy_objective_workspace_bytes(n), dtype=torch.uint8, device=DEV)
            vb.vla_policy_objective(ln, lo, adv, False, m, n, T, 0.2, 0.28, per_traj, ws, obj, per, frac)
        torch.cuda.synchronize()
        outs.append((obj.cpu().numpy(), frac.cpu().numpy(), per.cpu().numpy()))
    return outs


def test_noalloc_objective_matches_the_workspace_form_on_two_calls():
    for n, T, seed in ((4096, 80, 1), (37, 13, 2)):            # the second call is smaller than the first
        for per_traj in (True, False):
            (o0, f0, p0), (o1, f1, p1) = _run_both(n, T, seed, per_traj)
            assert np.isfinite(o0).all() and np.array_equal(o0, o1), (n, T, per_traj, o0, o1)
            assert np.array_equal(f0, f1) and np.array_equal(p0, p1)


def test_noalloc_objective_rejects_sizes_beyond_its_scratch():
    cap = vb.vla_policy_objective_noalloc_max_traj()
    assert cap == 65536
    x = torch.zeros(8, device=DEV)
    with pytest.raises(vb.VlaError) as e:
        vb.vla_policy_objective_noalloc(x, x, x, False, None, cap + 1, 1, 0.2, 0.28, True, x)
    assert e.value.code == vb.VLA_ESHAPE
