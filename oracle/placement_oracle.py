"""Oracle (test infrastructure, CPU only) for the rollout-time model of the GPU allocation modes and
the automatic placement search (section IV-A: collocated mode, hybrid mode with fine-grained
pipelining, auto-placement algorithm).  Plain Python, written as an event-by-event simulation of the
schedule the section describes; the library's closed forms are checked against it.

Readings of the section (it gives t_1 in closed form and no formula for t_2, only that it is an estimate for
pipelined execution):
  * one rollout epoch is m chunk steps; in each, Generation turns observations into actions (time
    t_G(b) for b environments per Generation GPU) and the Simulator turns actions into the next
    observations (t_S(b) per Simulator GPU); observations o_0 are available at time 0;
  * k = 1 (collocated): all N GPUs hold both components, each handles n_S / N environments, the two
    phases alternate: t_1 = m (t_G(n_S / N) + t_S(n_S / N));
  * k = 2 (hybrid, pipelined): N_G GPUs generate, N_S = N - N_G simulate, the environments of every
    GPU are split into k sub-batches that take turns in a fixed round-robin order; the Generation
    partition works on one sub-batch at a time and so does the Simulator partition; a sub-batch's
    simulator step starts when its actions are ready and the simulator is free, its next generation
    when its observations are ready and the generator is free;
  * a partition of n GPUs splits the n_S environments evenly, the time is that of the fullest GPU:
    ceil(n_S / (k n)) environments per sub-batch (at least one per GPU, or the split is not used);
  * t_G, t_S are profiled at batch sizes 1, 2, 4, ...; other sizes are interpolated linearly between
    the two neighbouring profiled sizes (sizes above the largest profiled one are not allowed).
Only tests/, the smoke check and the benchmark's baseline leg may import this module."""
from __future__ import annotations

from typing import List, Optional, Sequence, Tuple


def opipeline_time(g: float, s: float, k: int, m: int) -> float:
    """Makespan of m chunk steps over k sub-batches (generation g and simulation s per sub-batch
    step), simulated event by event."""
    gen_free = 0.0          # when the Generation partition is idle again
    sim_free = 0.0
    ready = [0.0] * k       # when sub-batch j's current observation exists
    for _ in range(m):
        for j in range(k):
            start_g = max(gen_free, ready[j])
            end_g = start_g + g
            gen_free = end_g
            start_s = max(sim_free, end_g)
            end_s = start_s + s
            sim_free = end_s
            ready[j] = end_s
    return max(ready) if k > 0 and m > 0 else 0.0


def oprofile_lookup(profile: Sequence[float], b: float) -> float:
    """profile[i] is the time at batch 2**i; linear interpolation in b between neighbours."""
    if b < 1 or b > 2 ** (len(profile) - 1):
        raise ValueError("batch outside the profiled range")
    i = 0
    while 2 ** (i + 1) <= b and i + 1 < len(profile):
        i += 1
    lo = 2 ** i
    if b == lo:
        return float(profile[i])
    hi = 2 ** (i + 1)
    w = (b - lo) / (hi - lo)
    return float(profile[i]) * (1 - w) + float(profile[i + 1]) * w


def oplacement_candidates(t_gen: Sequence[float], t_sim: Sequence[float], n_envs: int, n_gpus: int,
                          m: int) -> List[Tuple[int, int, int, float]]:
    """Every feasible (k, N_G, N_S, time): k = 1 collocated on all GPUs; k = 2 for every split
    N_G + N_S = N.  A candidate needs at least one environment per GPU and sub-batch."""
    out = []
    if n_envs >= n_gpus:
        b = -(-n_envs // n_gpus)
        out.append((1, n_gpus, n_gpus, opipeline_time(oprofile_lookup(t_gen, b), oprofile_lookup(t_sim, b), 1, m)))
    for n_g in range(1, n_gpus):
        n_s = n_gpus - n_g
        if n_envs < 2 * n_g or n_envs < 2 * n_s:
            continue
        g = oprofile_lookup(t_gen, -(-n_envs // (2 * n_g)))
        s = oprofile_lookup(t_sim, -(-n_envs // (2 * n_s)))
        out.append((2, n_g, n_s, opipeline_time(g, s, 2, m)))
    return out


def oauto_placement(t_gen, t_sim, n_envs: int, n_gpus: int, m: int) -> Optional[Tuple[int, int, int, float]]:
    """The candidate with the smallest time (first one in enumeration order on ties)."""
    best = None
    for c in oplacement_candidates(t_gen, t_sim, n_envs, n_gpus, m):
        if best is None or c[3] < best[3]:
            best = c
    return best
