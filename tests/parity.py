"""Helpers shared by the GPU parity tests: run one workload through the oracle (CPU, fp64) and
through the library (GPU), and compare element by element with the near-tie rule for sampled bins."""
from __future__ import annotations

import numpy as np
import torch

import vla_inputs as vi
from oracle import vla_oracle as vo
from oracle.from_inputs import oracle_config, oracle_weights, to_f64

# tolerances of the parity bar: max-abs on logits / log-probs, fp32 storage vs bf16 storage
TOL = {"f32": dict(logits=1e-4, logp=1e-4, ent=1e-4, value=1e-4),
       "bf16": dict(logits=2e-2, logp=1e-2, ent=1e-2, value=2e-2)}
NEAR_TIE = 1e-2


def oracle_rollout(wl: vi.Workload, seed: int, env0: int = 0, envs=None, sampled=True, weights=None):
    """Oracle prefill + decode for environments [env0, env0+envs)."""
    envs = wl.batch - env0 if envs is None else envs
    model = vi.SynthModel(wl.shape, seed)
    cfg = oracle_config(wl.shape)
    w = weights if weights is not None else oracle_weights(model, vi.VALUE_BIAS)
    patch, ids = vi.observation(wl, seed, env0=env0, envs=envs)
    g = to_f64(vi.gumbel_noise(wl, seed, env0=env0, envs=envs)) if sampled else None
    slot = to_f64(model.slot_embed(wl.n_action)) if wl.mode == 1 else None
    kv, h_last, value = vo.ovla_prefill(cfg, w, to_f64(patch), ids.numpy().astype(np.int64))
    bins, logp, ent, logits, _ = vo.ovla_decode_actions(cfg, w, kv, h_last, wl.prefix, wl.n_action, wl.mode,
                                                        slot, wl.temperature, g)
    y = logits / wl.temperature
    t = np.sort(y.astype(np.float32) + (g.astype(np.float32) if g is not None else 0), axis=-1)
    return dict(h_last=h_last, value=value, bins=bins, logp=logp, ent=ent, logits=logits,
                gap=(t[..., -1] - t[..., -2]).astype(np.float64))


def oracle_recompute(wl: vi.Workload, seed: int, bins: np.ndarray, env0: int = 0, envs=None, weights=None):
    envs = wl.batch - env0 if envs is None else envs
    model = vi.SynthModel(wl.shape, seed)
    cfg = oracle_config(wl.shape)
    w = weights if weights is not None else oracle_weights(model, vi.VALUE_BIAS)
    patch, ids = vi.observation(wl, seed, env0=env0, envs=envs)
    slot = to_f64(model.slot_embed(wl.n_action)) if wl.mode == 1 else None
    logp, ent, value, logits = vo.ovla_logprob_recompute(cfg, w, to_f64(patch), ids.numpy().astype(np.int64),
                                                         bins, wl.n_action, wl.mode, slot, wl.temperature)
    return dict(logp=logp, ent=ent, value=value, logits=logits)


class GpuCase:
    """The library on cuda:0 for one workload (weights generated on the device)."""

    def __init__(self, wl: vi.Workload, seed: int, max_batch=None, max_seq=None):
        from paper_2510_06710_amd.harness import Rollout
        self.wl, self.seed = wl, seed
        self.synth = vi.SynthModel(wl.shape, seed, device="cuda:0")
        rows = wl.prefix + wl.n_action
        self.run = Rollout(self.synth, max_batch or wl.batch, max_seq or rows, value_b=vi.VALUE_BIAS)
        self.slot = self.synth.slot_embed(wl.n_action) if wl.mode == 1 else None

    def rollout(self, sampled=True, env0=0, envs=None):
        wl = self.wl
        patch, ids = vi.observation(wl, self.seed, device="cuda:0", env0=env0, envs=envs)
        g = vi.gumbel_noise(wl, self.seed, device="cuda:0", env0=env0, envs=envs) if sampled else None
        h_last, value = self.run.prefill(patch, ids)
        bins, logp, ent, logits = self.run.decode(h_last, wl.prefix, wl.n_action, wl.mode, self.slot,
                                                  wl.temperature, g)
        torch.cuda.synchronize()
        c = lambda t: t.cpu().numpy()
        return dict(h_last=c(h_last), value=c(value), bins=c(bins), logp=c(logp), ent=c(ent), logits=c(logits))

    def recompute(self, bins: np.ndarray, env0=0, envs=None):
        wl = self.wl
        patch, ids = vi.observation(wl, self.seed, device="cuda:0", env0=env0, envs=envs)
        b = torch.from_numpy(np.ascontiguousarray(bins.astype(np.int32))).to("cuda:0")
        logp, ent, value, logits = self.run.recompute(patch, ids, b, wl.n_action, wl.mode, self.slot,
                                                      wl.temperature)
        torch.cuda.synchronize()
        c = lambda t: t.cpu().numpy()
        return dict(logp=c(logp), ent=c(ent), value=c(value), logits=c(logits))


def compare_rollout(gpu, ref, dtype: str, autoregressive: bool):
    """Element-by-element comparison.  A sampled bin may differ only where the oracle's top-2 gap of
    y + g is below NEAR_TIE; such cases are counted, and in autoregressive mode the later tokens of
    that environment (which now follow a different prefix) are left out."""
    tol = TOL[dtype]
    B, A = ref["bins"].shape
    stats = dict(max_logit_err=0.0, max_logp_err=0.0, max_ent_err=0.0, near_ties=0, compared=0)
    if "value" in gpu and gpu["value"] is not None and ref.get("value") is not None:
        stats["max_value_err"] = float(np.max(np.abs(gpu["value"] - ref["value"])))
        assert stats["max_value_err"] <= tol["value"], stats
    for b in range(B):
        for j in range(A):
            stats["compared"] += 1
            stats["max_logit_err"] = max(stats["max_logit_err"], float(np.max(np.abs(gpu["logits"][b, j] - ref["logits"][b, j]))))
            stats["max_ent_err"] = max(stats["max_ent_err"], float(abs(gpu["ent"][b, j] - ref["ent"][b, j])))
            if gpu["bins"][b, j] == ref["bins"][b, j]:
                stats["max_logp_err"] = max(stats["max_logp_err"], float(abs(gpu["logp"][b, j] - ref["logp"][b, j])))
                continue
            assert ref["gap"][b, j] < NEAR_TIE, (b, j, gpu["bins"][b, j], ref["bins"][b, j], ref["gap"][b, j])
            stats["near_ties"] += 1
            if autoregressive:
                break
    assert stats["max_logit_err"] <= tol["logits"], stats
    assert stats["max_logp_err"] <= tol["logp"], stats
    assert stats["max_ent_err"] <= tol["ent"], stats
    return stats


def compare_recompute(gpu, ref, dtype: str):
    tol = TOL[dtype]
    stats = dict(max_logit_err=float(np.max(np.abs(gpu["logits"] - ref["logits"]))),
                 max_logp_err=float(np.max(np.abs(gpu["logp"] - ref["logp"]))),
                 max_ent_err=float(np.max(np.abs(gpu["ent"] - ref["ent"]))),
                 max_value_err=float(np.max(np.abs(gpu["value"] - ref["value"]))))
    assert stats["max_logit_err"] <= tol["logits"], stats
    assert stats["max_logp_err"] <= tol["logp"], stats
    assert stats["max_ent_err"] <= tol["ent"], stats
    assert stats["max_value_err"] <= tol["value"], stats
    return stats
