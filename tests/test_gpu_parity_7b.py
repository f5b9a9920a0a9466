"""GPU parity at the 7B shape (bf16), in the launch configurations the benchmark times: full batches of
64 / 256 / 128 environments and 512 stored rollouts.

The oracle cannot run whole batches at this size, so
(a) one-layer models of 7B width run at the FULL batch sizes (256 autoregressive environments, 128 x 56 chunk
    slots, 512 rollouts in two passes) and the first, a middle and the LAST environment are compared with the
    oracle on the same bf16-stored tensors at the stated bar (logits 2e-2, log-prob 1e-2, near-tie gap 1e-2);
(b) the 32-layer model is compared on sampled environments (again including the last one) against oracle outputs
    stored by tests/golden/make_golden.py (a committed script that calls only oracle/ and the input generator).
    Through 32 layers of bf16 operands the stated bar cannot hold for any implementation; the bounds are per depth
    and per oracle mode, 1.5 times the deviation that tests/bf16_drift.py measures on the CPU between correct
    evaluations (parity.deep_tol), on the RMS as well as on the maximum;
(c) properties that hold at any size are checked on the full outputs."""
import math
import os

import numpy as np
import pytest
import torch

import vla_inputs as vi
from oracle.from_inputs import oracle_weights
from parity import (GpuCase, assert_rms, compare_recompute, compare_rollout, deep_tol, oracle_recompute, oracle_rollout)

pytestmark = pytest.mark.gpu

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "oracle_7b.npz")
LN256 = math.log(256.0)


@pytest.fixture(scope="module")
def golden():
    if not os.path.exists(GOLDEN):
        pytest.skip("tests/golden/oracle_7b.npz not generated")
    return np.load(GOLDEN, allow_pickle=False)


@pytest.fixture(scope="module")
def golden_ops():
    path = GOLDEN.replace("oracle_7b.npz", "oracle_7b_bf16ops.npz")
    if not os.path.exists(path):
        return None          # optional: only the exact-oracle comparisons run without it
    return np.load(path, allow_pickle=False)


@pytest.fixture(scope="module")
def model7b():
    """One 7B-shape model on the GPU (13 GB of weights), shared by the tests of this module."""
    wl = vi.WORKLOADS["cfg3_7b_b256"]
    print("\n[7b] generating weights on the GPU", flush=True)
    case = GpuCase(wl, 0, max_batch=256, max_seq=344)
    yield case
    del case
    torch.cuda.empty_cache()


def _golden_rollout(golden, prefix, env):
    keys = ("h_last", "value", "bins", "logp", "ent", "logits", "gap")
    return {k: golden[f"{prefix}_{env}_{k}"] for k in keys}


def _have(golden, prefix, env):
    return golden is not None and f"{prefix}_{env}_logits" in golden


def _take(d, e):
    return {k: v[e:e + 1] for k, v in d.items()}


def _check_properties(out, B, A):
    assert out["bins"].shape == (B, A) and out["bins"].min() >= 0 and out["bins"].max() < 256
    for k in ("logp", "ent", "logits", "value"):
        assert np.isfinite(out[k]).all(), k
    assert (out["logp"] <= 1e-6).all()
    assert (out["ent"] >= -1e-5).all() and (out["ent"] <= LN256 + 1e-5).all()
    z = out["logits"].astype(np.float64)
    lse = np.log(np.exp(z - z.max(-1, keepdims=True)).sum(-1)) + z.max(-1)
    lp = np.take_along_axis(z, out["bins"][..., None].astype(np.int64), -1)[..., 0] - lse
    assert np.max(np.abs(lp - out["logp"])) < 1e-4          # temperature 1 in these workloads


# ------------------------------------------------------------------------------------------------------------
# (a) one layer of 7B width at the full launch geometry, stated bar
# ------------------------------------------------------------------------------------------------------------
def test_one_layer_7b_width_every_env_meets_the_stated_bar():
    wl = vi.scaled(vi.WORKLOADS["cfg2_7b_b64"], n_layers=1, batch=6)
    print("\n[7b] oracle on 6 envs x 1 layer", flush=True)
    gpu = GpuCase(wl, 1).rollout()
    st = compare_rollout(gpu, oracle_rollout(wl, 1, operand_dtype="bf16"), "bf16", autoregressive=True)
    print(f"[parity] 1-layer 7B width vs bf16-stored oracle: {st}", flush=True)


def _one_layer_weights(wl, seed):
    return oracle_weights(vi.SynthModel(wl.shape, seed), vi.VALUE_BIAS)


def test_one_layer_full_batch_256_autoregressive_stated_bar():
    """The benchmarked geometry of the rollout step: 73,728 prefill rows (288 GEMM row tiles, the XCD-strided tile
    walk with its column panels, 256 x 32 attention items) and decode forwards of 256 rows at K = 4096 / 11008."""
    wl = vi.scaled(vi.WORKLOADS["cfg3_7b_b256"], n_layers=1)
    print("\n[7b] 1 layer, B = 256 autoregressive", flush=True)
    out = GpuCase(wl, 2).rollout()
    _check_properties(out, wl.batch, wl.n_action)
    w = _one_layer_weights(wl, 2)
    for e in (0, 131, 255):
        ref = oracle_rollout(wl, 2, env0=e, envs=1, weights=w, operand_dtype="bf16")
        st = compare_rollout(_take(out, e), ref, "bf16", autoregressive=True)
        print(f"[parity] 1 layer B=256 env {e} vs bf16-stored oracle: {st}", flush=True)


def test_one_layer_full_batch_128_chunk_of_56_stated_bar():
    wl = vi.scaled(vi.WORKLOADS["cfg4_7b_oft_b128"], n_layers=1)
    print("\n[7b] 1 layer, B = 128 x 56 slots", flush=True)
    out = GpuCase(wl, 2).rollout(sampled=False)
    _check_properties(out, wl.batch, wl.n_action)
    w = _one_layer_weights(wl, 2)
    for e in (0, 77, 127):
        ref = oracle_rollout(wl, 2, env0=e, envs=1, sampled=False, weights=w, operand_dtype="bf16")
        st = compare_rollout(_take(out, e), ref, "bf16", autoregressive=False)
        print(f"[parity] 1 layer B=128 chunk env {e} vs bf16-stored oracle: {st}", flush=True)


def test_one_layer_512_rollouts_in_two_passes_stated_bar():
    """The recompute geometry: 512 rollouts x 294 rows in two passes of 256 (75,264 rows each: a ragged last
    GEMM row tile and ten attention query blocks per rollout); the last rollout of each pass and the first of the
    second are among those compared."""
    wl = vi.scaled(vi.WORKLOADS["cfg5_7b_recompute_n512"], n_layers=1)
    print("\n[7b] 1 layer, N = 512 recompute in two passes", flush=True)
    bins = vi.stored_bins(wl, 2).numpy()
    out = GpuCase(wl, 2, max_batch=256).recompute(bins)
    assert np.isfinite(out["logp"]).all() and (out["logp"] <= 1e-6).all()
    w = _one_layer_weights(wl, 2)
    for e in (0, 255, 256, 511):
        ref = oracle_recompute(wl, 2, bins[e:e + 1], env0=e, envs=1, weights=w, operand_dtype="bf16")
        st = compare_recompute({k: v[e:e + 1] for k, v in out.items()}, ref, "bf16")
        print(f"[parity] 1 layer N=512 rollout {e} vs bf16-stored oracle: {st}", flush=True)


def test_two_layer_7b_width_every_env():
    wl = vi.scaled(vi.WORKLOADS["cfg2_7b_b64"], n_layers=2, batch=6)
    print("\n[7b] oracle on 6 envs x 2 layers", flush=True)
    gpu = GpuCase(wl, 1).rollout()
    for mode, against in (("bf16", "ops"), ("exact", "exact")):
        tol = deep_tol(2, against, n_logits=6 * 7 * 256, n_tokens=6 * 7)
        st = compare_rollout(gpu, oracle_rollout(wl, 1, operand_dtype=mode), tol, autoregressive=True)
        print(f"[parity] 2-layer 7B width vs {mode} oracle: {st}\n         bounds {tol}", flush=True)


# ------------------------------------------------------------------------------------------------------------
# (b) all 32 layers at the full batch sizes against stored oracle outputs, per-depth derived bounds
# ------------------------------------------------------------------------------------------------------------
def _compare_envs(out, goldens, prefix, envs, A, autoregressive, name):
    for ref, against in goldens:
        if ref is None:
            continue
        present = [e for e in envs if _have(ref, prefix, e)]
        assert present, f"no stored oracle output for {prefix} envs {envs}"
        tol = deep_tol(32, against, n_logits=len(present) * A * 256, n_tokens=len(present) * A)
        tot = dict(near_ties=0, max_logit_err=0.0, max_logp_err=0.0, max_ent_err=0.0, max_value_err=0.0)
        pool = {}
        for e in present:
            st = compare_rollout(_take(out, e), _golden_rollout(ref, prefix, e), tol, autoregressive=autoregressive, pooled_rms=pool)
            tot["near_ties"] += st["near_ties"]
            for k in ("max_logit_err", "max_logp_err", "max_ent_err", "max_value_err"):
                tot[k] = max(tot[k], st[k])
        tot["rms_logit_err"] = math.sqrt(pool["sq_logit"] / max(pool["n_logit"], 1))
        tot["rms_logp_err"] = math.sqrt(pool["sq_logp"] / max(pool["n_logp"], 1))
        tot["n_logp"] = pool["n_logp"]
        assert_rms(tot["rms_logit_err"], pool["n_logit"], tot["rms_logp_err"], pool["n_logp"], tol, tot)
        which = "bf16-stored oracle" if against == "ops" else "exact oracle"
        print(f"[parity] {name} envs {present} vs {which}: {tot}\n         bounds {tol}", flush=True)


@pytest.mark.parametrize("name,envs", [("cfg2_7b_b64", [0, 37, 63]), ("cfg3_7b_b256", [0, 37, 200, 255])])
def test_ar_rollout_sampled_envs_vs_golden(model7b, golden, golden_ops, name, envs):
    wl = vi.WORKLOADS[name]
    model7b.wl = wl
    model7b.slot = None
    print(f"\n[7b] {name} rollout", flush=True)
    out = model7b.rollout()
    _check_properties(out, wl.batch, wl.n_action)
    _compare_envs(out, ((golden_ops, "ops"), (golden, "exact")), "ar", envs, wl.n_action, True, name)


def test_oft_chunk_sampled_envs_vs_golden(model7b, golden, golden_ops):
    wl = vi.WORKLOADS["cfg4_7b_oft_b128"]
    model7b.wl = wl
    model7b.slot = model7b.synth.slot_embed(wl.n_action)
    print("\n[7b] cfg4 parallel chunk", flush=True)
    out = model7b.rollout(sampled=False)
    _check_properties(out, wl.batch, wl.n_action)
    _compare_envs(out, ((golden_ops, "ops"), (golden, "exact")), "oft", [0, 100, 127], wl.n_action, False, "cfg4")


def test_chunk_rollout_then_chunk_recompute_rho_one_at_7b(model7b):
    """The parallel-chunk recompute (prefix and slot rows in one teacher-forced pass of 344 rows per environment:
    eleven query blocks, so the prefill attention merges a ragged group into the workgroup before it) against the
    chunk decode of the same model (slot rows at an offset against the cached prefix): rho = 1 for all 128 x 56
    slots, within the bound for two bf16 evaluations of the same rows."""
    wl = vi.WORKLOADS["cfg4_7b_oft_b128"]
    model7b.wl = wl
    model7b.slot = model7b.synth.slot_embed(wl.n_action)
    out = model7b.rollout(sampled=False)
    rc = model7b.recompute(out["bins"])
    n = wl.batch * wl.n_action
    tol = deep_tol(32, "impl", n_logits=n * 256, n_tokens=n)
    dlp = rc["logp"].astype(np.float64) - out["logp"]
    rho = np.exp(dlp)
    err = np.max(np.abs(rc["logits"] - out["logits"]))
    print(f"\n[parity] 7B chunk rho range {rho.min():.5f} .. {rho.max():.5f}, log-prob difference rms "
          f"{np.sqrt(np.mean(dlp ** 2)):.5f}, max logit difference {err:.4f}\n         bounds {tol}", flush=True)
    assert rho.shape == (wl.batch, wl.n_action)
    assert np.sqrt(np.mean(dlp ** 2)) <= tol["logp_rms"] and np.max(np.abs(dlp)) <= tol["logp"]
    assert err <= tol["logits"]
    assert np.max(np.abs(rc["value"] - out["value"])) <= tol["value"]
    assert np.max(np.abs(rc["ent"] - out["ent"])) <= tol["ent"]


def test_recompute_sampled_rollouts_vs_golden(model7b, golden, golden_ops):
    wl = vi.WORKLOADS["cfg5_7b_recompute_n512"]
    model7b.wl = wl
    model7b.slot = None
    bins = vi.stored_bins(wl, 0).numpy()
    print("\n[7b] cfg5 recompute, 512 rollouts in micro-batches of 256", flush=True)
    out = model7b.recompute(bins)
    assert np.isfinite(out["logp"]).all() and (out["logp"] <= 1e-6).all()
    assert (out["ent"] >= -1e-5).all() and (out["ent"] <= LN256 + 1e-5).all()
    for g, against in ((golden_ops, "ops"), (golden, "exact")):
        if g is None:
            continue
        present = [e for e in (0, 256, 300, 511) if f"rc_{e}_logits" in g]
        tol = deep_tol(32, against, n_logits=len(present) * wl.n_action * 256, n_tokens=len(present) * wl.n_action)
        for e in present:
            assert np.array_equal(bins[e:e + 1], g[f"rc_{e}_bins"])
        ref = {k: np.concatenate([g[f"rc_{e}_{k}"] for e in present]) for k in ("logp", "ent", "value", "logits")}
        got = {k: np.concatenate([v[e:e + 1] for e in present]) for k, v in out.items()}
        st = compare_recompute(got, ref, tol)
        which = "bf16-stored oracle" if against == "ops" else "exact oracle"
        print(f"[parity] cfg5 rollouts {present} vs {which}: {st}\n         bounds {tol}", flush=True)


def test_rollout_then_recompute_rho_one_at_7b(model7b):
    """rho = pi_theta / pi_theta_old = 1 on the GPU's own rollout (appendix I-B), 64 environments: the decode
    path (single-row GEMM and attention kernels) and the recompute path (large-tile kernels) are two bf16
    evaluations of the same rows, so log rho is bounded, in RMS and in maximum, by 1.5 times the deviation the
    CPU model finds between two fp32 evaluations that differ in summation order."""
    wl = vi.WORKLOADS["cfg2_7b_b64"]
    model7b.wl = wl
    model7b.slot = None
    out = model7b.rollout()
    rc = model7b.recompute(out["bins"])
    n = wl.batch * wl.n_action
    tol = deep_tol(32, "impl", n_logits=n * 256, n_tokens=n)
    dlp = rc["logp"].astype(np.float64) - out["logp"]
    rho = np.exp(dlp)
    print(f"\n[parity] 7B rho range {rho.min():.5f} .. {rho.max():.5f}, log rho rms {np.sqrt(np.mean(dlp ** 2)):.5f}, "
          f"max {np.max(np.abs(dlp)):.5f}; bounds rms {tol['logp_rms']:.5f} max {tol['logp']:.5f}", flush=True)
    assert np.sqrt(np.mean(dlp ** 2)) <= tol["logp_rms"]
    assert np.max(np.abs(dlp)) <= tol["logp"]
    assert np.max(np.abs(rc["value"] - out["value"])) < 1e-3
