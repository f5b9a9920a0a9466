"""Pins of the model behind the deep-bf16 parity tolerances (tests/bf16_drift.py), CPU only.

(1) The fp32 evaluation used by the model is the decoder's definition: without its bf16 roundings it agrees with
    the fp64 oracle on the tiny workload to fp32 accuracy, with a different K summation order as well.
(2) The committed table tests/golden/bf16_drift_7b.json (written by tests/golden/make_bf16_drift_table.py) is
    reproduced at depths 1, 2 and 4 of the 7B-width model on one stored rollout: what the tolerances rest on can be
    re-derived from code in this repository in about a minute.
(3) The stated parity bar (logits 2e-2) sits inside the model's prediction at one layer and outside it from a few
    layers on, which is why the deep tests carry per-depth bounds; the bounds handed to the tests are 1.5 times the
    table, for every depth and oracle mode."""
import dataclasses
import math

import numpy as np
import pytest

import bf16_drift as bd
import vla_inputs as vi
from oracle import vla_oracle as vo
from oracle.from_inputs import oracle_config, oracle_weights, to_f64


@pytest.mark.parametrize("k_chunks", [1, 3])
def test_fp32_evaluation_is_the_decoder_definition(k_chunks):
    wl = vi.WORKLOADS["cfg1_tiny_fp32"]
    model = vi.SynthModel(wl.shape, 4)
    cfg = oracle_config(wl.shape)
    w = oracle_weights(model, vi.VALUE_BIAS)
    patch, ids = vi.observation(wl, 4)
    x = vo.embed_prefix(w, to_f64(patch), ids.numpy().astype(np.int64))
    S = x.shape[1]
    allowed = np.tril(np.ones((S, S), dtype=bool))
    ref, _ = vo.decoder_layers(cfg, w, x, np.arange(S), allowed, None)
    dec = bd.Fp32Decoder(wl.shape.n_heads, wl.shape.rms_eps, wl.shape.rope_theta, k_chunks, round_stored=False)
    y = x.astype(np.float32)
    for l in range(wl.shape.n_layers):
        y = dec.layer(y, {k: v.astype(np.float32) for k, v in w.layer(l).items()}, allowed)
    assert y.dtype == np.float32
    assert np.max(np.abs(y - ref)) < 2e-5 * max(1.0, np.abs(ref).max())


def test_rounded_evaluation_differs_from_the_exact_one_by_bf16_sized_errors():
    """With the stored tensors rounded, the tiny model's residual stream moves by a few bf16 ulps, no more."""
    wl = vi.WORKLOADS["cfg1_tiny_fp32"]
    model = vi.SynthModel(wl.shape, 4)
    w = oracle_weights(model, vi.VALUE_BIAS)
    patch, ids = vi.observation(wl, 4)
    x = vo.embed_prefix(w, to_f64(patch), ids.numpy().astype(np.int64)).astype(np.float32)
    S = x.shape[1]
    allowed = np.tril(np.ones((S, S), dtype=bool))
    ys = []
    for rs in (False, True):
        dec = bd.Fp32Decoder(wl.shape.n_heads, wl.shape.rms_eps, wl.shape.rope_theta, 1, round_stored=rs)
        y = x
        for l in range(wl.shape.n_layers):
            y = dec.layer(y, {k: v.astype(np.float32) for k, v in w.layer(l).items()}, allowed)
        ys.append(y)
    rel = np.sqrt(np.mean((ys[1] - ys[0]) ** 2) / np.mean(ys[0] ** 2))
    assert 1e-4 < rel < 2e-2, rel


def test_table_is_reproduced_at_depths_1_2_4():
    table = bd.load_table()
    rows = bd.drift_by_depth(4, 1, seed=table["seed"])
    by_depth = {r["depth"]: r for r in table["depths"]}
    for r in rows:
        if r["depth"] not in (1, 2, 4):
            continue
        t = by_depth[r["depth"]]
        for against in ("ops", "exact", "impl"):
            got, want = r[against]["logits_rms"], t[against]["logits_rms"]
            # one rollout here against the table's four: the RMS agrees to the spread between rollouts
            assert 0.7 * want < got < 1.4 * want, (r["depth"], against, got, want)
        assert abs(r["logit_sigma"] - t["logit_sigma"]) < 0.1


def test_table_shape_and_what_it_says_about_the_stated_bar():
    table = bd.load_table()
    depths = [r["depth"] for r in table["depths"]]
    assert depths == list(range(1, 33))
    for against in ("ops", "exact", "impl"):
        rms = [r[against]["logits_rms"] for r in table["depths"]]
        assert all(v > 0 for v in rms)
        assert rms[31] > 3 * rms[0]                              # carried forward and amplified, not damped
        assert rms[31] < 40 * rms[0]                             # but no blow-up either
    one = table["depths"][0]["ops"]
    # one layer: 2e-2 is more than five times the RMS deviation, so the stated bar holds for shallow models
    assert 5 * one["logits_rms"] < 2e-2
    # depth 32: even the RMS deviation from the oracle that rounds the same tensors exceeds the stated bar
    assert table["depths"][31]["ops"]["logits_rms"] > 2e-2


def test_tolerance_is_one_and_a_half_times_the_table():
    table = bd.load_table()
    for depth in (1, 2, 32):
        for against in ("ops", "exact", "impl"):
            t = bd.tolerance(depth, against, n_logits=5376, n_tokens=21)
            row = table["depths"][depth - 1][against]
            assert t["depth_used"] == depth
            assert math.isclose(t["logits_rms"], 1.5 * row["logits_rms"])
            assert math.isclose(t["logp_rms"], 1.5 * row["logp_rms"])
            assert math.isclose(t["logits"], t["logits_rms"] * math.sqrt(2 * math.log(2 * 5376)))
            assert math.isclose(t["logp"], t["logp_rms"] * 3.0)           # fewer than 45 values: the floor of 3 sigma
            # the model's own largest deviation lies inside the bound it yields
            assert row["logits_max"] < bd.tolerance(depth, against, row["logits_n"], row["logp_n"])["logits"]
