"""Pins of oracle/backward_oracle.py (CPU only): the analytic LoRA gradients of L = sum(coef * logp) against things
that are not the backward code itself -- central finite differences of the *forward* oracle through merged weights,
identity-layer reductions, linearity and batch structure."""
import dataclasses

import numpy as np
import pytest

from oracle import backward_oracle as bo
from oracle import vla_oracle as vo

CFG = vo.OracleConfig(n_layers=2, hidden=32, n_heads=2, ffn=48, vocab=300)
RANK, SCALE = 4, 0.5


def _model(seed, cfg=CFG, zero_o_down=False):
    """Random base weights, random LoRA factors, and the merged weights the forward runs on."""
    rng = np.random.default_rng(seed)
    H, F, V = cfg.hidden, cfg.ffn, cfg.vocab
    shapes = {"wq": (H, H), "wk": (H, H), "wv": (H, H), "wo": (H, H), "w_gate": (F, H), "w_up": (F, H), "w_down": (H, F)}
    base, lora = [], []
    for _ in range(cfg.n_layers):
        lw = {k: rng.normal(0, 0.15, s) for k, s in shapes.items()}
        lw["attn_norm"] = 1 + rng.normal(0, 0.05, H)
        lw["ffn_norm"] = 1 + rng.normal(0, 0.05, H)
        ll = {}
        for p in bo.PROJ:
            out, inn = shapes[bo.WEIGHT_OF[p]]
            ll[p] = (rng.normal(0, 0.2, (RANK, inn)), rng.normal(0, 0.2, (out, RANK)))
        if zero_o_down:
            for p in ("o", "down"):
                lw[bo.WEIGHT_OF[p]] = np.zeros_like(lw[bo.WEIGHT_OF[p]])
                ll[p] = (ll[p][0], np.zeros_like(ll[p][1]))
        base.append(lw)
        lora.append(ll)
    head = dict(embed=rng.normal(0, 0.5, (V, H)), lm_head=rng.normal(0, 0.3, (V, H)), final_norm=1 + rng.normal(0, 0.05, H))
    return base, lora, head


def _weights(base, lora, head, scale=SCALE):
    merged = [bo.merged_layer(b, l, scale) for b, l in zip(base, lora)]
    return vo.OracleWeights(embed=head["embed"], lm_head=head["lm_head"], final_norm=head["final_norm"],
                            layer=lambda l: merged[l])


def _inputs(seed, N=3, P=5, T=3, A=4, cfg=CFG):
    rng = np.random.default_rng(100 + seed)
    patch = rng.normal(0, 1, (N, P, cfg.hidden))
    ids = rng.integers(0, cfg.vocab - 256, (N, T))
    bins = rng.integers(0, 256, (N, A)).astype(np.int32)
    coef = rng.normal(0, 1, (N, A))
    slot = rng.normal(0, 0.5, (A, cfg.hidden))
    return patch, ids, bins, coef, slot


def _objective(cfg, w, patch, ids, bins, coef, A, mode, slot, tau):
    logp, _, _, _ = vo.ovla_logprob_recompute(cfg, w, patch, ids, bins, A, mode, slot, tau)
    return float(np.sum(coef * logp))


@pytest.mark.parametrize("mode,tau", [(0, 1.0), (0, 1.6), (1, 1.0)])
def test_forward_inside_the_backward_is_the_recompute_forward(mode, tau):
    base, lora, head = _model(1)
    w = _weights(base, lora, head)
    patch, ids, bins, coef, slot = _inputs(1)
    for cfg in (CFG, dataclasses.replace(CFG, operand_dtype="bf16")):
        _, logp = bo.ovla_logprob_backward(cfg, w, lora, SCALE, patch, ids, bins, coef, 4, mode, slot, tau)
        ref, _, _, _ = vo.ovla_logprob_recompute(cfg, w, patch, ids, bins, 4, mode, slot, tau)
        assert np.array_equal(logp, ref)


@pytest.mark.parametrize("mode,tau", [(0, 1.0), (0, 1.6), (1, 1.0)])
def test_central_finite_differences_of_the_forward_oracle(mode, tau):
    """Every projection of every layer, three entries of A and three of B each: perturb the factor, merge, run the
    plain forward oracle, difference the objective."""
    base, lora, head = _model(2)
    patch, ids, bins, coef, slot = _inputs(2)
    grads, _ = bo.ovla_logprob_backward(CFG, _weights(base, lora, head), lora, SCALE, patch, ids, bins, coef, 4, mode, slot, tau)
    rng = np.random.default_rng(5)
    eps = 1e-5
    worst = 0.0
    for l in range(CFG.n_layers):
        for p in bo.PROJ:
            for which in (0, 1):
                M = lora[l][p][which]
                for _ in range(3):
                    i, j = rng.integers(0, M.shape[0]), rng.integers(0, M.shape[1])
                    vals = []
                    for sgn in (+1, -1):
                        pert = [dict(x) for x in lora]
                        Mp = M.copy()
                        Mp[i, j] += sgn * eps
                        pert[l][p] = (Mp, lora[l][p][1]) if which == 0 else (lora[l][p][0], Mp)
                        vals.append(_objective(CFG, _weights(base, pert, head), patch, ids, bins, coef, 4, mode, slot, tau))
                    fd = (vals[0] - vals[1]) / (2 * eps)
                    an = grads[l][p][which][i, j]
                    worst = max(worst, abs(fd - an) / max(1e-3, abs(an)))
    assert worst < 2e-6, worst


def test_building_blocks_against_finite_differences():
    rng = np.random.default_rng(3)
    x, g, dn = rng.normal(0, 1, 12), 1 + rng.normal(0, 0.1, 12), rng.normal(0, 1, 12)
    an = bo.rmsnorm_backward(x, g, 1e-5, dn)
    for i in range(12):
        e = np.zeros(12); e[i] = 1e-6
        fd = np.sum(dn * (vo.rmsnorm(x + e, g, 1e-5) - vo.rmsnorm(x - e, g, 1e-5))) / 2e-6
        assert abs(fd - an[i]) < 1e-7
    t = np.linspace(-6, 6, 25)
    assert np.max(np.abs((vo.silu(t + 1e-6) - vo.silu(t - 1e-6)) / 2e-6 - bo.dsilu(t))) < 1e-8
    # rotating by the negative angle undoes the rotation (the rotary map is orthogonal)
    u, pos = rng.normal(0, 1, (1, 1, 5, 16)), np.arange(3, 8)
    assert np.max(np.abs(vo.rotary(vo.rotary(u, pos, 10000.0), -pos, 10000.0) - u)) < 1e-12


def test_identity_layers_leave_only_the_o_and_down_gradients():
    """W_o = W_d = 0: every layer is the identity, so the gradient at every layer's output is the head's own, nothing
    reaches q, k, v, gate, up, and dL/dB of the o and down projections is scale * dx^T (input A^T) with dx obtained here
    by finite differences of the head alone and the inputs from the forward building blocks."""
    base, lora, head = _model(4, zero_o_down=True)
    w = _weights(base, lora, head)
    patch, ids, bins, coef, _ = _inputs(4)
    A = 4
    grads, _ = bo.ovla_logprob_backward(CFG, w, lora, SCALE, patch, ids, bins, coef, A, 0, None, 1.0)
    x = np.concatenate([vo.embed_prefix(w, patch, ids), w.embed[CFG.vocab - 256 + bins[:, :A - 1]]], axis=1)
    S = patch.shape[1] + ids.shape[1]
    rows = np.arange(S - 1, S - 1 + A)

    def head_objective(xr):
        z = vo.bin_logits(CFG, w, vo.rmsnorm(xr, w.final_norm, CFG.rms_eps))
        _, lp, _ = vo.token_distribution(z, 1.0)
        return np.sum(coef * np.take_along_axis(lp, bins[..., None].astype(np.int64), -1)[..., 0])

    dx = np.zeros_like(x)
    xr = x[:, rows]
    for idx in np.ndindex(*xr.shape):
        e = np.zeros_like(xr); e[idx] = 1e-6
        dx[idx[0], rows[idx[1]], idx[2]] = (head_objective(xr + e) - head_objective(xr - e)) / 2e-6
    R = x.shape[1]
    allowed = np.tril(np.ones((R, R), dtype=bool))
    for l in range(CFG.n_layers):
        lw = w.layer(l)
        for p in ("q", "k", "v", "gate", "up"):
            assert np.max(np.abs(grads[l][p][0])) == 0 and np.max(np.abs(grads[l][p][1])) == 0
        for p in ("o", "down"):
            assert np.max(np.abs(grads[l][p][0])) == 0            # B = 0: nothing flows back to A
        n = vo.rmsnorm(x, lw["attn_norm"], CFG.rms_eps)
        q = vo.rotary(vo.split_heads(n @ lw["wq"].T, CFG.n_heads), np.arange(R), CFG.rope_theta)
        k = vo.rotary(vo.split_heads(n @ lw["wk"].T, CFG.n_heads), np.arange(R), CFG.rope_theta)
        ao = vo.merge_heads(vo.attention(q, k, vo.split_heads(n @ lw["wv"].T, CFG.n_heads), allowed))
        want_o = SCALE * np.einsum("nro,nrj->oj", dx, ao @ lora[l]["o"][0].T)
        n2 = vo.rmsnorm(x, lw["ffn_norm"], CFG.rms_eps)
        act = vo.silu(n2 @ lw["w_gate"].T) * (n2 @ lw["w_up"].T)
        want_d = SCALE * np.einsum("nro,nrj->oj", dx, act @ lora[l]["down"][0].T)
        assert np.max(np.abs(grads[l]["o"][1] - want_o)) < 1e-7 * max(1.0, np.abs(want_o).max())
        assert np.max(np.abs(grads[l]["down"][1] - want_d)) < 1e-7 * max(1.0, np.abs(want_d).max())


def _flat(grads):
    return np.concatenate([g[l][p][i].ravel() for g in [grads] for l in range(len(grads)) for p in bo.PROJ for i in (0, 1)])


def test_linearity_in_coef_zero_coef_and_batch_independence():
    base, lora, head = _model(6)
    w = _weights(base, lora, head)
    patch, ids, bins, c1, _ = _inputs(6)
    c2 = np.random.default_rng(9).normal(0, 1, c1.shape)
    run = lambda c, sel=slice(None): _flat(bo.ovla_logprob_backward(CFG, w, lora, SCALE, patch[sel], ids[sel], bins[sel], c[sel], 4)[0])
    g1, g2, g12 = run(c1), run(c2), run(c1 + 2 * c2)
    assert np.max(np.abs(g12 - (g1 + 2 * g2))) < 1e-9 * max(1.0, np.abs(g12).max())
    assert np.max(np.abs(run(np.zeros_like(c1)))) == 0
    per = sum(run(c1, slice(i, i + 1)) for i in range(patch.shape[0]))
    assert np.max(np.abs(per - g1)) < 1e-9 * max(1.0, np.abs(g1).max())
    # a rollout whose coefficients are zero changes nothing
    c0 = c1.copy(); c0[1] = 0
    assert np.max(np.abs(run(c0) - (run(c1, slice(0, 1)) + run(c1, slice(2, 3))))) < 1e-9 * max(1.0, np.abs(g1).max())


def test_rounded_forward_keeps_the_gradients_close():
    """Straight-through rounding: the "bf16" operand mode changes the gradients by bf16-sized relative amounts."""
    base, lora, head = _model(7)
    w = _weights(base, lora, head)
    patch, ids, bins, coef, _ = _inputs(7)
    ge = _flat(bo.ovla_logprob_backward(CFG, w, lora, SCALE, patch, ids, bins, coef, 4)[0])
    gb = _flat(bo.ovla_logprob_backward(dataclasses.replace(CFG, operand_dtype="bf16"), w, lora, SCALE, patch, ids, bins, coef, 4)[0])
    rel = np.linalg.norm(gb - ge) / np.linalg.norm(ge)
    assert 0 < rel < 3e-2, rel
