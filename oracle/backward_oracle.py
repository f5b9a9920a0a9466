"""CPU oracle for the gradient of the policy objective's log-probability term with respect to LoRA factors.

TEST INFRASTRUCTURE ONLY, like the rest of ``oracle/``: plain fp64 numpy, the chain rule written out step by
step through the decoder that ``vla_oracle`` defines.  Shares no code with the HIP path.

What it computes.  The policy update differentiates the clipped surrogate (appendix I-B, I-C) through
rho = pi_theta / pi_theta_old = exp(logp_theta - logp_old): every term reaches the parameters only through the
recomputed token log-probabilities (section IV-C.1), so the update needs

    dL / dtheta   with   L = sum_{n, j} coef[n, j] * logp_theta[n, j],

where coef = dJ / dlogp is what the objective's elementwise part hands back (rho * A-hat on the unclipped
branch, 0 on the clipped one).  The paper trains LoRA adapters (section IV-B.2): each of the seven projections
of a decoder layer is W_eff = W + scale * B A with A [r, in], B [out, r], and theta = {A, B}.  The forward runs
on the effective weights (the caller merges them); with dY the gradient at a projection's output and X its
input,

    dL / dB = scale * dY^T (X A^T),        dL / dA = scale * (dY B)^T X,

and dX = dY W_eff carries the gradient on.  Everything else is the textbook backward of RMSNorm, rotary
(an orthogonal map: its transpose is the rotation by the negative angle), causal softmax attention, SwiGLU,
the residual sums, the final norm and the log-softmax over the 256 action bins at temperature tau.

Readings where the paper is silent: LoRA on all seven projections of every layer and on nothing else (embeddings,
norm gains and the action head are frozen); only the log-probability term is differentiated (the printed
objectives carry no entropy or value-loss term); in the "bf16" operand mode the forward rounds the stored tensors
as ``vla_oracle`` does and the backward treats each rounding as the identity (straight-through), all of it in
fp64.

Pins (tests/test_oracle_backward_pins.py): the cached forward here reproduces ``ovla_logprob_recompute`` bit for
bit; central finite differences of that forward through merged weights, for entries of every A and B; identity
layers (W_o = W_d = 0) reduce the o / down gradients to a one-line closed form and zero all others; coef = 0 rows
contribute nothing; linearity in coef; batch independence.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Tuple

import numpy as np

from . import vla_oracle as vo

F64 = np.float64
PROJ = ("q", "k", "v", "o", "gate", "up", "down")
WEIGHT_OF = {"q": "wq", "k": "wk", "v": "wv", "o": "wo", "gate": "w_gate", "up": "w_up", "down": "w_down"}
Lora = List[Dict[str, Tuple[np.ndarray, np.ndarray]]]     # per layer: projection -> (A [r, in], B [out, r])


def merged_layer(base: Dict[str, np.ndarray], lora_l, scale: float) -> Dict[str, np.ndarray]:
    """W_eff = W + scale * B A for the seven projections; norm gains unchanged."""
    out = dict(base)
    for p in PROJ:
        A, B = lora_l[p]
        out[WEIGHT_OF[p]] = base[WEIGHT_OF[p]] + scale * (B @ A)
    return out


def rmsnorm_backward(x: np.ndarray, gain: np.ndarray, eps: float, dn: np.ndarray) -> np.ndarray:
    """n = x r g with r = (mean(x^2) + eps)^(-1/2):  dx = r (g dn) - x r^3 mean(x g dn)."""
    r = 1.0 / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)
    gd = gain * dn
    return r * gd - x * (r ** 3) * np.mean(x * gd, axis=-1, keepdims=True)


def dsilu(t: np.ndarray) -> np.ndarray:
    s = 1.0 / (1.0 + np.exp(-t))
    return s * (1.0 + t * (1.0 - s))


def _layer_forward(cfg, lw, x, positions, allowed):
    """One decoder layer exactly as ``vla_oracle.decoder_layers`` computes it (no cache of earlier rows), keeping
    what the backward needs."""
    st = lambda t: vo.stored(cfg, t)
    n = st(vo.rmsnorm(x, lw["attn_norm"], cfg.rms_eps))
    q = st(vo.rotary(vo.split_heads(n @ lw["wq"].T, cfg.n_heads), positions, cfg.rope_theta))
    k = st(vo.rotary(vo.split_heads(n @ lw["wk"].T, cfg.n_heads), positions, cfg.rope_theta))
    v = st(vo.split_heads(n @ lw["wv"].T, cfg.n_heads))
    d = q.shape[-1]
    s = np.einsum("nhrd,nhkd->nhrk", q, k) / np.sqrt(float(d))
    s = np.where(allowed[None, None], s, -np.inf)
    s = s - s.max(axis=-1, keepdims=True)
    p = np.exp(s)
    p = p / p.sum(axis=-1, keepdims=True)
    ao = st(vo.merge_heads(np.einsum("nhrk,nhkd->nhrd", p, v)))
    x_mid = x + ao @ lw["wo"].T
    n2 = st(vo.rmsnorm(x_mid, lw["ffn_norm"], cfg.rms_eps))
    g, u = n2 @ lw["w_gate"].T, n2 @ lw["w_up"].T
    act = st(vo.silu(g) * u)
    x_out = x_mid + act @ lw["w_down"].T
    return x_out, dict(x=x, n=n, q=q, k=k, v=v, p=p, ao=ao, x_mid=x_mid, n2=n2, g=g, u=u, act=act)


def _lora_grads(X, dY, A, B, scale):
    """dL/dA [r, in] and dL/dB [out, r] of Y = X (W + scale B A)^T given dY; X [.., in], dY [.., out]."""
    X2, dY2 = X.reshape(-1, X.shape[-1]), dY.reshape(-1, dY.shape[-1])
    dB = scale * dY2.T @ (X2 @ A.T)
    dA = scale * (dY2 @ B).T @ X2
    return dA, dB


def _layer_backward(cfg, lw, lora_l, scale, c, positions, dx):
    """Gradient at the layer's input and the LoRA gradients of its seven projections, given dx at its output."""
    grads = {}
    # x_out = x_mid + act W_d^T
    grads["down"] = _lora_grads(c["act"], dx, *lora_l["down"], scale)
    d_act = dx @ lw["w_down"]
    dg = d_act * c["u"] * dsilu(c["g"])
    du = d_act * vo.silu(c["g"])
    grads["gate"] = _lora_grads(c["n2"], dg, *lora_l["gate"], scale)
    grads["up"] = _lora_grads(c["n2"], du, *lora_l["up"], scale)
    dn2 = dg @ lw["w_gate"] + du @ lw["w_up"]
    dx_mid = dx + rmsnorm_backward(c["x_mid"], lw["ffn_norm"], cfg.rms_eps, dn2)
    # x_mid = x + ao W_o^T
    grads["o"] = _lora_grads(c["ao"], dx_mid, *lora_l["o"], scale)
    d_o = vo.split_heads(dx_mid @ lw["wo"], cfg.n_heads)                    # [n, nh, R, d]
    p, q, k, v = c["p"], c["q"], c["k"], c["v"]
    d = q.shape[-1]
    dP = np.einsum("nhrd,nhkd->nhrk", d_o, v)
    dv = np.einsum("nhrk,nhrd->nhkd", p, d_o)
    dS = p * (dP - np.sum(p * dP, axis=-1, keepdims=True))                  # masked keys have p = 0
    dq = np.einsum("nhrk,nhkd->nhrd", dS, k) / np.sqrt(float(d))
    dk = np.einsum("nhrk,nhrd->nhkd", dS, q) / np.sqrt(float(d))
    # the rotation is orthogonal: its transpose rotates by the negative angle
    dq_pre = vo.merge_heads(vo.rotary(dq, -positions, cfg.rope_theta))
    dk_pre = vo.merge_heads(vo.rotary(dk, -positions, cfg.rope_theta))
    dv_m = vo.merge_heads(dv)
    grads["q"] = _lora_grads(c["n"], dq_pre, *lora_l["q"], scale)
    grads["k"] = _lora_grads(c["n"], dk_pre, *lora_l["k"], scale)
    grads["v"] = _lora_grads(c["n"], dv_m, *lora_l["v"], scale)
    dn = dq_pre @ lw["wq"] + dk_pre @ lw["wk"] + dv_m @ lw["wv"]
    dx_in = dx_mid + rmsnorm_backward(c["x"], lw["attn_norm"], cfg.rms_eps, dn)
    return dx_in, grads


def ovla_logprob_backward(cfg: vo.OracleConfig, w: vo.OracleWeights, lora: Lora, scale: float, patch: np.ndarray,
                          ids: np.ndarray, bins: np.ndarray, coef: np.ndarray, A: int, mode: int = 0,
                          slot_embed: Optional[np.ndarray] = None, temperature: float = 1.0):
    """Gradients of L = sum(coef * logp) over N stored rollouts, teacher-forced as in ``ovla_logprob_recompute``.

    ``w`` holds the weights the forward runs on (for a LoRA model: the merged ones); ``lora[l][p] = (A, B)`` are the
    factors the gradients are taken with respect to.  coef [N, A].  Returns (grads, logp) with grads[l][p] =
    (dL/dA [r, in], dL/dB [out, r]) and logp [N, A] the forward's log-probabilities of the stored bins."""
    N = patch.shape[0]
    K = cfg.n_bins
    x = vo.embed_prefix(w, patch, ids)
    S = x.shape[1]
    if mode == 0:
        if A > 1:
            x = np.concatenate([x, w.embed[cfg.vocab - K + bins[:, :A - 1]]], axis=1)
        R = S + A - 1
        allowed = np.tril(np.ones((R, R), dtype=bool))
        rows = np.arange(S - 1, S - 1 + A)
    else:
        x = np.concatenate([x, np.broadcast_to(slot_embed.astype(F64)[None], (N, A, cfg.hidden))], axis=1)
        R = S + A
        allowed = vo.chunk_mask(S, A)
        rows = np.arange(S, S + A)
    positions = np.arange(R)
    caches = []
    for l in range(cfg.n_layers):
        x, c = _layer_forward(cfg, w.layer(l), x, positions, allowed)
        caches.append(c)
    # head: logp = y_bin - logsumexp(y), y = z / tau, z = h W_bins^T, h = RMSNorm(x[rows])
    Wb = w.lm_head[cfg.vocab - K:]
    xr = x[:, rows]
    z = vo.rmsnorm(xr, w.final_norm, cfg.rms_eps) @ Wb.T
    _, lp, _ = vo.token_distribution(z, temperature)
    logp = np.take_along_axis(lp, bins[:, :A, None].astype(np.int64), axis=-1)[..., 0]
    onehot = np.zeros_like(lp)
    np.put_along_axis(onehot, bins[:, :A, None].astype(np.int64), 1.0, axis=-1)
    dz = coef[..., None] * (onehot - np.exp(lp)) / temperature
    dx = np.zeros_like(x)
    dx[:, rows] = rmsnorm_backward(xr, w.final_norm, cfg.rms_eps, dz @ Wb)
    grads = [None] * cfg.n_layers
    for l in range(cfg.n_layers - 1, -1, -1):
        dx, grads[l] = _layer_backward(cfg, w.layer(l), lora[l], scale, caches[l], positions, dx)
    return grads, logp
