"""How far apart two correct bf16 implementations of the decoder may be: the model behind the parity
tolerances of deep bf16 models.  Test infrastructure; imports the oracle, never the HIP library.

The stated parity bar (logits 2e-2, log-prob 1e-2) is what one rounding of the result costs.  A model whose
projections take bf16 *operands* rounds seven stored tensors per layer (norm outputs, rotated q and k, v,
attention output, SwiGLU output), and an implementation that accumulates in fp32 lands on the other side of a
rounding boundary than one that accumulates in fp64 for a small share of those elements; each such flip is a
full bf16 ulp that the following layers of a random-weight decoder carry forward undamped.  This module measures
that, on the CPU, with three evaluations of the same teacher-forced forward (section IV-C.1 row alignment):

  * the oracle in its "bf16" mode (fp64 arithmetic, stored tensors rounded to bf16),
  * the oracle in its "exact" mode (fp64 arithmetic, nothing rounded),
  * ``Fp32Decoder``: the same definition evaluated in fp32 arithmetic with the same stored tensors rounded to
    bf16 -- a stand-in for *any* implementation of the kind the HIP kernels are (bf16 operands, fp32
    accumulation); ``k_chunks`` changes the order in which every projection sums over K, which is how two
    such implementations (the single-row decode path and the multi-row recompute path) differ.

It is written from the decoder's definition, shares nothing with the kernels, and claims nothing about their
exact rounding; only the *size* of the deviation is taken from it (``drift_by_depth``), and the parity tests
allow 1.5 times that (``tolerance``).
"""
from __future__ import annotations

import dataclasses
import json
import math
import os

import numpy as np

import vla_inputs as vi
from oracle import vla_oracle as vo
from oracle.from_inputs import oracle_config, to_f64

F32 = np.float32
TABLE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "bf16_drift_7b.json")


def _bf16(x: np.ndarray) -> np.ndarray:
    """Nearest bfloat16 (ties to even) of an fp32 array, as fp32."""
    u = np.ascontiguousarray(x, dtype=F32).view(np.uint32)
    u = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return u.view(F32)


class Fp32Decoder:
    """One decoder layer at a time in fp32 arithmetic on bf16-rounded stored tensors."""

    def __init__(self, n_heads: int, eps: float, theta: float, k_chunks: int = 1, round_stored: bool = True):
        self.nh, self.eps, self.theta, self.k_chunks = n_heads, F32(eps), theta, k_chunks
        self.st = _bf16 if round_stored else (lambda t: t)     # without rounding: the plain definition in fp32

    def proj(self, a: np.ndarray, w: np.ndarray) -> np.ndarray:
        """a [.., K] . w [N, K]^T with the K range summed in ``k_chunks`` pieces, in order."""
        K = a.shape[-1]
        step = -(-K // self.k_chunks)
        out = None
        for k0 in range(0, K, step):
            part = a[..., k0:k0 + step] @ w[:, k0:k0 + step].T
            out = part if out is None else out + part
        return out

    def norm(self, x, gain):
        return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True, dtype=F32) + self.eps) * gain

    def rope(self, u, pos):
        d = u.shape[-1]
        half = d // 2
        phi = pos.astype(np.float64)[:, None] * self.theta ** (-2.0 * np.arange(half) / d)
        c, s = np.cos(phi).astype(F32), np.sin(phi).astype(F32)
        a, b = u[..., :half], u[..., half:]
        return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)

    def heads(self, x):
        n, r, h = x.shape
        return x.reshape(n, r, self.nh, h // self.nh).transpose(0, 2, 1, 3)

    def layer(self, x: np.ndarray, lw: dict, allowed: np.ndarray) -> np.ndarray:
        pos = np.arange(x.shape[1])
        n = self.st(self.norm(x, lw["attn_norm"]))
        q = self.st(self.rope(self.heads(self.proj(n, lw["wq"])), pos))
        k = self.st(self.rope(self.heads(self.proj(n, lw["wk"])), pos))
        v = self.st(self.heads(self.proj(n, lw["wv"])))
        s = np.einsum("nhrd,nhkd->nhrk", q, k) / F32(math.sqrt(q.shape[-1]))
        s = np.where(allowed[None, None], s, F32(-np.inf))
        p = np.exp(s - s.max(axis=-1, keepdims=True))
        o = np.einsum("nhrk,nhkd->nhrd", p, v) / p.sum(axis=-1, keepdims=True)
        nn, nh, r, d = o.shape
        x = x + self.proj(self.st(o.transpose(0, 2, 1, 3).reshape(nn, r, nh * d)), lw["wo"])
        n2 = self.st(self.norm(x, lw["ffn_norm"]))
        g, u = self.proj(n2, lw["w_gate"]), self.proj(n2, lw["w_up"])
        return x + self.proj(self.st(g / (F32(1) + np.exp(-g)) * u), lw["w_down"])


def _readout(cfg, w, x, rows, bins, S):
    """Logits, log-prob of the stored bins, entropy (fp64 head on whatever residual stream it is handed) and value."""
    x = np.asarray(x, dtype=np.float64)
    z = vo.bin_logits(cfg, w, vo.rmsnorm(x[:, rows], w.final_norm, cfg.rms_eps))
    _, lp, ent = vo.token_distribution(z, 1.0)
    logp = np.take_along_axis(lp, bins[..., None].astype(np.int64), axis=-1)[..., 0]
    value = vo.value_head(cfg, w, vo.rmsnorm(x[:, S - 1], w.final_norm, cfg.rms_eps))
    return dict(logits=z, logp=logp, ent=ent, value=value)


def _stats(a: dict, b: dict) -> dict:
    out = {}
    for k in ("logits", "logp", "ent", "value"):
        d = np.asarray(a[k], dtype=np.float64) - b[k]
        out[k + "_rms"] = float(np.sqrt(np.mean(d * d)))
        out[k + "_max"] = float(np.max(np.abs(d)))
        out[k + "_n"] = int(d.size)
    return out


def drift_by_depth(n_layers: int, envs: int, seed: int = 0, k_chunks_b: int = 4, progress=None) -> list:
    """Teacher-forced forward (288-row prefix + 6 stored action tokens, the recompute workload's rows) over
    ``envs`` stored rollouts of the 7B-width model, read out after every depth 1..n_layers.  Returns one dict
    per depth with the deviations fp32-vs-bf16-stored-oracle ("ops"), fp32-vs-exact-oracle ("exact"), and
    between two fp32 evaluations that sum K in one piece and in ``k_chunks_b`` pieces ("impl")."""
    wl = vi.scaled(vi.WORKLOADS["cfg5_7b_recompute_n512"], n_layers=n_layers)
    model = vi.SynthModel(wl.shape, seed)
    cfgs = {m: dataclasses.replace(oracle_config(wl.shape, m), n_layers=1) for m in ("bf16", "exact")}
    patch, ids = vi.observation(wl, seed, envs=envs)
    bins = vi.stored_bins(wl, seed, envs=envs).numpy()
    S, A = wl.prefix, wl.n_action
    V, H, nb = wl.shape.vocab, wl.shape.hidden, wl.shape.n_bins

    def rows_of(tag, wanted):
        # only the rows that are read, in an otherwise untouched [V, H] array (any row regenerates on its own)
        full = np.zeros((V, H))
        for i in sorted(set(int(v) for v in wanted)):
            full[i] = to_f64(vi.normal(seed, tag, (V, H), sigma=vi.WEIGHT_SIGMA, dtype=wl.shape.torch_dtype,
                                       row0=i, rows=1))[0]
        return full

    head = vo.OracleWeights(embed=rows_of(vi.TAG_EMBED, list(ids.numpy().ravel()) + list((V - nb + bins).ravel())),
                            lm_head=rows_of(vi.TAG_LM_HEAD, range(V - nb, V)),
                            final_norm=to_f64(model.final_norm()), layer=None,
                            value_w=to_f64(model.value_w(1)), value_b=vi.VALUE_BIAS)
    x0 = np.concatenate([vo.embed_prefix(head, to_f64(patch), ids.numpy().astype(np.int64)),
                         head.embed[wl.shape.vocab - wl.shape.n_bins + bins[:, :A - 1]]], axis=1)
    R = S + A - 1
    allowed = np.tril(np.ones((R, R), dtype=bool))
    rows = np.arange(S - 1, S - 1 + A)
    xs = {"bf16": x0.copy(), "exact": x0.copy(), "a": x0.astype(F32), "b": x0.astype(F32)}
    dec = {"a": Fp32Decoder(wl.shape.n_heads, wl.shape.rms_eps, wl.shape.rope_theta, 1),
           "b": Fp32Decoder(wl.shape.n_heads, wl.shape.rms_eps, wl.shape.rope_theta, k_chunks_b)}
    out = []
    for l in range(n_layers):
        l32 = {k: v.float().numpy() for k, v in model.layer(l).items()}
        l64 = {k: v.astype(np.float64) for k, v in l32.items()}
        for m in ("bf16", "exact"):
            w1 = dataclasses.replace(head, layer=lambda _l, l64=l64: l64)
            xs[m], _ = vo.decoder_layers(cfgs[m], w1, xs[m], np.arange(R), allowed, None)
        for v in ("a", "b"):
            xs[v] = dec[v].layer(xs[v], l32, allowed)
        rd = {k: _readout(cfgs["exact"], head, xs[k], rows, bins, S) for k in xs}
        rec = dict(depth=l + 1, ops=_stats(rd["a"], rd["bf16"]), exact=_stats(rd["a"], rd["exact"]),
                   impl=_stats(rd["a"], rd["b"]), logit_sigma=float(rd["exact"]["logits"].std()))
        out.append(rec)
        if progress:
            progress(rec)
    return out


# ------------------------------------------------------------------------------------------------ tolerances
def load_table() -> dict:
    with open(TABLE) as f:
        return json.load(f)


def _gauss_max(n: int) -> float:
    """Expected largest |x| among n standard normal draws, to leading order: sqrt(2 ln 2n), at least 3."""
    return max(3.0, math.sqrt(2.0 * math.log(2.0 * max(n, 1))))


def tolerance(depth: int, against: str, n_logits: int, n_tokens: int, margin: float = 1.5) -> dict:
    """Bounds for a bf16 model of 7B width and ``depth`` layers compared with ``against``: "ops" (the oracle that
    rounds the stored tensors), "exact" (the plain fp64 oracle) or "impl" (another bf16 evaluation of the same rows,
    e.g. rollout against recompute).  RMS bounds are ``margin`` times the table's RMS at the nearest tabulated
    depth at or above ``depth``; max bounds are the RMS bound times the expected largest of as many normal draws as the
    test compares (``n_logits`` logits, ``n_tokens`` log-probs / entropies / values).  A sampled bin may differ
    where the oracle's top-2 gap is below the bound on the difference of two logit errors."""
    table = load_table()
    rows = [r for r in table["depths"] if r["depth"] >= depth]
    row = rows[0] if rows else table["depths"][-1]
    s = row[against]
    out = dict(depth_used=row["depth"])
    for k, n in (("logits", n_logits), ("logp", n_tokens), ("ent", n_tokens), ("value", n_tokens)):
        out[k + "_rms"] = margin * s[k + "_rms"]
        out[k] = margin * s[k + "_rms"] * _gauss_max(n)
    out["near_tie"] = margin * math.sqrt(2.0) * s["logits_rms"] * _gauss_max(n_tokens)
    return out
