"""CPU oracle for the batched VLA policy rollout step and the log-prob recompute.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the HIP library is
checked against.  Only the tests, the smoke check and the benchmark's CPU-baseline leg may
import it; the product path never does.  It shares no code with the HIP path.

What it computes (all arithmetic in fp64 on whatever values it is handed; for the bf16
workloads the caller hands it weights and patch embeddings already rounded to bf16):

* the generation step of the RL pipeline (paper section III-C: the policy infers an action
  chunk from the current observation, a_t ~ pi_theta(. | o_t) of section III-A), for a
  Llama-style pre-norm decoder whose action tokens are restricted to the last ``n_bins``
  vocabulary ids, one token per action dimension (section III-B);
* token-level log-probabilities pi(d_{t,i,j} | o_t, d_{t,i,:j-1}) (section IV-C.1) of the
  sampled / stored tokens and the entropy of each token distribution;
* the log-probability recompute under the current parameters that the importance ratio
  rho = pi_theta / pi_theta_old of the PPO / GRPO objectives needs (appendix I-B, I-C),
  with the scalar value head attached to the language model (section IV-C.2, critic
  design).

Precision: the paper never states one.  The benchmark's bf16 workloads fix what is *stored* in
bf16 -- weights, patch embeddings, the KV cache and the operands of the projections -- so the oracle
has two modes (``OracleConfig.operand_dtype``): "exact" keeps every intermediate in fp64 (only the
inputs are bf16 valued); "bf16" also rounds those stored tensors to bf16 while all arithmetic stays
fp64.  The fp32 workload uses "exact".

The method is exact, so the oracle is the textbook definition written out; a key/value
cache is used between the prefill and the action tokens (the three entry points mirror the
library's), and the tests pin that against a from-scratch, loop-only recomputation.

Readings taken where the paper is silent (decoder details come from the benchmark
configuration, not the paper): multi-head attention without biases; patches first, then
instruction tokens, causal throughout; RMSNorm eps 1e-5; rotary with half-split pairing
(i, i + d/2), base 10000, absolute positions from 0; softmax, log-prob, entropy and
sampling over the ``n_bins`` slice only, all at temperature tau; Gumbel-max with the lowest
index winning ties, the argmax taken in fp32 (the precision the kernel decides it in);
action token 1 is read from the last prefix row and token j+1 from the row of token j;
the value head reads the final-norm output of the last prefix row.

Pins (tests/test_oracle_*.py): scalar-loop brute force without a cache and with an explicit
boolean mask; a PyTorch-CPU library composition of the same model; closed forms (zero head,
identity layers, single key); rotary invariants; rho = 1 between rollout and recompute;
Monte-Carlo frequencies of the Gumbel-max sampler; batch permutation.  The bf16 rounding
path of the HIP kernels has no closed form: "parity unpinned" beyond the stated tolerance.
"""
from __future__ import annotations

import dataclasses
from typing import Callable, Dict, List, Optional, Tuple

import numpy as np

F64 = np.float64


@dataclasses.dataclass
class OracleConfig:
    n_layers: int
    hidden: int
    n_heads: int
    ffn: int
    vocab: int
    n_bins: int = 256
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0
    # "exact": every intermediate stays fp64 (the plain definition).  "bf16": the tensors that the
    # bf16 workloads *store* -- the operands of every projection (norm outputs, attention output,
    # SwiGLU output) and the rotated q and the k, v that go to the KV cache -- are rounded to bf16
    # (round to nearest even) exactly like the bf16 weights and patch embeddings already are;
    # all arithmetic on them is still exact fp64.
    operand_dtype: str = "exact"

    @property
    def head_dim(self) -> int:
        return self.hidden // self.n_heads


def round_bf16(x: np.ndarray) -> np.ndarray:
    """Round to the nearest bfloat16 (ties to even), returned as fp64."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(F64).reshape(np.shape(x))


def stored(cfg: "OracleConfig", x: np.ndarray) -> np.ndarray:
    """A tensor as the workload stores it: unchanged, or rounded to bf16."""
    return round_bf16(x) if cfg.operand_dtype == "bf16" else x


@dataclasses.dataclass
class OracleWeights:
    """fp64 arrays, matrices row-major [out, in].  ``layer(l)`` returns the nine tensors of
    decoder layer l (attn_norm, wq, wk, wv, wo, ffn_norm, w_gate, w_up, w_down); it is a
    callable so that 7B-shape weights can be produced one layer at a time."""

    embed: np.ndarray        # [V, H]
    lm_head: np.ndarray      # [V, H]
    final_norm: np.ndarray   # [H]
    layer: Callable[[int], Dict[str, np.ndarray]]
    value_w: Optional[np.ndarray] = None   # [H] (chunk-level scalar) or [C, H] (action-level)
    value_b: object = 0.0                  # scalar, or [C]


KV = List[Tuple[np.ndarray, np.ndarray]]   # per layer (K, V), each [n, n_heads, rows, d]

# ----------------------------------------------------------------------------------------
# building blocks (textbook definitions)
# ----------------------------------------------------------------------------------------


def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """n_i = x_i / sqrt(mean_i(x_i^2) + eps) * g_i over the last axis."""
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps) * gain


def rotary(u: np.ndarray, positions: np.ndarray, theta: float) -> np.ndarray:
    """Rotate the pairs (u_i, u_{i+d/2}) of each head vector by the angle
    position * theta^(-2i/d).  u: [..., rows, d]; positions: [rows]."""
    d = u.shape[-1]
    half = d // 2
    i = np.arange(half, dtype=F64)
    phi = positions.astype(F64)[:, None] * theta ** (-2.0 * i / d)      # [rows, d/2]
    c, s = np.cos(phi), np.sin(phi)
    a, b = u[..., :half], u[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def silu(t: np.ndarray) -> np.ndarray:
    return t / (1.0 + np.exp(-t))


def split_heads(x: np.ndarray, n_heads: int) -> np.ndarray:
    """[n, rows, H] -> [n, n_heads, rows, d]."""
    n, r, h = x.shape
    return x.reshape(n, r, n_heads, h // n_heads).transpose(0, 2, 1, 3)


def merge_heads(x: np.ndarray) -> np.ndarray:
    """[n, n_heads, rows, d] -> [n, rows, H]."""
    n, nh, r, d = x.shape
    return x.transpose(0, 2, 1, 3).reshape(n, r, nh * d)


def attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, allowed: np.ndarray) -> np.ndarray:
    """softmax(q k^T / sqrt(d)) v over the allowed keys of each query row.
    q: [n, nh, R, d]; k, v: [n, nh, Rk, d]; allowed: bool [R, Rk]."""
    d = q.shape[-1]
    s = np.einsum("nhrd,nhkd->nhrk", q, k) / np.sqrt(float(d))
    s = np.where(allowed[None, None], s, -np.inf)
    s = s - s.max(axis=-1, keepdims=True)
    p = np.exp(s)
    p = p / p.sum(axis=-1, keepdims=True)
    return np.einsum("nhrk,nhkd->nhrd", p, v)


def decoder_layers(cfg: OracleConfig, w: OracleWeights, x: np.ndarray, positions: np.ndarray,
                   allowed: np.ndarray, past: Optional[KV]) -> Tuple[np.ndarray, KV]:
    """All decoder layers over the rows x [n, R, H] at absolute ``positions`` [R].  Keys are
    the cached rows of ``past`` (if any) followed by the current rows; ``allowed`` is bool
    [R, R_past + R].  Returns the residual stream after the last layer and the K, V of all
    rows seen so far."""
    kv: KV = []
    for l in range(cfg.n_layers):
        lw = w.layer(l)
        n = stored(cfg, rmsnorm(x, lw["attn_norm"], cfg.rms_eps))
        q = stored(cfg, rotary(split_heads(n @ lw["wq"].T, cfg.n_heads), positions, cfg.rope_theta))
        k = stored(cfg, rotary(split_heads(n @ lw["wk"].T, cfg.n_heads), positions, cfg.rope_theta))
        v = stored(cfg, split_heads(n @ lw["wv"].T, cfg.n_heads))
        if past is not None:
            k = np.concatenate([past[l][0], k], axis=2)
            v = np.concatenate([past[l][1], v], axis=2)
        kv.append((k, v))
        x = x + stored(cfg, merge_heads(attention(q, k, v, allowed))) @ lw["wo"].T
        n2 = stored(cfg, rmsnorm(x, lw["ffn_norm"], cfg.rms_eps))
        x = x + stored(cfg, silu(n2 @ lw["w_gate"].T) * (n2 @ lw["w_up"].T)) @ lw["w_down"].T
    return x, kv


def bin_logits(cfg: OracleConfig, w: OracleWeights, h: np.ndarray) -> np.ndarray:
    """Logits over the action bins only: z_k = h . lm_head[V - n_bins + k]."""
    return h @ w.lm_head[cfg.vocab - cfg.n_bins:].T


def token_distribution(z: np.ndarray, temperature: float):
    """Log-probabilities and entropy (nats) of softmax(z / tau) over the last axis."""
    y = z / temperature
    m = y.max(axis=-1, keepdims=True)
    lse = m + np.log(np.exp(y - m).sum(axis=-1, keepdims=True))
    logp = y - lse
    ent = -(np.exp(logp) * logp).sum(axis=-1)
    return y, logp, ent


def gumbel_argmax(y: np.ndarray, g: Optional[np.ndarray]) -> np.ndarray:
    """argmax_k (y_k + g_k), lowest k on ties, decided in fp32; g None means greedy."""
    t = y.astype(np.float32)
    if g is not None:
        t = t + g.astype(np.float32)
    return np.argmax(t, axis=-1).astype(np.int32)


def embed_prefix(w: OracleWeights, patch: np.ndarray, ids: np.ndarray) -> np.ndarray:
    """x_p = patch[p] for p < P, x_{P+t} = E[ids[t]]."""
    return np.concatenate([patch.astype(F64), w.embed[ids]], axis=1)


def chunk_mask(S: int, A: int) -> np.ndarray:
    """Parallel-chunk mask over S prefix rows followed by A slot rows: prefix rows are
    causal, slot rows see every prefix row and every slot row."""
    m = np.tril(np.ones((S + A, S + A), dtype=bool))
    m[S:, :] = True
    return m


def value_head(cfg: OracleConfig, w: OracleWeights, h_last: np.ndarray) -> Optional[np.ndarray]:
    """Linear value head on the final-norm output of the last prefix row (section IV-C.2): one scalar
    per observation (chunk-level, V: S -> R) or one value per atomic action (action-level, S -> R^C)."""
    if w.value_w is None:
        return None
    return h_last @ np.asarray(w.value_w).T + w.value_b


# ----------------------------------------------------------------------------------------
# the three entry points
# ----------------------------------------------------------------------------------------


def ovla_prefill(cfg: OracleConfig, w: OracleWeights, patch: np.ndarray, ids: np.ndarray):
    """Causal forward over the observation prefix (patch [B, P, H], ids [B, T]).
    Returns (kv, h_last [B, H], value [B] or None): the K, V of every prefix row, the
    final-norm output of the last prefix row and the value-head output on it."""
    x = embed_prefix(w, patch, ids)
    S = x.shape[1]
    pos = np.arange(S)
    x, kv = decoder_layers(cfg, w, x, pos, np.tril(np.ones((S, S), dtype=bool)), None)
    h_last = rmsnorm(x[:, S - 1], w.final_norm, cfg.rms_eps)
    return kv, h_last, value_head(cfg, w, h_last)


def ovla_decode_actions(cfg: OracleConfig, w: OracleWeights, kv: KV, h_last: np.ndarray, S: int,
                        A: int, mode: int = 0, slot_embed: Optional[np.ndarray] = None,
                        temperature: float = 1.0, gumbel: Optional[np.ndarray] = None):
    """Decode A action tokens per environment after a prefill.

    mode 0 (autoregressive): token 1 from ``h_last``; for j = 1..A-1 the sampled token id
    V - n_bins + bin_j is embedded at position S + j - 1 and run through the decoder against
    the cache; token j+1 is read from that row.  The last token is never fed back.
    mode 1 (parallel chunk): one pass over A slot rows whose inputs are ``slot_embed`` [A, H]
    at positions S..S+A-1; slot rows see all prefix rows and all slot rows; slot s is read
    from its own row.

    gumbel: [B, A, n_bins] or None (greedy).  Returns bins int32 [B, A], logp [B, A],
    entropy [B, A], logits [B, A, n_bins] (untempered), kv (extended)."""
    B = h_last.shape[0]
    K = cfg.n_bins
    bins = np.zeros((B, A), dtype=np.int32)
    logp = np.zeros((B, A), dtype=F64)
    ent = np.zeros((B, A), dtype=F64)
    logits = np.zeros((B, A, K), dtype=F64)

    def emit(j, h):
        z = bin_logits(cfg, w, h)
        y, lp, e = token_distribution(z, temperature)
        b = gumbel_argmax(y, None if gumbel is None else gumbel[:, j])
        bins[:, j], ent[:, j], logits[:, j] = b, e, z
        logp[:, j] = lp[np.arange(B), b]
        return b

    if mode == 0:
        h = h_last
        for j in range(A):
            b = emit(j, h)
            if j == A - 1:
                break
            x = w.embed[cfg.vocab - K + b][:, None, :]                # [B, 1, H]
            pos = np.array([S + j])
            x, kv = decoder_layers(cfg, w, x, pos, np.ones((1, S + j + 1), dtype=bool), kv)
            h = rmsnorm(x[:, 0], w.final_norm, cfg.rms_eps)
    else:
        x = np.broadcast_to(slot_embed.astype(F64)[None], (B, A, cfg.hidden)).copy()
        pos = np.arange(S, S + A)
        x, kv = decoder_layers(cfg, w, x, pos, np.ones((A, S + A), dtype=bool), kv)
        h = rmsnorm(x, w.final_norm, cfg.rms_eps)
        for s in range(A):
            emit(s, h[:, s])
    return bins, logp, ent, logits, kv


def ovla_logprob_recompute(cfg: OracleConfig, w: OracleWeights, patch: np.ndarray,
                           ids: np.ndarray, bins: np.ndarray, A: int, mode: int = 0,
                           slot_embed: Optional[np.ndarray] = None, temperature: float = 1.0):
    """Teacher-forced forward over stored rollouts: log-prob of each stored bin under the
    current weights, entropy of each token distribution, value on the last prefix row.

    mode 0: rows = prefix followed by the stored action tokens 1..A-1 (the last token is
    only a target), causal; token j is read from row S + j - 2 (1-based j).
    mode 1: rows = prefix followed by the A slot inputs under the parallel-chunk mask.
    Returns logp [N, A], entropy [N, A], value [N] or None, logits [N, A, n_bins]."""
    N = patch.shape[0]
    K = cfg.n_bins
    x = embed_prefix(w, patch, ids)
    S = x.shape[1]
    if mode == 0:
        if A > 1:
            x = np.concatenate([x, w.embed[cfg.vocab - K + bins[:, :A - 1]]], axis=1)
        R = S + A - 1
        allowed = np.tril(np.ones((R, R), dtype=bool))
        rows = np.arange(S - 1, S - 1 + A)
    else:
        x = np.concatenate([x, np.broadcast_to(slot_embed.astype(F64)[None], (N, A, cfg.hidden))],
                           axis=1)
        R = S + A
        allowed = chunk_mask(S, A)
        rows = np.arange(S, S + A)
    x, _ = decoder_layers(cfg, w, x, np.arange(R), allowed, None)
    h = rmsnorm(x[:, rows], w.final_norm, cfg.rms_eps)                 # [N, A, H]
    z = bin_logits(cfg, w, h)
    _, lp, ent = token_distribution(z, temperature)
    logp = np.take_along_axis(lp, bins[:, :A, None].astype(np.int64), axis=-1)[..., 0]
    h_last = rmsnorm(x[:, S - 1], w.final_norm, cfg.rms_eps)
    return logp, ent, value_head(cfg, w, h_last), z
