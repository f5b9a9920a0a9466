"""Seeded synthetic inputs for the VLA rollout / log-prob-recompute hot path.

This module only *generates data*: model shapes, random-init weights, observation
prefixes, stored action bins and Gumbel noise.  It holds none of the method's
arithmetic (no norm, no attention, no softmax) and is the one piece shared by the CPU
oracle's tests and the HIP path's tests and benchmark, so both always see bit-identical
inputs.

Everything is counter based: element ``i`` of the logical tensor ``tag`` under ``seed``
depends only on ``(seed, tag, i)``, so any row slice of a 7B-shape tensor can be
regenerated on its own (the oracle checks a few environments of a 256-env batch without
ever holding the rest), and the same integer code runs on the CPU and on the GPU through
``torch`` integer ops with identical results.

Distributions (the recipe stands in for trained OpenVLA / OpenVLA-OFT checkpoints and
for ManiSkill / LIBERO / RoboTwin observations, none of which are available):

* ``normal``: N(mean, sigma) discretised to 65,536 equiprobable quantile midpoints.  The
  table is computed once on the host in fp64, scaled, rounded to the storage dtype and
  only then gathered, so host and device values agree bit for bit.
* ``randint``: uniform integers (token ids, stored bins).
* ``gumbel``: g = -ln(-ln u), u = (r + 0.5) / 2**24 with r a 24-bit integer, so u lies
  strictly inside (0, 1); evaluated on the host in fp64, stored as fp32.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, Optional, Sequence

import numpy as np
import torch

# ----------------------------------------------------------------------------------------
# shapes
# ----------------------------------------------------------------------------------------


@dataclasses.dataclass(frozen=True)
class ModelShape:
    """Decoder shape.  ``dtype`` is the storage type of weights, KV cache and GEMM
    operands ("f32" or "bf16")."""

    n_layers: int
    hidden: int
    n_heads: int
    ffn: int
    vocab: int
    n_bins: int = 256
    dtype: str = "bf16"
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0

    @property
    def head_dim(self) -> int:
        return self.hidden // self.n_heads

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def layer_params(self) -> int:
        return 4 * self.hidden * self.hidden + 3 * self.hidden * self.ffn


@dataclasses.dataclass(frozen=True)
class Workload:
    """One synthetic workload: a model shape plus batch / prefix / action sizes."""

    name: str
    shape: ModelShape
    batch: int          # parallel environments (or stored rollouts for recompute)
    n_patches: int      # P vision-patch embeddings per observation
    n_instr: int        # T instruction token ids per observation
    n_action: int       # A action tokens per environment step
    mode: int = 0       # 0 autoregressive, 1 parallel action chunk
    temperature: float = 1.0
    kind: str = "rollout"   # "rollout" or "recompute"

    @property
    def prefix(self) -> int:
        return self.n_patches + self.n_instr


TINY = ModelShape(n_layers=2, hidden=256, n_heads=4, ffn=688, vocab=1024, dtype="f32")
SHAPE_7B = ModelShape(n_layers=32, hidden=4096, n_heads=32, ffn=11008, vocab=32000, dtype="bf16")

WORKLOADS: Dict[str, Workload] = {
    # tiny fp32 decoder, 8 envs, 48 patches + 16 instruction ids, 7 action tokens
    "cfg1_tiny_fp32": Workload("cfg1_tiny_fp32", TINY, 8, 48, 16, 7),
    # OpenVLA shape, 64 envs, 256 patches + 32 instruction ids, 7 autoregressive tokens
    "cfg2_7b_b64": Workload("cfg2_7b_b64", SHAPE_7B, 64, 256, 32, 7),
    # same shape at the ManiSkill-scale batch of 256 parallel envs
    "cfg3_7b_b256": Workload("cfg3_7b_b256", SHAPE_7B, 256, 256, 32, 7),
    # OFT-style parallel chunk: 8 steps x 7 dims = 56 slots in one forward, 128 envs
    "cfg4_7b_oft_b128": Workload("cfg4_7b_oft_b128", SHAPE_7B, 128, 256, 32, 56, mode=1),
    # PPO/GRPO log-prob recompute over 512 stored rollouts
    "cfg5_7b_recompute_n512": Workload("cfg5_7b_recompute_n512", SHAPE_7B, 512, 256, 32, 7,
                                       kind="recompute"),
}

# ----------------------------------------------------------------------------------------
# counter-based integer stream
# ----------------------------------------------------------------------------------------

_M1 = -7046029254386353131   # 0x9E3779B97F4A7C15 as a signed 64-bit integer
_M2 = -4658895280553007687   # 0xBF58476D1CE4E5B9
_M3 = -7723592293110705685   # 0x94D049BB133111EB
_CHUNK = 1 << 22


def _wrap64(v: int) -> int:
    v &= (1 << 64) - 1
    return v - (1 << 64) if v >= (1 << 63) else v


def _mix_int(v: int) -> int:
    """The 64-bit finaliser below on one Python integer (used for stream bases)."""
    m = (1 << 64) - 1
    v = (v * (_M1 & m)) & m
    v = ((v ^ (v >> 30)) * (_M2 & m)) & m
    v = ((v ^ (v >> 27)) * (_M3 & m)) & m
    return v ^ (v >> 31)


def _mix_(z: torch.Tensor) -> torch.Tensor:
    """In-place 64-bit avalanche finaliser on an int64 tensor (two's-complement wraparound
    multiplies; the arithmetic right shifts are masked back to logical shifts)."""
    z.mul_(_M1)
    t = z >> 30
    t.bitwise_and_((1 << 34) - 1)
    z.bitwise_xor_(t)
    z.mul_(_M2)
    t = z >> 27
    t.bitwise_and_((1 << 37) - 1)
    z.bitwise_xor_(t)
    z.mul_(_M3)
    t = z >> 31
    t.bitwise_and_((1 << 33) - 1)
    z.bitwise_xor_(t)
    return z


def _stream_base(seed: int, tag: int) -> int:
    return _wrap64(_mix_int(_mix_int(seed + 1) ^ (tag * 0x632BE59BD9B4E019 + 0x1234567)))


def _bits(seed: int, tag: int, start: int, count: int, device) -> torch.Tensor:
    """64 hashed bits for logical elements [start, start+count) of stream (seed, tag)."""
    base = _stream_base(seed, tag)
    out = torch.empty(count, dtype=torch.int64, device=device)
    for s in range(0, count, _CHUNK):
        e = min(count, s + _CHUNK)
        z = torch.arange(start + s, start + e, dtype=torch.int64, device=device)
        z.add_(base)
        out[s:e] = _mix_(z)
    return out


def _slice_of(shape: Sequence[int], row0: int, rows: Optional[int]):
    shape = tuple(int(v) for v in shape)
    inner = int(np.prod(shape[1:])) if len(shape) > 1 else 1
    rows = shape[0] - row0 if rows is None else rows
    assert 0 <= row0 and row0 + rows <= shape[0]
    return (rows,) + shape[1:], row0 * inner, rows * inner


_QUANTILES: Optional[np.ndarray] = None


def _quantiles() -> np.ndarray:
    """Standard-normal quantile midpoints, 65,536 levels, fp64."""
    global _QUANTILES
    if _QUANTILES is None:
        from scipy.special import ndtri

        _QUANTILES = ndtri((np.arange(65536, dtype=np.float64) + 0.5) / 65536.0)
    return _QUANTILES


def normal(seed: int, tag: int, shape: Sequence[int], *, sigma: float, mean: float = 0.0,
           dtype: torch.dtype = torch.float32, device="cpu", row0: int = 0,
           rows: Optional[int] = None) -> torch.Tensor:
    """Rows [row0, row0+rows) of the logical tensor ``shape`` ~ N(mean, sigma), rounded to
    ``dtype`` (round to nearest even for bf16)."""
    out_shape, start, count = _slice_of(shape, row0, rows)
    table = torch.from_numpy(mean + sigma * _quantiles()).to(torch.float32).to(dtype).to(device)
    out = torch.empty(count, dtype=dtype, device=device)
    base = _stream_base(seed, tag)
    for s in range(0, count, _CHUNK):
        e = min(count, s + _CHUNK)
        z = torch.arange(start + s, start + e, dtype=torch.int64, device=device)
        z.add_(base)
        _mix_(z).bitwise_and_(0xFFFF)
        out[s:e] = table[z]
    return out.view(out_shape)


def randint(seed: int, tag: int, shape: Sequence[int], n: int, *, device="cpu", row0: int = 0,
            rows: Optional[int] = None) -> torch.Tensor:
    """Uniform int32 in [0, n)."""
    out_shape, start, count = _slice_of(shape, row0, rows)
    z = _bits(seed, tag, start, count, device)
    z.bitwise_and_(0x7FFFFFFF)
    return (z % n).to(torch.int32).view(out_shape)


def gumbel(seed: int, tag: int, shape: Sequence[int], *, device="cpu", row0: int = 0,
           rows: Optional[int] = None) -> torch.Tensor:
    """Standard Gumbel noise as fp32; always evaluated on the host, then moved."""
    out_shape, start, count = _slice_of(shape, row0, rows)
    r = _bits(seed, tag, start, count, "cpu").bitwise_and_(0xFFFFFF).numpy().astype(np.float64)
    u = (r + 0.5) / float(1 << 24)
    g = -np.log(-np.log(u))
    return torch.from_numpy(g.astype(np.float32)).view(out_shape).to(device)


# ----------------------------------------------------------------------------------------
# tensors of the synthetic model and workloads
# ----------------------------------------------------------------------------------------

TAG_EMBED, TAG_LM_HEAD, TAG_FINAL_NORM, TAG_VALUE_W, TAG_SLOT_EMBED = 1, 2, 3, 4, 5
TAG_PATCH, TAG_IDS, TAG_BINS, TAG_GUMBEL = 6, 7, 8, 9
_LAYER_TENSORS = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")
VALUE_BIAS = 0.25
WEIGHT_SIGMA = 0.02


def layer_tensor_shape(shape: ModelShape, name: str):
    H, F = shape.hidden, shape.ffn
    return {"attn_norm": (H,), "ffn_norm": (H,), "wq": (H, H), "wk": (H, H), "wv": (H, H),
            "wo": (H, H), "w_gate": (F, H), "w_up": (F, H), "w_down": (H, F)}[name]


class SynthModel:
    """Random-init weights of a ``ModelShape``: matrices N(0, 0.02) stored row-major
    [out, in]; RMSNorm gains 1 + N(0, 0.02) (gains of pure N(0, 0.02) would collapse the
    activations, gains of exactly one would not exercise the multiply); the value head is
    a length-H vector N(0, 0.02) plus the scalar bias ``VALUE_BIAS``.  Matrices use the
    shape's storage dtype; gains and the value head stay fp32."""

    def __init__(self, shape: ModelShape, seed: int = 0, device="cpu"):
        self.shape, self.seed, self.device = shape, seed, device

    def _mat(self, tag, shp):
        return normal(self.seed, tag, shp, sigma=WEIGHT_SIGMA, dtype=self.shape.torch_dtype,
                      device=self.device)

    def _gain(self, tag, n):
        return normal(self.seed, tag, (n,), sigma=WEIGHT_SIGMA, mean=1.0, dtype=torch.float32,
                      device=self.device)

    def embed(self):
        return self._mat(TAG_EMBED, (self.shape.vocab, self.shape.hidden))

    def lm_head(self):
        return self._mat(TAG_LM_HEAD, (self.shape.vocab, self.shape.hidden))

    def final_norm(self):
        return self._gain(TAG_FINAL_NORM, self.shape.hidden)

    def value_w(self, dim: int = 1):
        """Value head weights: [H] for the scalar head, [dim, H] for the action-level head (row 0 of
        the latter equals the scalar head)."""
        shp = (self.shape.hidden,) if dim == 1 else (dim, self.shape.hidden)
        return normal(self.seed, TAG_VALUE_W, shp, sigma=WEIGHT_SIGMA, dtype=torch.float32, device=self.device)

    def value_bias(self, dim: int):
        """Per-output bias of the action-level value head, added to ``VALUE_BIAS``: 0.125 * c."""
        return (0.125 * torch.arange(dim, dtype=torch.float32)).to(self.device)

    def slot_embed(self, n_action: int):
        return self._mat(TAG_SLOT_EMBED, (n_action, self.shape.hidden))

    def layer(self, l: int) -> Dict[str, torch.Tensor]:
        out = {}
        for k, name in enumerate(_LAYER_TENSORS):
            tag = 100 + 16 * l + k
            shp = layer_tensor_shape(self.shape, name)
            out[name] = self._gain(tag, shp[0]) if name.endswith("norm") else self._mat(tag, shp)
        return out


def observation(wl: Workload, seed: int = 0, *, device="cpu", env0: int = 0,
                envs: Optional[int] = None):
    """Observation prefixes of environments [env0, env0+envs): patch embeddings
    [envs, P, H] ~ N(0, 1) in the storage dtype and instruction ids [envs, T] uniform in
    [0, vocab - n_bins) (never an action-bin id)."""
    s = wl.shape
    patch = normal(seed, TAG_PATCH, (wl.batch, wl.n_patches, s.hidden), sigma=1.0,
                   dtype=s.torch_dtype, device=device, row0=env0, rows=envs)
    ids = randint(seed, TAG_IDS, (wl.batch, wl.n_instr), s.vocab - s.n_bins, device=device,
                  row0=env0, rows=envs)
    return patch, ids


def stored_bins(wl: Workload, seed: int = 0, *, device="cpu", env0: int = 0,
                envs: Optional[int] = None) -> torch.Tensor:
    """Stored rollout actions for the recompute workload: bins uniform in [0, n_bins)."""
    return randint(seed, TAG_BINS, (wl.batch, wl.n_action), wl.shape.n_bins, device=device,
                   row0=env0, rows=envs)


def gumbel_noise(wl: Workload, seed: int = 0, *, device="cpu", env0: int = 0,
                 envs: Optional[int] = None) -> torch.Tensor:
    """Gumbel noise [envs, A, n_bins] shared by the oracle and the HIP sampler."""
    return gumbel(seed, TAG_GUMBEL, (wl.batch, wl.n_action, wl.shape.n_bins), device=device,
                  row0=env0, rows=envs)


def scaled(wl: Workload, **kw) -> Workload:
    """A copy of a workload with some fields replaced (smaller batch, fewer layers ...)."""
    shape_kw = {k: kw.pop(k) for k in list(kw) if k in ModelShape.__dataclass_fields__}
    shape = dataclasses.replace(wl.shape, **shape_kw) if shape_kw else wl.shape
    return dataclasses.replace(wl, shape=shape, **kw)


__all__ = ["ModelShape", "Workload", "WORKLOADS", "TINY", "SHAPE_7B", "SynthModel", "normal",
           "randint", "gumbel", "observation", "stored_bins", "gumbel_noise", "scaled",
           "VALUE_BIAS", "WEIGHT_SIGMA", "layer_tensor_shape"]
