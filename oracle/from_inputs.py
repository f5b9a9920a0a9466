"""Adapter: hand the seeded synthetic model (``vla_inputs.SynthModel``) to the oracle as fp64
arrays.  Test infrastructure only, like the rest of ``oracle/``; no arithmetic of the method
lives here, only dtype conversion (bf16 -> fp64 is exact)."""
from __future__ import annotations

import numpy as np

from .vla_oracle import OracleConfig, OracleWeights


def to_f64(t) -> np.ndarray:
    return t.detach().to("cpu").float().numpy().astype(np.float64)


def oracle_config(shape, operand_dtype: str = "exact") -> OracleConfig:
    return OracleConfig(n_layers=shape.n_layers, hidden=shape.hidden, n_heads=shape.n_heads,
                        ffn=shape.ffn, vocab=shape.vocab, n_bins=shape.n_bins,
                        rms_eps=shape.rms_eps, rope_theta=shape.rope_theta,
                        operand_dtype=operand_dtype)


def oracle_weights(model, value_b: float, cache_layers: bool = True, value_dim: int = 1) -> OracleWeights:
    """``model`` is a CPU ``SynthModel``.  Layers are generated on first use; with
    ``cache_layers`` they are kept in their storage dtype and widened per call, so a 7B-shape
    model costs 13 GB of host memory instead of 52 GB."""
    cache = {}

    def layer(l):
        if cache_layers:
            if l not in cache:
                cache[l] = model.layer(l)
            src = cache[l]
        else:
            src = model.layer(l)
        return {k: to_f64(v) for k, v in src.items()}

    return OracleWeights(embed=to_f64(model.embed()), lm_head=to_f64(model.lm_head()),
                         final_norm=to_f64(model.final_norm()), layer=layer,
                         value_w=to_f64(model.value_w(value_dim)),
                         value_b=value_b if value_dim == 1 else value_b + to_f64(model.value_bias(value_dim)))
