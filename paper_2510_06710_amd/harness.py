"""Device-buffer plumbing around the C ABI for the tests and the benchmark: uploads the seeded
synthetic model, allocates the KV buffer, workspace and outputs as torch tensors, and calls the
library.  No arithmetic of the method happens here."""
from __future__ import annotations

import torch

from . import binding as vb


class Rollout:
    """One model on one GPU plus the buffers for a (B, S, A) rollout problem."""

    def __init__(self, synth_model, max_batch: int, max_seq: int, device="cuda:0", with_value=True,
                 value_b: float = 0.0, value_dim: int = 1):
        self.shape = synth_model.shape
        self.device = torch.device(device)
        assert str(synth_model.device).startswith("cuda"), "weights must be generated on the GPU"
        self.value_dim = value_dim
        self.cfg = vb.make_config(self.shape, max_batch, max_seq, value_dim)
        layers = [synth_model.layer(l) for l in range(self.shape.n_layers)]
        self.embed = synth_model.embed()
        self.model = vb.DeviceModel(self.cfg, self.embed, synth_model.lm_head(), synth_model.final_norm(),
                                    layers, synth_model.value_w(value_dim) if with_value else None, value_b,
                                    synth_model.value_bias(value_dim) if with_value and value_dim > 1 else None)
        self._bufs = {}

    def _buf(self, name, nbytes):
        t = self._bufs.get(name)
        if t is None or t.numel() < nbytes:
            self._bufs[name] = t = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        return t

    def _value_out(self, n):
        shape = (n,) if self.value_dim == 1 else (n, self.value_dim)
        return torch.empty(*shape, dtype=torch.float32, device=self.device)

    def kv(self, B, max_pos):
        return self._buf("kv", vb.vla_kv_bytes(self.cfg, B, max_pos))

    def prefill(self, patch, ids, want_value=True, stream=None):
        B, P = patch.shape[0], patch.shape[1]
        T = ids.shape[1]
        kv = self.kv(B, self.cfg.max_seq)
        ws = self._buf("ws", vb.vla_workspace_bytes(self.cfg, vb.VLA_ENTRY_PREFILL, B, P + T, 0))
        h_last = torch.empty(B, self.shape.hidden, dtype=torch.float32, device=self.device)
        value = self._value_out(B) if want_value else None
        vb.vla_prefill(self.model.handle, kv, ws, patch, ids, B, P, T, h_last, value, stream)
        return h_last, value

    def decode(self, h_last, S, A, mode=0, slot_embed=None, temperature=1.0, gumbel=None,
               want_logits=True, stream=None):
        B = h_last.shape[0]
        kv = self.kv(B, self.cfg.max_seq)
        ws = self._buf("ws", vb.vla_workspace_bytes(self.cfg, vb.VLA_ENTRY_DECODE, B, S, A))
        dev = self.device
        bins = torch.empty(B, A, dtype=torch.int32, device=dev)
        logp = torch.empty(B, A, dtype=torch.float32, device=dev)
        ent = torch.empty(B, A, dtype=torch.float32, device=dev)
        logits = torch.empty(B, A, 256, dtype=torch.float32, device=dev) if want_logits else None
        vb.vla_decode_actions(self.model.handle, kv, ws, h_last, B, S, A, mode, slot_embed, temperature,
                              gumbel, bins, logp, ent, logits, stream)
        return bins, logp, ent, logits

    def recompute(self, patch, ids, bins, A, mode=0, slot_embed=None, temperature=1.0, want_value=True,
                  want_logits=True, stream=None):
        N, P = patch.shape[0], patch.shape[1]
        T = ids.shape[1]
        ws = self._buf("ws", vb.vla_workspace_bytes(self.cfg, vb.VLA_ENTRY_RECOMPUTE, N, P + T, A))
        dev = self.device
        logp = torch.empty(N, A, dtype=torch.float32, device=dev)
        ent = torch.empty(N, A, dtype=torch.float32, device=dev)
        value = self._value_out(N) if want_value else None
        logits = torch.empty(N, A, 256, dtype=torch.float32, device=dev) if want_logits else None
        vb.vla_logprob_recompute(self.model.handle, ws, patch, ids, bins, N, P, T, A, mode, slot_embed,
                                 temperature, logp, ent, value, logits, stream)
        return logp, ent, value, logits
