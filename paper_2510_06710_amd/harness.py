"""Device-buffer plumbing around the C ABI for the tests and the benchmark: uploads the seeded
synthetic model, allocates the KV buffer, workspace and outputs as torch tensors, and calls the
library.  No arithmetic of the method happens here."""
from __future__ import annotations

import torch

from . import binding as vb


class Rollout:
    """One model on one GPU plus the buffers for a (B, S, A) rollout problem."""

    def __init__(self, synth_model, max_batch: int, max_seq: int, device="cuda:0", with_value=True,
                 value_b: float = 0.0, value_dim: int = 1, prepack: bool = True):
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
        # repacked projection weights for the multi-row forwards (bf16 models with tile-aligned widths)
        self.packed = None
        nbytes = vb.vla_prepack_bytes(self.cfg)
        if nbytes and prepack:
            self.packed = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
            vb.vla_prepack(self.model.handle, self.packed)
            torch.cuda.synchronize(self.device)

    def _buf(self, name, nbytes):
        t = self._bufs.get(name)
        if t is None or t.numel() < nbytes:
            self._bufs[name] = t = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        return t

    def _value_out(self, n):
        shape = (n,) if self.value_dim == 1 else (n, self.value_dim)
        return torch.empty(*shape, dtype=torch.float32, device=self.device)

    def kv(self, B, max_pos, lane=0):
        return self._buf(f"kv{lane}", vb.vla_kv_bytes(self.cfg, B, max_pos))

    # `lane` selects a private KV buffer and workspace, so that calls on different streams can overlap.
    def prefill(self, patch, ids, want_value=True, stream=None, lane=0):
        B, P = patch.shape[0], patch.shape[1]
        T = ids.shape[1]
        kv = self.kv(B, self.cfg.max_seq, lane)
        ws = self._buf(f"ws{lane}", vb.vla_workspace_bytes(self.cfg, vb.VLA_ENTRY_PREFILL, B, P + T, 0))
        h_last = torch.empty(B, self.shape.hidden, dtype=torch.float32, device=self.device)
        value = self._value_out(B) if want_value else None
        vb.vla_prefill(self.model.handle, kv, ws, patch, ids, B, P, T, h_last, value, stream)
        return h_last, value

    def decode(self, h_last, S, A, mode=0, slot_embed=None, temperature=1.0, gumbel=None,
               want_logits=True, stream=None, lane=0):
        B = h_last.shape[0]
        kv = self.kv(B, self.cfg.max_seq, lane)
        ws = self._buf(f"ws{lane}", vb.vla_workspace_bytes(self.cfg, vb.VLA_ENTRY_DECODE, B, S, A))
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
        ws = self._buf("ws0", vb.vla_workspace_bytes(self.cfg, vb.VLA_ENTRY_RECOMPUTE, N, P + T, A))
        dev = self.device
        logp = torch.empty(N, A, dtype=torch.float32, device=dev)
        ent = torch.empty(N, A, dtype=torch.float32, device=dev)
        value = self._value_out(N) if want_value else None
        logits = torch.empty(N, A, 256, dtype=torch.float32, device=dev) if want_logits else None
        vb.vla_logprob_recompute(self.model.handle, ws, patch, ids, bins, N, P, T, A, mode, slot_embed,
                                 temperature, logp, ent, value, logits, stream)
        return logp, ent, value, logits


    def backward(self, patch, ids, bins, coef, A, lora, rank, scale, mode=0, slot_embed=None, temperature=1.0, stream=None,
                 keep_activations=False):
        """LoRA gradients of sum(coef * logp): lora[l][p] = (a, b) device tensors in the storage dtype.  Returns
        (grads, logp) with grads[l][p] = (da, db) fp32 device tensors.  keep_activations: hand the library the larger
        workspace with which it keeps every layer's activations instead of running each layer a second time."""
        N, P = patch.shape[0], patch.shape[1]
        T = ids.shape[1]
        size = vb.vla_backward_keep_workspace_bytes if keep_activations else vb.vla_backward_workspace_bytes
        ws = self._buf("ws_bw", size(self.cfg, N, P + T, A, rank))
        grads = [{p: (torch.empty(f[0].shape, dtype=torch.float32, device=self.device),
                      torch.empty(f[1].shape, dtype=torch.float32, device=self.device)) for p, f in layer.items()}
                 for layer in lora]
        logp = torch.empty(N, A, dtype=torch.float32, device=self.device)
        vb.vla_logprob_backward(self.model.handle, ws, patch, ids, bins, coef, N, P, T, A, mode, slot_embed, temperature,
                                rank, scale, keep_activations, lora, grads, logp, stream)
        return grads, logp


class PipelinedRollout:
    """Rollout epoch with fine-grained pipelining on one GPU (section IV-A, hybrid mode, figure with
    k = 2): the environments are split into k sub-batches; while the simulator steps one sub-batch, the
    policy generates the actions of the next.  Each sub-batch has its own stream, KV buffer and
    workspace.  The simulator is the caller's: ``sim_step(j, t, bins_host)`` is called on a worker thread
    once the actions of sub-batch j at step t are on the host, and returns when that sub-batch's next
    observation exists (here the observation tensors stay the same; what the simulator computes is
    outside this library).  k = 1 is the collocated schedule: generation and simulation alternate."""

    def __init__(self, run: Rollout, k: int):
        import concurrent.futures
        self.run, self.k = run, k
        self.streams = [torch.cuda.Stream(device=run.device) for _ in range(k)]      # default priority
        self.pool = concurrent.futures.ThreadPoolExecutor(max_workers=k)

    def epoch(self, obs, m_chunks: int, S: int, A: int, sim_step, mode=0, slot_embed=None, temperature=1.0,
              gumbel=None):
        """obs[j] = (patch, ids) of sub-batch j (device tensors); gumbel[j] its noise or None.
        Returns (outputs, log): outputs[t][j] = (bins, logp, entropy) device tensors, log a list of
        (event, j, t, time) host timestamps in seconds from the start."""
        import time
        torch.cuda.synchronize(self.run.device)      # inputs made on other streams are complete
        t0 = time.perf_counter()
        log = []
        gen_done = None                              # the Generation side takes one sub-batch at a time
        pending = [None] * self.k
        outputs = []
        host_bins = [torch.empty(obs[j][0].shape[0], A, dtype=torch.int32).pin_memory() for j in range(self.k)]

        def simulate(j, t, ready):
            ready.synchronize()                      # the actions of (j, t) are on the host
            log.append(("actions", j, t, time.perf_counter() - t0))
            sim_step(j, t, host_bins[j])
            log.append(("observation", j, t, time.perf_counter() - t0))

        for t in range(m_chunks):
            row = []
            for j in range(self.k):
                if pending[j] is not None:
                    pending[j].result()              # o_t of sub-batch j exists
                patch, ids = obs[j]
                st = self.streams[j]
                log.append(("generate", j, t, time.perf_counter() - t0))
                with torch.cuda.stream(st):
                    if gen_done is not None:
                        st.wait_event(gen_done)
                    h_last, _ = self.run.prefill(patch, ids, want_value=False, stream=st, lane=j)
                    bins, logp, ent, _ = self.run.decode(h_last, S, A, mode, slot_embed, temperature,
                                                         None if gumbel is None else gumbel[j], want_logits=False,
                                                         stream=st, lane=j)
                    host_bins[j].copy_(bins, non_blocking=True)
                    ready = torch.cuda.Event()
                    ready.record(st)
                    gen_done = ready
                row.append((bins, logp, ent))
                pending[j] = self.pool.submit(simulate, j, t, ready)
            outputs.append(row)
        for f in pending:
            if f is not None:
                f.result()
        return outputs, log, time.perf_counter() - t0

    def close(self):
        self.pool.shutdown(wait=True)
