"""GPU parity of vla_logprob_backward (LoRA gradients of sum(coef * logp), section IV-B.2 / appendix I-B, I-C)
against oracle/backward_oracle.py on the same seeded inputs.

The synthetic model's weights play the role of the effective (merged) weights; the LoRA factors A, B are seeded
normal tensors in the storage dtype (the gradient formulas need nothing else).  fp32 storage: every gradient tensor
within 2e-4 of its largest entry.  bf16 storage: the GEMM operands of the backward (activations and gradients) are
rounded to bf16 (2^-9 relative per element, averaged down by the sums over rows), so each gradient tensor is compared
with the oracle that rounds the forward's stored tensors (straight-through): relative RMS error at most 1e-2 and
largest deviation at most 2e-2 of the tensor's largest entry (observed: 4e-3 and 5e-3).

The log-probs the pass returns come from the recompute's own forward kernels.  Here they are taken at seeded random
bins, not at sampled ones: such a bin can sit far in the tail (log-prob below -9 where a flat distribution gives
-ln 256 = -5.5), and a bf16 logit error grows with the distance z_j - logsumexp(z) = logp_j it is measured over, so
the bf16 bound of 1e-2 is scaled by max(1, |logp| / ln 256) per token."""
import numpy as np
import pytest
import torch

import vla_inputs as vi
from oracle import backward_oracle as bo
from oracle.from_inputs import oracle_config, oracle_weights, to_f64
from parity import GpuCase

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _lora(shape, rank, seed, sigma=0.05):
    """Per layer and projection (A [rank, in], B [out, rank]) as CPU tensors in the storage dtype."""
    g = torch.Generator().manual_seed(seed)
    dims = {"q": (shape.hidden, shape.hidden), "k": (shape.hidden, shape.hidden), "v": (shape.hidden, shape.hidden),
            "o": (shape.hidden, shape.hidden), "gate": (shape.ffn, shape.hidden), "up": (shape.ffn, shape.hidden),
            "down": (shape.hidden, shape.ffn)}
    out = []
    for _ in range(shape.n_layers):
        out.append({p: ((sigma * torch.randn(rank, i, generator=g)).to(shape.torch_dtype),
                        (sigma * torch.randn(o, rank, generator=g)).to(shape.torch_dtype)) for p, (o, i) in dims.items()})
    return out


def _run(wl, seed, rank, scale, n=None, max_batch=None, keep=False):
    n = wl.batch if n is None else n
    case = GpuCase(wl, seed, max_batch=max_batch or wl.batch)
    lora = _lora(wl.shape, rank, seed + 50)
    patch, ids = vi.observation(wl, seed, device=DEV, envs=n)
    bins = vi.stored_bins(wl, seed, envs=n)
    coef = torch.randn(n, wl.n_action, generator=torch.Generator().manual_seed(seed + 7))
    dev_lora = [{p: (a.to(DEV), b.to(DEV)) for p, (a, b) in layer.items()} for layer in lora]
    slot = case.synth.slot_embed(wl.n_action) if wl.mode == 1 else None
    grads, logp = case.run.backward(patch, ids, bins.to(DEV), coef.to(DEV), wl.n_action, dev_lora, rank, scale, wl.mode, slot,
                                    wl.temperature, keep_activations=keep)
    torch.cuda.synchronize()
    return case, lora, bins.numpy(), coef.numpy().astype(np.float64), grads, logp.cpu().numpy()


def _oracle(wl, seed, lora, bins, coef, n, scale, operand_dtype="exact"):
    model = vi.SynthModel(wl.shape, seed)
    cfg = oracle_config(wl.shape, operand_dtype)
    w = oracle_weights(model, vi.VALUE_BIAS)
    patch, ids = vi.observation(wl, seed, envs=n)
    lo = [{p: (to_f64(a), to_f64(b)) for p, (a, b) in layer.items()} for layer in lora]
    slot = to_f64(model.slot_embed(wl.n_action)) if wl.mode == 1 else None
    return bo.ovla_logprob_backward(cfg, w, lo, scale, to_f64(patch), ids.numpy().astype(np.int64), bins, coef, wl.n_action,
                                    wl.mode, slot, wl.temperature)


def _assert_logp_bf16(logp, ref_logp):
    tol = 1e-2 * np.maximum(1.0, np.abs(ref_logp) / np.log(256.0))
    assert np.all(np.abs(logp - ref_logp) < tol), float(np.max(np.abs(logp - ref_logp) / tol))


def _compare(grads, ref, rel_max, rel_rms=None):
    worst = dict(max=0.0, rms=0.0)
    for l, layer in enumerate(ref):
        for p in bo.PROJ:
            for i in (0, 1):
                got, want = grads[l][p][i].cpu().numpy().astype(np.float64), layer[p][i]
                assert got.shape == want.shape and np.isfinite(got).all(), (l, p, i)
                e_max = np.max(np.abs(got - want)) / max(np.max(np.abs(want)), 1e-30)
                e_rms = np.sqrt(np.mean((got - want) ** 2)) / max(np.sqrt(np.mean(want ** 2)), 1e-30)
                worst["max"], worst["rms"] = max(worst["max"], e_max), max(worst["rms"], e_rms)
                assert e_max <= rel_max, (l, p, "dA" if i == 0 else "dB", e_max, e_rms)
                if rel_rms is not None:
                    assert e_rms <= rel_rms, (l, p, "dA" if i == 0 else "dB", e_max, e_rms)
    return worst


@pytest.mark.parametrize("keep", [False, True])
@pytest.mark.parametrize("mode,tau", [(0, 1.0), (0, 1.6), (1, 1.0)])
def test_tiny_fp32_lora_gradients(mode, tau, keep):
    """keep: the first pass keeps every layer's activations (larger workspace) instead of running each layer twice."""
    wl = vi.scaled(vi.WORKLOADS["cfg1_tiny_fp32"], batch=4, mode=mode, temperature=tau)
    _, lora, bins, coef, grads, logp = _run(wl, 3, rank=8, scale=0.5, keep=keep)
    ref, ref_logp = _oracle(wl, 3, lora, bins, coef, 4, 0.5)
    assert np.max(np.abs(logp - ref_logp)) < 1e-4
    print(f"\n[parity] backward tiny fp32 mode={mode} tau={tau}: {_compare(grads, ref, 2e-4)}", flush=True)


@pytest.mark.parametrize("B,P,T,A", [(1, 0, 1, 1), (2, 0, 3, 2), (1, 4, 0, 3), (3, 5, 2, 1)])
def test_degenerate_sizes_lora_gradients(B, P, T, A):
    """One rollout, no patches or no instruction tokens, a single action token (one row: softmax over one key)."""
    wl = vi.scaled(vi.WORKLOADS["cfg1_tiny_fp32"], batch=B, n_patches=P, n_instr=T, n_action=A)
    _, lora, bins, coef, grads, logp = _run(wl, 8, rank=3, scale=0.7)
    ref, ref_logp = _oracle(wl, 8, lora, bins, coef, B, 0.7)
    assert np.max(np.abs(logp - ref_logp)) < 1e-4
    _compare(grads, ref, 2e-4)


@pytest.mark.parametrize("keep", [False, True])
def test_micro_batches_sum_to_the_whole_and_runs_are_bit_identical(keep):
    wl = vi.scaled(vi.WORKLOADS["cfg1_tiny_fp32"], batch=5)
    _, lora, bins, coef, g_all, _ = _run(wl, 4, rank=4, scale=1.0, keep=keep)
    _, _, _, _, g_again, _ = _run(wl, 4, rank=4, scale=1.0, keep=keep)
    _, _, _, _, g_mb, _ = _run(wl, 4, rank=4, scale=1.0, max_batch=2, keep=keep)   # passes of 2, 2 and 1 rollouts
    for l in range(wl.shape.n_layers):
        for p in bo.PROJ:
            for i in (0, 1):
                a, b, c = (g[l][p][i].cpu().numpy() for g in (g_all, g_again, g_mb))
                assert np.array_equal(a, b)
                assert np.max(np.abs(a - c)) <= 2e-5 * max(np.max(np.abs(a)), 1e-30)


@pytest.mark.parametrize("keep", [False, True])
@pytest.mark.parametrize("mode", [0, 1])
def test_aligned_bf16_lora_gradients_mfma_gemms(mode, keep):
    """hidden 256 / ffn 512 / head_dim 128: the forward and input-gradient GEMMs, the attention matrices and the LoRA
    products take the MFMA kernels; autoregressive rows and the parallel chunk (slot rows see every key)."""
    wl = vi.Workload("aligned_bw", vi.ModelShape(n_layers=2, hidden=256, n_heads=2, ffn=512, vocab=640, dtype="bf16"),
                     batch=5, n_patches=40, n_instr=9, n_action=4, mode=mode)
    _, lora, bins, coef, grads, logp = _run(wl, 5, rank=16, scale=0.25, keep=keep)
    ref, ref_logp = _oracle(wl, 5, lora, bins, coef, 5, 0.25, operand_dtype="bf16")
    _assert_logp_bf16(logp, ref_logp)
    print(f"\n[parity] backward aligned bf16 mode {mode}: {_compare(grads, ref, 2e-2, 1e-2)}", flush=True)


@pytest.mark.parametrize("keep", [False, True])
def test_one_layer_7b_width_lora_gradients(keep):
    wl = vi.scaled(vi.WORKLOADS["cfg5_7b_recompute_n512"], n_layers=1, batch=2)
    print(f"\n[7b] backward: 1 layer of 7B width, 2 rollouts x 294 rows, rank 32, keep={keep}", flush=True)
    _, lora, bins, coef, grads, logp = _run(wl, 6, rank=32, scale=0.5, keep=keep)
    ref, ref_logp = _oracle(wl, 6, lora, bins, coef, 2, 0.5, operand_dtype="bf16")
    _assert_logp_bf16(logp, ref_logp)
    print(f"[parity] backward 1-layer 7B width: {_compare(grads, ref, 2e-2, 1e-2)}", flush=True)
