"""The seeded input generator: slices regenerate exactly, distributions are as documented."""
import math

import numpy as np
import torch

import vla_inputs as vi


def test_row_slices_regenerate_exactly():
    full = vi.normal(3, 42, (10, 7, 5), sigma=1.0, dtype=torch.bfloat16)
    part = vi.normal(3, 42, (10, 7, 5), sigma=1.0, dtype=torch.bfloat16, row0=4, rows=3)
    assert torch.equal(full[4:7], part)
    ids = vi.randint(3, 43, (10, 6), 768)
    assert torch.equal(ids[8:], vi.randint(3, 43, (10, 6), 768, row0=8))
    g = vi.gumbel(3, 44, (6, 7, 256))
    assert torch.equal(g[2:5], vi.gumbel(3, 44, (6, 7, 256), row0=2, rows=3))


def test_streams_differ_by_seed_and_tag():
    a = vi.normal(0, 1, (1000,), sigma=1.0)
    assert not torch.equal(a, vi.normal(1, 1, (1000,), sigma=1.0))
    assert not torch.equal(a, vi.normal(0, 2, (1000,), sigma=1.0))
    assert abs(float(np.corrcoef(a.numpy(), vi.normal(0, 2, (1000,), sigma=1.0).numpy())[0, 1])) < 0.12


def test_normal_moments_and_gain_mean():
    x = vi.normal(0, 5, (400_000,), sigma=0.02).double()
    assert abs(x.mean().item()) < 2e-4 and abs(x.std().item() - 0.02) < 2e-4
    kurt = ((x / x.std()) ** 4).mean().item()
    assert abs(kurt - 3.0) < 0.05
    g = vi.normal(0, 6, (100_000,), sigma=0.02, mean=1.0).double()
    assert abs(g.mean().item() - 1.0) < 3e-4


def test_ids_and_bins_ranges_and_gumbel_moments():
    wl = vi.WORKLOADS["cfg1_tiny_fp32"]
    patch, ids = vi.observation(wl, 0)
    assert patch.shape == (8, 48, 256) and ids.shape == (8, 16) and ids.dtype == torch.int32
    assert int(ids.min()) >= 0 and int(ids.max()) < wl.shape.vocab - 256
    bins = vi.stored_bins(wl, 0)
    assert int(bins.min()) >= 0 and int(bins.max()) < 256
    g = vi.gumbel(1, 9, (200_000,)).double()
    assert torch.isfinite(g).all()
    assert abs(g.mean().item() - 0.5772156649) < 0.01           # Euler-Mascheroni
    assert abs(g.var().item() - math.pi ** 2 / 6) < 0.03


def test_bf16_values_are_exact_in_bf16():
    w = vi.SynthModel(vi.scaled(vi.WORKLOADS["cfg2_7b_b64"], n_layers=1, hidden=64, n_heads=2,
                                ffn=96, vocab=512).shape, 0).layer(0)
    assert w["wq"].dtype == torch.bfloat16 and w["attn_norm"].dtype == torch.float32
    assert torch.equal(w["wq"].float().bfloat16(), w["wq"])
    assert w["w_gate"].shape == (96, 64) and w["w_down"].shape == (64, 96)


def test_workload_table_matches_benchmark_configs():
    w = vi.WORKLOADS
    assert w["cfg3_7b_b256"].batch == 256 and w["cfg3_7b_b256"].prefix == 288
    assert w["cfg4_7b_oft_b128"].n_action == 56 and w["cfg4_7b_oft_b128"].mode == 1
    assert w["cfg5_7b_recompute_n512"].batch == 512
    assert vi.SHAPE_7B.layer_params * 32 == 6_476_005_376
