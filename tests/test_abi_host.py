"""Host-only checks of the C ABI: the library loads, exports every symbol the header declares,
and rejects bad arguments with the documented codes before touching any device."""
import ctypes as C
import os
import re

import pytest

import vla_inputs as vi
from paper_2510_06710_amd import binding as vb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_symbols():
    text = open(os.path.join(ROOT, "include", "vla.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(vla_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = vb.lib()
    names = header_symbols()
    assert {"vla_prefill", "vla_decode_actions", "vla_logprob_recompute", "vla_create", "vla_destroy",
            "vla_kv_bytes", "vla_workspace_bytes", "vla_last_error", "vla_version", "vla_profile_enable",
            "vla_profile_report", "vla_calibration_copy", "vla_gae", "vla_grpo_advantage",
            "vla_policy_objective", "vla_policy_objective_workspace_bytes", "vla_logp_aggregate",
            "vla_pipeline_time", "vla_profile_lookup", "vla_auto_placement", "vla_prepack", "vla_prepack_bytes"} <= set(names)
    for n in names:
        assert hasattr(L, n), n
    assert vb.vla_version() == 1


def fake_model(cfg):
    lw = (vb.vla_layer_weights * cfg.n_layers)()
    for a in lw:
        for name, _ in vb.vla_layer_weights._fields_:
            setattr(a, name, 0x1000)
    w = vb.vla_weights(0x1000, 0x1000, 0x1000, None, 0.0, lw, None)
    return vb.vla_create(cfg, w), lw


def test_config_validation_codes():
    good = vb.make_config(vi.TINY, 8, 80)
    h, _ = fake_model(good)
    vb.vla_destroy(h)
    for field, val, code in [("n_bins", 128, vb.VLA_ESHAPE), ("dtype", 7, vb.VLA_EDTYPE),
                             ("hidden", 250, vb.VLA_ESHAPE), ("n_layers", 0, vb.VLA_EINVAL),
                             ("vocab", 100, vb.VLA_ESHAPE), ("max_seq", 100000, vb.VLA_ESHAPE)]:
        cfg = vb.make_config(vi.TINY, 8, 80)
        setattr(cfg, field, val)
        with pytest.raises(vb.VlaError) as e:
            fake_model(cfg)
        assert e.value.code == code, field
        assert vb.vla_last_error() != ""


def test_null_weight_pointer_rejected():
    cfg = vb.make_config(vi.TINY, 8, 80)
    lw = (vb.vla_layer_weights * cfg.n_layers)()
    w = vb.vla_weights(0x1000, 0x1000, 0x1000, None, 0.0, lw, None)
    with pytest.raises(vb.VlaError) as e:
        vb.vla_create(cfg, w)
    assert e.value.code == vb.VLA_EINVAL and "layer 0" in str(e.value)


def test_rl_entry_points_reject_bad_arguments_without_a_device():
    L = vb.lib()
    p = C.c_void_p(0x1000)
    assert L.vla_gae(None, p, None, 4, 8, 0.99, 0.95, p, None, None) == vb.VLA_EINVAL
    assert L.vla_gae(p, p, None, 0, 8, 0.99, 0.95, p, None, None) == vb.VLA_EINVAL
    assert L.vla_grpo_advantage(p, 4, 0, p, None, None) == vb.VLA_EINVAL
    assert L.vla_policy_objective(p, p, p, 0, None, 4, 8, 0.2, 0.28, 1, p, 8, p, None, None, None) == vb.VLA_EWORKSPACE
    assert L.vla_policy_objective(p, p, p, 0, None, 4, 8, -0.1, 0.28, 1, p, 1 << 20, p, None, None, None) == vb.VLA_EINVAL
    assert L.vla_policy_objective_workspace_bytes(10) == 120
    assert L.vla_logp_aggregate(p, 0, 7, p, None) == vb.VLA_EINVAL


def test_size_queries():
    cfg = vb.make_config(vi.SHAPE_7B, 256, 296)
    kv = vb.vla_kv_bytes(cfg, 256, 294)
    assert kv == 2 * 32 * 256 * 4096 * 296 * 2
    assert vb.vla_workspace_bytes(cfg, vb.VLA_ENTRY_PREFILL, 256, 288, 7) > 256 * 288 * 4096 * 4
    small = vb.vla_workspace_bytes(cfg, vb.VLA_ENTRY_RECOMPUTE, 64, 288, 7)
    big = vb.vla_workspace_bytes(cfg, vb.VLA_ENTRY_RECOMPUTE, 512, 288, 7)
    capped = vb.vla_workspace_bytes(cfg, vb.VLA_ENTRY_RECOMPUTE, 4096, 288, 7)
    assert small < big == capped                 # micro-batched beyond max_batch
    with pytest.raises(vb.VlaError):
        vb.vla_kv_bytes(cfg, 257, 10)
    # one pass holds at most 97,254 rows at this shape (activation buffers below 2 GiB)
    wide = vb.make_config(vi.SHAPE_7B, 512, 296)
    assert vb.vla_workspace_bytes(wide, vb.VLA_ENTRY_PREFILL, 330, 294, 7) > 0          # 97,020 rows
    with pytest.raises(vb.VlaError, match="split the batch"):
        vb.vla_workspace_bytes(wide, vb.VLA_ENTRY_PREFILL, 331, 294, 7)                  # 97,314 rows
    # the recompute cuts its micro-batch to what fits instead: 329 rollouts of 295 rows (the longer of its two
    # modes), not 512
    assert (vb.vla_workspace_bytes(wide, vb.VLA_ENTRY_RECOMPUTE, 512, 288, 7)
            == vb.vla_workspace_bytes(wide, vb.VLA_ENTRY_RECOMPUTE, 329, 288, 7)
            > vb.vla_workspace_bytes(wide, vb.VLA_ENTRY_RECOMPUTE, 328, 288, 7))
    with pytest.raises(vb.VlaError):
        vb.vla_workspace_bytes(cfg, 9, 1, 1, 1)


def test_hot_calls_reject_bad_arguments_without_a_device():
    cfg = vb.make_config(vi.TINY, 8, 80)
    h, keep = fake_model(cfg)
    L = vb.lib()
    p = C.c_void_p(0x1000)
    big = 1 << 40
    # prefill
    assert L.vla_prefill(h, None, p, big, p, p, 8, 48, 16, p, None, None) == vb.VLA_EINVAL
    assert L.vla_prefill(h, p, p, big, p, p, 9, 48, 16, p, None, None) == vb.VLA_ESHAPE
    assert L.vla_prefill(h, p, p, big, p, p, 8, 70, 16, p, None, None) == vb.VLA_ESHAPE
    assert L.vla_prefill(h, p, p, 16, p, p, 8, 48, 16, p, None, None) == vb.VLA_EWORKSPACE
    assert L.vla_prefill(h, p, p, big, p, p, 8, 0, 0, p, None, None) == vb.VLA_EINVAL
    assert L.vla_prefill(h, p, p, big, p, p, 8, 48, 16, p, p, None) == vb.VLA_EINVAL   # no value head
    # decode
    args = lambda **k: [h, p, p, k.get("ws", big), p, k.get("B", 8), k.get("S", 64), k.get("A", 7), k.get("mode", 0),
                        k.get("slot", None), k.get("tau", 1.0), None, p, p, p, None, None]
    assert L.vla_decode_actions(*args(tau=0.0)) == vb.VLA_EINVAL
    assert L.vla_decode_actions(*args(mode=3)) == vb.VLA_EINVAL
    assert L.vla_decode_actions(*args(mode=1)) == vb.VLA_EINVAL          # slot_embed missing
    assert L.vla_decode_actions(*args(S=75)) == vb.VLA_ESHAPE            # 75 + 7 - 1 > 80
    assert L.vla_decode_actions(*args(ws=8)) == vb.VLA_EWORKSPACE
    assert L.vla_decode_actions(*args(A=0)) == vb.VLA_EINVAL
    # recompute
    r = lambda **k: [h, p, k.get("ws", big), p, p, k.get("bins", p), k.get("N", 4), 48, 16, k.get("A", 7),
                     k.get("mode", 0), None, 1.0, p, p, None, None, None]
    assert L.vla_logprob_recompute(*r(bins=None)) == vb.VLA_EINVAL
    assert L.vla_logprob_recompute(*r(A=30)) == vb.VLA_ESHAPE
    assert L.vla_logprob_recompute(*r(ws=100)) == vb.VLA_EWORKSPACE
    assert L.vla_logprob_recompute(*r(mode=1)) == vb.VLA_EINVAL
    assert "slot_embed" in vb.vla_last_error()
    vb.vla_destroy(h)


def test_backward_rejects_bad_arguments_without_a_device():
    cfg = vb.make_config(vi.TINY, 8, 80)
    h, keep = fake_model(cfg)
    L = vb.lib()
    p = C.c_void_p(0x1000)
    big = 1 << 40
    n_layers = cfg.n_layers
    lora = (vb.vla_lora_layer * n_layers)()
    grads = (vb.vla_lora_layer_grads * n_layers)()
    for l in range(n_layers):
        for name in vb.LORA_PROJECTIONS:
            f, g = getattr(lora[l], name), getattr(grads[l], name)
            f.a = f.b = g.da = g.db = 0x1000
    b = lambda **k: [h, p, k.get("ws", big), p, p, k.get("bins", p), k.get("coef", p), k.get("N", 4), 48, 16, k.get("A", 7),
                     k.get("mode", 0), None, k.get("tau", 1.0), k.get("rank", 8), 0.5, k.get("keep", 0), k.get("lora", lora), grads, None, None]
    assert L.vla_logprob_backward(*b(coef=None)) == vb.VLA_EINVAL
    assert L.vla_logprob_backward(*b(lora=None)) == vb.VLA_EINVAL
    assert L.vla_logprob_backward(*b(tau=0.0)) == vb.VLA_EINVAL
    assert L.vla_logprob_backward(*b(rank=0)) == vb.VLA_EINVAL
    assert L.vla_logprob_backward(*b(mode=1)) == vb.VLA_EINVAL           # slot_embed missing
    assert L.vla_logprob_backward(*b(A=30)) == vb.VLA_ESHAPE             # 64 + 30 - 1 rows > max_seq 80
    assert L.vla_logprob_backward(*b(rank=100)) == vb.VLA_ESHAPE         # three stacked factors exceed 256 rows
    assert L.vla_logprob_backward(*b(ws=100)) == vb.VLA_EWORKSPACE
    small, large = vb.vla_backward_workspace_bytes(cfg, 4, 64, 7, 8), vb.vla_backward_keep_workspace_bytes(cfg, 4, 64, 7, 8)
    # (the size queries cover the longer of the two modes' rows, so only clearly smaller buffers are certain to fail)
    assert L.vla_logprob_backward(*b(ws=small // 2)) == vb.VLA_EWORKSPACE
    assert L.vla_logprob_backward(*b(ws=large // 2, keep=1)) == vb.VLA_EWORKSPACE
    lora[1].gate.b = None
    assert L.vla_logprob_backward(*b()) == vb.VLA_EINVAL and "layer 1" in vb.vla_last_error()
    assert vb.vla_backward_workspace_bytes(cfg, 4, 64, 7, 8) > 4 * 70 * 256 * 4 * cfg.n_layers
    with pytest.raises(vb.VlaError):
        vb.vla_backward_workspace_bytes(cfg, 4, 64, 7, 0)
    assert L.vla_debug_force_generic(32) == vb.VLA_EINVAL and L.vla_debug_force_generic(0) == vb.VLA_OK
    vb.vla_destroy(h)
