"""ctypes binding of libvla.so: the same entry points as include/vla.h, argument marshalling only.

Every step of the path runs in the library's HIP kernels; PyTorch appears here solely as the owner
of device memory (``tensor.data_ptr()``) and of the stream the work is enqueued on.  If the library
has not been built this module raises on first use -- there is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libvla.so")

VLA_OK, VLA_EINVAL, VLA_ESHAPE, VLA_EWORKSPACE, VLA_EDTYPE, VLA_EHIP = 0, -1, -2, -3, -4, -5
VLA_DTYPE_F32, VLA_DTYPE_BF16 = 0, 1
VLA_MODE_AR, VLA_MODE_PARALLEL_CHUNK = 0, 1
VLA_ENTRY_PREFILL, VLA_ENTRY_DECODE, VLA_ENTRY_RECOMPUTE = 0, 1, 2
VLA_N_BINS = 256


class vla_config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("hidden", C.c_int32), ("n_heads", C.c_int32),
                ("ffn", C.c_int32), ("vocab", C.c_int32), ("n_bins", C.c_int32),
                ("dtype", C.c_int32), ("rms_eps", C.c_float), ("rope_theta", C.c_float),
                ("max_batch", C.c_int32), ("max_seq", C.c_int32), ("value_dim", C.c_int32)]


class vla_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm",
                                          "w_gate", "w_up", "w_down")]


class vla_weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p),
                ("value_w", C.c_void_p), ("value_b", C.c_float),
                ("layers", C.POINTER(vla_layer_weights)), ("value_bias", C.c_void_p)]


class vla_lora_factor(C.Structure):
    _fields_ = [("a", C.c_void_p), ("b", C.c_void_p)]


class vla_lora_grad(C.Structure):
    _fields_ = [("da", C.c_void_p), ("db", C.c_void_p)]


LORA_PROJECTIONS = ("q", "k", "v", "o", "gate", "up", "down")


class vla_lora_layer(C.Structure):
    _fields_ = [(n, vla_lora_factor) for n in LORA_PROJECTIONS]


class vla_lora_layer_grads(C.Structure):
    _fields_ = [(n, vla_lora_grad) for n in LORA_PROJECTIONS]


class vla_placement(C.Structure):
    _fields_ = [("k", C.c_int32), ("n_gen", C.c_int32), ("n_sim", C.c_int32), ("time", C.c_double)]


class VlaError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"libvla error {code}: {message}")
        self.code = code


_lib = None


def lib() -> C.CDLL:
    """Load libvla.so (built in-tree by ``paper_2510_06710_amd.build``); fails loudly if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(f"{_LIB_PATH} is not built; run `python -m paper_2510_06710_amd.build`")
        # The device pointers and streams this library is handed belong to PyTorch's HIP runtime, so that runtime must
        # be the one in the process: loaded first, the library's own dependency on libamdhip64 resolves to it (loaded
        # the other way round, the system copy comes in first and the kernels then find no device).
        import torch  # noqa: F401
        L = C.CDLL(_LIB_PATH)
        vp, i32, f32, sz = C.c_void_p, C.c_int, C.c_float, C.c_size_t
        L.vla_version.restype = C.c_int
        L.vla_last_error.restype = C.c_char_p
        L.vla_create.argtypes = [C.POINTER(vla_config), C.POINTER(vla_weights), C.POINTER(vp)]
        L.vla_destroy.argtypes = [vp]
        L.vla_prepack_bytes.argtypes = [C.POINTER(vla_config)]
        L.vla_prepack_bytes.restype = sz
        L.vla_prepack.argtypes = [vp, vp, sz, vp]
        L.vla_kv_bytes.argtypes = [C.POINTER(vla_config), i32, i32]
        L.vla_kv_bytes.restype = sz
        L.vla_workspace_bytes.argtypes = [C.POINTER(vla_config), i32, i32, i32, i32]
        L.vla_workspace_bytes.restype = sz
        L.vla_prefill.argtypes = [vp, vp, vp, sz, vp, vp, i32, i32, i32, vp, vp, vp]
        L.vla_decode_actions.argtypes = [vp, vp, vp, sz, vp, i32, i32, i32, i32, vp, f32, vp, vp, vp, vp, vp, vp]
        L.vla_logprob_recompute.argtypes = [vp, vp, sz, vp, vp, vp, i32, i32, i32, i32, i32, vp, f32,
                                            vp, vp, vp, vp, vp]
        L.vla_backward_workspace_bytes.argtypes = [C.POINTER(vla_config), i32, i32, i32, i32]
        L.vla_backward_workspace_bytes.restype = sz
        L.vla_backward_keep_workspace_bytes.argtypes = [C.POINTER(vla_config), i32, i32, i32, i32]
        L.vla_backward_keep_workspace_bytes.restype = sz
        L.vla_logprob_backward.argtypes = [vp, vp, sz, vp, vp, vp, vp, i32, i32, i32, i32, i32, vp, f32, i32, f32, i32,
                                           C.POINTER(vla_lora_layer), C.POINTER(vla_lora_layer_grads), vp, vp]
        L.vla_debug_force_generic.argtypes = [i32]
        L.vla_profile_enable.argtypes = [i32]
        L.vla_profile_report.argtypes = [C.c_char_p, sz]
        L.vla_calibration_copy.argtypes = [vp, vp, sz, vp]
        L.vla_gae.argtypes = [vp, vp, vp, i32, i32, f32, f32, vp, vp, vp]
        L.vla_grpo_advantage.argtypes = [vp, i32, i32, vp, vp, vp]
        L.vla_policy_objective_workspace_bytes.argtypes = [i32]
        L.vla_policy_objective_workspace_bytes.restype = sz
        L.vla_policy_objective.argtypes = [vp, vp, vp, i32, vp, i32, i32, f32, f32, i32, vp, sz, vp, vp, vp, vp]
        L.vla_policy_objective_noalloc_max_traj.restype = C.c_int
        L.vla_policy_objective_noalloc.argtypes = [vp, vp, vp, i32, vp, i32, i32, f32, f32, i32, vp, vp, vp, vp]
        L.vla_logp_aggregate.argtypes = [vp, sz, i32, vp, vp]
        dp = C.POINTER(C.c_double)
        L.vla_pipeline_time.argtypes = [C.c_double, C.c_double, i32, i32, dp]
        L.vla_profile_lookup.argtypes = [dp, i32, C.c_double, dp]
        L.vla_auto_placement.argtypes = [dp, dp, i32, i32, i32, i32, C.POINTER(vla_placement),
                                         C.POINTER(vla_placement), i32, C.POINTER(C.c_int)]
        _lib = L
    return _lib


def vla_last_error() -> str:
    return lib().vla_last_error().decode()


def _check(rc: int) -> None:
    if rc != VLA_OK:
        raise VlaError(rc, vla_last_error())


def _ptr(t) -> Optional[int]:
    """Device (or host) address of a tensor, None for None."""
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def vla_version() -> int:
    return lib().vla_version()


def vla_kv_bytes(cfg: vla_config, B: int, max_pos: int) -> int:
    n = lib().vla_kv_bytes(C.byref(cfg), B, max_pos)
    if n == 0:
        raise VlaError(VLA_EINVAL, vla_last_error())
    return n


def vla_workspace_bytes(cfg: vla_config, entry: int, B: int, S: int, A: int) -> int:
    n = lib().vla_workspace_bytes(C.byref(cfg), entry, B, S, A)
    if n == 0:
        raise VlaError(VLA_EINVAL, vla_last_error())
    return n


def vla_create(cfg: vla_config, weights: vla_weights) -> int:
    out = C.c_void_p()
    _check(lib().vla_create(C.byref(cfg), C.byref(weights), C.byref(out)))
    return out.value


def vla_destroy(model: int) -> None:
    _check(lib().vla_destroy(model))


def vla_prepack_bytes(cfg: vla_config) -> int:
    return lib().vla_prepack_bytes(C.byref(cfg))


def vla_prepack(model: int, buffer, stream=None) -> None:
    nbytes = 0 if buffer is None else buffer.numel() * buffer.element_size()
    _check(lib().vla_prepack(model, _ptr(buffer), nbytes, _stream(stream)))


def vla_prefill(model, kv, ws, patch, ids, B, P, T, h_last, value=None, stream=None) -> None:
    _check(lib().vla_prefill(model, _ptr(kv), _ptr(ws), ws.numel() * ws.element_size(), _ptr(patch),
                             _ptr(ids), B, P, T, _ptr(h_last), _ptr(value), _stream(stream)))


def vla_decode_actions(model, kv, ws, h_last, B, S, A, mode, slot_embed, temperature, gumbel, bins,
                       logp, entropy, logits=None, stream=None) -> None:
    _check(lib().vla_decode_actions(model, _ptr(kv), _ptr(ws), ws.numel() * ws.element_size(),
                                    _ptr(h_last), B, S, A, mode, _ptr(slot_embed), temperature,
                                    _ptr(gumbel), _ptr(bins), _ptr(logp), _ptr(entropy), _ptr(logits),
                                    _stream(stream)))


def vla_logprob_recompute(model, ws, patch, ids, bins, N, P, T, A, mode, slot_embed, temperature,
                          logp, entropy, value=None, logits=None, stream=None) -> None:
    _check(lib().vla_logprob_recompute(model, _ptr(ws), ws.numel() * ws.element_size(), _ptr(patch),
                                       _ptr(ids), _ptr(bins), N, P, T, A, mode, _ptr(slot_embed),
                                       temperature, _ptr(logp), _ptr(entropy), _ptr(value),
                                       _ptr(logits), _stream(stream)))


def vla_backward_workspace_bytes(cfg: vla_config, N: int, S: int, A: int, rank: int) -> int:
    n = lib().vla_backward_workspace_bytes(C.byref(cfg), N, S, A, rank)
    if n == 0:
        raise VlaError(VLA_EINVAL, vla_last_error())
    return n


def vla_backward_keep_workspace_bytes(cfg: vla_config, N: int, S: int, A: int, rank: int) -> int:
    n = lib().vla_backward_keep_workspace_bytes(C.byref(cfg), N, S, A, rank)
    if n == 0:
        raise VlaError(VLA_EINVAL, vla_last_error())
    return n


def vla_logprob_backward(model, ws, patch, ids, bins, coef, N, P, T, A, mode, slot_embed, temperature, rank, scale,
                         keep_activations, lora, grads, logp=None, stream=None) -> None:
    """lora[l][p] = (a, b) and grads[l][p] = (da, db): device tensors per layer and projection name."""
    n_layers = len(lora)
    la = (vla_lora_layer * n_layers)()
    ga = (vla_lora_layer_grads * n_layers)()
    for l in range(n_layers):
        for p in LORA_PROJECTIONS:
            f, g = getattr(la[l], p), getattr(ga[l], p)
            f.a, f.b = lora[l][p][0].data_ptr(), lora[l][p][1].data_ptr()
            g.da, g.db = grads[l][p][0].data_ptr(), grads[l][p][1].data_ptr()
    _check(lib().vla_logprob_backward(model, _ptr(ws), ws.numel() * ws.element_size(), _ptr(patch), _ptr(ids), _ptr(bins),
                                      _ptr(coef), N, P, T, A, mode, _ptr(slot_embed), temperature, rank, scale, int(bool(keep_activations)), la, ga,
                                      _ptr(logp), _stream(stream)))


def vla_debug_force_generic(mask: int) -> None:
    _check(lib().vla_debug_force_generic(mask))


def vla_calibration_copy(dst, src, nbytes: int, stream=None) -> None:
    _check(lib().vla_calibration_copy(_ptr(dst), _ptr(src), nbytes, _stream(stream)))


def vla_gae(rewards, values, dones, n, T, gamma, lam, adv, returns=None, stream=None) -> None:
    _check(lib().vla_gae(_ptr(rewards), _ptr(values), _ptr(dones), n, T, gamma, lam, _ptr(adv), _ptr(returns),
                         _stream(stream)))


def vla_grpo_advantage(total_reward, n_groups, G, adv, keep=None, stream=None) -> None:
    _check(lib().vla_grpo_advantage(_ptr(total_reward), n_groups, G, _ptr(adv), _ptr(keep), _stream(stream)))


def vla_policy_objective_workspace_bytes(n_traj: int) -> int:
    return lib().vla_policy_objective_workspace_bytes(n_traj)


def vla_policy_objective(logp_new, logp_old, adv, adv_per_step, mask, n_traj, T, clip_low, clip_high,
                         per_trajectory, ws, objective, per_step=None, clip_frac=None, stream=None) -> None:
    _check(lib().vla_policy_objective(_ptr(logp_new), _ptr(logp_old), _ptr(adv), int(adv_per_step), _ptr(mask),
                                      n_traj, T, clip_low, clip_high, int(per_trajectory), _ptr(ws),
                                      ws.numel() * ws.element_size(), _ptr(objective), _ptr(per_step),
                                      _ptr(clip_frac), _stream(stream)))


def vla_policy_objective_noalloc_max_traj() -> int:
    return lib().vla_policy_objective_noalloc_max_traj()


def vla_policy_objective_noalloc(logp_new, logp_old, adv, adv_per_step, mask, n_traj, T, clip_low, clip_high,
                                 per_trajectory, objective, per_step=None, clip_frac=None, stream=None) -> None:
    _check(lib().vla_policy_objective_noalloc(_ptr(logp_new), _ptr(logp_old), _ptr(adv), int(adv_per_step),
                                              _ptr(mask), n_traj, T, clip_low, clip_high, int(per_trajectory),
                                              _ptr(objective), _ptr(per_step), _ptr(clip_frac), _stream(stream)))


def vla_logp_aggregate(logp, n_out, inner, out, stream=None) -> None:
    _check(lib().vla_logp_aggregate(_ptr(logp), n_out, inner, _ptr(out), _stream(stream)))


def _doubles(values):
    return (C.c_double * len(values))(*[float(v) for v in values])


def vla_pipeline_time(t_gen: float, t_sim: float, k: int, m_chunks: int) -> float:
    out = C.c_double()
    _check(lib().vla_pipeline_time(t_gen, t_sim, k, m_chunks, C.byref(out)))
    return out.value


def vla_profile_lookup(profile, batch: float) -> float:
    out = C.c_double()
    _check(lib().vla_profile_lookup(_doubles(profile), len(profile), batch, C.byref(out)))
    return out.value


def vla_auto_placement(t_gen, t_sim, n_envs: int, n_gpus: int, m_chunks: int):
    """Returns (best, candidates), each candidate a (k, n_gen, n_sim, time) tuple."""
    if len(t_gen) != len(t_sim):
        raise ValueError("t_gen and t_sim must cover the same batch sizes")
    best = vla_placement()
    cap = n_gpus
    arr = (vla_placement * cap)()
    n = C.c_int()
    _check(lib().vla_auto_placement(_doubles(t_gen), _doubles(t_sim), len(t_gen), n_envs, n_gpus, m_chunks,
                                    C.byref(best), arr, cap, C.byref(n)))
    tup = lambda c: (c.k, c.n_gen, c.n_sim, c.time)
    return tup(best), [tup(arr[i]) for i in range(min(n.value, cap))]


def make_config(shape, max_batch: int, max_seq: int, value_dim: int = 1) -> vla_config:
    """``shape`` is any object with the decoder fields (n_layers, hidden, ..., dtype "f32"/"bf16")."""
    return vla_config(shape.n_layers, shape.hidden, shape.n_heads, shape.ffn, shape.vocab, shape.n_bins,
                      VLA_DTYPE_F32 if shape.dtype == "f32" else VLA_DTYPE_BF16, shape.rms_eps,
                      shape.rope_theta, max_batch, max_seq, value_dim)


class DeviceModel:
    """Keeps device weight tensors alive and owns the library's model handle.  ``layers`` is a list
    of dicts of device tensors with the nine per-layer names of ``vla_layer_weights``."""

    def __init__(self, cfg: vla_config, embed, lm_head, final_norm, layers, value_w=None, value_b=0.0,
                 value_bias=None):
        self.cfg = cfg
        self._keep = (embed, lm_head, final_norm, layers, value_w, value_bias)
        arr = (vla_layer_weights * len(layers))()
        for a, d in zip(arr, layers):
            for name, _ in vla_layer_weights._fields_:
                setattr(a, name, d[name].data_ptr())
        self._layers = arr
        w = vla_weights(embed.data_ptr(), lm_head.data_ptr(), final_norm.data_ptr(), _ptr(value_w),
                        float(value_b), arr, _ptr(value_bias))
        self.handle = vla_create(cfg, w)

    def close(self):
        if self.handle:
            vla_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
