"""Pins for the CPU oracle: each test checks oracle/vla_oracle.py against something other
than itself -- a scalar-loop recomputation without any cache, a PyTorch-CPU library
composition, closed forms, invariants, Monte-Carlo frequencies."""
import math

import numpy as np
import pytest
import torch

import vla_inputs as vi
from oracle import vla_oracle as vo
from oracle.from_inputs import oracle_config, oracle_weights, to_f64

LN256 = math.log(256.0)


# ----------------------------------------------------------------------------------------
# helpers
# ----------------------------------------------------------------------------------------

def small_shape(**kw):
    base = dict(n_layers=2, hidden=16, n_heads=2, ffn=24, vocab=272, dtype="f32")
    base.update(kw)
    return vi.ModelShape(**base)


def small_workload(B=2, P=3, T=2, A=3, mode=0, **kw):
    return vi.Workload("small", small_shape(**kw), B, P, T, A, mode=mode)


def setup(wl, seed=0, sigma_boost=None):
    model = vi.SynthModel(wl.shape, seed)
    w = oracle_weights(model, vi.VALUE_BIAS)
    if sigma_boost:   # larger weights make attention / softmax far from uniform
        inner = w.layer

        def layer(l):
            d = inner(l)
            return {k: (v if k.endswith("norm") else v * sigma_boost) for k, v in d.items()}
        w.layer = layer
        w.lm_head = w.lm_head * sigma_boost
    cfg = oracle_config(wl.shape)
    patch, ids = vi.observation(wl, seed)
    return cfg, w, to_f64(patch), ids.numpy().astype(np.int64)


# ----------------------------------------------------------------------------------------
# scalar-loop brute force: whole sequence from scratch, explicit boolean mask, no cache
# ----------------------------------------------------------------------------------------

def _dot(a, b):
    s = 0.0
    for x, y in zip(a, b):
        s += x * y
    return s


def _matvec(W, x):
    return [_dot(row, x) for row in W]


def _norm(x, g, eps):
    ms = sum(v * v for v in x) / len(x)
    r = 1.0 / math.sqrt(ms + eps)
    return [v * r * gi for v, gi in zip(x, g)]


def _rope(u, pos, theta):
    d = len(u)
    out = list(u)
    for i in range(d // 2):
        phi = pos * theta ** (-2.0 * i / d)
        a, b = u[i], u[i + d // 2]
        out[i] = a * math.cos(phi) - b * math.sin(phi)
        out[i + d // 2] = b * math.cos(phi) + a * math.sin(phi)
    return out


def bf16_scalar(x):
    """Round one Python float to bfloat16 (nearest, ties to even) through its fp32 bit pattern."""
    import struct
    (u,) = struct.unpack("<I", struct.pack("<f", x))
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return struct.unpack("<f", struct.pack("<I", u))[0]


def brute_rows(cfg, w, rows, positions, allowed, rnd=None):
    """rows: list of H-vectors (python lists); allowed[r][c] bool.  Returns residual rows.
    rnd: optional scalar rounding applied to the stored tensors (norm outputs, rotated q, k, v,
    attention output, SwiGLU output)."""
    H, nh, d = cfg.hidden, cfg.n_heads, cfg.head_dim
    st = (lambda v: [rnd(t) for t in v]) if rnd else (lambda v: v)
    x = [list(r) for r in rows]
    R = len(x)
    for l in range(cfg.n_layers):
        lw = {k: v.tolist() for k, v in w.layer(l).items()}
        q, k, v = [], [], []
        for r in range(R):
            n = st(_norm(x[r], lw["attn_norm"], cfg.rms_eps))
            qr, kr, vr = _matvec(lw["wq"], n), _matvec(lw["wk"], n), _matvec(lw["wv"], n)
            q.append([st(_rope(qr[h * d:(h + 1) * d], positions[r], cfg.rope_theta)) for h in range(nh)])
            k.append([st(_rope(kr[h * d:(h + 1) * d], positions[r], cfg.rope_theta)) for h in range(nh)])
            v.append([st(vr[h * d:(h + 1) * d]) for h in range(nh)])
        for r in range(R):
            o = []
            for h in range(nh):
                cols = [c for c in range(R) if allowed[r][c]]
                sc = [_dot(q[r][h], k[c][h]) / math.sqrt(d) for c in cols]
                m = max(sc)
                e = [math.exp(s - m) for s in sc]
                z = sum(e)
                acc = [0.0] * d
                for pc, c in zip(e, cols):
                    for i in range(d):
                        acc[i] += pc / z * v[c][h][i]
                o.extend(acc)
            att = _matvec(lw["wo"], st(o))
            x[r] = [a + b for a, b in zip(x[r], att)]
        for r in range(R):
            n = st(_norm(x[r], lw["ffn_norm"], cfg.rms_eps))
            g, u = _matvec(lw["w_gate"], n), _matvec(lw["w_up"], n)
            act = st([gi / (1.0 + math.exp(-gi)) * ui for gi, ui in zip(g, u)])
            dn = _matvec(lw["w_down"], act)
            x[r] = [a + b for a, b in zip(x[r], dn)]
    return x


def brute_head(cfg, w, xrow, tau):
    h = _norm(xrow, w.final_norm.tolist(), cfg.rms_eps)
    head = w.lm_head[cfg.vocab - cfg.n_bins:].tolist()
    z = _matvec(head, h)
    y = [v / tau for v in z]
    m = max(y)
    lse = m + math.log(sum(math.exp(v - m) for v in y))
    logp = [v - lse for v in y]
    ent = -sum(math.exp(v) * v for v in logp)
    return h, z, y, logp, ent


def brute_rollout_ar(cfg, w, patch_b, ids_b, A, tau, g_b, rnd=None):
    """One environment, autoregressive, every token recomputed from scratch."""
    S = patch_b.shape[0] + ids_b.shape[0]
    rows = [r.tolist() for r in patch_b] + [w.embed[i].tolist() for i in ids_b]
    out = []
    for j in range(A):
        R = len(rows)
        allowed = [[c <= r for c in range(R)] for r in range(R)]
        x = brute_rows(cfg, w, rows, list(range(R)), allowed, rnd)
        _, z, y, logp, ent = brute_head(cfg, w, x[-1], tau)
        t = [np.float32(yv) + (np.float32(g_b[j][k]) if g_b is not None else np.float32(0))
             for k, yv in enumerate(y)]
        b = max(range(len(t)), key=lambda k: (t[k], -k))
        out.append((b, logp[b], ent, z))
        rows.append(w.embed[cfg.vocab - cfg.n_bins + b].tolist())
    assert len(rows) == S + A
    return out


@pytest.mark.parametrize("tau,sampled", [(1.0, True), (1.6, False)])
def test_cached_rollout_matches_scalar_brute_force(tau, sampled):
    wl = small_workload(B=2, P=3, T=2, A=3)
    cfg, w, patch, ids = setup(wl, seed=3, sigma_boost=12.0)
    g = to_f64(vi.gumbel_noise(wl, 3)) if sampled else None
    kv, h_last, _ = vo.ovla_prefill(cfg, w, patch, ids)
    bins, logp, ent, logits, _ = vo.ovla_decode_actions(cfg, w, kv, h_last, wl.prefix, wl.n_action,
                                                        temperature=tau, gumbel=g)
    for b in range(wl.batch):
        ref = brute_rollout_ar(cfg, w, patch[b], ids[b], wl.n_action, tau, None if g is None else g[b])
        for j, (rb, rlp, rent, rz) in enumerate(ref):
            assert bins[b, j] == rb
            assert abs(logp[b, j] - rlp) < 1e-10
            assert abs(ent[b, j] - rent) < 1e-10
            assert np.max(np.abs(logits[b, j] - np.array(rz))) < 1e-10
    # attention must not be near uniform for this to pin anything: logits spread out
    assert np.std(logits) > 0.3


def test_round_bf16_against_torch_and_known_values():
    rng = np.random.default_rng(0)
    x = rng.standard_normal(50_000) * np.exp(rng.uniform(-30, 30, 50_000))
    assert np.array_equal(vo.round_bf16(x), torch.from_numpy(x).float().bfloat16().double().numpy())
    assert np.array_equal(vo.round_bf16(x[:200]), np.array([bf16_scalar(v) for v in x[:200]]))
    # ties to even at the 8-bit mantissa: 1 + 2^-8 -> 1, 1 + 3*2^-8 -> 1 + 2^-6, just above a tie -> up
    assert vo.round_bf16(np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 1 + 2.0 ** -8 + 2.0 ** -20])).tolist() == \
        [1.0, 1.015625, 1.0078125]
    assert vo.round_bf16(np.array([0.0, -2.5, 3.140625])).tolist() == [0.0, -2.5, 3.140625]


def test_bf16_stored_mode_matches_scalar_brute_force_with_the_same_roundings():
    """The "bf16" operand mode rounds exactly the stored tensors: norm outputs, rotated q, k, v,
    attention output, SwiGLU output -- and nothing else."""
    wl = small_workload(B=2, P=3, T=2, A=3)
    cfg, w, patch, ids = setup(wl, seed=3, sigma_boost=12.0)
    cfg.operand_dtype = "bf16"
    g = to_f64(vi.gumbel_noise(wl, 3))
    kv, h_last, _ = vo.ovla_prefill(cfg, w, patch, ids)
    bins, logp, ent, logits, _ = vo.ovla_decode_actions(cfg, w, kv, h_last, wl.prefix, wl.n_action, gumbel=g)
    exact_cfg = oracle_config(wl.shape)
    _, h_exact, _ = vo.ovla_prefill(exact_cfg, w, patch, ids)
    assert 1e-4 < np.max(np.abs(h_exact - h_last)) < 0.2          # the mode does change the result
    for b in range(wl.batch):
        ref = brute_rollout_ar(cfg, w, patch[b], ids[b], wl.n_action, 1.0, g[b], rnd=bf16_scalar)
        for j, (rb, rlp, rent, rz) in enumerate(ref):
            assert bins[b, j] == rb
            assert abs(logp[b, j] - rlp) < 1e-9 and abs(ent[b, j] - rent) < 1e-9
            assert np.max(np.abs(logits[b, j] - np.array(rz))) < 1e-9
    lp2, ent2, _, z2 = vo.ovla_logprob_recompute(cfg, w, patch, ids, bins, wl.n_action)
    assert np.max(np.abs(z2 - logits)) < 1e-9 and np.max(np.abs(lp2 - logp)) < 1e-9


def test_parallel_chunk_matches_scalar_brute_force_with_explicit_mask():
    wl = small_workload(B=2, P=3, T=2, A=4, mode=1)
    cfg, w, patch, ids = setup(wl, seed=5, sigma_boost=12.0)
    S, A = wl.prefix, wl.n_action
    slot = to_f64(vi.SynthModel(wl.shape, 5).slot_embed(A)) * 12.0
    kv, h_last, _ = vo.ovla_prefill(cfg, w, patch, ids)
    bins, logp, ent, logits, _ = vo.ovla_decode_actions(cfg, w, kv, h_last, S, A, mode=1,
                                                        slot_embed=slot)
    lp_rc, ent_rc, _, z_rc = vo.ovla_logprob_recompute(cfg, w, patch, ids, bins, A, mode=1,
                                                       slot_embed=slot)
    for b in range(wl.batch):
        rows = [r.tolist() for r in patch[b]] + [w.embed[i].tolist() for i in ids[b]] + slot.tolist()
        allowed = [[(c <= r) or (r >= S) for c in range(S + A)] for r in range(S + A)]
        x = brute_rows(cfg, w, rows, list(range(S + A)), allowed)
        for s in range(A):
            _, z, y, lp, e = brute_head(cfg, w, x[S + s], 1.0)
            assert np.max(np.abs(logits[b, s] - np.array(z))) < 1e-10
            assert np.max(np.abs(z_rc[b, s] - np.array(z))) < 1e-10
            assert bins[b, s] == int(np.argmax(np.array(y, dtype=np.float32)))
            assert abs(logp[b, s] - lp[bins[b, s]]) < 1e-10 and abs(lp_rc[b, s] - lp[bins[b, s]]) < 1e-10
            assert abs(ent[b, s] - e) < 1e-10 and abs(ent_rc[b, s] - e) < 1e-10


def test_recompute_matches_scalar_brute_force_and_value():
    wl = small_workload(B=2, P=2, T=2, A=3)
    cfg, w, patch, ids = setup(wl, seed=7, sigma_boost=10.0)
    bins = vi.stored_bins(wl, 7).numpy()
    lp, ent, val, z = vo.ovla_logprob_recompute(cfg, w, patch, ids, bins, wl.n_action, temperature=1.3)
    S = wl.prefix
    for b in range(wl.batch):
        rows = [r.tolist() for r in patch[b]] + [w.embed[i].tolist() for i in ids[b]]
        rows += [w.embed[cfg.vocab - 256 + bins[b, j]].tolist() for j in range(wl.n_action - 1)]
        R = len(rows)
        x = brute_rows(cfg, w, rows, list(range(R)), [[c <= r for c in range(R)] for r in range(R)])
        for j in range(wl.n_action):
            h, zz, _, l, e = brute_head(cfg, w, x[S - 1 + j], 1.3)
            assert np.max(np.abs(z[b, j] - np.array(zz))) < 1e-10
            assert abs(lp[b, j] - l[bins[b, j]]) < 1e-10 and abs(ent[b, j] - e) < 1e-10
            if j == 0:
                assert abs(val[b] - (_dot(h, w.value_w.tolist()) + vi.VALUE_BIAS)) < 1e-10


# ----------------------------------------------------------------------------------------
# PyTorch-CPU library composition of the tiny fp32 workload
# ----------------------------------------------------------------------------------------

def torch_forward(shape, model, x, positions, mask):
    """x [n, R, H] fp64 torch; library ops only: F.rms_norm, F.linear, SDPA, F.silu; the
    rotation is done as a complex multiplication by unit phasors."""
    F = torch.nn.functional
    nh, d = shape.n_heads, shape.head_dim
    ang = positions.double()[:, None] * shape.rope_theta ** (-torch.arange(0, d, 2).double() / d)
    phasor = torch.polar(torch.ones_like(ang), ang)                       # [R, d/2]

    def rot(u):                                                           # [n, nh, R, d]
        c = torch.complex(u[..., :d // 2], u[..., d // 2:]) * phasor
        return torch.cat([c.real, c.imag], dim=-1)

    for l in range(shape.n_layers):
        lw = {k: v.double() for k, v in model.layer(l).items()}
        n = F.rms_norm(x, (shape.hidden,), lw["attn_norm"], shape.rms_eps)
        hv = lambda t: t.view(t.shape[0], t.shape[1], nh, d).transpose(1, 2)
        q, k, v = rot(hv(F.linear(n, lw["wq"]))), rot(hv(F.linear(n, lw["wk"]))), hv(F.linear(n, lw["wv"]))
        o = F.scaled_dot_product_attention(q, k, v, attn_mask=mask)
        x = x + F.linear(o.transpose(1, 2).reshape(x.shape), lw["wo"])
        n = F.rms_norm(x, (shape.hidden,), lw["ffn_norm"], shape.rms_eps)
        x = x + F.linear(F.silu(F.linear(n, lw["w_gate"])) * F.linear(n, lw["w_up"]), lw["w_down"])
    return x


def test_tiny_config_matches_torch_library_composition():
    wl = vi.WORKLOADS["cfg1_tiny_fp32"]
    shape = wl.shape
    model = vi.SynthModel(shape, 0)
    cfg, w = oracle_config(shape), oracle_weights(model, vi.VALUE_BIAS)
    patch, ids = vi.observation(wl, 0)
    g = vi.gumbel_noise(wl, 0)
    kv, h_last, val = vo.ovla_prefill(cfg, w, to_f64(patch), ids.numpy())
    bins, logp, ent, logits, _ = vo.ovla_decode_actions(cfg, w, kv, h_last, wl.prefix, wl.n_action,
                                                        gumbel=to_f64(g))
    # teacher-forced torch forward over prefix + the oracle's own first A-1 tokens
    F = torch.nn.functional
    E = model.embed().double()
    S, A = wl.prefix, wl.n_action
    tok = torch.from_numpy(bins[:, :A - 1].astype(np.int64)) + shape.vocab - 256
    x = torch.cat([patch.double(), E[ids.long()], E[tok]], dim=1)
    R = S + A - 1
    mask = torch.tril(torch.ones(R, R, dtype=torch.bool))
    x = torch_forward(shape, model, x, torch.arange(R), mask)
    h = F.rms_norm(x[:, S - 1:], (shape.hidden,), model.final_norm().double(), shape.rms_eps)
    z = F.linear(h, model.lm_head().double()[-256:])
    dist = torch.distributions.Categorical(logits=z)
    assert np.max(np.abs(logits - z.numpy())) < 1e-9
    assert np.max(np.abs(ent - dist.entropy().numpy())) < 1e-9
    assert np.max(np.abs(logp - dist.log_prob(torch.from_numpy(bins.astype(np.int64))).numpy())) < 1e-9
    want = torch.argmax((z.float() + g), dim=-1).numpy()
    assert np.array_equal(bins, want)
    v = F.linear(h[:, 0], model.value_w().double()[None])[:, 0] + vi.VALUE_BIAS
    assert np.max(np.abs(val - v.numpy())) < 1e-10


def test_parallel_chunk_matches_torch_library_composition():
    wl = vi.scaled(vi.WORKLOADS["cfg1_tiny_fp32"], batch=3, n_action=8, mode=1)
    shape = wl.shape
    model = vi.SynthModel(shape, 1)
    cfg, w = oracle_config(shape), oracle_weights(model, vi.VALUE_BIAS)
    patch, ids = vi.observation(wl, 1)
    slot = model.slot_embed(wl.n_action)
    S, A = wl.prefix, wl.n_action
    kv, h_last, _ = vo.ovla_prefill(cfg, w, to_f64(patch), ids.numpy())
    bins, logp, ent, logits, _ = vo.ovla_decode_actions(cfg, w, kv, h_last, S, A, mode=1,
                                                        slot_embed=to_f64(slot))
    F = torch.nn.functional
    x = torch.cat([patch.double(), model.embed().double()[ids.long()],
                   slot.double()[None].expand(wl.batch, A, shape.hidden)], dim=1)
    mask = torch.tril(torch.ones(S + A, S + A, dtype=torch.bool))
    mask[S:] = True
    x = torch_forward(shape, model, x, torch.arange(S + A), mask)
    h = F.rms_norm(x[:, S:], (shape.hidden,), model.final_norm().double(), shape.rms_eps)
    z = F.linear(h, model.lm_head().double()[-256:])
    assert np.max(np.abs(logits - z.numpy())) < 1e-9
    assert np.array_equal(bins, torch.argmax(z.float(), -1).numpy())
    assert np.max(np.abs(logp - F.log_softmax(z, -1).max(-1).values.numpy())) < 1e-9


# ----------------------------------------------------------------------------------------
# closed forms and invariants
# ----------------------------------------------------------------------------------------

def test_zero_head_gives_uniform_distribution_and_bin_zero():
    wl = small_workload()
    cfg, w, patch, ids = setup(wl)
    w.lm_head = np.zeros_like(w.lm_head)
    kv, h_last, _ = vo.ovla_prefill(cfg, w, patch, ids)
    bins, logp, ent, _, _ = vo.ovla_decode_actions(cfg, w, kv, h_last, wl.prefix, wl.n_action)
    assert np.all(bins == 0)
    assert np.allclose(logp, -LN256, atol=1e-12) and np.allclose(ent, LN256, atol=1e-12)


def test_identity_layers_closed_form():
    """W_o = W_down = 0 makes every layer the identity: z = W_head . norm(E[last id])."""
    wl = small_workload()
    cfg, w, patch, ids = setup(wl)
    inner = w.layer

    def layer(l):
        d = dict(inner(l))
        d["wo"] = np.zeros_like(d["wo"])
        d["w_down"] = np.zeros_like(d["w_down"])
        return d
    w.layer = layer
    kv, h_last, val = vo.ovla_prefill(cfg, w, patch, ids)
    _, _, _, logits, _ = vo.ovla_decode_actions(cfg, w, kv, h_last, wl.prefix, 1)
    e = w.embed[ids[:, -1]]
    h = e / np.sqrt((e * e).mean(-1, keepdims=True) + cfg.rms_eps) * w.final_norm
    assert np.allclose(logits[:, 0], h @ w.lm_head[-256:].T, atol=1e-12)
    assert np.allclose(val, h @ w.value_w + vi.VALUE_BIAS, atol=1e-12)


def test_single_key_attention_is_wo_wv():
    """S = 1 (no patches, one id): softmax over one key is 1, so after layer 0's attention
    the residual is x + W_o W_v norm(x)."""
    wl = small_workload(B=2, P=0, T=1, A=1, n_layers=1)
    cfg, w, patch, ids = setup(wl, sigma_boost=8.0)
    lw = w.layer(0)
    x = w.embed[ids[:, 0]]
    n = vo.rmsnorm(x, lw["attn_norm"], cfg.rms_eps)
    x1 = x + n @ lw["wv"].T @ lw["wo"].T
    n2 = vo.rmsnorm(x1, lw["ffn_norm"], cfg.rms_eps)
    g = n2 @ lw["w_gate"].T
    x2 = x1 + ((g / (1 + np.exp(-g))) * (n2 @ lw["w_up"].T)) @ lw["w_down"].T
    _, h_last, _ = vo.ovla_prefill(cfg, w, patch, ids)
    assert np.allclose(h_last, vo.rmsnorm(x2, w.final_norm, cfg.rms_eps), atol=1e-12)


def test_rotary_invariants():
    rng = np.random.default_rng(0)
    u = rng.standard_normal((2, 3, 5, 8))
    pos = np.array([0, 1, 7, 100, 287])
    r = vo.rotary(u, pos, 10000.0)
    assert np.allclose(r[..., 0, :], u[..., 0, :], atol=0)            # position 0: identity
    assert np.allclose(np.linalg.norm(r, axis=-1), np.linalg.norm(u, axis=-1))
    # rotation by position p then dotting with a key at p' depends on p - p' only
    q, k = rng.standard_normal(8), rng.standard_normal(8)
    f = lambda a, b: vo.rotary(q[None], np.array([a]), 10000.0)[0] @ vo.rotary(k[None], np.array([b]), 10000.0)[0]
    assert abs(f(9, 4) - f(105, 100)) < 1e-9
    assert abs(f(9, 4) - f(4, 9)) > 1e-3                               # sign of the angle matters
    # pair (i, i + d/2), angle p * theta^(-2i/d): one hand-computed component
    e = np.zeros(8); e[1] = 1.0
    out = vo.rotary(e[None], np.array([3]), 10000.0)[0]
    phi = 3 * 10000.0 ** (-2.0 / 8)
    assert np.allclose(out[[1, 5]], [math.cos(phi), math.sin(phi)]) and np.allclose(np.delete(out, [1, 5]), 0)


def test_position_offset_leaves_logits_unchanged():
    """Adding a constant to all positions changes no logit (relative-position property)."""
    wl = small_workload(B=1, P=4, T=3, A=1)
    cfg, w, patch, ids = setup(wl, sigma_boost=10.0)
    x = vo.embed_prefix(w, patch, ids)
    S = x.shape[1]
    mask = np.tril(np.ones((S, S), dtype=bool))
    a, _ = vo.decoder_layers(cfg, w, x, np.arange(S), mask, None)
    b, _ = vo.decoder_layers(cfg, w, x, np.arange(S) + 37, mask, None)
    assert np.max(np.abs(a - b)) < 1e-9


def test_rollout_equals_recompute_rho_is_one():
    """Appendix I-B: rho = pi_theta / pi_theta_old; with theta = theta_old the recomputed
    log-probs equal the rollout's."""
    wl = vi.scaled(vi.WORKLOADS["cfg1_tiny_fp32"], batch=4)
    cfg, w, patch, ids = setup(wl, seed=2, sigma_boost=3.0)
    g = to_f64(vi.gumbel_noise(wl, 2))
    kv, h_last, val = vo.ovla_prefill(cfg, w, patch, ids)
    bins, logp, ent, logits, _ = vo.ovla_decode_actions(cfg, w, kv, h_last, wl.prefix, wl.n_action,
                                                        temperature=1.6, gumbel=g)
    lp2, ent2, val2, z2 = vo.ovla_logprob_recompute(cfg, w, patch, ids, bins, wl.n_action, temperature=1.6)
    assert np.max(np.abs(np.exp(lp2 - logp) - 1.0)) < 1e-10
    assert np.max(np.abs(ent2 - ent)) < 1e-10 and np.max(np.abs(z2 - logits)) < 1e-10
    assert np.max(np.abs(val2 - val)) < 1e-12


def test_distribution_normalises_and_temperature():
    rng = np.random.default_rng(1)
    z = rng.standard_normal((5, 256)) * 3
    y, lp, ent = vo.token_distribution(z, 1.6)
    assert np.allclose(np.exp(lp).sum(-1), 1.0, atol=1e-12)
    assert np.all(ent >= 0) and np.all(ent <= LN256 + 1e-12)
    y1, lp1, ent1 = vo.token_distribution(z / 1.6, 1.0)
    assert np.allclose(lp, lp1, atol=1e-14) and np.allclose(ent, ent1, atol=1e-14)
    # a two-point distribution with known entropy
    z2 = np.full((1, 256), -1e9); z2[0, 3] = 0.0; z2[0, 200] = math.log(3.0)
    _, lp2, e2 = vo.token_distribution(z2, 1.0)
    assert abs(lp2[0, 200] - math.log(0.75)) < 1e-12
    assert abs(e2[0] - (-(0.25 * math.log(0.25) + 0.75 * math.log(0.75)))) < 1e-12


def test_gumbel_max_samples_from_softmax():
    """Empirical bin frequencies over 10^5 noise draws match softmax(z / tau) (chi-square)."""
    rng = np.random.default_rng(2)
    z = rng.standard_normal(256) * 2.0
    tau = 1.6
    y, lp, _ = vo.token_distribution(z[None], tau)
    p = np.exp(lp[0])
    n = 100_000
    g = vi.gumbel(11, 77, (n, 256)).numpy()
    picks = vo.gumbel_argmax(np.broadcast_to(y, (n, 256)), g)
    counts = np.bincount(picks, minlength=256)
    big = p * n >= 5
    chi2 = (((counts - p * n) ** 2) / (p * n))[big].sum()
    dof = big.sum() - 1
    assert chi2 < dof + 4.5 * math.sqrt(2 * dof)
    assert np.max(np.abs(counts / n - p)) < 4.5 * math.sqrt(p.max() / n)
    # greedy and tie rule
    assert vo.gumbel_argmax(y, None)[0] == np.argmax(z)
    assert vo.gumbel_argmax(np.zeros((1, 256)), None)[0] == 0


def test_batch_permutation_and_duplication():
    wl = vi.scaled(vi.WORKLOADS["cfg1_tiny_fp32"], batch=5)
    cfg, w, patch, ids = setup(wl, seed=4)
    g = to_f64(vi.gumbel_noise(wl, 4))

    def run(p, i, gg):
        kv, h, v = vo.ovla_prefill(cfg, w, p, i)
        b, lp, e, z, _ = vo.ovla_decode_actions(cfg, w, kv, h, wl.prefix, wl.n_action, gumbel=gg)
        return b, lp, e, z, v
    base = run(patch, ids, g)
    perm = np.array([3, 0, 4, 4, 1])       # permutation with env 4 duplicated
    out = run(patch[perm], ids[perm], g[perm])
    assert np.array_equal(out[0], base[0][perm])
    for a, b in zip(out[1:], base[1:]):
        assert np.max(np.abs(a - b[perm])) < 1e-12
    one = run(patch[2:3], ids[2:3], g[2:3])
    assert np.array_equal(one[0], base[0][2:3]) and np.max(np.abs(one[3] - base[3][2:3])) < 1e-12


def test_parallel_chunk_single_slot_reduces_to_one_ar_forward():
    """A = 1 in chunk mode is one decode forward whose input is slot_embed[0]; the prefix
    rows' K, V are those of the causal prefill (slots are invisible to the prefix)."""
    wl = small_workload(B=2, P=3, T=2, A=1, mode=1)
    cfg, w, patch, ids = setup(wl, sigma_boost=10.0)
    S = wl.prefix
    slot = np.random.default_rng(3).standard_normal((1, cfg.hidden))
    kv, h_last, _ = vo.ovla_prefill(cfg, w, patch, ids)
    _, _, _, z_chunk, kv2 = vo.ovla_decode_actions(cfg, w, kv, h_last, S, 1, mode=1, slot_embed=slot)
    # the same through the AR machinery: overwrite the embedding of bin 0's token with the slot
    w2 = vo.OracleWeights(embed=w.embed.copy(), lm_head=np.zeros_like(w.lm_head),
                          final_norm=w.final_norm, layer=w.layer)
    w2.embed[cfg.vocab - 256] = slot[0]      # zero head => greedy bin 0 => feeds that row
    _, _, _, _, kv3 = vo.ovla_decode_actions(cfg, w2, kv, h_last, S, 2, mode=0)
    for (k2, v2), (k3, v3) in zip(kv2, kv3):
        assert np.allclose(k2, k3, atol=1e-12) and np.allclose(v2, v3, atol=1e-12)
    lp, _, _, z_rc = vo.ovla_logprob_recompute(cfg, w, patch, ids, np.zeros((2, 1), np.int32), 1,
                                               mode=1, slot_embed=slot)
    assert np.allclose(z_rc, z_chunk, atol=1e-10)
    for l in range(cfg.n_layers):
        assert np.array_equal(kv2[l][0][:, :, :S], kv[l][0]) and np.array_equal(kv2[l][1][:, :, :S], kv[l][1])


def test_value_head_closed_forms():
    wl = small_workload()
    cfg, w, patch, ids = setup(wl)
    _, h_last, v = vo.ovla_prefill(cfg, w, patch, ids)
    assert np.allclose(v, h_last @ w.value_w + vi.VALUE_BIAS)
    w.value_w = np.zeros_like(w.value_w)
    _, _, v0 = vo.ovla_prefill(cfg, w, patch, ids)
    assert np.allclose(v0, vi.VALUE_BIAS, atol=0)


def test_action_level_value_head_is_one_dot_product_per_action():
    wl = small_workload()
    cfg, _, patch, ids = setup(wl)
    w = oracle_weights(vi.SynthModel(wl.shape, 0), vi.VALUE_BIAS, value_dim=4)
    _, h_last, v = vo.ovla_prefill(cfg, w, patch, ids)
    assert v.shape == (wl.batch, 4)
    for b in range(wl.batch):
        for c in range(4):
            assert abs(v[b, c] - (_dot(h_last[b].tolist(), w.value_w[c].tolist()) + vi.VALUE_BIAS + 0.125 * c)) < 1e-12
