#!/usr/bin/env python3
"""Benchmark of the batched VLA rollout step on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic observations: vla_prefill
(observation prefix -> KV cache) followed by vla_decode_actions (7 autoregressive action tokens with
Gumbel-max sampling, or the parallel chunk pass), with every input already resident in HBM.
Prints one JSON line: env-actions/s plus the roofline of the dominant kernel (measured with HIP
events recorded by the library around each launch, in a separate instrumented pass) and the CPU
oracle timed on a bounded sample of the same workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg3_7b_b256]
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MI355X_HBM_GBPS = 8000.0          # published peak HBM3E bandwidth
MI355X_BF16_TFLOPS = 2500.0       # published dense bf16 MFMA peak


def profile_report(vb):
    buf = ctypes.create_string_buffer(1 << 16)
    n = vb.lib().vla_profile_report(buf, len(buf))
    if n < 0:
        raise RuntimeError(vb.vla_last_error())
    out = {}
    for line in buf.value.decode().splitlines():
        label, count, ms, work = line.rsplit(" ", 3)
        out[label] = dict(count=int(count), ms=float(ms), work=float(work))
    return out


def read_traffic(path, kernel, source):
    """HBM bytes per launch of `kernel`, measured in separate rocprofv3 --pmc runs (hardware counters cannot be
    read inside a timed run) and kept in profiles/*.txt as 'key: value' lines.  The figure is only quoted while the
    file names this kernel and carries the SHA-256 of the kernel's source file as it is in the tree now; after any
    change to that source the traffic is reported as null until the counters have been collected again.
    Returns (bytes or None, provenance dict)."""
    import hashlib
    prov = {"file": os.path.relpath(path, ROOT), "how": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, separate runs, "
            "scaled by the same counters on a 1 GiB copy kernel", "kernel_source": os.path.relpath(source, ROOT)}
    try:
        vals = {}
        for line in open(path):
            if ":" in line and not line.startswith("#"):
                k, v = line.split(":", 1)
                vals[k.strip()] = v.strip()
        sha = hashlib.sha256(open(source, "rb").read()).hexdigest()
        prov["source_sha256_in_tree"] = sha[:16]
        prov["source_sha256_measured"] = vals.get("kernel_source_sha256", "")[:16]
        prov["current"] = vals.get("kernel") == kernel and vals.get("kernel_source_sha256") == sha
        if not prov["current"]:
            return None, prov
        return float(vals["hbm_bytes_per_launch"]), prov
    except Exception as e:                      # missing or unreadable file: no figure
        prov["current"] = False
        prov["error"] = str(e)
        return None, prov


def forward_flops(shape, n_seq, rows, tail_rows):
    """Projection flops a multi-row forward executes: all rows through all layers but the last; in the last layer K and
    V for all rows and the rest (q, o, gate, up, down) for the `tail_rows` rows per sequence whose output is read
    (the library skips what nothing reads; the skipped work is not counted here).  tail_rows = rows: no skipping."""
    H, F = shape.hidden, shape.ffn
    full = 2.0 * shape.layer_params
    last = 2.0 * (2 * H * H) * rows + 2.0 * (2 * H * H + 3 * H * F) * tail_rows
    return n_seq * (rows * full * (shape.n_layers - 1) + last)


def cpu_baseline(wl, vi, sample_layers=8):
    """The CPU oracle as it stands, on 1 environment x `sample_layers` of the model's layers
    (prefill + decode), scaled linearly to all layers; the head and embedding cost is negligible."""
    import numpy as np
    import torch
    from oracle import vla_oracle as vo
    from oracle.from_inputs import oracle_config, oracle_weights, to_f64

    shape = vi.scaled(wl, n_layers=sample_layers).shape
    model = vi.SynthModel(shape, 0)
    cfg = oracle_config(shape)
    w = oracle_weights(model, vi.VALUE_BIAS)
    for l in range(sample_layers):
        w.layer(l)                                   # generate the weights outside the timed region
    patch, ids = vi.observation(wl, 0, envs=1)
    g = to_f64(vi.gumbel_noise(wl, 0, envs=1))
    slot = to_f64(model.slot_embed(wl.n_action)) if wl.mode == 1 else None
    t0 = time.perf_counter()
    kv, h_last, _ = vo.ovla_prefill(cfg, w, to_f64(patch), ids.numpy().astype(np.int64))
    vo.ovla_decode_actions(cfg, w, kv, h_last, wl.prefix, wl.n_action, wl.mode, slot, wl.temperature, g)
    dt = time.perf_counter() - t0
    per_env = dt * wl.shape.n_layers / sample_layers
    return {"value": 1.0 / per_env, "unit": "env-actions/s", "cores": torch.get_num_threads(), "kind": "oracle",
            "sample": f"1 env x {sample_layers} of {wl.shape.n_layers} layers (prefill {wl.prefix} rows + "
                      f"{wl.n_action} action tokens), fp64 numpy, {dt:.1f} s measured, scaled by layers"}


RECOMPUTE_MICRO_BATCH = 256


def bench_recompute(args, wl, torch, vi, vb, Rollout):
    """The log-prob recompute workload (cfg5): a step is one vla_logprob_recompute call over all stored
    rollouts, internally micro-batched by max_batch = 256 (75,264 rows per pass: 294 row tiles of the GEMMs, whose
    O / down projections then fill 18.4 rounds of the 256 CUs instead of the 9.2 rounds that 128 rollouts give)."""
    dev = "cuda:0"
    torch.cuda.set_device(0)
    N, S, A, shape = wl.batch, wl.prefix, wl.n_action, wl.shape
    synth = vi.SynthModel(shape, 0, device=dev)
    run = Rollout(synth, min(N, RECOMPUTE_MICRO_BATCH), S + A, device=dev, value_b=vi.VALUE_BIAS)
    patch, ids = vi.observation(wl, 0, device=dev)
    bins = vi.stored_bins(wl, 0, device=dev)
    slot = synth.slot_embed(A) if wl.mode == 1 else None
    stream = torch.cuda.current_stream()

    def step():
        return run.recompute(patch, ids, bins, A, wl.mode, slot, wl.temperature, want_value=True,
                             want_logits=False, stream=stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    vb.lib().vla_profile_enable(1)
    step()
    torch.cuda.synchronize()
    prof = profile_report(vb)
    vb.lib().vla_profile_enable(0)
    rows = S + A - 1 if wl.mode == 0 else S + A
    tail = A if (wl.mode == 0 and A * 4 <= rows) else rows          # autoregressive form: only the A read-out rows finish the last layer
    flops = forward_flops(shape, N, rows, tail)
    dom = prof.get("gemm_bf16_dma<swiglu>")
    roofline = None
    if dom:
        ach = dom["work"] / (dom["ms"] * 1e-3) / 1e12
        roofline = {"bound": "mfma", "kernel": "gemm_bf16_dma_kernel<EPI_SWIGLU, k-blocked, unit barrier> (gate/up projection)",
                    "achieved": ach, "peak": MI355X_BF16_TFLOPS, "unit": "TFLOP/s", "frac": ach / MI355X_BF16_TFLOPS,
                    "launches": dom["count"], "avg_launch_ms": dom["ms"] / dom["count"], "traffic": None}
    out = {"metric": "stored rollouts/sec, log-prob recompute (7B shape), % MFMA roofline", "value": N / (ms * 1e-3),
           "unit": "rollouts/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "bf16" if shape.dtype == "bf16" else "f32", "data": "synthetic",
           "config": {"workload": wl.name, "rollouts": N, "prefix": S, "action_tokens": A, "rows_per_rollout": rows,
                      "micro_batch": min(N, RECOMPUTE_MICRO_BATCH), "layers": shape.n_layers, "hidden": shape.hidden},
           "roofline": roofline,
           "phases": {"recompute_tokens_per_s": N * rows / (ms * 1e-3), "mfma_TFLOPs": flops / (ms * 1e-3) / 1e12,
                      "mfma_frac": flops / (ms * 1e-3) / 1e12 / MI355X_BF16_TFLOPS},
           "kernels": {k: {"n": v["count"], "ms": round(v["ms"], 3)} for k, v in sorted(prof.items(), key=lambda kv: -kv[1]["ms"])}}
    print(json.dumps(out))


def bench_backward(args, wl, torch, vi, vb, Rollout):
    """LoRA-gradient pass (vla_logprob_backward) over a sample of the recompute workload's stored rollouts: a step is
    one call over `--backward-rollouts` rollouts in micro-batches of `--backward-micro-batch`.  Reports rollouts/s and
    the rate of the projection flops it executes (the forward once, every layer again without its down projection, and
    the input-gradient products once; with --backward-keep the forward once and the input-gradient products), against
    the bf16 MFMA peak."""
    dev = "cuda:0"
    torch.cuda.set_device(0)
    N, mb, rank = args.backward_rollouts, args.backward_micro_batch, args.lora_rank
    S, A, shape = wl.prefix, wl.n_action, wl.shape
    wl_n = vi.scaled(wl, batch=N)
    synth = vi.SynthModel(shape, 0, device=dev)
    run = Rollout(synth, mb, S + A, device=dev, value_b=vi.VALUE_BIAS)
    patch, ids = vi.observation(wl_n, 0, device=dev)
    bins = vi.stored_bins(wl_n, 0, device=dev)
    g = torch.Generator(device="cpu").manual_seed(1)
    coef = torch.randn(N, A, generator=g).to(dev)
    dims = {"q": (shape.hidden, shape.hidden), "k": (shape.hidden, shape.hidden), "v": (shape.hidden, shape.hidden),
            "o": (shape.hidden, shape.hidden), "gate": (shape.ffn, shape.hidden), "up": (shape.ffn, shape.hidden),
            "down": (shape.hidden, shape.ffn)}
    lora = [{p: ((0.05 * torch.randn(rank, i, generator=g)).to(shape.torch_dtype).to(dev),
                 (0.05 * torch.randn(o, rank, generator=g)).to(shape.torch_dtype).to(dev)) for p, (o, i) in dims.items()}
            for _ in range(shape.n_layers)]
    stream = torch.cuda.current_stream()

    def step():
        return run.backward(patch, ids, bins, coef, A, lora, rank, 0.5, wl.mode, None, wl.temperature, stream=stream,
                            keep_activations=args.backward_keep)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    vb.lib().vla_profile_enable(1)
    step()
    torch.cuda.synchronize()
    prof = profile_report(vb)
    vb.lib().vla_profile_enable(0)
    rows = S + A - 1 if wl.mode == 0 else S + A
    down_share = shape.hidden * shape.ffn / shape.layer_params          # the recomputed forward skips the down projection
    passes = 2.0 if args.backward_keep else 3.0 - down_share            # forward (+ forward again) + input gradients
    flops = passes * N * rows * 2.0 * shape.layer_params * shape.n_layers
    out = {"metric": "stored rollouts/sec, LoRA-gradient pass of the log-prob recompute (7B shape)", "value": N / (ms * 1e-3),
           "unit": "rollouts/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "bf16" if shape.dtype == "bf16" else "f32", "data": "synthetic",
           "config": {"workload": wl.name + " (backward)", "rollouts": N, "micro_batch": mb, "keep_activations": bool(args.backward_keep),
                      "rows_per_rollout": rows,
                      "lora_rank": rank, "layers": shape.n_layers, "hidden": shape.hidden},
           "phases": {"projection_TFLOPs": flops / (ms * 1e-3) / 1e12, "mfma_frac": flops / (ms * 1e-3) / 1e12 / MI355X_BF16_TFLOPS},
           "kernels": {k: {"n": v["count"], "ms": round(v["ms"], 3)} for k, v in sorted(prof.items(), key=lambda kv: -kv[1]["ms"])}}
    print(json.dumps(out))


def bench_pipeline(args, wl, torch, vb, run, patch, ids, gumbel, slot):
    """t_1 vs t_2 of section IV-A on one GPU: Generation on the GPU, a CPU-parallel stub simulator that
    takes sim_ms_per_env * (environments in the sub-batch) per step on the host."""
    from paper_2510_06710_amd.harness import PipelinedRollout
    B, S, A, m = wl.batch, wl.prefix, wl.n_action, args.chunks

    def halves(k):
        n = B // k
        return ([(patch[j * n:(j + 1) * n].contiguous(), ids[j * n:(j + 1) * n].contiguous()) for j in range(k)],
                [gumbel[j * n:(j + 1) * n].contiguous() for j in range(k)])

    def gen_ms(k):                                    # t_G at the sub-batch size, generation alone
        obs, g = halves(k)
        pr = PipelinedRollout(run, 1)
        pr.epoch([obs[0]], 1, S, A, lambda j, t, b: None, wl.mode, slot, wl.temperature, [g[0]])
        _, _, dt = pr.epoch([obs[0]], 2, S, A, lambda j, t, b: None, wl.mode, slot, wl.temperature, [g[0]])
        pr.close()
        return dt * 1e3 / 2

    t_gen = {k: gen_ms(k) for k in (1, 2)}
    per_env = args.sim_ms_per_env if args.sim_ms_per_env is not None else t_gen[1] / B
    out = {"metric": "rollout epoch time, collocated (k=1) vs pipelined (k=2), stub host simulator",
           "workload": wl.name, "chunks": m, "sim_ms_per_env": per_env, "modes": {}}
    for k in (1, 2):
        obs, g = halves(k)
        t_sim = per_env * (B // k)
        pr = PipelinedRollout(run, k)
        _, log, dt = pr.epoch(obs, m, S, A, lambda j, t, b: time.sleep(t_sim * 1e-3), wl.mode, slot, wl.temperature, g)
        pr.close()
        out["modes"][f"k{k}"] = {"measured_ms": dt * 1e3, "t_gen_ms": t_gen[k], "t_sim_ms": t_sim,
                                 "modelled_ms": vb.vla_pipeline_time(t_gen[k], t_sim, k, m),
                                 "env_actions_per_s": B * m / dt}
    out["speedup_measured"] = out["modes"]["k1"]["measured_ms"] / out["modes"]["k2"]["measured_ms"]
    out["speedup_modelled"] = out["modes"]["k1"]["modelled_ms"] / out["modes"]["k2"]["modelled_ms"]
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="cfg3_7b_b256")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sweep-batch", action="store_true",
                    help="time the step at batch sizes 1, 2, 4, ... up to the workload's batch: the t_G(.) "
                         "profile that the paper's auto-placement measures (section IV-A.3)")
    ap.add_argument("--pipeline", action="store_true",
                    help="rollout epoch against a timed stub simulator on the host: collocated schedule (k = 1) "
                         "vs fine-grained pipelining with two sub-batches (k = 2), measured and as modelled "
                         "(section IV-A)")
    ap.add_argument("--chunks", type=int, default=4, help="--pipeline: chunk steps per epoch (m)")
    ap.add_argument("--sim-ms-per-env", type=float, default=None,
                    help="--pipeline: stub simulator time per environment and step (default: the measured "
                         "generation time per environment, i.e. a 1:1 Generation:Simulator ratio)")
    ap.add_argument("--backward", action="store_true",
                    help="recompute workload only: time vla_logprob_backward (LoRA gradients) instead of the forward recompute")
    ap.add_argument("--backward-rollouts", type=int, default=64)
    ap.add_argument("--backward-micro-batch", type=int, default=32)
    ap.add_argument("--lora-rank", type=int, default=32)
    ap.add_argument("--backward-keep", action="store_true",
                    help="--backward: keep every layer's activations in the first pass (larger workspace) instead of "
                         "running each layer a second time")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also launch one 1 GiB plain copy kernel (reference for rocprofv3 --pmc traffic counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (environments shard "
              "by environment without any exchange, each GPU with a full weight replica). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    import vla_inputs as vi
    from paper_2510_06710_amd import binding as vb
    from paper_2510_06710_amd.harness import Rollout

    wl = vi.WORKLOADS[args.workload]
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    if wl.kind == "recompute":
        if args.backward:
            bench_backward(args, wl, torch, vi, vb, Rollout)
        else:
            bench_recompute(args, wl, torch, vi, vb, Rollout)
        return
    dev = "cuda:0"
    torch.cuda.set_device(0)
    B, S, A = wl.batch, wl.prefix, wl.n_action
    synth = vi.SynthModel(wl.shape, 0, device=dev)
    run = Rollout(synth, B, S + A + 1, device=dev, value_b=vi.VALUE_BIAS)
    patch, ids = vi.observation(wl, 0, device=dev)
    gumbel = vi.gumbel_noise(wl, 0, device=dev)
    slot = synth.slot_embed(A) if wl.mode == 1 else None
    stream = torch.cuda.current_stream()

    def prefill():
        return run.prefill(patch, ids, want_value=True, stream=stream)

    def decode(h_last):
        return run.decode(h_last, S, A, wl.mode, slot, wl.temperature, gumbel, want_logits=False, stream=stream)

    def step():
        h_last, _ = prefill()
        return decode(h_last)

    if args.sweep_batch:
        rows = []
        b = 1
        while b <= B:
            pb, ib, gb = patch[:b].contiguous(), ids[:b].contiguous(), gumbel[:b].contiguous()

            def step_b():
                h, _ = run.prefill(pb, ib, want_value=True, stream=stream)
                return run.decode(h, S, A, wl.mode, slot, wl.temperature, gb, want_logits=False, stream=stream)
            step_b()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                step_b()
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3 / args.steps
            rows.append({"batch": b, "ms_per_step": ms, "env_actions_per_s": b / (ms * 1e-3)})
            b *= 2
        print(json.dumps({"metric": "t_G(batch): generation step time vs batch size", "workload": wl.name,
                          "steps": args.steps, "sweep": rows}))
        return

    if args.pipeline:
        bench_pipeline(args, wl, torch, vb, run, patch, ids, gumbel, slot)
        return

    if args.calibration_copy:
        a = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        b = torch.zeros(1 << 30, dtype=torch.uint8, device=dev)
        vb.vla_calibration_copy(a, b, 1 << 30, stream)
        torch.cuda.synchronize()
        del a, b

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    # phase split (one more step, events on the launch stream)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    ev[0].record(stream)
    h_last, _ = prefill()
    ev[1].record(stream)
    decode(h_last)
    ev[2].record(stream)
    torch.cuda.synchronize()
    prefill_ms, decode_ms = ev[0].elapsed_time(ev[1]), ev[1].elapsed_time(ev[2])

    # instrumented passes: per-kernel time from HIP events recorded by the library around each launch
    vb.lib().vla_profile_enable(1)
    h_last, _ = prefill()
    torch.cuda.synchronize()
    prof_prefill = profile_report(vb)
    vb.lib().vla_profile_enable(1)
    decode(h_last)
    torch.cuda.synchronize()
    prof_decode = profile_report(vb)
    vb.lib().vla_profile_enable(0)

    shape = wl.shape
    dom = "gemm_bf16_dma<swiglu>"           # gate/up projection: the largest share of the step
    roofline = None
    if dom in prof_prefill:
        r = prof_prefill[dom]
        achieved = r["work"] / (r["ms"] * 1e-3) / 1e12
        traffic, traffic_source = read_traffic(os.path.join(ROOT, "profiles", "gemm_swiglu_cfg3_traffic.txt"),
                                               "gemm_bf16_dma_kernel<2, true, true>",
                                               os.path.join(ROOT, "paper_2510_06710_amd", "csrc", "gemm_dma.hip"))
        roofline = {"bound": "mfma", "kernel": "gemm_bf16_dma_kernel<EPI_SWIGLU, k-blocked, unit barrier> (gate/up projection, prefill)",
                    "achieved": achieved, "peak": MI355X_BF16_TFLOPS, "unit": "TFLOP/s",
                    "frac": achieved / MI355X_BF16_TFLOPS, "launches": r["count"],
                    "avg_launch_ms": r["ms"] / r["count"],
                    "flops_per_launch": r["work"] / r["count"],
                    "traffic": traffic if wl.name == "cfg3_7b_b256" else None, "traffic_source": traffic_source}
    # decode HBM accounting: weights once per forward + each environment's own K, V rows per forward
    kv_tok = 2 * shape.n_layers * shape.hidden * 2
    fwd = A - 1 if wl.mode == 0 else 1
    weight_bytes = shape.layer_params * shape.n_layers * 2
    if wl.mode == 0:
        kv_bytes = B * sum(S + j + 1 for j in range(A - 1)) * kv_tok
    else:
        kv_bytes = B * (S + A) * kv_tok
    decode_bytes = fwd * weight_bytes + kv_bytes
    decode_gbps = decode_bytes / (decode_ms * 1e-3) / 1e9
    prefill_flops = forward_flops(shape, B, S, 1 if S >= 4 else S)       # the last layer finishes the last prefix row only

    def table(p):
        return {k: {"n": v["count"], "ms": round(v["ms"], 3),
                    "rate": (round(v["work"] / (v["ms"] * 1e-3) / 1e12, 3) if v["work"] and v["ms"] else None)}
                for k, v in sorted(p.items(), key=lambda kv: -kv[1]["ms"])}

    out = {
        "metric": "env-actions/sec at batch 256 (7B shape), % HBM/MFMA roofline",
        "value": B / (ms_per_step * 1e-3), "unit": "env-actions/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if shape.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": wl.name, "batch": B, "prefix": S, "action_tokens": A,
                   "mode": "autoregressive" if wl.mode == 0 else "parallel_chunk", "layers": shape.n_layers,
                   "hidden": shape.hidden, "heads": shape.n_heads, "ffn": shape.ffn, "vocab": shape.vocab},
        "roofline": roofline,
        "phases": {"prefill_ms": prefill_ms, "decode_ms": decode_ms,
                   "decode_only_env_actions_per_s": B / (decode_ms * 1e-3),
                   "prefill_tokens_per_s": B * S / (prefill_ms * 1e-3),
                   "decode_tokens_per_s": B * A / (decode_ms * 1e-3),
                   "prefill_mfma_TFLOPs": prefill_flops / (prefill_ms * 1e-3) / 1e12,
                   "prefill_mfma_frac": prefill_flops / (prefill_ms * 1e-3) / 1e12 / MI355X_BF16_TFLOPS,
                   "decode_hbm_GBps": decode_gbps, "decode_hbm_frac": decode_gbps / MI355X_HBM_GBPS,
                   "decode_algorithmic_GB": decode_bytes / 1e9,
                   "prefill_executed_TFLOP": prefill_flops / 1e12,
                   "note": "last layer of the prefill: K, V for all rows, the rest for the last prefix row only (nothing else "
                           "is read); prefill_mfma_* count the executed flops"},
        "kernels_prefill": table(prof_prefill), "kernels_decode": table(prof_decode),
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, vi)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
