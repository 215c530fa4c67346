#!/usr/bin/env python3
"""Benchmark of the action-conditioned decoder-layer path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2|c2p|c3|c5|c4|c5d|c4p|refresh|episode|episodep]

A step is one pass of the measured unit over one batch of seeded synthetic input that is already
resident in HBM. Default workload: the Llama-3.2-1B-shaped decoder layer, 4 inputs x 8 schedules
x 1024 tokens, bf16, i.i.d. actions from the 4x4x4 action space (one sol_layer_forward call).
Prints ONE JSON line (metric, value, roofline of the dominant kernel measured with HIP events
around the library's stages, and the CPU oracle timed on a bounded sample).
"""
import argparse
import json
import math
import sys
import time

import numpy as np
import torch

from paper_2605_10875_amd import sol, synth

PEAK_BF16_TFLOPS = 2500.0    # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0        # MI355X HBM3E


def _dev(a, bf16=True):
    if np.issubdtype(a.dtype, np.integer):
        return torch.from_numpy(np.ascontiguousarray(a, np.int32)).cuda()
    t = torch.from_numpy(np.ascontiguousarray(a, np.float32)).cuda()
    return t.to(torch.bfloat16).contiguous() if bf16 else t


def layer_flops(shape, table, ids, pos):
    """Algorithmic FLOPs of one decoder layer for the realised actions (per-token terms: q/k/v,
    o, gate/up dense; down counted on the kept channels; all causal scores; P.V on the kept keys)."""
    d, hq, hkv, dh, dff = shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ff
    t = np.array(table, dtype=np.int64)[ids.reshape(-1)]
    n = pos.reshape(-1).astype(np.int64) + 1
    m = np.clip(-(-(t[:, 2] * dff) // t[:, 3]), 1, dff)
    k = np.clip(-(-(t[:, 0] * n) // t[:, 1]), 1, n)
    lin = 2 * d * (hq + 2 * hkv) * dh + 2 * hq * dh * d + 4 * d * dff
    return {"linear_dense": float(lin * len(n)), "down": float((2 * m * d).sum()),
            "qk": float((2 * hq * dh * n).sum()), "pv": float((2 * hq * dh * k).sum())}


def copy_calibration():
    """One plain device copy of known size (1 GiB read + 1 GiB written). It gives the hardware
    counters FETCH_SIZE / WRITE_SIZE a reference point in the same rocprofv3 --pmc run."""
    src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    del src, dst


def measured_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary (None if absent)."""
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "hbm_traffic.json")
    try:
        with open(path) as f:
            return json.load(f).get(workload, {}).get(kernel)
    except (OSError, ValueError):
        return None


def time_steps(fn, steps, warmup):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def stage_times(ctx, fn, steps):
    ctx.profile_enable(512 * steps + 64)
    for _ in range(steps):
        fn()
    st = ctx.profile_read()
    ctx.profile_enable(0)
    return {k: v[0] / steps for k, v in st.items()}, {k: v[1] // steps for k, v in st.items()}


def run_layer(args, shape, n_inputs, G, T, table, name, preset=None):
    n_seq = n_inputs * G
    w = synth.layer_weights(shape, args.seed, bf16=True)
    x = synth.hidden_states(n_seq, T, shape.d_model, args.seed + 1, bf16=True)
    ids = synth.iid_actions(len(table), (n_seq, T), args.seed + 2)
    ctx = sol.Sol(shape, table, dtype=sol.BF16, max_positions=T, **(preset or {}))
    wd = {k: _dev(v) for k, v in w.items()}
    xd, idd = _dev(x), _dev(ids)
    kc = torch.zeros((n_seq, shape.n_kv_heads, T, shape.head_dim), dtype=torch.bfloat16, device="cuda")
    vc = torch.zeros_like(kc)
    out = torch.empty_like(xd)
    ws = ctx.workspace(sol.OP_LAYER_FORWARD, n_seq, T, T)

    def step():
        ctx.layer_forward(wd, xd, idd, kc, vc, x_out=out, workspace=ws)

    sec = time_steps(step, args.steps, args.warmup)
    assert ctx.device_status() == sol.OK and bool(torch.isfinite(out.float()).all())
    stages, launches = stage_times(ctx, step, max(2, min(args.steps, 5)))
    tokens = n_seq * T
    pos = np.tile(np.arange(T), (n_seq, 1))
    fl = layer_flops(shape, table, ids, pos)
    alg = fl["linear_dense"] + fl["down"] + fl["qk"] + fl["pv"]
    dense = fl["linear_dense"] + 2.0 * shape.d_ff * shape.d_model * tokens + 2 * fl["qk"]
    dom = "gate_up_gemm"
    dom_flops = 4.0 * shape.d_model * shape.d_ff * tokens           # 4 d d_ff per token
    ach = dom_flops / (stages[dom] * 1e-3) / 1e12
    res = {
        "metric": "schedule_tokens_per_s", "value": tokens / sec, "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": sec * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": name, "entry_point": "sol_layer_forward", "n_inputs": n_inputs, "schedules": G,
                   "seq_len": T, "tokens_per_step": tokens, "actions": "iid uniform over %d" % len(table)},
        "roofline": {"bound": "mfma", "kernel": dom, "achieved": ach, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": ach / PEAK_BF16_TFLOPS, "traffic": measured_traffic(args.workload, dom),
                     "kernel_ms": stages[dom],
                     "launches_per_step": launches.get(dom)},
        "layer": {"algorithmic_tflop": alg / 1e12, "algorithmic_tflops": alg / sec / 1e12,
                  "algorithmic_frac_of_peak": alg / sec / 1e12 / PEAK_BF16_TFLOPS,
                  "dense_equivalent_tflops": dense / sec / 1e12},
        "stage_ms": {k: round(v, 4) for k, v in stages.items()},
    }
    if not args.no_cpu_baseline:
        import oracle
        cfg = oracle.make_cfg(shape, act_bf16=True)
        ns = min(n_seq, max(1, (6 * 1024 * 2048) // (T * shape.d_model)))   # about 15 s of oracle work on 16 cores
        kco = np.zeros((ns, shape.n_kv_heads, T, shape.head_dim), np.float32)
        t0 = time.perf_counter()
        ref, _ = oracle.layer_forward(cfg, oracle.make_table(table), w, x[:ns], ids[:ns], kco, kco.copy())
        dt = time.perf_counter() - t0
        got = out[:ns].float().cpu().numpy()
        err = (np.abs(got - ref).max(axis=2) / np.abs(ref).max()).ravel()
        res["cpu_baseline"] = {"value": ns * T / dt, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": "sequences 0..%d of %d, all %d tokens, one layer (%.1f s)" % (ns - 1, n_seq, T, dt),
                               "gpu_vs_oracle_row_err_median": float(np.median(err))}
    ctx.close()
    return res


def run_stack(args, shape, B, G, T, table, name):
    """Full stack + LM head + NLL (sol_schedule_loglik). Weights are drawn on the GPU (2.5 GB of them)."""
    gen = torch.Generator(device="cuda").manual_seed(args.seed)

    def rnd(*sz, std=0.02, mean=0.0):
        return (torch.randn(sz, generator=gen, device="cuda") * std + mean).to(torch.bfloat16)

    d, hq, hkv, dh, dff = shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ff
    layers = [{"w_in_norm": rnd(d, std=0.1, mean=1.0), "wq": rnd(hq * dh, d), "wk": rnd(hkv * dh, d),
               "wv": rnd(hkv * dh, d), "wo": rnd(d, hq * dh), "w_post_norm": rnd(d, std=0.1, mean=1.0),
               "w_gate": rnd(dff, d), "w_up": rnd(dff, d), "w_down": rnd(d, dff)} for _ in range(shape.n_layers)]
    head = {"embed": rnd(shape.vocab, d), "w_final_norm": rnd(d, std=0.1, mean=1.0), "lm_head": rnd(shape.vocab, d)}
    tokens, targets = synth.tokens_and_targets(B, T, shape.vocab, args.seed + 1)
    ids = synth.markov_actions(len(table), B * G, T, args.seed + 2).reshape(B, G, T)
    ctx = sol.Sol(shape, table, dtype=sol.BF16, max_positions=T)
    tk, tg, idd = _dev(tokens), _dev(targets), _dev(ids)
    nll = torch.empty((B, G, T), dtype=torch.float32, device="cuda")
    ws = ctx.workspace(sol.OP_SCHEDULE_LOGLIK, B * G, T, T)

    def step():
        ctx.schedule_loglik(layers, head, tk, tg, idd, nll_out=nll, workspace=ws)

    sec = time_steps(step, args.steps, args.warmup)
    assert ctx.device_status() == sol.OK and bool(torch.isfinite(nll).all())
    stages, launches = stage_times(ctx, step, 2)
    tokens_n = B * G * T
    pos = np.tile(np.arange(T), (B * G, 1))
    fl = layer_flops(shape, table, ids.reshape(B * G, T), pos)
    alg = shape.n_layers * (fl["linear_dense"] + fl["down"] + fl["qk"] + fl["pv"]) + 2.0 * d * shape.vocab * tokens_n
    dom = "gate_up_gemm"
    dom_flops = 4.0 * d * dff * tokens_n                             # per launch (one layer)
    per_launch_ms = stages[dom] / max(1, launches.get(dom, shape.n_layers))
    ach = dom_flops / (per_launch_ms * 1e-3) / 1e12
    res = {
        "metric": "schedule_tokens_per_s", "value": tokens_n / sec, "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": sec * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": name, "entry_point": "sol_schedule_loglik", "n_inputs": B, "schedules": G, "seq_len": T,
                   "layers": shape.n_layers, "vocab": shape.vocab, "tokens_per_step": tokens_n,
                   "actions": "Markov chain over %d actions, stay-probability 0.8" % len(table)},
        "roofline": {"bound": "mfma", "kernel": dom, "achieved": ach, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": ach / PEAK_BF16_TFLOPS, "traffic": None, "kernel_ms": per_launch_ms,
                     "launches_per_step": launches.get(dom)},
        "stack": {"algorithmic_tflop": alg / 1e12, "algorithmic_tflops": alg / sec / 1e12,
                  "algorithmic_frac_of_peak": alg / sec / 1e12 / PEAK_BF16_TFLOPS,
                  "mean_nll_nats": float(nll.mean()), "log_vocab": float(np.log(shape.vocab))},
        "stage_ms": {k: round(v, 4) for k, v in stages.items()},
    }
    # the step right after this pass: reward reduction on its NLL tensor (not part of the timed step)
    tg3 = torch.full((B, 3), 0.6, dtype=torch.float32, device="cuda")
    rw = lambda: ctx.reward_advantages(nll, idd, tg3, (4.0, 4.0, 4.0), 0.02, 0.85)
    rw()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        adv = rw()["adv"]
    e1.record()
    torch.cuda.synchronize()
    assert bool(torch.isfinite(adv).all())
    res["reward_reduction"] = {"entry_point": "sol_reward_advantages", "ms": e0.elapsed_time(e1) / 10,
                               "values": tokens_n, "note": "includes the binding's five output allocations"}
    ctx.close()
    return res


def run_decode(args, shape, B, L, table, name, n_layers, preset=None):
    """preset: None = exact per-key top-k, quantiser on the linear-layer inputs; a dict of configuration fields
    (sol.PAPER_PRESET) = that configuration, decoded with caller-kept page metadata."""
    import dataclasses
    shape = dataclasses.replace(shape, n_layers=n_layers)
    gen = torch.Generator(device="cuda").manual_seed(args.seed)
    layers = [synth.layer_weights(shape, args.seed + l, bf16=True) for l in range(1)]
    lw = [{k: _dev(v) for k, v in layers[0].items()} for _ in range(1)]
    # every layer gets its own weight tensors (distinct HBM) with the same seeded values
    lw = lw + [{k: v.clone() for k, v in lw[0].items()} for _ in range(n_layers - 1)]
    head = None
    L_max = L + 8
    kcs = [torch.randn((B, shape.n_kv_heads, L_max, shape.head_dim), generator=gen, device="cuda",
                       dtype=torch.float32).to(torch.bfloat16) for _ in range(n_layers)]
    vcs = [torch.randn((B, shape.n_kv_heads, L_max, shape.head_dim), generator=gen, device="cuda",
                       dtype=torch.float32).to(torch.bfloat16) for _ in range(n_layers)]
    ids = synth.iid_actions(len(table), (B,), args.seed + 2)
    x = _dev(synth.hidden_states(1, B, shape.d_model, args.seed + 3, bf16=True)[0])
    cache_len = torch.full((B,), L, dtype=torch.int32, device="cuda")
    ctx = sol.Sol(shape, table, dtype=sol.BF16, max_positions=L_max, **(preset or {}))
    idd = _dev(ids)
    ws = ctx.workspace(sol.OP_DECODE_STEP, B, 1, L_max)
    metas = [ctx.page_meta_build(k, cache_len) for k in kcs] if preset and preset.get("page_size", 1) > 1 else None

    def step():
        return ctx.decode_step(lw, head, idd, cache_len, kcs, vcs, x_in=x, workspace=ws, page_meta=metas)[0]

    # The step is ~200 short kernels; replaying them as one HIP graph removes the host launch gaps
    # (the library only enqueues kernels on the caller's stream, so the caller may capture it).
    x_out = torch.empty((B, shape.d_model), dtype=torch.bfloat16, device="cuda")
    for _ in range(2):
        step()
    torch.cuda.synchronize()
    sec_eager = time_steps(step, max(2, args.steps // 2), 1)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        hid_g = step()
    sec = time_steps(graph.replay, args.steps, args.warmup)
    hid = step()
    torch.cuda.synchronize()
    assert ctx.device_status() == sol.OK and bool(torch.isfinite(hid.float()).all())
    assert torch.equal(hid, hid_g), "graph replay and eager step disagree"
    del x_out
    stages, launches = stage_times(ctx, step, 2)
    # algorithmic bytes: weights once per layer, all of K, the V rows kept by at least one head of a group
    d, hq, hkv, dh, dff = shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ff
    wbytes = 2 * (d * (hq + 2 * hkv) * dh + hq * dh * d + 3 * d * dff)
    t = np.array(table, dtype=np.int64)[ids]
    n = L + 1
    kk = np.clip(-(-(t[:, 0] * n) // t[:, 1]), 1, n)
    g = hq // hkv
    union = n * (1.0 - (1.0 - kk / n) ** g)                  # expected distinct rows over g independent heads
    kv_bytes = float((hkv * dh * 2 * (n + union)).sum())
    if metas is not None:
        # page rule: the metadata rows (2 * dh values per page), then K and V rows of the pages kept by at least one
        # head of a group (expected distinct pages over g independent heads) and of the sink / window keys
        S = preset["page_size"]
        n_pages = -(-n // S)
        npg = np.minimum(-(-kk // S), n_pages)
        upages = np.where(kk >= n, n_pages, n_pages * (1.0 - (1.0 - npg / n_pages) ** g))
        rows = np.minimum(upages * S + preset.get("n_sink", 0) + preset.get("n_window", 0), n)
        kv_bytes = float((hkv * dh * 2 * (2 * n_pages + 2 * rows)).sum())
    alg_bytes = n_layers * (wbytes + kv_bytes)
    dom = "attention_topk"
    ach = (n_layers * kv_bytes) / (stages[dom] * 1e-3) / 1e9
    res = {
        "metric": "decode_tokens_per_s", "value": B / sec, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": sec * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": name, "entry_point": "sol_decode_step_paged" if metas is not None else "sol_decode_step",
                   "batch": B, "cache_len": L, "layers": n_layers,
                   "launch": "one HIP graph replay per step", "ms_per_step_eager_launches": sec_eager * 1e3},
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": ach / PEAK_HBM_GBS, "traffic": measured_traffic(args.workload, dom),
                     "kernel_ms": stages[dom] / n_layers,
                     "launches_per_step": launches.get(dom)},
        "step": {"algorithmic_gb": alg_bytes / 1e9, "algorithmic_gbs": alg_bytes / sec / 1e9,
                 "algorithmic_frac_of_peak": alg_bytes / sec / 1e9 / PEAK_HBM_GBS},
        "stage_ms": {k: round(v, 4) for k, v in stages.items()},
    }
    if not args.no_cpu_baseline:
        import oracle
        o_opts = dict(preset or {})
        k0 = [kcs[0][:1].float().cpu().numpy().copy()]
        v0 = [vcs[0][:1].float().cpu().numpy().copy()]
        one = dataclasses.replace(shape, n_layers=1)
        t0 = time.perf_counter()
        oracle.decode_step(oracle.make_cfg(one, act_bf16=True, **o_opts), oracle.make_table(table), layers[:1],
                           x[:1].float().cpu().numpy(), ids[:1], np.array([L], np.int32), k0, v0)
        dt = time.perf_counter() - t0
        res["cpu_baseline"] = {"value": 1.0 / (dt * n_layers), "unit": "tokens/s", "cores": oracle.num_threads(),
                               "kind": "oracle", "sample": "sequence 0 of %d, one layer timed (%.2f s), scaled to %d layers"
                               % (B, dt, n_layers)}
        del o_opts
    ctx.close()
    return res


def run_episode(args, shape, B, K, P, T, table, name, preset=None):
    """Episode pass (sol_episode_loglik): dense prefill of P tokens once per input, K schedules of T steps on it."""
    gen = torch.Generator(device="cuda").manual_seed(args.seed)

    def rnd(*sz, std=0.02, mean=0.0):
        return (torch.randn(sz, generator=gen, device="cuda") * std + mean).to(torch.bfloat16)

    d, hq, hkv, dh, dff = shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ff
    layers = [{"w_in_norm": rnd(d, std=0.1, mean=1.0), "wq": rnd(hq * dh, d), "wk": rnd(hkv * dh, d),
               "wv": rnd(hkv * dh, d), "wo": rnd(d, hq * dh), "w_post_norm": rnd(d, std=0.1, mean=1.0),
               "w_gate": rnd(dff, d), "w_up": rnd(dff, d), "w_down": rnd(d, dff)} for _ in range(shape.n_layers)]
    head = {"embed": rnd(shape.vocab, d), "w_final_norm": rnd(d, std=0.1, mean=1.0), "lm_head": rnd(shape.vocab, d)}
    rng = np.random.default_rng(args.seed)
    prefix = _dev(rng.integers(0, shape.vocab, (B, P)).astype(np.int32))
    tokens, targets = synth.tokens_and_targets(B, T, shape.vocab, args.seed + 1)
    ids = synth.markov_actions(len(table), B * K, T, args.seed + 2).reshape(B, K, T)
    ctx = sol.Sol(shape, table, dtype=sol.BF16, max_positions=P + T, **(preset or {}))
    tk, tg, idd = _dev(tokens), _dev(targets), _dev(ids)
    nll = torch.empty((B, K, T), dtype=torch.float32, device="cuda")
    need = int(ctx.L.sol_episode_workspace_bytes(ctx.cfg, B, K, P, T))
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")

    def step():
        ctx.episode_loglik(layers, head, prefix, tk, tg, idd, nll_out=nll, workspace=ws)

    sec = time_steps(step, args.steps, args.warmup)
    assert ctx.device_status() == sol.OK and bool(torch.isfinite(nll).all())
    stages, launches = stage_times(ctx, step, 2)
    dom = max(stages, key=stages.get)
    # dense flops: every linear layer for the B*P prefix tokens and the B*K*T controlled tokens, plus the LM head on the latter
    lin = 2.0 * (d * (hq + 2 * hkv) * dh + hq * dh * d + 3 * d * dff)
    alg = shape.n_layers * lin * (B * P + B * K * T) + 2.0 * d * shape.vocab * B * K * T
    res = {
        "metric": "controlled_steps_per_s", "value": B * K * T / sec, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": sec * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": name, "entry_point": "sol_episode_loglik", "n_inputs": B, "schedules": K, "prefix": P,
                   "steps_per_episode": T, "layers": shape.n_layers, "vocab": shape.vocab,
                   "tokens_through_the_stack": B * P + B * K * T, "same_work_without_sharing": B * K * (P + T),
                   "workspace_gb": need / 1e9},
        "roofline": {"bound": "mfma", "kernel": "whole pass (linear layers + LM head, dense flops)", "achieved": alg / sec / 1e12,
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": alg / sec / 1e12 / PEAK_BF16_TFLOPS, "traffic": None},
        "stage_ms": {k: round(v, 4) for k, v in stages.items()}, "slowest_stage": dom,
    }
    ctx.close()
    return res


def run_refresh(args, shape, B, L, T, n_layers, name):
    """Periodic KV-cache refresh: dense pass of the stack over the last T tokens of B sequences with L-token caches."""
    import dataclasses
    shape = dataclasses.replace(shape, n_layers=n_layers)
    gen = torch.Generator(device="cuda").manual_seed(args.seed)
    w0 = {k: _dev(v) for k, v in synth.layer_weights(shape, args.seed, bf16=True).items()}
    lw = [w0] + [{k: v.clone() for k, v in w0.items()} for _ in range(n_layers - 1)]
    L_max = L
    kcs = [torch.randn((B, shape.n_kv_heads, L_max, shape.head_dim), generator=gen, device="cuda",
                       dtype=torch.float32).to(torch.bfloat16) for _ in range(n_layers)]
    vcs = [torch.randn((B, shape.n_kv_heads, L_max, shape.head_dim), generator=gen, device="cuda",
                       dtype=torch.float32).to(torch.bfloat16) for _ in range(n_layers)]
    x = _dev(synth.hidden_states(B, T, shape.d_model, args.seed + 3, bf16=True))
    pos0 = torch.full((B,), L - T, dtype=torch.int32, device="cuda")
    ctx = sol.Sol(shape, [synth.DENSE_ACTION], dtype=sol.BF16, max_positions=L_max)
    ws = ctx.workspace(sol.OP_KV_REFRESH, B, T, L_max)

    def step():
        return ctx.kv_refresh(lw, None, pos0, kcs, vcs, x_in=x, workspace=ws)

    sec = time_steps(step, args.steps, args.warmup)
    out = step()
    torch.cuda.synchronize()
    assert ctx.device_status() == sol.OK and bool(torch.isfinite(out.float()).all())
    stages, launches = stage_times(ctx, step, 2)
    dom = max(stages, key=stages.get)
    d, hq, hkv, dh, dff = shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ff
    kv_bytes = 2.0 * B * hkv * L * dh * 2                        # all of K and V once per layer (T queries share them)
    ach = n_layers * kv_bytes / (stages["attention_topk"] * 1e-3) / 1e9
    return {
        "metric": "refreshed_tokens_per_s", "value": B * T / sec, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": sec * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": name, "entry_point": "sol_kv_refresh", "batch": B, "cache_len": L, "T": T, "layers": n_layers},
        "roofline": {"bound": "hbm", "kernel": "attention_topk", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": ach / PEAK_HBM_GBS, "traffic": None, "kernel_ms": stages["attention_topk"] / n_layers,
                     "launches_per_step": launches.get("attention_topk")},
        "stage_ms": {k: round(v, 4) for k, v in stages.items()}, "slowest_stage": dom,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c2", choices=["c2", "c2p", "c3", "c5", "c4", "c5d", "c4p", "refresh", "episode", "episodep"])
    ap.add_argument("--seed", type=int, default=1234)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (sequences are independent and would be sharded by input); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    copy_calibration()
    if args.workload == "c2":
        res = run_layer(args, synth.LLAMA_1B, 4, 8, 1024, synth.TABLE_C2,
                        "C2: Llama-3.2-1B-shaped decoder layer, bf16, 4 inputs x 8 schedules x 1024 tokens")
    elif args.workload == "c2p":
        res = run_layer(args, synth.LLAMA_1B, 4, 8, 1024, synth.TABLE_C2,
                        "C2 under the configuration of the paper's runs (pages of 16 keys, 4 sink + 2 window keys, pruning at the "
                        "MLP input, quantiser on the MLP output): Llama-3.2-1B-shaped decoder layer, bf16, 4 inputs x 8 schedules "
                        "x 1024 tokens", preset=sol.PAPER_PRESET)
    elif args.workload == "c3":
        import dataclasses
        shape = dataclasses.replace(synth.LLAMA_1B, n_layers=16, vocab=128256)
        res = run_stack(args, shape, 2, 8, 2048, synth.TABLE_C2,
                        "C3: Llama-3.2-1B-shaped 16-layer stack + LM head + NLL, bf16, 2 inputs x 8 schedules x 2048 tokens")
    elif args.workload == "c5":
        res = run_layer(args, synth.LLAMA_8B, 2, 4, 4096, synth.TABLE_C2,
                        "C5: Llama-3.1-8B-shaped decoder layer, bf16, 2 inputs x 4 schedules x 4096 tokens")
    elif args.workload == "c4":
        res = run_decode(args, synth.LLAMA_1B, 64, 8192, synth.TABLE_C4,
                         "C4: Llama-3.2-1B-shaped decode step, bf16, 64 sequences x 8192-token KV cache, 16 layers", 16)
    elif args.workload == "episode":
        import dataclasses
        shape = dataclasses.replace(synth.LLAMA_1B, n_layers=16, vocab=128256)
        res = run_episode(args, shape, 8, 32, 1024, 16, synth.TABLE_C2,
                          "Episode pass: Llama-3.2-1B-shaped 16-layer stack + LM head + NLL, bf16, 8 inputs, dense prefill of "
                          "1024 tokens once per input, 32 schedules x 16 controlled steps on it")
    elif args.workload == "episodep":
        import dataclasses
        shape = dataclasses.replace(synth.LLAMA_1B, n_layers=16, vocab=128256)
        res = run_episode(args, shape, 8, 32, 1024, 16, synth.TABLE_C2,
                          "Episode pass under the configuration of the paper's runs (pages of 16 keys, 4 sink + 2 window keys, "
                          "pruning at the MLP input, quantiser on the MLP output): Llama-3.2-1B-shaped 16-layer stack + LM head + "
                          "NLL, bf16, 8 inputs, dense prefill of 1024 tokens once per input, 32 schedules x 16 controlled steps "
                          "on it", preset=sol.PAPER_PRESET)
    elif args.workload == "refresh":
        res = run_refresh(args, synth.LLAMA_1B, 64, 4096, 16, 16,
                          "KV-cache refresh: Llama-3.2-1B-shaped 16-layer stack, bf16, 64 sequences x 4096-token caches, "
                          "dense pass over the last 16 tokens")
    elif args.workload == "c4p":
        res = run_decode(args, synth.LLAMA_1B, 64, 8192, synth.TABLE_C4,
                         "C4 under the configuration of the paper's runs (pages of 16 keys, 4 sink + 2 window keys, pruning at "
                         "the MLP input, quantiser on the MLP output), page metadata kept by the caller: Llama-3.2-1B-shaped "
                         "decode step, bf16, 64 sequences x 8192-token KV cache, 16 layers", 16, preset=sol.PAPER_PRESET)
    else:
        res = run_decode(args, synth.LLAMA_8B, 32, 8192, synth.TABLE_C2,
                         "C5-decode: Llama-3.1-8B-shaped decode step, bf16, 32 sequences x 8192-token KV cache, 1 layer", 1)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
