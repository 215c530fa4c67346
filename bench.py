#!/usr/bin/env python3
"""Benchmark of the action-conditioned decoder-layer path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload all|c2|c2p|c3|c5|c5p|c4|c5d|c4p|refresh|episode|episodep|libgemm]

A step is one pass of the measured unit over one batch of seeded synthetic input that is already
resident in HBM. Default (`all`): the headline is C3, the largest single-GPU configuration and the one
that runs the call the metric names (sol_schedule_loglik: Llama-3.2-1B-shaped 16-layer stack + LM head +
NLL, 2 inputs x 8 schedules x 2048 tokens, bursty Markov schedules); the other roofline configurations
(C2 and C5 layers, C4 and C5 decode steps) are timed in the same run and reported under "configs", each
with its own roofline and cpu_baseline, so that the one line covers both halves of the metric
(teacher-forced schedule-tokens/s and decode tokens/s). Prints ONE JSON line.

Timing: W warm-up steps, then K steps bracketed by synchronisations (`ms_per_step`, `value`); every step is
also bracketed by a pair of HIP events on the stream the library launches on, and the median of those K
intervals is reported beside it (`ms_per_step_event_median`). Kernel times for the roofline come from HIP
events the library records around its stages (sol_profile_*), on that same stream.
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


def kernel_sources_digest():
    """Digest of the kernel sources: counters collected for other sources than the ones that run are not quoted."""
    import glob
    import hashlib
    import os
    h = hashlib.sha1()
    root = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2605_10875_amd", "csrc")
    for p in sorted(glob.glob(os.path.join(root, "*.hip")) + glob.glob(os.path.join(root, "*.h"))):
        h.update(open(p, "rb").read())
    return h.hexdigest()[:16]


def measured_counters(workload, kernel):
    """What the committed rocprofv3 --pmc summaries (profiles/counters.json, written by bench_counters.py from
    runs of this file) hold for `kernel` of `workload`: {"traffic": HBM bytes per launch, "mfma_util": share of the
    kernel's busy cycles in which the matrix cores were busy, ...}; empty when absent or collected for other kernel
    sources than the ones that run now."""
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "counters.json")
    try:
        with open(path) as f:
            d = json.load(f)
    except (OSError, ValueError):
        return {}
    if d.get("kernel_sources_digest") != kernel_sources_digest():
        return {}
    return d.get(workload, {}).get(kernel, {})


def time_steps(fn, steps, warmup):
    """(seconds per step by the wall clock around `steps` steps, median seconds per step by HIP event pairs)"""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    t0 = time.perf_counter()
    for a, b in ev:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / steps
    return wall, float(np.median([a.elapsed_time(b) for a, b in ev])) * 1e-3


def roofline_counters(workload, kernel):
    c = measured_counters(workload, kernel)
    return {"traffic": c.get("traffic"), "mfma_util": c.get("mfma_util")}


def executed_mfma(workload, sec):
    """MFMA flops the step executed by the hardware counter (all kernels; profiles/counters.json), as TFLOP per step,
    TFLOP/s over this run's step time and fraction of the published peak; None without counters for these sources."""
    fl = measured_counters(workload, "step").get("mfma_executed_flops")
    if not fl:
        return {"mfma_executed_tflop": None, "mfma_executed_tflops": None, "mfma_executed_frac_of_peak": None}
    return {"mfma_executed_tflop": fl / 1e12, "mfma_executed_tflops": fl / sec / 1e12,
            "mfma_executed_frac_of_peak": fl / sec / 1e12 / PEAK_BF16_TFLOPS}


def stage_times(ctx, fn, steps):
    ctx.profile_enable(512 * steps + 64)
    for _ in range(steps):
        fn()
    st = ctx.profile_read()
    ctx.profile_enable(0)
    return {k: v[0] / steps for k, v in st.items()}, {k: v[1] // steps for k, v in st.items()}


def _record(metric, units, sec, sec_ev, args, name, config, dtype="bf16"):
    return {"metric": metric, "value": units / sec, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": sec * 1e3, "ms_per_step_event_median": sec_ev * 1e3,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": dtype, "data": "synthetic",
            "config": dict({"workload": name}, **config)}


def _mfma_roofline(workload, dom, flops_per_launch, stages, launches):
    per_launch_ms = stages[dom] / max(1, launches.get(dom, 1))
    ach = flops_per_launch / (per_launch_ms * 1e-3) / 1e12
    r = {"bound": "mfma", "kernel": dom, "achieved": ach, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
         "frac": ach / PEAK_BF16_TFLOPS, "kernel_ms": per_launch_ms, "launches_per_step": launches.get(dom)}
    r.update(roofline_counters(workload, dom))
    return r


def run_layer(args, shape, n_inputs, G, T, table, name, preset=None, workload="c2", oracle_tokens=2048):
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

    sec, sec_ev = time_steps(step, args.steps, args.warmup)
    assert ctx.device_status() == sol.OK and bool(torch.isfinite(out.float()).all())
    stages, launches = stage_times(ctx, step, max(2, min(args.steps, 5)))
    tokens = n_seq * T
    pos = np.tile(np.arange(T), (n_seq, 1))
    fl = layer_flops(shape, table, ids, pos)
    alg = fl["linear_dense"] + fl["down"] + fl["qk"] + fl["pv"]
    dense = fl["linear_dense"] + 2.0 * shape.d_ff * shape.d_model * tokens + 2 * fl["qk"]
    res = _record("schedule_tokens_per_s", tokens, sec, sec_ev, args, name,
                  {"entry_point": "sol_layer_forward", "n_inputs": n_inputs, "schedules": G, "seq_len": T,
                   "tokens_per_step": tokens, "actions": "iid uniform over %d" % len(table)})
    res["roofline"] = _mfma_roofline(workload, "gate_up_gemm", 4.0 * shape.d_model * shape.d_ff * tokens, stages, launches)
    res["layer"] = {"algorithmic_tflop": alg / 1e12, "algorithmic_tflops": alg / sec / 1e12,
                    "algorithmic_frac_of_peak": alg / sec / 1e12 / PEAK_BF16_TFLOPS,
                    "dense_equivalent_tflops": dense / sec / 1e12}
    res["layer"].update(executed_mfma(workload, sec))
    res["stage_ms"] = {k: round(v, 4) for k, v in stages.items()}
    if not args.no_cpu_baseline:
        import oracle
        cfg = oracle.make_cfg(shape, act_bf16=True, **(preset or {}))
        # a bounded sample: whole sequences while they fit `oracle_tokens` tokens of this shape, else the first
        # tokens of sequence 0 (causality: their results do not depend on the rest of the sequence)
        ns = max(1, min(n_seq, oracle_tokens // T))
        Tn = min(T, oracle_tokens)
        kco = np.zeros((ns, shape.n_kv_heads, Tn, shape.head_dim), np.float32)
        t0 = time.perf_counter()
        ref, _ = oracle.layer_forward(cfg, oracle.make_table(table), w, x[:ns, :Tn], ids[:ns, :Tn], kco, kco.copy())
        dt = time.perf_counter() - t0
        got = out[:ns, :Tn].float().cpu().numpy()
        err = (np.abs(got - ref).max(axis=2) / np.abs(ref).max()).ravel()
        res["cpu_baseline"] = {"value": ns * Tn / dt, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": "sequences 0..%d of %d, tokens 0..%d of %d, one layer (%.1f s)" % (ns - 1, n_seq, Tn - 1, T, dt),
                               "gpu_vs_oracle_row_err_median": float(np.median(err))}
    ctx.close()
    return res


def _gpu_stack_weights(args, shape):
    """Random-init stack drawn on the GPU (2.5 GB at the 1B shape): N(0, 0.02) matrices, norm gains 1 + N(0, 0.1)."""
    gen = torch.Generator(device="cuda").manual_seed(args.seed)

    def rnd(*sz, std=0.02, mean=0.0):
        return (torch.randn(sz, generator=gen, device="cuda") * std + mean).to(torch.bfloat16)

    d, hq, hkv, dh, dff = shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ff
    layers = [{"w_in_norm": rnd(d, std=0.1, mean=1.0), "wq": rnd(hq * dh, d), "wk": rnd(hkv * dh, d),
               "wv": rnd(hkv * dh, d), "wo": rnd(d, hq * dh), "w_post_norm": rnd(d, std=0.1, mean=1.0),
               "w_gate": rnd(dff, d), "w_up": rnd(dff, d), "w_down": rnd(d, dff)} for _ in range(shape.n_layers)]
    head = {"embed": rnd(shape.vocab, d), "w_final_norm": rnd(d, std=0.1, mean=1.0), "lm_head": rnd(shape.vocab, d)}
    return layers, head


def _host(t):
    return t.float().cpu().numpy()


def run_stack(args, shape, B, G, T, table, name, workload="c3"):
    """Full stack + LM head + NLL (sol_schedule_loglik). Weights are drawn on the GPU (2.5 GB of them)."""
    import dataclasses
    layers, head = _gpu_stack_weights(args, shape)
    d, dff = shape.d_model, shape.d_ff
    tokens, targets = synth.tokens_and_targets(B, T, shape.vocab, args.seed + 1)
    ids = synth.markov_actions(len(table), B * G, T, args.seed + 2).reshape(B, G, T)
    ctx = sol.Sol(shape, table, dtype=sol.BF16, max_positions=T)
    tk, tg, idd = _dev(tokens), _dev(targets), _dev(ids)
    nll = torch.empty((B, G, T), dtype=torch.float32, device="cuda")
    ws = ctx.workspace(sol.OP_SCHEDULE_LOGLIK, B * G, T, T)

    def step():
        ctx.schedule_loglik(layers, head, tk, tg, idd, nll_out=nll, workspace=ws)

    sec, sec_ev = time_steps(step, args.steps, args.warmup)
    assert ctx.device_status() == sol.OK and bool(torch.isfinite(nll).all())
    stages, launches = stage_times(ctx, step, 2)
    tokens_n = B * G * T
    pos = np.tile(np.arange(T), (B * G, 1))
    fl = layer_flops(shape, table, ids.reshape(B * G, T), pos)
    alg = shape.n_layers * (fl["linear_dense"] + fl["down"] + fl["qk"] + fl["pv"]) + 2.0 * d * shape.vocab * tokens_n
    res = _record("schedule_tokens_per_s", tokens_n, sec, sec_ev, args, name,
                  {"entry_point": "sol_schedule_loglik", "n_inputs": B, "schedules": G, "seq_len": T,
                   "layers": shape.n_layers, "vocab": shape.vocab, "tokens_per_step": tokens_n,
                   "actions": "Markov chain over %d actions, stay-probability 0.8" % len(table)})
    res["roofline"] = _mfma_roofline(workload, "gate_up_gemm", 4.0 * d * dff * tokens_n, stages, launches)
    res["stack"] = {"algorithmic_tflop": alg / 1e12, "algorithmic_tflops": alg / sec / 1e12,
                    "algorithmic_frac_of_peak": alg / sec / 1e12 / PEAK_BF16_TFLOPS,
                    "mean_nll_nats": float(nll.mean()), "log_vocab": float(np.log(shape.vocab))}
    res["stack"].update(executed_mfma(workload, sec))
    res["stage_ms"] = {k: round(v, 4) for k, v in stages.items()}
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
    if not args.no_cpu_baseline:
        # The oracle cannot run the whole stack in bounded time (2.4 GFLOP per token in fp64 loops): it is timed on
        # sequence 0 / schedule 0 through layer 0 at the full length, and on the final norm + LM head + NLL of the
        # first 128 positions, and the two are scaled to 16 layers and all positions of that sequence.
        import oracle
        w0 = {k: _host(v) for k, v in layers[0].items()}
        x0 = _host(head["embed"][tk[0].long()])[None]
        kco = np.zeros((1, shape.n_kv_heads, T, shape.head_dim), np.float32)
        t0 = time.perf_counter()
        oracle.layer_forward(oracle.make_cfg(shape, act_bf16=True), oracle.make_table(table), w0, x0, ids[0, :1], kco, kco.copy())
        t_layer = time.perf_counter() - t0
        n_head = 128
        none = dataclasses.replace(shape, n_layers=0)
        emb, wf, lm = _host(head["embed"]), _host(head["w_final_norm"]), _host(head["lm_head"])
        t0 = time.perf_counter()
        oracle.schedule_loglik(oracle.make_cfg(none, act_bf16=True), oracle.make_table(table), emb, [], wf, lm,
                               tokens[:1, :n_head], targets[:1, :n_head], ids[:1, :1, :n_head])
        t_head = time.perf_counter() - t0
        del emb, lm
        total = shape.n_layers * t_layer + t_head * T / n_head
        res["cpu_baseline"] = {"value": T / total, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": "sequence 0, schedule 0: layer 0 over all %d tokens (%.1f s) and final norm + LM head + "
                                         "NLL of %d positions (%.1f s), scaled to %d layers and %d positions"
                                         % (T, t_layer, n_head, t_head, shape.n_layers, T)}
    ctx.close()
    return res


def run_decode(args, shape, B, L, table, name, n_layers, preset=None, with_head=False, workload="c4"):
    """preset: None = exact per-key top-k, quantiser on the linear-layer inputs; a dict of configuration fields
    (sol.PAPER_PRESET) = that configuration, decoded with caller-kept page metadata. with_head: the step ends with the
    final norm, the LM head and the NLL of a target token."""
    import dataclasses
    shape = dataclasses.replace(shape, n_layers=n_layers)
    gen = torch.Generator(device="cuda").manual_seed(args.seed)
    layers = [synth.layer_weights(shape, args.seed + l, bf16=True) for l in range(1)]
    lw = [{k: _dev(v) for k, v in layers[0].items()} for _ in range(1)]
    # every layer gets its own weight tensors (distinct HBM) with the same seeded values
    lw = lw + [{k: v.clone() for k, v in lw[0].items()} for _ in range(n_layers - 1)]
    head, targets = None, None
    if with_head:
        head = {"embed": None,
                "w_final_norm": (torch.randn(shape.d_model, generator=gen, device="cuda") * 0.1 + 1.0).to(torch.bfloat16),
                "lm_head": (torch.randn((shape.vocab, shape.d_model), generator=gen, device="cuda") * 0.02).to(torch.bfloat16)}
        targets = _dev(np.random.default_rng(args.seed + 5).integers(0, shape.vocab, B).astype(np.int32))
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
    k0_before = kcs[0][:2].float().cpu().numpy().copy()         # for the oracle leg (the step appends to the caches)
    v0_before = vcs[0][:2].float().cpu().numpy().copy()

    def step():
        return ctx.decode_step(lw, head, idd, cache_len, kcs, vcs, x_in=x, workspace=ws, page_meta=metas, targets=targets)

    # The step is ~200 short kernels; replaying them as one HIP graph removes the host launch gaps
    # (the library only enqueues kernels on the caller's stream, so the caller may capture it).
    for _ in range(2):
        step()
    torch.cuda.synchronize()
    sec_eager, _ = time_steps(step, max(2, args.steps // 2), 1)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        hid_g, nll_g = step()
    sec, sec_ev = time_steps(graph.replay, args.steps, args.warmup)
    hid, nll = step()
    torch.cuda.synchronize()
    assert ctx.device_status() == sol.OK and bool(torch.isfinite(hid.float()).all())
    assert torch.equal(hid, hid_g), "graph replay and eager step disagree"
    if with_head:
        assert bool(torch.isfinite(nll).all()) and torch.equal(nll, nll_g)
    stages, launches = stage_times(ctx, step, 2)
    # algorithmic bytes: weights once per layer, all of K, the V rows kept by at least one head of a group
    d, hq, hkv, dh, dff = shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ff
    wbytes = 2 * (d * (hq + 2 * hkv) * dh + hq * dh * d + 3 * d * dff)
    t = np.array(table, dtype=np.int64)[ids]
    n = L + 1
    kk = np.clip(-(-(t[:, 0] * n) // t[:, 1]), 1, n)
    g = hq // hkv
    union = n * (1.0 - (1.0 - kk / n) ** g)                  # expected distinct rows over g independent heads
    union_note = "expected union over %d independent heads" % g
    cpu = None
    if not args.no_cpu_baseline:
        # oracle on sequences 0 and 1, layer 0: timed, and its realised kept sets give the distinct V rows per KV
        # group, which correct the expectation used for the other sequences
        import oracle
        o_opts = dict(preset or {})
        one = dataclasses.replace(shape, n_layers=1)
        ns = min(2, B)
        t0 = time.perf_counter()
        _, taps = oracle.layer_forward(oracle.make_cfg(one, act_bf16=True, **o_opts), oracle.make_table(table), layers[0],
                                       x[:ns].float().cpu().numpy()[:, None, :], ids[:ns, None], k0_before[:ns], v0_before[:ns],
                                       pos0=np.full(ns, L, np.int32), taps=("keep_mask",))
        dt = time.perf_counter() - t0
        km = taps["keep_mask"][:, 0].reshape(ns, hkv, g, L_max)           # [seq][kv head][head of the group][key]
        realised = km.any(axis=2).sum(axis=2).mean(axis=1)               # distinct rows per KV head, averaged over KV heads
        ratio = float((realised / union[:ns]).mean())
        union = union * ratio
        union_note = ("expected union over %d independent heads, scaled by %.4f = realised / expected distinct V rows of the "
                      "oracle's kept sets for sequences 0..%d in layer 0" % (g, ratio, ns - 1))
        cpu = {"value": ns / (dt * n_layers), "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": "sequences 0..%d of %d, one layer timed (%.2f s), scaled to %d layers%s"
               % (ns - 1, B, dt, n_layers, "; final norm + LM head + NLL not included" if with_head else "")}
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
        union_note = "expected distinct pages over %d independent heads" % g
    head_bytes = 2.0 * shape.vocab * d if with_head else 0.0
    alg_bytes = n_layers * (wbytes + kv_bytes) + head_bytes
    dom = "attention_topk"
    per_launch_ms = stages[dom] / n_layers
    ach = kv_bytes / (per_launch_ms * 1e-3) / 1e9
    res = _record("decode_tokens_per_s", B, sec, sec_ev, args, name,
                  {"entry_point": "sol_decode_step_paged" if metas is not None else "sol_decode_step",
                   "batch": B, "cache_len": L, "layers": n_layers, "lm_head_and_nll": bool(with_head),
                   "launch": "one HIP graph replay per step", "ms_per_step_eager_launches": sec_eager * 1e3})
    res["roofline"] = {"bound": "hbm", "kernel": dom, "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                       "frac": ach / PEAK_HBM_GBS, "kernel_ms": per_launch_ms, "launches_per_step": launches.get(dom),
                       "v_rows": union_note}
    res["roofline"].update(roofline_counters(workload, dom))
    res["step"] = {"algorithmic_gb": alg_bytes / 1e9, "algorithmic_gbs": alg_bytes / sec / 1e9,
                   "algorithmic_frac_of_peak": alg_bytes / sec / 1e9 / PEAK_HBM_GBS}
    # what the counters saw the whole step move (FETCH_SIZE + WRITE_SIZE over all kernels; profiles/counters.json)
    mc = measured_counters(workload, "step")
    moved = (mc.get("fetch_bytes") or 0) + (mc.get("write_bytes") or 0)
    res["step"].update({"measured_gb": moved / 1e9 if moved else None, "measured_gbs": moved / sec / 1e9 if moved else None,
                        "measured_frac_of_peak": moved / sec / 1e9 / PEAK_HBM_GBS if moved else None})
    res["stage_ms"] = {k: round(v, 4) for k, v in stages.items()}
    if cpu:
        res["cpu_baseline"] = cpu
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

    sec, sec_ev = time_steps(step, args.steps, args.warmup)
    assert ctx.device_status() == sol.OK and bool(torch.isfinite(nll).all())
    stages, launches = stage_times(ctx, step, 2)
    dom = max(stages, key=stages.get)
    # dense flops: every linear layer for the B*P prefix tokens and the B*K*T controlled tokens, plus the LM head on the latter
    lin = 2.0 * (d * (hq + 2 * hkv) * dh + hq * dh * d + 3 * d * dff)
    alg = shape.n_layers * lin * (B * P + B * K * T) + 2.0 * d * shape.vocab * B * K * T
    res = {
        "metric": "controlled_steps_per_s", "value": B * K * T / sec, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": sec * 1e3, "ms_per_step_event_median": sec_ev * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
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

    sec, sec_ev = time_steps(step, args.steps, args.warmup)
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
        "warmup": args.warmup, "ms_per_step": sec * 1e3, "ms_per_step_event_median": sec_ev * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": name, "entry_point": "sol_kv_refresh", "batch": B, "cache_len": L, "T": T, "layers": n_layers},
        "roofline": {"bound": "hbm", "kernel": "attention_topk", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": ach / PEAK_HBM_GBS, "traffic": None, "kernel_ms": stages["attention_topk"] / n_layers,
                     "launches_per_step": launches.get("attention_topk")},
        "stage_ms": {k: round(v, 4) for k, v in stages.items()}, "slowest_stage": dom,
    }


LAYER_1B = "Llama-3.2-1B-shaped decoder layer, bf16, 4 inputs x 8 schedules x 1024 tokens"
PAPER_CFG = ("the configuration of the paper's runs (pages of 16 keys, 4 sink + 2 window keys, pruning at the MLP input, "
             "quantiser on the MLP output)")


def run_workload(args, wl):
    import dataclasses
    stack_shape = dataclasses.replace(synth.LLAMA_1B, n_layers=16, vocab=128256)
    if wl == "c2":
        return run_layer(args, synth.LLAMA_1B, 4, 8, 1024, synth.TABLE_C2, "C2: " + LAYER_1B, workload=wl)
    if wl == "c2p":
        return run_layer(args, synth.LLAMA_1B, 4, 8, 1024, synth.TABLE_C2, "C2 under " + PAPER_CFG + ": " + LAYER_1B,
                         preset=sol.PAPER_PRESET, workload=wl)
    if wl == "c3":
        return run_stack(args, stack_shape, 2, 8, 2048, synth.TABLE_C2,
                         "C3: Llama-3.2-1B-shaped 16-layer stack + LM head + NLL, bf16, 2 inputs x 8 schedules x 2048 tokens",
                         workload=wl)
    if wl == "c5":
        return run_layer(args, synth.LLAMA_8B, 2, 4, 4096, synth.TABLE_C2,
                         "C5: Llama-3.1-8B-shaped decoder layer, bf16, 2 inputs x 4 schedules x 4096 tokens", workload=wl,
                         oracle_tokens=768)
    if wl == "c5p":
        return run_layer(args, synth.LLAMA_8B, 2, 4, 4096, synth.TABLE_C2,
                         "C5 under " + PAPER_CFG + ": Llama-3.1-8B-shaped decoder layer, bf16, 2 inputs x 4 schedules x 4096 "
                         "tokens", preset=sol.PAPER_PRESET, workload=wl, oracle_tokens=768)
    if wl == "c4":
        return run_decode(args, stack_shape, 64, 8192, synth.TABLE_C4,
                          "C4: Llama-3.2-1B-shaped decode step, bf16, 64 sequences x 8192-token KV cache, 16 layers + final "
                          "norm + LM head + NLL", 16, with_head=True, workload=wl)
    if wl == "c4p":
        return run_decode(args, stack_shape, 64, 8192, synth.TABLE_C4,
                          "C4 under " + PAPER_CFG + ", page metadata kept by the caller: Llama-3.2-1B-shaped decode step, "
                          "bf16, 64 sequences x 8192-token KV cache, 16 layers + final norm + LM head + NLL", 16,
                          preset=sol.PAPER_PRESET, with_head=True, workload=wl)
    if wl == "c5d":
        return run_decode(args, synth.LLAMA_8B, 32, 8192, synth.TABLE_C2,
                          "C5-decode: Llama-3.1-8B-shaped decode step, bf16, 32 sequences x 8192-token KV cache, 1 layer", 1,
                          workload=wl)
    if wl == "episode":
        return run_episode(args, stack_shape, 8, 32, 1024, 16, synth.TABLE_C2,
                           "Episode pass: Llama-3.2-1B-shaped 16-layer stack + LM head + NLL, bf16, 8 inputs, dense prefill of "
                           "1024 tokens once per input, 32 schedules x 16 controlled steps on it")
    if wl == "episodep":
        return run_episode(args, stack_shape, 8, 32, 1024, 16, synth.TABLE_C2,
                           "Episode pass under " + PAPER_CFG + ": Llama-3.2-1B-shaped 16-layer stack + LM head + NLL, bf16, 8 "
                           "inputs, dense prefill of 1024 tokens once per input, 32 schedules x 16 controlled steps on it",
                           preset=sol.PAPER_PRESET)
    if wl == "refresh":
        return run_refresh(args, synth.LLAMA_1B, 64, 4096, 16, 16,
                           "KV-cache refresh: Llama-3.2-1B-shaped 16-layer stack, bf16, 64 sequences x 4096-token caches, "
                           "dense pass over the last 16 tokens")
    raise ValueError(wl)


def run_libgemm(args):
    """For scale only, not part of the product path: the plain bf16 GEMM that PyTorch dispatches to the vendor library
    (no epilogue, C written as bf16) on the shapes of the layer GEMMs and the LM head, timed with events."""
    shapes = [("gate_up_1b", 32768, 16384, 2048), ("down_1b", 32768, 2048, 8192), ("qkv_1b", 32768, 3072, 2048),
              ("o_proj_1b", 32768, 2048, 2048), ("gate_up_8b", 32768, 28672, 4096), ("down_8b", 32768, 4096, 14336),
              ("lm_head_1b", 32768, 128256, 2048)]
    out = {}
    g = torch.Generator(device="cuda").manual_seed(args.seed)
    for name, M, N, K in shapes:
        a = torch.randn((M, K), device="cuda", dtype=torch.float32, generator=g).to(torch.bfloat16)
        w = torch.randn((N, K), device="cuda", dtype=torch.float32, generator=g).to(torch.bfloat16)
        iters = max(3, min(args.steps, 5 if N > 100000 else args.steps))
        for _ in range(max(1, min(args.warmup, 3))):
            c = a @ w.t()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(iters):
            c = a @ w.t()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / iters
        out[name] = {"M": M, "N": N, "K": K, "ms": ms, "tflops": 2.0 * M * N * K / ms / 1e9}
        del a, w, c
        torch.cuda.empty_cache()
    return {"metric": "library_gemm_tflops", "value": out["gate_up_1b"]["tflops"], "unit": "TFLOP/s", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "ms_per_step": out["gate_up_1b"]["ms"], "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": "plain bf16 GEMMs of the vendor library via torch.matmul on the layer's shapes (comparison only)"},
            "roofline": {"bound": "mfma", "achieved": out["gate_up_1b"]["tflops"], "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                         "frac": out["gate_up_1b"]["tflops"] / PEAK_BF16_TFLOPS, "traffic": None},
            "shapes": out}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="all",
                    choices=["all", "c2", "c2p", "c3", "c5", "c5p", "c4", "c5d", "c4p", "refresh", "episode", "episodep", "libgemm"])
    ap.add_argument("--seed", type=int, default=1234)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-peaks", action="store_true", help="skip the two peak microbenchmarks")
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
    peaks = None
    if not args.no_peaks:
        tf, gb, rd = sol.measure_peaks()
        peaks = {"mfma_bf16_tflops": tf, "mfma_bf16_published": PEAK_BF16_TFLOPS, "hbm_copy_gbs": gb, "hbm_read_gbs": rd,
                 "hbm_published": PEAK_HBM_GBS,
                 "note": "register-only 32x32x16 bf16 MFMA loop on every SIMD; 1 GiB device copy (bytes read + written); "
                         "read-only sweep of 1 GiB"}
    if args.workload == "all":
        res = run_workload(args, "c3")
        res["configs"] = {}
        for wl in ("c2", "c5", "c4", "c5d"):
            torch.cuda.empty_cache()
            sub = run_workload(args, wl)
            for k in ("n_gpus", "steps", "warmup", "higher_is_better", "scaling", "vs_baseline", "data"):
                sub.pop(k, None)
            res["configs"][wl] = sub
    elif args.workload == "libgemm":
        res = run_libgemm(args)
    else:
        res = run_workload(args, args.workload)
    if peaks:
        res["measured_peaks"] = peaks
        for rec in [res] + list(res.get("configs", {}).values()):
            r = rec["roofline"]
            if r.get("bound") in ("mfma", "hbm") and "achieved" in r:
                r["frac_of_measured_peak"] = r["achieved"] / (peaks["mfma_bf16_tflops"] if r["bound"] == "mfma" else max(peaks["hbm_copy_gbs"], peaks["hbm_read_gbs"]))
    print(json.dumps(res))


if __name__ == "__main__":
    main()
