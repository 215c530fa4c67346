"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times, checked on
sampled sequences the oracle can compute on its own (sequences are independent), plus the long-row
variants of the tiled attention kernel."""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
from paper_2605_10875_amd import sol, synth

from gpu_util import check_rows, dev, dev_weights, host

pytestmark = pytest.mark.gpu


def _check_by_bits(out, ref, ids, table, what, pages=False):
    bits = np.array([a[4] for a in table])[ids]
    for b in sorted(set(bits.reshape(-1).tolist())):
        if b >= 16:     # selection / pruning flips only: 2e-2, with a per-cent of rows allowed up to 5e-2 (a swapped
            # key weighs ~1/k of a short row; 1 row in 256 was seen at 2.06e-2 at this size); a swapped page of 16
            # keys weighs more: 5 % of the rows up to 5e-2 under the page rule
            check_rows(out[bits == b], ref[bits == b], 2e-2, 5e-2, 0.05 if pages else 0.01, f"{what}: rows of {b}-bit actions")
        else:
            cap = max(2e-2, 6.0 / 2 ** (b - 1))
            check_rows(out[bits == b], ref[bits == b], cap, cap, 0.0, f"{what}: rows of {b}-bit actions")


@pytest.mark.parametrize("preset", [None, sol.PAPER_PRESET], ids=["exact-topk", "paper-configuration"])
def test_c2_full_size_layer_sampled_sequences(preset):
    """Llama-3.2-1B layer, 32 sequences x 1024 tokens (bench.py's default step), sequences 0 and 17. Second case: the
    configuration of the paper's runs (bench.py's c2p: the tiled kernels under the page rule)."""
    shape, table, n_seq, T, seed = synth.LLAMA_1B, synth.TABLE_C2, 32, 1024, 1234
    opts = dict(preset or {})
    qs = opts.pop("quant_sites", oracle.QS_NORTHSTAR)
    w = synth.layer_weights(shape, seed, bf16=True)
    x = synth.hidden_states(n_seq, T, shape.d_model, seed + 1, bf16=True)
    ids = synth.iid_actions(len(table), (n_seq, T), seed + 2)
    ctx = sol.Sol(shape, table, dtype=sol.BF16, max_positions=T, quant_sites=qs, **opts)
    kc = torch.zeros((n_seq, shape.n_kv_heads, T, shape.head_dim), dtype=torch.bfloat16, device="cuda")
    vc = torch.zeros_like(kc)
    out = ctx.layer_forward(dev_weights(w, sol.BF16), dev(x, sol.BF16), dev(ids), kc, vc)
    assert ctx.device_status() == sol.OK
    for s in (0, 17):
        kr = np.zeros((1, shape.n_kv_heads, T, shape.head_dim), np.float32)
        vr = kr.copy()
        ref, _ = oracle.layer_forward(oracle.make_cfg(shape, quant_sites=qs, act_bf16=True, **opts), oracle.make_table(table),
                                      w, x[s:s + 1], ids[s:s + 1], kr, vr)
        check_rows(host(kc[s]).transpose(1, 0, 2), kr[0].transpose(1, 0, 2), 2e-2, 0.3, 0.02, f"seq {s} K cache")
        check_rows(host(vc[s]).transpose(1, 0, 2), vr[0].transpose(1, 0, 2), 2e-2, 0.3, 0.02, f"seq {s} V cache")
        _check_by_bits(host(out[s]), ref[0], ids[s], table, f"seq {s}", pages=bool(preset))
    # a sequence's result does not depend on the batch around it: rerun sequence 17 alone, compare bits
    solo_k = torch.zeros((1, shape.n_kv_heads, T, shape.head_dim), dtype=torch.bfloat16, device="cuda")
    solo = ctx.layer_forward(dev_weights(w, sol.BF16), dev(x[17:18], sol.BF16), dev(ids[17:18]), solo_k,
                             torch.zeros_like(solo_k))
    assert torch.equal(solo[0], out[17])
    ctx.close()


@pytest.mark.parametrize("preset", [None, sol.PAPER_PRESET], ids=["exact-topk", "paper-configuration"])
def test_c4_full_size_decode_sampled_sequence(preset):
    """Llama-3.2-1B decode step, 64 sequences x 8192-token caches x 16 layers; sequence 5 against the oracle.
    Second case: the configuration of the paper's runs, decoded with caller-kept page metadata (bench.py's c4p)."""
    opts = dict(preset or {})
    qs = opts.pop("quant_sites", oracle.QS_NORTHSTAR)
    shape = dataclasses.replace(synth.LLAMA_1B, n_layers=16, vocab=4096)
    table, B, L, seed = synth.TABLE_C4, 64, 8192, 1234
    L_max = L + 8
    gen = torch.Generator(device="cuda").manual_seed(seed)
    layers = [synth.layer_weights(shape, seed + l, bf16=True) for l in range(shape.n_layers)]
    head = synth.head_weights(shape, seed + 100, bf16=True)
    kcs = [torch.randn((B, shape.n_kv_heads, L_max, shape.head_dim), generator=gen, device="cuda").to(torch.bfloat16)
           for _ in range(shape.n_layers)]
    vcs = [torch.randn((B, shape.n_kv_heads, L_max, shape.head_dim), generator=gen, device="cuda").to(torch.bfloat16)
           for _ in range(shape.n_layers)]
    ids = synth.iid_actions(len(table), (B,), seed + 2)
    x = synth.hidden_states(1, B, shape.d_model, seed + 3, bf16=True)[0]
    rng = np.random.default_rng(seed + 4)
    cache_len = rng.integers(L // 2, L + 1, B).astype(np.int32)
    cache_len[5] = L
    targets = rng.integers(0, shape.vocab, B).astype(np.int32)
    s = 5
    k_host = [k[s:s + 1].float().cpu().numpy().copy() for k in kcs]
    v_host = [v[s:s + 1].float().cpu().numpy().copy() for v in vcs]
    ctx = sol.Sol(shape, table, dtype=sol.BF16, max_positions=L_max, quant_sites=qs, **opts)
    metas = [ctx.page_meta_build(k, dev(cache_len)) for k in kcs] if preset else None
    hid, nll = ctx.decode_step([dev_weights(w, sol.BF16) for w in layers], dev_weights(head, sol.BF16), dev(ids),
                               dev(cache_len), kcs, vcs, x_in=dev(x, sol.BF16), targets=dev(targets), page_meta=metas)
    assert ctx.device_status() == sol.OK
    # oracle with one quantising-free copy of the action is not needed: compare layer 0's committed K/V
    # exactly-ish and the final hidden state with the bit-width bound of the sequence's action
    h_ref, nll_ref = oracle.decode_step(oracle.make_cfg(shape, quant_sites=qs, act_bf16=True, **opts), oracle.make_table(table), layers,
                                        x[s:s + 1], ids[s:s + 1], cache_len[s:s + 1], k_host, v_host,
                                        head["w_final_norm"], head["lm_head"], targets[s:s + 1])
    p = int(cache_len[s])
    check_rows(host(kcs[0][s, :, p]), k_host[0][0, :, p], 2e-2, 2e-2, 0.0, "layer-0 K row of the new token")
    check_rows(host(vcs[0][s, :, p]), v_host[0][0, :, p], 2e-2, 2e-2, 0.0, "layer-0 V row of the new token")
    bits = table[ids[s]][4]
    cap = 2e-2 if bits >= 16 else max(2e-2, 6.0 / 2 ** (bits - 1))
    err = float(np.abs(host(hid)[s] - h_ref[0]).max() / np.abs(h_ref).max())
    print(f"decode seq {s}: action {table[ids[s]]}, hidden max-rel {err:.3e} (cap {cap:.2e}), "
          f"nll gpu {float(nll[s]):.4f} oracle {float(nll_ref[0]):.4f}")
    assert err < 16 * cap            # 16 layers: every layer may flip codes of its own
    assert np.isfinite(host(nll)).all() and np.isfinite(host(hid)).all()
    ctx.close()


LONG = synth.ModelShape(d_model=256, n_q_heads=8, n_kv_heads=2, head_dim=64, d_ff=512, n_layers=1, vocab=100)
NOQUANT = synth.action_table((0.125, 0.25, 0.5, 1.0), (0.0, 0.5), (16,))


@pytest.mark.parametrize("T", [1100, 2100, 4096])
def test_long_rows_of_the_tiled_attention(T):
    """Rows of 1025..2048 and 2049..4096 keys take the 16- and 8-row variants of the tiled kernel."""
    shape, table = LONG, NOQUANT
    w = synth.layer_weights(shape, 7000, bf16=True, std=0.05)
    x = synth.hidden_states(1, T, shape.d_model, 7001, bf16=True)
    ids = synth.iid_actions(len(table), (1, T), 7002)
    ctx = sol.Sol(shape, table, dtype=sol.BF16, max_positions=T)
    kc = torch.zeros((1, shape.n_kv_heads, T, shape.head_dim), dtype=torch.bfloat16, device="cuda")
    vc = torch.zeros_like(kc)
    out = host(ctx.layer_forward(dev_weights(w, sol.BF16), dev(x, sol.BF16), dev(ids), kc, vc))
    assert ctx.device_status() == sol.OK
    kr = np.zeros((1, shape.n_kv_heads, T, shape.head_dim), np.float32)
    ref, _ = oracle.layer_forward(oracle.make_cfg(shape, act_bf16=True), oracle.make_table(table), w, x, ids, kr,
                                  kr.copy())
    check_rows(out, ref, 2e-2, 2e-2, 0.0, f"T={T}, selection and pruning only", median=1e-2)
    ctx.close()
