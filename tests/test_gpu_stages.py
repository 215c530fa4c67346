"""Stage-wise GPU parity: one stage of the layer at a time, fed with the ORACLE's inputs of that stage, so that
a row crosses at most one quantiser before it is compared and the bound does not have to absorb flips that
earlier stages amplified.

Attention stage (q, K, V -> o): no quantiser inside. Both sides read the same bf16 q, K, V. The GPU forms scores
by bf16 MFMA with fp32 sums, probabilities in fp32 split into two bf16 halves, and sums P.V in fp32; the oracle
sums in fp64. Expected difference of a row: about 2^-17 (the split of the probabilities) plus fp32 summation noise,
far below 1e-4 of the row's largest value, unless a near-tie at the threshold swaps one key, which moves the row by
at most that key's weight (it is the smallest kept weight, so at most 1 / budget). Asserted: every row within 2e-2,
median row within 1e-4, at most 1 % of rows over 1e-3. The codes of the quantiser that follows (input of the output
projection) are compared as integers: with eps the relative difference of the two inputs, a code flips by one step
with probability about 2 q_max eps per element (the chance that a rounding boundary lies between the two values),
never by more; asserted with eps = 1e-4: off-by-one share <= 2 q_max 1e-4 + 1e-4, none beyond one step.

MLP stage (h2, x2 -> a -> out): one quantiser (input of the down projection). Both sides read the same bf16 h2.
gate / up sums are fp32 (GPU) against fp64 (oracle): relative difference about sqrt(d) 2^-24 ~ 3e-6, then both
round SiLU(gate)*up to bf16: a share of about 3e-6 / 2^-9 ~ 2e-3 of the elements lands on neighbouring bf16 values
(0.4 - 0.8 % apart). Such an element changes its code with probability ~ |code| * 0.6 %, and if it is the row's
largest it rescales the whole row by one bf16 step. Asserted per bit class: no code differs by more than one step,
at most 1 % of the codes differ by one step, the kept-channel sets differ in at most 0.1 % of their members, 16-bit
rows agree to one bf16 step on top of the summation noise (2e-5 of the row's largest value); the stage output (one more GEMM and the residual) within 2e-2 for EVERY row of every
class, median within 5e-3."""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_10875_amd import sol, synth

from gpu_util import dev, dev_weights, host

pytestmark = pytest.mark.gpu


def _row_err(got, ref):
    ref = np.asarray(ref, np.float64).reshape(-1, ref.shape[-1])
    got = np.asarray(got, np.float64).reshape(-1, ref.shape[-1])
    return np.abs(got - ref).max(axis=1) / np.maximum(np.abs(ref).max(axis=1), 1e-30)


def _oracle_taps(shape, table, w, x, ids, T, taps):
    n = x.shape[0]
    kc = np.zeros((n, shape.n_kv_heads, T, shape.head_dim), np.float32)
    vc = np.zeros_like(kc)
    out, tp = oracle.layer_forward(oracle.make_cfg(shape, act_bf16=True), oracle.make_table(table), w, x, ids, kc, vc,
                                   taps=taps)
    return out, tp, kc, vc


HD64 = synth.ModelShape(d_model=256, n_q_heads=8, n_kv_heads=2, head_dim=64, d_ff=512, n_layers=1, vocab=100)
HD128 = synth.ModelShape(d_model=256, n_q_heads=4, n_kv_heads=1, head_dim=128, d_ff=512, n_layers=1, vocab=100)
HD128_G8 = synth.ModelShape(d_model=256, n_q_heads=8, n_kv_heads=1, head_dim=128, d_ff=512, n_layers=1, vocab=100)


# T picks the variant of the threshold kernel: <= 256, <= 1024, <= 1280, <= 2048, <= 4096 keys
@pytest.mark.parametrize("shape,n_seq,T", [
    (HD64, 3, 70), (HD64, 2, 300), (HD64, 1, 1100), (HD64, 1, 1500), (HD64, 1, 2100),
    (HD128, 3, 72), (HD128, 2, 300), (HD128, 1, 1100), (HD128, 1, 1500), (HD128, 1, 2100), (HD128, 1, 4096),
    (HD128_G8, 1, 530),
], ids=lambda v: getattr(v, "head_dim", v))
def test_attention_stage_on_the_oracles_q_k_v(shape, n_seq, T):
    table = synth.TABLE_C2
    w = synth.layer_weights(shape, 9000, bf16=True, std=0.05)
    x = synth.hidden_states(n_seq, T, shape.d_model, 9001, bf16=True)
    ids = synth.iid_actions(len(table), (n_seq, T), 9002)
    _, tp, kc, vc = _oracle_taps(shape, table, w, x, ids, T, ("q_rot", "attn_out"))
    ctx = sol.Sol(shape, table, dtype=sol.BF16, max_positions=T)
    o = host(ctx.test_attention_stage(dev(tp["q_rot"], sol.BF16), dev(ids), dev(kc, sol.BF16), dev(vc, sol.BF16)))
    assert ctx.device_status() == sol.OK
    ctx.close()
    err = _row_err(o, tp["attn_out"])
    print(f"attention stage dh={shape.head_dim} T={T}: row err median {np.median(err):.2e} q99 {np.quantile(err, .99):.2e} "
          f"max {err.max():.2e}; rows over 1e-3: {(err > 1e-3).mean():.4f}")
    assert err.max() < 2e-2 and np.median(err) < 1e-4 and (err > 1e-3).mean() <= 0.01
    # the quantiser that follows, as integer codes
    bits = np.array([a[4] for a in table], np.int32)[ids.reshape(-1)]
    rows_gpu = o.reshape(-1, o.shape[-1])
    codes_gpu = host(sol.quant_codes(dev(rows_gpu), dev(bits))[0]).astype(np.int32)
    rows_ref = tp["attn_out"].reshape(-1, o.shape[-1])
    for b in (4, 6, 8):
        sel = np.flatnonzero(bits == b)
        diff = np.concatenate([np.abs(codes_gpu[r] - oracle.fake_quant(rows_ref[r], b)[1]) for r in sel])
        q_max = 2 ** (b - 1) - 1
        share = float((diff == 1).mean())
        print(f"  {b}-bit codes of the o-proj input: {diff.size} codes, off by one {share:.2e}, beyond {int((diff > 1).sum())}")
        assert (diff > 1).sum() == 0 and share <= 2 * q_max * 1e-4 + 1e-4


@pytest.mark.parametrize("shape,L_max,starts,T", [
    (HD64, 1300, (1200, 1000, 0), 70),          # 2048-key variant, cache lengths 1270 / 1070 / 70 in one launch
    (HD128, 2500, (2400, 17), 96),              # 4096-key variant, head size 128
], ids=["dh64-L1300", "dh128-L2500"])
def test_attention_stage_on_a_chunk_behind_a_cache_prefix(shape, L_max, starts, T):
    """The chunk's T rows sit at positions pos0[s] .. pos0[s] + T - 1 of caches that already hold pos0[s] keys (different
    per sequence, L_max not a multiple of the kernels' tiles): the oracle first runs the prefix to fill the caches, then
    the chunk; the GPU stage gets the oracle's rotated q of the chunk and the oracle's caches."""
    table = synth.TABLE_C2
    n_seq = len(starts)
    w = synth.layer_weights(shape, 9200, bf16=True, std=0.05)
    cfg, tab = oracle.make_cfg(shape, act_bf16=True), oracle.make_table(table)
    kc = np.zeros((n_seq, shape.n_kv_heads, L_max, shape.head_dim), np.float32)
    vc = np.zeros_like(kc)
    for s, p in enumerate(starts):               # prefixes of different lengths, one sequence at a time
        if p:
            xp = synth.hidden_states(1, p, shape.d_model, 9210 + s, bf16=True)
            idp = synth.iid_actions(len(table), (1, p), 9220 + s)
            oracle.layer_forward(cfg, tab, w, xp, idp, kc[s:s + 1], vc[s:s + 1])
    x = synth.hidden_states(n_seq, T, shape.d_model, 9201, bf16=True)
    ids = synth.iid_actions(len(table), (n_seq, T), 9202)
    pos0 = np.array(starts, np.int32)
    _, tp = oracle.layer_forward(cfg, tab, w, x, ids, kc, vc, pos0=pos0, taps=("q_rot", "attn_out"))
    ctx = sol.Sol(shape, table, dtype=sol.BF16, max_positions=L_max)
    o = host(ctx.test_attention_stage(dev(tp["q_rot"], sol.BF16), dev(ids), dev(kc, sol.BF16), dev(vc, sol.BF16), pos0=dev(pos0)))
    assert ctx.device_status() == sol.OK
    ctx.close()
    err = _row_err(o, tp["attn_out"])
    print(f"attention stage behind a prefix, dh={shape.head_dim} L_max={L_max}: row err median {np.median(err):.2e} "
          f"max {err.max():.2e}; rows over 1e-3: {(err > 1e-3).mean():.4f}")
    assert err.max() < 2e-2 and np.median(err) < 1e-4 and (err > 1e-3).mean() <= 0.01


def _codes(a, bits):
    """integer codes of a stored (dequantised) row: the row's largest magnitude is q_max steps"""
    q_max = 2 ** (bits - 1) - 1
    amax = np.abs(a).max()
    return np.zeros(a.shape, np.int64) if amax == 0 else np.rint(a.astype(np.float64) / (amax / q_max)).astype(np.int64)


@pytest.mark.parametrize("shape,n_seq,T", [
    (synth.ModelShape(d_model=256, n_q_heads=8, n_kv_heads=2, head_dim=64, d_ff=768, n_layers=1, vocab=100), 3, 70),
    (synth.LLAMA_1B, 2, 160),
    (synth.LLAMA_8B, 1, 72),
    (synth.LLAMA_1B, 1, 40),                   # few rows: the weight-streaming GEMMs of the decode step
], ids=["small", "1B", "8B", "1B-skinny"])
def test_mlp_stage_on_the_oracles_h2(shape, n_seq, T):
    table = synth.TABLE_C2
    w = synth.layer_weights(shape, 9100, bf16=True)
    x = synth.hidden_states(n_seq, T, shape.d_model, 9101, bf16=True)
    ids = synth.iid_actions(len(table), (n_seq, T), 9102)
    ref, tp, _, _ = _oracle_taps(shape, table, w, x, ids, T, ("h2", "x_mid", "mlp_act"))
    ctx = sol.Sol(shape, table, dtype=sol.BF16, max_positions=max(T, 16))
    a, out = ctx.test_mlp_stage(dev_weights(w, sol.BF16), dev(tp["h2"], sol.BF16), dev(tp["x_mid"]), dev(ids))
    assert ctx.device_status() == sol.OK
    ctx.close()
    a, out = host(a).reshape(-1, shape.d_ff), host(out).reshape(-1, shape.d_model)
    a_ref, out_ref = tp["mlp_act"].reshape(-1, shape.d_ff), ref.reshape(-1, shape.d_model)
    bits = np.array([t[4] for t in table], np.int32)[ids.reshape(-1)]
    kept_gpu, kept_ref = a != 0, a_ref != 0
    for b in (4, 6, 8, 16):
        sel = np.flatnonzero(bits == b)
        if b >= 16:      # no quantiser: kept channels agree to one bf16 step (plus the fp32 summation noise, which is
            # relative to the row's scale, not to a small element), a handful of swapped near-ties
            both = kept_gpu[sel] & kept_ref[sel]
            noise = 2e-5 * np.abs(a_ref[sel]).max(axis=1, keepdims=True)
            excess = (np.abs(a[sel] - a_ref[sel]) - noise)[both] / np.abs(a_ref[sel])[both]
            swapped = float((kept_gpu[sel] != kept_ref[sel]).sum() / max(1, kept_ref[sel].sum()))
            print(f"MLP stage {b}-bit rows: kept values, largest step {excess.max():.2e} of the value, over half a bf16 step "
                  f"{(excess > 2 ** -9).mean():.2e}, kept-set difference {swapped:.2e}")
            assert excess.max() <= 2 ** -7 and (excess > 2 ** -9).mean() < 1e-2 and swapped <= 1e-3
            continue
        diff = np.concatenate([np.abs(_codes(a[r], b) - _codes(a_ref[r], b)) for r in sel])
        share = float((diff == 1).mean())
        print(f"MLP stage {b}-bit rows: {diff.size} codes of the down-proj input, off by one {share:.2e}, beyond {int((diff > 1).sum())}")
        assert (diff > 1).sum() == 0 and share <= 1e-2
    err = _row_err(out, out_ref)
    for b in (4, 6, 8, 16):
        e = err[bits == b]
        print(f"MLP stage output, rows of {b}-bit actions: median {np.median(e):.2e} max {e.max():.2e}")
        assert e.max() < 2e-2 and np.median(e) < 5e-3
