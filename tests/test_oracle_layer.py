"""Pins of the CPU oracle's layer / stack functions (CPU only).

Witness: a float64 decoder layer assembled from tensor-library primitives (matmul,
scaled_dot_product_attention, silu, complex multiplication for the rotary embedding) plus
the single operators that tests/test_oracle_ops.py pins on their own."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from paper_2605_10875_amd import synth

SHAPE = synth.ModelShape(d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, d_ff=96, n_layers=2, vocab=50)
DENSE = [synth.DENSE_ACTION]


def _rms(x, w, eps):
    return x * torch.rsqrt(x.pow(2).mean(-1, keepdim=True) + eps) * w


def _rope_complex(x, pos, theta):
    # x [..., T, H, dh]; pairs (c, c + dh/2) seen as complex numbers rotated by pos * theta^(-2c/dh)
    dh = x.shape[-1]
    half = dh // 2
    inv = theta ** (-torch.arange(half, dtype=torch.float64) * 2.0 / dh)
    ang = pos.double()[:, None] * inv[None, :]                       # [T, half]
    rot = torch.polar(torch.ones_like(ang), ang)[:, None, :]         # [T, 1, half]
    xc = torch.complex(x[..., :half], x[..., half:]) * rot
    return torch.cat([xc.real, xc.imag], -1)


def witness_layer(shape, w, x, table, ids, keep_mask=None, quant_sites=oracle.QS_NORTHSTAR, prune_site=0,
                  act_bf16=False, drop=None, full=False):
    """float64 layer for pos0 = 0. keep_mask [n,T,Hq,T] (from the oracle's tap) or None = causal dense.
    Values are narrowed to float32 wherever the method stores a tensor (storage is fp32, sums are fp64).
    act_bf16: the tensors handed from one operator to the next (h1, q, k, v, o, h2, a before and after the
    prune / quantiser, layer output) make a round trip through torch.bfloat16; the residual x2 does not.
    drop: name of one of those hand-over points whose rounding is left out (to show that the comparison notices).
    full: return a dict of every intermediate instead of (out, scores, a)."""
    W = {k: torch.from_numpy(v).double() for k, v in w.items()}
    x = torch.from_numpy(x).double()
    n, T, d = x.shape
    Hq, Hkv, dh = shape.n_q_heads, shape.n_kv_heads, shape.head_dim

    def f32(t):
        return t.float().double()

    def bf(t, name):
        if not act_bf16 or name in (drop if isinstance(drop, tuple) else (drop,)):
            return t
        return t.float().to(torch.bfloat16).double()

    def fq(t, site):
        if not (quant_sites & site):
            return t
        out = t.clone()
        for s in range(n):
            for i in range(T):
                bits = table[ids[s, i]][4]
                out[s, i] = torch.from_numpy(oracle.fake_quant(t[s, i].float().numpy(), bits)[0]).double()
        return out

    def prune(t):
        out = t.clone()
        for s in range(n):
            for i in range(T):
                num, den = table[ids[s, i]][2:4]
                m = max(1, min(t.shape[-1], math.ceil(num * t.shape[-1] / den)))
                keep = oracle.topm_mask(t[s, i].float().numpy(), m)
                out[s, i] = t[s, i] * torch.from_numpy(keep).double()
        return out

    h1 = bf(fq(f32(_rms(x, W["w_in_norm"], shape.rms_eps)), oracle.QS_QKV_IN), "h1")
    pos = torch.arange(T)
    q = bf(f32(_rope_complex(f32(h1 @ W["wq"].T).view(n, T, Hq, dh), pos, shape.rope_theta)), "q")
    k = bf(f32(_rope_complex(f32(h1 @ W["wk"].T).view(n, T, Hkv, dh), pos, shape.rope_theta)), "k")
    v = bf(f32(h1 @ W["wv"].T).view(n, T, Hkv, dh), "v")
    qh = q.permute(0, 2, 1, 3)
    kh = k.permute(0, 2, 1, 3).repeat_interleave(Hq // Hkv, dim=1)
    vh = v.permute(0, 2, 1, 3).repeat_interleave(Hq // Hkv, dim=1)
    if keep_mask is None:
        o = F.scaled_dot_product_attention(qh, kh, vh, is_causal=True)
    else:
        km = torch.from_numpy(keep_mask[:, :, :, :T].astype(bool)).permute(0, 2, 1, 3)   # [n,Hq,T,T]
        bias = torch.where(km, 0.0, -math.inf).double()
        o = F.scaled_dot_product_attention(qh, kh, vh, attn_mask=bias)
    o_raw = f32(o.permute(0, 2, 1, 3).reshape(n, T, Hq * dh))
    o = bf(fq(o_raw, oracle.QS_O_IN), "o")
    x2 = f32(x + f32(o @ W["wo"].T))
    h2 = f32(_rms(x2, W["w_post_norm"], shape.rms_eps))
    if prune_site == 1:
        h2 = prune(h2)
    h2 = bf(fq(h2, oracle.QS_GATEUP_IN), "h2")
    gate, up = f32(h2 @ W["w_gate"].T), f32(h2 @ W["w_up"].T)
    a = bf(f32(F.silu(gate) * up), "a")
    if prune_site == 0:
        a = prune(a)
    a = bf(fq(a, oracle.QS_DOWN_IN), "a_quant")
    z = f32(a @ W["w_down"].T)
    z = fq(z, oracle.QS_MLP_OUT)
    out = bf(f32(x2 + z), "out")
    scores = (qh @ kh.transpose(-1, -2)) / math.sqrt(dh)
    if full:
        return dict(out=out.numpy(), scores=scores.numpy(), a=a.numpy(), q=q.numpy(), k=k.numpy(), v=v.numpy(),
                    h1=h1.numpy(), h2=h2.numpy(), x2=x2.numpy(), o_raw=o_raw.numpy())
    return out.numpy(), scores.numpy(), a.numpy()


def _caches(shape, n_seq, L):
    z = np.zeros((n_seq, shape.n_kv_heads, L, shape.head_dim), np.float32)
    return z, z.copy()


def test_dense_action_is_the_textbook_layer():
    w = synth.layer_weights(SHAPE, 11, std=0.15)
    x = synth.hidden_states(2, 12, SHAPE.d_model, 12)
    cfg, tab = oracle.make_cfg(SHAPE), oracle.make_table(DENSE)
    kc, vc = _caches(SHAPE, 2, 12)
    out, _ = oracle.layer_forward(cfg, tab, w, x, np.zeros((2, 12), np.int32), kc, vc)
    want, _, _ = witness_layer(SHAPE, w, x, DENSE, np.zeros((2, 12), np.int32))
    assert np.abs(out - want).max() < 1e-5 * np.abs(want).max()
    # the paper's preset (pages, sinks, MLP-input prune, MLP-output quant) is dense too under a dense action
    cfg_p = oracle.make_cfg(SHAPE, page_size=4, n_sink=4, n_window=2, prune_site=1, quant_sites=oracle.QS_PAPER)
    kc2, vc2 = _caches(SHAPE, 2, 12)
    out_p, _ = oracle.layer_forward(cfg_p, tab, w, x, np.zeros((2, 12), np.int32), kc2, vc2)
    assert np.array_equal(out_p, out) and np.array_equal(kc2, kc)


@pytest.mark.parametrize("preset", ["linear_input_sites", "paper_sites"])
def test_action_conditioned_layer_against_witness(preset):
    table = synth.action_table((0.25, 0.5, 1.0), (0.0, 0.25, 0.5), (4, 8, 16))
    w = synth.layer_weights(SHAPE, 21, std=0.15)
    n, T = 2, 14
    x = synth.hidden_states(n, T, SHAPE.d_model, 22)
    ids = synth.iid_actions(len(table), (n, T), 23)
    if preset == "linear_input_sites":
        kw = dict()
        wkw = dict()
    else:
        kw = dict(prune_site=1, quant_sites=oracle.QS_PAPER)
        wkw = dict(prune_site=1, quant_sites=oracle.QS_PAPER)
    cfg, tab = oracle.make_cfg(SHAPE, **kw), oracle.make_table(table)
    kc, vc = _caches(SHAPE, n, T)
    out, taps = oracle.layer_forward(cfg, tab, w, x, ids, kc, vc, taps=("keep_mask", "mlp_act"))
    want, scores, a = witness_layer(SHAPE, w, x, table, ids, keep_mask=taps["keep_mask"], **wkw)
    assert np.abs(out - want).max() < 2e-5 * np.abs(want).max()
    assert np.abs(taps["mlp_act"] - a).max() < 2e-5 * np.abs(a).max()
    # the attended sets are the top-ceil(kappa*n) causal scores of the witness
    km = taps["keep_mask"]
    for s in range(n):
        for i in range(T):
            num, den = table[ids[s, i]][:2]
            b = max(1, math.ceil(num * (i + 1) / den))
            for h in range(SHAPE.n_q_heads):
                row = scores[s, h, i, :i + 1].astype(np.float32)
                top = sorted(range(i + 1), key=lambda j: (-row[j], j))[:b]
                assert km[s, i, h, :i + 1].sum() == b and km[s, i, h, i + 1:].sum() == 0
                assert set(np.nonzero(km[s, i, h])[0]) == set(top)
            if preset == "linear_input_sites" and table[ids[s, i]][4] >= 16:   # small codes round to 0
                mnum, mden = table[ids[s, i]][2:4]
                m = math.ceil(mnum * SHAPE.d_ff / mden)
                assert np.count_nonzero(taps["mlp_act"][s, i]) == m


HAND_OVER_POINTS = ("h1", "q", "k", "v", "o", "h2", "a", "a_quant", "out")


def _bf16_case():
    table = synth.action_table((0.25, 0.5, 1.0), (0.0, 0.25, 0.5), (4, 8, 16))
    w = synth.layer_weights(SHAPE, 121, std=0.15, bf16=True)
    n, T = 2, 14
    x = synth.hidden_states(n, T, SHAPE.d_model, 122, bf16=True)
    ids = synth.iid_actions(len(table), (n, T), 123)
    return table, w, x, ids, n, T


def _bf16_diffs(o_out, o_taps, o_kc, o_vc, wit):
    """largest |oracle - witness| of every tensor the oracle exposes, relative to that tensor's largest value"""
    pairs = {"out": (o_out, wit["out"]), "x2": (o_taps["x_mid"], wit["x2"]), "a": (o_taps["mlp_act"], wit["a"]),
             "q": (o_taps["q_rot"], wit["q"].reshape(o_taps["q_rot"].shape)), "h1": (o_taps["h1"], wit["h1"]),
             "h2": (o_taps["h2"], wit["h2"]), "o_raw": (o_taps["attn_out"], wit["o_raw"]),
             "k": (o_kc.transpose(0, 2, 1, 3), wit["k"]), "v": (o_vc.transpose(0, 2, 1, 3), wit["v"])}
    return {name: float(np.abs(a - b).max() / np.abs(b).max()) for name, (a, b) in pairs.items()}


@pytest.mark.parametrize("sites", ["linear_input_sites", "paper_sites"])
def test_bf16_store_mode_rounds_exactly_at_the_hand_over_points(sites):
    """The bf16-store mode is the reference of every bf16 GPU comparison, so its rounding points are pinned: a
    float64 witness that sends exactly the tensors handed from one operator to the next (h1, q, k, v, o, h2, the
    SiLU(gate)*up product before and after prune + quantiser, the layer output; not the residual x2) through
    torch.bfloat16 must reproduce every exposed tensor, and leaving out any single one of those roundings in the
    witness must break the agreement, i.e. the comparison notices a missing rounding anywhere."""
    table, w, x, ids, n, T = _bf16_case()
    kw = dict() if sites == "linear_input_sites" else dict(prune_site=1, quant_sites=oracle.QS_PAPER)
    cfg, tab = oracle.make_cfg(SHAPE, act_bf16=True, **kw), oracle.make_table(table)
    kc, vc = _caches(SHAPE, n, T)
    out, taps = oracle.layer_forward(cfg, tab, w, x, ids, kc, vc,
                                     taps=("keep_mask", "mlp_act", "x_mid", "q_rot", "h1", "h2", "attn_out"))
    wit = witness_layer(SHAPE, w, x, table, ids, keep_mask=taps["keep_mask"], act_bf16=True, full=True, **kw)
    diffs = _bf16_diffs(out, taps, kc, vc, wit)
    assert max(diffs.values()) < 1e-6, diffs
    for t in (out, kc, vc, taps["mlp_act"], taps["q_rot"], taps["h1"], taps["h2"]):
        assert np.array_equal(t, synth.round_to_bf16(t))
    assert not np.array_equal(taps["x_mid"], synth.round_to_bf16(taps["x_mid"]))        # the residual stays fp32
    points = list(HAND_OVER_POINTS)
    if sites == "paper_sites":       # nothing sits between the two roundings of the SiLU(gate)*up product there: one point
        points = [p for p in points if p not in ("a", "a_quant")] + [("a", "a_quant")]
    for point in points:
        mutant = witness_layer(SHAPE, w, x, table, ids, keep_mask=taps["keep_mask"], act_bf16=True, drop=point,
                               full=True, **kw)
        worst = max(_bf16_diffs(out, taps, kc, vc, mutant).values())
        assert worst > 1e-4, (point, worst)


def _page_rule_sets(q, k, i, num, den, S, n_sink, n_window):
    """Appendix "Quest masking", written out in numpy for one (query, head): pages of S keys from key 0 over the
    n = i + 1 allowed keys, bound sum_c max(q_c max_c, q_c min_c), the ceil(b / S) best pages (ties to the lower
    page) kept whole, plus the first n_sink and last n_window allowed keys; b >= n keeps everything."""
    n = i + 1
    b = max(1, min(n, -(-num * n // den)))
    if b >= n:
        return set(range(n))
    pages = -(-n // S)
    bound = []
    for u in range(pages):
        rows = k[u * S:min(u * S + S, n)]
        bound.append(float(np.maximum(q * rows.max(axis=0), q * rows.min(axis=0)).sum()))
    best = sorted(range(pages), key=lambda u: (-bound[u], u))[:-(-b // S)]
    kept = {j for u in best for j in range(u * S, min(u * S + S, n))}
    return kept | set(range(min(n_sink, n))) | set(range(max(0, n - n_window), n))


@pytest.mark.parametrize("S,n_sink,n_window,T", [(4, 4, 2, 40), (16, 4, 2, 50), (16, 0, 0, 70), (8, 3, 5, 33)])
@pytest.mark.parametrize("sites", ["linear_input_sites", "paper_sites"])
def test_page_rule_layer_against_witness(S, n_sink, n_window, T, sites):
    """The page rule at layer level: which query, which keys and how many of them reach the page selection inside
    the layer. The attended sets tapped from the layer must equal the page ranking recomputed in numpy from the
    witness's own rotated q and k (unscaled q, pages over the allowed keys only, forced keys on top), and the layer
    output must equal the witness layer run with those sets."""
    table = synth.action_table((0.125, 0.25, 0.5, 1.0), (0.0, 0.5), (4, 16))
    w = synth.layer_weights(SHAPE, 131, std=0.15)
    n = 2
    x = synth.hidden_states(n, T, SHAPE.d_model, 132)
    ids = synth.iid_actions(len(table), (n, T), 133)
    kw = dict() if sites == "linear_input_sites" else dict(prune_site=1, quant_sites=oracle.QS_PAPER)
    cfg = oracle.make_cfg(SHAPE, page_size=S, n_sink=n_sink, n_window=n_window, **kw)
    kc, vc = _caches(SHAPE, n, T)
    out, taps = oracle.layer_forward(cfg, oracle.make_table(table), w, x, ids, kc, vc, taps=("keep_mask", "mlp_act"))
    wit = witness_layer(SHAPE, w, x, table, ids, keep_mask=taps["keep_mask"], full=True, **kw)
    assert np.abs(out - wit["out"]).max() < 2e-5 * np.abs(wit["out"]).max()
    assert np.abs(taps["mlp_act"] - wit["a"]).max() < 2e-5 * np.abs(wit["a"]).max()
    km = taps["keep_mask"]
    grp = SHAPE.n_q_heads // SHAPE.n_kv_heads
    sparse_rows = 0
    for s in range(n):
        for i in range(T):
            num, den = table[ids[s, i]][:2]
            for h in range(SHAPE.n_q_heads):
                want = _page_rule_sets(wit["q"][s, i, h], wit["k"][s, :, h // grp], i, num, den, S, n_sink, n_window)
                got = set(np.nonzero(km[s, i, h])[0].tolist())
                assert got == want, (s, i, h, sorted(got ^ want))
                sparse_rows += len(want) < i + 1
    assert sparse_rows > n * T * SHAPE.n_q_heads // 4          # the case really exercises the page selection


def test_keep_all_budget_is_bitwise_dense_attention():
    # a keep fraction so close to 1 that ceil(kappa*n) = n for every row: same bits as kappa = 1
    table = [(1, 1, 1, 1, 16), (4095, 4096, 1, 1, 16)]
    w = synth.layer_weights(SHAPE, 31, std=0.15)
    x = synth.hidden_states(1, 20, SHAPE.d_model, 32)
    cfg, tab = oracle.make_cfg(SHAPE), oracle.make_table(table)
    outs = []
    for a in (0, 1):
        kc, vc = _caches(SHAPE, 1, 20)
        outs.append(oracle.layer_forward(cfg, tab, w, x, np.full((1, 20), a, np.int32), kc, vc)[0])
    assert np.array_equal(outs[0], outs[1])


def test_single_axis_actions_leave_the_other_paths_alone():
    w = synth.layer_weights(SHAPE, 41, std=0.15)
    x = synth.hidden_states(1, 16, SHAPE.d_model, 42)
    table = [(1, 1, 1, 1, 16), (1, 4, 1, 1, 16), (1, 1, 1, 2, 16), (1, 1, 1, 1, 4)]
    cfg, tab = oracle.make_cfg(SHAPE), oracle.make_table(table)
    res = []
    for a in range(4):
        kc, vc = _caches(SHAPE, 1, 16)
        out, taps = oracle.layer_forward(cfg, tab, w, x, np.full((1, 16), a, np.int32), kc, vc,
                                         taps=("attn_out", "x_mid", "mlp_act"))
        res.append((out, taps, kc.copy(), vc.copy()))
    dense = res[0]
    # sparse attention only: K/V identical (projections untouched), attention output differs
    assert np.array_equal(res[1][2], dense[2]) and np.array_equal(res[1][3], dense[3])
    assert not np.array_equal(res[1][1]["attn_out"], dense[1]["attn_out"])
    assert np.array_equal(res[1][1]["attn_out"][0, :1], dense[1]["attn_out"][0, :1])   # one allowed key: kept
    # MLP pruning only: everything up to the MLP input identical; half of the channels zero
    assert np.array_equal(res[2][1]["x_mid"], dense[1]["x_mid"])
    assert np.all(np.count_nonzero(res[2][1]["mlp_act"], axis=-1) == SHAPE.d_ff // 2)
    kept = res[2][1]["mlp_act"] != 0
    assert np.array_equal(res[2][1]["mlp_act"][kept], dense[1]["mlp_act"][kept])
    # quantisation only: at most 2*q_max+1 = 15 distinct values per token at the down-proj input
    for i in range(16):
        assert len(np.unique(res[3][1]["mlp_act"][0, i])) <= 15
    assert not np.array_equal(res[3][2], dense[2])                   # K/V are committed under the action


def test_row_zero_of_sparse_attention_matches_dense_row():
    # with one allowed key every budget keeps it
    w = synth.layer_weights(SHAPE, 41, std=0.15)
    x = synth.hidden_states(1, 3, SHAPE.d_model, 43)
    table = [(1, 1, 1, 1, 16), (1, 16, 1, 1, 16)]
    cfg, tab = oracle.make_cfg(SHAPE), oracle.make_table(table)
    o = []
    for a in (0, 1):
        kc, vc = _caches(SHAPE, 1, 3)
        o.append(oracle.layer_forward(cfg, tab, w, x, np.full((1, 3), a, np.int32), kc, vc, taps=("attn_out",))[1]["attn_out"])
    assert np.array_equal(o[0][0, 0], o[1][0, 0]) and not np.array_equal(o[0][0, 2], o[1][0, 2])


def _stack(shape, seed, std=0.15):
    layers = [synth.layer_weights(shape, seed + l, std=std) for l in range(shape.n_layers)]
    head = synth.head_weights(shape, seed + 100, std=std)
    return layers, head


def test_batched_pass_equals_stepwise_decode_bitwise():
    table = synth.TABLE_C1
    layers, head = _stack(SHAPE, 51)
    B, G, T = 2, 2, 9
    tokens, targets = synth.tokens_and_targets(B, T, SHAPE.vocab, 52)
    ids = synth.iid_actions(len(table), (B, G, T), 53)
    for kw in (dict(), dict(page_size=4, n_sink=2, n_window=1, prune_site=1, quant_sites=oracle.QS_PAPER),
               dict(act_bf16=True)):
        cfg, tab = oracle.make_cfg(SHAPE, **kw), oracle.make_table(table)
        nll, hid = oracle.schedule_loglik(cfg, tab, head["embed"], layers, head["w_final_norm"], head["lm_head"],
                                          tokens, targets, ids, want_hidden=True)
        N = B * G
        kcs = [np.zeros((N, SHAPE.n_kv_heads, T, SHAPE.head_dim), np.float32) for _ in layers]
        vcs = [np.zeros((N, SHAPE.n_kv_heads, T, SHAPE.head_dim), np.float32) for _ in layers]
        flat_ids = ids.reshape(N, T)
        tok_n = np.repeat(tokens, G, axis=0)
        tgt_n = np.repeat(targets, G, axis=0)
        for t in range(T):
            x0 = head["embed"][tok_n[:, t]]
            h, nl = oracle.decode_step(cfg, tab, layers, x0, flat_ids[:, t], np.full(N, t, np.int32), kcs, vcs,
                                       head["w_final_norm"], head["lm_head"], tgt_n[:, t])
            assert np.array_equal(h, hid.reshape(N, T, -1)[:, t])
            assert np.array_equal(nl, nll.reshape(N, T)[:, t])


def test_identical_schedules_identical_likelihoods_and_batch_independence():
    table = synth.TABLE_C1
    layers, head = _stack(SHAPE, 61)
    B, G, T = 2, 3, 10
    tokens, targets = synth.tokens_and_targets(B, T, SHAPE.vocab, 62)
    one = synth.iid_actions(len(table), (B, 1, T), 63)
    ids = np.repeat(one, G, axis=1)
    cfg, tab = oracle.make_cfg(SHAPE), oracle.make_table(table)
    nll = oracle.schedule_loglik(cfg, tab, head["embed"], layers, head["w_final_norm"], head["lm_head"],
                                 tokens, targets, ids)
    for g in range(1, G):
        assert np.array_equal(nll[:, g], nll[:, 0])
    # a sequence's result does not depend on what else is in the batch, nor on its slot
    solo = oracle.schedule_loglik(cfg, tab, head["embed"], layers, head["w_final_norm"], head["lm_head"],
                                  tokens[1:], targets[1:], ids[1:])
    assert np.array_equal(solo[0], nll[1])
    # dense schedule == plain stack: NLL equals -log_softmax of a float64 witness stack
    dense_ids = np.zeros((B, 1, T), np.int32)
    cfg_d, tab_d = oracle.make_cfg(SHAPE), oracle.make_table(DENSE)
    nll_d = oracle.schedule_loglik(cfg_d, tab_d, head["embed"], layers, head["w_final_norm"], head["lm_head"],
                                   tokens, targets, dense_ids)
    x = head["embed"][tokens]
    for w in layers:
        x = witness_layer(SHAPE, w, x.astype(np.float32), DENSE, np.zeros((B, T), np.int32))[0]
    hf = _rms(torch.from_numpy(x).double(), torch.from_numpy(head["w_final_norm"]).double(), SHAPE.rms_eps)
    lsm = torch.log_softmax(hf @ torch.from_numpy(head["lm_head"]).double().T, -1)
    want = -torch.gather(lsm, -1, torch.from_numpy(targets).long()[..., None])[..., 0]
    assert np.abs(nll_d[:, 0] - want.numpy()).max() < 5e-5


def test_causality_and_kv_pollution_impulse():
    # compress a burst of steps, then return to dense: positions before the burst keep their bits,
    # positions after it differ because they attend to K/V committed under the compressed actions
    table = [synth.DENSE_ACTION, (1, 4, 1, 2, 4)]
    layers, head = _stack(SHAPE, 71)
    T, t0, burst = 16, 5, 4
    tokens, targets = synth.tokens_and_targets(1, T, SHAPE.vocab, 72)
    ids = np.zeros((1, 2, T), np.int32)
    ids[0, 1, t0:t0 + burst] = 1
    cfg, tab = oracle.make_cfg(SHAPE), oracle.make_table(table)
    nll, hid = oracle.schedule_loglik(cfg, tab, head["embed"], layers, head["w_final_norm"], head["lm_head"],
                                      tokens, targets, ids, want_hidden=True)
    assert np.array_equal(hid[0, 0, :t0], hid[0, 1, :t0]) and np.array_equal(nll[0, 0, :t0], nll[0, 1, :t0])
    for t in range(t0, T):
        assert not np.array_equal(hid[0, 0, t], hid[0, 1, t])


def test_prefix_cache_positions():
    # running tokens [0,T) in one call equals running [0,T1) then [T1,T) with pos0 = T1 on the same cache
    table = synth.TABLE_C1
    w = synth.layer_weights(SHAPE, 81, std=0.15)
    T, T1 = 12, 7
    x = synth.hidden_states(1, T, SHAPE.d_model, 82)
    ids = synth.iid_actions(len(table), (1, T), 83)
    cfg, tab = oracle.make_cfg(SHAPE), oracle.make_table(table)
    kc, vc = _caches(SHAPE, 1, T)
    full, _ = oracle.layer_forward(cfg, tab, w, x, ids, kc, vc)
    kc2, vc2 = _caches(SHAPE, 1, T)
    a, _ = oracle.layer_forward(cfg, tab, w, x[:, :T1], ids[:, :T1], kc2, vc2)
    b, _ = oracle.layer_forward(cfg, tab, w, x[:, T1:], ids[:, T1:], kc2, vc2, pos0=np.array([T1], np.int32))
    assert np.array_equal(np.concatenate([a, b], 1), full) and np.array_equal(kc2, kc)


def test_bf16_mode_rounds_the_handed_over_tensors():
    table = synth.TABLE_C1
    w = synth.layer_weights(SHAPE, 91, std=0.15, bf16=True)
    x = synth.hidden_states(1, 8, SHAPE.d_model, 92, bf16=True)
    ids = synth.iid_actions(len(table), (1, 8), 93)
    cfg, tab = oracle.make_cfg(SHAPE, act_bf16=True), oracle.make_table(table)
    kc, vc = _caches(SHAPE, 1, 8)
    out, taps = oracle.layer_forward(cfg, tab, w, x, ids, kc, vc, taps=("mlp_act",))
    for t in (out, kc, vc, taps["mlp_act"]):
        assert np.array_equal(t, synth.round_to_bf16(t))
    cfg32 = oracle.make_cfg(SHAPE)
    kc3, vc3 = _caches(SHAPE, 1, 8)
    out32, _ = oracle.layer_forward(cfg32, tab, w, x, ids, kc3, vc3)
    assert np.abs(out - out32).max() < 0.2 * np.abs(out32).max()


def test_argument_errors():
    w = synth.layer_weights(SHAPE, 1)
    x = synth.hidden_states(1, 4, SHAPE.d_model, 2)
    cfg = oracle.make_cfg(SHAPE)
    kc, vc = _caches(SHAPE, 1, 4)
    with pytest.raises(ValueError, match="-4"):
        oracle.layer_forward(cfg, oracle.make_table(DENSE), w, x, np.full((1, 4), 3, np.int32), kc, vc)
    with pytest.raises(ValueError, match="-4"):
        oracle.layer_forward(cfg, oracle.make_table([(0, 1, 1, 1, 16)]), w, x, np.zeros((1, 4), np.int32), kc, vc)
    with pytest.raises(ValueError, match="-5"):
        oracle.layer_forward(cfg, oracle.make_table(DENSE), w, x, np.zeros((1, 4), np.int32), kc, vc,
                             pos0=np.array([1], np.int32))


def test_kv_refresh_restores_the_dense_cache():
    """Background, "Episodes and control horizon": after T steps under aggressive actions the K/V entries of those
    steps differ from the dense ones (they are written as produced under each step's action); the refresh pass over
    the same T tokens rebuilds exactly the entries of a dense pass over the whole sequence, and leaves the prefix alone."""
    import dataclasses
    shape = dataclasses.replace(synth.TINY, n_layers=2)
    table = synth.action_table((0.25, 1.0), (0.0, 0.75), (4, 16))
    dense_id = table.index(synth.DENSE_ACTION)
    harsh_id = table.index((1, 4, 1, 4, 4))
    cfg = oracle.make_cfg(shape)
    tab = oracle.make_table(table)
    layers = [synth.layer_weights(shape, 900 + l) for l in range(2)]
    T0, T, L = 24, 8, 40
    x = synth.hidden_states(1, T0 + T, shape.d_model, 910, std=0.5)

    def run(ids):
        kc = [np.zeros((1, shape.n_kv_heads, L, shape.head_dim), np.float32) for _ in range(2)]
        vc = [np.zeros_like(kc[0]) for _ in range(2)]
        h = x
        for l in range(2):
            h, _ = oracle.layer_forward(cfg, tab, layers[l], h, ids, kc[l], vc[l])
        return kc, vc

    ids_dense = np.full((1, T0 + T), dense_id, np.int32)
    ids_mixed = ids_dense.copy()
    ids_mixed[0, T0:] = harsh_id
    k_ref, v_ref = run(ids_dense)
    k_pol, v_pol = run(ids_mixed)
    for l in range(2):                                              # the steps' entries are polluted, the prefix is not
        assert np.abs(k_pol[l][:, :, T0:T0 + T] - k_ref[l][:, :, T0:T0 + T]).max() > 1e-3
        assert np.array_equal(k_pol[l][:, :, :T0], k_ref[l][:, :, :T0])
    out = oracle.kv_refresh(cfg, layers, x[:, T0:], np.array([T0], np.int32), k_pol, v_pol)
    for l in range(2):
        np.testing.assert_allclose(k_pol[l], k_ref[l], rtol=0, atol=1e-6)
        np.testing.assert_allclose(v_pol[l], v_ref[l], rtol=0, atol=1e-6)
    assert out.shape == (1, T, shape.d_model)
    # a second refresh changes nothing
    k2 = [k.copy() for k in k_pol]
    oracle.kv_refresh(cfg, layers, x[:, T0:], np.array([T0], np.int32), k_pol, v_pol)
    assert all(np.array_equal(a, b) for a, b in zip(k2, k_pol))


def test_episode_pass_equals_prefill_then_stepwise_decode():
    """Method, "GRPO with per-sequence budget sampling": the episode NLLs (batched definition) against the same
    episode walked the way it is deployed: dense prefill of the prefix layer by layer, then one decode step per token
    under the schedule's action."""
    import dataclasses
    shape = dataclasses.replace(synth.TINY, n_layers=2, vocab=97)
    table = synth.action_table((0.25, 1.0), (0.0, 0.75), (4, 16))
    dense_id = table.index(synth.DENSE_ACTION)
    cfg, tab = oracle.make_cfg(shape), oracle.make_table(table)
    layers = [synth.layer_weights(shape, 950 + l) for l in range(2)]
    head = synth.head_weights(shape, 960)
    B, K, P, T = 1, 2, 10, 5
    rng = np.random.default_rng(961)
    prefix = rng.integers(0, shape.vocab, (B, P)).astype(np.int32)
    tokens, targets = synth.tokens_and_targets(B, T, shape.vocab, 962)
    ids = synth.iid_actions(len(table), (B, K, T), 963)
    nll = oracle.episode_loglik(cfg, tab, dense_id, head["embed"], layers, head["w_final_norm"], head["lm_head"], prefix,
                                tokens, targets, ids)
    assert nll.shape == (B, K, T)
    L = P + T
    for k in range(K):
        kc = [np.zeros((1, shape.n_kv_heads, L, shape.head_dim), np.float32) for _ in range(2)]
        vc = [np.zeros_like(kc[0]) for _ in range(2)]
        h = head["embed"][prefix[0]][None]
        for l in range(2):
            h, _ = oracle.layer_forward(cfg, tab, layers[l], h, np.full((1, P), dense_id, np.int32), kc[l], vc[l])
        for t in range(T):
            x0 = head["embed"][tokens[0, t]][None]
            _, step_nll = oracle.decode_step(cfg, tab, layers, x0, ids[0, k, t:t + 1], np.array([P + t], np.int32), kc, vc,
                                             head["w_final_norm"], head["lm_head"], targets[0, t:t + 1])
            assert abs(float(step_nll[0]) - float(nll[0, k, t])) < 1e-4, (k, t)
