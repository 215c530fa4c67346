"""ctypes binding of the CPU oracle (oracle/sol_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg. The product package never imports this module.
All arrays are numpy float32 / int32 / uint8 on the host.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

QS_QKV_IN, QS_O_IN, QS_GATEUP_IN, QS_DOWN_IN, QS_MLP_OUT = 1, 2, 4, 8, 16
QS_NORTHSTAR = QS_QKV_IN | QS_O_IN | QS_GATEUP_IN | QS_DOWN_IN
QS_PAPER = QS_MLP_OUT


class Cfg(C.Structure):
    _fields_ = [("d_model", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("d_ff", C.c_int32), ("n_layers", C.c_int32),
                ("vocab", C.c_int32), ("rms_eps", C.c_float), ("rope_theta", C.c_float),
                ("page_size", C.c_int32), ("n_sink", C.c_int32), ("n_window", C.c_int32),
                ("prune_site", C.c_int32), ("quant_sites", C.c_uint32), ("act_bf16", C.c_int32)]


class Action(C.Structure):
    _fields_ = [("keep_num", C.c_uint32), ("keep_den", C.c_uint32),
                ("mlp_keep_num", C.c_uint32), ("mlp_keep_den", C.c_uint32), ("bits", C.c_uint32)]


_FP = C.POINTER(C.c_float)


class LayerWeights(C.Structure):
    _fields_ = [(n, _FP) for n in ("w_in_norm", "wq", "wk", "wv", "wo", "w_post_norm",
                                   "w_gate", "w_up", "w_down")]


class Taps(C.Structure):
    _fields_ = [("keep_mask", C.POINTER(C.c_uint8)), ("attn_out", _FP), ("mlp_act", _FP), ("x_mid", _FP),
                ("q_rot", _FP), ("h2", _FP), ("h1", _FP)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        # SOL_ORACLE_SANITIZE=1: the AddressSanitizer / UndefinedBehaviorSanitizer build (the process must have the
        # sanitizer runtime preloaded; see tests/test_oracle_sanitizers.py)
        path = _build.build(force=False, sanitize=os.environ.get("SOL_ORACLE_SANITIZE") == "1")
        _lib = C.CDLL(path)
        _lib.orc_budget.restype = C.c_int32
        _lib.orc_budget.argtypes = [C.c_uint32, C.c_uint32, C.c_int32]
        _lib.orc_nll_row.restype = C.c_float
        _lib.orc_round_bf16.restype = C.c_float
        _lib.orc_round_bf16.argtypes = [C.c_float]
        _lib.orc_num_threads.restype = C.c_int32
        for f in ("orc_layer_forward", "orc_decode_step", "orc_schedule_loglik"):
            getattr(_lib, f).restype = C.c_int32
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _p(a, ty=C.c_float):
    return a.ctypes.data_as(C.POINTER(ty)) if a is not None else None


def make_cfg(shape, page_size=1, n_sink=0, n_window=0, prune_site=0,
             quant_sites=QS_NORTHSTAR, act_bf16=False):
    """shape: any object with d_model, n_q_heads, n_kv_heads, head_dim, d_ff, n_layers, vocab,
    rms_eps, rope_theta attributes."""
    return Cfg(shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ff,
               shape.n_layers, shape.vocab, shape.rms_eps, shape.rope_theta,
               page_size, n_sink, n_window, prune_site, quant_sites, int(bool(act_bf16)))


def make_table(actions):
    """actions: sequence of (keep_num, keep_den, mlp_keep_num, mlp_keep_den, bits)."""
    arr = (Action * len(actions))()
    for i, a in enumerate(actions):
        arr[i] = Action(*[int(v) for v in a])
    return arr


_W_NAMES = ("w_in_norm", "wq", "wk", "wv", "wo", "w_post_norm", "w_gate", "w_up", "w_down")


def _layer_struct(w, keepalive):
    s = LayerWeights()
    for n in _W_NAMES:
        a = _f32(w[n])
        keepalive.append(a)
        setattr(s, n, _p(a))
    return s


def num_threads():
    return int(lib().orc_num_threads())


def budget(num, den, n):
    return int(lib().orc_budget(num, den, n))


def round_bf16(x):
    x = _f32(x)
    out = np.empty_like(x)
    flat_in, flat_out = x.reshape(-1), out.reshape(-1)
    f = lib().orc_round_bf16
    for i in range(flat_in.size):
        flat_out[i] = f(float(flat_in[i]))
    return out


def fake_quant(z, bits):
    z = _f32(z)
    n = z.size
    out = np.empty(n, np.float32)
    codes = np.empty(n, np.int32)
    scale = C.c_float(0)
    lib().orc_fake_quant(_p(z), C.c_int32(n), C.c_int32(bits), _p(out), _p(codes, C.c_int32), C.byref(scale))
    return out, codes, float(scale.value)


def topm_mask(a, m):
    a = _f32(a)
    keep = np.zeros(a.size, np.uint8)
    lib().orc_topm_mask(_p(a), C.c_int32(a.size), C.c_int32(m), _p(keep, C.c_uint8))
    return keep


def select_keys(score, b, n_sink=0, n_window=0):
    score = _f32(score)
    keep = np.zeros(score.size, np.uint8)
    lib().orc_select_keys(_p(score), C.c_int32(score.size), C.c_int32(b), C.c_int32(n_sink),
                          C.c_int32(n_window), _p(keep, C.c_uint8))
    return keep


def select_pages(q, k_rows, b, S, n_sink=0, n_window=0):
    q, k_rows = _f32(q), _f32(k_rows)
    n, dh = k_rows.shape
    keep = np.zeros(n, np.uint8)
    ps = np.zeros((n + S - 1) // S, np.float32)
    lib().orc_select_pages(_p(q), _p(k_rows), C.c_int64(dh), C.c_int32(dh), C.c_int32(n), C.c_int32(b),
                           C.c_int32(S), C.c_int32(n_sink), C.c_int32(n_window), _p(keep, C.c_uint8), _p(ps))
    return keep, ps


def softmax_v(score, keep, v_rows):
    score, v_rows = _f32(score), _f32(v_rows)
    keep = np.ascontiguousarray(keep, np.uint8)
    n, dh = v_rows.shape
    o = np.empty(dh, np.float32)
    prob = np.empty(n, np.float32)
    lib().orc_softmax_v(_p(score), _p(keep, C.c_uint8), C.c_int32(n), _p(v_rows), C.c_int64(dh),
                        C.c_int32(dh), _p(o), _p(prob))
    return o, prob


def nll_row(hf, w_lm, target):
    hf, w_lm = _f32(hf), _f32(w_lm)
    V, d = w_lm.shape
    return float(lib().orc_nll_row(_p(hf), _p(w_lm), C.c_int32(d), C.c_int32(V), C.c_int32(target)))


def rmsnorm(x, w, eps):
    x, w = _f32(x), _f32(w)
    out = np.empty_like(x)
    lib().orc_rmsnorm(_p(x), _p(w), C.c_int32(x.size), C.c_float(eps), _p(out))
    return out


def layer_forward(cfg, table, w, x_in, action_ids, k_cache, v_cache, pos0=None, taps=()):
    """x_in [n_seq][T][d]; action_ids [n_seq][T]; caches [n_seq][Hkv][L_max][dh] float32, updated
    in place. Returns (x_out, dict of requested taps)."""
    x_in = _f32(x_in)
    n_seq, T, d = x_in.shape
    assert k_cache.dtype == np.float32 and k_cache.flags.c_contiguous
    assert v_cache.dtype == np.float32 and v_cache.flags.c_contiguous
    L_max = k_cache.shape[2]
    ids = _i32(action_ids).reshape(n_seq, T)
    p0 = _i32(pos0) if pos0 is not None else None
    keepalive = []
    ws = _layer_struct(w, keepalive)
    x_out = np.empty_like(x_in)
    M = n_seq * T
    tp = Taps()
    res = {}
    if "keep_mask" in taps:
        res["keep_mask"] = np.zeros((n_seq, T, cfg.n_q_heads, L_max), np.uint8)
        tp.keep_mask = _p(res["keep_mask"], C.c_uint8)
    if "attn_out" in taps:
        res["attn_out"] = np.zeros((n_seq, T, cfg.n_q_heads * cfg.head_dim), np.float32)
        tp.attn_out = _p(res["attn_out"])
    if "mlp_act" in taps:
        res["mlp_act"] = np.zeros((n_seq, T, cfg.d_ff), np.float32)
        tp.mlp_act = _p(res["mlp_act"])
    if "x_mid" in taps:
        res["x_mid"] = np.zeros((n_seq, T, d), np.float32)
        tp.x_mid = _p(res["x_mid"])
    if "q_rot" in taps:
        res["q_rot"] = np.zeros((n_seq, T, cfg.n_q_heads * cfg.head_dim), np.float32)
        tp.q_rot = _p(res["q_rot"])
    if "h2" in taps:
        res["h2"] = np.zeros((n_seq, T, d), np.float32)
        tp.h2 = _p(res["h2"])
    if "h1" in taps:
        res["h1"] = np.zeros((n_seq, T, d), np.float32)
        tp.h1 = _p(res["h1"])
    rc = lib().orc_layer_forward(C.byref(cfg), table, C.c_int32(len(table)), C.byref(ws),
                                 _p(x_in), _p(x_out), _p(ids, C.c_int32),
                                 _p(p0, C.c_int32) if p0 is not None else None,
                                 _p(k_cache), _p(v_cache), C.c_int32(n_seq), C.c_int32(T),
                                 C.c_int32(L_max), C.byref(tp))
    if rc != 0:
        raise ValueError(f"orc_layer_forward returned {rc}")
    del M
    return x_out, res


def episode_loglik(cfg, table, dense_id, embed, layers, w_final_norm, lm_head, prefix_tokens, tokens, targets, action_ids):
    """Episode pass (Method, "GRPO with per-sequence budget sampling"): dense prefill of the P-token prefix, then K
    schedules of T teacher-forced steps. Written as its definition: the teacher-forced pass over the P + T tokens with
    the dense action (table row dense_id) on the prefix, of which the last T positions are the episode.
    prefix_tokens [B][P], tokens / targets [B][T], action_ids [B][K][T] -> nll [B][K][T]."""
    prefix_tokens, tokens, targets = _i32(prefix_tokens), _i32(tokens), _i32(targets)
    ids = _i32(action_ids)
    B, K, T = ids.shape
    P = prefix_tokens.shape[1]
    full_tokens = np.concatenate([prefix_tokens, tokens], axis=1)
    full_targets = np.concatenate([np.zeros((B, P), np.int32), targets], axis=1)      # prefix targets are not used
    full_ids = np.concatenate([np.full((B, K, P), dense_id, np.int32), ids], axis=2)
    nll = schedule_loglik(cfg, table, embed, layers, w_final_norm, lm_head, full_tokens, full_targets, full_ids)
    return nll[:, :, P:]


def kv_refresh(cfg, layers, x_in, pos0, k_caches, v_caches):
    """Periodic KV-cache refresh (Background, "Episodes and control horizon"): a fully dense pass of the whole
    stack over the T already-known tokens x_in [n_seq][T][d] at positions pos0[s].., which overwrites their K/V in
    every layer's cache with the dense values. Written as the layer pass under the one-row table of the dense
    action with every quantiser site off. Returns the last layer's output."""
    dense = make_table([(1, 1, 1, 1, 16)])
    x = _f32(x_in)
    ids = np.zeros(x.shape[:2], np.int32)
    for l, w in enumerate(layers):
        x, _ = layer_forward(cfg, dense, w, x, ids, k_caches[l], v_caches[l], pos0=pos0)
    return x


def decode_step(cfg, table, layers, x0, action_ids, cache_len, k_caches, v_caches,
                w_final_norm=None, lm_head=None, targets=None):
    """x0 [B][d]; k_caches / v_caches: lists (one per layer) of [B][Hkv][L_max][dh] float32 arrays,
    updated in place. Returns (hidden [B][d], nll [B] or None)."""
    x0 = _f32(x0)
    B, d = x0.shape
    L_max = k_caches[0].shape[2]
    keepalive = []
    larr = (LayerWeights * len(layers))()
    for i, w in enumerate(layers):
        larr[i] = _layer_struct(w, keepalive)
    kp = (_FP * len(layers))(*[_p(k) for k in k_caches])
    vp = (_FP * len(layers))(*[_p(v) for v in v_caches])
    ids, cl = _i32(action_ids), _i32(cache_len)
    hidden = np.empty((B, d), np.float32)
    want_nll = targets is not None
    nll = np.empty(B, np.float32) if want_nll else None
    wf = _f32(w_final_norm) if w_final_norm is not None else None
    lm = _f32(lm_head) if lm_head is not None else None
    tg = _i32(targets) if want_nll else None
    rc = lib().orc_decode_step(C.byref(cfg), table, C.c_int32(len(table)), larr, _p(wf), _p(lm),
                               _p(x0), _p(ids, C.c_int32), _p(cl, C.c_int32), kp, vp,
                               C.c_int32(B), C.c_int32(L_max), _p(hidden),
                               _p(tg, C.c_int32) if want_nll else None, _p(nll) if want_nll else None)
    if rc != 0:
        raise ValueError(f"orc_decode_step returned {rc}")
    return hidden, nll


def schedule_loglik(cfg, table, embed, layers, w_final_norm, lm_head, tokens, targets, action_ids,
                    want_hidden=False):
    """tokens/targets [B][T]; action_ids [B][G][T]. Returns nll [B][G][T] (and hidden)."""
    tokens, targets, ids = _i32(tokens), _i32(targets), _i32(action_ids)
    B, G, T = ids.shape
    keepalive = []
    larr = (LayerWeights * len(layers))()
    for i, w in enumerate(layers):
        larr[i] = _layer_struct(w, keepalive)
    embed, wf, lm = _f32(embed), _f32(w_final_norm), _f32(lm_head)
    nll = np.empty((B, G, T), np.float32)
    hid = np.empty((B, G, T, cfg.d_model), np.float32) if want_hidden else None
    rc = lib().orc_schedule_loglik(C.byref(cfg), table, C.c_int32(len(table)), _p(embed), larr,
                                   _p(wf), _p(lm), _p(tokens, C.c_int32), _p(targets, C.c_int32),
                                   _p(ids, C.c_int32), C.c_int32(B), C.c_int32(G), C.c_int32(T),
                                   _p(nll), _p(hid) if want_hidden else None)
    if rc != 0:
        raise ValueError(f"orc_schedule_loglik returned {rc}")
    return (nll, hid) if want_hidden else nll


# ---------------------------------------------------------------------------------------------------
# reward reduction (Method, "Actions and controlled compute", Eqs. 2-5; "GRPO with per-sequence budget
# sampling"): plain numpy in float64, loops written out in the paper's order.
# ---------------------------------------------------------------------------------------------------
def hinge_penalty(delta, tau):
    """psi(delta; tau) = (max(0, |delta| - tau))^2."""
    return max(0.0, abs(float(delta)) - float(tau)) ** 2


def reward_advantages(nll, action_ids, actions, targets, alpha, tau, gamma, eff=None, eps=1e-8):
    """nll [B][K][T] (nats; the task reward is r_t = -nll, Eq. 2); action_ids [B][K][T] into `actions`, rows
    (keep_num, keep_den, mlp_keep_num, mlp_keep_den, bits); targets [B][3] = (C_kappa, C_rho, C_eta) per input;
    alpha = (a_kappa, a_rho, a_eta); eff [B][T] in {0, 1} or None (every step effective).
    Returns dict: avg [B][K][3] (realised kappa, rho, eta averaged over the effective steps; an episode without
    effective steps takes the targets, i.e. no penalty), penalty [B][K] (Eq. 3), returns [B][K][T] (Eq. 4),
    signal [B][K][T] = returns - penalty (Eq. 5), adv [B][K][T]: the signal mean-centred over the K schedules of an
    input at fixed t, then whitened over the whole batch, (x - mean) / (std + eps) with the population std."""
    nll = np.asarray(nll, np.float64)
    ids = np.asarray(action_ids)
    B, K, T = nll.shape
    tab = np.asarray(actions, np.float64)
    knob = np.stack([tab[:, 0] / tab[:, 1], tab[:, 2] / tab[:, 3], np.minimum(tab[:, 4], 16.0) / 16.0], axis=1)   # kappa, rho, eta = q/16
    targets = np.asarray(targets, np.float64)
    e = np.ones((B, T)) if eff is None else np.asarray(eff, np.float64)
    avg = np.zeros((B, K, 3))
    pen = np.zeros((B, K))
    ret = np.zeros((B, K, T))
    for b in range(B):
        n_eff = e[b].sum()
        for k in range(K):
            for ax in range(3):
                if n_eff > 0:
                    avg[b, k, ax] = sum(e[b, t] * knob[ids[b, k, t], ax] for t in range(T)) / n_eff
                else:
                    avg[b, k, ax] = targets[b, ax]
                pen[b, k] += alpha[ax] * hinge_penalty(avg[b, k, ax] - targets[b, ax], tau)
            g = 0.0
            for t in range(T - 1, -1, -1):               # G_t = r_t + gamma * G_{t+1}
                g = -nll[b, k, t] + gamma * g
                ret[b, k, t] = g
    signal = ret - pen[:, :, None]
    centred = signal - signal.mean(axis=1, keepdims=True)
    adv = (centred - centred.mean()) / (centred.std() + eps)
    return {"avg": avg, "penalty": pen, "returns": ret, "signal": signal, "adv": adv}
