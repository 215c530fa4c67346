"""Seeded synthetic inputs for the action-conditioned decoder-layer path.

This module only draws random numbers and shapes them; it holds none of the method's
arithmetic, so both the GPU library's tests and the CPU oracle's tests may use it.
The tensors stand in for Llama weights and for tokenised text windows, neither of which
is available offline. Every generator is a pure function of (shape, seed).
"""
from dataclasses import dataclass, replace
from fractions import Fraction
from itertools import product

import numpy as np
import torch


@dataclass(frozen=True)
class ModelShape:
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ff: int
    n_layers: int = 1
    vocab: int = 0
    rms_eps: float = 1e-5
    rope_theta: float = 500000.0


# Llama-3.2-1B and Llama-3.1-8B decoder-layer shapes, and the tiny parity shape.
TINY = ModelShape(256, 4, 4, 64, 1024, 1, 1000)
LLAMA_1B = ModelShape(2048, 32, 8, 64, 8192, 16, 128256)
LLAMA_8B = ModelShape(4096, 32, 8, 128, 14336, 32, 128256)

W_NAMES = ("w_in_norm", "wq", "wk", "wv", "wo", "w_post_norm", "w_gate", "w_up", "w_down")


def action_table(keep_levels, prune_levels, bit_levels):
    """Cartesian action table. keep_levels are attention keep fractions, prune_levels are the
    pruned fractions of MLP channels (keep = 1 - prune), bit_levels are bit-widths.
    Returns a list of (keep_num, keep_den, mlp_keep_num, mlp_keep_den, bits); the action id
    is the list index, ordered keep-major, then prune, then bits."""
    table = []
    for k, p, b in product(keep_levels, prune_levels, bit_levels):
        kf = Fraction(k).limit_denominator(1 << 16)
        rf = 1 - Fraction(p).limit_denominator(1 << 16)
        table.append((kf.numerator, kf.denominator, rf.numerator, rf.denominator, int(b)))
    return table


TABLE_C1 = action_table((0.25, 0.5, 1.0), (0.0, 0.25, 0.5), (4, 8, 16))
TABLE_C2 = action_table((0.125, 0.25, 0.5, 1.0), (0.0, 0.25, 0.5, 0.75), (4, 6, 8, 16))
TABLE_C4 = action_table((0.0625, 0.125, 0.25, 0.5, 1.0), (0.0, 0.25, 0.5, 0.75), (4, 6, 8, 16))
DENSE_ACTION = (1, 1, 1, 1, 16)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Nearest bfloat16 of each float32, returned widened to float32 (a storage-format
    conversion done by the tensor library)."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32))
    return t.to(torch.bfloat16).to(torch.float32).numpy()


def layer_weights(shape: ModelShape, seed: int, std: float = 0.02, bf16: bool = False):
    """Random-init decoder-layer weights: projections N(0, std), norm gains 1 + N(0, 0.1)
    so that a dropped gain multiplication is visible. Row-major [out][in] float32."""
    rng = np.random.default_rng(seed)
    d, hq, hkv, dh, dff = shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ff
    w = {
        "w_in_norm": (1.0 + 0.1 * rng.standard_normal(d)).astype(np.float32),
        "wq": (std * rng.standard_normal((hq * dh, d))).astype(np.float32),
        "wk": (std * rng.standard_normal((hkv * dh, d))).astype(np.float32),
        "wv": (std * rng.standard_normal((hkv * dh, d))).astype(np.float32),
        "wo": (std * rng.standard_normal((d, hq * dh))).astype(np.float32),
        "w_post_norm": (1.0 + 0.1 * rng.standard_normal(d)).astype(np.float32),
        "w_gate": (std * rng.standard_normal((dff, d))).astype(np.float32),
        "w_up": (std * rng.standard_normal((dff, d))).astype(np.float32),
        "w_down": (std * rng.standard_normal((d, dff))).astype(np.float32),
    }
    if bf16:
        w = {k: round_to_bf16(v) for k, v in w.items()}
    return w


def head_weights(shape: ModelShape, seed: int, std: float = 0.02, bf16: bool = False):
    """Embedding table, final norm gain and LM head ([vocab][d_model])."""
    rng = np.random.default_rng(seed)
    e = (std * rng.standard_normal((shape.vocab, shape.d_model))).astype(np.float32)
    f = (1.0 + 0.1 * rng.standard_normal(shape.d_model)).astype(np.float32)
    h = (std * rng.standard_normal((shape.vocab, shape.d_model))).astype(np.float32)
    if bf16:
        e, f, h = round_to_bf16(e), round_to_bf16(f), round_to_bf16(h)
    return {"embed": e, "w_final_norm": f, "lm_head": h}


def hidden_states(n_seq: int, T: int, d: int, seed: int, std: float = 1.0, bf16: bool = False):
    rng = np.random.default_rng(seed)
    x = (std * rng.standard_normal((n_seq, T, d))).astype(np.float32)
    return round_to_bf16(x) if bf16 else x


def iid_actions(n_actions: int, shape_, seed: int) -> np.ndarray:
    """Action ids drawn independently and uniformly per token."""
    rng = np.random.default_rng(seed)
    return rng.integers(0, n_actions, size=shape_, dtype=np.int32)


def markov_actions(n_actions: int, n_seq: int, T: int, seed: int, stay: float = 0.8) -> np.ndarray:
    """Bursty schedules: a_0 uniform; a_t = a_{t-1} with probability `stay`, else a fresh
    uniform draw over all joint action ids; independent per sequence."""
    rng = np.random.default_rng(seed)
    fresh = rng.integers(0, n_actions, size=(n_seq, T), dtype=np.int32)
    hold = rng.random((n_seq, T)) < stay
    ids = np.empty((n_seq, T), np.int32)
    ids[:, 0] = fresh[:, 0]
    for t in range(1, T):
        ids[:, t] = np.where(hold[:, t], ids[:, t - 1], fresh[:, t])
    return ids


def tokens_and_targets(B: int, T: int, vocab: int, seed: int):
    rng = np.random.default_rng(seed)
    return (rng.integers(0, vocab, size=(B, T), dtype=np.int32),
            rng.integers(0, vocab, size=(B, T), dtype=np.int32))


def kv_cache(n_seq: int, n_kv_heads: int, L: int, head_dim: int, seed: int, bf16: bool = False):
    """A filled cache of random N(0,1) keys and values, [n_seq][Hkv][L][dh]."""
    rng = np.random.default_rng(seed)
    k = rng.standard_normal((n_seq, n_kv_heads, L, head_dim), dtype=np.float32)
    v = rng.standard_normal((n_seq, n_kv_heads, L, head_dim), dtype=np.float32)
    if bf16:
        k, v = round_to_bf16(k), round_to_bf16(v)
    return k, v


def with_layers(shape: ModelShape, n_layers: int, vocab: int = None) -> ModelShape:
    return replace(shape, n_layers=n_layers, vocab=shape.vocab if vocab is None else vocab)
