"""GPU parity of the episode pass (dense prefill once per input, K schedules of T controlled steps on top of it)
against the oracle's definition; tolerances of test_gpu_parity.py."""
import dataclasses

import numpy as np
import pytest

import oracle
from paper_2605_10875_amd import sol, synth

from gpu_util import dev, dev_weights, host

pytestmark = pytest.mark.gpu

SMALL_GQA = synth.ModelShape(d_model=256, n_q_heads=8, n_kv_heads=2, head_dim=64, d_ff=768, n_layers=2, vocab=1024)


def _run(shape, table, dt, B, K, P, T, seed, **opts):
    bf = dt == sol.BF16
    layers = [synth.layer_weights(shape, seed + l, bf16=bf) for l in range(shape.n_layers)]
    head = synth.head_weights(shape, seed + 10, bf16=bf)
    rng = np.random.default_rng(seed + 11)
    prefix = rng.integers(0, shape.vocab, (B, P)).astype(np.int32)
    tokens, targets = synth.tokens_and_targets(B, T, shape.vocab, seed + 12)
    ids = synth.iid_actions(len(table), (B, K, T), seed + 13)
    o_opts = dict(opts)
    qs = o_opts.pop("quant_sites", oracle.QS_NORTHSTAR)
    ref = oracle.episode_loglik(oracle.make_cfg(shape, quant_sites=qs, act_bf16=bf, **o_opts), oracle.make_table(table),
                                table.index(synth.DENSE_ACTION), head["embed"], layers, head["w_final_norm"],
                                head["lm_head"], prefix, tokens, targets, ids)
    ctx = sol.Sol(shape, table, dtype=dt, max_positions=P + T, quant_sites=qs, **o_opts)
    nll = ctx.episode_loglik([dev_weights(w, dt) for w in layers], dev_weights(head, dt), dev(prefix), dev(tokens),
                             dev(targets), dev(ids))
    assert ctx.device_status() == sol.OK
    ctx.close()
    return host(nll), ref, ids


def test_fp32_episode_pass():
    shape = dataclasses.replace(synth.TINY, n_layers=2)
    nll, ref, _ = _run(shape, synth.TABLE_C1, sol.F32, 2, 3, 20, 6, 8000)
    err = np.abs(nll - ref)
    assert np.quantile(err, 0.95) < 1e-3 and err.max() < 2e-2, (np.quantile(err, 0.95), err.max())


@pytest.mark.parametrize("P,T,K", [(64, 16, 4), (50, 4, 3)])
def test_bf16_episode_pass(P, T, K):
    """(64, 16): the tiled attention at pos0 = P; (50, 4): fewer than 16 steps take the row-per-workgroup kernel."""
    table = synth.action_table((0.125, 0.5, 1.0), (0.0, 0.75), (6, 16))
    nll, ref, ids = _run(SMALL_GQA, table, sol.BF16, 2, K, P, T, 8100 + T)
    bits = np.array([a[4] for a in table])[ids]
    err = np.abs(nll - ref)
    # a step is held to 2e-2 nats if no step of its schedule so far quantised (a flipped code in an earlier step's K/V
    # entries moves every later step of that schedule)
    clean = np.logical_and.accumulate(bits >= 16, axis=2)
    assert (err[clean] < 2e-2).all() and np.median(err) < 1e-2 and err.max() < 0.5, (np.median(err), err.max())


def test_bf16_episode_pass_paper_configuration():
    table = synth.action_table((0.125, 0.5, 1.0), (0.0, 0.75), (6, 16))
    nll, ref, ids = _run(SMALL_GQA, table, sol.BF16, 1, 3, 48, 8, 8200, **sol.PAPER_PRESET)
    err = np.abs(nll - ref)
    assert np.median(err) < 1e-2 and err.max() < 0.5, (np.median(err), err.max())


def test_identical_schedules_give_identical_likelihoods():
    table = synth.action_table((0.25, 1.0), (0.0, 0.5), (8, 16))
    shape = SMALL_GQA
    layers = [dev_weights(synth.layer_weights(shape, 8300 + l, bf16=True), sol.BF16) for l in range(2)]
    head = dev_weights(synth.head_weights(shape, 8310, bf16=True), sol.BF16)
    rng = np.random.default_rng(8311)
    prefix = rng.integers(0, shape.vocab, (1, 32)).astype(np.int32)
    tokens, targets = synth.tokens_and_targets(1, 16, shape.vocab, 8312)
    one = synth.iid_actions(len(table), (1, 1, 16), 8313)
    ids = np.repeat(one, 5, axis=1)
    ctx = sol.Sol(shape, table, dtype=sol.BF16, max_positions=48)
    nll = host(ctx.episode_loglik(layers, head, dev(prefix), dev(tokens), dev(targets), dev(ids)))
    ctx.close()
    assert all(np.array_equal(nll[0, 0], nll[0, k]) for k in range(1, 5))
