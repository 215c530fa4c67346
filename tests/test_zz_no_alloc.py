"""The decode step for callers that cannot allocate (sol_decode_step_static: the step's scratch lives in a file-scope
device array of the library) against sol_decode_step with a caller workspace: same kernels on the same inputs, so the
outputs and the appended K/V rows must agree bit for bit; two calls in a row, the second with a smaller input, so that
what the first call left in the shared array is shown not to leak into the second."""
import dataclasses

import numpy as np
import pytest
import torch

from paper_2605_10875_amd import sol, synth

from gpu_util import dev, dev_weights

pytestmark = pytest.mark.gpu


def _case(shape, table, B, L, seed):
    L_max = L + 8
    rng = np.random.default_rng(seed)
    cache_len = rng.integers(1, L + 1, B).astype(np.int32)
    ids = synth.iid_actions(len(table), (B,), seed + 1)
    tokens, targets = synth.tokens_and_targets(B, 1, shape.vocab, seed + 2)
    kcs, vcs = [], []
    for l in range(shape.n_layers):
        k, v = synth.kv_cache(B, shape.n_kv_heads, L_max, shape.head_dim, seed + 10 + l, bf16=True)
        kcs.append(k); vcs.append(v)
    return cache_len, ids, tokens[:, 0], targets[:, 0], kcs, vcs


def test_static_scratch_decode_step_equals_the_workspace_one():
    shape = dataclasses.replace(synth.LLAMA_1B, n_layers=2, vocab=2048)
    table = synth.TABLE_C4
    layers = [dev_weights(synth.layer_weights(shape, 6000 + l, bf16=True), sol.BF16) for l in range(shape.n_layers)]
    head = dev_weights(synth.head_weights(shape, 6100, bf16=True), sol.BF16)
    ctx = sol.Sol(shape, table, dtype=sol.BF16, max_positions=1300)
    assert sol.lib().sol_static_scratch_bytes() == 64 << 20
    for B, L, seed in ((24, 1200, 6200), (5, 300, 6300)):                 # the second call is the smaller one
        cache_len, ids, tokens, targets, kcs, vcs = _case(shape, table, B, L, seed)
        res = []
        for static in (False, True):
            kd = [dev(k, sol.BF16) for k in kcs]
            vd = [dev(v, sol.BF16) for v in vcs]
            fn = ctx.decode_step_static if static else ctx.decode_step
            hid, nll = fn(layers, head, dev(ids), dev(cache_len), kd, vd, token_ids=dev(tokens), targets=dev(targets))
            assert ctx.device_status() == sol.OK
            res.append((hid, nll, kd, vd))
        (h0, n0, k0, v0), (h1, n1, k1, v1) = res
        assert torch.isfinite(h0.float()).all() and torch.isfinite(n0).all()
        assert torch.equal(h0, h1) and torch.equal(n0, n1)
        for l in range(shape.n_layers):
            assert torch.equal(k0[l], k1[l]) and torch.equal(v0[l], v1[l])
    # a step that does not fit the static array is refused before any launch, with a message that says so
    big = sol.Sol(dataclasses.replace(shape, vocab=128256), table, dtype=sol.BF16, max_positions=64)
    B = 200
    need = sol.workspace_bytes(big.cfg, sol.OP_DECODE_STEP, B, 1, 64)
    assert need > 64 << 20
    cache_len, ids, tokens, targets, kcs, vcs = _case(shape, table, B, 40, 6400)
    with pytest.raises(sol.SolError) as e:
        big.decode_step_static(layers, head, dev(ids), dev(cache_len), [dev(k, sol.BF16) for k in kcs],
                               [dev(v, sol.BF16) for v in vcs], token_ids=dev(tokens))
    assert e.value.code == sol.ERR_WORKSPACE and "static" in str(e.value)
    big.close()
    ctx.close()
