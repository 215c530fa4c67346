"""Edge cases and error paths of the entry points beyond the three main operations: empty inputs are no-ops, bad
configurations come back as status codes before anything is launched, a sequence that does not fit its cache is
skipped and flagged."""
import dataclasses

import numpy as np
import pytest
import torch

from paper_2605_10875_amd import sol, synth

from gpu_util import dev, dev_weights, host

pytestmark = pytest.mark.gpu

SMALL_GQA = synth.ModelShape(d_model=256, n_q_heads=8, n_kv_heads=2, head_dim=64, d_ff=768, n_layers=2, vocab=1024)
TABLE = [synth.DENSE_ACTION, (1, 4, 1, 4, 4)]


def _model(shape, seed, dt=sol.BF16):
    bf = dt == sol.BF16
    layers = [dev_weights(synth.layer_weights(shape, seed + l, bf16=bf), dt) for l in range(shape.n_layers)]
    head = dev_weights(synth.head_weights(shape, seed + 10, bf16=bf), dt)
    return layers, head


def _caches(shape, n_seq, L_max, n_layers=2):
    mk = lambda: torch.zeros((n_seq, shape.n_kv_heads, L_max, shape.head_dim), dtype=torch.bfloat16, device="cuda")
    return [mk() for _ in range(n_layers)], [mk() for _ in range(n_layers)]


def test_empty_inputs_are_no_ops():
    shape = SMALL_GQA
    layers, head = _model(shape, 9000)
    ctx = sol.Sol(shape, TABLE, dtype=sol.BF16, max_positions=64)
    kc, vc = _caches(shape, 2, 64)
    x = torch.zeros((2, 0, shape.d_model), dtype=torch.bfloat16, device="cuda")
    out = ctx.kv_refresh(layers, None, dev(np.zeros(2, np.int32)), kc, vc, x_in=x)          # T = 0
    assert out.shape == (2, 0, shape.d_model) and float(kc[0].abs().max()) == 0.0
    empty_ids = torch.zeros((0, 3, 4), dtype=torch.int32, device="cuda")                     # B = 0
    nll = ctx.episode_loglik(layers, head, torch.zeros((0, 8), dtype=torch.int32, device="cuda"),
                             torch.zeros((0, 4), dtype=torch.int32, device="cuda"),
                             torch.zeros((0, 4), dtype=torch.int32, device="cuda"), empty_ids)
    assert nll.shape == (0, 3, 4)
    r = ctx.reward_advantages(torch.zeros((2, 0, 5), dtype=torch.float32, device="cuda"),
                              torch.zeros((2, 0, 5), dtype=torch.int32, device="cuda"),
                              torch.zeros((2, 3), dtype=torch.float32, device="cuda"), (1, 1, 1), 0.0, 0.85)
    assert r["adv"].shape == (2, 0, 5)
    assert ctx.device_status() == sol.OK
    ctx.close()


def test_refresh_skips_and_flags_a_sequence_that_does_not_fit():
    shape = SMALL_GQA
    layers, _ = _model(shape, 9100)
    ctx = sol.Sol(shape, TABLE, dtype=sol.BF16, max_positions=32)
    kc, vc = _caches(shape, 2, 32)
    x = dev(synth.hidden_states(2, 8, shape.d_model, 9101, bf16=True), sol.BF16)
    ctx.kv_refresh(layers, None, dev(np.array([4, 28], np.int32)), kc, vc, x_in=x)          # 28 + 8 > 32
    assert ctx.device_status() == sol.ERR_CACHE_OVERFLOW
    k0 = host(kc[0])
    assert np.abs(k0[0, :, 4:12]).max() > 0 and np.abs(k0[1]).max() == 0.0                   # sequence 1 untouched
    ctx.close()


def test_page_metadata_entry_points_reject_what_they_do_not_cover():
    shape = SMALL_GQA
    layers, head = _model(shape, 9200)
    kc, vc = _caches(shape, 1, 64)
    lens, ids = dev(np.array([5], np.int32)), dev(np.array([0], np.int32))
    x = dev(synth.hidden_states(1, 1, shape.d_model, 9201, bf16=True)[0], sol.BF16)
    plain = sol.Sol(shape, TABLE, dtype=sol.BF16, max_positions=64)                          # page size 1: no metadata
    with pytest.raises(sol.SolError) as e:
        plain.page_meta_build(kc[0], lens)
    assert e.value.code == sol.ERR_UNSUPPORTED
    with pytest.raises(sol.SolError) as e:
        plain.decode_step(layers, head, ids, lens, kc, vc, x_in=x, page_meta=[kc[0], kc[1]])
    assert e.value.code == sol.ERR_UNSUPPORTED
    plain.close()
    three = dataclasses.replace(shape, n_q_heads=6)                                          # 3 query heads per KV head
    l3, h3 = _model(three, 9210)
    ctx = sol.Sol(three, TABLE, dtype=sol.BF16, max_positions=64, page_size=16)
    meta = [ctx.page_meta_build(k, lens) for k in kc]                                        # building is fine
    with pytest.raises(sol.SolError) as e:
        ctx.decode_step(l3, h3, ids, lens, kc, vc, x_in=x, page_meta=meta)
    assert e.value.code == sol.ERR_UNSUPPORTED
    out, _ = ctx.decode_step(l3, h3, ids, lens, kc, vc, x_in=x)                              # without metadata: general kernel
    assert bool(torch.isfinite(out.float()).all())
    ctx.close()


def test_workspace_too_small_is_reported():
    shape = SMALL_GQA
    layers, head = _model(shape, 9300)
    ctx = sol.Sol(shape, TABLE, dtype=sol.BF16, max_positions=64)
    tiny = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(sol.SolError) as e:
        ctx.episode_loglik(layers, head, dev(np.zeros((1, 16), np.int32)), dev(np.zeros((1, 4), np.int32)),
                           dev(np.zeros((1, 4), np.int32)), dev(np.zeros((1, 2, 4), np.int32)), workspace=tiny)
    assert e.value.code == sol.ERR_WORKSPACE
    kc, vc = _caches(shape, 1, 64)
    with pytest.raises(sol.SolError) as e:
        ctx.kv_refresh(layers, None, dev(np.zeros(1, np.int32)), kc, vc,
                       x_in=torch.zeros((1, 4, shape.d_model), dtype=torch.bfloat16, device="cuda"), workspace=tiny)
    assert e.value.code == sol.ERR_WORKSPACE
    ctx.close()
