"""GPU parity of the reward reduction (Method, Eqs. 2-5, group-relative whitened advantages) against the oracle.
fp32 on the GPU (fp64 for the sums that decide the whitening), fp64 in the oracle: returns within 1e-5 of the
largest return, advantages (unit variance) within 1e-4."""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_10875_amd import sol, synth

from gpu_util import dev, host

pytestmark = pytest.mark.gpu

TABLE = synth.action_table((0.125, 0.25, 0.5, 1.0), (0.0, 0.5, 0.75), (4, 8, 16))


def _case(B, G, T, seed, with_eff):
    rng = np.random.default_rng(seed)
    nll = rng.uniform(0.2, 11.0, (B, G, T)).astype(np.float32)
    ids = rng.integers(0, len(TABLE), (B, G, T)).astype(np.int32)
    targets = rng.uniform(0.3, 1.0, (B, 3)).astype(np.float32)
    eff = None
    if with_eff:
        eff = (rng.uniform(size=(B, T)) < 0.7).astype(np.int32)
        eff[0] = 0                                             # an input without any effective step
    return nll, ids, targets, eff


@pytest.mark.parametrize("B,G,T,with_eff,gamma", [(3, 5, 7, False, 0.85), (2, 8, 2048, True, 0.85), (4, 32, 64, True, 1.0),
                                                  (1, 2, 1, False, 0.5), (2, 3, 300, False, 0.999)])
def test_reward_advantages(B, G, T, with_eff, gamma):
    nll, ids, targets, eff = _case(B, G, T, 7000 + T, with_eff)
    alpha, tau, eps = (3.0, 2.0, 5.0), 0.05, 1e-8
    ref = oracle.reward_advantages(nll, ids, TABLE, targets, alpha, tau, gamma, eff=eff, eps=eps)
    ctx = sol.Sol(synth.TINY, TABLE, dtype=sol.F32, max_positions=16)
    out = ctx.reward_advantages(dev(nll, sol.F32), dev(ids), dev(targets, sol.F32), alpha, tau, gamma,
                                eff=dev(eff) if eff is not None else None, eps=eps)
    assert ctx.device_status() == sol.OK
    ctx.close()
    np.testing.assert_allclose(host(out["avg"]), ref["avg"], rtol=0, atol=2e-7)
    np.testing.assert_allclose(host(out["penalty"]), ref["penalty"], rtol=1e-4, atol=1e-7)
    scale = np.abs(ref["returns"]).max()
    assert np.abs(host(out["returns"]) - ref["returns"]).max() < 1e-5 * scale
    assert np.abs(host(out["signal"]) - ref["signal"]).max() < 1e-5 * max(scale, np.abs(ref["signal"]).max())
    assert np.abs(host(out["adv"]) - ref["adv"]).max() < 1e-4


def test_reward_flags_an_action_outside_the_table_and_rejects_bad_settings():
    nll, ids, targets, _ = _case(1, 2, 5, 7100, False)
    ids[0, 1, 3] = len(TABLE)
    ctx = sol.Sol(synth.TINY, TABLE, dtype=sol.F32, max_positions=16)
    ctx.reward_advantages(dev(nll, sol.F32), dev(ids), dev(targets, sol.F32), (1, 1, 1), 0.0, 0.85)
    assert ctx.device_status() == sol.ERR_ACTION
    with pytest.raises(sol.SolError):
        ctx.reward_advantages(dev(nll, sol.F32), dev(ids), dev(targets, sol.F32), (1, 1, 1), 0.0, 1.5)
    with pytest.raises(sol.SolError):
        ctx.reward_advantages(dev(nll, sol.F32), dev(ids), dev(targets, sol.F32), (-1, 1, 1), 0.0, 0.85)
    ctx.close()
