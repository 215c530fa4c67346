"""The oracle's C code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only): every entry point on small
inputs with ragged sizes, both selection rules, both site presets, both storage modes, prefix positions, ties and the
error returns, in a child process that has the sanitizer runtime preloaded. Any report aborts the child."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

CHILD = r'''
import dataclasses
import numpy as np
import oracle
from paper_2605_10875_amd import synth

shape = synth.ModelShape(d_model=48, n_q_heads=4, n_kv_heads=2, head_dim=8, d_ff=72, n_layers=2, vocab=37)
table = synth.action_table((0.125, 0.5, 1.0), (0.0, 0.5), (4, 7, 16))
tab = oracle.make_table(table)
rng = np.random.default_rng(5)
for kw in (dict(), dict(act_bf16=True), dict(page_size=4, n_sink=2, n_window=3, prune_site=1, quant_sites=oracle.QS_PAPER),
           dict(page_size=16, n_sink=0, n_window=1), dict(n_sink=3, n_window=2)):
    cfg = oracle.make_cfg(shape, **kw)
    w = synth.layer_weights(shape, 1, std=0.2)
    for n_seq, T, L, p0 in ((1, 1, 1, 0), (2, 13, 20, 7), (3, 17, 17, 0)):
        x = synth.hidden_states(n_seq, T, shape.d_model, 2)
        ids = synth.iid_actions(len(table), (n_seq, T), 3)
        kc = rng.standard_normal((n_seq, shape.n_kv_heads, L, shape.head_dim)).astype(np.float32)
        vc = rng.standard_normal(kc.shape).astype(np.float32)
        out, taps = oracle.layer_forward(cfg, tab, w, x, ids, kc, vc, pos0=np.full(n_seq, p0, np.int32),
                                         taps=("keep_mask", "attn_out", "mlp_act", "x_mid", "q_rot", "h1", "h2"))
        assert np.isfinite(out).all()
    layers = [synth.layer_weights(shape, 10 + l, std=0.2) for l in range(2)]
    head = synth.head_weights(shape, 20, std=0.2)
    tokens, targets = synth.tokens_and_targets(2, 9, shape.vocab, 21)
    ids = synth.iid_actions(len(table), (2, 3, 9), 22)
    nll, hid = oracle.schedule_loglik(cfg, tab, head["embed"], layers, head["w_final_norm"], head["lm_head"], tokens,
                                      targets, ids, want_hidden=True)
    assert np.isfinite(nll).all()
    kcs = [np.zeros((2, shape.n_kv_heads, 12, shape.head_dim), np.float32) for _ in layers]
    vcs = [np.zeros_like(kcs[0]) for _ in layers]
    h, nl = oracle.decode_step(cfg, tab, layers, head["embed"][tokens[:, 0]], ids[:, 0, 0], np.array([0, 11], np.int32), kcs,
                               vcs, head["w_final_norm"], head["lm_head"], targets[:, 0])
    assert np.isfinite(h).all() and np.isfinite(nl).all()
# single operators at the edges: one element, all ties, budget = all / one, zero rows
for n in (1, 2, 31, 64):
    s = (rng.integers(-2, 3, n) * 0.5).astype(np.float32)
    for b in (1, max(1, n // 2), n):
        assert oracle.select_keys(s, b).sum() == b
        assert oracle.select_keys(s, b, n_sink=2, n_window=1).sum() >= min(b, n)
        assert oracle.topm_mask(s, b).sum() == b
    oracle.fake_quant(s, 4); oracle.fake_quant(np.zeros(n, np.float32), 8); oracle.fake_quant(s, 16)
    k = rng.standard_normal((n, 8)).astype(np.float32)
    for S in (1, 4, 16):
        oracle.select_pages(k[0], k, max(1, n // 3), S, n_sink=1, n_window=1)
    oracle.softmax_v(s, np.ones(n, np.uint8), k)
    oracle.nll_row(k[0], k, 0); oracle.rmsnorm(k[0], k[0], 1e-5); oracle.budget(1, 8, n)
# error returns leave no damage behind
for bad in ((lambda: oracle.layer_forward(oracle.make_cfg(shape), tab, w, x, np.full(ids.shape[:1] + (17,), 99, np.int32)[:3], kc, vc)),
            (lambda: oracle.layer_forward(oracle.make_cfg(shape), oracle.make_table([(0, 1, 1, 1, 16)]), w, x, np.zeros((3, 17), np.int32), kc, vc))):
    try:
        bad()
        raise SystemExit("expected an error return")
    except ValueError:
        pass
print("SANITIZED-OK")
'''


def test_oracle_under_address_and_undefined_behaviour_sanitizers():
    from oracle import build
    build.build(force=False, sanitize=True)
    libasan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True, check=True).stdout.strip()
    assert os.path.isabs(libasan), "gcc has no AddressSanitizer runtime"
    env = dict(os.environ, SOL_ORACLE_SANITIZE="1", PYTHONPATH=ROOT, OMP_NUM_THREADS="2",
               ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0:abort_on_error=1",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    env["LD_PRELOAD"] = libasan + (":" + os.environ["LD_PRELOAD"] if os.environ.get("LD_PRELOAD") else "")
    r = subprocess.run([sys.executable, "-c", CHILD], env=env, capture_output=True, text=True, timeout=600, cwd=ROOT)
    assert r.returncode == 0 and "SANITIZED-OK" in r.stdout, (r.returncode, r.stdout[-2000:], r.stderr[-4000:])
