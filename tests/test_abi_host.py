"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol that
include/sol.h declares, validates configurations and sizes workspaces by pure host arithmetic."""
import ctypes as C
import os
import re

import pytest

from paper_2605_10875_amd import sol, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "sol.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sol_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = sol.lib()
    names = _declared_symbols()
    assert set(names) == set(sol.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def test_no_cpu_fallback_in_binding():
    # the binding marshals arguments only: it must not import the oracle or compute anything itself
    src = open(os.path.join(ROOT, "paper_2605_10875_amd", "sol.py")).read()
    assert "oracle" not in src.replace("no CPU fallback", "")
    csrc = os.path.join(ROOT, "paper_2605_10875_amd", "csrc")
    for f in os.listdir(csrc):
        if os.path.isfile(os.path.join(csrc, f)):
            assert "oracle" not in open(os.path.join(csrc, f)).read()


def test_validate_config_accepts_benchmark_tables():
    for shape, table, dt in ((synth.TINY, synth.TABLE_C1, sol.F32), (synth.LLAMA_1B, synth.TABLE_C2, sol.BF16),
                             (synth.LLAMA_1B, synth.TABLE_C4, sol.BF16), (synth.LLAMA_8B, synth.TABLE_C2, sol.BF16)):
        rc, msg = sol.validate_config(sol.make_cfg(shape, dt, 8192), table)
        assert rc == sol.OK, msg


@pytest.mark.parametrize("bad,code", [
    ((0, 1, 1, 1, 16), sol.ERR_ACTION),       # kappa = 0: softmax over no keys
    ((2, 1, 1, 1, 16), sol.ERR_ACTION),       # kappa > 1
    ((1, 0, 1, 1, 16), sol.ERR_ACTION),
    ((1, 1, 0, 1, 16), sol.ERR_ACTION),       # rho = 0
    ((1, 1, 3, 2, 16), sol.ERR_ACTION),
    ((1, 1, 1, 1, 3), sol.ERR_ACTION),        # fewer than 4 bits
])
def test_validate_config_rejects_bad_actions(bad, code):
    rc, msg = sol.validate_config(sol.make_cfg(synth.TINY, sol.F32, 128), [synth.DENSE_ACTION, bad])
    assert rc == code and "action 1" in msg


def test_validate_config_rejects_bad_shapes_and_accepts_every_variant():
    ok = dict(shape=synth.TINY, dtype=sol.F32, max_positions=128)
    tab = [synth.DENSE_ACTION]
    import dataclasses
    for field, val in (("d_model", 0), ("n_kv_heads", 3), ("head_dim", 63)):
        shp = dataclasses.replace(synth.TINY, **{field: val})
        rc, _ = sol.validate_config(sol.make_cfg(shp, sol.F32, 128), tab)
        assert rc == sol.ERR_INVALID_ARG
    rc, _ = sol.validate_config(sol.make_cfg(synth.TINY, 7, 128), tab)
    assert rc == sol.ERR_INVALID_ARG
    rc, _ = sol.validate_config(sol.make_cfg(synth.TINY, sol.F32, 128), [])
    assert rc == sol.ERR_INVALID_ARG
    for kw in (dict(page_size=4), dict(n_sink=4), dict(n_window=2), dict(prune_site=1), dict(quant_sites=16),
               sol.PAPER_PRESET):
        rc, msg = sol.validate_config(sol.make_cfg(ok["shape"], ok["dtype"], ok["max_positions"], **kw), tab)
        assert rc == sol.OK, msg
    for kw in (dict(page_size=0), dict(n_sink=-1), dict(n_window=-2), dict(prune_site=2), dict(quant_sites=32)):
        rc, _ = sol.validate_config(sol.make_cfg(ok["shape"], ok["dtype"], ok["max_positions"], **kw), tab)
        assert rc == sol.ERR_INVALID_ARG


def test_workspace_bytes_is_host_arithmetic():
    cfg = sol.make_cfg(synth.LLAMA_1B, sol.BF16, 8192)
    a = sol.workspace_bytes(cfg, sol.OP_LAYER_FORWARD, 4, 128, 128)
    b = sol.workspace_bytes(cfg, sol.OP_LAYER_FORWARD, 8, 128, 128)
    assert 0 < a < b
    assert sol.workspace_bytes(cfg, sol.OP_LAYER_FORWARD, 0, 128, 128) == 0
    assert sol.workspace_bytes(cfg, 99, 4, 128, 128) == 0
    assert sol.workspace_bytes(cfg, sol.OP_DECODE_STEP, 64, 1, 8192) > 0
    assert sol.workspace_bytes(cfg, sol.OP_SCHEDULE_LOGLIK, 16, 2048, 2048) > sol.workspace_bytes(
        cfg, sol.OP_LAYER_FORWARD, 16, 2048, 2048)


def test_null_context_is_an_error_not_a_crash():
    L = sol.lib()
    assert L.sol_layer_forward(None, None, None, None, None, None, None, None, 1, 1, 1, None, 0, None) == sol.ERR_INVALID_ARG
    assert L.sol_device_status(None, None) == sol.ERR_INVALID_ARG
    assert L.sol_test_topk_select(None, 1, 1, None, None, None, None) == sol.ERR_INVALID_ARG
    out = C.c_void_p()
    cfg = sol.make_cfg(synth.TINY, sol.F32, 128)
    assert L.sol_create(C.byref(cfg), sol.make_table([(0, 1, 1, 1, 16)]), 1, C.byref(out)) == sol.ERR_ACTION
    assert not out.value


def test_page_meta_bytes_is_host_arithmetic():
    cfg = sol.make_cfg(synth.LLAMA_1B, sol.BF16, 8200, **sol.PAPER_PRESET)
    pages = -(-8200 // 16)
    assert sol.lib().sol_page_meta_bytes(C.byref(cfg), 64, 8200) == 64 * 8 * pages * 2 * 64 * 2
    plain = sol.make_cfg(synth.LLAMA_1B, sol.BF16, 8200)
    assert sol.lib().sol_page_meta_bytes(C.byref(plain), 64, 8200) == 0          # page size 1 has no metadata
    assert sol.lib().sol_page_meta_bytes(C.byref(cfg), 0, 8200) == 0
