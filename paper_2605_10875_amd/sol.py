"""Thin ctypes binding of libsol.so (the C ABI declared in include/sol.h).

Argument marshalling only: every step of the path runs in the library's HIP kernels. torch is
used for device memory and streams. There is no CPU fallback: a missing library is an error.
"""
import ctypes as C
import os

import torch

from . import build as _build

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_ACTION, ERR_CACHE_OVERFLOW, ERR_HIP = 0, -1, -2, -3, -4, -5, -6
F32, BF16 = 0, 1
QS_QKV_IN, QS_O_IN, QS_GATEUP_IN, QS_DOWN_IN, QS_MLP_OUT = 1, 2, 4, 8, 16
QS_ALL_LINEAR_INPUTS = 15
# the configuration of the paper's own runs (Appendix "Quest masking", "Activation quantization"; sink / window
# sizes from the experiment set-up): pages of 16 keys, 4 sink and 2 window keys, pruning at the MLP input,
# quantiser on the MLP output only
PAPER_PRESET = dict(page_size=16, n_sink=4, n_window=2, prune_site=1, quant_sites=QS_MLP_OUT)
OP_LAYER_FORWARD, OP_DECODE_STEP, OP_SCHEDULE_LOGLIK, OP_KV_REFRESH, OP_REWARD = 0, 1, 2, 3, 4

EXPORTS = ("sol_validate_config", "sol_create", "sol_destroy", "sol_last_error", "sol_workspace_bytes",
           "sol_layer_forward", "sol_decode_step", "sol_schedule_loglik", "sol_device_status",
           "sol_page_meta_bytes", "sol_page_meta_build", "sol_decode_step_paged", "sol_kv_refresh",
           "sol_reward_advantages", "sol_episode_workspace_bytes", "sol_episode_loglik",
           "sol_profile_enable", "sol_profile_read",
           "sol_test_topk_select", "sol_test_prune_mask", "sol_test_prune_quant", "sol_test_quant_codes",
           "sol_test_gemm", "sol_test_attn_threshold", "sol_test_attention_stage", "sol_test_mlp_stage",
           "sol_test_episode_copies_workspace_bytes", "sol_test_episode_loglik_copies",
           "sol_static_scratch_bytes", "sol_decode_step_static", "sol_measure_peaks")


class RewardCfg(C.Structure):
    _fields_ = [("alpha_kappa", C.c_float), ("alpha_rho", C.c_float), ("alpha_eta", C.c_float), ("tau", C.c_float),
                ("gamma", C.c_float), ("eps", C.c_float)]


class ActionDef(C.Structure):
    _fields_ = [("keep_num", C.c_uint32), ("keep_den", C.c_uint32), ("mlp_keep_num", C.c_uint32),
                ("mlp_keep_den", C.c_uint32), ("bits", C.c_uint32)]


class ModelCfg(C.Structure):
    _fields_ = [("d_model", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("d_ff", C.c_int32), ("n_layers", C.c_int32), ("vocab", C.c_int32),
                ("rms_eps", C.c_float), ("rope_theta", C.c_float), ("dtype", C.c_int32),
                ("max_positions", C.c_int32), ("page_size", C.c_int32), ("n_sink", C.c_int32),
                ("n_window", C.c_int32), ("prune_site", C.c_int32), ("quant_sites", C.c_uint32)]


_W_NAMES = ("w_in_norm", "wq", "wk", "wv", "wo", "w_post_norm", "w_gate", "w_up", "w_down")


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _W_NAMES]


class ModelWeights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("layers", C.POINTER(LayerWeights)), ("w_final_norm", C.c_void_p),
                ("lm_head", C.c_void_p)]


class SolError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"sol status {code}: {msg}")
        self.code = code


_lib = None


def lib_path():
    return _build.LIB


def lib():
    """Loads libsol.so, building it first only if it has never been built. A library older than its sources is
    still loaded (a GPU machine runs what was built beforehand) but reported, so that stale results are not mistaken
    for current ones."""
    global _lib
    if _lib is None:
        if not os.path.exists(_build.LIB):
            _build.build()
        elif _build.is_stale():
            import warnings
            warnings.warn("libsol.so is older than its sources: run paper_2605_10875_amd/build.py", RuntimeWarning)
        L = C.CDLL(_build.LIB)
        L.sol_last_error.restype = C.c_char_p
        L.sol_last_error.argtypes = [C.c_void_p]
        L.sol_workspace_bytes.restype = C.c_size_t
        L.sol_workspace_bytes.argtypes = [C.POINTER(ModelCfg), C.c_int, C.c_int, C.c_int, C.c_int]
        L.sol_validate_config.argtypes = [C.POINTER(ModelCfg), C.POINTER(ActionDef), C.c_int]
        L.sol_create.argtypes = [C.POINTER(ModelCfg), C.POINTER(ActionDef), C.c_int, C.POINTER(C.c_void_p)]
        L.sol_destroy.argtypes = [C.c_void_p]
        L.sol_destroy.restype = None
        L.sol_device_status.argtypes = [C.c_void_p, C.c_void_p]
        L.sol_layer_forward.argtypes = [C.c_void_p, C.POINTER(LayerWeights), C.c_void_p, C.c_void_p, C.c_void_p,
                                        C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int,
                                        C.c_void_p, C.c_size_t, C.c_void_p]
        L.sol_decode_step.argtypes = [C.c_void_p, C.POINTER(ModelWeights), C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.c_int, C.c_int,
                                      C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.sol_static_scratch_bytes.restype = C.c_size_t
        L.sol_static_scratch_bytes.argtypes = []
        L.sol_decode_step_static.argtypes = [C.c_void_p, C.POINTER(ModelWeights), C.c_void_p, C.c_void_p, C.c_void_p,
                                             C.c_void_p, C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.c_int, C.c_int,
                                             C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.sol_decode_step_paged.argtypes = [C.c_void_p, C.POINTER(ModelWeights), C.c_void_p, C.c_void_p, C.c_void_p,
                                            C.c_void_p, C.POINTER(C.c_void_p), C.POINTER(C.c_void_p),
                                            C.POINTER(C.c_void_p), C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p,
                                            C.c_void_p, C.c_size_t, C.c_void_p]
        L.sol_kv_refresh.argtypes = [C.c_void_p, C.POINTER(ModelWeights), C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.c_int, C.c_int,
                                     C.c_int, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.sol_reward_advantages.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                            C.POINTER(RewardCfg), C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                            C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.sol_episode_workspace_bytes.restype = C.c_size_t
        L.sol_episode_workspace_bytes.argtypes = [C.POINTER(ModelCfg), C.c_int, C.c_int, C.c_int, C.c_int]
        L.sol_episode_loglik.argtypes = [C.c_void_p, C.POINTER(ModelWeights), C.c_void_p, C.c_void_p, C.c_void_p,
                                         C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                         C.c_size_t, C.c_void_p]
        L.sol_test_episode_copies_workspace_bytes.restype = C.c_size_t
        L.sol_test_episode_copies_workspace_bytes.argtypes = L.sol_episode_workspace_bytes.argtypes
        L.sol_test_episode_loglik_copies.argtypes = L.sol_episode_loglik.argtypes
        L.sol_test_attention_stage.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                               C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.sol_test_mlp_stage.argtypes = [C.c_void_p, C.POINTER(LayerWeights), C.c_void_p, C.c_void_p, C.c_void_p,
                                         C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.sol_page_meta_bytes.restype = C.c_size_t
        L.sol_page_meta_bytes.argtypes = [C.POINTER(ModelCfg), C.c_int, C.c_int]
        L.sol_page_meta_build.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        L.sol_schedule_loglik.argtypes = [C.c_void_p, C.POINTER(ModelWeights), C.c_void_p, C.c_void_p, C.c_void_p,
                                          C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.sol_profile_enable.argtypes = [C.c_void_p, C.c_int]
        L.sol_profile_read.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.POINTER(C.c_char_p), C.POINTER(C.c_float),
                                       C.POINTER(C.c_int)]
        L.sol_test_topk_select.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.sol_test_attn_threshold.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.sol_test_gemm.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p]
        L.sol_test_prune_mask.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]
        L.sol_test_prune_quant.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p,
                                           C.c_size_t, C.c_void_p]
        L.sol_test_quant_codes.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p,
                                           C.c_void_p, C.c_void_p]
        _lib = L
    return _lib


def make_cfg(shape, dtype, max_positions, quant_sites=QS_ALL_LINEAR_INPUTS, page_size=1, n_sink=0, n_window=0,
             prune_site=0):
    return ModelCfg(shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ff, shape.n_layers,
                    shape.vocab, shape.rms_eps, shape.rope_theta, dtype, max_positions, page_size, n_sink, n_window,
                    prune_site, quant_sites)


def make_table(actions):
    arr = (ActionDef * len(actions))()
    for i, a in enumerate(actions):
        arr[i] = ActionDef(*[int(v) for v in a])
    return arr


def validate_config(cfg, actions):
    L = lib()
    tab = make_table(actions) if len(actions) else None
    rc = L.sol_validate_config(C.byref(cfg), tab, len(actions))
    return rc, (L.sol_last_error(None) or b"").decode() if rc else ""


def workspace_bytes(cfg, op, n_seq, T, L_max):
    return int(lib().sol_workspace_bytes(C.byref(cfg), op, n_seq, T, L_max))


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else None


def _stream(stream):
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def _dtype_code(t):
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float32:
        return F32
    raise TypeError(f"unsupported dtype {t.dtype}")


def _i32(t):
    assert t is None or (t.dtype == torch.int32 and t.is_cuda and t.is_contiguous())
    return t


class Sol:
    """One library context: a model configuration plus an action table, on the current device."""

    def __init__(self, shape, actions, dtype=BF16, max_positions=8192, quant_sites=QS_ALL_LINEAR_INPUTS, **kw):
        self.L = lib()
        self.cfg = make_cfg(shape, dtype, max_positions, quant_sites, **kw)
        self.dtype = dtype
        self.tdtype = torch.bfloat16 if dtype == BF16 else torch.float32
        self.table = make_table(actions)
        self.handle = C.c_void_p()
        rc = self.L.sol_create(C.byref(self.cfg), self.table, len(actions), C.byref(self.handle))
        if rc:
            raise SolError(rc, (self.L.sol_last_error(None) or b"").decode())
        self._ws = None

    def close(self):
        if self.handle:
            self.L.sol_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc):
        if rc:
            raise SolError(rc, (self.L.sol_last_error(self.handle) or b"").decode())

    def workspace(self, op, n_seq, T, L_max):
        need = workspace_bytes(self.cfg, op, n_seq, T, L_max)
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        return self._ws

    def _layer_struct(self, w):
        s = LayerWeights()
        for n in _W_NAMES:
            t = w[n]
            assert t.is_cuda and t.is_contiguous() and t.dtype == self.tdtype, n
            setattr(s, n, t.data_ptr())
        return s

    def _model_struct(self, layers, head):
        arr = (LayerWeights * len(layers))()
        for i, w in enumerate(layers):
            arr[i] = self._layer_struct(w)
        mw = ModelWeights()
        mw.layers = C.cast(arr, C.POINTER(LayerWeights))
        if head is not None:
            for n in ("embed", "w_final_norm", "lm_head"):
                t = head.get(n)
                if t is not None:
                    assert t.is_cuda and t.is_contiguous() and t.dtype == self.tdtype, n
                    setattr(mw, n, t.data_ptr())
        return mw, arr

    def layer_forward(self, w, x_in, action_ids, k_cache, v_cache, pos0=None, x_out=None, workspace=None,
                      stream=None):
        """x_in [n_seq][T][d]; action_ids int32 [n_seq][T]; caches [n_seq][Hkv][L_max][dh] (updated)."""
        n_seq, T, d = x_in.shape
        L_max = k_cache.shape[2]
        assert x_in.is_contiguous() and k_cache.is_contiguous() and v_cache.is_contiguous()
        assert x_in.dtype == self.tdtype and k_cache.dtype == self.tdtype and v_cache.dtype == self.tdtype
        if x_out is None:
            x_out = torch.empty_like(x_in)
        ws = workspace if workspace is not None else self.workspace(OP_LAYER_FORWARD, n_seq, T, L_max)
        ls = self._layer_struct(w)
        rc = self.L.sol_layer_forward(self.handle, C.byref(ls), _ptr(x_in), _ptr(x_out), _ptr(_i32(action_ids)),
                                      _ptr(_i32(pos0)), _ptr(k_cache), _ptr(v_cache), n_seq, T, L_max,
                                      _ptr(ws), ws.numel(), _stream(stream))
        self._check(rc)
        return x_out

    def test_attention_stage(self, q, action_ids, k_cache, v_cache, pos0=None, stream=None):
        """Stage hook: q [n_seq][T][Hq*dh] (storage dtype, after the rotary embedding) against caches that already
        hold positions [0, pos0 + T). Returns the attention output float32 [n_seq][T][Hq*dh]."""
        n_seq, T, _ = q.shape
        L_max = k_cache.shape[2]
        assert q.is_contiguous() and q.dtype == self.tdtype and k_cache.dtype == self.tdtype
        o = torch.empty(q.shape, dtype=torch.float32, device="cuda")
        ws = self.workspace(OP_LAYER_FORWARD, n_seq, T, L_max)
        self._check(self.L.sol_test_attention_stage(self.handle, _ptr(q), _ptr(_i32(action_ids)), _ptr(_i32(pos0)),
                                                    _ptr(k_cache), _ptr(v_cache), n_seq, T, L_max, _ptr(o), _ptr(ws),
                                                    ws.numel(), _stream(stream)))
        return o

    def test_mlp_stage(self, w, h2, x2, action_ids, stream=None):
        """Stage hook: h2 [n_seq][T][d] (storage dtype, the MLP input as the projections read it), x2 float32
        [n_seq][T][d] (residual after attention). Returns (a [n_seq][T][d_ff], x_out [n_seq][T][d]), storage dtype."""
        n_seq, T, d = h2.shape
        assert h2.is_contiguous() and h2.dtype == self.tdtype and x2.dtype == torch.float32 and x2.is_contiguous()
        a = torch.empty((n_seq, T, self.cfg.d_ff), dtype=self.tdtype, device="cuda")
        out = torch.empty_like(h2)
        ws = self.workspace(OP_LAYER_FORWARD, n_seq, T, T)
        ls = self._layer_struct(w)
        self._check(self.L.sol_test_mlp_stage(self.handle, C.byref(ls), _ptr(h2), _ptr(x2), _ptr(_i32(action_ids)),
                                              n_seq, T, _ptr(a), _ptr(out), _ptr(ws), ws.numel(), _stream(stream)))
        return a, out

    def page_meta_build(self, k_cache, cache_len, stream=None):
        """Page metadata (channel-wise maxima and minima per page) of one layer's key cache for keys
        [0, cache_len[s]); returns the new buffer [n_seq][Hkv][pages][2 * head_dim]."""
        n_seq, hkv, L_max, dh = k_cache.shape
        pages = (L_max + self.cfg.page_size - 1) // self.cfg.page_size
        need = self.L.sol_page_meta_bytes(C.byref(self.cfg), n_seq, L_max)
        assert need in (0, n_seq * hkv * pages * 2 * dh * k_cache.element_size())     # 0: no metadata for this configuration
        meta = torch.zeros((n_seq, hkv, pages, 2 * dh), dtype=k_cache.dtype, device="cuda")
        self._check(self.L.sol_page_meta_build(self.handle, _ptr(k_cache), _ptr(_i32(cache_len)), n_seq, L_max,
                                               _ptr(meta), _stream(stream)))
        return meta

    def decode_step(self, layers, head, action_ids, cache_len, k_caches, v_caches, token_ids=None, x_in=None,
                    targets=None, want_hidden=True, workspace=None, stream=None, page_meta=None):
        """One token per sequence through all layers. Returns (hidden [B][d] or None, nll [B] or None).
        page_meta: per-layer metadata buffers (page_meta_build), updated in place, for the page rule."""
        B = action_ids.shape[0]
        L_max = k_caches[0].shape[2]
        mw, keep = self._model_struct(layers, head)
        kp = (C.c_void_p * len(k_caches))(*[t.data_ptr() for t in k_caches])
        vp = (C.c_void_p * len(v_caches))(*[t.data_ptr() for t in v_caches])
        x_out = torch.empty((B, self.cfg.d_model), dtype=self.tdtype, device="cuda") if want_hidden else None
        nll = torch.empty(B, dtype=torch.float32, device="cuda") if targets is not None else None
        ws = workspace if workspace is not None else self.workspace(OP_DECODE_STEP, B, 1, L_max)
        if page_meta is not None:
            mp = (C.c_void_p * len(page_meta))(*[t.data_ptr() for t in page_meta])
            rc = self.L.sol_decode_step_paged(self.handle, C.byref(mw), _ptr(_i32(token_ids)), _ptr(x_in),
                                              _ptr(_i32(action_ids)), _ptr(_i32(cache_len)), kp, vp, mp, B, L_max,
                                              _ptr(x_out), _ptr(_i32(targets)), _ptr(nll), _ptr(ws), ws.numel(),
                                              _stream(stream))
        else:
            rc = self.L.sol_decode_step(self.handle, C.byref(mw), _ptr(_i32(token_ids)), _ptr(x_in),
                                        _ptr(_i32(action_ids)), _ptr(_i32(cache_len)), kp, vp, B, L_max, _ptr(x_out),
                                        _ptr(_i32(targets)), _ptr(nll), _ptr(ws), ws.numel(), _stream(stream))
        del keep
        self._check(rc)
        return x_out, nll

    def decode_step_static(self, layers, head, action_ids, cache_len, k_caches, v_caches, token_ids=None, x_in=None,
                           targets=None, x_out=None, nll_out=None, stream=None):
        """decode_step without a workspace: the library's static device scratch is used and nothing is allocated by
        the library (outputs given by the caller are written in place; missing ones are created here, by torch)."""
        B = action_ids.shape[0]
        L_max = k_caches[0].shape[2]
        mw, keep = self._model_struct(layers, head)
        kp = (C.c_void_p * len(k_caches))(*[t.data_ptr() for t in k_caches])
        vp = (C.c_void_p * len(v_caches))(*[t.data_ptr() for t in v_caches])
        if x_out is None:
            x_out = torch.empty((B, self.cfg.d_model), dtype=self.tdtype, device="cuda")
        if nll_out is None and targets is not None:
            nll_out = torch.empty(B, dtype=torch.float32, device="cuda")
        rc = self.L.sol_decode_step_static(self.handle, C.byref(mw), _ptr(_i32(token_ids)), _ptr(x_in),
                                           _ptr(_i32(action_ids)), _ptr(_i32(cache_len)), kp, vp, B, L_max, _ptr(x_out),
                                           _ptr(_i32(targets)), _ptr(nll_out) if targets is not None else None,
                                           _stream(stream))
        del keep
        self._check(rc)
        return x_out, (nll_out if targets is not None else None)

    def kv_refresh(self, layers, head, pos0, k_caches, v_caches, token_ids=None, x_in=None, page_meta=None,
                   want_hidden=True, workspace=None, stream=None):
        """Dense pass of all layers over the T known tokens at positions pos0[s].., rewriting their K/V (and the
        pages of page_meta that hold them). Returns the last layer's output [n_seq][T][d] or None."""
        src = token_ids if token_ids is not None else x_in
        n_seq, T = src.shape[0], src.shape[1]
        L_max = k_caches[0].shape[2]
        mw, keep = self._model_struct(layers, head)
        kp = (C.c_void_p * len(k_caches))(*[t.data_ptr() for t in k_caches])
        vp = (C.c_void_p * len(v_caches))(*[t.data_ptr() for t in v_caches])
        mp = (C.c_void_p * len(page_meta))(*[t.data_ptr() for t in page_meta]) if page_meta is not None else None
        x_out = torch.empty((n_seq, T, self.cfg.d_model), dtype=self.tdtype, device="cuda") if want_hidden else None
        ws = workspace if workspace is not None else self.workspace(OP_KV_REFRESH, n_seq, T, L_max)
        rc = self.L.sol_kv_refresh(self.handle, C.byref(mw), _ptr(_i32(token_ids)), _ptr(x_in), _ptr(_i32(pos0)), kp, vp,
                                   mp, n_seq, T, L_max, _ptr(x_out), _ptr(ws), ws.numel(), _stream(stream))
        del keep
        self._check(rc)
        return x_out

    def episode_loglik(self, layers, head, prefix_tokens, tokens, targets, action_ids, nll_out=None, workspace=None,
                       stream=None, force_copies=False):
        """prefix_tokens int32 [B][P]; tokens/targets int32 [B][T]; action_ids int32 [B][K][T]: dense prefill once per
        input, then K schedules of T controlled steps on it. Returns nll float32 [B][K][T] (nats).
        force_copies: the test hook that gives every schedule its own copy of the prefix cache."""
        B, K, T = action_ids.shape
        P = prefix_tokens.shape[1]
        mw, keep = self._model_struct(layers, head)
        if nll_out is None:
            nll_out = torch.empty((B, K, T), dtype=torch.float32, device="cuda")
        size_fn = self.L.sol_test_episode_copies_workspace_bytes if force_copies else self.L.sol_episode_workspace_bytes
        run_fn = self.L.sol_test_episode_loglik_copies if force_copies else self.L.sol_episode_loglik
        need = int(size_fn(C.byref(self.cfg), B, K, P, T))
        ws = workspace if workspace is not None else torch.empty(need, dtype=torch.uint8, device="cuda")
        rc = run_fn(self.handle, C.byref(mw), _ptr(_i32(prefix_tokens)), _ptr(_i32(tokens)),
                    _ptr(_i32(targets)), _ptr(_i32(action_ids)), B, K, P, T, _ptr(nll_out), _ptr(ws),
                    ws.numel(), _stream(stream))
        del keep
        self._check(rc)
        return nll_out

    def reward_advantages(self, nll, action_ids, targets, alpha, tau, gamma, eff=None, eps=1e-8, stream=None):
        """nll float32 / action_ids int32 [B][G][T], targets float32 [B][3], eff int32 [B][T] or None.
        Returns dict of device tensors: avg [B][G][3], penalty [B][G], returns, signal, adv [B][G][T]."""
        B, G, T = nll.shape
        f = lambda *sh: torch.empty(sh, dtype=torch.float32, device="cuda")
        out = {"avg": f(B, G, 3), "penalty": f(B, G), "returns": f(B, G, T), "signal": f(B, G, T), "adv": f(B, G, T)}
        rc = RewardCfg(float(alpha[0]), float(alpha[1]), float(alpha[2]), float(tau), float(gamma), float(eps))
        need = workspace_bytes(self.cfg, OP_REWARD, B, T, 0)
        ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        assert nll.dtype == torch.float32 and nll.is_contiguous() and targets.dtype == torch.float32
        self._check(self.L.sol_reward_advantages(self.handle, _ptr(nll), _ptr(_i32(action_ids)), _ptr(_i32(eff)),
                                                 _ptr(targets), C.byref(rc), B, G, T, _ptr(out["avg"]),
                                                 _ptr(out["penalty"]), _ptr(out["returns"]), _ptr(out["signal"]),
                                                 _ptr(out["adv"]), _ptr(ws), ws.numel(), _stream(stream)))
        return out

    def schedule_loglik(self, layers, head, tokens, targets, action_ids, nll_out=None, workspace=None, stream=None):
        """tokens/targets int32 [B][T]; action_ids int32 [B][G][T]. Returns nll float32 [B][G][T] (nats)."""
        B, G, T = action_ids.shape
        mw, keep = self._model_struct(layers, head)
        if nll_out is None:
            nll_out = torch.empty((B, G, T), dtype=torch.float32, device="cuda")
        ws = workspace if workspace is not None else self.workspace(OP_SCHEDULE_LOGLIK, B * G, T, T)
        rc = self.L.sol_schedule_loglik(self.handle, C.byref(mw), _ptr(_i32(tokens)), _ptr(_i32(targets)),
                                        _ptr(_i32(action_ids)), B, G, T, _ptr(nll_out), _ptr(ws), ws.numel(),
                                        _stream(stream))
        del keep
        self._check(rc)
        return nll_out

    def profile_enable(self, max_stage_records):
        self._check(self.L.sol_profile_enable(self.handle, max_stage_records))

    def profile_read(self, stream=None):
        """Returns {stage name: (total ms, brackets)} since the last read (synchronises the stream)."""
        n = 32
        names = (C.c_char_p * n)()
        ms = (C.c_float * n)()
        calls = (C.c_int * n)()
        got = self.L.sol_profile_read(self.handle, _stream(stream), n, names, ms, calls)
        if got < 0:
            self._check(got)
        return {names[i].decode(): (float(ms[i]), int(calls[i])) for i in range(got) if calls[i]}

    def device_status(self, stream=None):
        return int(self.L.sol_device_status(self.handle, _stream(stream)))


def measure_peaks(scratch_bytes=2 << 30, reps=10, stream=None):
    """(bf16 MFMA TFLOP/s, device copy GB/s, device read GB/s) this GPU reaches in the library's peak microbenchmarks."""
    buf = torch.empty(scratch_bytes, dtype=torch.uint8, device="cuda").zero_()
    tf, gb, rd = C.c_float(0), C.c_float(0), C.c_float(0)
    L = lib()
    L.sol_measure_peaks.argtypes = [C.c_void_p, C.c_size_t, C.c_int, C.POINTER(C.c_float), C.POINTER(C.c_float),
                                    C.POINTER(C.c_float), C.c_void_p]
    rc = L.sol_measure_peaks(_ptr(buf), buf.numel(), reps, C.byref(tf), C.byref(gb), C.byref(rd), _stream(stream))
    if rc:
        raise SolError(rc, "sol_measure_peaks")
    return float(tf.value), float(gb.value), float(rd.value)


def topk_select(scores, n_valid, k, stream=None):
    """scores float32 [rows][n_cols] (cuda); n_valid, k int32 [rows]. Returns uint8 keep mask."""
    rows, n_cols = scores.shape
    keep = torch.zeros((rows, n_cols), dtype=torch.uint8, device="cuda")
    rc = lib().sol_test_topk_select(_ptr(scores), rows, n_cols, _ptr(_i32(n_valid)), _ptr(_i32(k)), _ptr(keep),
                                    _stream(stream))
    if rc:
        raise SolError(rc, "sol_test_topk_select")
    return keep


def attn_threshold(scores, n_valid, k, stream=None):
    """As topk_select, through the row stage of the batched threshold kernel (n_cols <= 4096)."""
    rows, n_cols = scores.shape
    keep = torch.zeros((rows, n_cols), dtype=torch.uint8, device="cuda")
    rc = lib().sol_test_attn_threshold(_ptr(scores), rows, n_cols, _ptr(_i32(n_valid)), _ptr(_i32(k)), _ptr(keep),
                                       _stream(stream))
    if rc:
        raise SolError(rc, "sol_test_attn_threshold")
    return keep


def gemm(a, w, stream=None):
    """a bf16 [M][K], w bf16 [N][K] (cuda): fp32 [M][N] = a * w^T by the layer's MFMA GEMM."""
    M, K = a.shape
    N = w.shape[0]
    c = torch.empty((M, N), dtype=torch.float32, device="cuda")
    rc = lib().sol_test_gemm(_ptr(a), _ptr(w), _ptr(c), M, N, K, _stream(stream))
    if rc:
        raise SolError(rc, "sol_test_gemm")
    return c


def prune_mask(a, m, stream=None):
    rows, n = a.shape
    keep = torch.zeros((rows, n), dtype=torch.uint8, device="cuda")
    rc = lib().sol_test_prune_mask(_ptr(a), rows, n, _ptr(_i32(m)), _ptr(keep), _stream(stream))
    if rc:
        raise SolError(rc, "sol_test_prune_mask")
    return keep


def prune_quant(a, m, bits, stream=None):
    """Runs the layer's prune + quantise kernel in place on a copy of a [rows][n] (bf16 or fp32)."""
    rows, n = a.shape
    out = a.clone().contiguous()
    scratch = torch.empty(max(16 * rows, 16), dtype=torch.uint8, device="cuda")
    rc = lib().sol_test_prune_quant(_ptr(out), _dtype_code(out), rows, n, _ptr(_i32(m)), _ptr(_i32(bits)),
                                    _ptr(scratch), scratch.numel(), _stream(stream))
    if rc:
        raise SolError(rc, "sol_test_prune_quant")
    return out


def quant_codes(z, bits, stream=None):
    rows, n = z.shape
    codes = torch.zeros((rows, n), dtype=torch.int32, device="cuda")
    scale = torch.zeros(rows, dtype=torch.float32, device="cuda")
    zhat = torch.zeros((rows, n), dtype=torch.float32, device="cuda")
    rc = lib().sol_test_quant_codes(_ptr(z), rows, n, _ptr(_i32(bits)), _ptr(codes), _ptr(scale), _ptr(zhat),
                                    _stream(stream))
    if rc:
        raise SolError(rc, "sol_test_quant_codes")
    return codes, scale, zhat
