"""ctypes binding of libtide_draft.so: the same names as the C ABI, argument marshalling only.

Every step of the draft-training path runs in the library's HIP kernels; nothing here computes.
Importing this module fails loudly if the library has not been built (there is no fallback path).
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtide_draft.so")

TIDE_OK = 0
TIDE_ERR_NULL = -1
TIDE_ERR_CONFIG = -2
TIDE_ERR_WORKSPACE = -3
TIDE_ERR_HIP = -4
TIDE_DTYPE_FP32 = 0
TIDE_DTYPE_BF16 = 1
LAYOUT_NT, LAYOUT_NN, LAYOUT_TN = 0, 1, 2

TENSOR_NAMES = ("w_fc", "g1", "w_qkv", "w_o", "g2", "w_gate", "w_up", "w_down", "g3", "w_lm")


class TideDraftConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("batch", "seq", "n_capture", "target_hidden", "hidden",
                                         "n_heads", "n_kv_heads", "head_dim", "ffn", "vocab")] + \
               [(n, C.c_float) for n in ("rope_theta", "rms_eps", "beta1", "beta2", "adam_eps",
                                         "weight_decay")] + [("dtype", C.c_int32), ("lm_block_rows", C.c_int32),
                                                               ("lm_keep_all_rows", C.c_int32)]


class TideDraftTensors(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in TENSOR_NAMES]


class TideAdamState(C.Structure):
    _fields_ = [("m", TideDraftTensors), ("v", TideDraftTensors), ("master", TideDraftTensors),
                ("step", C.c_int64)]


class TideTokenInput(C.Structure):
    """tide_token_input: the token-input variant's frozen embedding table, ids, W_in and its training state."""
    _fields_ = [("embed", C.c_void_p), ("embed_rows", C.c_int32), ("input_ids", C.c_void_p), ("w_in", C.c_void_p),
                ("grad_w_in", C.c_void_p), ("m_w_in", C.c_void_p), ("v_w_in", C.c_void_p), ("master_w_in", C.c_void_p)]


class TideError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"tide error {code}: {msg}")
        self.code = code


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it first (python -m paper_2602_05145_amd.build or "
            "__graft_entry__.build()); there is no non-HIP fallback")
    return C.CDLL(LIB_PATH)


_lib = _load()
_cfgp, _tp, _ap = C.POINTER(TideDraftConfig), C.POINTER(TideDraftTensors), C.POINTER(TideAdamState)
_vp, _i64, _i32, _f32, _sz = C.c_void_p, C.c_int64, C.c_int, C.c_float, C.c_size_t

_lib.tide_last_error.restype = C.c_char_p
_lib.tide_last_error.argtypes = []
_lib.tide_draft_workspace_bytes.restype = _sz
_lib.tide_draft_workspace_bytes.argtypes = [_cfgp]
_lib.tide_draft_workspace_offset.restype = _i64
_lib.tide_draft_workspace_offset.argtypes = [_cfgp, C.c_char_p]
_lib.tide_draft_forward.restype = _i32
_lib.tide_draft_forward.argtypes = [_cfgp, _tp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.tide_draft_forward_packed.restype = _i32
_lib.tide_draft_forward_packed.argtypes = [_cfgp, _tp, _vp, _vp, _vp, _vp, _i32, _i32, _vp, _vp, _vp, _sz, _vp]
_lib.tide_draft_train_step_packed.restype = _i32
_lib.tide_draft_train_step_packed.argtypes = [_cfgp, _tp, _tp, _ap, _vp, _vp, _vp, _vp, _i32, _i32,
                                              C.c_float, _vp, _vp, _sz, _vp]
_lib.tide_draft_train_step_dev.restype = _i32
_lib.tide_draft_train_step_dev.argtypes = [_cfgp, _tp, _tp, _ap, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.tide_draft_eval.restype = _i32
_lib.tide_draft_eval.argtypes = [_cfgp, _tp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.tide_draft_train_step.restype = _i32
_lib.tide_draft_train_step.argtypes = [_cfgp, _tp, _tp, _ap, _vp, _vp, _vp, _f32, _vp, _vp, _sz, _vp]
_tokp = C.POINTER(TideTokenInput)
_lib.tide_draft_forward_tok.restype = _i32
_lib.tide_draft_forward_tok.argtypes = [_cfgp, _tp, _tokp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.tide_draft_train_step_tok.restype = _i32
_lib.tide_draft_train_step_tok.argtypes = [_cfgp, _tp, _tp, _ap, _tokp, _vp, _vp, _vp, _f32, _vp, _vp, _sz, _vp]
_lib.tide_draft_unroll_workspace_bytes.restype = _sz
_lib.tide_draft_unroll_workspace_bytes.argtypes = [_cfgp, _i32]
_lib.tide_draft_unroll_workspace_offset.restype = _i64
_lib.tide_draft_unroll_workspace_offset.argtypes = [_cfgp, _i32, _i32, C.c_char_p]
_lib.tide_draft_eval_unroll.restype = _i32
_lib.tide_draft_eval_unroll.argtypes = [_cfgp, _tp, _tokp, _vp, _vp, _vp, _i32, _vp, _vp, _vp, _sz, _vp]
_lib.tide_draft_train_step_unroll.restype = _i32
_lib.tide_draft_train_step_unroll.argtypes = [_cfgp, _tp, _tp, _ap, _tokp, _vp, _vp, _vp, _i32, C.POINTER(C.c_float), _f32, _vp, _vp, _sz, _vp]
_lib.tide_draft_eval_unroll_packed.restype = _i32
_lib.tide_draft_eval_unroll_packed.argtypes = [_cfgp, _tp, _tokp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _vp, _vp, _vp, _sz, _vp]
_lib.tide_draft_train_step_unroll_packed.restype = _i32
_lib.tide_draft_train_step_unroll_packed.argtypes = [_cfgp, _tp, _tp, _ap, _tokp, _vp, _vp, _vp, _vp, _i32, _i32, _i32,
                                                     C.POINTER(C.c_float), _f32, _vp, _vp, _sz, _vp]
_lib.tide_gemm_workspace_bytes.restype = _sz
_lib.tide_gemm_workspace_bytes.argtypes = [_i32, _i64, _i64, _i64, _i32]
_lib.tide_gemm.restype = _i32
_lib.tide_gemm.argtypes = [_i32, _i64, _i64, _i64, _f32, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _vp, _sz, _vp]
_lib.tide_rmsnorm_fwd.restype = _i32
_lib.tide_rmsnorm_fwd.argtypes = [_i64, _i64, _vp, _vp, _f32, _vp, _vp, _i32, _vp]
_lib.tide_rmsnorm_bwd_scratch_bytes.restype = _sz
_lib.tide_rmsnorm_bwd_scratch_bytes.argtypes = [_i64, _i64]
_lib.tide_rmsnorm_bwd.restype = _i32
_lib.tide_rmsnorm_bwd.argtypes = [_i64, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _vp]
_lib.tide_rmsnorm_bwd_static.restype = _i32
_lib.tide_rmsnorm_bwd_static.argtypes = [_i64, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _vp]
_lib.tide_attention_fwd.restype = _i32
_lib.tide_attention_fwd.argtypes = [_i32] * 5 + [_vp, _vp, _vp, _i32, _vp]
_lib.tide_attention_bwd.restype = _i32
_lib.tide_attention_bwd.argtypes = [_i32] * 5 + [_vp, _vp, _vp, _vp, _vp, _vp, _i32, _vp]
_lib.tide_ce_train.restype = _i32
_lib.tide_ce_train.argtypes = [_i64, _i32, _vp, _i64, _vp, _vp, _vp, _vp, _i32, _vp]
_lib.tide_rope.restype = _i32
_lib.tide_rope.argtypes = [_i32] * 5 + [_f32, _vp, _vp, _i32, _i32, _vp]

_lib.tide_profile_start.restype = _i32
_lib.tide_profile_start.argtypes = []
_lib.tide_profile_stop.restype = _i32
_lib.tide_profile_stop.argtypes = [C.c_char_p, _sz]

EXPORTED = ("tide_last_error", "tide_draft_workspace_bytes", "tide_draft_workspace_offset",
            "tide_draft_forward", "tide_draft_eval", "tide_draft_train_step", "tide_draft_train_step_dev", "tide_draft_forward_packed",
    "tide_draft_train_step_packed", "tide_draft_forward_tok", "tide_draft_train_step_tok",
    "tide_draft_unroll_workspace_bytes", "tide_draft_unroll_workspace_offset", "tide_draft_eval_unroll", "tide_draft_train_step_unroll",
    "tide_draft_eval_unroll_packed", "tide_draft_train_step_unroll_packed",
    "tide_mfma_probe",
    "tide_ingest_create", "tide_ingest_destroy", "tide_ingest_acquire", "tide_ingest_submit", "tide_ingest_wait",
    "tide_ingest_done", "tide_ingest_last_error", "tide_gemm_workspace_bytes", "tide_gemm",
            "tide_rmsnorm_fwd", "tide_rmsnorm_bwd_scratch_bytes", "tide_rmsnorm_bwd", "tide_rmsnorm_bwd_static",
            "tide_attention_fwd", "tide_attention_bwd", "tide_rope", "tide_ce_train", "tide_profile_start",
            "tide_profile_stop")


def lib():
    """The loaded ctypes library (for calls that need raw arguments)."""
    return _lib


def tide_last_error() -> str:
    return _lib.tide_last_error().decode()


def _check(rc):
    if rc != TIDE_OK:
        raise TideError(rc, tide_last_error())
    return rc


def make_config(cfg: dict) -> TideDraftConfig:
    """dict (see workloads.CONFIGS) -> C struct."""
    c = TideDraftConfig()
    for n in ("batch", "seq", "n_capture", "target_hidden", "hidden", "n_heads", "n_kv_heads",
              "head_dim", "ffn", "vocab"):
        setattr(c, n, int(cfg[n]))
    for n in ("rope_theta", "rms_eps", "beta1", "beta2", "adam_eps", "weight_decay"):
        setattr(c, n, float(cfg[n]))
    dt = cfg["dtype"]
    c.dtype = {"fp32": TIDE_DTYPE_FP32, "bf16": TIDE_DTYPE_BF16}.get(dt, dt)
    c.lm_block_rows = int(cfg.get("lm_block_rows", 0))
    c.lm_keep_all_rows = int(cfg.get("lm_keep_all_rows", 0))
    return c


def _ptr(x):
    """device pointer of a torch tensor / raw int / None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def make_tensors(d) -> TideDraftTensors:
    """dict name -> torch tensor (or int pointer); missing names become NULL."""
    t = TideDraftTensors()
    for n in TENSOR_NAMES:
        setattr(t, n, _ptr(d.get(n)) if d is not None else None)
    return t


def make_token_input(embed, input_ids, w_in, grad_w_in=None, m_w_in=None, v_w_in=None, master_w_in=None) -> TideTokenInput:
    """torch tensors (or int pointers / None) -> C struct; embed_rows is embed's first dimension."""
    t = TideTokenInput()
    t.embed, t.embed_rows, t.input_ids, t.w_in = _ptr(embed), int(embed.shape[0]), _ptr(input_ids), _ptr(w_in)
    t.grad_w_in, t.m_w_in, t.v_w_in, t.master_w_in = _ptr(grad_w_in), _ptr(m_w_in), _ptr(v_w_in), _ptr(master_w_in)
    return t


def tide_draft_forward_tok(cfg, params, tok, hidden_buf, tokens, loss_mask, loss_out, top1_out, workspace,
                           workspace_bytes, stream, check=True):
    rc = _lib.tide_draft_forward_tok(C.byref(cfg) if cfg is not None else None,
                                     C.byref(params) if params is not None else None,
                                     C.byref(tok) if tok is not None else None,
                                     _ptr(hidden_buf), _ptr(tokens), _ptr(loss_mask), _ptr(loss_out),
                                     _ptr(top1_out), _ptr(workspace), int(workspace_bytes), stream)
    return _check(rc) if check else rc


def tide_draft_train_step_dev(cfg, params, grads, adam_state, hidden_buf, tokens, loss_mask, lr_dev, step_dev, loss_out,
                              workspace, workspace_bytes, stream, check=True):
    rc = _lib.tide_draft_train_step_dev(C.byref(cfg) if cfg is not None else None,
                                        C.byref(params) if params is not None else None,
                                        C.byref(grads) if grads is not None else None,
                                        C.byref(adam_state) if adam_state is not None else None,
                                        _ptr(hidden_buf), _ptr(tokens), _ptr(loss_mask), _ptr(lr_dev), _ptr(step_dev),
                                        _ptr(loss_out), _ptr(workspace), int(workspace_bytes), stream)
    return _check(rc) if check else rc


def tide_draft_train_step_tok(cfg, params, grads, adam_state, tok, hidden_buf, tokens, loss_mask, lr, loss_out,
                              workspace, workspace_bytes, stream, check=True):
    rc = _lib.tide_draft_train_step_tok(C.byref(cfg) if cfg is not None else None,
                                        C.byref(params) if params is not None else None,
                                        C.byref(grads) if grads is not None else None,
                                        C.byref(adam_state) if adam_state is not None else None,
                                        C.byref(tok) if tok is not None else None,
                                        _ptr(hidden_buf), _ptr(tokens), _ptr(loss_mask), float(lr), _ptr(loss_out),
                                        _ptr(workspace), int(workspace_bytes), stream)
    return _check(rc) if check else rc


def tide_draft_unroll_workspace_bytes(cfg: TideDraftConfig, n_steps: int) -> int:
    return int(_lib.tide_draft_unroll_workspace_bytes(C.byref(cfg), int(n_steps)))


def tide_draft_unroll_workspace_offset(cfg: TideDraftConfig, n_steps: int, step: int, name: str) -> int:
    return int(_lib.tide_draft_unroll_workspace_offset(C.byref(cfg), int(n_steps), int(step), name.encode()))


def tide_draft_eval_unroll(cfg, params, tok, hidden_buf, tokens, loss_mask, n_steps, loss_out, accuracy_out, workspace,
                           workspace_bytes, stream, check=True):
    rc = _lib.tide_draft_eval_unroll(C.byref(cfg) if cfg is not None else None,
                                     C.byref(params) if params is not None else None,
                                     C.byref(tok) if tok is not None else None,
                                     _ptr(hidden_buf), _ptr(tokens), _ptr(loss_mask), int(n_steps), _ptr(loss_out),
                                     _ptr(accuracy_out), _ptr(workspace), int(workspace_bytes), stream)
    return _check(rc) if check else rc


def tide_draft_train_step_unroll(cfg, params, grads, adam_state, tok, hidden_buf, tokens, loss_mask, n_steps, step_weights,
                                 lr, loss_out, workspace, workspace_bytes, stream, check=True):
    """step_weights: None or a host sequence of n_steps floats."""
    w = None if step_weights is None else (C.c_float * len(step_weights))(*[float(x) for x in step_weights])
    rc = _lib.tide_draft_train_step_unroll(C.byref(cfg) if cfg is not None else None,
                                           C.byref(params) if params is not None else None,
                                           C.byref(grads) if grads is not None else None,
                                           C.byref(adam_state) if adam_state is not None else None,
                                           C.byref(tok) if tok is not None else None,
                                           _ptr(hidden_buf), _ptr(tokens), _ptr(loss_mask), int(n_steps), w, float(lr),
                                           _ptr(loss_out), _ptr(workspace), int(workspace_bytes), stream)
    return _check(rc) if check else rc


def tide_draft_eval_unroll_packed(cfg, params, tok, hidden_buf, tokens, loss_mask, cu_seqlens, n_seqs, max_seqlen, n_steps,
                                  loss_out, accuracy_out, workspace, workspace_bytes, stream, check=True):
    rc = _lib.tide_draft_eval_unroll_packed(C.byref(cfg) if cfg is not None else None,
                                            C.byref(params) if params is not None else None,
                                            C.byref(tok) if tok is not None else None,
                                            _ptr(hidden_buf), _ptr(tokens), _ptr(loss_mask), _ptr(cu_seqlens), int(n_seqs),
                                            int(max_seqlen), int(n_steps), _ptr(loss_out), _ptr(accuracy_out),
                                            _ptr(workspace), int(workspace_bytes), stream)
    return _check(rc) if check else rc


def tide_draft_train_step_unroll_packed(cfg, params, grads, adam_state, tok, hidden_buf, tokens, loss_mask, cu_seqlens,
                                        n_seqs, max_seqlen, n_steps, step_weights, lr, loss_out, workspace,
                                        workspace_bytes, stream, check=True):
    w = None if step_weights is None else (C.c_float * len(step_weights))(*[float(x) for x in step_weights])
    rc = _lib.tide_draft_train_step_unroll_packed(C.byref(cfg) if cfg is not None else None,
                                                  C.byref(params) if params is not None else None,
                                                  C.byref(grads) if grads is not None else None,
                                                  C.byref(adam_state) if adam_state is not None else None,
                                                  C.byref(tok) if tok is not None else None,
                                                  _ptr(hidden_buf), _ptr(tokens), _ptr(loss_mask), _ptr(cu_seqlens),
                                                  int(n_seqs), int(max_seqlen), int(n_steps), w, float(lr),
                                                  _ptr(loss_out), _ptr(workspace), int(workspace_bytes), stream)
    return _check(rc) if check else rc


def tide_draft_workspace_bytes(cfg: TideDraftConfig) -> int:
    return int(_lib.tide_draft_workspace_bytes(C.byref(cfg)))


def tide_draft_workspace_offset(cfg: TideDraftConfig, name: str) -> int:
    return int(_lib.tide_draft_workspace_offset(C.byref(cfg), name.encode()))


def tide_draft_forward(cfg, params, hidden_buf, tokens, loss_mask, loss_out, top1_out, workspace,
                       workspace_bytes, stream, check=True):
    rc = _lib.tide_draft_forward(C.byref(cfg) if cfg is not None else None,
                                 C.byref(params) if params is not None else None,
                                 _ptr(hidden_buf), _ptr(tokens), _ptr(loss_mask), _ptr(loss_out),
                                 _ptr(top1_out), _ptr(workspace), int(workspace_bytes), stream)
    return _check(rc) if check else rc


def tide_draft_forward_packed(cfg, params, hidden_buf, tokens, loss_mask, cu_seqlens, n_seqs, max_seqlen, loss_out,
                              top1_out, workspace, workspace_bytes, stream, check=True):
    rc = _lib.tide_draft_forward_packed(C.byref(cfg) if cfg is not None else None,
                                        C.byref(params) if params is not None else None,
                                        _ptr(hidden_buf), _ptr(tokens), _ptr(loss_mask), _ptr(cu_seqlens),
                                        int(n_seqs), int(max_seqlen), _ptr(loss_out), _ptr(top1_out),
                                        _ptr(workspace), int(workspace_bytes), stream)
    return _check(rc) if check else rc


def tide_draft_train_step_packed(cfg, params, grads, adam_state, hidden_buf, tokens, loss_mask, cu_seqlens, n_seqs,
                                 max_seqlen, lr, loss_out, workspace, workspace_bytes, stream, check=True):
    rc = _lib.tide_draft_train_step_packed(C.byref(cfg) if cfg is not None else None,
                                           C.byref(params) if params is not None else None,
                                           C.byref(grads) if grads is not None else None,
                                           C.byref(adam_state) if adam_state is not None else None,
                                           _ptr(hidden_buf), _ptr(tokens), _ptr(loss_mask), _ptr(cu_seqlens),
                                           int(n_seqs), int(max_seqlen), float(lr), _ptr(loss_out),
                                           _ptr(workspace), int(workspace_bytes), stream)
    return _check(rc) if check else rc


def tide_draft_eval(cfg, params, hidden_buf, tokens, loss_mask, loss_out, accuracy_out, workspace,
                    workspace_bytes, stream, check=True):
    rc = _lib.tide_draft_eval(C.byref(cfg) if cfg is not None else None,
                              C.byref(params) if params is not None else None,
                              _ptr(hidden_buf), _ptr(tokens), _ptr(loss_mask), _ptr(loss_out),
                              _ptr(accuracy_out), _ptr(workspace), int(workspace_bytes), stream)
    return _check(rc) if check else rc


def tide_draft_train_step(cfg, params, grads, adam_state, hidden_buf, tokens, loss_mask, lr, loss_out,
                          workspace, workspace_bytes, stream, check=True):
    rc = _lib.tide_draft_train_step(C.byref(cfg) if cfg is not None else None,
                                    C.byref(params) if params is not None else None,
                                    C.byref(grads) if grads is not None else None,
                                    C.byref(adam_state) if adam_state is not None else None,
                                    _ptr(hidden_buf), _ptr(tokens), _ptr(loss_mask), float(lr),
                                    _ptr(loss_out), _ptr(workspace), int(workspace_bytes), stream)
    return _check(rc) if check else rc


def tide_gemm_workspace_bytes(layout, M, N, K, out_dtype):
    return int(_lib.tide_gemm_workspace_bytes(layout, M, N, K, out_dtype))


def tide_gemm(layout, M, N, K, alpha, A, B, Cmat, residual, in_dtype, out_dtype, accumulate, stream,
              check=True, workspace=None, workspace_bytes=0):
    rc = _lib.tide_gemm(layout, M, N, K, float(alpha), _ptr(A), _ptr(B), _ptr(Cmat), _ptr(residual),
                        in_dtype, out_dtype, int(accumulate), _ptr(workspace), int(workspace_bytes), stream)
    return _check(rc) if check else rc


def tide_rmsnorm_fwd(rows, d, x, g, eps, y, rstd, dtype, stream):
    return _check(_lib.tide_rmsnorm_fwd(rows, d, _ptr(x), _ptr(g), float(eps), _ptr(y), _ptr(rstd), dtype, stream))


def tide_rmsnorm_bwd_scratch_bytes(rows, d):
    return int(_lib.tide_rmsnorm_bwd_scratch_bytes(rows, d))


def tide_rmsnorm_bwd(rows, d, dy, x, g, rstd, residual_grad, dx, dg, dg_partial, dtype, stream):
    return _check(_lib.tide_rmsnorm_bwd(rows, d, _ptr(dy), _ptr(x), _ptr(g), _ptr(rstd), _ptr(residual_grad),
                                        _ptr(dx), _ptr(dg), _ptr(dg_partial), dtype, stream))


def tide_rmsnorm_bwd_static(rows, d, dy, x, g, rstd, residual_grad, dx, dg, dtype, stream, check=True):
    rc = _lib.tide_rmsnorm_bwd_static(rows, d, _ptr(dy), _ptr(x), _ptr(g), _ptr(rstd), _ptr(residual_grad),
                                      _ptr(dx), _ptr(dg), dtype, stream)
    return _check(rc) if check else rc


def tide_attention_fwd(B, S, nh, nkv, dh, qkv, out, lse, dtype, stream):
    return _check(_lib.tide_attention_fwd(B, S, nh, nkv, dh, _ptr(qkv), _ptr(out), _ptr(lse), dtype, stream))


def tide_attention_bwd(B, S, nh, nkv, dh, qkv, out, dout, lse, delta, dqkv, dtype, stream):
    return _check(_lib.tide_attention_bwd(B, S, nh, nkv, dh, _ptr(qkv), _ptr(out), _ptr(dout), _ptr(lse),
                                          _ptr(delta), _ptr(dqkv), dtype, stream))


def tide_rope(B, S, nh, nkv, dh, theta, qkv, table, inverse, dtype, stream):
    return _check(_lib.tide_rope(B, S, nh, nkv, dh, float(theta), _ptr(qkv), _ptr(table), int(inverse), dtype, stream))


def tide_ce_train(rows, vocab, z, ldz, tokens, mask, lse, loss_rows, dtype, stream, check=True):
    rc = _lib.tide_ce_train(int(rows), int(vocab), _ptr(z), int(ldz), _ptr(tokens), _ptr(mask), _ptr(lse), _ptr(loss_rows), dtype, stream)
    return _check(rc) if check else rc


def tide_profile_start():
    return _check(_lib.tide_profile_start())


def tide_profile_stop():
    """Returns the per-kernel records as a list of dicts."""
    import json
    buf = C.create_string_buffer(1 << 16)
    _check(_lib.tide_profile_stop(buf, len(buf)))
    return json.loads(buf.value.decode())


_lib.tide_mfma_probe.restype = _i32
_lib.tide_mfma_probe.argtypes = [_i32, _i32, _vp, C.POINTER(C.c_double), _vp]


def tide_mfma_probe(blocks, iters, sink, stream):
    """Enqueues the pure-MFMA probe; returns the flop count of the launch."""
    fl = C.c_double(0.0)
    _check(_lib.tide_mfma_probe(int(blocks), int(iters), _ptr(sink), C.byref(fl), stream))
    return float(fl.value)


# ---- signal ingest ring (include/tide_ingest.h) ----
TIDE_INGEST_ERR_NULL, TIDE_INGEST_ERR_ARG, TIDE_INGEST_ERR_HIP, TIDE_INGEST_ERR_BUSY = -1, -2, -4, -5
_lib.tide_ingest_create.restype = _i32
_lib.tide_ingest_create.argtypes = [C.POINTER(_vp), _sz, _i32]
_lib.tide_ingest_destroy.restype = _i32
_lib.tide_ingest_destroy.argtypes = [_vp]
_lib.tide_ingest_acquire.restype = _i32
_lib.tide_ingest_acquire.argtypes = [_vp, C.POINTER(C.c_int32), C.POINTER(_vp)]
_lib.tide_ingest_submit.restype = _i32
_lib.tide_ingest_submit.argtypes = [_vp, _i32, _vp, _sz, _vp, _i32]
_lib.tide_ingest_wait.restype = _i32
_lib.tide_ingest_wait.argtypes = [_vp, _i32, _vp]
_lib.tide_ingest_done.restype = _i32
_lib.tide_ingest_done.argtypes = [_vp, _i32]
_lib.tide_ingest_last_error.restype = C.c_char_p
_lib.tide_ingest_last_error.argtypes = []


def tide_ingest_create(slot_bytes, n_slots):
    """Returns (rc, handle)."""
    h = _vp()
    rc = _lib.tide_ingest_create(C.byref(h), int(slot_bytes), int(n_slots))
    return rc, h


def tide_ingest_destroy(h):
    return _lib.tide_ingest_destroy(h)


def tide_ingest_acquire(h):
    """Returns (rc, slot, host address)."""
    slot, ptr = C.c_int32(-1), _vp()
    rc = _lib.tide_ingest_acquire(h, C.byref(slot), C.byref(ptr))
    return rc, int(slot.value), ptr.value


def tide_ingest_submit(h, slot, device_dst, nbytes, reader_stream=None, after_reader=False):
    return _lib.tide_ingest_submit(h, int(slot), _ptr(device_dst), int(nbytes), reader_stream, int(bool(after_reader)))


def tide_ingest_wait(h, slot, stream):
    return _lib.tide_ingest_wait(h, int(slot), stream)


def tide_ingest_done(h, slot):
    return _lib.tide_ingest_done(h, int(slot))


def tide_ingest_last_error() -> str:
    return _lib.tide_ingest_last_error().decode()
