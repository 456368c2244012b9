"""ctypes binding of libnmt.so: one Python function per C entry point, same names, argument
marshalling only.  Device buffers are torch tensors (their data_ptr() is passed through); the HIP
stream is torch's current stream unless one is given.  The library must have been built
(`python -m paper_1806_00187_amd.build`); there is no fallback of any kind."""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libnmt.so")

NMT_OK, NMT_EINVAL, NMT_ESTATE, NMT_ENOMEM, NMT_EHIP = 0, -1, -2, -3, -4


class NmtError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"libnmt error {code}: {msg}")
        self.code = code


class nmt_config(C.Structure):
    _fields_ = [("enc_layers", C.c_int32), ("dec_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32),
                ("d_ff", C.c_int32), ("vocab", C.c_int32), ("pad_id", C.c_int32), ("dropout", C.c_float),
                ("attn_dropout", C.c_float), ("act_dropout", C.c_float), ("label_smoothing", C.c_float), ("ln_eps", C.c_float), ("seed", C.c_uint64),
                ("max_sentences", C.c_int32), ("max_len", C.c_int32)]


class nmt_dropout(C.Structure):
    _fields_ = [("p", C.c_float), ("site", C.c_uint32), ("step", C.c_uint32), ("micro", C.c_uint32), ("seed", C.c_uint64),
                ("n_pos", C.c_int32), ("d_sent_uid", C.c_void_p)]


class nmt_segment(C.Structure):
    _fields_ = [("B", C.c_int32), ("S", C.c_int32), ("T", C.c_int32), ("micro_idx", C.c_uint32)]


_P, _I32, _I64, _F, _U32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float, C.c_uint32
_DP = C.POINTER(nmt_dropout)
_SP = C.POINTER(nmt_segment)

_SIGNATURES = {
    "nmt_last_error": (C.c_char_p, []),
    "nmt_create": (C.c_int, [C.POINTER(nmt_config), C.POINTER(_P)]),
    "nmt_destroy": (None, [_P]),
    "nmt_param_count": (_I64, [_P]),
    "nmt_param_tensors": (_I32, [_P]),
    "nmt_grad_scale": (C.c_float, [_P]),
    "nmt_param_info": (C.c_int, [_P, _I32, C.POINTER(C.c_char_p), C.POINTER(_I64), C.POINTER(_I32), C.POINTER(_I32)]),
    "nmt_workspace_bytes": (_I64, [_P, _I32, _I32, _I32]),
    "nmt_workspace_bytes_group": (_I64, [_P, _I32, _SP]),
    "nmt_bind": (C.c_int, [_P, _P, _P, _P, _P, _P, _P, _P, _I64]),
    "nmt_forward_loss": (C.c_int, [_P, _P, _P, _P, _I32, _I32, _I32, _F, _U32, _U32, _P, _I32, _P, _P, _P]),
    "nmt_forward_loss_group": (C.c_int, [_P, _I32, _SP, _P, _P, _P, _F, _U32, _P, _I32, _P, _P, _P]),
    "nmt_workspace_bytes_packed": (_I64, [_P, _I32, _I64, _I64]),
    "nmt_forward_loss_packed": (C.c_int, [_P, _I32, _P, _I64, _I64, _I32, _I32, _P, _P, _P, _F, _U32, _I32, _P, _P, _P]),
    "nmt_backward": (C.c_int, [_P, _P]),
    "nmt_accumulate": (C.c_int, [_P, _I32, _P]),
    "nmt_accumulate_loss": (C.c_int, [_P, _I32, _P, _P, _P]),
    "nmt_tuning": (C.c_int, [C.c_char_p, _I32]),
    "nmt_gemm_timing": (C.c_int, [C.POINTER(C.c_double), C.POINTER(_I64), C.POINTER(C.c_double)]),
    "nmt_debug_activation": (C.c_int, [_P, C.c_char_p, C.POINTER(_P), C.POINTER(_I64), C.POINTER(_I64)]),
    "nmt_check_overflow": (C.c_int, [_P, _F, _P, _P]),
    "nmt_adam_step": (C.c_int, [_P, _F, _F, _F, _F, _I32, _P, _P]),
    "nmt_scaler_update": (C.c_int, [C.POINTER(C.c_float), C.POINTER(_I32), _I32, _I32]),
    "nmt_lr_schedule": (C.c_double, [_I64, C.c_double, _I64]),
    "nmt_op_gemm": (C.c_int, [_P, _I32, _I32, _P, _I32, _I32, _P, _I32, _I32, _I32, _I32, _P, _I32, _DP, _P, _P, _F, _P]),
    "nmt_op_gemm_f32": (C.c_int, [_P, _I32, _I32, _P, _I32, _I32, _P, _I32, _I32, _I32, _I32, _I32, _P]),
    "nmt_op_gemm_splitk": (C.c_int, [_P, _I32, _I32, _P, _I32, _I32, _P, _I32, _I32, _I32, _I32, _P, _I64, _I32, _P]),
    "nmt_op_attention_fwd": (C.c_int, [_P, _I32, _P, _I32, _P, _I32, _P, _I32, _P, _P, _I32, _I32, _I32, _I32, _I32, _I32, _I32, _P]),
    "nmt_op_attention_bwd": (C.c_int, [_P, _I32, _P, _I32, _P, _I32, _P, _I32, _P, _I32, _P, _P, _I32, _P, _I32, _P, _I32, _P,
                                       _I32, _I32, _I32, _I32, _I32, _I32, _I32, _P]),
    "nmt_op_residual_layernorm_fwd": (C.c_int, [_P, _P, _P, _P, _P, _P, _I32, _I32, _F, _DP, _P]),
    "nmt_op_layernorm_bwd_scratch": (_I64, [_I32]),
    "nmt_op_residual_layernorm_bwd": (C.c_int, [_P, _P, _P, _P, _P, _P, _P, _P, _P, _P, _P, _I32, _I32, _DP, _P]),
    "nmt_op_embed_fwd": (C.c_int, [_P, _P, _P, _I32, _I32, _I32, _DP, _P]),
    "nmt_op_softmax_xent": (C.c_int, [_P, _P, _P, _I32, _I32, _I32, _F, _F, _P, _P, _P]),
    "nmt_op_colsum_scratch": (_I64, [_I32]),
    "nmt_op_colsum": (C.c_int, [_P, _I32, _P, _P, _I32, _I32, _P]),
    "nmt_op_colsum_static": (C.c_int, [_P, _I32, _P, _I32, _I32, _P]),
    "nmt_op_embed_bwd_scratch": (_I64, [_I32, _I32, _I32]),
    "nmt_op_embed_bwd": (C.c_int, [_P, _P, _I32, _DP, _P, _P, _I32, _DP, _P, _I32, _I32, _P, _P]),
    "nmt_op_accumulate": (C.c_int, [_P, _P, _I64, _I32, _P]),
    "nmt_op_check_overflow": (C.c_int, [_P, _I64, _F, _P, _P]),
    "nmt_op_adam": (C.c_int, [_P, _P, _P, _P, _F, _P, _I64, _F, _F, _F, _F, _I32, _P, _P]),
    "nmt_op_dropout_mask": (C.c_int, [_P, _I32, _I32, _DP, _P]),
}

_lib = None


def load():
    """Loads libnmt.so and declares every entry point; raises if the library has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_1806_00187_amd.build`")
        # torch first: the library then binds to the HIP runtime torch has already loaded, the one that owns
        # the tensors' memory and streams (loaded the other way round, the process ends up with two runtimes
        # and the library's own sees no device)
        import torch  # noqa: F401
        lib = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib


def exported_symbols():
    return sorted(_SIGNATURES)


def _check(rc):
    if rc != NMT_OK:
        raise NmtError(rc, load().nmt_last_error().decode())


def _p(t):
    """Device (or host) address of a torch tensor, or NULL."""
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is not None:
        return C.c_void_p(stream)
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _drop(drop):
    """drop: None or dict(p, site, step, micro, seed, n_pos, sent_uid=tensor|None)."""
    if drop is None:
        return None
    uid = drop.get("sent_uid")
    return C.byref(nmt_dropout(drop.get("p", 0.0), drop.get("site", 0), drop.get("step", 0), drop.get("micro", 0),
                               drop.get("seed", 0), drop["n_pos"], None if uid is None else uid.data_ptr()))


# ---- context ------------------------------------------------------------------------------------
def nmt_create(**cfg):
    c = nmt_config(**cfg)
    out = C.c_void_p()
    _check(load().nmt_create(C.byref(c), C.byref(out)))
    return out


def nmt_destroy(ctx):
    load().nmt_destroy(ctx)


def nmt_param_count(ctx):
    return load().nmt_param_count(ctx)


def nmt_grad_scale(ctx):
    return load().nmt_grad_scale(ctx)


def nmt_param_tensors(ctx):
    return load().nmt_param_tensors(ctx)


def nmt_param_info(ctx, idx):
    name, off, rows, cols = C.c_char_p(), C.c_int64(), C.c_int32(), C.c_int32()
    _check(load().nmt_param_info(ctx, idx, C.byref(name), C.byref(off), C.byref(rows), C.byref(cols)))
    return name.value.decode(), off.value, rows.value, cols.value


def nmt_workspace_bytes(ctx, B, S, T):
    n = load().nmt_workspace_bytes(ctx, B, S, T)
    if n < 0:
        _check(int(n))
    return n


def _segments(segs):
    """segs: sequence of (B, S, T, micro_idx)."""
    arr = (nmt_segment * len(segs))()
    for i, (B, S, T, micro) in enumerate(segs):
        arr[i] = nmt_segment(B, S, T, micro)
    return arr


def nmt_workspace_bytes_group(ctx, segs):
    n = load().nmt_workspace_bytes_group(ctx, len(segs), _segments(segs))
    if n < 0:
        _check(int(n))
    return n


def nmt_bind(ctx, w16, g16, master32=None, acc32=None, adam_m=None, adam_v=None, workspace=None):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().nmt_bind(ctx, _p(w16), _p(g16), _p(master32), _p(acc32), _p(adam_m), _p(adam_v), _p(workspace), ws_bytes))


# ---- the training step --------------------------------------------------------------------------
def nmt_forward_loss(ctx, src, tgt_in, tgt_out, loss_scale, step, micro_idx, loss_sum, ntok, sent_uid=None, training=True,
                     stream=None):
    B, S = src.shape
    T = tgt_in.shape[1]
    _check(load().nmt_forward_loss(ctx, _p(src), _p(tgt_in), _p(tgt_out), B, S, T, loss_scale, step, micro_idx, _p(sent_uid),
                                   1 if training else 0, _p(loss_sum), _p(ntok), _stream(stream)))


def nmt_forward_loss_group(ctx, segs, src, tgt_in, tgt_out, loss_scale, step, loss_sum, ntok, sent_uid=None, training=True,
                           stream=None):
    """segs: sequence of (B, S, T, micro_idx); src / tgt_in / tgt_out: flat int32 tensors holding the sub-batches one after
    another; sent_uid: one uint32 per sentence in the same order, or None."""
    _check(load().nmt_forward_loss_group(ctx, len(segs), _segments(segs), _p(src), _p(tgt_in), _p(tgt_out), loss_scale, step,
                                         _p(sent_uid), 1 if training else 0, _p(loss_sum), _p(ntok), _stream(stream)))


def nmt_workspace_bytes_packed(ctx, n_sent, n_src_tokens, n_tgt_tokens):
    n = load().nmt_workspace_bytes_packed(ctx, n_sent, n_src_tokens, n_tgt_tokens)
    if n < 0:
        _check(int(n))
    return n


def nmt_forward_loss_packed(ctx, sentences, n_src_tokens, n_tgt_tokens, max_src_len, max_tgt_len, src, tgt_in, tgt_out, loss_scale,
                            step, loss_sum, ntok, training=True, stream=None):
    """sentences: int32 device tensor [n_sent, 4] = (src_len, tgt_len, uid, micro_idx) per sentence; src / tgt_in / tgt_out: flat
    int32 device tensors of n_src_tokens / n_tgt_tokens ids, sentences back to back."""
    _check(load().nmt_forward_loss_packed(ctx, sentences.shape[0], _p(sentences), n_src_tokens, n_tgt_tokens, max_src_len, max_tgt_len,
                                          _p(src), _p(tgt_in), _p(tgt_out), loss_scale, step, 1 if training else 0, _p(loss_sum),
                                          _p(ntok), _stream(stream)))


def nmt_backward(ctx, stream=None):
    _check(load().nmt_backward(ctx, _stream(stream)))


def nmt_accumulate(ctx, first, stream=None):
    _check(load().nmt_accumulate(ctx, 1 if first else 0, _stream(stream)))


def nmt_accumulate_loss(ctx, first, loss_total, ntok_total, stream=None):
    _check(load().nmt_accumulate_loss(ctx, 1 if first else 0, _p(loss_total), _p(ntok_total), _stream(stream)))


def nmt_debug_activation(ctx, name):
    """(device address, rows, cols) of a saved fp16 activation of the last forward pass."""
    ptr, rows, cols = C.c_void_p(), C.c_int64(), C.c_int64()
    _check(load().nmt_debug_activation(ctx, name.encode(), C.byref(ptr), C.byref(rows), C.byref(cols)))
    return ptr.value, rows.value, cols.value


def nmt_gemm_timing():
    """(milliseconds, products, algorithmic FLOPs) of the GEMM products launched since the last call with "gemm_timing" on."""
    ms, n, fl = C.c_double(), C.c_int64(), C.c_double()
    _check(load().nmt_gemm_timing(C.byref(ms), C.byref(n), C.byref(fl)))
    return ms.value, n.value, fl.value


_TUNING_SET = {}   # what this process has set through nmt_tuning (the library has no call that reads a switch back)


def nmt_tuning(name, value=0):
    _check(load().nmt_tuning(name.encode(), int(value)))
    if name == "defaults":
        _TUNING_SET.clear()
    else:
        _TUNING_SET[name] = int(value)


def tuning_value(name, default):
    """The value last set for a launch-form switch through nmt_tuning, or `default` (the library's) if none was."""
    return _TUNING_SET.get(name, default)


def nmt_check_overflow(ctx, inv_scale, flag, stream=None):
    _check(load().nmt_check_overflow(ctx, inv_scale, _p(flag), _stream(stream)))


def nmt_adam_step(ctx, lr, beta1, beta2, eps, t, flag, stream=None):
    _check(load().nmt_adam_step(ctx, lr, beta1, beta2, eps, t, _p(flag), _stream(stream)))


def nmt_scaler_update(scale, clean, overflow, window=2000):
    s, c = C.c_float(scale), C.c_int32(clean)
    _check(load().nmt_scaler_update(C.byref(s), C.byref(c), 1 if overflow else 0, window))
    return s.value, c.value


def nmt_lr_schedule(t, peak, warmup=4000):
    return load().nmt_lr_schedule(t, peak, warmup)


# ---- kernel-level entry points -------------------------------------------------------------------
def nmt_op_gemm(A, a_t, lda, B, b_t, ldb, Cout, ldc, M, N, K, bias=None, relu=False, drop=None, add=None, relu_src=None,
                mask_scale=1.0, stream=None):
    _check(load().nmt_op_gemm(_p(A), int(a_t), lda, _p(B), int(b_t), ldb, _p(Cout), ldc, M, N, K, _p(bias), int(relu), _drop(drop),
                              _p(add), _p(relu_src), mask_scale, _stream(stream)))


def nmt_op_gemm_f32(A, a_t, lda, B, b_t, ldb, Cout, ldc, M, N, K, splits=1, stream=None):
    _check(load().nmt_op_gemm_f32(_p(A), int(a_t), lda, _p(B), int(b_t), ldb, _p(Cout), ldc, M, N, K, splits, _stream(stream)))


def nmt_op_gemm_splitk(A, a_t, lda, B, b_t, ldb, Cout, ldc, M, N, K, partial, splits=0, stream=None):
    _check(load().nmt_op_gemm_splitk(_p(A), int(a_t), lda, _p(B), int(b_t), ldb, _p(Cout), ldc, M, N, K, _p(partial), partial.numel(),
                                     splits, _stream(stream)))


def nmt_op_attention_fwd(Q, ldq, K, ldk, V, ldv, O, ldo, lse, key_ids, pad_id, causal, B, H, dh, Tq, Tk, stream=None):
    _check(load().nmt_op_attention_fwd(_p(Q), ldq, _p(K), ldk, _p(V), ldv, _p(O), ldo, _p(lse), _p(key_ids), pad_id, int(causal),
                                       B, H, dh, Tq, Tk, _stream(stream)))


def nmt_op_attention_bwd(Q, ldq, K, ldk, V, ldv, O, ldo, dO, lddo, lse, dQ, lddq, dK, lddk, dV, lddv, key_ids, pad_id, causal, B, H,
                         dh, Tq, Tk, stream=None):
    _check(load().nmt_op_attention_bwd(_p(Q), ldq, _p(K), ldk, _p(V), ldv, _p(O), ldo, _p(dO), lddo, _p(lse), _p(dQ), lddq, _p(dK),
                                       lddk, _p(dV), lddv, _p(key_ids), pad_id, int(causal), B, H, dh, Tq, Tk, _stream(stream)))


def nmt_op_residual_layernorm_fwd(sub, resid, gamma, beta, out, stats, rows, d, eps, drop=None, stream=None):
    _check(load().nmt_op_residual_layernorm_fwd(_p(sub), _p(resid), _p(gamma), _p(beta), _p(out), _p(stats), rows, d, eps, _drop(drop),
                                                _stream(stream)))


def nmt_op_layernorm_bwd_scratch(d):
    return load().nmt_op_layernorm_bwd_scratch(d)


def nmt_op_residual_layernorm_bwd(dout, sub, resid, gamma, stats, dy, dym, dgamma, dbeta, dbias, partial, rows, d, drop=None,
                                  stream=None):
    _check(load().nmt_op_residual_layernorm_bwd(_p(dout), _p(sub), _p(resid), _p(gamma), _p(stats), _p(dy), _p(dym), _p(dgamma),
                                                _p(dbeta), _p(dbias), _p(partial), rows, d, _drop(drop), _stream(stream)))


def nmt_op_embed_fwd(ids, E, x, rows, d, vocab, drop, stream=None):
    _check(load().nmt_op_embed_fwd(_p(ids), _p(E), _p(x), rows, d, vocab, _drop(drop), _stream(stream)))


def nmt_op_softmax_xent(logits, targets, row_loss, rows, V, pad_id, label_smoothing, loss_scale, loss_sum, ntok, stream=None):
    _check(load().nmt_op_softmax_xent(_p(logits), _p(targets), _p(row_loss), rows, V, pad_id, label_smoothing, loss_scale,
                                      _p(loss_sum), _p(ntok), _stream(stream)))


def nmt_op_colsum_scratch(cols):
    return load().nmt_op_colsum_scratch(cols)


def nmt_op_colsum(src, ld, dst, partial, rows, cols, stream=None):
    _check(load().nmt_op_colsum(_p(src), ld, _p(dst), _p(partial), rows, cols, _stream(stream)))


def nmt_op_colsum_static(src, ld, dst, rows, cols, stream=None):
    _check(load().nmt_op_colsum_static(_p(src), ld, _p(dst), rows, cols, _stream(stream)))


def nmt_op_embed_bwd_scratch(vocab, rows_total, d):
    return load().nmt_op_embed_bwd_scratch(vocab, rows_total, d)


def nmt_op_embed_bwd(ids_a, dx_a, rows_a, drop_a, ids_b, dx_b, rows_b, drop_b, gE, d, vocab, scratch, stream=None):
    _check(load().nmt_op_embed_bwd(_p(ids_a), _p(dx_a), rows_a, _drop(drop_a), _p(ids_b), _p(dx_b), rows_b, _drop(drop_b), _p(gE), d,
                                   vocab, _p(scratch), _stream(stream)))


def nmt_op_accumulate(g16, acc32, n, first, stream=None):
    _check(load().nmt_op_accumulate(_p(g16), _p(acc32), n, 1 if first else 0, _stream(stream)))


def nmt_op_check_overflow(acc32, n, inv_scale, flag, stream=None):
    _check(load().nmt_op_check_overflow(_p(acc32), n, inv_scale, _p(flag), _stream(stream)))


def nmt_op_adam(master32, m, v, g32, w16, n, lr, beta1, beta2, eps, t, flag, grad_scale=1.0, stream=None):
    _check(load().nmt_op_adam(_p(master32), _p(m), _p(v), _p(g32), grad_scale, _p(w16), n, lr, beta1, beta2, eps, t, _p(flag),
                              _stream(stream)))


def nmt_op_dropout_mask(keep, rows, n_cols, drop, stream=None):
    _check(load().nmt_op_dropout_mask(_p(keep), rows, n_cols, _drop(drop), _stream(stream)))
