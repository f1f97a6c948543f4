"""Thin ctypes binding of libtemplora.so: argument marshalling only.

Every function has the name of the C entry point it calls (include/templora.h)
and passes device pointers of torch tensors straight through; no step of the
chunk update is computed in Python.  torch is used for device memory and the
HIP stream handle, nothing else.  If the shared library has not been built the
import of this module fails loudly: there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtemplora.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python -m paper_2401_11504_amd.build` "
        "(the Temp-Lora path has no CPU or PyTorch fallback)")
_lib = C.CDLL(LIB_PATH)

TL_OK = 0
STATUS = {0: "TL_OK", -1: "TL_ERR_ARG", -2: "TL_ERR_SHAPE", -3: "TL_ERR_TOKEN_RANGE", -4: "TL_ERR_WINDOW",
          -5: "TL_ERR_NONFINITE", -6: "TL_ERR_DEVICE", -7: "TL_ERR_DISCARDED", -8: "TL_ERR_OOM"}
(FACTOR_A, FACTOR_B, GRAD_A, GRAD_B, M_A, M_B, V_A, V_B) = range(8)
PROJ = ("q", "k", "v", "o", "gate", "up", "down")


class TlError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"{STATUS.get(status, status)}: {msg}")
        self.status = status


class tl_model_cfg(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32), ("d_head", C.c_int32),
                ("d_ffn", C.c_int32), ("vocab", C.c_int32), ("max_tokens", C.c_int32), ("rms_eps", C.c_float),
                ("rope_base", C.c_float)]


class tl_lora_cfg(C.Structure):
    _fields_ = [("rank", C.c_int32), ("alpha", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float),
                ("eps", C.c_float), ("weight_decay", C.c_float), ("a_init_std", C.c_float), ("seed", C.c_uint64),
                ("dropout", C.c_float)]


class tl_train_cfg(C.Structure):
    _fields_ = [("n_ctx_max", C.c_int32), ("batch", C.c_int32), ("epochs", C.c_int32), ("warmup_steps", C.c_int32),
                ("lr", C.c_float)]


class tl_generate_cfg(C.Structure):
    _fields_ = [("window", C.c_int32), ("chunk", C.c_int32), ("train", tl_train_cfg)]


_vp, _i32, _i64, _f32, _sz = C.c_void_p, C.c_int32, C.c_int64, C.c_float, C.c_size_t
_SIGS = {
    "tl_model_create": [C.POINTER(tl_model_cfg), C.POINTER(_vp), _vp, C.POINTER(_vp)],
    "tl_model_destroy": [_vp],
    "tl_lora_init": [_vp, C.POINTER(tl_lora_cfg), C.POINTER(_vp)],
    "tl_chunk_update": [_vp, _vp, _i32, _i32, _f32, C.POINTER(_f32), C.POINTER(_i32)],
    "tl_chunk_loss": [_vp, _vp, _i32, _i32, C.POINTER(_f32), C.POINTER(_i32)],
    "tl_chunk_train": [_vp, _vp, _i32, _i32, C.POINTER(tl_train_cfg), _vp, C.POINTER(_i32)],
    "tl_prefill": [_vp, _vp, _i32, C.POINTER(_i32), _vp],
    "tl_decode_step": [_vp, _i32, C.POINTER(_i32), _vp],
    "tl_kv_length": [_vp, C.POINTER(_i32)],
    "tl_generate": [_vp, _vp, _i32, _i32, C.POINTER(tl_generate_cfg), _vp, _vp, C.POINTER(_i32)],
    "tl_cache_reuse": [_vp, _i32],
    "tl_discard": [_vp],
    "tl_lora_free": [_vp],
    "tl_get_factor": [_vp, _i32, _i32, _i32, _vp, _sz],
    "tl_set_factor": [_vp, _i32, _i32, _i32, _vp, _sz],
    "tl_get_step": [_vp, C.POINTER(_i64)],
    "tl_get_nll": [_vp, _vp, _sz],
    "tl_get_dh": [_vp, _i32, _vp, _sz],
    "tl_keep_input_grad": [_vp, _i32],
    "tl_profile_enable": [_vp, _i32],
    "tl_profile_read": [_vp, C.POINTER(C.c_double), C.POINTER(_i64), C.POINTER(C.c_double)],
    "tl_layer_step": [_vp, _i32, _vp, _vp, _i32, _vp, _vp, _f32, _i32],
    "tl_linear_step": [_vp] * 5 + [_i32] * 4 + [_f32] * 6 + [_i32] + [_vp] * 6 + [_vp],
    "tl_linear_step_static": [_vp] * 5 + [_i32] * 4 + [_f32] * 6 + [_i32] + [_vp] * 6 + [_vp],
    "tl_k_gemm_nt": [_vp, _i32, _vp, _i32, _i32, _i32, _i32, _vp, _i32, _vp, _i32, _i32, _f32, _vp, _vp, _i32, _i32, _vp,
                     _sz, _vp],
    "tl_k_gemm_nt_plan": [_i32, _i32, _i32, _i32, _sz, C.c_char_p, _sz, C.POINTER(_i32), C.POINTER(_i32)],
    "tl_k_gemm_tn": [_vp, _i32, _vp, _i32, _i32, _i32, _i32, _f32, _vp, _i32, _vp],
    "tl_k_rmsnorm_fwd": [_vp, _vp, _i32, _i32, _f32, _vp, _vp],
    "tl_k_rmsnorm_bwd": [_vp, _vp, _vp, _vp, _i32, _i32, _f32, _vp, _vp, _vp],
    "tl_k_rope": [_vp, _i32, _i32, _i32, _i32, _f32, _i32, _i32, _vp],
    "tl_k_rope_table": [_vp, _i32, _i32, _i32, _i32, _f32, _i32, _i32, _vp, _sz, _vp],
    "tl_k_dropout": [_vp, _i32, _i32, _f32, C.c_uint64, _i64, _i32, _i32, _vp, _vp],
    "tl_k_swiglu_fwd": [_vp, _i32, _i32, _vp, _vp],
    "tl_k_swiglu_bwd": [_vp, _vp, _i32, _i32, _vp, _vp],
    "tl_k_gemv": [_vp, _i32, _vp, _i32, _i32, _vp, _vp, _i32, _i32, _f32, _vp, _vp, _i32, _vp],
    "tl_k_gemv_pre": [_vp, _i32, _i32, _i32, _i32, _vp, _vp, _f32, _vp, _vp, _vp, _vp],
    "tl_k_attention_decode": [_vp, _vp, _vp, _i32, _i32, _i32, _i32, _vp, _vp, _sz, _vp],
    "tl_k_argmax": [_vp, _i32, _vp, _vp],
    "tl_k_attention_fwd": [_vp, _vp, _vp, _i32, _i32, _i32, _i32, _vp, _i32, _vp, _vp],
    "tl_k_attention_bwd": [_vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _vp],
    "tl_k_cross_entropy": [_vp, _vp, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp],
    "tl_k_adamw": [_vp, _vp, _vp, _vp, _vp, _sz, _i64, _f32, _f32, _f32, _f32, _f32, _vp],
    "tl_k_embed": [_vp, _vp, _i32, _i32, _vp, _vp],
}
EXPORTS = tuple(_SIGS) + ("tl_warmup_lr", "tl_last_error", "tl_version")
for _n, _a in _SIGS.items():
    _f = getattr(_lib, _n)
    _f.argtypes = _a
    _f.restype = C.c_int
_lib.tl_warmup_lr.argtypes = [_f32, _i64, _i32]
_lib.tl_warmup_lr.restype = _f32
_lib.tl_last_error.restype = C.c_char_p
_lib.tl_version.restype = C.c_char_p


def tl_last_error() -> str:
    return _lib.tl_last_error().decode()


def tl_version() -> str:
    return _lib.tl_version().decode()


def _chk(status: int):
    if status != TL_OK:
        raise TlError(status, tl_last_error())


def _dp(t):
    """device pointer of a torch tensor (None -> NULL)"""
    if t is None:
        return None
    assert t.is_cuda and (t.dim() == 0 or t.stride(-1) == 1), "device tensor with unit inner stride expected"
    return C.c_void_p(t.data_ptr())


def current_stream_handle():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


# ------------------------------------------------------------------ life cycle
def tl_model_create(n_layers, d_model, n_heads, d_head, d_ffn, vocab, max_tokens, weight_tensors, rms_eps=1e-5,
                    rope_base=10000.0, stream=None):
    """weight_tensors: flat list in the order of the header (9 per layer, then embedding, final gain, lm_head;
    entries may be None where the header allows).  Returns an opaque model handle."""
    cfg = tl_model_cfg(n_layers, d_model, n_heads, d_head, d_ffn, vocab, max_tokens, rms_eps, rope_base)
    n = 9 * n_layers + 3
    assert len(weight_tensors) == n
    arr = (_vp * n)(*[(t.data_ptr() if t is not None else None) for t in weight_tensors])
    out = _vp()
    _chk(_lib.tl_model_create(C.byref(cfg), arr, stream if stream is not None else current_stream_handle(),
                              C.byref(out)))
    return out


def tl_model_destroy(model):
    _chk(_lib.tl_model_destroy(model))


def tl_lora_init(model, rank, alpha, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, a_init_std=0.02, seed=0,
                 dropout=0.0):
    cfg = tl_lora_cfg(rank, alpha, beta1, beta2, eps, weight_decay, a_init_std, seed, dropout)
    out = _vp()
    _chk(_lib.tl_lora_init(model, C.byref(cfg), C.byref(out)))
    return out


def _tok(tokens):
    a = np.ascontiguousarray(np.asarray(tokens), dtype=np.int32)
    return a, a.ctypes.data_as(_vp)


def tl_chunk_update(lora, tokens, n_ctx=0, lr=5e-5):
    """-> (loss, n_targets)"""
    a, p = _tok(tokens)
    loss, n = _f32(), _i32()
    _chk(_lib.tl_chunk_update(lora, p, a.size, n_ctx, lr, C.byref(loss), C.byref(n)))
    return loss.value, n.value


def tl_chunk_loss(lora, tokens, n_ctx=0):
    a, p = _tok(tokens)
    loss, n = _f32(), _i32()
    _chk(_lib.tl_chunk_loss(lora, p, a.size, n_ctx, C.byref(loss), C.byref(n)))
    return loss.value, n.value


def tl_chunk_train(lora, tokens, n_chunk, n_ctx_max=1024, batch=0, epochs=2, lr=5e-5, warmup_steps=0):
    """-> list of per-step losses (epochs * ceil(n_chunk / batch) of them)"""
    a, p = _tok(tokens)
    cfg = tl_train_cfg(n_ctx_max, batch, epochs, warmup_steps, lr)
    b = batch if 0 < batch < n_chunk else max(n_chunk, 1)
    losses = np.zeros(max(epochs, 1) * (-(-max(n_chunk, 1) // b)), dtype=np.float32)
    n = _i32()
    _chk(_lib.tl_chunk_train(lora, p, a.size, n_chunk, C.byref(cfg), losses.ctypes.data_as(_vp), C.byref(n)))
    return [float(x) for x in losses[:n.value]]


def tl_warmup_lr(lr, step, warmup_steps):
    return float(_lib.tl_warmup_lr(lr, step, warmup_steps))


def tl_prefill(lora, tokens, vocab=0):
    """-> (next_token, logits fp32[vocab] or None)"""
    a, p = _tok(tokens)
    nxt = _i32()
    logits = np.empty(vocab, np.float32) if vocab else None
    _chk(_lib.tl_prefill(lora, p, a.size, C.byref(nxt), logits.ctypes.data if vocab else None))
    return nxt.value, logits


def tl_decode_step(lora, token, vocab=0):
    """-> (next_token, logits fp32[vocab] or None)"""
    nxt = _i32()
    logits = np.empty(vocab, np.float32) if vocab else None
    _chk(_lib.tl_decode_step(lora, int(token), C.byref(nxt), logits.ctypes.data if vocab else None))
    return nxt.value, logits


def tl_generate(lora, prompt, n_new, window, chunk, n_ctx_max=1024, batch=0, epochs=2, lr=5e-5, warmup_steps=0):
    """-> (generated tokens int32[n_new], per-step training losses)"""
    a, p = _tok(prompt)
    cfg = tl_generate_cfg(window, chunk, tl_train_cfg(n_ctx_max, batch, epochs, warmup_steps, lr))
    out = np.zeros(max(n_new, 1), np.int32)
    b = batch if 0 < batch < chunk else max(chunk, 1)
    losses = np.zeros(max(1, (n_new // max(chunk, 1)) * max(epochs, 1) * (-(-max(chunk, 1) // b))), np.float32)
    n = _i32()
    _chk(_lib.tl_generate(lora, p, a.size, n_new, C.byref(cfg), out.ctypes.data_as(_vp), losses.ctypes.data_as(_vp),
                          C.byref(n)))
    return out[:n_new], [float(x) for x in losses[:n.value]]


def tl_cache_reuse(lora, on=True):
    _chk(_lib.tl_cache_reuse(lora, int(on)))


def tl_kv_length(lora):
    n = _i32()
    _chk(_lib.tl_kv_length(lora, C.byref(n)))
    return n.value


def tl_discard(lora):
    _chk(_lib.tl_discard(lora))


def tl_lora_free(lora):
    _chk(_lib.tl_lora_free(lora))


# ------------------------------------------------------------------ inspection
def tl_get_factor(lora, layer, proj, which, shape):
    out = np.empty(shape, dtype=np.float32)
    _chk(_lib.tl_get_factor(lora, layer, proj, which, out.ctypes.data_as(_vp), out.size))
    return out


def tl_set_factor(lora, layer, proj, which, values):
    a = np.ascontiguousarray(values, dtype=np.float32)
    _chk(_lib.tl_set_factor(lora, layer, proj, which, a.ctypes.data_as(_vp), a.size))


def tl_get_step(lora) -> int:
    s = _i64()
    _chk(_lib.tl_get_step(lora, C.byref(s)))
    return s.value


def tl_get_nll(lora, n_tokens):
    out = np.empty(n_tokens, dtype=np.float32)
    _chk(_lib.tl_get_nll(lora, out.ctypes.data_as(_vp), out.size))
    return out


def tl_get_dh(lora, boundary, n_tokens, d_model):
    out = np.empty((n_tokens, d_model), dtype=np.float32)
    _chk(_lib.tl_get_dh(lora, boundary, out.ctypes.data_as(_vp), out.size))
    return out


def tl_keep_input_grad(lora, on=True):
    _chk(_lib.tl_keep_input_grad(lora, int(on)))


def tl_profile_enable(lora, on=True):
    _chk(_lib.tl_profile_enable(lora, int(on)))


def tl_profile_read(lora):
    """-> (milliseconds, launches, flop) of the frozen-weight GEMM launches since the last read"""
    ms, n, fl = C.c_double(), _i64(), C.c_double()
    _chk(_lib.tl_profile_read(lora, C.byref(ms), C.byref(n), C.byref(fl)))
    return ms.value, n.value, fl.value


def tl_layer_step(lora, layer, h_in, dh_out, h_out, dh_in, lr=0.0, apply_adamw=False):
    _chk(_lib.tl_layer_step(lora, layer, _dp(h_in), _dp(dh_out), h_in.shape[0], _dp(h_out), _dp(dh_in), lr,
                            int(apply_adamw)))


def tl_linear_step(X, W, A, B, dY, s, lr, beta1, beta2, eps, weight_decay, apply_adamw, Y, dX, dA, dB, A_new, B_new,
                   stream=None):
    T, d_in = X.shape
    d_out, r = B.shape
    _chk(_lib.tl_linear_step(_dp(X), _dp(W), _dp(A), _dp(B), _dp(dY), T, d_in, d_out, r, s, lr, beta1, beta2, eps,
                             weight_decay, int(apply_adamw), _dp(Y), _dp(dX), _dp(dA), _dp(dB), _dp(A_new),
                             _dp(B_new), stream if stream is not None else current_stream_handle()))


def tl_linear_step_static(X, W, A, B, dY, s, lr, beta1, beta2, eps, weight_decay, apply_adamw, Y, dX, dA, dB, A_new,
                          B_new, stream=None):
    T, d_in = X.shape
    d_out, r = B.shape
    _chk(_lib.tl_linear_step_static(_dp(X), _dp(W), _dp(A), _dp(B), _dp(dY), T, d_in, d_out, r, s, lr, beta1, beta2, eps,
                                    weight_decay, int(apply_adamw), _dp(Y), _dp(dX), _dp(dA), _dp(dB), _dp(A_new),
                                    _dp(B_new), stream if stream is not None else current_stream_handle()))


# ------------------------------------------------------------------ single kernels (not synchronised)
def _s(stream):
    return stream if stream is not None else current_stream_handle()


def tl_k_gemm_nt(A, B, C_out, A2=None, B2=None, alpha=1.0, R=None, workspace=None, stream=None):
    M, K = A.shape
    N = B.shape[0]
    K2 = A2.shape[1] if A2 is not None else 0
    _chk(_lib.tl_k_gemm_nt(_dp(A), A.stride(0), _dp(B), B.stride(0), M, N, K, _dp(A2),
                           A2.stride(0) if A2 is not None else 0, _dp(B2), B2.stride(0) if B2 is not None else 0, K2,
                           alpha, _dp(R), _dp(C_out), C_out.stride(0), int(C_out.dtype == torch.float32),
                           _dp(workspace), workspace.numel() if workspace is not None else 0, _s(stream)))


def tl_k_gemm_nt_plan(M, N, K, K2=0, workspace_elems=0):
    """-> (configuration name, contraction split, launches)"""
    buf = C.create_string_buffer(32)
    sp, nl = _i32(0), _i32(0)
    _chk(_lib.tl_k_gemm_nt_plan(M, N, K, K2, workspace_elems, buf, 32, C.byref(sp), C.byref(nl)))
    return buf.value.decode(), sp.value, nl.value


def tl_k_gemm_tn(P, Q, C_out, alpha=1.0, stream=None):
    T, Mo = P.shape
    No = Q.shape[1]
    _chk(_lib.tl_k_gemm_tn(_dp(P), P.stride(0), _dp(Q), Q.stride(0), T, Mo, No, alpha, _dp(C_out), C_out.stride(0),
                           _s(stream)))


def tl_k_rmsnorm_fwd(h, g, eps, y, stream=None):
    _chk(_lib.tl_k_rmsnorm_fwd(_dp(h), _dp(g), h.shape[0], h.shape[1], eps, _dp(y), _s(stream)))


def tl_k_rmsnorm_bwd(dy, h, g, dres, eps, dh_out, dh_out_bf16=None, stream=None):
    _chk(_lib.tl_k_rmsnorm_bwd(_dp(dy), _dp(h), _dp(g), _dp(dres), h.shape[0], h.shape[1], eps, _dp(dh_out),
                               _dp(dh_out_bf16), _s(stream)))


def tl_k_rope(x, n_heads, d_head, base=10000.0, pos0=0, sign=1, stream=None):
    _chk(_lib.tl_k_rope(_dp(x), x.stride(0), x.shape[0], n_heads, d_head, base, pos0, sign, _s(stream)))


def tl_k_rope_table(x, n_heads, d_head, table, base=10000.0, pos0=0, sign=1, stream=None):
    _chk(_lib.tl_k_rope_table(_dp(x), x.stride(0), x.shape[0], n_heads, d_head, base, pos0, sign, _dp(table),
                              table.numel(), _s(stream)))


def tl_k_dropout(x, y, p, seed, step, layer, group, stream=None):
    _chk(_lib.tl_k_dropout(_dp(x), x.shape[0], x.shape[1], p, seed, step, layer, group, _dp(y), _s(stream)))


def tl_k_swiglu_fwd(gu, a, stream=None):
    _chk(_lib.tl_k_swiglu_fwd(_dp(gu), gu.shape[0], gu.shape[1] // 2, _dp(a), _s(stream)))


def tl_k_swiglu_bwd(da, gu, dgu, stream=None):
    _chk(_lib.tl_k_swiglu_bwd(_dp(da), _dp(gu), gu.shape[0], gu.shape[1] // 2, _dp(dgu), _s(stream)))


def tl_k_gemv(W, x, y, lora_b=None, lora_h=None, rows_per_group=0, alpha=1.0, resid=None, stream=None):
    N, K = W.shape
    r = lora_b.shape[1] if lora_b is not None else 0
    _chk(_lib.tl_k_gemv(_dp(W), W.stride(0), _dp(x), N, K, _dp(lora_b), _dp(lora_h), r, rows_per_group, alpha, _dp(resid),
                        _dp(y), int(y.dtype == torch.float32), _s(stream)))


def tl_k_gemv_pre(W, y, mode, h=None, gain=None, eps=0.0, gu=None, x_out=None, stream=None):
    N, K = W.shape
    _chk(_lib.tl_k_gemv_pre(_dp(W), W.stride(0), N, K, mode, _dp(h), _dp(gain), eps, _dp(gu), _dp(x_out), _dp(y), _s(stream)))


def tl_k_attention_decode(q, k, v, n_heads, d_head, o, workspace=None, stream=None):
    _chk(_lib.tl_k_attention_decode(_dp(q), _dp(k), _dp(v), k.stride(0), k.shape[0], n_heads, d_head, _dp(o),
                                    _dp(workspace), workspace.numel() if workspace is not None else 0, _s(stream)))


def tl_k_argmax(x, out, stream=None):
    _chk(_lib.tl_k_argmax(_dp(x), x.numel(), _dp(out), _s(stream)))


def tl_k_attention_fwd(q, k, v, n_heads, d_head, o, lse, stream=None):
    _chk(_lib.tl_k_attention_fwd(_dp(q), _dp(k), _dp(v), q.stride(0), q.shape[0], n_heads, d_head, _dp(o),
                                 o.stride(0), _dp(lse), _s(stream)))


def tl_k_attention_bwd(q, k, v, o, d_o, lse, n_heads, d_head, dq, dk, dv, delta, stream=None):
    _chk(_lib.tl_k_attention_bwd(_dp(q), _dp(k), _dp(v), _dp(o), _dp(d_o), _dp(lse), q.stride(0), o.stride(0),
                                 q.shape[0], n_heads, d_head, _dp(dq), _dp(dk), _dp(dv), _dp(delta), _s(stream)))


def tl_k_cross_entropy(logits, labels, first_target, n_targets, nll, dlogits, loss_sum, stream=None):
    _chk(_lib.tl_k_cross_entropy(_dp(logits), _dp(labels), logits.shape[0], logits.shape[1], first_target, n_targets,
                                 _dp(nll), _dp(dlogits), _dp(loss_sum), _s(stream)))


def tl_k_adamw(p, g, m, v, shadow, step, lr, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, stream=None):
    _chk(_lib.tl_k_adamw(_dp(p), _dp(g), _dp(m), _dp(v), _dp(shadow), p.numel(), step, lr, beta1, beta2, eps,
                         weight_decay, _s(stream)))


def tl_k_embed(E, tokens, h, stream=None):
    _chk(_lib.tl_k_embed(_dp(E), _dp(tokens), tokens.shape[0], E.shape[1], _dp(h), _s(stream)))
