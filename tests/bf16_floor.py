"""A bf16-boundary replay of the oracle's chunk update (TEST INFRASTRUCTURE, CPU only).

Section 3 "Setup" says the module is trained in bfloat16.  This build reads that as: frozen weights, activations and
activation gradients are bf16 wherever one kernel hands a tensor to the next; accumulation, softmax, norm statistics,
the loss and the residual stream are fp32; the LoRA factors are fp32 with bf16 copies for the products.  ANY
implementation with those storage types differs from the fp64 oracle by the rounding it does at those hand-over
points -- however exact its arithmetic in between is.  This module measures that difference on the CPU: it runs the
oracle's own functions (norm, RoPE, attention, SwiGLU, cross-entropy, AdamW: oracle/templora_oracle.py) in fp64 and
rounds to bf16 (nearest even) or fp32 at exactly the hand-over points listed below, nowhere else.  The result is the
error floor of the storage format on a given workload, with no kernel involved; GPU tests at depth hold the HIP path to
a small multiple of it where the benchmark spec's tolerance of 2e-2 is below the floor.

Hand-over points (`rb` = to bf16, `rf` = to fp32):
  forward   x1 = rb(RMSNorm(h));  Hs = rb(s x rb(A)^T);  q|k|v = rb(x W^T + Hs rb(B)^T);  q, k = rb(RoPE(.));
            o = rb(attention);  h1 = rf(h + o W_o^T + ..);  x2, gate, up likewise;  act = rb(SwiGLU);  h_out = rf(..);
            hf = rb(final norm);  logits = rf(hf W_lm^T)
  backward  dlogits = rb(.);  dhf = rb(dlogits W_lm);  every dY entering a product is rb(fp32 gradient);
            dH = rb(s dY rb(B));  dX = rb(dY W + dH rb(A));  dgate|dup = rb(SwiGLU');  dq, dk = rb(RoPE^T(.)), dv = rb(.);
            residual-stream gradients rf(.);  dA = rf(dH^T X), dB = rf(dY^T Hs) from the rounded operands
With `exact=True` every rounding is the identity and the replay must reproduce oracle.model_fwd_bwd to fp64 rounding
(tests/test_bf16_floor.py checks that, so a wiring mistake here cannot pass as "rounding error").

`inner=True` additionally rounds what a bf16 matrix unit needs as an operand inside the attention kernels (the
probabilities before P V and P^T dO, dS before dS K and dS^T Q); the default is boundaries only.
"""
from __future__ import annotations

import numpy as np

from oracle import templora_oracle as O

F64 = np.float64
PROJ = O.PROJ


def round_bf16(x):
    """fp64 -> nearest fp32 -> nearest-even bf16, returned as fp64 (finite inputs)."""
    y = np.ascontiguousarray(x, dtype=np.float32).copy()
    u = y.reshape(-1).view(np.uint32)
    step = 1 << 22
    for i in range(0, u.size, step):
        blk = u[i:i + step]
        t = (blk >> np.uint32(16)) & np.uint32(1)
        t += np.uint32(0x7FFF)
        blk += t
        blk &= np.uint32(0xFFFF0000)
    return y.astype(F64)


def round_f32(x):
    return np.asarray(x, dtype=np.float32).astype(F64)


class Rounding:
    def __init__(self, exact: bool = False, inner: bool = False):
        ident = lambda x: np.asarray(x, dtype=F64)
        self.b = ident if exact else round_bf16
        self.f = ident if exact else round_f32
        self.inner = inner and not exact


def _lin_fwd(X, W, A, B, s, R):
    """X already bf16-valued.  Returns (Y unrounded fp64, Hs = rb(s X rb(A)^T))."""
    Hs = R.b(s * (X @ R.b(A).T))
    return X @ O._f(W).T + Hs @ R.b(B).T, Hs


def _lin_bwd(dY, X, Hs, W, A, B, s, R):
    """dY, X, Hs bf16-valued.  Returns (dX unrounded, dA, dB)."""
    dH = R.b(s * (dY @ R.b(B)))
    dX = dY @ O._f(W) + dH @ R.b(A)
    return dX, R.f(dH.T @ X), R.f(dY.T @ Hs)


def _attention_fwd(q, k, v, R):
    if not R.inner:
        return O.attention_fwd(q, k, v)
    o, P = O.attention_fwd(q, k, v)
    Pb = R.b(P)
    for h in range(q.shape[1]):
        o[:, h, :] = Pb[h] @ v[:, h, :]
    return o, P


def _attention_bwd(do, q, k, v, P, R):
    if not R.inner:
        return O.attention_bwd(do, q, k, v, P)
    T, nh, dh = q.shape
    dq, dk, dv = np.empty_like(q), np.empty_like(k), np.empty_like(v)
    for h in range(nh):
        dv[:, h, :] = R.b(P[h]).T @ do[:, h, :]
        dP = do[:, h, :] @ v[:, h, :].T
        dS = R.b(P[h] * (dP - np.sum(dP * P[h], axis=-1, keepdims=True)))
        dq[:, h, :] = (dS @ k[:, h, :]) / np.sqrt(dh)
        dk[:, h, :] = (dS.T @ q[:, h, :]) / np.sqrt(dh)
    return dq, dk, dv


def layer_fwd(h, W, L, shape, R, store=np.float32):
    """One decoder layer; h fp32-valued.  Returns (h_out, cache); cache tensors are kept in `store` precision (bf16
    values are exact in fp32; the probabilities lose nothing that matters)."""
    T = h.shape[0]
    nh, dh, s = shape.n_heads, shape.d_head, shape.scale
    keep = (lambda x: x) if store is F64 else (lambda x: np.asarray(x, dtype=store))
    c = {"h0": keep(h)}
    x1 = R.b(O.rmsnorm_fwd(h, W["g1"], shape.rms_eps))
    y, hs = {}, {}
    for p in ("q", "k", "v"):
        y[p], hs[p] = _lin_fwd(x1, W[p], *L[p], s, R)
        y[p] = R.b(y[p])
    q = R.b(O.rope_fwd(y["q"].reshape(T, nh, dh), shape.rope_base))
    k = R.b(O.rope_fwd(y["k"].reshape(T, nh, dh), shape.rope_base))
    v = y["v"].reshape(T, nh, dh)
    o, P = _attention_fwd(q, k, v, R)
    o = R.b(o.reshape(T, nh * dh))
    yo, hs["o"] = _lin_fwd(o, W["o"], *L["o"], s, R)
    h1 = R.f(h + yo)
    x2 = R.b(O.rmsnorm_fwd(h1, W["g2"], shape.rms_eps))
    g, hs["gate"] = _lin_fwd(x2, W["gate"], *L["gate"], s, R)
    u, hs["up"] = _lin_fwd(x2, W["up"], *L["up"], s, R)
    g, u = R.b(g), R.b(u)
    a = R.b(O.swiglu_fwd(g, u))
    yd, hs["down"] = _lin_fwd(a, W["down"], *L["down"], s, R)
    c.update(x1=keep(x1), q=keep(q), k=keep(k), v=keep(v), P=keep(P), o=keep(o), h1=keep(h1), x2=keep(x2), g=keep(g),
             u=keep(u), a=keep(a), hs={p: keep(hs[p]) for p in PROJ})
    return R.f(h1 + yd), c


def layer_bwd(dh_out, c, W, L, shape, R):
    """dh_out fp32-valued gradient at the layer's output -> (gradient at its input, {p: (dA, dB)})."""
    T = dh_out.shape[0]
    nh, dh, s = shape.n_heads, shape.d_head, shape.scale
    f = lambda x: np.asarray(x, dtype=F64)
    G = {}
    dy = R.b(dh_out)
    da, *G["down"] = _lin_bwd(dy, f(c["a"]), f(c["hs"]["down"]), W["down"], *L["down"], s, R)
    dg, du = O.swiglu_bwd(R.b(da), f(c["g"]), f(c["u"]))
    dg, du = R.b(dg), R.b(du)
    dx_g, *G["gate"] = _lin_bwd(dg, f(c["x2"]), f(c["hs"]["gate"]), W["gate"], *L["gate"], s, R)
    dx_u, *G["up"] = _lin_bwd(du, f(c["x2"]), f(c["hs"]["up"]), W["up"], *L["up"], s, R)
    dh1 = R.f(dh_out + O.rmsnorm_bwd(R.b(dx_g + dx_u), f(c["h1"]), W["g2"], shape.rms_eps))
    d_o, *G["o"] = _lin_bwd(R.b(dh1), f(c["o"]), f(c["hs"]["o"]), W["o"], *L["o"], s, R)
    dq, dk, dv = _attention_bwd(R.b(d_o).reshape(T, nh, dh), f(c["q"]), f(c["k"]), f(c["v"]), f(c["P"]), R)
    dq = R.b(O.rope_bwd(dq, shape.rope_base).reshape(T, nh * dh))
    dk = R.b(O.rope_bwd(dk, shape.rope_base).reshape(T, nh * dh))
    dv = R.b(dv.reshape(T, nh * dh))
    x1 = f(c["x1"])
    dx_q, *G["q"] = _lin_bwd(dq, x1, f(c["hs"]["q"]), W["q"], *L["q"], s, R)
    dx_k, *G["k"] = _lin_bwd(dk, x1, f(c["hs"]["k"]), W["k"], *L["k"], s, R)
    dx_v, *G["v"] = _lin_bwd(dv, x1, f(c["hs"]["v"]), W["v"], *L["v"], s, R)
    dh0 = R.f(dh1 + O.rmsnorm_bwd(R.b(dx_q + dx_k + dx_v), f(c["h0"]), W["g1"], shape.rms_eps))
    return dh0, {p: tuple(G[p]) for p in PROJ}


def model_fwd_bwd(tokens, n_ctx, shape, emb, head, g_final, get_layer, lora, keep=(), exact=False, inner=False,
                  on_layer=None):
    """Same contract as oracle.model_fwd_bwd (no dropout), with the roundings above.  on_layer(l, dh_in, grads) is
    called as the backward pass leaves layer l (so that a caller can reduce a layer's results and drop them)."""
    R = Rounding(exact, inner)
    tok = np.asarray(tokens, dtype=np.int64)
    labels, mask, N = O.labels_and_mask(tok, n_ctx)
    h = O._f(emb)[tok]
    caches = []
    for l in range(shape.n_layers):
        h, c = layer_fwd(h, get_layer(l), lora[l], shape, R, F64 if exact else np.float32)
        caches.append(c)
    hf = R.b(O.rmsnorm_fwd(h, g_final, shape.rms_eps))
    logits = R.f(hf @ O._f(head).T)
    loss, nll, dlogits = O.cross_entropy(logits, labels, mask)
    dhf = R.b(R.b(dlogits) @ O._f(head))
    dh = R.f(O.rmsnorm_bwd(dhf, h, g_final, shape.rms_eps))
    out = {"loss": loss, "nll": nll, "n_targets": N, "dh": {"final": dh}, "grads": [None] * shape.n_layers}
    del logits, dlogits
    for l in reversed(range(shape.n_layers)):
        dh, G = layer_bwd(dh, caches[l], get_layer(l), lora[l], shape, R)
        caches[l] = None
        if on_layer is not None:
            on_layer(l, dh, G)
        else:
            out["grads"][l] = G
        if l in keep:
            out["dh"][l] = dh
    return out


def chunk_update(tokens, n_ctx, shape, emb, head, g_final, get_layer, lora, opt, lr, keep=(), inner=False,
                 beta1=0.9, beta2=0.999, eps=1e-8, wd=0.0):
    """One optimizer step of the replay: gradients from model_fwd_bwd above, the oracle's AdamW on fp32-valued state."""
    res = model_fwd_bwd(tokens, n_ctx, shape, emb, head, g_final, get_layer, lora, keep, False, inner)
    tau = opt["tau"] + 1
    new_lora, new_m, new_v = [], [], []
    for l in range(shape.n_layers):
        Ll, Ml, Vl = {}, {}, {}
        for p in PROJ:
            facs, ms, vs = [], [], []
            for i in range(2):
                pn, mn, vn = O.adamw_step(lora[l][p][i], res["grads"][l][p][i], opt["m"][l][p][i], opt["v"][l][p][i],
                                          tau, lr, beta1, beta2, eps, wd)
                facs.append(round_f32(pn)), ms.append(round_f32(mn)), vs.append(round_f32(vn))
            Ll[p], Ml[p], Vl[p] = tuple(facs), tuple(ms), tuple(vs)
        new_lora.append(Ll), new_m.append(Ml), new_v.append(Vl)
    return res, new_lora, {"tau": tau, "m": new_m, "v": new_v}


def chunk_train(tokens, n_chunk, L_T, batch, epochs, lr, warmup_steps, shape, emb, head, g_final, get_layer, lora, opt):
    """The replay of oracle.chunk_train: same samples, same warm-up, steps made by chunk_update above."""
    tok = np.asarray(tokens, dtype=np.int64)
    losses = []
    for _ in range(epochs):
        for first, n_ctx, end in O.training_samples(tok.size - n_chunk, n_chunk, L_T, batch):
            rate = O.warmup_lr(lr, opt["tau"], warmup_steps)
            res, lora, opt = chunk_update(tok[first:end], n_ctx, shape, emb, head, g_final, get_layer, lora, opt, rate)
            losses.append(res["loss"])
    return losses, lora, opt


def rel_err(x, ref):
    x, ref = np.asarray(x, dtype=F64), np.asarray(ref, dtype=F64)
    n = np.linalg.norm(ref)
    return float(np.linalg.norm(x - ref) / n) if n > 0 else float(np.linalg.norm(x))
