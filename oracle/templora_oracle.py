"""CPU oracle for the Temp-Lora chunk update (TEST INFRASTRUCTURE, not a product path).

A plain, slow, fp64 numpy statement of what one "Train Theta_k: In X_T -> Out
Chunk_k" step of Algorithm 1 computes for a Llama2-style decoder (Section 3,
"Baselines") whose projections carry a LoRA module (Section 2; rank and alpha
from Section 3 "Setup"): forward, next-token loss on the chunk, backward to the
LoRA factors only, one AdamW step at the paper's learning rate.

Rules this file keeps:
  * every function takes the algorithm's steps in order, in fp64, with a numpy
    matmul / exp / sum as the only primitives; no blocking, fusion or reuse
    tricks, so that it can be checked against the paper by eye;
  * it imports nothing from the HIP package and shares no code with it;
  * only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may
    import it.

Pins (tests/test_oracle_pins.py): B = 0 gives the base model exactly; merged
weight W + s*B*A gives the same forward; central finite differences and an
independent autograd graph agree with every gradient; the loss is a valid NLL
(ln V on uniform logits, agreement with a library log-softmax); AdamW agrees
with its step-1 closed form and with a library optimizer over several steps;
RoPE and RMSNorm invariants; causality; window_logits agrees with the autograd
graph's logits and is causal (a longer window leaves earlier rows unchanged);
window_logits_reuse with the same module on both sides is window_logits, and
with different ones its old positions are untouched by the new module;
chunk_train's samples cover every chunk position exactly once per epoch with at
most L_T conditioning tokens, its warm-up is checked against hand-computed
rates, and with one piece, one epoch and no warm-up it is chunk_update; the
dropout generator reproduces SplitMix64's published first outputs, its masks
drop a fraction p and keep the mean, p = 0 is exactly the path without dropout,
and gradients under a fixed mask agree with the autograd graph given the same
mask.  Absolute loss / gradient values at the
workload shapes are printed nowhere in the paper: they are pinned only through
these properties.

Layouts: activations [T, width]; W [d_out, d_in]; A [r, d_in]; B [d_out, r].
"""
from __future__ import annotations

import numpy as np

PROJ = ("q", "k", "v", "o", "gate", "up", "down")
F64 = np.float64


def _f(x):
    return np.asarray(x, dtype=F64)


# --------------------------------------------------------------------------
# Labels and loss mask (Section 2: the preceding L_T tokens are the input, the
# chunk is the output; Algorithm 1, the "Train" line).
# --------------------------------------------------------------------------
def labels_and_mask(tokens, n_ctx: int):
    """label[t] = tokens[t+1]; position t carries loss iff its label is a chunk token.

    tokens = n_ctx conditioning tokens followed by the chunk.  Position t
    predicts token t+1, so it is a target iff t+1 >= max(n_ctx, 1) and t+1 < T.
    Returns (labels int64[T] with labels[T-1] = -1, mask bool[T], N targets).
    """
    tok = np.asarray(tokens, dtype=np.int64)
    T = tok.shape[0]
    labels = np.full(T, -1, dtype=np.int64)
    labels[: T - 1] = tok[1:]
    t = np.arange(T)
    mask = (t + 1 >= max(int(n_ctx), 1)) & (t + 1 < T)
    return labels, mask, int(mask.sum())


# --------------------------------------------------------------------------
# LoRA-adapted linear layer (Section 2: a temporary LoRA module on a frozen LM).
# --------------------------------------------------------------------------
def lora_linear_fwd(X, W, A, B, s: float, D=None):
    """Y = X W^T + s ((D o X) A^T) B^T.  Returns (Y, H) with H = (D o X) A^T.

    D is the dropout factor on the input of the low-rank branch (Section 3 "Setup": dropout 0.05): 0 where an
    element is dropped, 1 / (1 - p) where it is kept; None means no dropout (D = 1)."""
    X, W, A, B = _f(X), _f(W), _f(A), _f(B)
    Xl = X if D is None else X * _f(D)
    H = Xl @ A.T
    Y = X @ W.T + s * (H @ B.T)
    return Y, H


def lora_linear_bwd(dY, X, W, A, B, s: float, D=None):
    """Gradients of <dY, Y> w.r.t. X, A, B; W is frozen so no dW exists.

    dH = s dY B;  dX = dY W + D o (dH A);  dA = dH^T (D o X);  dB = s dY^T ((D o X) A^T).
    """
    dY, X, W, A, B = _f(dY), _f(X), _f(W), _f(A), _f(B)
    Xl = X if D is None else X * _f(D)
    dH = s * (dY @ B)
    dX = dY @ W + (dH @ A if D is None else _f(D) * (dH @ A))
    dA = dH.T @ Xl
    dB = s * (dY.T @ (Xl @ A.T))
    return dX, dA, dB


# --------------------------------------------------------------------------
# Dropout masks.  The paper only names the rate; which elements fall is an encoding this build fixes so that two
# implementations can draw the same mask: a counter-based generator (the 64-bit finaliser of the SplitMix64
# generator) keyed by (seed, optimizer step, layer, projection group) and indexed by the element.
# --------------------------------------------------------------------------
GROUPS = ("qkv", "o", "gu", "down")      # projection groups that share an input, in mask-stream order 0..3
_M64 = (1 << 64) - 1


def _mix64(z):
    """SplitMix64's output function of the state z + golden-ratio increment, on numpy uint64 (wrap-around)."""
    z = np.asarray(z, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = z + np.uint64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        return z ^ (z >> np.uint64(31))


def dropout_factor(seed: int, step: int, layer: int, group: int, T: int, d_in: int, p: float):
    """D [T, d_in]: 0 where element (t, c) is dropped, 1 / (1 - p) where it is kept.  p is taken in fp32."""
    p32 = float(np.float32(p))
    stream = ((1 << 63) | (int(step) << 16) | (int(layer) << 3) | int(group)) & _M64
    key = _mix64(np.uint64(int(seed) & _M64) ^ _mix64(np.uint64(stream)))
    with np.errstate(over="ignore"):
        bits = _mix64(key + np.arange(T * d_in, dtype=np.uint64)) >> np.uint64(32)
    thr = min(int(np.floor(p32 * 4294967296.0)), 4294967295)
    keep = bits >= np.uint64(max(thr, 0))
    return (keep.astype(F64) / (1.0 - p32)).reshape(T, d_in)


# --------------------------------------------------------------------------
# RMSNorm, RoPE, SwiGLU (Llama2 decoder blocks, Section 3 "Baselines").
# --------------------------------------------------------------------------
def rmsnorm_fwd(h, g, eps: float):
    h, g = _f(h), _f(g)
    rho = 1.0 / np.sqrt(np.mean(h * h, axis=-1, keepdims=True) + eps)
    return h * rho * g


def rmsnorm_bwd(dy, h, g, eps: float):
    """dh = rho (g*dy) - h rho^3 mean_j(h_j g_j dy_j); the gain is frozen (no dg)."""
    dy, h, g = _f(dy), _f(h), _f(g)
    rho = 1.0 / np.sqrt(np.mean(h * h, axis=-1, keepdims=True) + eps)
    gd = g * dy
    return rho * gd - h * rho ** 3 * np.mean(h * gd, axis=-1, keepdims=True)


def _rope_angles(T: int, d_head: int, base: float, pos0: int = 0):
    i = np.arange(d_head // 2, dtype=F64)
    theta = base ** (-2.0 * i / d_head)
    p = np.arange(pos0, pos0 + T, dtype=F64)
    return np.outer(p, theta)  # [T, d_head/2]


def rope_fwd(x, base: float, pos0: int = 0, sign: float = 1.0):
    """x [T, n_heads, d_head]; pair (i, i + d_head/2) rotated by angle p*theta_i."""
    x = _f(x)
    T, _, dh = x.shape
    ang = sign * _rope_angles(T, dh, base, pos0)
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    x1, x2 = x[..., : dh // 2], x[..., dh // 2:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def rope_bwd(dy, base: float, pos0: int = 0):
    """The rotation is orthogonal: its transpose is the rotation by the negated angle."""
    return rope_fwd(dy, base, pos0, sign=-1.0)


def swiglu_fwd(g, u):
    g, u = _f(g), _f(u)
    return g / (1.0 + np.exp(-g)) * u


def swiglu_bwd(da, g, u):
    da, g, u = _f(da), _f(g), _f(u)
    sig = 1.0 / (1.0 + np.exp(-g))
    dg = da * u * sig * (1.0 + g * (1.0 - sig))
    du = da * g * sig
    return dg, du


# --------------------------------------------------------------------------
# Causal self-attention within the call's tokens.
# --------------------------------------------------------------------------
def attention_fwd(q, k, v):
    """q, k, v [T, n_heads, d_head] -> (o [T, n_heads, d_head], P [n_heads, T, T]).

    Per head: S = q k^T / sqrt(d_head), S_tu = -inf for u > t, P = softmax over u, o = P v.
    """
    q, k, v = _f(q), _f(k), _f(v)
    T, nh, dh = q.shape
    future = np.triu(np.ones((T, T), dtype=bool), k=1)
    P = np.empty((nh, T, T), dtype=F64)
    o = np.empty((T, nh, dh), dtype=F64)
    for h in range(nh):
        S = (q[:, h, :] @ k[:, h, :].T) / np.sqrt(dh)
        S[future] = -np.inf
        S -= S.max(axis=-1, keepdims=True)
        E = np.exp(S)
        P[h] = E / E.sum(axis=-1, keepdims=True)
        o[:, h, :] = P[h] @ v[:, h, :]
    return o, P


def attention_bwd(do, q, k, v, P):
    """dv = P^T do; dP = do v^T; dS = P * (dP - rowsum(dP * P)); dq = dS k / sqrt(d); dk = dS^T q / sqrt(d)."""
    do, q, k, v = _f(do), _f(q), _f(k), _f(v)
    T, nh, dh = q.shape
    dq, dk, dv = np.empty_like(q), np.empty_like(k), np.empty_like(v)
    for h in range(nh):
        dv[:, h, :] = P[h].T @ do[:, h, :]
        dP = do[:, h, :] @ v[:, h, :].T
        dS = P[h] * (dP - np.sum(dP * P[h], axis=-1, keepdims=True))
        dq[:, h, :] = (dS @ k[:, h, :]) / np.sqrt(dh)
        dk[:, h, :] = (dS.T @ q[:, h, :]) / np.sqrt(dh)
    return dq, dk, dv


# --------------------------------------------------------------------------
# Next-token cross-entropy on the chunk positions (perplexity = exp(loss),
# Section 3 "Evaluation Metric").
# --------------------------------------------------------------------------
def cross_entropy(logits, labels, mask):
    """loss = mean over masked positions of (logsumexp(logits_t) - logits_t[label_t]).

    Returns (loss, nll [T] (0 where unmasked), dlogits [T, V] = d loss / d logits).
    """
    z = _f(logits)
    T, V = z.shape
    N = int(np.sum(mask))
    zmax = z.max(axis=-1, keepdims=True)
    lse = np.log(np.exp(z - zmax).sum(axis=-1)) + zmax[:, 0]
    nll = np.zeros(T, dtype=F64)
    dlogits = np.zeros_like(z)
    for t in range(T):
        if mask[t]:
            nll[t] = lse[t] - z[t, labels[t]]
            p = np.exp(z[t] - lse[t])
            p[labels[t]] -= 1.0
            dlogits[t] = p / N
    loss = nll.sum() / N
    return loss, nll, dlogits


# --------------------------------------------------------------------------
# AdamW on the LoRA factors (Section 3 "Setup": learning rate 5e-5).
# --------------------------------------------------------------------------
def adamw_step(p, g, m, v, tau: int, lr: float, beta1=0.9, beta2=0.999, eps=1e-8, wd=0.0):
    """One decoupled-weight-decay Adam step with bias correction; tau is 1-based."""
    p, g, m, v = _f(p), _f(g), _f(m), _f(v)
    p = p * (1.0 - lr * wd)
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** tau)
    vhat = v / (1.0 - beta2 ** tau)
    p = p - lr * mhat / (np.sqrt(vhat) + eps)
    return p, m, v


# --------------------------------------------------------------------------
# One decoder layer with LoRA on q, k, v, o, gate, up, down.
# --------------------------------------------------------------------------
def layer_fwd(h, W: dict, L: dict, shape, pos0: int = 0, D=None):
    """h [T, d] -> (h_out, cache).  W[p] frozen [d_out, d_in], W['g1'|'g2'] gains; L[p] = (A, B).
    D: None, or {group: dropout factor of that group's input} for the groups in GROUPS."""
    h = _f(h)
    D = D or {}
    Dq, Do, Dg, Dd = (D.get(g) for g in GROUPS)
    T = h.shape[0]
    nh, dh, s = shape.n_heads, shape.d_head, shape.scale
    c = {"h0": h, "D": (Dq, Do, Dg, Dd)}
    c["x1"] = rmsnorm_fwd(h, W["g1"], shape.rms_eps)
    q, _ = lora_linear_fwd(c["x1"], W["q"], *L["q"], s, Dq)
    k, _ = lora_linear_fwd(c["x1"], W["k"], *L["k"], s, Dq)
    v, _ = lora_linear_fwd(c["x1"], W["v"], *L["v"], s, Dq)
    c["q"] = rope_fwd(q.reshape(T, nh, dh), shape.rope_base, pos0)
    c["k"] = rope_fwd(k.reshape(T, nh, dh), shape.rope_base, pos0)
    c["v"] = v.reshape(T, nh, dh)
    o, c["P"] = attention_fwd(c["q"], c["k"], c["v"])
    c["o"] = o.reshape(T, nh * dh)
    yo, _ = lora_linear_fwd(c["o"], W["o"], *L["o"], s, Do)
    c["h1"] = h + yo
    c["x2"] = rmsnorm_fwd(c["h1"], W["g2"], shape.rms_eps)
    c["g"], _ = lora_linear_fwd(c["x2"], W["gate"], *L["gate"], s, Dg)
    c["u"], _ = lora_linear_fwd(c["x2"], W["up"], *L["up"], s, Dg)
    c["a"] = swiglu_fwd(c["g"], c["u"])
    yd, _ = lora_linear_fwd(c["a"], W["down"], *L["down"], s, Dd)
    return c["h1"] + yd, c


def layer_bwd(dh_out, c: dict, W: dict, L: dict, shape, pos0: int = 0):
    """Upstream d loss / d h_out -> (d loss / d h_in, {p: (dA, dB)})."""
    dh_out = _f(dh_out)
    T = dh_out.shape[0]
    nh, dh, s = shape.n_heads, shape.d_head, shape.scale
    G = {}
    Dq, Do, Dg, Dd = c["D"]
    da, *G["down"] = lora_linear_bwd(dh_out, c["a"], W["down"], *L["down"], s, Dd)
    dg, du = swiglu_bwd(da, c["g"], c["u"])
    dx2_g, *G["gate"] = lora_linear_bwd(dg, c["x2"], W["gate"], *L["gate"], s, Dg)
    dx2_u, *G["up"] = lora_linear_bwd(du, c["x2"], W["up"], *L["up"], s, Dg)
    dh1 = dh_out + rmsnorm_bwd(dx2_g + dx2_u, c["h1"], W["g2"], shape.rms_eps)
    do, *G["o"] = lora_linear_bwd(dh1, c["o"], W["o"], *L["o"], s, Do)
    dq, dk, dv = attention_bwd(do.reshape(T, nh, dh), c["q"], c["k"], c["v"], c["P"])
    dq = rope_bwd(dq, shape.rope_base, pos0).reshape(T, nh * dh)
    dk = rope_bwd(dk, shape.rope_base, pos0).reshape(T, nh * dh)
    dv = dv.reshape(T, nh * dh)
    dx1_q, *G["q"] = lora_linear_bwd(dq, c["x1"], W["q"], *L["q"], s, Dq)
    dx1_k, *G["k"] = lora_linear_bwd(dk, c["x1"], W["k"], *L["k"], s, Dq)
    dx1_v, *G["v"] = lora_linear_bwd(dv, c["x1"], W["v"], *L["v"], s, Dq)
    dh0 = dh1 + rmsnorm_bwd(dx1_q + dx1_k + dx1_v, c["h0"], W["g1"], shape.rms_eps)
    return dh0, {p: tuple(G[p]) for p in PROJ}


# --------------------------------------------------------------------------
# The whole chunk update.
# --------------------------------------------------------------------------
def layer_dropout(drop, shape, layer: int, T: int):
    """drop = None or (p, seed, optimizer step index) -> {group: factor} for one layer's four group inputs."""
    if not drop or drop[0] <= 0.0:
        return None
    p, seed, step = drop
    d_in = {"qkv": shape.d_model, "o": shape.d_model, "gu": shape.d_model, "down": shape.d_ffn}
    return {g: dropout_factor(seed, step, layer, gi, T, d_in[g], p) for gi, g in enumerate(GROUPS)}


def model_fwd_bwd(tokens, n_ctx, shape, emb, head, g_final, get_layer, lora, keep=(), drop=None):
    """Forward + backward of one call's tokens.

    get_layer(l) returns layer l's frozen dict (so a 7B-shape caller can build
    layers on demand); lora[l][p] = (A, B).  Returns a dict with loss, nll,
    n_targets, grads[l][p] = (dA, dB), and dh at the layer inputs listed in
    `keep` (plus 'final' = gradient at the last layer's output).
    """
    tok = np.asarray(tokens, dtype=np.int64)
    if tok.min() < 0 or tok.max() >= shape.vocab:
        raise ValueError("token id out of range")
    labels, mask, N = labels_and_mask(tok, n_ctx)
    if N < 1:
        raise ValueError("no target positions")
    h = _f(emb)[tok]
    caches = []
    for l in range(shape.n_layers):
        h, c = layer_fwd(h, get_layer(l), lora[l], shape, 0, layer_dropout(drop, shape, l, tok.size))
        caches.append(c)
    hf = rmsnorm_fwd(h, g_final, shape.rms_eps)
    logits = hf @ _f(head).T
    loss, nll, dlogits = cross_entropy(logits, labels, mask)
    dhf = dlogits @ _f(head)
    dh = rmsnorm_bwd(dhf, h, g_final, shape.rms_eps)
    out = {"loss": loss, "nll": nll, "n_targets": N, "labels": labels, "mask": mask,
           "logits": logits, "dh": {"final": dh}, "grads": [None] * shape.n_layers}
    for l in reversed(range(shape.n_layers)):
        dh, out["grads"][l] = layer_bwd(dh, caches[l], get_layer(l), lora[l], shape)
        caches[l] = None
        if l in keep:
            out["dh"][l] = dh
    return out


# --------------------------------------------------------------------------
# Generation side (Algorithm 1: the token loop between two updates).
# --------------------------------------------------------------------------
def window_logits(tokens, shape, emb, head, g_final, get_layer, lora):
    """Logits of every position of a window under the LoRA-adapted model (no cache, no shortcuts:
    the whole window is recomputed, which is what a key/value cache must reproduce)."""
    tok = np.asarray(tokens, dtype=np.int64)
    if tok.size < 1 or tok.min() < 0 or tok.max() >= shape.vocab:
        raise ValueError("token id out of range")
    h = _f(emb)[tok]
    for l in range(shape.n_layers):
        h, _ = layer_fwd(h, get_layer(l), lora[l], shape)
    return rmsnorm_fwd(h, g_final, shape.rms_eps) @ _f(head).T


def greedy_next(tokens, shape, emb, head, g_final, get_layer, lora):
    """(next token, last-position logits): the largest logit, lowest index among equals."""
    logits = window_logits(tokens, shape, emb, head, g_final, get_layer, lora)[-1]
    return int(np.argmax(logits)), logits


def greedy_decode(prompt, n_new, shape, emb, head, g_final, get_layer, lora):
    """Algorithm 1's inner loop: append the greedy token n_new times, recomputing the window each time."""
    seq = [int(t) for t in prompt]
    for _ in range(n_new):
        nxt, _ = greedy_next(seq, shape, emb, head, g_final, get_layer, lora)
        seq.append(nxt)
    return seq[len(prompt):]


def _layer_with_past(h, W, L, shape, past_k, past_v):
    """One layer over new positions n_past .. n_past + T - 1 whose attention also sees the given keys and values of
    positions 0 .. n_past - 1 (past_k rotated, both [n_past, n_heads, d_head]).  Returns (h_out, k, v) of the new rows.
    Written from the definition: softmax over every visible key, no running statistics."""
    T, n_past = h.shape[0], past_k.shape[0]
    nh, dh, s = shape.n_heads, shape.d_head, shape.scale
    x1 = rmsnorm_fwd(h, W["g1"], shape.rms_eps)
    q = rope_fwd(lora_linear_fwd(x1, W["q"], *L["q"], s)[0].reshape(T, nh, dh), shape.rope_base, n_past)
    k = rope_fwd(lora_linear_fwd(x1, W["k"], *L["k"], s)[0].reshape(T, nh, dh), shape.rope_base, n_past)
    v = lora_linear_fwd(x1, W["v"], *L["v"], s)[0].reshape(T, nh, dh)
    K = np.concatenate([_f(past_k), k], 0)
    V = np.concatenate([_f(past_v), v], 0)
    o = np.zeros((T, nh, dh), F64)
    for i in range(T):
        vis = n_past + i + 1                                   # query i sits at position n_past + i
        sc = np.einsum("hd,uhd->hu", q[i], K[:vis]) / np.sqrt(dh)
        sc = np.exp(sc - sc.max(1, keepdims=True))
        o[i] = np.einsum("hu,uhd->hd", sc / sc.sum(1, keepdims=True), V[:vis])
    h1 = h + lora_linear_fwd(o.reshape(T, nh * dh), W["o"], *L["o"], s)[0]
    x2 = rmsnorm_fwd(h1, W["g2"], shape.rms_eps)
    a = swiglu_fwd(lora_linear_fwd(x2, W["gate"], *L["gate"], s)[0], lora_linear_fwd(x2, W["up"], *L["up"], s)[0])
    return h1 + lora_linear_fwd(a, W["down"], *L["down"], s)[0], k, v


def window_logits_reuse(tokens, n_stale, shape, emb, head, g_final, get_layer, lora_old, lora_new):
    """Cache reuse (Section 2): logits of positions n_stale .. under lora_new, attending over the keys and values that
    lora_old computed for positions 0 .. n_stale - 1 (every layer's cache is the old module's forward pass over the old
    positions; nothing of the old positions is recomputed)."""
    tok = np.asarray(tokens, dtype=np.int64)
    nh, dh = shape.n_heads, shape.d_head
    empty = np.zeros((0, nh, dh), F64)
    h_old, h_new = _f(emb)[tok[:n_stale]], _f(emb)[tok[n_stale:]]
    for l in range(shape.n_layers):
        W = get_layer(l)
        h_old, k_old, v_old = _layer_with_past(h_old, W, lora_old[l], shape, empty, empty)
        h_new, _, _ = _layer_with_past(h_new, W, lora_new[l], shape, k_old, v_old)
    return rmsnorm_fwd(h_new, g_final, shape.rms_eps) @ _f(head).T


def new_opt_state(lora):
    """Zero first/second moments for every factor; step counter 0."""
    return {"tau": 0,
            "m": [{p: (np.zeros_like(_f(a)), np.zeros_like(_f(b))) for p, (a, b) in L.items()} for L in lora],
            "v": [{p: (np.zeros_like(_f(a)), np.zeros_like(_f(b))) for p, (a, b) in L.items()} for L in lora]}


def chunk_update(tokens, n_ctx, shape, emb, head, g_final, get_layer, lora, opt, lr,
                 beta1=0.9, beta2=0.999, eps=1e-8, wd=0.0, keep=(), dropout=0.0, seed=0):
    """One optimizer step on one chunk: returns (result dict, new lora, new opt).
    With dropout > 0 the masks of this step are those of (seed, number of steps taken so far)."""
    res = model_fwd_bwd(tokens, n_ctx, shape, emb, head, g_final, get_layer, lora, keep,
                        (dropout, seed, opt["tau"]) if dropout > 0.0 else None)
    tau = opt["tau"] + 1
    new_lora, new_m, new_v = [], [], []
    for l in range(shape.n_layers):
        Ll, Ml, Vl = {}, {}, {}
        for p in PROJ:
            facs, ms, vs = [], [], []
            for i in range(2):  # 0: A, 1: B
                pn, mn, vn = adamw_step(lora[l][p][i], res["grads"][l][p][i], opt["m"][l][p][i],
                                        opt["v"][l][p][i], tau, lr, beta1, beta2, eps, wd)
                facs.append(pn), ms.append(mn), vs.append(vn)
            Ll[p], Ml[p], Vl[p] = tuple(facs), tuple(ms), tuple(vs)
        new_lora.append(Ll), new_m.append(Ml), new_v.append(Vl)
    return res, new_lora, {"tau": tau, "m": new_m, "v": new_v}


# --------------------------------------------------------------------------
# The whole module update for one chunk (Algorithm 1, "Train Theta_k"; Section 3 "Setup": n epochs,
# linear warm-up; Table 5: a chunk of Delta tokens trained in Delta / batch steps per epoch).
# --------------------------------------------------------------------------
def warmup_lr(lr: float, step: int, warmup_steps: int) -> float:
    """Rate of the optimizer step with 0-based index `step`: rises linearly and reaches lr at step warmup_steps - 1."""
    if warmup_steps <= 0:
        return lr
    return lr * min(1.0, (max(step, 0) + 1) / warmup_steps)


def training_samples(n_before: int, n_chunk: int, L_T: int, batch: int):
    """[(first token, n_ctx, end)] of one epoch: the chunk occupies positions n_before .. n_before + n_chunk - 1 of the
    stream; each piece of `batch` chunk tokens is trained with the up to L_T tokens before it as conditioning."""
    if batch <= 0 or batch > n_chunk:
        batch = n_chunk
    out = []
    for start in range(n_before, n_before + n_chunk, batch):
        end = min(start + batch, n_before + n_chunk)
        n_ctx = min(start, L_T)
        out.append((start - n_ctx, n_ctx, end))
    return out


def chunk_train(tokens, n_chunk, L_T, batch, epochs, lr, warmup_steps, shape, emb, head, g_final, get_layer, lora, opt,
                beta1=0.9, beta2=0.999, eps=1e-8, wd=0.0, dropout=0.0, seed=0):
    """-> (losses of every step in order, new lora, new opt).  tokens: the stream so far, the chunk last."""
    tok = np.asarray(tokens, dtype=np.int64)
    losses = []
    for _ in range(epochs):
        for first, n_ctx, end in training_samples(tok.size - n_chunk, n_chunk, L_T, batch):
            rate = warmup_lr(lr, opt["tau"], warmup_steps)
            res, lora, opt = chunk_update(tok[first:end], n_ctx, shape, emb, head, g_final, get_layer, lora, opt, rate,
                                          beta1, beta2, eps, wd, (), dropout, seed)
            losses.append(res["loss"])
    return losses, lora, opt


def linear_step(X, W, A, B, dY, s, lr, beta1=0.9, beta2=0.999, eps=1e-8, wd=0.0):
    """Single LoRA-adapted linear layer: forward, backward, first AdamW step on A and B."""
    Y, _ = lora_linear_fwd(X, W, A, B, s)
    dX, dA, dB = lora_linear_bwd(dY, X, W, A, B, s)
    z = np.zeros_like
    A1, _, _ = adamw_step(A, dA, z(_f(A)), z(_f(A)), 1, lr, beta1, beta2, eps, wd)
    B1, _, _ = adamw_step(B, dB, z(_f(B)), z(_f(B)), 1, lr, beta1, beta2, eps, wd)
    return {"Y": Y, "dX": dX, "dA": dA, "dB": dB, "A1": A1, "B1": B1}
