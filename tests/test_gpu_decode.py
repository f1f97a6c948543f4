"""Generation side of Algorithm 1 (greedy decoding with the temporary module over a key/value cache) against the
oracle, which recomputes the whole window for every token (no cache): logits to the bf16 tolerance at every step, the
chosen token wherever the oracle's two best logits are further apart than that tolerance allows to confuse, cache
consistency on the GPU itself, and the error paths."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from oracle import templora_oracle as O  # noqa: E402
from paper_2401_11504_amd import synth  # noqa: E402
from test_gpu_kernels import BF16_TOL, H, api, check, rnd  # noqa: E402,F401


# ------------------------------------------------------------------ kernels
@pytest.mark.parametrize("N,K,r,G", [(64, 64, 0, 1), (1000, 4096, 16, 1), (3 * 256, 256, 8, 3), (776, 11008, 64, 1),
                                     (192, 4096, 64, 3), (512, 11008, 16, 1), (516, 256, 8, 1), (1, 8, 0, 1)])
def test_gemv_with_lora_term(api, H, N, K, r, G):
    W, x = rnd(1, (N, K), 0.05), rnd(2, (1, K))[0]
    ref = W.astype(np.float64) @ x.astype(np.float64)
    lb = lh = None
    if r:
        lb = rnd(3, (N, r), 0.05)
        lh = rnd(4, (G, r), 1.0, False)
        rows = N // G
        ref = ref + np.concatenate([lb[g * rows:(g + 1) * rows].astype(np.float64) @ lh[g].astype(np.float64) for g in range(G)])
    res = rnd(5, (1, N), 1.0, False)[0]
    y32 = torch.empty(N, dtype=torch.float32, device="cuda")
    ybf = torch.empty(N, dtype=torch.bfloat16, device="cuda")
    args = dict(lora_b=H.to_dev_bf16(lb) if r else None, lora_h=H.to_dev_f32(lh.reshape(-1)) if r else None, rows_per_group=N // G)
    api.tl_k_gemv(H.to_dev_bf16(W), H.to_dev_bf16(x), y32, alpha=0.5, resid=H.to_dev_f32(res), **args)
    api.tl_k_gemv(H.to_dev_bf16(W), H.to_dev_bf16(x), ybf, alpha=1.0, **args)
    torch.cuda.synchronize()
    check(y32.cpu().numpy(), 0.5 * ref + res, 1e-4, "y fp32 + resid")      # bf16 products are exact; fp32 sums
    check(H.bf16_to_np(ybf), ref, BF16_TOL, "y bf16")


@pytest.mark.parametrize("N,K", [(64, 4096), (192, 264), (1000, 4096), (128, 11008)])
def test_gemv_with_norm_and_swiglu_prologues(api, H, N, K):
    """The input vector formed inside the launch: RMSNorm of an fp32 row, SwiGLU of a gate|up row."""
    W = rnd(1, (N, K), 0.05)
    h, gain = rnd(2, (1, K), 2.0, False), 1.0 + rnd(3, (1, K), 0.1, False)[0]
    gu = rnd(4, (1, 2 * K), 1.5)
    y = torch.empty(N, dtype=torch.float32, device="cuda")
    xo = torch.empty(K, dtype=torch.bfloat16, device="cuda")
    api.tl_k_gemv_pre(H.to_dev_bf16(W), y, 1, h=H.to_dev_f32(h[0]), gain=H.to_dev_f32(gain), eps=1e-5, x_out=xo)
    torch.cuda.synchronize()
    x_ref = O.rmsnorm_fwd(h, gain, 1e-5)[0]
    check(H.bf16_to_np(xo), x_ref, BF16_TOL, "x (norm)")
    # the product is taken with the bf16-rounded vector the kernel stored, so that only the summation differs
    check(y.cpu().numpy(), W.astype(np.float64) @ H.bf16_to_np(xo).astype(np.float64), 1e-4, "y (norm)")
    api.tl_k_gemv_pre(H.to_dev_bf16(W), y, 2, gu=H.to_dev_bf16(gu[0]), x_out=xo)
    torch.cuda.synchronize()
    a_ref = O.swiglu_fwd(gu[:, :K], gu[:, K:])[0]
    check(H.bf16_to_np(xo), a_ref, BF16_TOL, "x (swiglu)")
    check(y.cpu().numpy(), W.astype(np.float64) @ H.bf16_to_np(xo).astype(np.float64), 1e-4, "y (swiglu)")


@pytest.mark.parametrize("ws_splits", [0, 32, 3])      # no scratch (one workgroup per head); full scratch; a short one
@pytest.mark.parametrize("n_keys,nh,dh", [(1, 2, 64), (77, 3, 64), (129, 2, 64), (384, 2, 64), (1000, 4, 64), (1024, 2, 128),
                                          (2048, 1, 128), (3000, 2, 128)])
def test_attention_decode_is_last_row_of_causal_attention(api, H, n_keys, nh, dh, ws_splits):
    d = nh * dh
    qkv = rnd(1, (n_keys, 3 * d), 1.0)
    q, k, v = (qkv[:, i * d:(i + 1) * d].reshape(n_keys, nh, dh) for i in range(3))
    ro, _ = O.attention_fwd(q, k, v)
    dev = H.to_dev_bf16(qkv)
    o = torch.zeros(d, dtype=torch.bfloat16, device="cuda")
    ws = torch.zeros(nh * ws_splits * (dh + 2), device="cuda") if ws_splits else None
    api.tl_k_attention_decode(dev[n_keys - 1, :d], dev[:, d:2 * d], dev[:, 2 * d:], nh, dh, o, ws)
    torch.cuda.synchronize()
    check(H.bf16_to_np(o), ro[-1].reshape(d), BF16_TOL, "o")


def test_argmax_lowest_index_among_equals(api, H):
    x = rnd(1, (1, 32000), 1.0, False)[0]
    x[[17, 4000, 31999]] = x.max() + 1.0          # three equal maxima
    out = torch.zeros(1, dtype=torch.int32, device="cuda")
    api.tl_k_argmax(H.to_dev_f32(x), out)
    assert int(out.item()) == 17                   # integer work: exact
    x[5] = np.inf
    api.tl_k_argmax(H.to_dev_f32(x), out)
    assert int(out.item()) == 5


# ------------------------------------------------------------------ prefill + decode against the oracle
def _oracle_args(model, facs):
    shape = model.shape
    return (shape, model.emb, model.head, np.ones(shape.d_model), lambda l: model.host_layers[l], facs)


@pytest.mark.parametrize("name,n_prompt,n_new", [("small", 37, 12), ("small128", 130, 8), ("small", 420, 4)])
def test_prefill_and_decode_follow_the_oracle(api, H, name, n_prompt, n_new):
    shape = synth.SHAPES[name]
    seed = 4100
    model = H.Model(shape, seed, max_tokens=n_prompt + n_new + 1)
    lora, facs = H.new_lora(model, seed, b_std=0.01)
    prompt = synth.zipf_tokens(seed, n_prompt, shape.vocab)
    seq = [int(t) for t in prompt]
    nxt, logits = api.tl_prefill(lora, prompt, shape.vocab)
    assert api.tl_kv_length(lora) == n_prompt
    for step in range(n_new + 1):
        ref_next, ref = O.greedy_next(seq, *_oracle_args(model, facs))
        check(logits, ref, BF16_TOL, f"logits at step {step}")
        assert nxt == int(np.argmax(logits))                               # the GPU's own argmax: exact
        top = np.sort(ref)[-2:]
        if top[1] - top[0] > 4 * BF16_TOL * np.sqrt(np.mean(ref * ref)):    # unambiguous for a bf16 path
            assert nxt == ref_next, f"step {step}"
        if step == n_new:
            break
        seq.append(nxt)                                                    # teacher forcing with the GPU's choice
        nxt, logits = api.tl_decode_step(lora, nxt, shape.vocab)
        assert api.tl_kv_length(lora) == len(seq)
    # the cache is what a fresh prefill of the same window computes
    nxt2, logits2 = api.tl_prefill(lora, np.array(seq, np.int32), shape.vocab)
    check(logits2, logits, 1e-2, "cached decode vs prefill of the whole window")
    api.tl_lora_free(lora)
    model.close()


def test_decode_lifecycle_and_errors(api, H):
    shape = synth.SHAPES["small"]
    model = H.Model(shape, 4200, max_tokens=16)
    lora, _ = H.new_lora(model, 4200, b_std=0.01)
    tok = synth.uniform_tokens(4200, 12, shape.vocab)
    with pytest.raises(api.TlError) as e:
        api.tl_decode_step(lora, 1)
    assert e.value.status == -1                                # no cache yet
    with pytest.raises(api.TlError) as e:
        api.tl_prefill(lora, np.arange(17) % shape.vocab)
    assert e.value.status == -4
    with pytest.raises(api.TlError) as e:
        api.tl_prefill(lora, np.array([0, shape.vocab]))
    assert e.value.status == -3
    nxt, _ = api.tl_prefill(lora, tok)
    for _ in range(4):
        nxt, _ = api.tl_decode_step(lora, nxt)
    assert api.tl_kv_length(lora) == 16
    with pytest.raises(api.TlError) as e:
        api.tl_decode_step(lora, nxt)
    assert e.value.status == -4                             # window full
    # an update invalidates the cache (the paper recomputes it with the new module)
    api.tl_chunk_update(lora, tok, 0, 5e-5)
    assert api.tl_kv_length(lora) == 0
    with pytest.raises(api.TlError) as e:
        api.tl_decode_step(lora, 1)
    assert e.value.status == -1
    # the updated module changes the continuation's logits; a second prefill is deterministic
    a1, l1 = api.tl_prefill(lora, tok, shape.vocab)
    a2, l2 = api.tl_prefill(lora, tok, shape.vocab)
    assert a1 == a2 and np.array_equal(l1, l2)
    api.tl_discard(lora)
    with pytest.raises(api.TlError) as e:
        api.tl_prefill(lora, tok)
    assert e.value.status == -7
    api.tl_lora_free(lora)
    model.close()


def test_algorithm1_stream_decode_then_update(api, H):
    """Algorithm 1 end to end at a small size: decode a chunk greedily over the window, train the module on
    (preceding L_T tokens -> chunk) for two epochs, rebuild the cache from the last L_X tokens with the updated module,
    and go on.  The oracle replays the same token stream (teacher forcing with the GPU's choices) with its own module
    and AdamW state, so every step's logits are compared under an independently evolved module."""
    shape = synth.SHAPES["small"]
    seed, L_X, L_T, DELTA, N_CHUNKS, EPOCHS, lr = 4300, 24, 24, 16, 2, 2, 5e-5
    model = H.Model(shape, seed, max_tokens=L_X + DELTA)
    lora, facs = H.new_lora(model, seed, b_std=0.01)
    args = lambda f: (shape, model.emb, model.head, np.ones(shape.d_model), lambda l: model.host_layers[l], f)
    opt = O.new_opt_state(facs)
    stream = [int(t) for t in synth.zipf_tokens(seed, L_X, shape.vocab)]
    for k in range(N_CHUNKS):
        window = stream[-L_X:]
        nxt, logits = api.tl_prefill(lora, np.array(window, np.int32), shape.vocab)
        for i in range(DELTA):
            _, ref = O.greedy_next(window, *args(facs))
            check(logits, ref, BF16_TOL, f"chunk {k} token {i}")
            window.append(nxt)
            stream.append(nxt)
            if i + 1 < DELTA:
                nxt, logits = api.tl_decode_step(lora, nxt, shape.vocab)
        sample = np.array(stream[-(L_T + DELTA):], np.int32)               # X_T followed by the chunk
        for e in range(EPOCHS):
            loss, n = api.tl_chunk_update(lora, sample, L_T, lr)
            res, facs, opt = O.chunk_update(sample, L_T, *args(facs)[:5], facs, opt, lr)
            assert n == res["n_targets"] == DELTA
            assert abs(loss - res["loss"]) <= BF16_TOL * res["loss"], (k, e, loss, res["loss"])
        assert api.tl_kv_length(lora) == 0                                 # the cache must be rebuilt with the new module
    assert api.tl_get_step(lora) == N_CHUNKS * EPOCHS
    api.tl_discard(lora)
    api.tl_lora_free(lora)
    model.close()


def _gpu_factors(api, lora, shape):
    return [{p: (api.tl_get_factor(lora, l, i, api.FACTOR_A, (shape.rank, shape.proj_dims(p)[1])).astype(np.float64),
                 api.tl_get_factor(lora, l, i, api.FACTOR_B, (shape.proj_dims(p)[0], shape.rank)).astype(np.float64))
             for i, p in enumerate(synth.PROJ)} for l in range(shape.n_layers)]


def test_cache_reuse_decodes_over_the_old_modules_keys_and_values(api, H):
    """Section 2's cache reuse: after an update the cached keys and values stay (computed by the module as it was),
    new positions use the updated module.  The learning rate is large on purpose, so that the two modules differ by
    far more than the tolerance and reuse is distinguishable from recomputing."""
    shape = synth.SHAPES["small"]
    seed, n_prompt, n_new = 4400, 40, 5
    model = H.Model(shape, seed, max_tokens=n_prompt + n_new + 1)
    lora, facs_old = H.new_lora(model, seed, b_std=0.01)
    base = (shape, model.emb, model.head, np.ones(shape.d_model), lambda l: model.host_layers[l])
    prompt = synth.zipf_tokens(seed, n_prompt, shape.vocab)
    api.tl_cache_reuse(lora, True)
    nxt, _ = api.tl_prefill(lora, prompt)
    api.tl_chunk_update(lora, prompt, 0, 2e-2)
    assert api.tl_kv_length(lora) == n_prompt                   # the cache survived the update
    facs_new = _gpu_factors(api, lora, shape)                   # the module the GPU now holds, for like with like
    seq = [int(t) for t in prompt]
    for step in range(n_new):
        seq.append(nxt)
        nxt, logits = api.tl_decode_step(lora, seq[-1], shape.vocab)
        ref = O.window_logits_reuse(seq, n_prompt, *base, facs_old, facs_new)[-1]
        check(logits, ref, BF16_TOL, f"reuse logits at step {step}")
        fresh = O.window_logits(seq, *base, facs_new)[-1]
        assert np.linalg.norm(ref - fresh) > 10 * BF16_TOL * np.linalg.norm(ref)     # recomputing would be different
    # the paper's default is one call away: a prefill rebuilds the cache with the current module
    nxt2, logits2 = api.tl_prefill(lora, np.array(seq, np.int32), shape.vocab)
    check(logits2, O.window_logits(seq, *base, facs_new)[-1], BF16_TOL, "prefill after reuse")
    api.tl_cache_reuse(lora, False)
    assert api.tl_kv_length(lora) == 0
    api.tl_lora_free(lora)
    model.close()


def test_cache_reuse_switched_on_after_a_prefill_keeps_the_cache(api, H):
    shape = synth.SHAPES["small"]
    seed, n_prompt = 4500, 33
    model = H.Model(shape, seed, max_tokens=n_prompt + 4)
    la, _ = H.new_lora(model, seed, b_std=0.01)
    lb, _ = H.new_lora(model, seed, b_std=0.01)
    prompt = synth.zipf_tokens(seed, n_prompt, shape.vocab)
    na, _ = api.tl_prefill(la, prompt)
    nb, _ = api.tl_prefill(lb, prompt)
    api.tl_cache_reuse(lb, True)                                # moves the existing cache into its own buffers
    assert na == nb and api.tl_kv_length(lb) == n_prompt
    for _ in range(3):
        na, xa = api.tl_decode_step(la, na, shape.vocab)
        nb, xb = api.tl_decode_step(lb, nb, shape.vocab)
        assert na == nb and np.array_equal(xa, xb)              # same kernels on the same values: bit-identical
    for h in (la, lb):
        api.tl_lora_free(h)
    model.close()


def test_generate_is_algorithm1_made_of_the_same_calls(api, H):
    """tl_generate against the same loop written out with tl_prefill / tl_decode_step / tl_chunk_train on a second
    module: identical kernels on identical values, so tokens and losses must agree bit for bit (the loop itself is
    checked against the oracle in test_algorithm1_stream_decode_then_update)."""
    shape = synth.SHAPES["small"]
    seed, L_X, L_T, DELTA, n_new, lr = 4600, 20, 12, 8, 21, 2e-3        # two full chunks and a tail of five tokens
    model = H.Model(shape, seed, max_tokens=L_X + DELTA)
    la, _ = H.new_lora(model, seed, b_std=0.01)
    lb, _ = H.new_lora(model, seed, b_std=0.01)
    prompt = [int(t) for t in synth.zipf_tokens(seed, 30, shape.vocab)]
    toks, losses = api.tl_generate(la, prompt, n_new, L_X, DELTA, n_ctx_max=L_T, batch=4, epochs=2, lr=lr, warmup_steps=3)
    text, want_tok, want_loss = list(prompt), [], []
    while len(want_tok) < n_new:
        nxt, _ = api.tl_prefill(lb, np.array(text[-L_X:], np.int32))
        got = 0
        while got < DELTA and len(want_tok) < n_new:
            text.append(nxt)
            want_tok.append(nxt)
            got += 1
            if got < DELTA and len(want_tok) < n_new:
                nxt, _ = api.tl_decode_step(lb, nxt)
        if got < DELTA:
            break
        want_loss += api.tl_chunk_train(lb, np.array(text[-(L_T + DELTA):], np.int32), DELTA, L_T, 4, 2, lr, 3)
    assert list(toks) == want_tok
    assert losses == want_loss and len(losses) == 2 * 2 * 2            # two chunks x two epochs x two pieces
    assert api.tl_get_step(la) == api.tl_get_step(lb) == 8
    # geometry errors come before anything runs
    for kwargs, code in ((dict(window=L_X + 1, chunk=DELTA), -4), (dict(window=L_X, chunk=DELTA, n_ctx_max=L_X + DELTA), -4),
                         (dict(window=0, chunk=DELTA), -1)):
        with pytest.raises(api.TlError) as e:
            api.tl_generate(la, prompt, 4, **kwargs)
        assert e.value.status == code
    assert api.tl_get_step(la) == 8
    for h in (la, lb):
        api.tl_lora_free(h)
    model.close()


def test_error_paths_of_the_measurement_and_cache_calls(api, H):
    shape = synth.SHAPES["small"]
    model = H.Model(shape, 4700, max_tokens=32)
    lora, _ = H.new_lora(model, 4700, b_std=0.01)
    # dropout kernel arguments
    x = torch.zeros(4, 16, dtype=torch.bfloat16, device="cuda")
    for kw in (dict(p=1.0), dict(p=-0.1), dict(group=4), dict(step=-1)):
        a = dict(p=0.1, seed=1, step=0, layer=0, group=0)
        a.update(kw)
        with pytest.raises(api.TlError) as e:
            api.tl_k_dropout(x, torch.empty_like(x), **a)
        assert e.value.status == -1
    # cache reuse on a discarded module
    api.tl_cache_reuse(lora, True)
    api.tl_cache_reuse(lora, True)          # idempotent
    api.tl_discard(lora)
    for fn in (lambda: api.tl_cache_reuse(lora, True), lambda: api.tl_generate(lora, [1, 2], 4, 8, 8)):
        with pytest.raises(api.TlError) as e:
            fn()
        assert e.value.status == -7
    api.tl_lora_free(lora)
    model.close()
