"""LoRA dropout (Section 3 "Setup": dropout 0.05) through the C ABI against the oracle: the mask itself bit for bit,
then one layer and whole updates with the masks both sides derive from (seed, step, layer, group)."""
import os
import sys

import numpy as np
import pytest
import torch

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))

from oracle import templora_oracle as O  # noqa: E402
from paper_2401_11504_amd import synth  # noqa: E402
from test_gpu_kernels import BF16_TOL, H, api, check, rnd  # noqa: E402,F401

pytestmark = pytest.mark.gpu
PROJ = synth.PROJ
LR = 5e-5


@pytest.mark.parametrize("T,d_in,p,seed,step,layer,group", [
    (37, 264, 0.05, 1, 0, 0, 0), (5, 8, 0.5, 2 ** 63 + 12345, 70000, 31, 3), (1024, 11008, 0.05, 77, 3, 17, 3),
    (333, 4096, 0.999, 9, 1, 2, 1), (64, 512, 0.0, 9, 1, 2, 1)])
def test_dropout_mask_is_bit_exact(api, H, T, d_in, p, seed, step, layer, group):
    x = rnd(seed % 1000, (T, d_in))
    x[x == 0] = 1.0                                    # so that a zero in the output can only be a dropped element
    xd = H.to_dev_bf16(x)
    y = torch.empty_like(xd)
    api.tl_k_dropout(xd, y, p, seed, step, layer, group)
    torch.cuda.synchronize()
    got = H.bf16_to_np(y)
    D = O.dropout_factor(seed, step, layer, group, T, d_in, p)
    assert np.array_equal(got == 0, D == 0)            # which elements fall: integer work, exact
    xb = H.bf16_to_np(xd)                             # the bf16 values the kernel read
    keep = D != 0
    # kept values: x / (1 - p) in fp32, rounded to bf16 (half an ulp = 2^-9 relative)
    assert np.all(np.abs(got[keep] - xb[keep] * D[keep]) <= 2.0 ** -8 * np.abs(xb[keep] * D[keep]))
    if p == 0.0:
        assert np.array_equal(got, xb)


@pytest.mark.parametrize("name,T,p", [("small", 200, 0.05), ("small128", 333, 0.25), ("layer", 1024, 0.05)])
def test_layer_step_with_dropout(api, H, name, T, p):
    shape = synth.SHAPES[name].with_layers(1)
    seed = 6100
    model = H.Model(shape, seed, max_tokens=T)
    lora, facs = H.new_lora(model, seed, b_std=0.01, dropout=p)
    h = synth.hidden(seed, T, shape.d_model)
    dy = synth.upstream_grad(seed, T, shape.d_model)
    h_out = torch.zeros(T, shape.d_model, device="cuda")
    dh_in = torch.zeros(T, shape.d_model, device="cuda")
    W = model.host_layers[0]
    for step in range(2):                              # the second call must draw the masks of step 1
        api.tl_layer_step(lora, 0, H.to_dev_f32(h), H.to_dev_f32(dy), h_out, dh_in, 0.0, True)
        D = O.layer_dropout((p, seed, step), shape, 0, T)
        ref_out, cache = O.layer_fwd(h, W, facs[0], shape, 0, D)
        ref_dh, G = O.layer_bwd(dy, cache, W, facs[0], shape)
        check(h_out.cpu().numpy(), ref_out, BF16_TOL, f"h_out step {step}")
        check(dh_in.cpu().numpy(), ref_dh, BF16_TOL, f"dh_in step {step}")
        for i, pj in enumerate(PROJ):
            dout, din = shape.proj_dims(pj)
            check(api.tl_get_factor(lora, 0, i, api.GRAD_A, (shape.rank, din)), G[pj][0], BF16_TOL, f"dA {pj} step {step}")
            check(api.tl_get_factor(lora, 0, i, api.GRAD_B, (dout, shape.rank)), G[pj][1], BF16_TOL, f"dB {pj} step {step}")
        if step == 0:
            first = h_out.cpu().numpy().copy()
        else:
            assert not np.array_equal(first, h_out.cpu().numpy())      # lr = 0: only the masks changed
    api.tl_lora_free(lora)
    model.close()


@pytest.mark.parametrize("name,T,n_ctx,p", [("small", 200, 0, 0.05), ("small", 256, 100, 0.05), ("small128", 130, 0, 0.3)])
def test_chunk_update_with_dropout_matches_oracle(api, H, name, T, n_ctx, p):
    shape = synth.SHAPES[name]
    seed = 6200
    model = H.Model(shape, seed, max_tokens=T)
    lora, facs = H.new_lora(model, seed, b_std=0.01, dropout=p)
    tok = synth.uniform_tokens(seed, T, shape.vocab)
    args = (shape, model.emb, model.head, np.ones(shape.d_model), lambda l: model.host_layers[l])
    opt = O.new_opt_state(facs)
    for step in range(2):
        loss, n = api.tl_chunk_update(lora, tok, n_ctx, LR)
        old = facs
        res, facs, opt = O.chunk_update(tok, n_ctx, *args, facs, opt, LR, keep=range(shape.n_layers), dropout=p, seed=seed)
        assert n == res["n_targets"]
        assert abs(loss - res["loss"]) <= BF16_TOL * abs(res["loss"])
        check(api.tl_get_nll(lora, T), res["nll"], BF16_TOL, "nll")
        for l in range(shape.n_layers):
            check(api.tl_get_dh(lora, l, T, shape.d_model), res["dh"][l], BF16_TOL, f"dh layer {l} step {step}")
            for i, pj in enumerate(PROJ):
                dout, din = shape.proj_dims(pj)
                check(api.tl_get_factor(lora, l, i, api.GRAD_A, (shape.rank, din)), res["grads"][l][pj][0], BF16_TOL,
                      f"dA l{l} {pj} step {step}")
                check(api.tl_get_factor(lora, l, i, api.GRAD_B, (dout, shape.rank)), res["grads"][l][pj][1], BF16_TOL,
                      f"dB l{l} {pj} step {step}")
        if step == 0:
            # scoring runs without dropout: the loss of the updated module equals the oracle's plain forward
            score, _ = api.tl_chunk_loss(lora, tok, n_ctx)
            plain = O.model_fwd_bwd(tok, n_ctx, *args, facs)["loss"]
            assert abs(score - plain) <= BF16_TOL * plain
            assert abs(plain - res["loss"]) > 1e-7 or p == 0
        # carry the GPU's own factors into the oracle so that the second step compares like with like
        facs = [{pj: (api.tl_get_factor(lora, l, i, api.FACTOR_A, (shape.rank, shape.proj_dims(pj)[1])).astype(np.float64),
                      api.tl_get_factor(lora, l, i, api.FACTOR_B, (shape.proj_dims(pj)[0], shape.rank)).astype(np.float64))
                 for i, pj in enumerate(PROJ)} for l in range(shape.n_layers)]
        del old
    assert api.tl_get_step(lora) == 2
    api.tl_lora_free(lora)
    model.close()


def test_dropout_zero_is_bit_identical_to_the_default_path_and_bad_rates_are_rejected(api, H):
    shape = synth.SHAPES["small"]
    model = H.Model(shape, 6300, max_tokens=96)
    tok = synth.uniform_tokens(6300, 96, shape.vocab)
    la, _ = H.new_lora(model, 6300, b_std=0.01)
    lb, _ = H.new_lora(model, 6300, b_std=0.01, dropout=0.0)
    assert api.tl_chunk_update(la, tok, 0, LR) == api.tl_chunk_update(lb, tok, 0, LR)
    for i, pj in enumerate(PROJ):
        dout, din = shape.proj_dims(pj)
        assert np.array_equal(api.tl_get_factor(la, 0, i, api.FACTOR_B, (dout, shape.rank)),
                              api.tl_get_factor(lb, 0, i, api.FACTOR_B, (dout, shape.rank)))
    for bad in (-0.1, 1.0, float("nan")):
        with pytest.raises(api.TlError) as e:
            api.tl_lora_init(model.handle, shape.rank, shape.alpha, dropout=bad)
        assert e.value.status == -1
    for h in (la, lb):
        api.tl_lora_free(h)
    model.close()
