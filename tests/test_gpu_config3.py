"""Full-size parity: the 7B-shaped chunk update (32 layers, r = 64, 1024 tokens) in the launch configuration
bench.py times, against values the CPU oracle computed once for the same seeded inputs
(tests/golden/config3_7b_seed3000.npz, written by tests/golden/make_config3_golden.py, which calls only the
oracle).  The oracle needs ~14 minutes and ~30 GB for this size, so its loss, per-position nll and samples of
the gradients -- the hidden-state gradient at EVERY layer boundary, dB of every projection of every layer --
are stored; everything else is checked through properties that hold at any size
(B = 0  =>  dA == 0 exactly and A untouched; first AdamW step moves every B entry by lr).

Tolerances.  Loss, per-position nll, the gradient at the final norm and every tensor norm meet the bf16 bar
(2e-2).  Tensors that sit behind many layers cannot, whatever the kernels do: the same file stores, next to every
sample, the error that a bf16-boundary replay of the ORACLE (its fp64 arithmetic, rounded to bf16 / fp32 only where
the storage format of Section 3 "Setup" stores a tensor -- tests/bf16_floor.py, no kernel involved) has against
the fp64 oracle on that sample: 0.2 % at the final norm, 1.6 % one layer down, 6 % at layer 16, 8 % at layer 0 for dX
and 7-14 % for dB at every depth (Hs at layer l carries the forward rounding of l layers).  Each deep tensor is
therefore held to max(2e-2, 1.5 x its own stored floor).  A single 7B-shaped layer from exact inputs meets 2e-2 on
every output (test_config3_single_layer_full_shape)."""
import os

import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from paper_2401_11504_amd import synth  # noqa: E402
from test_gpu_kernels import BF16_TOL, check  # noqa: E402
from test_gpu_depth import floor_tol  # noqa: E402

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "config3_7b_seed3000.npz")
LR = 5e-5


def _cos(a, b):
    a, b = np.asarray(a, np.float64).ravel(), np.asarray(b, np.float64).ravel()
    return float(a @ b / (np.linalg.norm(a) * np.linalg.norm(b)))


def test_config3_full_update_matches_stored_oracle():
    from paper_2401_11504_amd import api, harness
    gold = np.load(GOLD)
    seed, T = int(gold["seed"]), 1024
    shape = synth.SHAPES["7b"]
    assert int(gold["n_layers"]) == shape.n_layers and int(gold["n_tokens"]) == T
    print("building the 7B-shaped synthetic model ...", flush=True)
    model = harness.Model(shape, seed, max_tokens=T, keep_host=False, workers=16)
    lora, facs = harness.new_lora(model, seed, b_std=0.0)
    tok = synth.uniform_tokens(seed, T, shape.vocab)
    assert np.array_equal(tok, gold["tokens"])                          # same input bytes on both sides
    print("chunk update ...", flush=True)
    loss, n = api.tl_chunk_update(lora, tok, 0, LR)
    assert n == int(gold["n_targets"]) == T - 1                        # integer work: exact
    assert abs(loss - float(gold["loss"])) <= BF16_TOL * float(gold["loss"]), (loss, float(gold["loss"]))
    assert abs(loss - float(gold["loss"])) <= 2e-3 * float(gold["loss"])   # in practice far tighter
    nll = api.tl_get_nll(lora, T)
    check(nll, gold["nll"], BF16_TOL, "per-position nll")
    assert nll[-1] == 0.0
    rows, cols = gold["dh_rows"], gold["dh_cols"]
    worst_dh = worst_db = 0.0
    for name, boundary in [("dh_final", shape.n_layers)] + [(f"dh_{l}", l) for l in reversed(range(shape.n_layers))]:
        dh = api.tl_get_dh(lora, boundary, T, shape.d_model)
        s = dh[np.ix_(rows, cols)]
        floor = gold["floor_" + name]
        check(s, gold[name], BF16_TOL if boundary == shape.n_layers else floor_tol(floor), name)
        worst_dh = max(worst_dh, np.linalg.norm(s - gold[name]) / np.linalg.norm(gold[name]) / float(floor[0]))
        norm_key = "dh_final_norm" if name == "dh_final" else f"dh_norm_{boundary}"
        assert abs(np.linalg.norm(dh.astype(np.float64)) - float(gold[norm_key])) <= BF16_TOL * float(gold[norm_key])
    for l in range(shape.n_layers):
        for i, p in enumerate(synth.PROJ):
            dout, din = shape.proj_dims(p)
            dA = api.tl_get_factor(lora, l, i, api.GRAD_A, (shape.rank, din))
            assert not dA.any(), f"dA l{l} {p} must be exactly zero while B = 0"
            assert np.array_equal(api.tl_get_factor(lora, l, i, api.FACTOR_A, (shape.rank, din)), facs[l][p][0])
            dB = api.tl_get_factor(lora, l, i, api.GRAD_B, (dout, shape.rank))
            r = gold[f"dB_rows_{l}_{i}"]
            floor = gold[f"floor_dB_{l}_{i}"]
            check(dB[r], gold[f"dB_{l}_{i}"], floor_tol(floor), f"dB l{l} {p} (sampled rows)")
            worst_db = max(worst_db, np.linalg.norm(dB[r] - gold[f"dB_{l}_{i}"]) / np.linalg.norm(gold[f"dB_{l}_{i}"]) / float(floor[0]))
            gn = float(gold[f"dB_norm_{l}_{i}"])
            assert abs(np.linalg.norm(dB.astype(np.float64)) - gn) <= BF16_TOL * gn, f"|dB| l{l} {p}"
            # AdamW step 1 from B = 0: every entry lands on -lr * sign(g) (closed form)
            B1 = api.tl_get_factor(lora, l, i, api.FACTOR_B, (dout, shape.rank))
            g = gold[f"dB_{l}_{i}"]
            big = np.abs(g) > 0.5 * np.sqrt(np.mean(g * g))   # well clear of the depth-amplified gradient noise
            assert np.mean(np.sign(B1[r][big]) == -np.sign(g[big])) > 0.999
            ga = np.abs(dB.astype(np.float64))
            assert np.allclose(np.abs(B1), LR * ga / (ga + 1e-8), rtol=1e-3, atol=1e-12)
            assert np.median(np.abs(B1)) > 0.9 * LR
    print(f"largest GPU error / storage floor on the samples: dX {worst_dh:.3f}, dB {worst_db:.3f}", flush=True)
    assert api.tl_get_step(lora) == 1
    # second epoch on the same chunk: the loss must go down (B is no longer 0, dA becomes non-zero)
    loss2, _ = api.tl_chunk_update(lora, tok, 0, LR)
    assert loss2 < loss
    assert api.tl_get_factor(lora, 5, 0, api.GRAD_A, (shape.rank, shape.d_model)).any()
    api.tl_discard(lora)
    api.tl_lora_free(lora)
    model.close()


def test_config3_single_layer_full_shape():
    """One decoder layer at the 7B shape (d 4096, 32x128 heads, ffn 11008, r = 64, 1024 tokens) from exact
    seeded inputs: every output within the bf16 tolerance of the oracle computed here."""
    from oracle import templora_oracle as O
    from paper_2401_11504_amd import api, harness
    shape = synth.SHAPES["7b"].with_layers(1)
    T, seed = 1024, 3100
    model = harness.Model(shape, seed, max_tokens=T)
    lora, facs = harness.new_lora(model, seed, b_std=0.01)
    h = synth.hidden(seed, T, shape.d_model)
    dy = synth.upstream_grad(seed, T, shape.d_model)
    h_out = torch.zeros(T, shape.d_model, device="cuda")
    dh_in = torch.zeros(T, shape.d_model, device="cuda")
    api.tl_layer_step(lora, 0, harness.to_dev_f32(h), harness.to_dev_f32(dy), h_out, dh_in, LR, False)
    W = model.host_layers[0]
    ref_out, cache = O.layer_fwd(h, W, facs[0], shape)
    ref_dh, G = O.layer_bwd(dy, cache, W, facs[0], shape)
    check(h_out.cpu().numpy(), ref_out, BF16_TOL, "h_out")
    check(dh_in.cpu().numpy(), ref_dh, BF16_TOL, "dh_in")
    for i, p in enumerate(synth.PROJ):
        dout, din = shape.proj_dims(p)
        check(api.tl_get_factor(lora, 0, i, api.GRAD_A, (shape.rank, din)), G[p][0], BF16_TOL, f"dA {p}")
        check(api.tl_get_factor(lora, 0, i, api.GRAD_B, (dout, shape.rank)), G[p][1], BF16_TOL, f"dB {p}")
    api.tl_lora_free(lora)
    model.close()
