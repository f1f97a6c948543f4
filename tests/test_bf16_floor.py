"""The bf16-boundary replay of the oracle (tests/bf16_floor.py) is what the deep GPU tests take their bounds from, so it
is pinned here, on the CPU: with every rounding switched off it must BE the oracle (a wiring mistake cannot hide as
"rounding error"); with the roundings on it must stay within the bf16 bar on a shallow model; each rounding it applies
is the nearest bf16 / fp32 value; and the floors stored next to the deep expected values must look like what they
claim to be (finite, positive, growing with depth for the hidden-state gradient)."""
import glob
import os

import numpy as np

import bf16_floor as F
from oracle import templora_oracle as O
from paper_2401_11504_amd import synth

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _case(name, T, seed, n_ctx, b_std=0.01):
    shape = synth.SHAPES[name]
    tok = synth.zipf_tokens(seed, T, shape.vocab)
    emb, head = synth.embedding(seed, shape), synth.lm_head(seed, shape)
    lora = [synth.lora_factors(seed, shape, l, b_std=b_std) for l in range(shape.n_layers)]
    W = [synth.layer_weights(seed, shape, l) for l in range(shape.n_layers)]
    return shape, tok, n_ctx, emb, head, np.ones(shape.d_model), (lambda l: W[l]), lora


def test_replay_without_rounding_is_the_oracle():
    for name, T, n_ctx in (("tiny", 24, 0), ("small", 40, 7)):
        shape, tok, n_ctx, emb, head, g, get, lora = _case(name, T, 7, n_ctx)
        ref = O.model_fwd_bwd(tok, n_ctx, shape, emb, head, g, get, lora, keep=range(shape.n_layers))
        rep = F.model_fwd_bwd(tok, n_ctx, shape, emb, head, g, get, lora, keep=range(shape.n_layers), exact=True)
        assert rep["loss"] == ref["loss"] and rep["n_targets"] == ref["n_targets"]
        assert np.array_equal(rep["nll"], ref["nll"])
        for k in ref["dh"]:
            assert np.allclose(rep["dh"][k], ref["dh"][k], rtol=1e-12, atol=1e-300), k
        for l in range(shape.n_layers):
            for p in O.PROJ:
                for i in (0, 1):
                    assert np.allclose(rep["grads"][l][p][i], ref["grads"][l][p][i], rtol=1e-11, atol=1e-300), (l, p, i)


def test_replay_with_rounding_meets_the_bf16_bar_on_a_shallow_model():
    shape, tok, n_ctx, emb, head, g, get, lora = _case("small", 64, 11, 0)
    ref = O.model_fwd_bwd(tok, n_ctx, shape, emb, head, g, get, lora, keep=range(shape.n_layers))
    for inner in (False, True):
        rep = F.model_fwd_bwd(tok, n_ctx, shape, emb, head, g, get, lora, keep=range(shape.n_layers), inner=inner)
        assert 0 < abs(rep["loss"] - ref["loss"]) <= 2e-3 * ref["loss"]
        errs = [F.rel_err(rep["dh"][k], ref["dh"][k]) for k in ref["dh"]]
        errs += [F.rel_err(rep["grads"][l][p][i], ref["grads"][l][p][i])
                 for l in range(shape.n_layers) for p in O.PROJ for i in (0, 1)]
        assert 1e-4 < max(errs) <= 2e-2, max(errs)        # rounded somewhere, and within the bf16 tolerance


def test_rounding_helpers_are_nearest_even():
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 2.0 ** -7, 1.0 + 3 * 2.0 ** -8, -0.02, 3.0e38, 1e-30])
    y = F.round_bf16(x)
    # bf16 keeps 8 significant bits: 1 + 2^-8 is a tie and goes to the even neighbour 1, 1 + 3 * 2^-8 to 1 + 2^-6
    assert y[0] == 1.0 and y[1] == 1.0 and y[2] == 1.0 + 2.0 ** -7 and y[3] == 1.0 + 2.0 ** -6
    assert np.all(np.abs(y - x) <= np.abs(x) * 2.0 ** -8)
    bits = np.asarray(y, np.float32).view(np.uint32)
    assert np.all(bits & 0xFFFF == 0)                      # representable in bf16
    assert np.array_equal(F.round_f32(x), x.astype(np.float32).astype(np.float64))


def test_replay_chunk_train_makes_the_oracles_steps():
    """Same samples, same warm-up, same step count as oracle.chunk_train; losses within the bf16 bar."""
    shape, tok, _, emb, head, g, get, lora = _case("tiny", 40, 5, 0)
    a = O.chunk_train(tok, 24, 8, 8, 2, 1e-3, 3, shape, emb, head, g, get, lora, O.new_opt_state(lora))
    b = F.chunk_train(tok, 24, 8, 8, 2, 1e-3, 3, shape, emb, head, g, get, lora, O.new_opt_state(lora))
    assert len(a[0]) == len(b[0]) == 6 and a[2]["tau"] == b[2]["tau"] == 6
    assert np.allclose(a[0], b[0], rtol=2e-2)


def test_stored_floors_are_sane():
    files = sorted(glob.glob(os.path.join(GOLDEN, "*.npz")))
    assert files
    seen = 0
    for f in files:
        g = np.load(f)
        keys = [k for k in g.files if k.startswith("floor_")]
        for k in keys:
            v = np.asarray(g[k], np.float64)
            assert np.all(np.isfinite(v)) and np.all(v >= 0), (f, k)
            seen += 1
        if "floor_dh_0" in g.files and "floor_dh_final" in g.files:
            # rounding noise is amplified on its way down: the bottom boundary's floor exceeds the top one's
            assert g["floor_dh_0"][0] > g["floor_dh_final"][0], f
    assert seen > 500
    deep = np.load(os.path.join(GOLDEN, "config3_7b_seed3000.npz"))
    fl = np.array([deep[f"floor_dh_{l}"][0] for l in range(32)])
    assert fl[0] > 0.05 and fl[31] < 0.03 and np.all(np.diff(fl[::4]) < 0)     # 8 % at the bottom, 1.6 % one layer down
