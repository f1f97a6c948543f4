#!/usr/bin/env python3
"""Writes tests/golden/config3_7b_seed3000.npz: the CPU oracle's results for the full 7B-shaped chunk update.

Calls only oracle/ and the seeded input generator.  The paper prints no numbers for one update, so these
are the pinned oracle's values on the synthetic workload (32 layers, d 4096, 32x128 heads, ffn 11008,
vocab 32000, LoRA r=64 alpha=64 with A ~ N(0, 0.02^2), B = 0, 1024 uniform token ids, seed 3000):
loss, n_targets, per-position nll, and samples of dB (whose sign decides the first AdamW step) and of the
hidden-state gradients at the layer boundaries 0, 16, 31 and at the final norm.

    python tests/golden/make_config3_golden.py          (about 64 GB of host memory is NOT needed: layers are
                                                          generated on demand and caches are fp64, ~30 GB peak)
"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import templora_oracle as O  # noqa: E402
from paper_2401_11504_amd import synth  # noqa: E402

SEED, T = 3000, 1024
OUT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "config3_7b_seed3000.npz")
SAMPLE_ROWS = 8      # rows of each sampled dB
SAMPLE_DH_ROWS = 4   # rows and
SAMPLE_DH_COLS = 256  # columns of each sampled hidden-state gradient


def main(n_layers=32):
    shape = synth.SHAPES["7b"].with_layers(n_layers)
    tok = synth.uniform_tokens(SEED, T, shape.vocab)
    emb, head = synth.embedding(SEED, shape), synth.lm_head(SEED, shape)
    lora = [synth.lora_factors(SEED, shape, l) for l in range(shape.n_layers)]
    cache = {}

    def get_layer(l):
        # forward visits 0..L-1 then backward L-1..0: keep only the layer in use
        if l not in cache:
            cache.clear()
            cache[l] = synth.layer_weights(SEED, shape, l)
        return cache[l]

    t0 = time.time()
    keep = sorted({0, shape.n_layers // 2, shape.n_layers - 1})
    res = O.model_fwd_bwd(tok, 0, shape, emb, head, np.ones(shape.d_model), get_layer, lora, keep=keep)
    print(f"oracle forward+backward: {time.time() - t0:.1f} s, loss {res['loss']:.6f}", flush=True)
    rs = np.random.default_rng(SEED)
    f32 = lambda x: np.asarray(x, dtype=np.float32)
    out = {"loss": np.float64(res["loss"]), "n_targets": np.int64(res["n_targets"]), "nll": f32(res["nll"]),
           "n_layers": np.int64(shape.n_layers), "seed": np.int64(SEED), "keep": np.array(keep)}
    rows_t = np.sort(rs.choice(T, SAMPLE_DH_ROWS, replace=False))
    cols_d = np.sort(rs.choice(shape.d_model, SAMPLE_DH_COLS, replace=False))
    out["dh_rows"], out["dh_cols"] = rows_t, cols_d
    out["dh_final"] = f32(res["dh"]["final"][np.ix_(rows_t, cols_d)])
    out["dh_final_norm"] = np.float64(np.linalg.norm(res["dh"]["final"]))
    for l in keep:
        out[f"dh_{l}"] = f32(res["dh"][l][np.ix_(rows_t, cols_d)])
        out[f"dh_norm_{l}"] = np.float64(np.linalg.norm(res["dh"][l]))
    for l in keep:
        for i, p in enumerate(synth.PROJ):
            dA, dB = res["grads"][l][p]
            assert np.all(dA == 0.0)     # B = 0  =>  dA = 0 exactly
            rows = np.sort(rs.choice(dB.shape[0], SAMPLE_ROWS, replace=False))
            out[f"dB_rows_{l}_{i}"] = rows
            out[f"dB_{l}_{i}"] = f32(dB[rows])
            out[f"dB_norm_{l}_{i}"] = np.float64(np.linalg.norm(dB))
    np.savez_compressed(OUT if n_layers == 32 else OUT.replace(".npz", f"_L{n_layers}.npz"), **out)
    print("wrote", OUT, flush=True)


if __name__ == "__main__":
    main(int(sys.argv[1]) if len(sys.argv) > 1 else 32)
