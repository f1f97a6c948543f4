#!/usr/bin/env python3
"""Writes tests/golden/train_7bwidth_L2_seed4096_b{4096,512}.npz: the CPU oracle's chunk_train on the long samples of
the paper's Table 5 -- a chunk of Delta = 4096 tokens behind L_T = 1024 conditioning tokens, trained with batch 4096
(one optimizer step on a 5120-token sample, the longest sample of the table) and with batch 512 (eight steps per epoch
on 1536-token samples) -- on a two-layer decoder of the 7B width (d 4096, 32x128 heads, ffn 11008, vocab 32000, r = 64)
so that the oracle finishes in minutes.  One epoch, warm-up over the first two steps.

Calls only oracle/, the seeded input generator and tests/bf16_floor.py (built from oracle functions only).  Zipf(1.1)
token ids, A ~ N(0, 0.02^2), B ~ N(0, 0.01^2).  Stored: the loss of every step; samples of B and of both first moments
after the last step for every projection of every layer; and `floor_*`: what the bf16-boundary replay of the oracle
(the storage format of Section 3 "Setup" alone, no kernel) differs from the fp64 oracle by on each of them.

    python tests/golden/make_train_golden.py 4096 | 512
"""
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.dirname(HERE))
import bf16_floor as F  # noqa: E402
from oracle import templora_oracle as O  # noqa: E402
from paper_2401_11504_amd import synth  # noqa: E402

SEED, N_LAYERS, N_BEFORE, N_CHUNK, L_T, EPOCHS, LR, WARMUP, B_STD = 4096, 2, 1024, 4096, 1024, 1, 5e-5, 2, 0.01
ROWS, COLS = 4, 256


def sample_err(x, ref):
    x, ref = np.asarray(x, np.float64), np.asarray(ref, np.float64)
    rms = np.sqrt(np.mean(ref * ref))
    return np.array([np.linalg.norm(x - ref) / np.linalg.norm(ref), np.max(np.abs(x - ref)) / (10.0 * rms)])


def main(batch):
    shape = synth.SHAPES["7b"].with_layers(N_LAYERS)
    tok = synth.zipf_tokens(SEED, N_BEFORE + N_CHUNK, shape.vocab)
    emb, head = synth.embedding(SEED, shape), synth.lm_head(SEED, shape)
    W = [synth.layer_weights(SEED, shape, l) for l in range(shape.n_layers)]
    get_layer = lambda l: W[l]
    g = np.ones(shape.d_model)
    mk = lambda: [synth.lora_factors(SEED, shape, l, b_std=B_STD) for l in range(shape.n_layers)]
    t0 = time.time()
    lora0 = mk()
    ref_losses, ref_lora, ref_opt = O.chunk_train(tok, N_CHUNK, L_T, batch, EPOCHS, LR, WARMUP, shape, emb, head, g,
                                                  get_layer, lora0, O.new_opt_state(lora0))
    print(f"oracle chunk_train (batch {batch}): {time.time() - t0:.1f} s, losses {np.round(ref_losses, 5)}", flush=True)
    t0 = time.time()
    lora1 = mk()
    rep_losses, rep_lora, rep_opt = F.chunk_train(tok, N_CHUNK, L_T, batch, EPOCHS, LR, WARMUP, shape, emb, head, g,
                                                  get_layer, lora1, O.new_opt_state(lora1))
    print(f"bf16-boundary replay: {time.time() - t0:.1f} s, losses {np.round(rep_losses, 5)}", flush=True)
    rs = np.random.default_rng(SEED + batch)
    f32 = lambda x: np.asarray(x, dtype=np.float32)
    out = {"seed": np.int64(SEED), "n_layers": np.int64(N_LAYERS), "n_before": np.int64(N_BEFORE),
           "n_chunk": np.int64(N_CHUNK), "L_T": np.int64(L_T), "batch": np.int64(batch), "epochs": np.int64(EPOCHS),
           "lr": np.float64(LR), "warmup": np.int64(WARMUP), "b_std": np.float64(B_STD), "tokens": tok,
           "losses": np.asarray(ref_losses, np.float64),
           "floor_losses": np.abs(np.asarray(rep_losses) - np.asarray(ref_losses)) / np.abs(np.asarray(ref_losses)),
           "n_steps": np.int64(ref_opt["tau"])}
    for l in range(shape.n_layers):
        for i, p in enumerate(synth.PROJ):
            d_out, d_in = shape.proj_dims(p)
            ra = np.sort(rs.choice(shape.rank, ROWS, replace=False))
            ca = np.sort(rs.choice(d_in, COLS, replace=False))
            rb = np.sort(rs.choice(d_out, ROWS, replace=False))
            out[f"rowsA_{l}_{i}"], out[f"colsA_{l}_{i}"], out[f"rowsB_{l}_{i}"] = ra, ca, rb
            B0 = np.asarray(lora0[l][p][1], np.float64)
            for tag, ref, rep in (("dB_total", np.asarray(ref_lora[l][p][1]) - B0, np.asarray(rep_lora[l][p][1]) - B0),
                                  ("mB", ref_opt["m"][l][p][1], rep_opt["m"][l][p][1])):
                out[f"{tag}_{l}_{i}"] = f32(np.asarray(ref)[rb])
                out[f"floor_{tag}_{l}_{i}"] = sample_err(np.asarray(rep)[rb], np.asarray(ref)[rb])
            out[f"mA_{l}_{i}"] = f32(np.asarray(ref_opt["m"][l][p][0])[np.ix_(ra, ca)])
            out[f"floor_mA_{l}_{i}"] = sample_err(np.asarray(rep_opt["m"][l][p][0])[np.ix_(ra, ca)],
                                                  np.asarray(ref_opt["m"][l][p][0])[np.ix_(ra, ca)])
    print("largest floors: loss %.2e, mA %.3f, mB %.3f, total B step %.3f" % (
        out["floor_losses"].max(), max(out[f"floor_mA_{l}_{i}"][0] for l in range(N_LAYERS) for i in range(7)),
        max(out[f"floor_mB_{l}_{i}"][0] for l in range(N_LAYERS) for i in range(7)),
        max(out[f"floor_dB_total_{l}_{i}"][0] for l in range(N_LAYERS) for i in range(7))), flush=True)
    path = os.path.join(HERE, f"train_7bwidth_L{N_LAYERS}_seed{SEED}_b{batch}.npz")
    np.savez_compressed(path, **out)
    print("wrote", path, flush=True)


if __name__ == "__main__":
    main(int(sys.argv[1]))
