#!/usr/bin/env python3
"""Writes tests/golden/prefix_7bwidth_L4_seed2048.npz (default) or, with the argument "piece", tests/golden/
prefix_7bwidth_L2_seed1357.npz.  The first holds the CPU oracle's results for one update on the paper's actual
training sample layout -- L_T = 1024 conditioning tokens followed by a chunk of 1024 (Section 2, "use the preceding
L_T tokens as the input and the chunk as the output"), i.e. 2048 tokens with n_ctx = 1024 so that only the chunk
positions carry loss -- on a decoder of the 7B width (d 4096, 32x128 heads, ffn 11008, vocab 32000, r = 64) cut to
four layers so that the oracle finishes in minutes and every tensor can be held to the bf16 tolerance.

Calls only oracle/, the seeded input generator and tests/bf16_floor.py (built from oracle functions only).  Zipf(1.1) token ids, A ~ N(0, 0.02^2), B ~ N(0, 0.01^2) (so that
dA != 0).  Stored: loss, n_targets, per-position nll, samples of the hidden-state gradient at every layer boundary and
of dA / dB of every projection of every layer, with full-tensor norms; and next to every sample `floor_*`: the error
of the bf16-boundary replay of the oracle (tests/bf16_floor.py) against the fp64 oracle on that sample, as (relative L2,
max-abs / 10 RMS) -- what the storage format of Section 3 "Setup" alone costs, no kernel involved.

The "piece" file is the layout of one of Table 5's smaller batches: the same 1024 conditioning tokens followed by a
ragged piece of 333 tokens (1357 in all, no multiple of any tile), on two layers of the same width.

    python tests/golden/make_prefix_golden.py [piece]
"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
import bf16_floor as F  # noqa: E402
from oracle import templora_oracle as O  # noqa: E402
from paper_2401_11504_amd import synth  # noqa: E402

B_STD = 0.01
if sys.argv[1:] == ["piece"]:
    SEED, T, N_CTX, N_LAYERS = 1357, 1357, 1024, 2
else:
    SEED, T, N_CTX, N_LAYERS = 2048, 2048, 1024, 4
OUT = os.path.join(os.path.dirname(os.path.abspath(__file__)), f"prefix_7bwidth_L{N_LAYERS}_seed{SEED}.npz")
ROWS, COLS = 2, 256


def main():
    shape = synth.SHAPES["7b"].with_layers(N_LAYERS)
    tok = synth.zipf_tokens(SEED, T, shape.vocab)
    emb, head = synth.embedding(SEED, shape), synth.lm_head(SEED, shape)
    lora = [synth.lora_factors(SEED, shape, l, b_std=B_STD) for l in range(shape.n_layers)]
    W = {}

    def get_layer(l):
        if l not in W:
            W[l] = synth.layer_weights(SEED, shape, l)
        return W[l]

    keep = list(range(shape.n_layers))
    t0 = time.time()
    res = O.model_fwd_bwd(tok, N_CTX, shape, emb, head, np.ones(shape.d_model), get_layer, lora, keep=keep)
    print(f"oracle forward+backward: {time.time() - t0:.1f} s, loss {res['loss']:.6f}, targets {res['n_targets']}", flush=True)
    rs = np.random.default_rng(SEED)
    f32 = lambda x: np.asarray(x, dtype=np.float32)
    out = {"loss": np.float64(res["loss"]), "n_targets": np.int64(res["n_targets"]), "nll": f32(res["nll"]),
           "n_layers": np.int64(shape.n_layers), "seed": np.int64(SEED), "n_ctx": np.int64(N_CTX), "b_std": np.float64(B_STD),
           "tokens": tok}
    if N_LAYERS == 4:
        rows_t = np.sort(rs.choice(T, 4, replace=False))
    else:       # two conditioning rows (their gradient arrives through dK / dV alone) and two rows of the piece
        rows_t = np.concatenate([np.sort(rs.choice(N_CTX - 1, 2, replace=False)),
                                 np.sort(N_CTX - 1 + rs.choice(T - N_CTX + 1, 2, replace=False))])
    cols_d = np.sort(rs.choice(shape.d_model, COLS, replace=False))
    out["dh_rows"], out["dh_cols"] = rows_t, cols_d
    out["dh_final"] = f32(res["dh"]["final"][np.ix_(rows_t, cols_d)])
    out["dh_final_norm"] = np.float64(np.linalg.norm(res["dh"]["final"]))
    for l in keep:
        out[f"dh_{l}"] = f32(res["dh"][l][np.ix_(rows_t, cols_d)])
        out[f"dh_norm_{l}"] = np.float64(np.linalg.norm(res["dh"][l]))
        for i, p in enumerate(synth.PROJ):
            dA, dB = res["grads"][l][p]
            d_out, d_in = shape.proj_dims(p)
            ra = np.sort(rs.choice(shape.rank, ROWS, replace=False))
            ca = np.sort(rs.choice(d_in, COLS, replace=False))
            rb = np.sort(rs.choice(d_out, ROWS, replace=False))
            out[f"rowsA_{l}_{i}"], out[f"colsA_{l}_{i}"], out[f"rowsB_{l}_{i}"] = ra, ca, rb
            out[f"dA_{l}_{i}"] = f32(dA[np.ix_(ra, ca)])
            out[f"dB_{l}_{i}"] = f32(dB[rb])
            out[f"dA_norm_{l}_{i}"] = np.float64(np.linalg.norm(dA))
            out[f"dB_norm_{l}_{i}"] = np.float64(np.linalg.norm(dB))

    def sample_err(x, ref):
        x, ref = np.asarray(x, np.float64), np.asarray(ref, np.float64)
        rms = np.sqrt(np.mean(ref * ref))
        if rms == 0.0:      # rows without any gradient (conditioning rows above the last layer): the replay gives zeros too
            return np.array([np.linalg.norm(x), np.max(np.abs(x))])
        return np.array([np.linalg.norm(x - ref) / np.linalg.norm(ref), np.max(np.abs(x - ref)) / (10.0 * rms)])

    t0 = time.time()
    rep = F.model_fwd_bwd(tok, N_CTX, shape, emb, head, np.ones(shape.d_model), get_layer, lora, keep=keep)
    out["floor_loss"] = np.float64(abs(rep["loss"] - res["loss"]) / abs(res["loss"]))
    out["floor_nll"] = sample_err(rep["nll"], res["nll"])
    out["floor_dh_final"] = sample_err(rep["dh"]["final"][np.ix_(rows_t, cols_d)], out["dh_final"])
    for l in keep:
        out[f"floor_dh_{l}"] = sample_err(rep["dh"][l][np.ix_(rows_t, cols_d)], res["dh"][l][np.ix_(rows_t, cols_d)])
        if N_LAYERS != 4:     # conditioning rows and piece rows are bounded separately in the test
            pre = rows_t < N_CTX - 1
            for tag, sel in (("cond", pre), ("piece", ~pre)):
                out[f"floor_dh_{tag}_{l}"] = sample_err(rep["dh"][l][np.ix_(rows_t[sel], cols_d)],
                                                        res["dh"][l][np.ix_(rows_t[sel], cols_d)])
        for i, p in enumerate(synth.PROJ):
            dA, dB = rep["grads"][l][p]
            rA, rB = res["grads"][l][p]
            ra, ca, rb = out[f"rowsA_{l}_{i}"], out[f"colsA_{l}_{i}"], out[f"rowsB_{l}_{i}"]
            out[f"floor_dA_{l}_{i}"] = sample_err(dA[np.ix_(ra, ca)], rA[np.ix_(ra, ca)])
            out[f"floor_dB_{l}_{i}"] = sample_err(dB[rb], rB[rb])
    if N_LAYERS != 4:
        pre = rows_t < N_CTX - 1
        for tag, sel in (("cond", pre), ("piece", ~pre)):
            out[f"floor_dh_{tag}_final"] = sample_err(rep["dh"]["final"][np.ix_(rows_t[sel], cols_d)],
                                                      res["dh"]["final"][np.ix_(rows_t[sel], cols_d)])
    print(f"bf16-boundary replay: {time.time() - t0:.1f} s, loss floor {out['floor_loss']:.2e}; dh floors "
          + " ".join(f"{out[f'floor_dh_{l}'][0]:.4f}" for l in keep) + "; largest dA / dB floor "
          + f"{max(out[f'floor_dA_{l}_{i}'][0] for l in keep for i in range(7)):.4f} / "
          + f"{max(out[f'floor_dB_{l}_{i}'][0] for l in keep for i in range(7)):.4f}", flush=True)
    np.savez_compressed(OUT, **out)
    print("wrote", OUT, flush=True)


if __name__ == "__main__":
    main()
