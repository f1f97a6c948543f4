#!/usr/bin/env python3
"""Throughput of the Temp-Lora chunk update on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

A "step" is one complete tl_chunk_update call: forward + loss + backward + AdamW over one
1024-token chunk on the 7B-shaped decoder with rank-64 LoRA on all seven projections
(Section 3 "Setup" of the paper; Table 5 is its cost table for this operation).  Tokens go in
as a host int32 array (4 KB) and the loss comes back as a host scalar; everything else is
resident in HBM before the timed region starts.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix peak (vendor figure, no sparsity)
# HBM bytes per launch of the dominant kernel, from two rocprofv3 --pmc passes over this same command
# (FETCH_SIZE, then WRITE_SIZE; summed over the kernel's launches of one update, divided by their number,
# each counter scaled by what it reads for --copy-calibration's 1 GiB copy).  The passes and the scaling
# factors are in profiles/chunk_update_7b_r64_T1024.md; counters cannot be read from inside this process.
GEMM_NT_HBM_BYTES_PER_LAUNCH = 202e6
# the same for the weight-streaming matrix-vector launches of the generation side (profiles/decode_7b_r64_window1024.md):
# 50 839 KiB of FETCH_SIZE per launch x 2.000 = 104.1 MB against 103.8 MB of algorithmic bytes; writes are negligible
GEMV_HBM_BYTES_PER_LAUNCH = 104.1e6


CPU_SAMPLE_LAYERS = 6


def cpu_baseline(shape, T, seed):
    """The fp64 oracle as it stands, timed on this host on a bounded sample of the same update (about ten seconds of CPU
    work): the embedding gather, the first CPU_SAMPLE_LAYERS layers of the 7B shape (forward + backward + the AdamW step
    of their 14 factors each; all 32 layers cost the same), and the final norm / lm_head / cross-entropy part once.
    Reported as trained tokens/s of the whole update = T / (t_gather + n_layers * mean(t_layer + t_adamw) + t_head)."""
    import numpy as np
    from oracle import templora_oracle as O
    from paper_2401_11504_amd import synth
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count() or 1])
    except Exception:
        cores = os.cpu_count() or 1
    emb = synth.embedding(seed, shape)
    tok = synth.uniform_tokens(seed, T, shape.vocab)
    t0 = time.perf_counter()
    h = np.asarray(emb, dtype=np.float64)[tok]                     # the oracle's gather (model_fwd_bwd, first line)
    t_gather = time.perf_counter() - t0
    del emb
    dy = synth.upstream_grad(seed, T, shape.d_model)
    n_sample = min(CPU_SAMPLE_LAYERS, shape.n_layers)
    t_layer = t_adamw = 0.0
    for l in range(n_sample):
        W = synth.layer_weights(seed, shape, l)
        facs = synth.lora_factors(seed, shape, l)
        t0 = time.perf_counter()
        h_next, cache = O.layer_fwd(h, W, facs, shape)
        _, G = O.layer_bwd(dy, cache, W, facs, shape)
        t_layer += time.perf_counter() - t0
        del cache, W
        t0 = time.perf_counter()
        for p in O.PROJ:
            for i in range(2):
                z = np.zeros_like(np.asarray(facs[p][i], dtype=np.float64))
                O.adamw_step(facs[p][i], G[p][i], z, z, 1, 5e-5)
        t_adamw += time.perf_counter() - t0
        del G
        h = h_next
    t_layer /= n_sample
    t_adamw /= n_sample
    head = synth.lm_head(seed, shape)
    t0 = time.perf_counter()
    labels, mask, _ = O.labels_and_mask(tok, 0)
    hf = O.rmsnorm_fwd(h, np.ones(shape.d_model), shape.rms_eps)
    logits = hf @ head.T.astype(np.float64)
    _, _, dlogits = O.cross_entropy(logits, labels, mask)
    dhf = dlogits @ head.astype(np.float64)
    O.rmsnorm_bwd(dhf, h, np.ones(shape.d_model), shape.rms_eps)
    t_head = time.perf_counter() - t0
    total = t_gather + shape.n_layers * (t_layer + t_adamw) + t_head
    return {"value": T / total, "unit": "trained tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"fp64 oracle: embedding gather ({t_gather:.3f} s) + layers 0..{n_sample - 1} fwd+bwd (mean {t_layer:.2f} s) "
                      f"and their AdamW steps (mean {t_adamw:.2f} s), the means counted x{shape.n_layers} layers + final "
                      f"norm/lm_head/CE fwd+bwd timed once ({t_head:.2f} s)"}


def stream_bench(args, torch, api, harness, synth):
    """configs[4]: a long synthetic input consumed as sequential 1024-token chunks, two epochs of updates per chunk,
    the module (and its AdamW state) carried from chunk to chunk and discarded at the end.  Sustained trained
    tokens/s = epochs * chunks * 1024 / total time, host-side token hand-over included."""
    shape = synth.SHAPES["7b"].with_layers(args.layers)
    seed, T, chunks, epochs, lr = 5000, 1024, args.stream, 2, 5e-5
    model = harness.Model(shape, seed, max_tokens=T, keep_host=False, device_random=True)
    lora = api.tl_lora_init(model.handle, shape.rank, shape.alpha, a_init_std=0.02, seed=seed)
    stream = synth.zipf_tokens(seed, chunks * T, shape.vocab)
    warm = synth.zipf_tokens(seed + 1, T, shape.vocab)
    for _ in range(2):
        api.tl_chunk_update(lora, warm, 0, lr)
    api.tl_discard(lora)                               # the warm-up module is thrown away: the stream starts from k = 0
    api.tl_lora_free(lora)
    lora = api.tl_lora_init(model.handle, shape.rank, shape.alpha, a_init_std=0.02, seed=seed)
    torch.cuda.synchronize()
    losses = []
    t0 = time.perf_counter()
    for c in range(chunks):
        tok = stream[c * T:(c + 1) * T]
        for _ in range(epochs):
            loss, _ = api.tl_chunk_update(lora, tok, 0, lr)
            losses.append(loss)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    steps = int(api.tl_get_step(lora))
    api.tl_discard(lora)
    api.tl_lora_free(lora)
    model.close()
    n = chunks * epochs
    second_lower = sum(1 for c in range(chunks) if losses[2 * c + 1] < losses[2 * c])
    print(json.dumps({
        "metric": "sustained trained tokens/sec over a stream of Temp-Lora chunk updates (7B-shape, r=64)",
        "value": round(n * T / dt, 1), "unit": "trained tokens/s", "n_gpus": 1, "steps": n, "warmup": 2,
        "ms_per_step": round(dt / n * 1e3, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"DEBUG (not the headline metric): configs[4] shape, {chunks} sequential 1024-token chunks of a "
                               f"Zipf(1.1) stream x {epochs} epochs, state carried, discarded at the end",
                   "n_layers": args.layers, "optimizer_steps": steps, "first_loss": round(float(losses[0]), 5),
                   "last_loss": round(float(losses[-1]), 5), "chunks_whose_second_epoch_loss_is_lower": second_lower}}))


def generate_bench(args, torch, api, harness, synth):
    """Algorithm 1 end to end (tl_generate, cascaded deployment): L_X = Delta = L_T = 1024, n = 2 epochs, greedy
    decoding, the cache recomputed after every update; seconds per 1024 generated tokens, everything included."""
    shape = synth.SHAPES["7b"].with_layers(args.layers)
    seed, chunks = 3000, args.generate
    model = harness.Model(shape, seed, max_tokens=2048, keep_host=False, device_random=True)
    lora = api.tl_lora_init(model.handle, shape.rank, shape.alpha, a_init_std=0.02, seed=seed)
    prompt = synth.uniform_tokens(seed, 1024, shape.vocab)
    api.tl_generate(lora, prompt, 8, 1024, 1024)                     # warm-up: a prefill and a few tokens
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    toks, losses = api.tl_generate(lora, prompt, 1024 * chunks, 1024, 1024, n_ctx_max=1024, batch=0, epochs=2, lr=5e-5,
                                   warmup_steps=4)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    api.tl_discard(lora)
    api.tl_lora_free(lora)
    model.close()
    print(json.dumps({
        "metric": "seconds per 1024 generated tokens, Algorithm 1 end to end (7B-shape, r=64, L_X = Delta = L_T = 1024, n = 2)",
        "value": round(dt / chunks, 3), "unit": "s per 1024 tokens", "n_gpus": 1, "steps": chunks, "warmup": 0,
        "ms_per_step": round(dt / chunks * 1e3, 1), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"configs[3] shape, {chunks} chunks: decode 1024 greedy tokens over a window growing from "
                               "1024 to 2048, then two training steps on (1024 conditioning + the chunk), then the cache "
                               "is recomputed; not the headline metric", "n_layers": args.layers,
                   "training_steps": len(losses), "generated": int(len(toks))},
        "generated_tokens_per_s": round(1024 * chunks / dt, 1)}))


def cycle_bench(args, torch, api, harness, synth):
    """configs[3]: the streaming cycle with its two halves timed separately.  Each cycle decodes 1024 greedy tokens over
    a key/value window that starts at the last 1024 tokens (and grows to 2048), then runs ONE chunk update on the 1024
    tokens just decoded, then recomputes the cache from them with the updated module (the paper's default).  Reports
    decode tokens/s, update trained tokens/s and the cache recomputation apart."""
    import numpy as np
    shape = synth.SHAPES["7b"].with_layers(args.layers)
    seed, cycles, W, D = 3000, args.cycle, 1024, 1024
    model = harness.Model(shape, seed, max_tokens=W + D + 1, keep_host=False, device_random=True)
    lora = api.tl_lora_init(model.handle, shape.rank, shape.alpha, a_init_std=0.02, seed=seed)
    window = synth.uniform_tokens(seed, W, shape.vocab)          # the stream so far (seeded stand-in for a prompt)
    nxt, _ = api.tl_prefill(lora, window)
    for _ in range(8):                                           # warm-up: a few tokens, one update, the prefill again
        nxt, _ = api.tl_decode_step(lora, nxt)
    api.tl_chunk_update(lora, window, 0, 5e-5)
    api.tl_discard(lora)
    api.tl_lora_free(lora)
    lora = api.tl_lora_init(model.handle, shape.rank, shape.alpha, a_init_std=0.02, seed=seed)
    nxt, _ = api.tl_prefill(lora, window)
    torch.cuda.synchronize()
    t_dec = t_upd = t_pre = 0.0
    losses = []
    for _ in range(cycles):
        chunk = np.empty(D, dtype=np.int32)
        t0 = time.perf_counter()
        for i in range(D):
            chunk[i] = nxt
            nxt, _ = api.tl_decode_step(lora, nxt)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        loss, _ = api.tl_chunk_update(lora, chunk, 0, 5e-5)
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        nxt, _ = api.tl_prefill(lora, chunk[-W:])
        torch.cuda.synchronize()
        t3 = time.perf_counter()
        t_dec += t1 - t0; t_upd += t2 - t1; t_pre += t3 - t2
        losses.append(round(loss, 5))
    api.tl_discard(lora)
    api.tl_lora_free(lora)
    model.close()
    total = t_dec + t_upd + t_pre
    print(json.dumps({
        "metric": "streaming Temp-Lora cycle (7B-shape, r=64): decode and update timed separately",
        "value": round(D * cycles / t_upd, 1), "unit": "trained tokens/s (update half)", "n_gpus": 1, "steps": cycles,
        "warmup": 1, "ms_per_step": round(1e3 * total / cycles, 1), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"DEBUG (not the headline metric): configs[3], {cycles} cycles of (decode 1024 greedy tokens over "
                               "a 1024..2048-token key/value window, one chunk update on them, cache recomputed from them)",
                   "n_layers": args.layers, "stream_tokens": D * cycles},
        "update_trained_tokens_per_s": round(D * cycles / t_upd, 1), "decode_tokens_per_s": round(D * cycles / t_dec, 1),
        "ms_per_update": round(1e3 * t_upd / cycles, 2), "ms_per_decoded_token": round(1e3 * t_dec / (D * cycles), 3),
        "ms_per_cache_recompute": round(1e3 * t_pre / cycles, 2), "s_per_1024_stream_tokens": round(total / cycles, 3),
        "first_update_loss": losses[0], "last_update_loss": losses[-1]}))


def decode_bench(args, torch, api, harness, synth):
    """Greedy decoding with the module over the key/value cache (Algorithm 1's token loop): tokens/s, and the
    matrix-vector kernel that streams the frozen weights against the HBM roofline."""
    shape = synth.SHAPES["7b"].with_layers(args.layers)
    seed, P, K = 3000, args.prompt, args.steps
    model = harness.Model(shape, seed, max_tokens=P + K + args.warmup + 1, keep_host=False, device_random=True)
    lora = api.tl_lora_init(model.handle, shape.rank, shape.alpha, a_init_std=0.02, seed=seed)
    # B = 0 would make the module a no-op numerically but not in work done: the kernels read A and B regardless
    prompt = synth.uniform_tokens(seed, P, shape.vocab)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    nxt, _ = api.tl_prefill(lora, prompt)
    t_prefill = time.perf_counter() - t0
    for _ in range(args.warmup):
        nxt, _ = api.tl_decode_step(lora, nxt)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(K):
        nxt, _ = api.tl_decode_step(lora, nxt)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    roof = None
    if not args.no_events:
        # a second window of the same length from the same start, with the weight-streaming launches bracketed
        nxt, _ = api.tl_prefill(lora, prompt)
        for _ in range(args.warmup):
            nxt, _ = api.tl_decode_step(lora, nxt)
        api.tl_profile_enable(lora, True)
        for _ in range(K):
            nxt, _ = api.tl_decode_step(lora, nxt)
        ms, launches, flop = api.tl_profile_read(lora)
        api.tl_profile_enable(lora, False)
        gbs = flop / (ms * 1e-3) / 1e9 if ms > 0 else 0.0     # 2 flop per bf16 element of 2 bytes: bytes read = flop
        roof = {"bound": "hbm", "achieved": round(gbs, 1), "peak": 8000.0, "unit": "GB/s", "frac": round(gbs / 8000.0, 4),
                "traffic": GEMV_HBM_BYTES_PER_LAUNCH if args.layers == 32 else None,
                "kernel": "gemv_kernel (frozen matrix + LoRA B rows, one token)",
                "launches_per_step": launches // max(K, 1), "avg_launch_us": round(ms * 1e3 / max(launches, 1), 2),
                "bytes_per_launch": flop / max(launches, 1),
                "share_of_step_time": round(ms * 1e-3 / dt, 4)}
    api.tl_discard(lora)
    api.tl_lora_free(lora)
    model.close()
    d, f, V, L, r = shape.d_model, shape.d_ffn, shape.vocab, shape.n_layers, shape.rank
    weight_bytes = 2.0 * (L * (4 * d * d + 3 * d * f) + d * V)
    lora_bytes = 2.0 * r * L * (4 * 2 * d + 3 * (d + f))
    kv_bytes = 2.0 * 2 * d * L * (P + args.warmup + K / 2.0)
    print(json.dumps({
        "metric": "greedy decode tokens/sec with the Temp-Lora module over a key/value cache (7B-shape, r=64)",
        "value": round(K / dt, 1), "unit": "decoded tokens/s", "n_gpus": 1, "steps": K, "warmup": args.warmup,
        "ms_per_step": round(dt / K * 1e3, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"generation side of configs[3] (not the headline metric): {args.layers} layers, window "
                               f"{P} tokens at the start, {K} tokens decoded", "prefill_ms": round(t_prefill * 1e3, 2)},
        "hbm_bytes_per_token": weight_bytes + lora_bytes + kv_bytes,
        "hbm_frac_whole_step": round((weight_bytes + lora_bytes + kv_bytes) / (dt / K) / 8e12, 4),
        "roofline": roof}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--layers", type=int, default=32, help="debug only: fewer layers (marks the line invalid)")
    ap.add_argument("--tokens", type=int, default=1024)
    ap.add_argument("--ctx", type=int, default=0,
                    help="debug only: the first CTX of --tokens are conditioning (L_T prefix, no loss on them)")
    ap.add_argument("--dropout", type=float, default=0.0,
                    help="debug only: LoRA dropout rate (the benchmark configuration has none; marks the line)")
    ap.add_argument("--stream", type=int, default=0, metavar="CHUNKS",
                    help="measure the long-input workload instead (configs[4]): CHUNKS sequential 1024-token chunks of a "
                         "Zipf(1.1) token stream, two epochs each, module state carried, discarded at the end")
    ap.add_argument("--generate", type=int, default=0, metavar="CHUNKS",
                    help="measure Algorithm 1 end to end instead: generate CHUNKS chunks of 1024 tokens with tl_generate")
    ap.add_argument("--cycle", type=int, default=0, metavar="CYCLES",
                    help="debug line: configs[3], CYCLES x (decode 1024 tokens, one update on them), halves timed separately")
    ap.add_argument("--decode", action="store_true",
                    help="measure the generation side instead (the step either side of the update): one step = one "
                         "greedily decoded token with the module applied, after a prefill of --prompt tokens")
    ap.add_argument("--prompt", type=int, default=1024, help="--decode: tokens in the window when decoding starts")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-events", action="store_true", help="do not bracket the GEMM launches with HIP events")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run one plain 1 GiB device-to-device copy kernel (reference for the rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE counters) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the chunk update has no CPU path", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    if args.copy_calibration:
        n = 1 << 28  # 2^28 fp32 = 1 GiB read + 1 GiB written by one elementwise copy kernel
        src = torch.ones(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_read": 4 * n, "copy_calibration_bytes_written": 4 * n}))
        return
    from paper_2401_11504_amd import api, harness, synth

    if args.stream > 0:
        stream_bench(args, torch, api, harness, synth)
        return
    if args.generate > 0:
        generate_bench(args, torch, api, harness, synth)
        return
    if args.cycle > 0:
        cycle_bench(args, torch, api, harness, synth)
        return
    if args.decode:
        decode_bench(args, torch, api, harness, synth)
        return
    shape = synth.SHAPES["7b"].with_layers(args.layers)
    T, seed = args.tokens, 3000
    headline = args.layers == 32 and T == 1024 and args.dropout == 0.0 and args.ctx == 0
    model = harness.Model(shape, seed, max_tokens=T, keep_host=False, device_random=True)
    # config: A ~ N(0, 0.02^2), B = 0, AdamW lr 5e-5, betas (0.9, 0.999), wd 0
    lora = api.tl_lora_init(model.handle, shape.rank, shape.alpha, a_init_std=0.02, seed=seed,
                            dropout=args.dropout)
    tok = synth.uniform_tokens(seed, T, shape.vocab)
    lr = 5e-5

    loss = first_loss = None
    for _ in range(args.warmup):
        loss, n_targets = api.tl_chunk_update(lora, tok, args.ctx, lr)
        if first_loss is None:
            first_loss = loss                    # the module's very first step: B = 0, so this is the base model's loss
    # timed region 1: exactly K steps, nothing but the update on the GPU -> `value`
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        loss, n_targets = api.tl_chunk_update(lora, tok, args.ctx, lr)
        if first_loss is None:
            first_loss = loss
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    # timed region 2: K more steps with every launch of the dominant kernel bracketed by HIP events on the
    # library's stream -> `roofline`.  Kept apart from region 1 because the 516 event packets per step
    # cost about 6 % of a step (each drains the queue), which would understate `value`.
    roof = None
    if not args.no_events:
        api.tl_profile_enable(lora, True)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(args.steps):
            api.tl_chunk_update(lora, tok, args.ctx, lr)
        torch.cuda.synchronize()
        dt_ev = time.perf_counter() - t1
        ms, launches, flop = api.tl_profile_read(lora)
        api.tl_profile_enable(lora, False)
        achieved = flop / (ms * 1e-3) / 1e12 if ms > 0 else 0.0
        roof = {"bound": "mfma", "achieved": round(achieved, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4),
                "traffic": GEMM_NT_HBM_BYTES_PER_LAUNCH if headline else None,
                "traffic_source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE passes recorded in profiles/ (not measured in this run)",
                "kernel": "gemm_nt_dl_kernel (frozen W GEMM + low-rank K-extension; all tile shapes)",
                "launches_per_step": launches // max(args.steps, 1),
                "avg_launch_us": round(ms * 1e3 / max(launches, 1), 2),
                "flop_per_launch": flop / max(launches, 1),
                "share_of_step_time": round(ms * 1e-3 / dt_ev, 4),
                "ms_per_step_with_events": round(dt_ev / args.steps * 1e3, 3)}
    api.tl_discard(lora)
    api.tl_lora_free(lora)
    model.close()

    ms_step = dt / args.steps * 1e3
    # whole-update algorithmic work: frozen GEMMs fwd + dX, LoRA low-rank products, causal attention fwd + bwd
    d, f, V, L, r = shape.d_model, shape.d_ffn, shape.vocab, shape.n_layers, shape.rank
    frozen = 2.0 * T * (L * (4 * d * d + 3 * d * f) + d * V)
    lora_fl = 6.0 * T * r * L * (4 * 2 * d + 3 * (d + f))
    attn = 3.5 * 2.0 * T * T * d * L
    # the gradient at the embedding output feeds nothing trainable: dX of layer 0's q|k|v (frozen part and its low-rank
    # extension) is not computed and not counted
    total_flop = 2 * frozen + lora_fl + attn - 2.0 * T * 3 * d * (d + r)
    out = {
        "metric": "trained tokens/sec per Temp-Lora chunk update (7B-shape, r=64); MFMA util %",
        "value": round((T - args.ctx) / (ms_step * 1e-3), 1),   # chunk tokens; conditioning tokens are not trained on
        "unit": "trained tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "configs[2]: full Temp-Lora chunk update, 7B-shaped decoder (32 layers, d 4096, 32x128 "
                               "heads, ffn 11008, vocab 32000), LoRA r=64 alpha=64 on q,k,v,o,gate,up,down, "
                               "one 1024-token chunk, AdamW lr 5e-5" if headline else
                               f"DEBUG (not the benchmark): {args.layers} layers, {T} tokens of which {args.ctx} conditioning, "
                               f"dropout {args.dropout}",
                   "n_tokens": T, "n_layers": args.layers, "rank": r, "first_step_loss": round(float(first_loss), 5),
                   "loss_after_all_steps_on_the_same_chunk": round(float(loss), 5), "n_targets": n_targets},
        "mfma_util_whole_update": round(total_flop / (ms_step * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
        "algorithmic_tflop_per_step": round(total_flop / 1e12, 3),
        "roofline": roof,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(synth.SHAPES["7b"], T, seed)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
