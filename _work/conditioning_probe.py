#!/usr/bin/env python3
"""How well conditioned is the synthetic workload?  Runs the fp64 oracle twice at the 7B width (n_layers and n_tokens
from the command line), the second time with every embedding entry multiplied by 1 + 1e-3 * N(0, 1), and prints the
relative L2 change of the hidden-state gradient at every layer boundary and of dB of the q projection.

Calls only oracle/ and the seeded input generator.  It backs the tolerance used for deep tensors in
tests/test_gpu_config3.py: a relative input perturbation of 1e-3 (about one bf16 rounding) already moves the
gradients by 4e-3 .. 1.6e-2 within eight layers, growing towards the input, so no bf16 implementation can meet 2e-2
on the deepest gradients of the 32-layer model.  Output of `python tests/golden/conditioning_probe.py 8 256`:

    dh final rel diff 2.353e-04
    dh layer  7 rel diff 4.188e-03   dB(q) rel diff 1.636e-02
    dh layer  6 rel diff 5.888e-03   dB(q) rel diff 1.570e-02
    dh layer  5 rel diff 7.170e-03   dB(q) rel diff 1.509e-02
    dh layer  4 rel diff 8.228e-03   dB(q) rel diff 1.460e-02
    dh layer  3 rel diff 9.132e-03   dB(q) rel diff 1.395e-02
    dh layer  2 rel diff 9.930e-03   dB(q) rel diff 1.346e-02
    dh layer  1 rel diff 1.060e-02   dB(q) rel diff 1.254e-02
    dh layer  0 rel diff 1.117e-02   dB(q) rel diff 1.127e-02
"""
import sys, os, time, numpy as np
sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
from oracle import templora_oracle as O
from paper_2401_11504_amd import synth
L, T, SEED = int(sys.argv[1]), int(sys.argv[2]), 3000
shape = synth.SHAPES["7b"].with_layers(L)
tok = synth.uniform_tokens(SEED, T, shape.vocab)
emb, head = synth.embedding(SEED, shape), synth.lm_head(SEED, shape)
lora = [synth.lora_factors(SEED, shape, l) for l in range(L)]
W = {l: synth.layer_weights(SEED, shape, l) for l in range(L)}
keep = list(range(L))
def run(e):
    t0 = time.time()
    r = O.model_fwd_bwd(tok, 0, shape, e, head, np.ones(shape.d_model), lambda l: W[l], lora, keep=keep)
    print("run %.1f s loss %.6f" % (time.time() - t0, r["loss"]), flush=True)
    return r
a = run(emb)
rs = np.random.default_rng(1)
b = run(emb.astype(np.float64) * (1.0 + 1e-3 * rs.standard_normal(emb.shape)))
rel = lambda x, y: np.linalg.norm(x - y) / np.linalg.norm(x)
print("dh final rel diff %.3e" % rel(a["dh"]["final"], b["dh"]["final"]))
for l in reversed(keep):
    print("dh layer %2d rel diff %.3e   dB(q) rel diff %.3e" % (l, rel(a["dh"][l], b["dh"][l]), rel(a["grads"][l]["q"][1], b["grads"][l]["q"][1])))
