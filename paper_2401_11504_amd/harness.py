"""Glue between the seeded synthetic inputs and the C ABI: uploads buffers, builds handles.

No arithmetic of the method lives here: tensors are drawn by `synth`, moved to the
device with torch, and handed to libtemplora through `api`.
"""
from __future__ import annotations

import numpy as np
import torch

from . import api, synth


def to_dev_bf16(x: np.ndarray) -> torch.Tensor:
    """fp32 numpy (bf16-representable or not) -> device bf16 tensor, nearest-even."""
    bits = synth.bf16_bits(x).view(np.int16)
    return torch.from_numpy(bits).cuda().view(torch.bfloat16)


def to_dev_f32(x: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()


def bf16_to_np(t: torch.Tensor) -> np.ndarray:
    return t.float().cpu().numpy()


class Model:
    """A frozen synthetic decoder on the device + the host copies the oracle needs (optional)."""

    def __init__(self, shape: synth.Shape, seed: int, max_tokens: int, keep_host: bool = True, workers: int = 8,
                 device_random: bool = False):
        self.shape, self.seed, self.max_tokens = shape, seed, max_tokens
        self.host_layers = [None] * shape.n_layers
        self.emb = self.head = None
        ptrs = []
        hold = []
        if device_random:
            # throughput runs only: values drawn on the device (same distribution, not reproducible on the host)
            g = torch.Generator(device="cuda").manual_seed(seed)
            for l in range(shape.n_layers):
                for p in synth.PROJ:
                    w = (torch.randn(shape.proj_dims(p), generator=g, device="cuda") * 0.02).bfloat16()
                    hold.append(w), ptrs.append(w)
                for _ in range(2):
                    gain = torch.ones(shape.d_model, device="cuda")
                    hold.append(gain), ptrs.append(gain)
            if shape.vocab:
                e = (torch.randn(shape.vocab, shape.d_model, generator=g, device="cuda") * 0.02).bfloat16()
                h = (torch.randn(shape.vocab, shape.d_model, generator=g, device="cuda") * 0.02).bfloat16()
                ptrs += [e, torch.ones(shape.d_model, device="cuda"), h]
            else:
                ptrs += [None, None, None]
        else:
            layers = synth.parallel_layers(lambda l: synth.layer_weights(seed, shape, l), shape.n_layers, workers)
            for l, W in enumerate(layers):
                for p in synth.PROJ:
                    ptrs.append(to_dev_bf16(W[p]))
                ptrs.append(to_dev_f32(W["g1"]))
                ptrs.append(to_dev_f32(W["g2"]))
                if keep_host:
                    self.host_layers[l] = W
            if shape.vocab:
                emb, head = synth.embedding(seed, shape), synth.lm_head(seed, shape)
                ptrs += [to_dev_bf16(emb), to_dev_f32(np.ones(shape.d_model, np.float32)), to_dev_bf16(head)]
                if keep_host:
                    self.emb, self.head = emb, head
            else:
                ptrs += [None, None, None]
        torch.cuda.synchronize()
        self.handle = api.tl_model_create(shape.n_layers, shape.d_model, shape.n_heads, shape.d_head, shape.d_ffn,
                                          shape.vocab, max_tokens, ptrs, shape.rms_eps, shape.rope_base)
        del ptrs, hold  # the library keeps its own packed copies
        torch.cuda.empty_cache()

    def close(self):
        if self.handle is not None:
            api.tl_model_destroy(self.handle)
            self.handle = None


def new_lora(model: Model, seed: int, b_std: float = 0.0, set_from_synth: bool = True, keep_input_grad: bool = True,
             **hyper):
    """tl_lora_init + (optionally) overwrite A, B with the synth draws the oracle also uses.
    Returns (handle, host factors [{proj: (A, B)}] or None).  keep_input_grad: updates also compute the gradient at
    the embedding output (off by default in the library), so that tl_get_dh(.., 0, ..) can be compared."""
    shape = model.shape
    h = api.tl_lora_init(model.handle, shape.rank, shape.alpha, seed=seed, **hyper)
    if keep_input_grad:
        api.tl_keep_input_grad(h, True)
    if not set_from_synth:
        return h, None
    facs = [synth.lora_factors(seed, shape, l, b_std=b_std) for l in range(shape.n_layers)]
    for l in range(shape.n_layers):
        for i, p in enumerate(synth.PROJ):
            a, b = facs[l][p]
            api.tl_set_factor(h, l, i, api.FACTOR_A, a)
            api.tl_set_factor(h, l, i, api.FACTOR_B, b)
    return h, facs
