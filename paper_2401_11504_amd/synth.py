"""Seeded synthetic inputs for the Temp-Lora chunk update.

This module only draws random buffers of the shapes the paper's workloads have
(Section 3 "Setup": Llama2-7B dimensions, chunks of 1024 tokens, LoRA rank 64)
and rounds them to the storage type.  It holds none of the method's arithmetic;
both the CPU oracle's tests and the HIP path's callers take their inputs from
here so that the two sides see identical bytes.

Every tensor has its own Philox stream keyed by (seed, a path of small
integers), so a tensor can be regenerated on its own, in any order, on any
number of threads.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from concurrent.futures import ThreadPoolExecutor

import numpy as np

# projection order used everywhere (index = "proj" in the C ABI)
PROJ = ("q", "k", "v", "o", "gate", "up", "down")

# path tags (first element of a stream path)
_TAG_W, _TAG_A, _TAG_B, _TAG_EMB, _TAG_HEAD, _TAG_TOK, _TAG_X, _TAG_DY = range(1, 9)


@dataclass(frozen=True)
class Shape:
    """Decoder + LoRA dimensions (notation: T tokens, d hidden, f FFN width, V vocab, r rank)."""
    n_layers: int
    d_model: int
    n_heads: int
    d_head: int
    d_ffn: int
    vocab: int
    rank: int
    alpha: float
    rms_eps: float = 1e-5
    rope_base: float = 10000.0

    @property
    def scale(self) -> float:
        return self.alpha / self.rank

    def proj_dims(self, p: str):
        """(d_out, d_in) of projection p."""
        d, f = self.d_model, self.d_ffn
        return {"q": (d, d), "k": (d, d), "v": (d, d), "o": (d, d),
                "gate": (f, d), "up": (f, d), "down": (d, f)}[p]

    def with_layers(self, n: int) -> "Shape":
        return replace(self, n_layers=n)


# Workload shapes.  "7b" is the paper's Llama2-7B setting with its LoRA
# hyper-parameters (Section 3 "Setup": alpha = 64, rank = 64).
SHAPES = {
    "tiny": Shape(2, 32, 2, 16, 48, 64, 4, 8.0),
    "small": Shape(2, 256, 4, 64, 704, 1000, 16, 16.0),
    "small128": Shape(2, 256, 2, 128, 448, 776, 8, 16.0),
    "layer": Shape(1, 1024, 16, 64, 2816, 0, 16, 16.0),
    "7b": Shape(32, 4096, 32, 128, 11008, 32000, 64, 64.0),
}


def rng(seed: int, *path: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(np.random.SeedSequence([int(seed), *map(int, path)])))


def _round_bf16_inplace(x: np.ndarray) -> np.ndarray:
    """Round a contiguous fp32 array to bf16-representable values in place (nearest-even; finite inputs)."""
    u = x.reshape(-1).view(np.uint32)
    step = 1 << 22  # bounded temporaries for multi-GB tensors
    for i in range(0, u.size, step):
        blk = u[i:i + step]
        t = blk >> np.uint32(16)
        t &= np.uint32(1)
        t += np.uint32(0x7FFF)
        blk += t
        blk &= np.uint32(0xFFFF0000)
    return x


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round-to-nearest-even. Inputs are finite."""
    y = _round_bf16_inplace(np.array(x, dtype=np.float32, order="C", copy=True))
    return (y.reshape(-1).view(np.uint32) >> np.uint32(16)).astype(np.uint16).reshape(np.shape(x))


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 array whose every value is exactly representable in bf16."""
    return _round_bf16_inplace(np.array(x, dtype=np.float32, order="C", copy=True))


def normal(seed: int, path, shape, std: float, bf16: bool) -> np.ndarray:
    x = rng(seed, *path).standard_normal(shape, dtype=np.float32)
    x *= np.float32(std)
    return _round_bf16_inplace(x) if bf16 else x


def uniform_tokens(seed: int, n: int, vocab: int, stream: int = 0) -> np.ndarray:
    return rng(seed, _TAG_TOK, stream).integers(0, vocab, size=n, dtype=np.int64).astype(np.int32)


def zipf_tokens(seed: int, n: int, vocab: int, exponent: float = 1.1, stream: int = 0) -> np.ndarray:
    """ids whose rank k = id + 1 is drawn with probability proportional to k^-exponent."""
    w = np.arange(1, vocab + 1, dtype=np.float64) ** (-exponent)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    u = rng(seed, _TAG_TOK, 1000 + stream).random(n)
    return np.minimum(np.searchsorted(cdf, u, side="right"), vocab - 1).astype(np.int32)


def proj_weight(seed: int, shape: Shape, layer: int, p: str, bf16: bool = True, std: float = 0.02):
    return normal(seed, (_TAG_W, layer, PROJ.index(p)), shape.proj_dims(p), std, bf16)


def layer_weights(seed: int, shape: Shape, layer: int, bf16: bool = True) -> dict:
    """Frozen matrices of one decoder layer, W[p] is [d_out, d_in]; norm gains are 1."""
    w = {p: proj_weight(seed, shape, layer, p, bf16) for p in PROJ}
    w["g1"] = np.ones(shape.d_model, np.float32)
    w["g2"] = np.ones(shape.d_model, np.float32)
    return w


def lora_factors(seed: int, shape: Shape, layer: int, b_std: float = 0.0, a_std: float = 0.02) -> dict:
    """Per projection (A [r, d_in], B [d_out, r]) in fp32; B is zero unless b_std > 0."""
    out = {}
    for i, p in enumerate(PROJ):
        d_out, d_in = shape.proj_dims(p)
        a = normal(seed, (_TAG_A, layer, i), (shape.rank, d_in), a_std, False)
        if b_std > 0:
            b = normal(seed, (_TAG_B, layer, i), (d_out, shape.rank), b_std, False)
        else:
            b = np.zeros((d_out, shape.rank), np.float32)
        out[p] = (a, b)
    return out


def embedding(seed: int, shape: Shape, bf16: bool = True):
    return normal(seed, (_TAG_EMB,), (shape.vocab, shape.d_model), 0.02, bf16)


def lm_head(seed: int, shape: Shape, bf16: bool = True):
    return normal(seed, (_TAG_HEAD,), (shape.vocab, shape.d_model), 0.02, bf16)


def hidden(seed: int, n_tokens: int, width: int, bf16: bool = False):
    return normal(seed, (_TAG_X,), (n_tokens, width), 1.0, bf16)


def upstream_grad(seed: int, n_tokens: int, width: int, bf16: bool = False):
    return normal(seed, (_TAG_DY,), (n_tokens, width), 1.0, bf16)


def parallel_layers(fn, n_layers: int, workers: int = 8) -> list:
    """fn(layer) for every layer on a small thread pool (numpy's generators release the GIL)."""
    with ThreadPoolExecutor(max_workers=max(1, workers)) as ex:
        return list(ex.map(fn, range(n_layers)))


def linear_case(seed: int, n_tokens=128, d_in=256, d_out=256, rank=8):
    """The single fp32 LoRA-linear workload: X, W, A, B, dY."""
    return dict(
        X=normal(seed, (_TAG_X,), (n_tokens, d_in), 1.0, False),
        W=normal(seed, (_TAG_W, 0, 0), (d_out, d_in), 0.02, False),
        A=normal(seed, (_TAG_A, 0, 0), (rank, d_in), 0.02, False),
        B=normal(seed, (_TAG_B, 0, 0), (d_out, rank), 0.01, False),
        dY=normal(seed, (_TAG_DY,), (n_tokens, d_out), 1.0, False),
    )
