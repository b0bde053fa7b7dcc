"""Seeded synthetic inputs for the ChunkFT hot path.

This module only draws numbers and picks ranges; it contains none of the
method's arithmetic, so the tests can hand the same arrays to the library and
to the checker they compare it with.

The paper's own workloads are fine-tuning runs of Llama-family models at a
maximum sequence length of 1024 (Section 4 and Table "Actual memory costs");
only the layer shapes, token counts and gradient scales of those runs reach
this path, so the inputs here are Gaussian arrays of those shapes:

* activations X ~ N(0, 1), output gradients dY ~ N(0, sigma_dY) with the second
  argument a standard deviation, parameters W0 ~ N(0, 0.02);
* values are drawn in fp32 and rounded ONCE to the storage dtype (torch's
  float32 -> bfloat16 conversion); both sides consume the rounded arrays;
* chunk offsets come from the same generator: numpy.random.default_rng(
  211770 + configuration index).
"""

from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np
import torch

SEED_BASE = 211770

# AdamW hyper-parameters used for every configuration
HPARAMS = dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)

F32 = 0
BF16 = 1
LINEAR = 0
VECTOR = 1
EMBEDDING = 2
RMSNORM = 3
LAYERNORM = 4

MiB = 1 << 20


def rng_for(config: int, stream: int = 0) -> np.random.Generator:
    return np.random.default_rng([SEED_BASE + config, stream])


def normal(rng: np.random.Generator, shape, sigma: float, dtype: int) -> torch.Tensor:
    """CPU tensor of N(0, sigma) draws stored as `dtype` (F32 or BF16)."""
    a = rng.standard_normal(size=shape, dtype=np.float32)
    if sigma != 1.0:
        a *= np.float32(sigma)
    t = torch.from_numpy(a)
    return t.to(torch.bfloat16) if dtype == BF16 else t


def two_scale_rows(rng: np.random.Generator, shape, sigma_lo: float, sigma_hi: float,
                   frac_hi: float, dtype: int) -> torch.Tensor:
    """[T, n] draws whose token rows are N(0, sigma_hi) with probability frac_hi
    (one seeded Bernoulli per row) and N(0, sigma_lo) otherwise."""
    T = shape[0]
    hot = rng.random(T) < frac_hi
    a = rng.standard_normal(size=shape, dtype=np.float32)
    scale = np.where(hot, np.float32(sigma_hi), np.float32(sigma_lo)).astype(np.float32)
    a *= scale[:, None]
    t = torch.from_numpy(a)
    return t.to(torch.bfloat16) if dtype == BF16 else t


def as_f64(t: torch.Tensor) -> np.ndarray:
    """Exact fp64 values of a CPU tensor (bf16 and fp32 embed in fp64)."""
    return t.detach().cpu().to(torch.float32).numpy().astype(np.float64)


def bits_u16(t: torch.Tensor) -> np.ndarray:
    """Raw bit patterns of a bf16 tensor."""
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16).copy()


def draw_offset(rng: np.random.Generator, numel: int, length: int, cols: int,
                mid_row: bool = True, odd: Optional[bool] = None) -> int:
    """Start of a range of `length` elements inside a tensor of `numel`.
    mid_row: neither end of the range falls on a row boundary.
    odd: force the parity of the offset (None = whatever is drawn)."""
    if length > numel:
        raise ValueError("range longer than the tensor")
    if length == numel:
        return 0
    for _ in range(10000):
        off = int(rng.integers(0, numel - length + 1))
        if odd is not None and (off % 2 == 1) != odd:
            off += 1 if off + 1 + length <= numel else -1
        if mid_row and (off % cols == 0 or (off + length) % cols == 0):
            continue
        return off
    raise RuntimeError("no admissible offset")


@dataclass
class LayerCase:
    """One tensor with the operands of its backward step (CPU tensors)."""
    name: str
    kind: int
    dtype: int
    out: int
    n_in: int
    T: int
    X: torch.Tensor          # [T, in]; EMBEDDING: the T token ids (int64)
    dY: torch.Tensor         # LINEAR [T, out]; others [T, in]
    W0: torch.Tensor         # LINEAR / EMBEDDING [out, in]; 1-D kinds [in]; storage dtype
    eps: float = 0.0         # RMSNORM / LAYERNORM

    @property
    def numel(self) -> int:
        return self.out * self.n_in

    def desc(self) -> Tuple[int, int, int]:
        return (self.out, self.n_in, self.dtype)


def linear_case(rng, name, out, n_in, T, dtype, sigma_dy, X: Optional[torch.Tensor] = None,
                dy_rows: Optional[Tuple[float, float, float]] = None) -> LayerCase:
    if X is None:
        X = normal(rng, (T, n_in), 1.0, dtype)
    if dy_rows is None:
        dY = normal(rng, (T, out), sigma_dy, dtype)
    else:
        dY = two_scale_rows(rng, (T, out), dy_rows[0], dy_rows[1], dy_rows[2], dtype)
    W0 = normal(rng, (out, n_in), 0.02, dtype)
    return LayerCase(name, LINEAR, dtype, out, n_in, T, X, dY, W0)


def vector_case(rng, name, n, T, dtype, sigma_dy) -> LayerCase:
    X = normal(rng, (T, n), 1.0, dtype)
    dY = normal(rng, (T, n), sigma_dy, dtype)
    W0 = normal(rng, (n,), 0.02, F32) + 1.0      # scale vectors sit around one
    if dtype == BF16:
        W0 = W0.to(torch.bfloat16)
    return LayerCase(name, VECTOR, dtype, 1, n, T, X, dY, W0)


def embedding_case(rng, name, vocab, dim, T, dtype, sigma_dy) -> LayerCase:
    """Embedding table [vocab, dim] with T token ids whose frequencies are heavy-tailed
    (rank r drawn with probability ~ 1/(r + 1), ranks scattered over the table), as token
    counts of text are: a few rows collect many tokens, most rows none."""
    ranks = np.minimum((np.exp(rng.random(T) * np.log(vocab + 1.0)) - 1.0).astype(np.int64), vocab - 1)
    perm = rng.permutation(vocab)
    ids = torch.from_numpy(perm[ranks].astype(np.int64))
    dY = normal(rng, (T, dim), sigma_dy, dtype)
    W0 = normal(rng, (vocab, dim), 0.02, dtype)
    return LayerCase(name, EMBEDDING, dtype, vocab, dim, T, ids, dY, W0)


def norm_case(rng, name, n, T, dtype, sigma_dy, kind, eps=1e-5) -> LayerCase:
    """Scale vector of RMSNorm / LayerNorm: raw activations with a per-token scale and,
    for LayerNorm, a non-zero mean."""
    a = rng.standard_normal(size=(T, n), dtype=np.float32)
    a *= (0.5 + 2.0 * rng.random(T).astype(np.float32))[:, None]
    if kind == LAYERNORM:
        a += rng.standard_normal(size=(T, 1), dtype=np.float32)
    X = torch.from_numpy(a)
    if dtype == BF16:
        X = X.to(torch.bfloat16)
    dY = normal(rng, (T, n), sigma_dy, dtype)
    W0 = normal(rng, (n,), 0.02, F32) + 1.0
    if dtype == BF16:
        W0 = W0.to(torch.bfloat16)
    return LayerCase(name, kind, dtype, 1, n, T, X, dY, W0, eps)


# --------------------------------------------------------------------------
# The five configurations.  `scale` divides the layer dimensions (not the
# structure) so that a CPU check of the same recipe finishes in seconds;
# scale = 1 is the configuration as stated.
# --------------------------------------------------------------------------
def config1():
    """Single fp32 linear layer, W 1024x512, T = 256, chunk [100000, 300000)."""
    rng = rng_for(1)
    layer = linear_case(rng, "fc", 1024, 512, 256, F32, 1.0)
    return layer, 100000, 300000


def config2(scale: int = 1, T: Optional[int] = None):
    """Llama-3-8B up_proj shape, bf16: W 14336x4096, T = 1024, one chunk of
    32 Mi elements (64 MiB of bf16) at a seeded mid-row offset."""
    rng = rng_for(2)
    out, n_in = 14336 // scale, 4096 // scale
    T = T or 1024
    layer = linear_case(rng, "up_proj", out, n_in, T, BF16, 1e-3)
    length = (32 * MiB) // (scale * scale)
    begin = draw_offset(rng, layer.numel, length, n_in, mid_row=True)
    return layer, begin, begin + length


def config3(scale: int = 1, T: Optional[int] = None) -> List[LayerCase]:
    """One Llama-3-8B-shaped transformer block, bf16, in model order:
    q, k, v, o, gate, up, down, and two RMSNorm scale vectors.
    q/k/v share one input, gate/up share one input."""
    rng = rng_for(3)
    h, kv, ff = 4096 // scale, 1024 // scale, 14336 // scale
    T = T or 1024
    x_attn = normal(rng, (T, h), 1.0, BF16)
    x_mlp = normal(rng, (T, h), 1.0, BF16)
    layers = [
        linear_case(rng, "q_proj", h, h, T, BF16, 1e-3, X=x_attn),
        linear_case(rng, "k_proj", kv, h, T, BF16, 1e-3, X=x_attn),
        linear_case(rng, "v_proj", kv, h, T, BF16, 1e-3, X=x_attn),
        linear_case(rng, "o_proj", h, h, T, BF16, 1e-3),
        linear_case(rng, "gate_proj", ff, h, T, BF16, 1e-3, X=x_mlp),
        linear_case(rng, "up_proj", ff, h, T, BF16, 1e-3, X=x_mlp),
        linear_case(rng, "down_proj", h, ff, T, BF16, 1e-3),
        vector_case(rng, "input_norm", h, T, BF16, 1e-3),
        vector_case(rng, "post_attn_norm", h, T, BF16, 1e-3),
    ]
    return layers


def config4(scale: int = 1, T: Optional[int] = None) -> List[LayerCase]:
    """Long-context 70B-shaped MLP, bf16: gate 28672x8192 and down 8192x28672,
    T = 8192 (the split over tokens is what this one exercises)."""
    rng = rng_for(4)
    h, ff = 8192 // scale, 28672 // scale
    T = T or 8192
    return [
        linear_case(rng, "gate_proj", ff, h, T, BF16, 1e-3),
        linear_case(rng, "down_proj", h, ff, T, BF16, 1e-3),
    ]


def config4_chunks(gate_numel: int, gate_cols: int, down_numel: int, length: int = 64 * MiB):
    """The chunks of configuration 4 as lists of (tensor, begin, end), tensor 0 = gate, 1 = down, in
    the concatenated [gate | down] element space: a 128 MiB chunk (`length` elements) at a seeded
    mid-row offset, one that straddles the gate -> down boundary, and the 1 GiB budget's chunk,
    which exceeds both tensors together and so takes each whole."""
    rng = rng_for(4, 1)
    off = draw_offset(rng, gate_numel + down_numel, length, gate_cols)
    straddle = gate_numel - length // 3 - 17

    def cut(o):
        segs = []
        if o < gate_numel:
            segs.append((0, o, min(o + length, gate_numel)))
        if o + length > gate_numel:
            segs.append((1, max(o, gate_numel) - gate_numel, o + length - gate_numel))
        return segs

    return {"seeded": cut(off), "straddling": cut(straddle), "whole": [(0, 0, gate_numel), (1, 0, down_numel)]}


def config5(scale: int = 1, T: Optional[int] = None) -> LayerCase:
    """Embedding / lm_head shape, bf16: W 128256x4096, T = 4096; 90% of the
    token rows of dY are N(0, 1e-4), 10% are N(0, 1e-2)."""
    rng = rng_for(5)
    out, n_in = 128256 // scale, 4096 // scale
    T = T or 4096
    return linear_case(rng, "lm_head", out, n_in, T, BF16, 0.0, dy_rows=(1e-4, 1e-2, 0.1))


CONFIG5_CHUNK_MIB = (4, 16, 64, 256, 512)


def config5_ranges(layer: LayerCase, scale: int = 1) -> List[Tuple[int, int]]:
    rng = rng_for(5, 1)
    out = []
    for mib in CONFIG5_CHUNK_MIB:
        length = (mib * MiB // 2) // (scale * scale)
        length = min(length, layer.numel)
        b = draw_offset(rng, layer.numel, length, layer.n_in, mid_row=(length < layer.numel))
        out.append((b, b + length))
    return out
