"""Synthetic OWQ layers shaped like OPT / LLaMA projections.

A layer in "plain" form is what the storage paragraph of the paper (section
"Outlier-Aware Weight Quantization", last paragraph before the configuration
search) lists: a full d_out x d_in grid of low-bit codes whose weak-column
positions are zero-filled, a step size and a zero point per output channel or
per group of input columns, the k weak columns in fp16 and one integer index
per weak column.

Recipe (every draw comes from numpy's PCG64 seeded with `seed`):
  W      ~ N(0, 0.02)            fp32, only used to pick weak columns and to
                                  fill them
  lambda ~ LogNormal(0, 2)       stand-in for the Hessian diagonal of Eq. (6)
  idx    = ascending sort of the top-k columns by lambda_j * ||W[:, j]||^2
           (ties: lower column index first)
  Ww     = fp16(W[:, idx])
  codes  ~ U{0 .. 2^bits - 1}    then set to 0 at the weak columns
  scale  ~ U(0.001, 0.01) -> fp16
  zero   ~ U{0 .. 2^bits - 1} -> fp16 (integer valued)
  x      = fp16(N(0, 1) * m),  m = outlier factor at the weak columns, else 1
The real checkpoints and calibration data the paper quantises are not
available; these draws stand in for them with the same shapes and layout.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np


@dataclass(frozen=True)
class LayerSpec:
    name: str
    d_in: int
    d_out: int
    bits: int
    group_size: int  # 0 = one (scale, zero) per output channel
    k: int
    seed: int
    outlier: float = 20.0  # factor on x at the weak columns


@dataclass
class Layer:
    spec: LayerSpec
    codes: np.ndarray      # uint8  [d_out, d_in], values < 2^bits, 0 at weak columns
    scale: np.ndarray      # fp16   [d_out, G]
    zero: np.ndarray       # fp16   [d_out, G]
    weak_idx: np.ndarray   # int32  [k], strictly ascending
    weak_w: np.ndarray     # fp16   [d_out, k]

    @property
    def d_in(self) -> int:
        return self.spec.d_in

    @property
    def d_out(self) -> int:
        return self.spec.d_out

    @property
    def bits(self) -> int:
        return self.spec.bits

    @property
    def group_size(self) -> int:
        return self.spec.group_size

    @property
    def k(self) -> int:
        return self.spec.k

    @property
    def n_groups(self) -> int:
        return 1 if self.spec.group_size == 0 else -(-self.spec.d_in // self.spec.group_size)


def _top_k_columns(score: np.ndarray, k: int) -> np.ndarray:
    """Indices of the k largest scores, ties broken towards the lower index, ascending."""
    if k == 0:
        return np.zeros(0, dtype=np.int32)
    order = np.lexsort((np.arange(score.size), -score))  # primary: -score, secondary: index
    return np.sort(order[:k]).astype(np.int32)


def make_layer(spec: LayerSpec, row_chunk: int = 2048) -> Layer:
    rng = np.random.default_rng(spec.seed)
    d_out, d_in, k = spec.d_out, spec.d_in, spec.k
    levels = 1 << spec.bits
    n_groups = 1 if spec.group_size == 0 else -(-d_in // spec.group_size)

    lam = rng.lognormal(mean=0.0, sigma=2.0, size=d_in)
    # W is drawn in row chunks from a child generator so that big layers never
    # hold the fp32 matrix whole; the weak columns are kept as they go by.
    w_rng = np.random.default_rng([spec.seed, 1])
    col_sq = np.zeros(d_in, dtype=np.float64)
    chunks = []
    for r0 in range(0, d_out, row_chunk):
        r1 = min(d_out, r0 + row_chunk)
        w = w_rng.normal(0.0, 0.02, size=(r1 - r0, d_in)).astype(np.float32)
        col_sq += np.einsum("ij,ij->j", w, w, dtype=np.float64)
        chunks.append(w if k else None)
    weak_idx = _top_k_columns(lam * col_sq, k)
    if k:
        weak_w = np.concatenate([c[:, weak_idx] for c in chunks], axis=0).astype(np.float16)
    else:
        weak_w = np.zeros((d_out, 0), dtype=np.float16)
    del chunks

    codes = rng.integers(0, levels, size=(d_out, d_in), dtype=np.uint8)
    codes[:, weak_idx] = 0
    scale = rng.uniform(0.001, 0.01, size=(d_out, n_groups)).astype(np.float16)
    zero = rng.integers(0, levels, size=(d_out, n_groups)).astype(np.float16)
    return Layer(spec, codes, scale, zero, weak_idx, weak_w)


def make_weights(d_out: int, d_in: int, k: int, seed: int, weak_gain: float = 6.0,
                 tail: float = 0.002, row_chunk: int = 2048):
    """fp16 weights for the configuration search and the weak columns to leave out.

    W ~ N(0, 0.02); a fraction `tail` of the entries is multiplied by U(3, 10) (the long tail
    that a narrowed range cuts off); the k weak columns (top-k of lambda_i * |W_:,i|^2 with
    lambda ~ LogNormal(0, 2), as for the layers) are multiplied by `weak_gain`: large values
    that would dominate the range if they were not left out.  Returns (w [d_out, d_in] fp16,
    weak_idx int32 [k] ascending)."""
    rng = np.random.default_rng([seed, 7])
    lam = rng.lognormal(mean=0.0, sigma=2.0, size=d_in)
    w16 = np.empty((d_out, d_in), dtype=np.float16)
    col_sq = np.zeros(d_in, dtype=np.float64)
    for r0 in range(0, d_out, row_chunk):
        r1 = min(d_out, r0 + row_chunk)
        w = rng.normal(0.0, 0.02, size=(r1 - r0, d_in)).astype(np.float32)
        big = rng.random(size=w.shape, dtype=np.float32) < tail
        w = np.where(big, w * rng.uniform(3.0, 10.0, size=w.shape).astype(np.float32), w)
        col_sq += np.einsum("ij,ij->j", w, w, dtype=np.float64)
        w16[r0:r1] = w.astype(np.float16)
    weak_idx = _top_k_columns(lam * col_sq, k)
    if k:
        w16[:, weak_idx] = (w16[:, weak_idx].astype(np.float32) * weak_gain).astype(np.float16)
    return w16, weak_idx


def make_x(layer: Layer, batch: int, seed: Optional[int] = None,
           mean: float = 0.0) -> np.ndarray:
    """fp16 activations [batch, d_in]; weak columns carry the outlier factor."""
    s = layer.spec.seed if seed is None else seed
    rng = np.random.default_rng([s, 2, batch])
    x = rng.normal(mean, 1.0, size=(batch, layer.d_in))
    m = np.ones(layer.d_in)
    m[layer.weak_idx] = layer.spec.outlier
    return (x * m).astype(np.float16)


def _seed(cfg: int, layer_id: int) -> int:
    return 1000 * cfg + layer_id


# The workload families: 0-4 = position in the benchmark's config list; 5 and 6 are extra layers.
CONFIGS = {
    0: [LayerSpec("tiny", 1024, 1024, 4, 0, 8, _seed(0, 0), outlier=1.0)],
    1: [LayerSpec("opt6.7b.attn", 4096, 4096, 3, 0, 32, _seed(1, 0))],
    2: [LayerSpec("opt6.7b.fc1", 4096, 16384, 3, 128, 32, _seed(2, 0)),
        LayerSpec("opt6.7b.fc2", 16384, 4096, 3, 128, 128, _seed(2, 1))],
    3: [LayerSpec("llama13b.qkvo", 5120, 5120, 4, 128, 51, _seed(3, 0)),
        LayerSpec("llama13b.gate_up", 5120, 13824, 4, 128, 51, _seed(3, 1)),
        LayerSpec("llama13b.down", 13824, 5120, 4, 128, 138, _seed(3, 2))],
    4: [LayerSpec("opt66b.fc1", 9216, 36864, 3, 0, 64, _seed(4, 0)),
        LayerSpec("opt66b.fc2", 36864, 9216, 3, 0, 256, _seed(4, 1))],
    # the layer the bandwidth target is stated on: 16384 -> 4096, per channel
    5: [LayerSpec("target.16384x4096", 16384, 4096, 3, 0, 128, _seed(5, 0))],
    # shapes no launch model was fitted on: a hidden size that is not a power of two, and a very wide FFN pair
    6: [LayerSpec("unseen.7168x7168", 7168, 7168, 3, 128, 72, 9001),
        LayerSpec("unseen.8192x28672", 8192, 28672, 4, 128, 82, 9002),
        LayerSpec("unseen.28672x8192", 28672, 8192, 4, 0, 287, 9003)],
}


def config_layers(cfg: int):
    return list(CONFIGS[cfg])
