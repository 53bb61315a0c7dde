"""Seeded synthetic LLaMA-shaped linear layers and activations.

The five workloads stand in for LLaMA-7B / 13B / 70B linear layers: only the public layer shapes are
used, every value is drawn from a seeded numpy generator.  Nothing in this module belongs to the
method (no scoring, pruning, binarisation or packing): it produces the inputs that both the library
and the CPU oracle are given.

Recipe for one layer (n outputs, k inputs, seed s):
    rng   = numpy.random.default_rng(s)
    W     = 0.02 * rng.standard_normal((n, k), float32)           weights, std 0.02
    S     = floor(0.05 * k); cols = sorted(rng.choice(k, S, replace=False))   salient columns
    'x8'  : W[:, cols] *= 8                                       salient columns 8x larger
    't3'  : W[:, cols]  = 0.02 * rng.standard_t(3, (n, S))        heavy-tailed salient columns
    xnorm = |1 + 0.3 * rng.standard_normal(k)|  (float32)         per-input-feature activation norm
Activations: x = default_rng(s + 7_000_000 + rows).standard_normal((rows, k)).astype(float16).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Tuple

import numpy as np

SALIENT_FRACTION = 0.05
WEIGHT_STD = 0.02


@dataclass(frozen=True)
class LayerSpec:
    name: str
    n: int          # output features (rows of W)
    k: int          # input features (columns of W)
    N: int          # kept weights ...
    M: int          # ... of every M consecutive input weights
    region_mode: int  # 0 = break-point search, 1 = tertile split
    salient_kind: str  # 'x8' or 't3'
    seed: int

    @property
    def n_salient(self) -> int:
        return int(np.floor(SALIENT_FRACTION * self.k))


def layer_seed(cfg: int, layer_idx: int) -> int:
    """Seed 0 for the single layer of workload 1, 1000*cfg + layer index otherwise."""
    return 0 if cfg == 1 else 1000 * cfg + layer_idx


def _specs(cfg: int, shapes: List[Tuple[str, int, int, int, int]], region_mode: int,
           salient_kind: str) -> List[LayerSpec]:
    return [LayerSpec(name, n, k, N, M, region_mode, salient_kind, layer_seed(cfg, i))
            for i, (name, n, k, N, M) in enumerate(shapes)]


# workload id -> dict(layers=[LayerSpec...], decode_batches=[...], prefill_tokens=[...])
WORKLOADS: Dict[int, dict] = {
    1: dict(
        title="single linear 4096x4096, 4:8",
        layers=_specs(1, [("linear", 4096, 4096, 4, 8)], 0, "x8"),
        decode_batches=[1], prefill_tokens=[]),
    2: dict(
        title="LLaMA-7B MLP linears, 2:4, heavy-tailed salient columns",
        layers=_specs(2, [("mlp_up", 11008, 4096, 2, 4), ("mlp_down", 4096, 11008, 2, 4)], 0, "t3"),
        decode_batches=[1, 4, 16], prefill_tokens=[]),
    3: dict(
        title="LLaMA-13B shapes, 6:8, tertile regions",
        layers=_specs(3, [("attn", 5120, 5120, 6, 8), ("mlp_up", 13824, 5120, 6, 8),
                          ("mlp_down", 5120, 13824, 6, 8)], 1, "x8"),
        decode_batches=[1, 2, 4, 8, 16, 32], prefill_tokens=[]),
    4: dict(
        title="prefill GEMM, 4:8",
        layers=_specs(4, [("attn", 4096, 4096, 4, 8), ("mlp_up", 11008, 4096, 4, 8)], 0, "x8"),
        decode_batches=[], prefill_tokens=[2048, 8192]),
    5: dict(
        title="one LLaMA-70B-shaped decoder layer, layer-wise N:M mix",
        layers=_specs(5, [("q", 8192, 8192, 6, 8), ("k", 1024, 8192, 6, 8),
                          ("v", 1024, 8192, 6, 8), ("o", 8192, 8192, 6, 8),
                          ("gate", 28672, 8192, 4, 8), ("up", 28672, 8192, 4, 8),
                          ("down", 8192, 28672, 2, 4)], 0, "x8"),
        decode_batches=[1], prefill_tokens=[2048]),
}


def cols_to_bitmap(cols: np.ndarray, k: int) -> np.ndarray:
    """uint32 words, bit b of word w set iff column 32*w + b is listed."""
    bits = np.zeros(k, dtype=np.uint8)
    bits[np.asarray(cols, dtype=np.int64)] = 1
    return np.packbits(bits, bitorder="little").view("<u4").copy()


def make_layer(n: int, k: int, seed: int, salient_kind: str = "x8",
               n_salient: int | None = None) -> dict:
    """Weights, activation-norm vector and salient column set of one synthetic layer."""
    rng = np.random.default_rng(seed)
    W = (WEIGHT_STD * rng.standard_normal((n, k), dtype=np.float32)).astype(np.float32)
    S = int(np.floor(SALIENT_FRACTION * k)) if n_salient is None else int(n_salient)
    cols = np.sort(rng.choice(k, S, replace=False)).astype(np.int64)
    if S > 0:
        if salient_kind == "x8":
            W[:, cols] *= np.float32(8.0)
        elif salient_kind == "t3":
            W[:, cols] = (WEIGHT_STD * rng.standard_t(3, (n, S))).astype(np.float32)
        else:
            raise ValueError(f"unknown salient_kind {salient_kind!r}")
    xnorm = np.abs(1.0 + 0.3 * rng.standard_normal(k)).astype(np.float32)
    return dict(W=np.ascontiguousarray(W), xnorm=xnorm, sal_cols=cols,
                sal_bitmap=cols_to_bitmap(cols, k))


def make_x(rows: int, k: int, seed: int) -> np.ndarray:
    """fp16 activations, standard normal, (rows, k) row-major."""
    rng = np.random.default_rng(seed + 7_000_000 + rows)
    return rng.standard_normal((rows, k)).astype(np.float16)
