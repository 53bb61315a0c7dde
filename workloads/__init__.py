"""Seeded synthetic inputs shared by the tests, the benchmark and the oracle's callers.

Holds no arithmetic of the method: only random matrices, vectors and the table of workloads.
"""
from .synth import (  # noqa: F401
    LayerSpec,
    WORKLOADS,
    layer_seed,
    make_layer,
    make_x,
    cols_to_bitmap,
)
