"""Seeded synthetic inputs for the VQ matrix-vector path.

This module is shared by the CPU oracle's tests and by the GPU library's
tests/bench.  It holds no arithmetic of the method: it only names the
workload shapes and draws random bytes / fp16 values of the right sizes.

Canonical storage (what the arrays returned here mean) follows the paper's
representation: a weight matrix W[out, in] is tiled into groups of
``group_rows x group_cols`` weights (Sec. 4, "a group of 2,048 weights is 8
rows by 256 columns"); every group owns a codebook of ``k`` centroids of
``d`` fp16 values (Sec. 2.1) and stores one ``index_bits``-bit index per run
of ``d`` consecutive columns (Sec. 4: d columns are quantised at a time).
The byte-level order inside those arrays is fixed by the oracle, not here:
the generators only need the total sizes, because a uniformly random byte
stream *is* a uniformly random stream of 4- or 8-bit indices.
"""
from __future__ import annotations

from dataclasses import dataclass
import numpy as np

__all__ = [
    "VQShape", "CONFIGS", "LLAMA7B_LAYER", "seed_for", "canonical_sizes",
    "make_weights", "make_x", "make_X", "llama7b_pass_shapes",
]


@dataclass(frozen=True)
class VQShape:
    """Shape parameters of one vector-quantised matrix (no data)."""
    out_features: int
    in_features: int
    k: int
    index_bits: int
    group_rows: int = 8
    group_cols: int = 256
    d: int = 2

    @property
    def n_groups(self) -> int:
        return (self.out_features // self.group_rows) * (self.in_features // self.group_cols)

    @property
    def vectors_per_group(self) -> int:
        return self.group_rows * self.group_cols // self.d


def canonical_sizes(s: VQShape) -> tuple[int, int]:
    """(index bytes, codebook bytes) of the canonical arrays for shape ``s``."""
    idx_group_bits = s.vectors_per_group * s.index_bits
    assert idx_group_bits % 8 == 0
    return s.n_groups * (idx_group_bits // 8), s.n_groups * s.k * s.d * 2


# The five workload families; names are used as bench/test ids.
CONFIGS = {
    "tiny_256x256_k16": VQShape(256, 256, 16, 4),
    "attn_4096x4096_k16": VQShape(4096, 4096, 16, 4),
    "mlp_up_11008x4096_k256": VQShape(11008, 4096, 256, 8),
    "mlp_down_4096x11008_k256": VQShape(4096, 11008, 256, 8),
    "mlp_up_11008x4096_k16": VQShape(11008, 4096, 16, 4),
    "mlp_down_4096x11008_k16": VQShape(4096, 11008, 16, 4),
}

# One Llama-7B decoder layer as (name, shape key) in execution order.
LLAMA7B_LAYER = (
    ("q_proj", "attn_4096x4096_k16"),
    ("k_proj", "attn_4096x4096_k16"),
    ("v_proj", "attn_4096x4096_k16"),
    ("o_proj", "attn_4096x4096_k16"),
    ("gate_proj", "mlp_up_11008x4096_k16"),
    ("up_proj", "mlp_up_11008x4096_k16"),
    ("down_proj", "mlp_down_4096x11008_k16"),
)
LLAMA7B_N_LAYERS = 32

_BASE_SEED = 15319 * 10


def seed_for(name: str, layer: int = 0, matrix: int = 0) -> int:
    """Deterministic seed for a named workload (and layer/matrix for the 7B pass)."""
    names = sorted(CONFIGS)
    return _BASE_SEED + 1000 * names.index(name) + 10 * layer + matrix


def make_weights(s: VQShape, seed: int, cb_std: float = 0.02):
    """Random canonical (idx_bytes uint8[...], codebooks float16[n_groups,k,d]).

    Indices are uniform (every byte uniform in [0,256) gives uniform 4- or 8-bit
    indices); centroids are N(0, cb_std) rounded to fp16.
    """
    assert s.index_bits in (4, 8), "byte-uniform draw is only uniform for 4/8-bit indices"
    rng = np.random.default_rng(seed)
    idx_bytes, _ = canonical_sizes(s)
    idx = rng.integers(0, 256, size=idx_bytes, dtype=np.uint8)
    cb = rng.normal(0.0, cb_std, size=(s.n_groups, s.k, s.d)).astype(np.float16)
    return idx, cb


def make_x(n: int, seed: int) -> np.ndarray:
    """Activation vector x[n], fp16, ~N(0,1)."""
    rng = np.random.default_rng(seed ^ 0x5EED)
    return rng.standard_normal(n).astype(np.float16)


def make_X(n: int, batch: int, seed: int) -> np.ndarray:
    """Activation matrix X[n, batch] (batch contiguous), fp16, ~N(0,1)."""
    rng = np.random.default_rng(seed ^ 0xBA7C)
    return rng.standard_normal((n, batch)).astype(np.float16)


def llama7b_pass_shapes():
    """The 224 (layer, name, VQShape, seed) items of one per-token weight pass."""
    items = []
    for layer in range(LLAMA7B_N_LAYERS):
        for m, (name, key) in enumerate(LLAMA7B_LAYER):
            items.append((layer, name, CONFIGS[key], seed_for(key, layer, m)))
    return items
