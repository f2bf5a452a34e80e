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
stream *is* a uniformly random stream of b-bit indices whenever k = 2^b.
"""
from __future__ import annotations

from dataclasses import dataclass
import numpy as np

__all__ = [
    "VQShape", "CONFIGS", "LLAMA7B_LAYER", "seed_for", "canonical_sizes",
    "make_weights", "make_weights_i8", "make_x", "make_X", "llama7b_pass_shapes",
    "tables_i8_bytes", "tables_bn_bytes",
    "LLAMA7B_LAYER_K64", "LLAMA7B_LAYER_K16_I8", "LLAMA7B_LAYER_K16_I8_G4", "LLAMA7B_LAYER_K32", "LLAMA7B_LAYER_D1_K16", "LLAMA7B_LAYER_K64_BN", "LLAMA7B_LAYER_K16_BN", "make_weights_bn", "LLAMA7B_LAYER_D4", "LLAMA7B_LAYER_D1_K8", "LLAMA7B_LAYER_D1_K8_BN", "LLAMA7B_LAYER_K256_BN", "LLAMA7B_LAYER_D4_BN", "LLAMA7B_LAYER_K256_I8", "LLAMA7B_LAYER_D1_K4",
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
    int8_tables: bool = False     # int8 centroids with one fp16 scale per group (Sec. 3.1)
    block_norm: bool = False      # blockwise normalisation on top (appendix): 16 levels per group,
                                  # one 4-bit code per 32 weights

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
    if s.block_norm:     # tables and scales padded to 16 bytes each, 32 bytes of levels per group, nibble codes
        return (s.n_groups * (idx_group_bits // 8),
                (s.n_groups * s.k * s.d + 15) // 16 * 16 + (2 * s.n_groups + 15) // 16 * 16 + 32 * s.n_groups
                + s.out_features * (s.in_features // 32) // 2)
    if s.int8_tables:    # int8 tables padded to 16 bytes, then one fp16 scale per group
        return s.n_groups * (idx_group_bits // 8), (s.n_groups * s.k * s.d + 15) // 16 * 16 + 2 * s.n_groups
    return s.n_groups * (idx_group_bits // 8), s.n_groups * s.k * s.d * 2


# The five workload families; names are used as bench/test ids.
CONFIGS = {
    "tiny_256x256_k16": VQShape(256, 256, 16, 4),
    "attn_4096x4096_k16": VQShape(4096, 4096, 16, 4),
    "mlp_up_11008x4096_k256": VQShape(11008, 4096, 256, 8),
    "mlp_down_4096x11008_k256": VQShape(4096, 11008, 256, 8),
    "mlp_up_11008x4096_k16": VQShape(11008, 4096, 16, 4),
    "mlp_down_4096x11008_k16": VQShape(4096, 11008, 16, 4),
    # the paper's deployed representation (Sec. 3.1, Sec. 5.1): 2-D VQ, 6-bit indices, int8
    # tables with a scale per group, groups of 8,192 weights (32 rows x 256 columns): 3.125 bpv
    # the paper's 2.125-bit setting: 2-D VQ, k = 16, int8 tables, groups of 2,048 weights
    "attn_4096x4096_k16_i8": VQShape(4096, 4096, 16, 4, 8, 256, 2, True),
    "mlp_up_11008x4096_k16_i8": VQShape(11008, 4096, 16, 4, 8, 256, 2, True),
    "mlp_down_4096x11008_k16_i8": VQShape(4096, 11008, 16, 4, 8, 256, 2, True),
    # the 2.5-bits-per-dimension 2D row of the appendix table: k = 32, 5-bit indices, int8 tables, 8 x 256 groups: 2.75 bpv
    "attn_4096x4096_k32": VQShape(4096, 4096, 32, 5, 8, 256, 2, True),
    "mlp_up_11008x4096_k32": VQShape(11008, 4096, 32, 5, 8, 256, 2, True),
    "mlp_down_4096x11008_k32": VQShape(4096, 11008, 32, 5, 8, 256, 2, True),
    # the paper's 2.25-bit 2D setting: the same with groups of 1,024 weights (4 rows x 256 columns)
    "attn_4096x4096_k16_i8_g4": VQShape(4096, 4096, 16, 4, 4, 256, 2, True),
    "mlp_up_11008x4096_k16_i8_g4": VQShape(11008, 4096, 16, 4, 4, 256, 2, True),
    "mlp_down_4096x11008_k16_i8_g4": VQShape(4096, 11008, 16, 4, 4, 256, 2, True),
    # the 4-bits-per-dimension 2D setting (the 2D 4.125 row of the appendix table): k = 256, 8-bit
    # indices, int8 tables + scale shared by groups of 32,768 weights (128 rows x 256 columns): 4.125 bpv
    "attn_4096x4096_k256_i8": VQShape(4096, 4096, 256, 8, 128, 256, 2, True),
    "mlp_up_11008x4096_k256_i8": VQShape(11008, 4096, 256, 8, 128, 256, 2, True),
    "mlp_down_4096x11008_k256_i8": VQShape(4096, 11008, 256, 8, 128, 256, 2, True),
    # four-dimensional vectors (d = 4): k = 256, one index byte per 4 weights, int8 tables + scale,
    # groups of 65,536 weights (256 rows x 256 columns): 2.125 bpv, the 4D row of the appendix table
    "attn_4096x4096_d4": VQShape(4096, 4096, 256, 8, 256, 256, 4, True),
    "mlp_up_11008x4096_d4": VQShape(11008, 4096, 256, 8, 256, 256, 4, True),
    "mlp_down_4096x11008_d4": VQShape(4096, 11008, 256, 8, 256, 256, 4, True),
    # scalar codebooks (d = 1): 16 fp16 values per 8 x 256 group, 4-bit indices: 4.125 bpv
    "attn_4096x4096_d1_k16": VQShape(4096, 4096, 16, 4, 8, 256, 1),
    "mlp_up_11008x4096_d1_k16": VQShape(11008, 4096, 16, 4, 8, 256, 1),
    "mlp_down_4096x11008_d1_k16": VQShape(4096, 11008, 16, 4, 8, 256, 1),
    # scalar codebooks at 3 bits: k = 8 int8 values + scale per 32 x 256 group (the 1D 3.125 row)
    "attn_4096x4096_d1_k8": VQShape(4096, 4096, 8, 3, 32, 256, 1, True),
    "mlp_up_11008x4096_d1_k8": VQShape(11008, 4096, 8, 3, 32, 256, 1, True),
    "mlp_down_4096x11008_d1_k8": VQShape(4096, 11008, 8, 3, 32, 256, 1, True),
    # scalar codebooks at 2 bits: k = 4 int8 values + scale per row of a col-block (groups of 1 x 256),
    # the 1D 2.125 row of the appendix table (2.1875 with the fp16 scale counted)
    "attn_4096x4096_d1_k4": VQShape(4096, 4096, 4, 2, 1, 256, 1, True),
    "mlp_up_11008x4096_d1_k4": VQShape(11008, 4096, 4, 2, 1, 256, 1, True),
    "mlp_down_4096x11008_d1_k4": VQShape(4096, 11008, 4, 2, 1, 256, 1, True),
    "tiny_64x512_k64_i8": VQShape(64, 512, 64, 6, 32, 256, 2, True),
    "attn_4096x4096_k64_i8": VQShape(4096, 4096, 64, 6, 32, 256, 2, True),
    "mlp_up_11008x4096_k64_i8": VQShape(11008, 4096, 64, 6, 32, 256, 2, True),
    "mlp_down_4096x11008_k64_i8": VQShape(4096, 11008, 64, 6, 32, 256, 2, True),
    # ... with blockwise normalisation (appendix): + 16 levels per group and a 4-bit code per 32 weights
    "attn_4096x4096_k64_bn": VQShape(4096, 4096, 64, 6, 32, 256, 2, True, True),
    "mlp_up_11008x4096_k64_bn": VQShape(11008, 4096, 64, 6, 32, 256, 2, True, True),
    "mlp_down_4096x11008_k64_bn": VQShape(4096, 11008, 64, 6, 32, 256, 2, True, True),
    # k = 16 (the 2.125 bpv setting) with blockwise normalisation: + 16 levels and 64 codes per group
    "attn_4096x4096_k16_bn": VQShape(4096, 4096, 16, 4, 8, 256, 2, True, True),
    "mlp_up_11008x4096_k16_bn": VQShape(11008, 4096, 16, 4, 8, 256, 2, True, True),
    "mlp_down_4096x11008_k16_bn": VQShape(4096, 11008, 16, 4, 8, 256, 2, True, True),
    # scalar codebooks at 3 bits with blockwise normalisation: 3.17 bpv at 32 x 256 groups
    "attn_4096x4096_d1_k8_bn": VQShape(4096, 4096, 8, 3, 32, 256, 1, True, True),
    "mlp_up_11008x4096_d1_k8_bn": VQShape(11008, 4096, 8, 3, 32, 256, 1, True, True),
    "mlp_down_4096x11008_d1_k8_bn": VQShape(4096, 11008, 8, 3, 32, 256, 1, True, True),
    # the 4.125 bpv 2D setting and the 2.125 bpv 4D setting with blockwise normalisation (+ 0.125 bpv of
    # codes and 16 levels per group)
    "attn_4096x4096_k256_bn": VQShape(4096, 4096, 256, 8, 128, 256, 2, True, True),
    "mlp_up_11008x4096_k256_bn": VQShape(11008, 4096, 256, 8, 128, 256, 2, True, True),
    "mlp_down_4096x11008_k256_bn": VQShape(4096, 11008, 256, 8, 128, 256, 2, True, True),
    "attn_4096x4096_d4_bn": VQShape(4096, 4096, 256, 8, 256, 256, 4, True, True),
    "mlp_up_11008x4096_d4_bn": VQShape(11008, 4096, 256, 8, 256, 256, 4, True, True),
    "mlp_down_4096x11008_d4_bn": VQShape(4096, 11008, 256, 8, 256, 256, 4, True, True),
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
LLAMA7B_LAYER_K64 = tuple((n, k.replace("_k16", "_k64_i8")) for n, k in LLAMA7B_LAYER)
LLAMA7B_LAYER_K256_I8 = tuple((n, k.replace("_k16", "_k256_i8")) for n, k in LLAMA7B_LAYER)
LLAMA7B_LAYER_K16_I8 = tuple((n, k + "_i8") for n, k in LLAMA7B_LAYER)
LLAMA7B_LAYER_K32 = tuple((n, k.replace("_k16", "_k32")) for n, k in LLAMA7B_LAYER)
LLAMA7B_LAYER_K16_I8_G4 = tuple((n, k + "_i8_g4") for n, k in LLAMA7B_LAYER)
LLAMA7B_LAYER_K64_BN = tuple((n, k.replace("_k16", "_k64_bn")) for n, k in LLAMA7B_LAYER)
LLAMA7B_LAYER_K16_BN = tuple((n, k + "_bn") for n, k in LLAMA7B_LAYER)
LLAMA7B_LAYER_D1_K8 = tuple((n, k.replace("_k16", "_d1_k8")) for n, k in LLAMA7B_LAYER)
LLAMA7B_LAYER_D1_K8_BN = tuple((n, k.replace("_k16", "_d1_k8_bn")) for n, k in LLAMA7B_LAYER)
LLAMA7B_LAYER_K256_BN = tuple((n, k.replace("_k16", "_k256_bn")) for n, k in LLAMA7B_LAYER)
LLAMA7B_LAYER_D4_BN = tuple((n, k.replace("_k16", "_d4_bn")) for n, k in LLAMA7B_LAYER)
LLAMA7B_LAYER_D1_K4 = tuple((n, k.replace("_k16", "_d1_k4")) for n, k in LLAMA7B_LAYER)
LLAMA7B_LAYER_D4 = tuple((n, k.replace("_k16", "_d4")) for n, k in LLAMA7B_LAYER)
LLAMA7B_LAYER_D1_K16 = tuple((n, k.replace("_k16", "_d1_k16")) for n, k in LLAMA7B_LAYER)
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
    assert s.k == 1 << s.index_bits, "a uniform byte stream is a uniform index stream only if k = 2^bits"
    assert not s.int8_tables
    rng = np.random.default_rng(seed)
    idx_bytes, _ = canonical_sizes(s)
    idx = rng.integers(0, 256, size=idx_bytes, dtype=np.uint8)
    cb = rng.normal(0.0, cb_std, size=(s.n_groups, s.k, s.d)).astype(np.float16)
    return idx, cb


def make_weights_i8(s: VQShape, seed: int, w_std: float = 0.02):
    """Random canonical (idx_bytes uint8[...], q int8[n_groups,k,d], scale float16[n_groups]).

    Indices uniform; table entries uniform in [-127, 127]; the scale of a group is drawn so
    that scale * 127 is about 3 standard deviations of an N(0, w_std) weight, varying by
    a factor of up to about 2 between groups.
    """
    assert s.k == 1 << s.index_bits and s.int8_tables
    rng = np.random.default_rng(seed)
    idx_bytes, _ = canonical_sizes(s)
    idx = rng.integers(0, 256, size=idx_bytes, dtype=np.uint8)
    q = rng.integers(-127, 128, size=(s.n_groups, s.k, s.d), dtype=np.int8)
    scale = (3.0 * w_std / 127.0 * np.exp2(rng.uniform(-0.5, 0.5, size=s.n_groups))).astype(np.float16)
    return idx, q, scale


def make_weights_bn(s: VQShape, seed: int, w_std: float = 0.02):
    """As make_weights_i8, plus the blockwise normalisation data: levels float16[n_groups, 16]
    = 2^(a_g * j + s0_g) with a_g in [0.1, 0.3] and s0_g in [-1.5, -0.5] (a log-scale grid
    spanning one to several octaves, as the appendix describes), rounded to fp16, and uniform
    4-bit codes uint8[out, in / 32]."""
    assert s.block_norm and s.int8_tables
    idx, q, scale = make_weights_i8(VQShape(s.out_features, s.in_features, s.k, s.index_bits, s.group_rows,
                                            s.group_cols, s.d, True), seed, w_std)
    rng = np.random.default_rng(seed ^ 0xB10C)
    a = rng.uniform(0.1, 0.3, size=(s.n_groups, 1))
    s0 = rng.uniform(-1.5, -0.5, size=(s.n_groups, 1))
    levels = np.exp2(a * np.arange(16)[None, :] + s0).astype(np.float16)
    codes = rng.integers(0, 16, size=(s.out_features, s.in_features // 32), dtype=np.uint8)
    return idx, q, scale, levels, codes


def tables_i8_bytes(s: VQShape, q: np.ndarray, scale: np.ndarray) -> np.ndarray:
    """The interchange table buffer of an int8-table matrix as raw bytes (byte copies only): the
    int8 tables q[n_groups, k, d] in array order, zero bytes up to a multiple of 16, then the
    fp16 scales scale[n_groups].  What the GPU library's pack step takes as input, and what the
    oracle's own reader parses back into arrays in the tests."""
    assert q.dtype == np.int8 and scale.dtype == np.float16 and s.int8_tables and not s.block_norm
    buf = np.zeros(canonical_sizes(s)[1], dtype=np.uint8)
    qb = np.ascontiguousarray(q).view(np.uint8).reshape(-1)
    sb = np.ascontiguousarray(scale).view(np.uint8).reshape(-1)
    off = (qb.size + 15) // 16 * 16
    assert off + sb.size == buf.size
    buf[:qb.size] = qb
    buf[off:] = sb
    return buf


def tables_bn_bytes(s: VQShape, q: np.ndarray, scale: np.ndarray, levels: np.ndarray,
                    codes: np.ndarray) -> np.ndarray:
    """The interchange table buffer of a block-normalised matrix as raw bytes: q and scale as in
    tables_i8_bytes, each zero-padded to a multiple of 16 bytes, then the fp16 levels[n_groups, 16],
    then the 4-bit block codes codes[out, in / 32], two per byte, even block in the low nibble
    (byte copies and nibble packing only)."""
    assert q.dtype == np.int8 and scale.dtype == np.float16 and levels.dtype == np.float16
    assert codes.dtype == np.uint8 and codes.shape[1] % 2 == 0 and s.block_norm
    buf = np.zeros(canonical_sizes(s)[1], dtype=np.uint8)
    off = 0
    for part in (q, scale):
        b = np.ascontiguousarray(part).view(np.uint8).reshape(-1)
        buf[off:off + b.size] = b
        off = (off + b.size + 15) // 16 * 16
    lb = np.ascontiguousarray(levels).view(np.uint8).reshape(-1)
    buf[off:off + lb.size] = lb
    off += lb.size
    packed = (codes[:, 0::2] | (codes[:, 1::2] << 4)).astype(np.uint8).reshape(-1)
    assert off + packed.size == buf.size
    buf[off:] = packed
    return buf


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
