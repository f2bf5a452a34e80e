"""Plain CPU oracle: what the VQ decode + matrix-vector path computes.

TEST INFRASTRUCTURE.  Slow, straightforward NumPy in fp64; imported only by
tests, the smoke check and the bench's CPU-baseline leg.  Nothing here is
shared with, derived from, or fed by the GPU library.

What is computed (paper passages followed, restated):

* Sec. 2.1: a codebook C_d = {c_1..c_k} holds k centroids of d values each;
  every run of d values of the tensor is replaced by the index of one
  centroid, stored in ceil(log2 k) bits.
* Sec. 3.1: the tensor is split into groups; each group is stored as a
  tuple (indices, lookup table, scale).  Two table types: fp16 centroids
  with the scale already folded in (a group is (indices, table)), or int8
  tables with an fp16 scale per group (dequantise_codebooks turns the
  latter into the former; everything downstream is shared).
* Sec. 4 (GPTVQ paragraph): a vector spans d consecutive *columns* of one
  row (the input dimension); groups are at most 256 columns wide, e.g.
  2,048 weights = 8 rows x 256 columns.
* Sec. 4 (Total bits per value): bpv = log2(k)/d + k*d*b_c/l.
* Sec. 3.2: at inference a block is decoded by table lookup to the native
  type and then used in the matrix-vector product.

Decoding is a table copy, so the result has a plain definition and the
oracle is that definition written out:

    W[r, c + t] = C_g[ I_g[v] ][t],   y = W x  (fp64 accumulate).

Canonical byte order (Sec. 3.2 says only that indices are stored without
padding bits between them; these are the readings this build fixes):

* groups tile W row-block-major: g = (r // gr) * (in // gc) + (c // gc);
* inside a group vectors are row-major: v = (r % gr) * (gc // d) + (c % gc) // d;
* a group's indices form a little-endian bit stream: vector v occupies bits
  [v*b, (v+1)*b) of the group's bytes, bit 0 = least significant bit of
  byte 0 (for b=4: even v in the low nibble, odd v in the high nibble;
  for b=8: byte v); groups are concatenated in g order;
* codebooks: cb[g, j, t] fp16, contiguous, same g order.

The quantiser's E- and M-step (paragraph "Codebook Initialization") follow at the end of the
file with their own header: em_assign, em_update, em_objective; then the blockwise
normalisation of the appendix: apply_block_scales, canonical_sizes_bn.

Parity pins (tests/test_oracle_*.py): hand-written tiny cases stored under
tests/golden/, a coordinate-revealing codebook, one-centroid and
identity-like codebooks, relabelling invariance, the bpv closed form,
unit-vector probes and a per-element scalar walk; hand-written hex dumps of the
int8-table buffers for read_tables_i8 / read_tables_bn; hand-worked vectors and a
planted wrong row for normwise_rel_err (the pass criterion of the product tests).
"""
from __future__ import annotations

from dataclasses import dataclass
import numpy as np


@dataclass(frozen=True)
class VQFormat:
    """Shape of one vector-quantised matrix W[out_features, in_features]."""
    out_features: int
    in_features: int
    k: int
    index_bits: int
    group_rows: int = 8
    group_cols: int = 256
    d: int = 2

    def __post_init__(self):
        if self.out_features % self.group_rows or self.in_features % self.group_cols:
            raise ValueError("matrix shape must be a multiple of the group shape")
        if self.group_cols % self.d:
            raise ValueError("group_cols must be a multiple of d")
        if self.k > (1 << self.index_bits):
            raise ValueError("index_bits too small for k")
        if (self.vectors_per_group * self.index_bits) % 8:
            raise ValueError("a group's index stream must end on a byte boundary")

    @property
    def groups_per_row(self) -> int:
        return self.in_features // self.group_cols

    @property
    def n_groups(self) -> int:
        return (self.out_features // self.group_rows) * self.groups_per_row

    @property
    def vectors_per_row(self) -> int:
        """Vectors of one row inside one group."""
        return self.group_cols // self.d

    @property
    def vectors_per_group(self) -> int:
        return self.group_rows * self.vectors_per_row

    @property
    def group_index_bytes(self) -> int:
        return self.vectors_per_group * self.index_bits // 8


def canonical_sizes(f: VQFormat) -> tuple[int, int]:
    """(bytes of packed indices, bytes of fp16 codebooks) for the whole matrix."""
    return f.n_groups * f.group_index_bytes, f.n_groups * f.k * f.d * 2


def bits_per_value(k: int, d: int, codebook_bits: int, group_size: int) -> float:
    """Sec. 4, Total bits per value: log2(k)/d + k*d*b_c/l."""
    return float(np.log2(k)) / d + k * d * codebook_bits / group_size


def unpack_indices(f: VQFormat, idx: np.ndarray) -> np.ndarray:
    """Packed index bytes -> int64[n_groups, vectors_per_group].

    Each group's bytes are expanded to a little-endian bit stream and cut into
    consecutive fields of ``index_bits`` bits (Sec. 2.1: one index of
    ceil(log2 k) bits per vector; Sec. 3.2: no padding between indices).
    """
    idx = np.ascontiguousarray(idx, dtype=np.uint8)
    if idx.size != f.n_groups * f.group_index_bytes:
        raise ValueError("index buffer has the wrong size")
    per_group = idx.reshape(f.n_groups, f.group_index_bytes)
    bits = np.unpackbits(per_group, axis=1, bitorder="little")
    fields = bits.reshape(f.n_groups, f.vectors_per_group, f.index_bits).astype(np.int64)
    weights = (1 << np.arange(f.index_bits, dtype=np.int64))
    out = fields @ weights
    if out.size and out.max() >= f.k:
        raise ValueError("index out of range for this codebook")
    return out


def decode_dense(f: VQFormat, idx: np.ndarray, cb: np.ndarray) -> np.ndarray:
    """Rebuild dense W as raw fp16 bit patterns, uint16[out, in] (Sec. 3.2 decode).

    W[r, c + t] = cb[g, I_g[v], t] with g, v as in the module header.  Pure
    copying of 16-bit patterns: subnormals, -0 and NaN payloads survive.
    """
    cb_bits = np.ascontiguousarray(cb).view(np.uint16).reshape(f.n_groups, f.k, f.d)
    I = unpack_indices(f, idx)                                  # [g, v]
    vecs = cb_bits[np.arange(f.n_groups)[:, None], I]           # [g, v, d]
    n_rb, n_cb = f.out_features // f.group_rows, f.groups_per_row
    # [row-block, col-block, row in group, vector in row, t] -> [row-block, row, col-block, vector, t]
    vecs = vecs.reshape(n_rb, n_cb, f.group_rows, f.vectors_per_row, f.d)
    W = vecs.transpose(0, 2, 1, 3, 4).reshape(f.out_features, f.in_features)
    return np.ascontiguousarray(W)


def decode_element(f: VQFormat, idx: np.ndarray, cb: np.ndarray, r: int, c: int) -> int:
    """One element of W (raw fp16 bits) by walking the definition with scalars.

    Used for sampled checks at sizes where a full decode is too slow elsewhere.
    """
    g = (r // f.group_rows) * f.groups_per_row + (c // f.group_cols)
    v = (r % f.group_rows) * f.vectors_per_row + (c % f.group_cols) // f.d
    t = (c % f.group_cols) % f.d
    base = g * f.group_index_bytes
    j = 0
    for b in range(f.index_bits):
        bit = v * f.index_bits + b
        byte = int(idx[base + bit // 8])
        j |= ((byte >> (bit % 8)) & 1) << b
    cb_bits = np.ascontiguousarray(cb).view(np.uint16).reshape(f.n_groups, f.k, f.d)
    return int(cb_bits[g, j, t])


def gemv(f: VQFormat, idx: np.ndarray, cb: np.ndarray, x: np.ndarray) -> np.ndarray:
    """y = W x in fp64, W decoded as above (fp16 -> fp64 widening is exact)."""
    W = decode_dense(f, idx, cb).view(np.float16).astype(np.float64)
    x64 = np.asarray(x, dtype=np.float16).astype(np.float64)
    if x64.shape != (f.in_features,):
        raise ValueError("x has the wrong shape")
    return W @ x64


def gemm(f: VQFormat, idx: np.ndarray, cb: np.ndarray, X: np.ndarray) -> np.ndarray:
    """Y[out, B] = W X[in, B] in fp64."""
    W = decode_dense(f, idx, cb).view(np.float16).astype(np.float64)
    X64 = np.asarray(X, dtype=np.float16).astype(np.float64)
    if X64.ndim != 2 or X64.shape[0] != f.in_features:
        raise ValueError("X has the wrong shape")
    return W @ X64


def gemv_lora(f: VQFormat, idx: np.ndarray, cb: np.ndarray, x: np.ndarray, A: np.ndarray,
              B: np.ndarray) -> np.ndarray:
    """y = W x + B (A x) in fp64: the frozen vector-quantised base matrix plus a low-rank adapter
    (Sec. 5, "Combination of GPTVQ with LoRA adapters": adapters are trained on top of the
    quantised representation and applied next to it at inference; the update is the usual
    product of a [out, rank] and a [rank, in] matrix, any scaling folded into B).

    A: fp16 [rank, in], B: fp16 [out, rank]; both widened exactly to fp64.
    """
    A64 = np.asarray(A, dtype=np.float16).astype(np.float64)
    B64 = np.asarray(B, dtype=np.float16).astype(np.float64)
    if A64.ndim != 2 or B64.ndim != 2 or A64.shape[1] != f.in_features or \
            B64.shape != (f.out_features, A64.shape[0]):
        raise ValueError("A is [rank, in], B is [out, rank]")
    x64 = np.asarray(x, dtype=np.float16).astype(np.float64)
    return gemv(f, idx, cb, x) + B64 @ (A64 @ x64)


def dequantise_codebooks(q: np.ndarray, scale: np.ndarray) -> np.ndarray:
    """Integer lookup tables with a scale factor per group -> fp16 codebooks.

    Sec. 3.1: a group is stored as the tuple (indices, lookup table, quantisation
    scale factor); the appendix on codebook compression makes 8-bit integer tables the
    default.  Sec. 3.2 decodes an index to a signed 8-bit integer.  On this path the
    native type is fp16, so a centroid value is the product scale_g * q taken exactly
    and rounded ONCE to fp16 (round to nearest even); this is what the dense
    reconstruction returns bit for bit.  q: int8[n_groups, k, d], scale: fp16[n_groups].
    """
    q = np.asarray(q)
    scale = np.asarray(scale)
    if q.dtype != np.int8 or scale.dtype != np.float16:
        raise ValueError("q must be int8 and scale fp16")
    if q.ndim != 3 or scale.shape != (q.shape[0],):
        raise ValueError("q is [n_groups, k, d], scale is [n_groups]")
    # fp16 (11 significant bits) times int8 is exact in fp64; the cast rounds once
    exact = scale.astype(np.float64)[:, None, None] * q.astype(np.float64)
    return exact.astype(np.float16)


def canonical_sizes_i8(f: VQFormat) -> tuple[int, int]:
    """(index bytes, table bytes) with int8 tables and one fp16 scale per group.

    The table buffer holds q[n_groups, k, d] int8, zero-padded to a multiple of 16
    bytes, followed by scale[n_groups] fp16.
    """
    q_bytes = f.n_groups * f.k * f.d
    return f.n_groups * f.group_index_bytes, (q_bytes + 15) // 16 * 16 + 2 * f.n_groups


def read_tables_i8(f: VQFormat, buf: np.ndarray) -> tuple[np.ndarray, np.ndarray]:
    """Canonical VQ_I8 table buffer (raw bytes) -> (q int8[n_groups, k, d], scale fp16[n_groups]).

    Sec. 3.1 stores a group as (indices, lookup table, scale).  Byte order of this build's
    interchange buffer: the tables of all groups first, group after group, inside a group
    centroid after centroid, inside a centroid coordinate after coordinate, one signed byte
    each; zero bytes up to the next multiple of 16; then one little-endian fp16 scale per
    group in the same group order.
    """
    buf = np.ascontiguousarray(buf, dtype=np.uint8).reshape(-1)
    n_q = f.n_groups * f.k * f.d
    off = (n_q + 15) // 16 * 16
    if buf.size != off + 2 * f.n_groups:
        raise ValueError("table buffer has the wrong size")
    if np.any(buf[n_q:off]):
        raise ValueError("padding bytes must be zero")
    q = buf[:n_q].view(np.int8).reshape(f.n_groups, f.k, f.d).copy()
    sb = buf[off:].reshape(f.n_groups, 2).astype(np.uint16)
    scale = (sb[:, 0] | (sb[:, 1] << 8)).astype(np.uint16).view(np.float16)
    return q, scale


def read_tables_bn(f: VQFormat, buf: np.ndarray, block: int = 32):
    """Canonical VQ_I8_BN table buffer (raw bytes) -> (q, scale, levels fp16[n_groups, 16],
    codes uint8[out, in / block]).

    Byte order: the int8 tables as in read_tables_i8, zero-padded to a multiple of 16 bytes;
    the fp16 scales, zero-padded to a multiple of 16 bytes; 16 little-endian fp16 levels per
    group, group after group; then the 4-bit block codes of the whole matrix (appendix
    "Blockwise data normalization": one code per sub-row block), row after row, block after
    block along a row, two per byte: the block with the even index in the LOW nibble.
    """
    buf = np.ascontiguousarray(buf, dtype=np.uint8).reshape(-1)
    n_q = f.n_groups * f.k * f.d
    q_end = (n_q + 15) // 16 * 16
    s_end = q_end + (2 * f.n_groups + 15) // 16 * 16
    l_end = s_end + 32 * f.n_groups
    n_blk = f.in_features // block
    if f.group_cols % block or n_blk % 2:
        raise ValueError("blocks must tile a group's columns and pair up into bytes")
    if buf.size != l_end + f.out_features * n_blk // 2:
        raise ValueError("table buffer has the wrong size")
    if np.any(buf[n_q:q_end]) or np.any(buf[q_end + 2 * f.n_groups:s_end]):
        raise ValueError("padding bytes must be zero")
    q = buf[:n_q].view(np.int8).reshape(f.n_groups, f.k, f.d).copy()
    sb = buf[q_end:q_end + 2 * f.n_groups].reshape(f.n_groups, 2).astype(np.uint16)
    scale = (sb[:, 0] | (sb[:, 1] << 8)).astype(np.uint16).view(np.float16)
    lb = buf[s_end:l_end].reshape(f.n_groups, 16, 2).astype(np.uint16)
    levels = (lb[..., 0] | (lb[..., 1] << 8)).astype(np.uint16).view(np.float16)
    cbytes = buf[l_end:].reshape(f.out_features, n_blk // 2)
    codes = np.empty((f.out_features, n_blk), dtype=np.uint8)
    codes[:, 0::2] = cbytes & 0x0F
    codes[:, 1::2] = cbytes >> 4
    return q, scale, levels, codes


def normwise_rel_err(y, y_ref) -> float:
    """||y - y_ref||_2 / ||y_ref||_2 (Frobenius for matrices), computed in fp64."""
    y = np.asarray(y, dtype=np.float64).ravel()
    y_ref = np.asarray(y_ref, dtype=np.float64).ravel()
    den = float(np.linalg.norm(y_ref))
    num = float(np.linalg.norm(y - y_ref))
    return num / den if den > 0 else (0.0 if num == 0 else float("inf"))


# ---------------------------------------------------------------------------------------------
# Codebook initialisation (Sec. 3.2 of the method, paragraph "Codebook Initialization"): the
# E- and M-step of the Hessian-weighted EM, for one matrix tiled into groups as above.
#
# Data points are the d-dimensional vectors x_i of a group (d consecutive columns of one row);
# D = diag(1 / [H^-1]_cc) has one weight per column, shared by all rows, and D_i is the d x d
# block of D on the columns of x_i.  `hdiag[c]` is that weight 1 / [H^-1]_cc.
#
#   E-step (eq. "hessian_e_step"):  a_i = argmin_m (x_i - c_m)^T D_i (x_i - c_m)
#   M-step (closed form below eq. "hessian_m_step"):
#          c_m = (sum_{i in I_m} D_i)^+ (sum_{i in I_m} D_i x_i)      (+ : pseudoinverse)
#
# With a diagonal D_i this is  sum_t h_t (x_t - c_t)^2  and a weighted mean per coordinate; the
# pseudoinverse of a zero diagonal entry is zero, so a coordinate no vector votes for (an empty
# cluster, or weights that are all zero) becomes 0.
#
# Precision: the assignment is a decision taken in floating point, and the paper does not fix
# the arithmetic.  The quantiser works on binary32 weights, so the reading taken here is the
# plainest binary32 evaluation of the printed expression: IEEE binary32, no fused operations,
# every operation rounded separately, in this order:
#   e_t = x_t - c_t;  q_t = e_t * e_t;  p_t = h_t * q_t;  dist = (p_0 + p_1) + ... ;
# the smallest distance wins and the lowest m wins a tie.  The M-step has a plain definition
# and is evaluated in binary64.
def em_assign(f: VQFormat, W: np.ndarray, hdiag: np.ndarray, cb: np.ndarray) -> np.ndarray:
    """E-step: index of the weighted-nearest centroid for every vector, uint8/uint16 [out, in/d]."""
    W = np.asarray(W)
    hdiag = np.asarray(hdiag)
    cb = np.asarray(cb)
    if W.dtype != np.float32 or hdiag.dtype != np.float32 or cb.dtype != np.float32:
        raise ValueError("the E-step is defined on binary32 inputs")
    if W.shape != (f.out_features, f.in_features) or hdiag.shape != (f.in_features,):
        raise ValueError("W is [out, in], hdiag is [in]")
    if cb.shape != (f.n_groups, f.k, f.d):
        raise ValueError("cb is [n_groups, k, d]")
    n_rb, n_cb = f.out_features // f.group_rows, f.groups_per_row
    out = np.zeros((f.out_features, f.in_features // f.d), dtype=np.uint16 if f.k > 256 else np.uint8)
    vpr = f.vectors_per_row
    for rb in range(n_rb):
        for cbk in range(n_cb):
            g = rb * n_cb + cbk
            rows = slice(rb * f.group_rows, (rb + 1) * f.group_rows)
            cols = slice(cbk * f.group_cols, (cbk + 1) * f.group_cols)
            x = W[rows, cols].reshape(f.group_rows, vpr, f.d)               # [r, v, t]
            h = hdiag[cols].reshape(vpr, f.d)                               # [v, t]
            e = x[:, :, None, :] - cb[g][None, None, :, :]                  # [r, v, m, t], binary32
            q = e * e
            p = h[None, :, None, :] * q
            dist = p[..., 0]
            for t in range(1, f.d):
                dist = dist + p[..., t]
            assert dist.dtype == np.float32
            out[rows, cbk * vpr:(cbk + 1) * vpr] = np.argmin(dist, axis=2)  # first minimum = lowest m
    return out


def em_update(f: VQFormat, W: np.ndarray, hdiag: np.ndarray, assign: np.ndarray) -> np.ndarray:
    """M-step: float64 centroids [n_groups, k, d] from the assignments of the E-step."""
    W = np.asarray(W, dtype=np.float64)
    hdiag = np.asarray(hdiag, dtype=np.float64)
    assign = np.asarray(assign)
    if W.shape != (f.out_features, f.in_features) or hdiag.shape != (f.in_features,):
        raise ValueError("W is [out, in], hdiag is [in]")
    if assign.shape != (f.out_features, f.in_features // f.d):
        raise ValueError("assign is [out, in/d]")
    if assign.size and int(assign.max()) >= f.k:
        raise ValueError("assignment out of range")
    n_rb, n_cb = f.out_features // f.group_rows, f.groups_per_row
    vpr = f.vectors_per_row
    cb = np.zeros((f.n_groups, f.k, f.d), dtype=np.float64)
    for rb in range(n_rb):
        for cbk in range(n_cb):
            g = rb * n_cb + cbk
            rows = slice(rb * f.group_rows, (rb + 1) * f.group_rows)
            cols = slice(cbk * f.group_cols, (cbk + 1) * f.group_cols)
            x = W[rows, cols].reshape(f.group_rows, vpr, f.d)
            h = np.broadcast_to(hdiag[cols].reshape(1, vpr, f.d), x.shape)
            a = assign[rows, cbk * vpr:(cbk + 1) * vpr]
            for m in range(f.k):
                sel = a == m
                den = h[sel].sum(axis=0)                                    # sum of D_i (diagonal)
                num = (h[sel] * x[sel]).sum(axis=0)                         # sum of D_i x_i
                nz = den != 0
                cb[g, m, nz] = num[nz] / den[nz]                            # pseudoinverse: 0 where den = 0
    return cb


def em_objective(f: VQFormat, W: np.ndarray, hdiag: np.ndarray, cb: np.ndarray,
                 assign: np.ndarray) -> float:
    """The EM objective (eq. "kmeans_objective") in binary64: sum_i (x_i - c_{a_i})^T D_i (x_i - c_{a_i})."""
    W = np.asarray(W, dtype=np.float64)
    hdiag = np.asarray(hdiag, dtype=np.float64)
    cb = np.asarray(cb, dtype=np.float64)
    n_cb = f.groups_per_row
    vpr = f.vectors_per_row
    total = 0.0
    for r in range(f.out_features):
        for cbk in range(n_cb):
            g = (r // f.group_rows) * n_cb + cbk
            x = W[r, cbk * f.group_cols:(cbk + 1) * f.group_cols].reshape(vpr, f.d)
            h = hdiag[cbk * f.group_cols:(cbk + 1) * f.group_cols].reshape(vpr, f.d)
            c = cb[g][assign[r, cbk * vpr:(cbk + 1) * vpr].astype(np.int64)]
            total += float((h * (x - c) ** 2).sum())
    return total


# ---------------------------------------------------------------------------------------------
# Blockwise data normalisation (appendix "Blockwise data normalization"): every sub-row of
# `block` consecutive weights inside a group has a 4-bit code, the code selects one of the
# group's 16 block scales (the appendix quantises the scales in the log domain, level j being
# 2^(a*j + s_0) with a shared by the group; here the 16 levels themselves are stored, as fp16,
# which contains that parameterisation and keeps the reconstruction exact to state), and the
# scaling is undone when a weight is decoded: the decoded weight is the centroid value times its
# block's scale.  On this path the native type is fp16: the product of the two fp16 values is
# taken exactly and rounded once to fp16 (nearest even).
def apply_block_scales(f: VQFormat, W_bits: np.ndarray, levels: np.ndarray, codes: np.ndarray,
                       block: int = 32) -> np.ndarray:
    """Dense W (raw fp16 bits, uint16[out, in]) -> W with the block scales applied (same form).

    levels: fp16[n_groups, 16]; codes: uint8[out, in / block], one 4-bit code per sub-row block
    (values 0..15), row-major like W.  The group of element (r, c) is the usual
    g = (r // group_rows) * (in // group_cols) + c // group_cols.
    """
    levels = np.asarray(levels)
    codes = np.asarray(codes)
    if levels.dtype != np.float16 or levels.shape != (f.n_groups, 16):
        raise ValueError("levels is fp16 [n_groups, 16]")
    if f.group_cols % block or codes.shape != (f.out_features, f.in_features // block):
        raise ValueError("codes is [out, in / block] and blocks must tile a group's columns")
    if codes.size and int(codes.max()) > 15:
        raise ValueError("block codes are 4-bit")
    W = np.ascontiguousarray(W_bits).view(np.float16).reshape(f.out_features, f.in_features)
    rows = np.arange(f.out_features)[:, None]
    blk = np.arange(f.in_features // block)[None, :]
    g = (rows // f.group_rows) * f.groups_per_row + (blk * block) // f.group_cols    # [out, in/block]
    S = levels[g, codes.astype(np.int64)]                                            # fp16 [out, in/block]
    S_full = np.repeat(S, block, axis=1)
    # fp16 x fp16 is exact in binary32 (22 significant bits); the cast rounds once
    with np.errstate(over="ignore", invalid="ignore"):     # products beyond fp16 become inf, as on the device
        out = (W.astype(np.float32) * S_full.astype(np.float32)).astype(np.float16)
    return np.ascontiguousarray(out).view(np.uint16)


def canonical_sizes_bn(f: VQFormat, block: int = 32) -> tuple[int, int]:
    """(index bytes, table bytes) with int8 tables, a scale per group and blockwise normalisation.

    Table buffer: q[n_groups, k, d] int8 padded to 16 bytes; scale[n_groups] fp16 padded to 16
    bytes; levels[n_groups, 16] fp16; then the 4-bit block codes of the whole matrix, row-major
    [out, in / block], two per byte (even block in the low nibble).
    """
    q_bytes = (f.n_groups * f.k * f.d + 15) // 16 * 16
    s_bytes = (2 * f.n_groups + 15) // 16 * 16
    code_bytes = f.out_features * (f.in_features // block) // 2
    return f.n_groups * f.group_index_bytes, q_bytes + s_bytes + 32 * f.n_groups + code_bytes
