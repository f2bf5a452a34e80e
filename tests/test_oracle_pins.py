"""Pins for the CPU oracle: values and identities fixed by the paper and by
arithmetic, none of them computed by the oracle itself.

Each test names the mistake it is meant to catch.
"""
import math
from fractions import Fraction

import numpy as np
import pytest

import oracle
from oracle import VQFormat
import workloads
from golden_io import read_case, read_bpv_table

GOLDEN_CASES = ["decode_2x4_k4_b2.txt", "decode_1x8_k16_b4.txt", "decode_1x16_k8_b3.txt",
                "decode_2x8_k4_b2_d1.txt"]


def _fmt(case):
    f = case["format"]
    return VQFormat(f["out"], f["in"], f["k"], f["index_bits"], f["group_rows"], f["group_cols"], f["d"])


# ---------------------------------------------------------------- hand-worked values
@pytest.mark.parametrize("name", GOLDEN_CASES)
def test_golden_decode(name):
    """Wrong group order, vector order, nibble/bit order or (j,t) transposition fails here."""
    case = read_case(name)
    f = _fmt(case)
    cb = case["codebook"].astype(np.float16)
    W = oracle.decode_dense(f, case["idx"], cb).view(np.float16).astype(np.float64)
    np.testing.assert_array_equal(W, case["W"])


@pytest.mark.parametrize("name", GOLDEN_CASES)
def test_golden_gemv_and_gemm(name):
    """Transposed operand / dropped column fails here (values are exact in fp64)."""
    case = read_case(name)
    f = _fmt(case)
    cb = case["codebook"].astype(np.float16)
    y = oracle.gemv(f, case["idx"], cb, case["x"].astype(np.float16))
    np.testing.assert_array_equal(y, case["y"])
    X = np.stack([case["x"], 2 * case["x"], -case["x"]], axis=1).astype(np.float16)
    Y = oracle.gemm(f, case["idx"], cb, X)
    np.testing.assert_array_equal(Y, np.stack([case["y"], 2 * case["y"], -case["y"]], axis=1))


@pytest.mark.parametrize("name", GOLDEN_CASES)
def test_golden_decode_element(name):
    case = read_case(name)
    f = _fmt(case)
    cb = case["codebook"].astype(np.float16)
    for r in range(f.out_features):
        for c in range(f.in_features):
            bits = oracle.decode_element(f, case["idx"], cb, r, c)
            assert np.array([bits], dtype=np.uint16).view(np.float16)[0] == case["W"][r, c]


# ---------------------------------------------------------------- closed forms
def test_bpv_paper_rows():
    """Sec. 4 formula against the bits-per-value the paper prints."""
    for bpv, d, k, l, bc in read_bpv_table():
        assert oracle.bits_per_value(k, d, bc, l) == pytest.approx(bpv, abs=1e-12), (bpv, d, k, l)


@pytest.mark.parametrize("key,bpv", [
    ("tiny_256x256_k16", 2.25), ("attn_4096x4096_k16", 2.25),
    ("mlp_up_11008x4096_k256", 8.0), ("mlp_down_4096x11008_k256", 8.0),
    ("mlp_up_11008x4096_k16", 2.25), ("mlp_down_4096x11008_k16", 2.25),
])
def test_buffer_sizes_reproduce_bpv(key, bpv):
    """Stored bytes*8/weights must equal the closed form with fp16 centroids (b_c = 16)."""
    s = workloads.CONFIGS[key]
    f = VQFormat(s.out_features, s.in_features, s.k, s.index_bits, s.group_rows, s.group_cols, s.d)
    ib, cb = oracle.canonical_sizes(f)
    assert (ib, cb) == workloads.canonical_sizes(s)
    assert (ib + cb) * 8 / (s.out_features * s.in_features) == bpv
    assert oracle.bits_per_value(s.k, s.d, 16, s.group_rows * s.group_cols) == bpv


def test_algorithmic_bytes_of_the_configs():
    """Byte counts used for the roofline (indices + codebooks + x + y as fp16)."""
    def total(key):
        s = workloads.CONFIGS[key]
        ib, cb = workloads.canonical_sizes(s)
        return ib + cb + 2 * s.in_features + 2 * s.out_features
    assert total("tiny_256x256_k16") == 19456
    assert total("attn_4096x4096_k16") == 4734976
    assert total("mlp_up_11008x4096_k256") == 45118976
    assert total("mlp_down_4096x11008_k256") == 45118976
    per_layer = sum(total(k) for _, k in workloads.LLAMA7B_LAYER)
    assert per_layer == 57074176
    assert per_layer * workloads.LLAMA7B_N_LAYERS == 1826373632
    assert len(workloads.llama7b_pass_shapes()) == 224


def test_fp16_widening_is_the_ieee_value():
    """fp16 -> fp64 spot values from the binary16 definition (sign, 5-bit exponent bias 15, 10-bit fraction)."""
    bits = np.array([0x3C00, 0xC000, 0x7BFF, 0x0001, 0x0400, 0x8000, 0x3555], dtype=np.uint16)
    want = [1.0, -2.0, 65504.0, 2.0 ** -24, 2.0 ** -14, -0.0, (1 + 0x155 / 1024) * 2.0 ** -2]
    got = bits.view(np.float16).astype(np.float64)
    assert list(got) == want
    assert math.copysign(1.0, got[5]) == -1.0


# ---------------------------------------------------------------- structural invariants
def _bit_pack(indices, bits):
    """Test-local packer (little-endian bit stream), scalar Python on purpose."""
    total = len(indices) * bits
    assert total % 8 == 0
    out = bytearray(total // 8)
    for v, j in enumerate(indices):
        for b in range(bits):
            if (int(j) >> b) & 1:
                pos = v * bits + b
                out[pos // 8] |= 1 << (pos % 8)
    return np.frombuffer(bytes(out), dtype=np.uint8)


SMALL_FORMATS = [
    VQFormat(16, 512, 16, 4),            # 2 x 2 groups of 8 x 256
    VQFormat(8, 768, 256, 8),            # 1 x 3 groups
    VQFormat(6, 24, 64, 6, 2, 12, 2),    # 6-bit indices, 3 x 2 groups of 2 x 12
    VQFormat(4, 16, 4, 2, 4, 8, 4),      # d = 4
    VQFormat(3, 8, 8, 3, 1, 8, 1),       # d = 1
]


@pytest.mark.parametrize("f", SMALL_FORMATS, ids=str)
def test_coordinate_revealing_codebook(f):
    """Centroid (g, j) stores values that spell out g, j and t, so each decoded element
    names the group, index and lane that produced it; the expected triple is
    recomputed here element by element with divmod."""
    rng = np.random.default_rng(7)
    per_group = [rng.integers(0, f.k, size=f.vectors_per_group) for _ in range(f.n_groups)]
    idx = np.concatenate([_bit_pack(p, f.index_bits) for p in per_group])
    # value = g*k*d + j*d + t  (all < 2048 for these formats, exact in fp16)
    cb = np.arange(f.n_groups * f.k * f.d, dtype=np.float64).reshape(f.n_groups, f.k, f.d)
    assert cb.max() < 2048
    W = oracle.decode_dense(f, idx, cb.astype(np.float16)).view(np.float16).astype(np.int64)
    for r in range(f.out_features):
        rb, lr = divmod(r, f.group_rows)
        for c in range(f.in_features):
            cblk, lc = divmod(c, f.group_cols)
            vec, t = divmod(lc, f.d)
            g = rb * (f.in_features // f.group_cols) + cblk
            j = per_group[g][lr * (f.group_cols // f.d) + vec]
            assert W[r, c] == (g * f.k + j) * f.d + t, (r, c)


@pytest.mark.parametrize("f", SMALL_FORMATS, ids=str)
def test_one_centroid_codebook_gives_constant_rows(f):
    """All k entries equal => W is the centroid tiled, whatever the indices; and
    y[r] = sum_t a_t * (sum of x over columns congruent to t mod d)."""
    rng = np.random.default_rng(11)
    nb = oracle.canonical_sizes(f)[0]
    if f.k == 1 << f.index_bits:
        idx = rng.integers(0, 256, size=nb, dtype=np.uint8)
    else:
        idx = np.zeros(nb, dtype=np.uint8)
    a = np.array([0.375, -1.25, 2.5, -0.0625][: f.d])
    cb = np.broadcast_to(a, (f.n_groups, f.k, f.d)).astype(np.float16)
    W = oracle.decode_dense(f, idx, cb).view(np.float16).astype(np.float64)
    np.testing.assert_array_equal(W, np.tile(a, (f.out_features, f.in_features // f.d)))
    x = rng.integers(-8, 9, size=f.in_features).astype(np.float16)
    y = oracle.gemv(f, idx, cb, x)
    want = sum(a[t] * x[t::f.d].astype(np.float64).sum() for t in range(f.d))
    np.testing.assert_array_equal(y, np.full(f.out_features, want))


@pytest.mark.parametrize("f", SMALL_FORMATS, ids=str)
def test_identity_like_codebook_reconstructs_exactly(f):
    """Build W whose d-vectors take at most k distinct values per group, encode it with
    a test-local encoder, and require decode == W bit for bit."""
    rng = np.random.default_rng(13)
    n_cb = f.in_features // f.group_cols
    W = np.zeros((f.out_features, f.in_features), dtype=np.float16)
    cb = np.zeros((f.n_groups, f.k, f.d), dtype=np.float16)
    chunks = []
    for g in range(f.n_groups):
        rb, cblk = divmod(g, n_cb)
        palette = rng.standard_normal((f.k, f.d)).astype(np.float16)
        cb[g] = palette
        choice = rng.integers(0, f.k, size=(f.group_rows, f.group_cols // f.d))
        tile = palette[choice].reshape(f.group_rows, f.group_cols)
        W[rb * f.group_rows:(rb + 1) * f.group_rows, cblk * f.group_cols:(cblk + 1) * f.group_cols] = tile
        chunks.append(_bit_pack(choice.ravel(), f.index_bits))
    idx = np.concatenate(chunks)
    got = oracle.decode_dense(f, idx, cb)
    np.testing.assert_array_equal(got, W.view(np.uint16))
    # and the matvec is the dense matvec of that W (brute force with exact rationals)
    x = rng.integers(-4, 5, size=f.in_features).astype(np.float16)
    y = oracle.gemv(f, idx, cb, x)
    for r in range(f.out_features):
        exact = sum(Fraction(float(W[r, c])) * Fraction(float(x[c])) for c in range(f.in_features))
        assert abs(Fraction(float(y[r])) - exact) <= abs(exact) * Fraction(1, 10 ** 12) + Fraction(1, 10 ** 15)


def test_relabelling_a_codebook_does_not_change_W():
    """Permute each codebook and remap its indices: the decoded matrix must not move."""
    f = VQFormat(16, 512, 256, 8)
    rng = np.random.default_rng(17)
    idx = rng.integers(0, 256, size=oracle.canonical_sizes(f)[0], dtype=np.uint8)
    cb = rng.standard_normal((f.n_groups, f.k, f.d)).astype(np.float16)
    W0 = oracle.decode_dense(f, idx, cb)
    idx2 = idx.copy().reshape(f.n_groups, -1)
    cb2 = cb.copy()
    for g in range(f.n_groups):
        perm = rng.permutation(f.k)          # new position of old entry j is perm[j]
        cb2[g, perm] = cb[g]
        idx2[g] = perm[idx2[g]].astype(np.uint8)
    np.testing.assert_array_equal(oracle.decode_dense(f, idx2.ravel(), cb2), W0)


def test_unit_vectors_pick_out_columns():
    """x = e_c must return column c of the decoded matrix (catches W^T x and index slips)."""
    s = workloads.CONFIGS["tiny_256x256_k16"]
    f = VQFormat(s.out_features, s.in_features, s.k, s.index_bits)
    idx, cb = workloads.make_weights(s, 3)
    W = oracle.decode_dense(f, idx, cb).view(np.float16).astype(np.float64)
    for c in (0, 1, 2, 127, 128, 255):
        e = np.zeros(f.in_features, dtype=np.float16)
        e[c] = 1
        np.testing.assert_array_equal(oracle.gemv(f, idx, cb, e), W[:, c])


def test_gemv_matches_scalar_walk_with_fsum():
    """Every y[r] against math.fsum over decode_element (different code path, exact summation)."""
    s = workloads.CONFIGS["tiny_256x256_k16"]
    f = VQFormat(s.out_features, s.in_features, s.k, s.index_bits)
    idx, cb = workloads.make_weights(s, 5)
    x = workloads.make_x(s.in_features, 5)
    y = oracle.gemv(f, idx, cb, x)
    x64 = x.astype(np.float64)
    for r in (0, 7, 8, 100, 255):
        row = [np.array([oracle.decode_element(f, idx, cb, r, c)], dtype=np.uint16).view(np.float16)[0]
               for c in range(f.in_features)]
        exact = math.fsum(float(w) * float(xc) for w, xc in zip(row, x64))
        assert y[r] == pytest.approx(exact, rel=1e-12, abs=1e-15)


def test_gemm_columns_are_gemvs():
    f = VQFormat(16, 512, 256, 8)
    rng = np.random.default_rng(19)
    idx = rng.integers(0, 256, size=oracle.canonical_sizes(f)[0], dtype=np.uint8)
    cb = (0.02 * rng.standard_normal((f.n_groups, f.k, f.d))).astype(np.float16)
    X = workloads.make_X(f.in_features, 5, 1)
    Y = oracle.gemm(f, idx, cb, X)
    for b in range(5):
        np.testing.assert_allclose(Y[:, b], oracle.gemv(f, idx, cb, X[:, b]), rtol=1e-13, atol=1e-16)


def test_planted_mistakes_are_caught_by_the_goldens():
    """Sanity of the pins themselves: plausible wrong readings disagree with the fixtures."""
    case = read_case("decode_1x8_k16_b4.txt")
    f = _fmt(case)
    swapped = ((case["idx"] << 4) | (case["idx"] >> 4)).astype(np.uint8)   # high nibble first
    W = oracle.decode_dense(f, swapped, case["codebook"].astype(np.float16)).view(np.float16)
    assert not np.array_equal(W.astype(np.float64), case["W"])
    case = read_case("decode_2x4_k4_b2.txt")
    f = _fmt(case)
    cb_t = case["codebook"].astype(np.float16)[:, :, ::-1].copy()           # (t) order flipped
    W = oracle.decode_dense(f, case["idx"], cb_t).view(np.float16)
    assert not np.array_equal(W.astype(np.float64), case["W"])


def test_bad_inputs_raise():
    with pytest.raises(ValueError):
        VQFormat(10, 256, 16, 4)
    with pytest.raises(ValueError):
        VQFormat(8, 256, 32, 4)
    f = VQFormat(8, 256, 16, 4)
    with pytest.raises(ValueError):
        oracle.unpack_indices(f, np.zeros(3, dtype=np.uint8))
    f3 = VQFormat(1, 16, 5, 3, 1, 16, 2)
    with pytest.raises(ValueError):
        oracle.unpack_indices(f3, np.full(3, 0xFF, dtype=np.uint8))


# ---------------------------------------------------------------- 6-bit indices, int8 tables with a scale
def test_golden_six_bit_indices():
    """The paper's deployed index width: fields that straddle byte boundaries in a 3-byte stream."""
    case = read_case("decode_1x8_k64_b6.txt")
    f = _fmt(case)
    cb = case["codebook"].astype(np.float16)
    np.testing.assert_array_equal(oracle.unpack_indices(f, case["idx"]), [[37, 2, 63, 40]])
    W = oracle.decode_dense(f, case["idx"], cb).view(np.float16).astype(np.float64)
    np.testing.assert_array_equal(W, case["W"])
    np.testing.assert_array_equal(oracle.gemv(f, case["idx"], cb, case["x"].astype(np.float16)), case["y"])


def test_golden_int8_tables_with_scale():
    """A dropped scale, a scale applied per matrix instead of per group, truncation instead of
    round-to-nearest-even (the 3*s entry is an exact tie) or a double rounding fails here."""
    case = read_case("decode_2x8_k4_b2_i8.txt")
    f = _fmt(case)
    cb = oracle.dequantise_codebooks(case["q"].astype(np.int8), case["scale"].astype(np.float16))
    assert cb.dtype == np.float16 and cb.shape == (2, 4, 2)
    W = oracle.decode_dense(f, case["idx"], cb).view(np.float16).astype(np.float64)
    np.testing.assert_array_equal(W, case["W"])
    np.testing.assert_array_equal(oracle.gemv(f, case["idx"], cb, case["x"].astype(np.float16)), case["y"])


def _fp16_nearest_even(value: Fraction) -> float:
    """Round an exact rational to fp16 by searching the table of all finite fp16 values
    (no float cast involved): nearest, ties to the value whose bit pattern is even."""
    bits = np.arange(0, 0x7C00, dtype=np.uint16)                 # non-negative finite patterns, ascending
    vals = bits.view(np.float16).astype(np.float64)
    sign = -1 if value < 0 else 1
    mag = abs(value)
    hi = int(np.searchsorted(vals, float(mag), side="left"))     # float(mag) is exact here (< 2^53 scale)
    if hi < len(vals) and Fraction(vals[hi]) == mag:
        return sign * vals[hi]
    lo = hi - 1
    assert 0 <= lo and hi < len(vals)
    d_lo, d_hi = mag - Fraction(vals[lo]), Fraction(vals[hi]) - mag
    pick = lo if d_lo < d_hi else hi if d_hi < d_lo else (lo if bits[lo] % 2 == 0 else hi)
    return sign * vals[pick]


def test_dequantise_is_one_correct_rounding_of_the_exact_product():
    """Exact rational product, rounded by table search, against the oracle on random and
    adversarial (scale, q) pairs: subnormal results, ties, the largest magnitudes."""
    rng = np.random.default_rng(7)
    scales = np.concatenate([
        rng.uniform(1e-4, 2.0, 40), [6.1e-5, 5.96e-8, 3e-7, 0.1, 1.0, 255.0, 500.0]]).astype(np.float16)
    q = rng.integers(-128, 128, size=(len(scales), 8, 2), dtype=np.int8)
    q[:, 0, 0], q[:, 0, 1], q[:, 1, 0], q[:, 1, 1] = 127, -128, 3, 1
    got = oracle.dequantise_codebooks(q, scales).astype(np.float64)
    for g in range(len(scales)):
        s = Fraction(float(scales[g]))
        for j in range(8):
            for t in range(2):
                assert got[g, j, t] == _fp16_nearest_even(s * int(q[g, j, t])), (float(scales[g]), int(q[g, j, t]))


def test_dequantise_special_scales():
    """scale 1 returns the integers, a power of two scales exactly, negating q negates W."""
    q = np.arange(-128, 128, dtype=np.int8).reshape(1, 128, 2)
    one = oracle.dequantise_codebooks(q, np.array([1.0], dtype=np.float16)).astype(np.float64)
    np.testing.assert_array_equal(one, q.astype(np.float64))
    eighth = oracle.dequantise_codebooks(q, np.array([0.125], dtype=np.float16)).astype(np.float64)
    np.testing.assert_array_equal(eighth, q.astype(np.float64) / 8)
    s = np.array([0.0371], dtype=np.float16)
    qq = np.arange(-127, 127, dtype=np.int8).reshape(1, 127, 2)
    np.testing.assert_array_equal(oracle.dequantise_codebooks((-qq).astype(np.int8), s).astype(np.float64),
                                  -oracle.dequantise_codebooks(qq, s).astype(np.float64))
    with pytest.raises(ValueError):
        oracle.dequantise_codebooks(q.astype(np.int16), np.array([1.0], dtype=np.float16))
    with pytest.raises(ValueError):
        oracle.dequantise_codebooks(q, np.array([1.0, 2.0], dtype=np.float16))


def test_deployed_format_sizes_follow_the_bpv_formula():
    """2-D VQ, 6-bit indices, int8 tables, groups of 8,192 weights: 3.125 bits per value
    (Sec. 5.1) plus the 16-bit scale per group that the formula leaves out."""
    for key in ("attn_4096x4096_k64_i8", "mlp_up_11008x4096_k64_i8", "mlp_down_4096x11008_k64_i8"):
        s = workloads.CONFIGS[key]
        f = VQFormat(s.out_features, s.in_features, s.k, s.index_bits, s.group_rows, s.group_cols, s.d)
        ib, tb = oracle.canonical_sizes_i8(f)
        assert (ib, tb) == workloads.canonical_sizes(s)
        n = s.out_features * s.in_features
        bits = Fraction((ib + tb) * 8, n)
        want = Fraction(6, 2) + Fraction(64 * 2 * 8 + 16, 8192)
        pad_bits = Fraction(((-(f.n_groups * 128)) % 16) * 8, n)
        assert bits == want + pad_bits
        assert math.isclose(oracle.bits_per_value(64, 2, 8, 8192), 3.125)


def test_i8_workload_generator_shapes():
    s = workloads.CONFIGS["tiny_64x512_k64_i8"]
    idx, q, scale = workloads.make_weights_i8(s, 3)
    assert idx.dtype == np.uint8 and idx.size == 2 * 2 * 3072
    assert q.dtype == np.int8 and q.shape == (4, 64, 2) and q.min() >= -127
    assert scale.dtype == np.float16 and scale.shape == (4,) and (scale > 0).all()
    f = VQFormat(64, 512, 64, 6, 32, 256, 2)
    I = oracle.unpack_indices(f, idx)
    assert I.shape == (4, 4096) and I.max() == 63 and I.min() == 0


# ---------------------------------------------------------------- scalar codebooks (d = 1)
def test_scalar_codebook_equals_pair_table_of_twice_the_index_width():
    """Two neighbouring b-bit indices of a d = 1 stream are one 2b-bit index of a d = 2 stream
    over the same bytes, with the table T[j] = (c[j % k], c[j // k]): the bit stream is
    little-endian, so the lower column's index is the low half of the pair index.  A swapped
    pair order or a big-endian reading of the stream fails here."""
    rng = np.random.default_rng(41)
    f1 = VQFormat(16, 512, 16, 4, 8, 256, 1)
    f2 = VQFormat(16, 512, 256, 8, 8, 256, 2)
    idx = rng.integers(0, 256, size=oracle.canonical_sizes(f1)[0], dtype=np.uint8)
    assert oracle.canonical_sizes(f2)[0] == idx.size
    c = rng.normal(0, 1, size=(f1.n_groups, 16, 1)).astype(np.float16)
    j = np.arange(256)
    T = np.stack([c[:, j % 16, 0], c[:, j // 16, 0]], axis=2)            # [g, 256, 2]
    np.testing.assert_array_equal(oracle.decode_dense(f1, idx, c), oracle.decode_dense(f2, idx, T))
    # and element by element against the nibbles read directly from the bytes
    W = oracle.decode_dense(f1, idx, c).view(np.float16)
    for (r, col) in [(0, 0), (0, 1), (3, 255), (9, 256), (15, 511), (8, 300)]:
        g = (r // 8) * 2 + col // 256
        v = (r % 8) * 256 + col % 256
        byte = int(idx[g * 1024 + v // 2])
        nib = (byte >> 4) if v % 2 else (byte & 15)
        assert W[r, col] == c[g, nib, 0]


def test_three_bit_scalar_codebook_equals_the_six_bit_pair_table():
    """The same identity one size down: d = 1, k = 8 (3-bit) over the bytes of d = 2, k = 64 (6-bit),
    T[j] = (c[j % 8], c[j // 8]); indices straddle byte boundaries here."""
    rng = np.random.default_rng(42)
    f1 = VQFormat(32, 512, 8, 3, 32, 256, 1)
    f2 = VQFormat(32, 512, 64, 6, 32, 256, 2)
    idx = rng.integers(0, 256, size=oracle.canonical_sizes(f1)[0], dtype=np.uint8)
    assert oracle.canonical_sizes(f2)[0] == idx.size
    q = rng.integers(-127, 128, size=(f1.n_groups, 8, 1), dtype=np.int8)
    scale = np.array([0.01, 0.02], dtype=np.float16)
    c = oracle.dequantise_codebooks(q, scale)
    j = np.arange(64)
    T = np.stack([c[:, j % 8, 0], c[:, j // 8, 0]], axis=2)
    np.testing.assert_array_equal(oracle.decode_dense(f1, idx, c), oracle.decode_dense(f2, idx, T))
    # the 3.125 row of the appendix table: 3 bits + (8 x 8-bit values per 8,192 weights) ~ 3.008; with the scale 3.0098
    ib, tb = oracle.canonical_sizes_i8(VQFormat(4096, 4096, 8, 3, 32, 256, 1))
    assert ib * 8 / 4096 ** 2 == 3.0 and tb == 2048 * 8 + 2048 * 2


def test_two_bit_scalar_codebook_per_row_equals_the_four_bit_pair_table():
    """One size further down, with one codebook per row of a col-block (groups of 1 x 256, the 1D
    2.125 row of the appendix table): d = 1, k = 4 over the bytes of d = 2, k = 16 with the same
    1 x 256 groups and T[j] = (c[j % 4], c[j // 4]); and element by element against the 2-bit
    fields read directly from the bytes, where a wrong group order (col-block-major instead of
    row-major) or a wrong field order inside a byte fails."""
    rng = np.random.default_rng(43)
    f1 = VQFormat(6, 512, 4, 2, 1, 256, 1)
    f2 = VQFormat(6, 512, 16, 4, 1, 256, 2)
    idx = rng.integers(0, 256, size=oracle.canonical_sizes(f1)[0], dtype=np.uint8)
    assert idx.size == 6 * 512 // 4 == oracle.canonical_sizes(f2)[0]
    q = rng.integers(-127, 128, size=(f1.n_groups, 4, 1), dtype=np.int8)
    scale = rng.uniform(0.001, 0.01, size=f1.n_groups).astype(np.float16)
    c = oracle.dequantise_codebooks(q, scale)
    j = np.arange(16)
    T = np.stack([c[:, j % 4, 0], c[:, j // 4, 0]], axis=2)
    np.testing.assert_array_equal(oracle.decode_dense(f1, idx, c), oracle.decode_dense(f2, idx, T))
    W = oracle.decode_dense(f1, idx, c).view(np.float16)
    for (r, col) in [(0, 0), (0, 1), (0, 3), (0, 4), (3, 255), (3, 256), (5, 511), (4, 300)]:
        g = r * 2 + col // 256
        v = col % 256
        field = (int(idx[g * 64 + v // 4]) >> (2 * (v % 4))) & 3
        assert W[r, col] == np.float16(np.float16(q[g, field, 0]) * scale[g])
    # 2 bits + (4 x 8-bit values per 256 weights) = 2.125, the figure the table prints; 2.1875 with the scale
    assert oracle.bits_per_value(4, 1, 8, 256) == 2.125
    # the 2D rows at 2 bits per dimension: groups of 2,048 weights give 2.125, groups of 1,024 give 2.25
    assert oracle.bits_per_value(16, 2, 8, 2048) == 2.125 and oracle.bits_per_value(16, 2, 8, 1024) == 2.25
    ib, tb = oracle.canonical_sizes_i8(VQFormat(4096, 4096, 4, 2, 1, 256, 1))
    assert (ib + tb) * 8 / 4096 ** 2 == 2.1875
    s = workloads.CONFIGS["attn_4096x4096_d1_k4"]
    assert workloads.canonical_sizes(s) == (ib, tb)


def test_four_bits_per_dimension_2d_setting_sizes_and_group_sharing():
    """The 2D 4.125 row of the appendix table: k = 256 (4 bits per dimension), 8-bit codebooks,
    one table per 32,768 weights (128 x 256): 4 + 256*2*8/32768 = 4.125 bits per value (the
    fp16 scale adds 16/32768).  And the rows of a tall group share its table: a group of 128
    rows decodes like 16 groups of 8 rows given copies of the table, on the same index bytes."""
    assert oracle.bits_per_value(256, 2, 8, 32768) == 4.125
    s = workloads.CONFIGS["mlp_up_11008x4096_k256_i8"]
    f = VQFormat(s.out_features, s.in_features, s.k, s.index_bits, s.group_rows, s.group_cols, s.d)
    ib, tb = oracle.canonical_sizes_i8(f)
    assert (ib, tb) == workloads.canonical_sizes(s)
    assert Fraction((ib + tb) * 8, s.out_features * s.in_features) == Fraction(4125, 1000) + Fraction(16, 32768)
    rng = np.random.default_rng(44)
    f_tall = VQFormat(256, 512, 256, 8, 128, 256, 2)
    f_flat = VQFormat(256, 512, 256, 8, 8, 256, 2)
    idx = rng.integers(0, 256, size=oracle.canonical_sizes(f_tall)[0], dtype=np.uint8)
    q = rng.integers(-127, 128, size=(f_tall.n_groups, 256, 2), dtype=np.int8)
    scale = rng.uniform(0.0005, 0.002, size=f_tall.n_groups).astype(np.float16)
    cb = oracle.dequantise_codebooks(q, scale)
    # tall group (gr, c) = rows 128*gr .. +127; its index bytes are those of flat groups (16*gr + j, c), j = 0..15
    idx_flat = np.empty_like(idx)
    cb_flat = np.empty((f_flat.n_groups, 256, 2), dtype=cb.dtype)
    for gr in range(2):
        for c in range(2):
            tall = idx[(gr * 2 + c) * 16384:(gr * 2 + c + 1) * 16384]
            for j in range(16):
                gf = (gr * 16 + j) * 2 + c
                idx_flat[gf * 1024:(gf + 1) * 1024] = tall[j * 1024:(j + 1) * 1024]
                cb_flat[gf] = cb[gr * 2 + c]
    np.testing.assert_array_equal(oracle.decode_dense(f_tall, idx, cb), oracle.decode_dense(f_flat, idx_flat, cb_flat))


def test_scalar_format_sizes_follow_the_bpv_formula():
    """d = 1, k = 16, fp16 codebooks, 8 x 256 groups: 4 + 16*16/2048 = 4.125 bits per value
    (the total of the 1D 4.125 row of the appendix table, which reaches the same overhead with
    8-bit codebooks and groups of 1,024)."""
    assert oracle.bits_per_value(16, 1, 16, 2048) == 4.125
    assert oracle.bits_per_value(16, 1, 8, 1024) == 4.125
    s = workloads.CONFIGS["mlp_up_11008x4096_d1_k16"]
    ib, cbb = workloads.canonical_sizes(s)
    assert (ib + cbb) * 8 / (s.out_features * s.in_features) == 4.125
    f = VQFormat(s.out_features, s.in_features, s.k, s.index_bits, s.group_rows, s.group_cols, s.d)
    assert oracle.canonical_sizes(f) == (ib, cbb)


# ---------------------------------------------------------------- blockwise normalisation
def test_block_scales_hand_worked_products_and_roundings():
    """Appendix "Blockwise data normalization": decoded weight = centroid value x the scale of
    its sub-row block, here fp16 x fp16 rounded once to fp16.  One group of 2 x 8, blocks of 4.
    Row 0: block 0 uses level 3 (= 2), block 1 level 0 (= 1/3 as fp16 = 1365/4096).
    Row 1: block 0 uses level 15 (= 1 + 2^-10), block 1 level 3 (= 2).
      3 x 1365/4096 = 4095/4096 needs 12 bits: a tie between 2047/2048 and 1 -> even -> 1.0
      (1 + 2^-10)^2 = 1 + 2^-9 + 2^-20 -> 1 + 2^-9;  -0.5 x 2 = -1;  0.1(fp16) x 2 = 2 x 0.1(fp16)."""
    f = VQFormat(2, 8, 4, 2, 2, 8, 2)
    tenth = float(np.float16(0.1))
    W = np.array([[1, -0.5, tenth, 4, 3, 3, -3, 0.75],
                  [1 + 2.0 ** -10, 1, -1, 2, 5, -0.5, tenth, 0]], dtype=np.float16)
    levels = np.ones((1, 16), dtype=np.float16)
    levels[0, 0] = np.float16(1 / 3)
    levels[0, 3] = 2
    levels[0, 15] = 1 + 2.0 ** -10
    codes = np.array([[3, 0], [15, 3]], dtype=np.uint8)
    third = 1365 / 4096
    assert float(levels[0, 0]) == third
    # 0.75 x 1365/4096 = 4095/16384: 4095 needs 12 bits, again a tie, to even: 4096/16384 = 0.25
    assert 0.75 * third == 4095 / 16384
    want = np.array([[2, -1, 2 * tenth, 8, 1.0, 1.0, -1.0, 0.25],
                     [1 + 2.0 ** -9, 1 + 2.0 ** -10, -(1 + 2.0 ** -10), 2 * (1 + 2.0 ** -10), 10, -1, 2 * tenth, 0]])
    got = oracle.apply_block_scales(f, W.view(np.uint16), levels, codes, block=4).view(np.float16).astype(np.float64)
    np.testing.assert_array_equal(got, want)


def test_block_scales_unit_levels_keep_every_bit_and_powers_of_two_are_exact():
    rng = np.random.default_rng(51)
    f = VQFormat(16, 512, 64, 6, 8, 256, 2)
    bits = rng.integers(0, 1 << 16, size=(16, 512), dtype=np.uint16)
    bits[(bits & 0x7C00) == 0x7C00] = 0x3C00            # no inf / NaN here
    codes = rng.integers(0, 16, size=(16, 16), dtype=np.uint8)
    ones = np.ones((f.n_groups, 16), dtype=np.float16)
    np.testing.assert_array_equal(oracle.apply_block_scales(f, bits, ones, codes), bits)   # subnormals, -0 included
    pw = np.tile(np.exp2(np.arange(-4, 12) // 2).astype(np.float16), (f.n_groups, 1))      # 2^-2 .. 2^5
    got = oracle.apply_block_scales(f, bits, pw, codes).view(np.float16).astype(np.float64)
    e = (np.arange(-4, 12) // 2)[codes.astype(np.int64)]
    want = np.ldexp(bits.view(np.float16).astype(np.float64), np.repeat(e, 32, axis=1))
    ok = (np.abs(want) < 65504) & ((np.abs(want) >= 2.0 ** -14) | (want == 0))             # stays a normal fp16
    np.testing.assert_array_equal(got[ok], want[ok])
    assert ok.mean() > 0.9


def test_block_scales_pick_the_level_of_the_right_group_and_block():
    """W = 1 everywhere and level (g, j) = 32*g + j + 1 (exact in fp16): every output element
    names its group and its block's code; expected values recomputed with divmod."""
    f = VQFormat(64, 768, 64, 6, 32, 256, 2)
    rng = np.random.default_rng(52)
    codes = rng.integers(0, 16, size=(64, 24), dtype=np.uint8)
    levels = (32 * np.arange(f.n_groups)[:, None] + np.arange(16)[None, :] + 1).astype(np.float16)
    W = np.ones((64, 768), dtype=np.float16)
    got = oracle.apply_block_scales(f, W.view(np.uint16), levels, codes).view(np.float16)
    for (r, c) in [(0, 0), (0, 31), (0, 32), (31, 255), (32, 0), (33, 256), (63, 767), (40, 500)]:
        g = (r // 32) * 3 + c // 256
        assert got[r, c] == 32 * g + int(codes[r, c // 32]) + 1
    with pytest.raises(ValueError):
        oracle.apply_block_scales(f, W.view(np.uint16), levels, codes, block=48)   # 48 does not tile 256 columns


def test_block_normalised_format_sizes():
    """32 x 256 groups, k = 64, 6-bit: 3 + (64*2*8 + 16 + 16*16)/8192 + 4/32 = 3.283 bits per value
    (index, int8 table, scale, 16 levels, one 4-bit code per 32 weights)."""
    f = VQFormat(4096, 4096, 64, 6, 32, 256, 2)
    ib, tb = oracle.canonical_sizes_bn(f)
    assert ib == oracle.canonical_sizes_i8(f)[0]
    assert tb == f.n_groups * 128 + f.n_groups * 2 + f.n_groups * 32 + 4096 * 128 // 2
    assert (ib + tb) * 8 / (4096 * 4096) == 3 + (1024 + 16 + 256) / 8192 + 4 / 32
    # 8 x 256 groups, k = 16, 4-bit (the 2.125 bpv setting): 2 + (16*2*8 + 16 + 16*16)/2048 + 4/32 = 2.383
    f = VQFormat(4096, 4096, 16, 4, 8, 256, 2)
    ib, tb = oracle.canonical_sizes_bn(f)
    assert ib == oracle.canonical_sizes_i8(f)[0]
    assert (ib + tb) * 8 / (4096 * 4096) == 2 + (256 + 16 + 256) / 2048 + 4 / 32 == 2.3828125


# ---------------------------------------------------------------- four-dimensional vectors (d = 4)
def test_golden_four_dimensional_vectors():
    """A vector taken down a column instead of along the row, centroid coordinates in the wrong
    order, or vectors of a group counted column-major fail here."""
    case = read_case("decode_2x8_k4_b2_d4_i8.txt")
    f = _fmt(case)
    assert f.d == 4 and f.vectors_per_group == 4
    cb = oracle.dequantise_codebooks(case["q"].astype(np.int8), case["scale"].astype(np.float16))
    assert cb.shape == (1, 4, 4)
    W = oracle.decode_dense(f, case["idx"], cb).view(np.float16).astype(np.float64)
    np.testing.assert_array_equal(W, case["W"])
    np.testing.assert_array_equal(oracle.gemv(f, case["idx"], cb, case["x"].astype(np.float16)), case["y"])
    for r in range(2):
        for c in range(8):
            bits = oracle.decode_element(f, case["idx"], cb, r, c)
            assert np.array([bits], dtype=np.uint16).view(np.float16)[0] == case["W"][r, c]


def test_four_dimensional_format_sizes_follow_the_bpv_formula():
    """The 4D rows of the appendix table: 8-bit indices per 4 weights, 256 x 4 int8 tables; groups of
    65,536 (256 x 256) give 2 + 256*4*8/65536 = 2.125 and groups of 32,768 (128 x 256) 2.25 bits
    per value; the fp16 scale per group adds 16 bits per group on top."""
    assert oracle.bits_per_value(256, 4, 8, 65536) == 2.125
    assert oracle.bits_per_value(256, 4, 8, 32768) == 2.25
    for rows, bpv in ((256, 2.125), (128, 2.25)):
        f = VQFormat(4096, 4096, 256, 8, rows, 256, 4)
        ib, tb = oracle.canonical_sizes_i8(f)
        assert ib == 4096 * 4096 // 4 and tb == f.n_groups * 1024 + 2 * f.n_groups
        assert (ib + tb - 2 * f.n_groups) * 8 / (4096 * 4096) == bpv


# ---------------------------------------------------------------- the bit stream against Python's big integers
def test_unpack_indices_against_big_integer_arithmetic():
    """A group's index bytes read as ONE little-endian integer: vector v is (N >> v*b) & (2^b - 1).
    Python's arbitrary-precision integers do the shifting here, for every index width from 1 to 12 bits
    (including widths that straddle one or two byte boundaries)."""
    rng = np.random.default_rng(77)
    for bits in range(1, 13):
        k = 1 << bits
        # group of 2 rows x 16 columns, d = 2 -> 16 vectors; 16 * bits is always a multiple of 8
        f = VQFormat(4, 32, k, bits, 2, 16, 2)
        nbytes = oracle.canonical_sizes(f)[0]
        idx = rng.integers(0, 256, size=nbytes, dtype=np.uint8)
        got = oracle.unpack_indices(f, idx)
        gb = f.group_index_bytes
        for g in range(f.n_groups):
            N = int.from_bytes(bytes(idx[g * gb:(g + 1) * gb]), "little")
            want = [(N >> (v * bits)) & (k - 1) for v in range(f.vectors_per_group)]
            assert list(got[g]) == want, (bits, g)
