"""Pins for two pieces of the oracle that every GPU parity test leans on:

* the readers of the interchange table buffers (int8 tables + scale, and the block-normalised
  variant): the bytes are written out by hand in tests/golden/tables_*.txt;
* normwise_rel_err, the pass criterion of every product test: hand-worked vectors, and a planted
  wrong row that the stated tolerances must catch.

Nothing here is computed by the functions under test.
"""
import math

import numpy as np
import pytest

import oracle
from oracle import VQFormat
import workloads
from golden_io import read_case


def _fmt(case):
    f = case["format"]
    return VQFormat(f["out"], f["in"], f["k"], f["index_bits"], f["group_rows"], f["group_cols"], f["d"])


# ---------------------------------------------------------------- int8 tables + scale
def test_read_tables_i8_hand_written_bytes():
    """Wrong order of (group, centroid, coordinate), unsigned bytes, big-endian scales, scales
    placed before the padding: each fails here."""
    case = read_case("tables_3x8_k4_i8.txt")
    f = _fmt(case)
    assert case["tables"].size == oracle.canonical_sizes_i8(f)[1] == 38
    q, scale = oracle.read_tables_i8(f, case["tables"])
    assert q.dtype == np.int8 and scale.dtype == np.float16
    np.testing.assert_array_equal(q.astype(np.int64), case["q"])
    np.testing.assert_array_equal(scale.astype(np.float64), case["scale"])


def test_read_tables_i8_rejects_bad_buffers():
    case = read_case("tables_3x8_k4_i8.txt")
    f = _fmt(case)
    with pytest.raises(ValueError):
        oracle.read_tables_i8(f, case["tables"][:-1])
    bad = case["tables"].copy()
    bad[25] = 1                                   # a padding byte
    with pytest.raises(ValueError):
        oracle.read_tables_i8(f, bad)


def test_tables_i8_writer_reproduces_the_hand_written_bytes_and_round_trips():
    """The generator-side writer (the bytes the GPU pack step is fed) against the same fixture,
    and reader(writer(arrays)) == arrays on random data of a size with padding."""
    case = read_case("tables_3x8_k4_i8.txt")
    s = workloads.VQShape(3, 8, 4, 2, 1, 8, 2, True)
    buf = workloads.tables_i8_bytes(s, case["q"].astype(np.int8), case["scale"].astype(np.float16))
    np.testing.assert_array_equal(buf, case["tables"])
    s2 = workloads.VQShape(24, 512, 16, 4, 8, 256, 2, True)      # 6 groups x 32 bytes, 12 bytes of scales
    idx, q, scale = workloads.make_weights_i8(s2, 5)
    f2 = VQFormat(24, 512, 16, 4)
    q2, sc2 = oracle.read_tables_i8(f2, workloads.tables_i8_bytes(s2, q, scale))
    np.testing.assert_array_equal(q2, q)
    np.testing.assert_array_equal(sc2.view(np.uint16), scale.view(np.uint16))


# ---------------------------------------------------------------- blockwise normalisation
def test_read_tables_bn_hand_written_bytes():
    """Swapped code nibbles, codes stored column-major, levels of the wrong group, a missing pad
    between scales and levels: each fails here."""
    case = read_case("tables_2x64_k2_bn.txt")
    f = _fmt(case)
    assert case["tables"].size == oracle.canonical_sizes_bn(f)[1] == 98
    q, scale, levels, codes = oracle.read_tables_bn(f, case["tables"])
    np.testing.assert_array_equal(q.astype(np.int64), case["q"])
    np.testing.assert_array_equal(scale.astype(np.float64), case["scale"])
    assert levels.dtype == np.float16 and levels.shape == (2, 16)
    np.testing.assert_array_equal(levels.astype(np.float64), case["levels"])
    np.testing.assert_array_equal(codes, case["codes"])
    # a reader that took the high nibble first would return (12, 3) and (0, 15)
    assert codes[0, 0] == 3 and codes[0, 1] == 12 and codes[1, 0] == 15 and codes[1, 1] == 0


def test_block_normalised_decode_of_the_hand_written_buffer():
    """The bytes, through reader, table decode and block scales, against weights worked by hand.
    Indices: group 0 (columns 0..31) all centroid 1 = (20,-20), group 1 all centroid 0 = (1,-1).
    Row 0: block 0 has code 3 -> group 0 level 2^-5: 20/32 = 0.625; block 1 code 12 -> group 1
    level 1 + 12/1024, times scale 0.5: 0.505859375.  Row 1: block 0 code 15 -> 2^7: 2560;
    block 1 code 0 -> level 1: 0.5."""
    case = read_case("tables_2x64_k2_bn.txt")
    f = _fmt(case)
    q, scale, levels, codes = oracle.read_tables_bn(f, case["tables"])
    idx = np.array([0xFF] * 4 + [0x00] * 4, dtype=np.uint8)      # 32 one-bit indices per group
    W = oracle.decode_dense(f, idx, oracle.dequantise_codebooks(q, scale))
    W = oracle.apply_block_scales(f, W, levels, codes).view(np.float16).astype(np.float64)
    sign = np.tile([1.0, -1.0], 16)
    np.testing.assert_array_equal(W[0, :32], 0.625 * sign)
    np.testing.assert_array_equal(W[0, 32:], 0.505859375 * sign)
    np.testing.assert_array_equal(W[1, :32], 2560.0 * sign)
    np.testing.assert_array_equal(W[1, 32:], 0.5 * sign)


def test_tables_bn_writer_reproduces_the_hand_written_bytes_and_round_trips():
    case = read_case("tables_2x64_k2_bn.txt")
    s = workloads.VQShape(2, 64, 2, 1, 2, 32, 2, True, True)
    buf = workloads.tables_bn_bytes(s, case["q"].astype(np.int8), case["scale"].astype(np.float16),
                                    case["levels"].astype(np.float16), case["codes"])
    np.testing.assert_array_equal(buf, case["tables"])
    s2 = workloads.VQShape(96, 768, 64, 6, 32, 256, 2, True, True)
    idx, q, scale, levels, codes = workloads.make_weights_bn(s2, 6)
    f2 = VQFormat(96, 768, 64, 6, 32, 256, 2)
    q2, sc2, lv2, cd2 = oracle.read_tables_bn(f2, workloads.tables_bn_bytes(s2, q, scale, levels, codes))
    np.testing.assert_array_equal(q2, q)
    np.testing.assert_array_equal(sc2.view(np.uint16), scale.view(np.uint16))
    np.testing.assert_array_equal(lv2.view(np.uint16), levels.view(np.uint16))
    np.testing.assert_array_equal(cd2, codes)


def test_read_tables_bn_rejects_bad_buffers():
    case = read_case("tables_2x64_k2_bn.txt")
    f = _fmt(case)
    with pytest.raises(ValueError):
        oracle.read_tables_bn(f, case["tables"][:-1])
    bad = case["tables"].copy()
    bad[21] = 7                                   # padding behind the scales
    with pytest.raises(ValueError):
        oracle.read_tables_bn(f, bad)


# ---------------------------------------------------------------- normwise_rel_err
def test_normwise_rel_err_hand_worked_vectors():
    """||y - ref|| / ||ref||: a wrong denominator (norm of y, of the sum), a 1-norm or a max-norm fails."""
    # y - ref = (3, -1), norm sqrt(10); ||ref|| = 5
    assert oracle.normwise_rel_err([3.0, 4.0], [0.0, 5.0]) == pytest.approx(math.sqrt(10) / 5, rel=1e-15)
    # ||y|| = 13 differs from ||ref|| = 5: dividing by the wrong one gives 12/13
    assert oracle.normwise_rel_err([5.0, 12.0], [5.0, 0.0]) == pytest.approx(12 / 5, rel=1e-15)
    # 2-norm, not 1-norm (2/4) or max-norm (1/1): differences (1,1,0,0), ref (1,1,1,1)
    assert oracle.normwise_rel_err([2.0, 2.0, 1.0, 1.0], [1.0, 1.0, 1.0, 1.0]) == pytest.approx(math.sqrt(2) / 2, rel=1e-15)
    assert oracle.normwise_rel_err([1.0, -2.0, 3.0], [1.0, -2.0, 3.0]) == 0.0


def test_normwise_rel_err_matrices_use_the_frobenius_norm():
    ref = np.array([[1.0, 2.0], [2.0, 4.0]])        # Frobenius 5, spectral 5 too (rank one)
    y = ref + np.array([[0.0, 3.0], [4.0, 0.0]])    # difference: Frobenius 5, spectral 4
    assert oracle.normwise_rel_err(y, ref) == pytest.approx(1.0, rel=1e-15)
    ref2 = np.array([[3.0, 0.0], [0.0, 4.0]])       # Frobenius 5, spectral 4
    y2 = ref2 + np.array([[0.0, 0.0], [0.0, 1.0]])
    assert oracle.normwise_rel_err(y2, ref2) == pytest.approx(1 / 5, rel=1e-15)
    # the layout must not matter
    assert oracle.normwise_rel_err(y2.T.copy(), ref2.T.copy()) == pytest.approx(1 / 5, rel=1e-15)


def test_normwise_rel_err_zero_reference_and_scaling():
    assert oracle.normwise_rel_err([0.0, 0.0], [0.0, 0.0]) == 0.0
    assert oracle.normwise_rel_err([0.0, 1e-30], [0.0, 0.0]) == float("inf")
    rng = np.random.default_rng(1)
    ref = rng.standard_normal(100)
    y = ref + 1e-3 * rng.standard_normal(100)
    e = oracle.normwise_rel_err(y, ref)
    for c in (2.0, -0.125, 1e6):                    # invariant under a common scale factor
        assert oracle.normwise_rel_err(c * y, c * ref) == pytest.approx(e, rel=1e-12)
    # widened to fp64 first: fp16 inputs whose squares overflow fp16 still give the exact ratio
    assert oracle.normwise_rel_err(np.array([300.0, 401.0], dtype=np.float16),
                                   np.array([300.0, 400.0], dtype=np.float16)) == pytest.approx(1 / 500, rel=1e-15)


def test_normwise_tolerances_catch_one_wrong_row_and_one_wrong_group():
    """What the tolerances written in the GPU tests can and cannot see, on outputs shaped like the
    workload's (4096 rows of 4096 N(0, 0.02) weights times N(0, 1) activations: |y_r| ~ 1.3).
    One row replaced by an unrelated value of the same distribution is ~ sqrt(2)/64 = 2.2e-2 normwise:
    above the fp16-output bound 2e-3.  One 8 x 256 group's contribution dropped from 8 rows of a
    4096-column matrix (each row off by ~ 0.32) is ~ 3.5e-3: above 2e-3 too, and two hundred times the
    fp32-output bound 2e-5, which is why the layer-sized tests run with fp32 output as well."""
    rng = np.random.default_rng(2)
    ref = rng.standard_normal(4096) * 0.02 * math.sqrt(4096)
    wrong_row = ref.copy()
    wrong_row[1234] = rng.standard_normal() * 0.02 * math.sqrt(4096) + 2.0
    assert oracle.normwise_rel_err(wrong_row, ref) > 2e-3
    wrong_group = ref.copy()
    wrong_group[800:808] -= rng.standard_normal(8) * 0.02 * math.sqrt(256)
    e = oracle.normwise_rel_err(wrong_group, ref)
    assert e > 2e-3 and e > 100 * 2e-5
    # a single wrong vector (2 weights of one row): invisible at 2e-3, visible at 2e-5
    wrong_vec = ref.copy()
    wrong_vec[77] += 0.04 * 1.0
    e = oracle.normwise_rel_err(wrong_vec, ref)
    assert 2e-5 < e < 2e-3


# ---------------------------------------------------------------- low-rank adapter next to the base matrix
def test_gemv_lora_hand_worked():
    """y = W x + B (A x) on the hand-written 4 x 8 decode fixture: W x is the fixture's y
    (49.75, 37.75, 76.25, 63.75) with x = (1, 2, -1, 0.5, 0, 1, 3, -2); the adapter is worked by hand:
    A row 0 = e_0 + 2 e_2 -> t_0 = 1 - 2 = -1;  A row 1 = 0.5 everywhere -> t_1 = 0.5 * 4.5 = 2.25;
    B rows (1, 2), (-1, 0), (0, 4), (2, -2) -> B t = (3.5, 1, 9, -6.5).
    A transposed A or B, a dropped base term, or (B A)^T fails."""
    case = read_case("decode_2x4_k4_b2.txt")
    f = _fmt(case)
    cb = case["codebook"].astype(np.float16)
    x = case["x"].astype(np.float16)
    A = np.array([[1, 0, 2, 0, 0, 0, 0, 0], [0.5] * 8], dtype=np.float16)           # rank 2, in 8
    B = np.array([[1, 2], [-1, 0], [0, 4], [2, -2]], dtype=np.float16)              # out 4, rank 2
    want = np.array([53.25, 38.75, 85.25, 57.25])
    np.testing.assert_array_equal(oracle.gemv_lora(f, case["idx"], cb, x, A, B), want)
    with pytest.raises(ValueError):
        oracle.gemv_lora(f, case["idx"], cb, x, A.T.copy(), B)
    with pytest.raises(ValueError):
        oracle.gemv_lora(f, case["idx"], cb, x, A, B.T.copy())


def test_gemv_lora_reduces_to_known_cases():
    """Zero adapter: the plain product.  Rank-one adapter u v^T: y = W x + u (v . x).  And the sum equals
    the product with the dense matrix W + B A formed in exact rational arithmetic on a tiny case."""
    from fractions import Fraction
    s = workloads.VQShape(16, 512, 16, 4)
    f = VQFormat(16, 512, 16, 4)
    idx, cb = workloads.make_weights(s, 77)
    x = workloads.make_x(512, 77)
    rng = np.random.default_rng(78)
    A = rng.normal(0, 0.05, (4, 512)).astype(np.float16)
    B = rng.normal(0, 0.05, (16, 4)).astype(np.float16)
    base = oracle.gemv(f, idx, cb, x)
    np.testing.assert_array_equal(oracle.gemv_lora(f, idx, cb, x, np.zeros_like(A), B), base)
    np.testing.assert_array_equal(oracle.gemv_lora(f, idx, cb, x, A, np.zeros_like(B)), base)
    u, v = B[:, :1], A[:1, :]
    got = oracle.gemv_lora(f, idx, cb, x, v, u)
    vx = float((v.astype(np.float64) @ x.astype(np.float64))[0])
    np.testing.assert_allclose(got, base + u[:, 0].astype(np.float64) * vx, rtol=1e-13, atol=1e-13)
    # exact rational check of two rows
    W = oracle.decode_dense(f, idx, cb).view(np.float16)
    for r in (0, 11):
        exact = sum(Fraction(float(W[r, c])) * Fraction(float(x[c])) for c in range(512))
        for j in range(4):
            tj = sum(Fraction(float(A[j, c])) * Fraction(float(x[c])) for c in range(512))
            exact += Fraction(float(B[r, j])) * tj
        assert abs(float(exact) - oracle.gemv_lora(f, idx, cb, x, A, B)[r]) <= 1e-12 * max(1.0, abs(float(exact)))
