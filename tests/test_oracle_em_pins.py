"""Pins for the oracle's E- and M-step (Hessian-weighted EM of the codebook initialisation):
hand-worked values, closed forms and invariants, none computed by the functions under test."""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from oracle import VQFormat
from golden_io import GOLDEN_DIR


def _read_em_case(name):
    out = {"W": [], "assign": []}
    with open(os.path.join(GOLDEN_DIR, name)) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, _, rest = line.partition(":")
            vals = rest.split()
            if key == "format":
                out["format"] = {k: int(v) for k, v in (kv.split("=") for kv in vals)}
            elif key in ("W", "assign"):
                out[key].append([float(v) for v in vals])
            else:
                out[key] = [float(v) for v in vals]
    return out


def _case(name="em_2x4_k2.txt"):
    c = _read_em_case(name)
    fm = c["format"]
    f = VQFormat(fm["out"], fm["in"], fm["k"], fm["index_bits"], fm["group_rows"], fm["group_cols"], fm["d"])
    W = np.array(c["W"], dtype=np.float32)
    h = np.array(c["hdiag"], dtype=np.float32)
    cb = np.array(c["codebook"], dtype=np.float32).reshape(1, fm["k"], fm["d"])
    return c, f, W, h, cb


def test_golden_e_step():
    """A dropped weight (plain Euclidean distance), weights taken from the wrong columns or a
    transposed centroid change at least one of the four hand-worked assignments."""
    c, f, W, h, cb = _case()
    a = oracle.em_assign(f, W, h, cb)
    np.testing.assert_array_equal(a, np.array(c["assign"], dtype=np.int64))
    assert oracle.em_objective(f, W, h, cb, a) == c["objective"][0]
    # the same data without the weights picks the other centroid for the first vector
    a_plain = oracle.em_assign(f, W, np.ones(4, dtype=np.float32), cb)
    assert a_plain[0, 0] == 0 and a[0, 0] == 1


def test_golden_m_step():
    """Unweighted means, weights of the other coordinate, or sums over the wrong cluster fail."""
    c, f, W, h, cb = _case()
    a = np.array(c["assign"], dtype=np.uint8)
    got = oracle.em_update(f, W, h, a)
    want = (np.array(c["updated_num"]) / np.array(c["updated_den"])).reshape(1, 2, 2)
    np.testing.assert_allclose(got, want, rtol=1e-15)
    n, d = c["objective_after_num_den"]
    assert abs(oracle.em_objective(f, W, h, got, a) - n / d) < 1e-12


@pytest.mark.parametrize("name", ["em_2x4_k2_d1.txt", "em_2x8_k2_d4.txt"])
def test_golden_e_and_m_step_other_dimensionalities(name):
    """Scalar codebooks (d = 1) and four-dimensional vectors (d = 4), worked by hand: the weights of
    the wrong columns, a sum over t that stops at two coordinates, vectors cut at the wrong column
    stride or an unweighted mean change an assignment, the objective or a centroid."""
    c, f, W, h, cb = _case(name)
    a = oracle.em_assign(f, W, h, cb)
    np.testing.assert_array_equal(a, np.array(c["assign"], dtype=np.int64))
    assert oracle.em_objective(f, W, h, cb, a) == c["objective"][0]
    got = oracle.em_update(f, W, h, a)
    want = (np.array(c["updated_num"]) / np.array(c["updated_den"])).reshape(1, f.k, f.d)
    np.testing.assert_allclose(got, want, rtol=1e-15)


def test_tall_groups_use_their_own_codebook_and_sum_over_all_their_rows():
    """Two groups of 2 rows x 2 columns stacked (out = 4): the same vector (1,1) is nearest to centroid 0
    of the upper group and to centroid 1 of the lower one, whose codebook is the upper one's swapped;
    the M-step of a group averages over both of its rows."""
    f = VQFormat(4, 2, 2, 4, 2, 2, 2)          # (4 index bits so that a group's two indices fill a byte)
    W = np.array([[1, 1], [3, 1], [1, 1], [9, 9]], dtype=np.float32)
    h = np.array([1, 3], dtype=np.float32)
    cb = np.array([[[0, 0], [10, 10]], [[10, 10], [0, 0]]], dtype=np.float32)
    a = oracle.em_assign(f, W, h, cb)
    np.testing.assert_array_equal(a, [[0], [0], [1], [0]])
    new = oracle.em_update(f, W, h, a)
    np.testing.assert_array_equal(new[0], [[2, 1], [0, 0]])       # rows 0 and 1 together: ((1+3)/2, (3*1+3*1)/6)
    np.testing.assert_array_equal(new[1], [[9, 9], [1, 1]])


def test_ties_go_to_the_lowest_index_and_empty_clusters_become_zero():
    f = VQFormat(1, 4, 4, 4, 1, 4, 2)      # (4 index bits only so that the group's indices fill a byte)
    W = np.array([[1, 1, 5, 5]], dtype=np.float32)
    h = np.ones(4, dtype=np.float32)
    cb = np.array([[[9, 9], [0, 1], [1, 0], [5, 5]]], dtype=np.float32)     # (1,1) is at distance 1 from both 1 and 2
    a = oracle.em_assign(f, W, h, cb)
    np.testing.assert_array_equal(a, [[1, 3]])
    new = oracle.em_update(f, W, h, a)
    np.testing.assert_array_equal(new[0, 0], [0, 0])      # nobody chose 0: the pseudoinverse gives 0
    np.testing.assert_array_equal(new[0, 2], [0, 0])
    np.testing.assert_array_equal(new[0, 1], [1, 1])
    # a coordinate whose weights are all zero also becomes 0, the other one is still a weighted mean
    h0 = np.array([0, 2, 0, 6], dtype=np.float32)
    new0 = oracle.em_update(f, W, h0, np.array([[1, 1]], dtype=np.uint8))
    np.testing.assert_array_equal(new0[0, 1], [0, (2 * 1 + 6 * 5) / 8])


def _exact_assign(f, W, h, cb):
    """Exact rational brute force over every vector and centroid; also returns the margin
    (second best minus best, relative) so that near-ties can be left out."""
    n_cb = f.groups_per_row
    a = np.zeros((f.out_features, f.in_features // f.d), dtype=np.int64)
    margin = np.zeros(a.shape)
    for r in range(f.out_features):
        for v in range(f.in_features // f.d):
            c0 = v * f.d
            g = (r // f.group_rows) * n_cb + c0 // f.group_cols
            ds = []
            for m in range(f.k):
                ds.append(sum(Fraction(float(h[c0 + t])) * (Fraction(float(W[r, c0 + t])) - Fraction(float(cb[g, m, t]))) ** 2
                              for t in range(f.d)))
            order = sorted(range(f.k), key=lambda m: (ds[m], m))
            a[r, v] = order[0]
            margin[r, v] = float((ds[order[1]] - ds[order[0]]) / (ds[order[1]] + 1)) if f.k > 1 else 1.0
    return a, margin


@pytest.mark.parametrize("f", [VQFormat(4, 16, 4, 2, 2, 8, 2), VQFormat(2, 24, 8, 3, 1, 24, 3),
                               VQFormat(3, 8, 4, 2, 1, 8, 1)], ids=str)
def test_e_step_against_exact_rational_brute_force(f):
    """Wrong group of a vector, wrong columns of the weights, a missing square: caught on every
    vector whose best and second-best distances are not within rounding of each other."""
    rng = np.random.default_rng(5)
    W = rng.normal(0, 1, (f.out_features, f.in_features)).astype(np.float32)
    h = rng.uniform(0.1, 4, f.in_features).astype(np.float32)
    cb = rng.normal(0, 1, (f.n_groups, f.k, f.d)).astype(np.float32)
    want, margin = _exact_assign(f, W, h, cb)
    got = oracle.em_assign(f, W, h, cb).astype(np.int64)
    clear = margin > 1e-5
    assert clear.mean() > 0.9
    np.testing.assert_array_equal(got[clear], want[clear])


def test_unit_weights_reduce_to_k_means():
    """D = I: nearest centroid in the Euclidean sense and the arithmetic mean of a cluster."""
    rng = np.random.default_rng(6)
    f = VQFormat(8, 32, 4, 2, 4, 16, 2)
    W = rng.normal(0, 1, (8, 32)).astype(np.float32)
    ones = np.ones(32, dtype=np.float32)
    cb = rng.normal(0, 1, (f.n_groups, 4, 2)).astype(np.float32)
    a = oracle.em_assign(f, W, ones, cb)
    new = oracle.em_update(f, W, ones, a)
    for g in range(f.n_groups):
        rb, cbk = divmod(g, 2)
        X = W[rb * 4:(rb + 1) * 4, cbk * 16:(cbk + 1) * 16].reshape(-1, 2).astype(np.float64)
        A = a[rb * 4:(rb + 1) * 4, cbk * 8:(cbk + 1) * 8].reshape(-1)
        d2 = ((X[:, None, :] - cb[g].astype(np.float64)[None]) ** 2).sum(-1)
        gap = np.sort(d2, axis=1)
        clear = gap[:, 1] - gap[:, 0] > 1e-5
        np.testing.assert_array_equal(A[clear], d2.argmin(1)[clear])
        for m in range(4):
            if (A == m).any():
                np.testing.assert_allclose(new[g, m], X[A == m].mean(0), rtol=1e-12)


def test_m_step_is_the_minimiser_and_em_never_increases_the_objective():
    """The weighted residuals of a cluster sum to zero at the M-step's centroid (first-order
    condition of the quadratic), any other centroid is worse, and alternating the two steps
    never increases the objective (a sign or weighting mistake in either step breaks this)."""
    rng = np.random.default_rng(8)
    f = VQFormat(16, 512, 16, 4)
    W = rng.normal(0, 0.02, (16, 512)).astype(np.float32)
    h = rng.uniform(0.2, 5, 512).astype(np.float32)
    cb = rng.normal(0, 0.02, (f.n_groups, 16, 2)).astype(np.float32)
    last = np.inf
    for _ in range(5):
        a = oracle.em_assign(f, W, h, cb)
        o_e = oracle.em_objective(f, W, h, cb, a)
        assert o_e <= last * (1 + 1e-6)
        new = oracle.em_update(f, W, h, a)
        o_m = oracle.em_objective(f, W, h, new, a)
        assert o_m <= o_e * (1 + 1e-12)
        for trial in range(3):
            bumped = new + rng.normal(0, 1e-3, new.shape) * (trial + 1)
            assert oracle.em_objective(f, W, h, bumped, a) >= o_m
        # first-order condition for one group, cluster by cluster
        X = W[:8, :256].reshape(8, 128, 2).astype(np.float64)
        H = np.broadcast_to(h[:256].reshape(1, 128, 2).astype(np.float64), X.shape)
        A = a[:8, :128]
        for m in range(16):
            sel = A == m
            if sel.any():
                resid = (H[sel] * (X[sel] - new[0, m])).sum(0)
                assert np.all(np.abs(resid) < 1e-12)
        last = o_m
        cb = new.astype(np.float32)


def test_scaling_all_weights_by_a_power_of_two_changes_nothing():
    rng = np.random.default_rng(9)
    f = VQFormat(8, 256, 16, 4)
    W = rng.normal(0, 0.02, (8, 256)).astype(np.float32)
    h = rng.uniform(0.2, 5, 256).astype(np.float32)
    cb = rng.normal(0, 0.02, (1, 16, 2)).astype(np.float32)
    a = oracle.em_assign(f, W, h, cb)
    np.testing.assert_array_equal(a, oracle.em_assign(f, W, h * np.float32(8), cb))
    np.testing.assert_allclose(oracle.em_update(f, W, h, a), oracle.em_update(f, W, h * np.float32(8), a), rtol=1e-13)
