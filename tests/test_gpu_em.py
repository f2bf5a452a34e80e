"""GPU parity of the quantiser kernels (E- and M-step of the Hessian-weighted EM) against the
CPU oracle, through the C ABI.  Assignments are compared bit for bit (both sides take the
decision in binary32 with the same operation order); centroids within the bound derived from
binary32 summation of at most 1,024 terms."""
import numpy as np
import pytest

import oracle
import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2402_15319_amd as vq
    from paper_2402_15319_amd import device as vqdev
    assert torch.cuda.is_available()
    vq.lib()
    return torch, vq, vqdev


def _inputs(out_f, in_f, k, seed, from_data=False):
    """Seeded synthetic quantiser inputs: N(0, 0.02) weights, column weights 1/[H^-1]_cc spread
    over a factor of 25, and a starting codebook (random, or k vectors drawn from the group)."""
    rng = np.random.default_rng(seed)
    W = rng.normal(0, 0.02, (out_f, in_f)).astype(np.float32)
    h = rng.uniform(0.2, 5.0, in_f).astype(np.float32)
    n_groups = (out_f // 8) * (in_f // 256)
    if from_data:
        cb = np.zeros((n_groups, k, 2), dtype=np.float32)
        n_cb = in_f // 256
        for g in range(n_groups):
            rb, c = divmod(g, n_cb)
            X = W[rb * 8:(rb + 1) * 8, c * 256:(c + 1) * 256].reshape(-1, 2)
            cb[g] = X[rng.choice(X.shape[0], size=k, replace=False)]
    else:
        cb = rng.normal(0, 0.02, (n_groups, k, 2)).astype(np.float32)
    return W, h, cb


def _fmt(out_f, in_f, k):
    return oracle.VQFormat(out_f, in_f, k, {16: 4, 64: 6, 256: 8}[k])


def _desc(vq, out_f, in_f, k):
    return vq.make_desc(out_f, in_f, k, {16: 4, 64: 6, 256: 8}[k])


def _gpu_assign(env, desc, W, h, cb):
    torch, vq, vqdev = env
    a = torch.full((desc.out_features, desc.in_features // 2), 255, dtype=torch.uint8, device="cuda:0")
    vq.vq_em_assign(desc, vqdev.to_device_bytes(W), vqdev.to_device_bytes(h), vqdev.to_device_bytes(cb), a)
    torch.cuda.synchronize()
    return a.cpu().numpy()


def _gpu_update(env, desc, W, h, assign, k):
    torch, vq, vqdev = env
    n_groups = (desc.out_features // 8) * (desc.in_features // 256)
    out = torch.full((n_groups, k, 2), 777.0, dtype=torch.float32, device="cuda:0")
    vq.vq_em_update(desc, vqdev.to_device_bytes(W), vqdev.to_device_bytes(h),
                    vqdev.to_device_bytes(assign.astype(np.uint8)), out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


# several groups, group counts that are not a multiple of the waves of a workgroup (4 for the
# E-step, 2 for the M-step), every codebook size
SHAPES = [(8, 256, 16), (16, 512, 16), (40, 768, 16), (24, 1280, 64), (8, 768, 256), (24, 256, 256)]


@pytest.mark.parametrize("from_data", [False, True], ids=["random_cb", "cb_from_data"])
@pytest.mark.parametrize("shape", SHAPES, ids=str)
def test_e_step_bit_exact(env, shape, from_data):
    out_f, in_f, k = shape
    W, h, cb = _inputs(out_f, in_f, k, 900 + out_f + k, from_data)
    got = _gpu_assign(env, _desc(env[1], out_f, in_f, k), W, h, cb)
    np.testing.assert_array_equal(got, oracle.em_assign(_fmt(out_f, in_f, k), W, h, cb))


@pytest.mark.parametrize("shape", SHAPES, ids=str)
def test_m_step_within_summation_bound(env, shape):
    """fp32 sequential summation of n <= 1,024 terms is off by at most n * 2^-24 relative to the
    sum of magnitudes, for numerator and denominator each: |error| <= 1.3e-4 * max|W| of the
    group; the test uses 1.5e-4.  Clusters nobody chose must come out as exact zeros."""
    out_f, in_f, k = shape
    # k = 256 starts from random centroids, so that some clusters stay empty
    W, h, cb = _inputs(out_f, in_f, k, 950 + out_f + k, from_data=(k != 256))
    f = _fmt(out_f, in_f, k)
    a = oracle.em_assign(f, W, h, cb)
    got = _gpu_update(env, _desc(env[1], out_f, in_f, k), W, h, a, k)
    want = oracle.em_update(f, W, h, a)
    assert np.abs(got - want).max() <= 1.5e-4 * np.abs(W).max()
    counts = np.zeros((f.n_groups, k), dtype=np.int64)
    n_cb = in_f // 256
    for g in range(f.n_groups):
        rb, c = divmod(g, n_cb)
        counts[g] = np.bincount(a[rb * 8:(rb + 1) * 8, c * 128:(c + 1) * 128].reshape(-1), minlength=k)
    assert np.all(got[counts == 0] == 0.0)
    if k == 256:
        assert (counts == 0).any()        # 1,024 vectors over 256 centroids: the case occurs


def test_tie_and_zero_weight_cases(env):
    """Two centroids at the same weighted distance -> the lower index, on the GPU as in the
    oracle; a column whose weight is zero contributes nothing and gives a zero coordinate."""
    torch, vq, vqdev = env
    out_f, in_f, k = 8, 256, 16
    W = np.ones((out_f, in_f), dtype=np.float32)
    h = np.ones(in_f, dtype=np.float32)
    h[1::2] = 0.0                                    # second coordinate of every vector has no weight
    cb = np.zeros((1, k, 2), dtype=np.float32)
    cb[0, :, 0] = np.array([5, 3, 0, 2, 2, 9, 9, 9, 9, 9, 9, 9, 9, 9, 9, 9], dtype=np.float32)
    cb[0, :, 1] = np.arange(k, dtype=np.float32)     # ignored: weight 0
    desc = _desc(vq, out_f, in_f, k)
    a = _gpu_assign(env, desc, W, h, cb)
    assert np.all(a == 2)                            # |1-0| = |1-2| = 1: index 2 comes before 3 and 4
    np.testing.assert_array_equal(a, oracle.em_assign(_fmt(out_f, in_f, k), W, h, cb))
    new = _gpu_update(env, desc, W, h, a, k)
    np.testing.assert_array_equal(new[0, 2], [1.0, 0.0])
    assert np.all(new[0, np.arange(k) != 2] == 0.0)


def test_em_iterations_track_the_oracle_and_lower_the_objective(env):
    """Five E/M rounds on the GPU: every E-step equals the oracle's on the GPU's own centroids,
    and the objective (evaluated by the oracle in fp64) never increases."""
    out_f, in_f, k = 32, 1024, 16
    W, h, cb = _inputs(out_f, in_f, k, 977, True)
    f = _fmt(out_f, in_f, k)
    desc = _desc(env[1], out_f, in_f, k)
    last = np.inf
    for _ in range(5):
        a = _gpu_assign(env, desc, W, h, cb)
        np.testing.assert_array_equal(a, oracle.em_assign(f, W, h, cb))
        obj_e = oracle.em_objective(f, W, h, cb, a)
        assert obj_e <= last * (1 + 1e-6)
        cb = _gpu_update(env, desc, W, h, a, k)
        last = oracle.em_objective(f, W, h, cb, a)
        assert last <= obj_e * (1 + 1e-6)


def test_full_size_layer(env):
    """4096 x 4096, k = 16 (8,192 groups), in the launch configuration the bench times: the
    E-step compared in full, the M-step on 64 sampled groups."""
    out_f, in_f, k = 4096, 4096, 16
    W, h, cb = _inputs(out_f, in_f, k, 990)
    f = _fmt(out_f, in_f, k)
    desc = _desc(env[1], out_f, in_f, k)
    a = _gpu_assign(env, desc, W, h, cb)
    np.testing.assert_array_equal(a, oracle.em_assign(f, W, h, cb))
    new = _gpu_update(env, desc, W, h, a, k)
    rng = np.random.default_rng(3)
    for g in rng.choice(f.n_groups, size=64, replace=False):
        rb, c = divmod(int(g), in_f // 256)
        sub = oracle.VQFormat(8, 256, k, 4)
        want = oracle.em_update(sub, W[rb * 8:(rb + 1) * 8, c * 256:(c + 1) * 256], h[c * 256:(c + 1) * 256],
                                a[rb * 8:(rb + 1) * 8, c * 128:(c + 1) * 128])
        assert np.abs(new[g] - want[0]).max() <= 1.5e-4 * np.abs(W).max()


# ---------------------------------------------------------------- other dimensionalities and group heights
def _inputs_any(out_f, in_f, k, d, group_rows, seed, from_data=True):
    rng = np.random.default_rng(seed)
    W = rng.normal(0, 0.02, (out_f, in_f)).astype(np.float32)
    h = rng.uniform(0.2, 5.0, in_f).astype(np.float32)
    n_cb = in_f // 256
    n_groups = (out_f // group_rows) * n_cb
    if from_data:
        cb = np.zeros((n_groups, k, d), dtype=np.float32)
        for g in range(n_groups):
            gr, c = divmod(g, n_cb)
            X = W[gr * group_rows:(gr + 1) * group_rows, c * 256:(c + 1) * 256].reshape(-1, d)
            cb[g] = X[rng.choice(X.shape[0], size=k, replace=X.shape[0] < k)]
    else:
        cb = rng.normal(0, 0.02, (n_groups, k, d)).astype(np.float32)
    return W, h, cb


# (out, in, k, d, group_rows): the group shapes of the decode formats, with block counts that are not
# multiples of the waves of a workgroup
ANY_SHAPES = [
    (8, 256, 16, 1, 8), (40, 768, 16, 1, 8),          # scalar codebooks, 4-bit
    (64, 512, 8, 1, 32), (96, 256, 8, 1, 16),         # 3-bit, 32- and 16-row groups
    (8, 512, 4, 1, 1), (24, 768, 4, 1, 1),            # 2-bit, a codebook per row
    (64, 512, 64, 2, 32), (48, 256, 64, 2, 16),       # d = 2 with taller groups
    (256, 512, 256, 2, 128), (64, 256, 256, 2, 64),
    (128, 512, 256, 4, 64), (256, 256, 256, 4, 256), (256, 768, 256, 4, 128),   # four-dimensional vectors
    (8, 256, 16, 2, 4), (40, 768, 16, 2, 4), (24, 512, 16, 1, 4),   # groups of 4 rows: two codebooks per 8-row block
    (8, 256, 32, 2, 8), (40, 768, 32, 2, 8),          # k = 32 (5-bit indices)
    (16, 256, 16, 4, 8), (8, 256, 4, 2, 1),           # combinations no decode format uses, same kernels
]


def _gpu_em_any(env, shape, W, h, cb):
    torch, vq, vqdev = env
    out_f, in_f, k, d, gr = shape
    bits = {4: 2, 8: 3, 16: 4, 32: 5, 64: 6, 256: 8}[k]
    desc = vq.make_desc(out_f, in_f, k, bits, group_rows=gr, d=d)
    a = torch.full((out_f, in_f // d), 255, dtype=torch.uint8, device="cuda:0")
    W_d, h_d = vqdev.to_device_bytes(W), vqdev.to_device_bytes(h)
    vq.vq_em_assign(desc, W_d, h_d, vqdev.to_device_bytes(cb), a)
    new = torch.full(cb.shape, 777.0, dtype=torch.float32, device="cuda:0")
    vq.vq_em_update(desc, W_d, h_d, a, new)
    torch.cuda.synchronize()
    return a.cpu().numpy(), new.cpu().numpy()


@pytest.mark.parametrize("shape", ANY_SHAPES, ids=str)
def test_e_and_m_step_any_dimensionality_and_group_height(env, shape):
    """E-step bit for bit; M-step (on the E-step's own assignments) within the binary32 summation
    bound: a lane sums at most n / 64 terms one after the other, then 64 lane totals are added, so the
    error is at most (n / 64 + 64) * 2^-24 relative to the sum of magnitudes, for numerator and
    denominator each; with weights within a factor 25 of each other that is below
    (n / 64 + 64) * 2^-24 * 2 * 25 * max|W| -- the test uses that bound, which is 1.5e-4 max|W| for the
    8 x 256 groups."""
    out_f, in_f, k, d, gr = shape
    # big codebooks start from random centroids, so that some clusters stay empty
    W, h, cb = _inputs_any(out_f, in_f, k, d, gr, 1200 + out_f + k + d, from_data=(k < 256))
    f = oracle.VQFormat(out_f, in_f, k, 8, gr, 256, d)
    want_a = oracle.em_assign(f, W, h, cb)
    a, new = _gpu_em_any(env, shape, W, h, cb)
    np.testing.assert_array_equal(a, want_a)
    want = oracle.em_update(f, W, h, want_a)
    n = gr * 256 // d
    bound = max(1.5e-4, (n / 64 + 64) * 2.0 ** -24 * 50) * np.abs(W).max()
    assert np.abs(new - want).max() <= bound
    n_cb = in_f // 256
    counts = np.zeros((f.n_groups, k), dtype=np.int64)
    for g in range(f.n_groups):
        gi, c = divmod(g, n_cb)
        counts[g] = np.bincount(want_a[gi * gr:(gi + 1) * gr, c * (256 // d):(c + 1) * (256 // d)].reshape(-1), minlength=k)
    assert np.all(new[counts == 0] == 0.0)


def test_em_rounds_on_a_deployed_group_shape(env):
    """Four E/M rounds with k = 64, 32 x 256 groups (the deployed representation's groups): each
    E-step equals the oracle's on the GPU's own centroids, the objective never rises."""
    shape = (64, 512, 64, 2, 32)
    out_f, in_f, k, d, gr = shape
    W, h, cb = _inputs_any(out_f, in_f, k, d, gr, 1300)
    f = oracle.VQFormat(out_f, in_f, k, 6, gr, 256, d)
    last = np.inf
    for _ in range(4):
        a, new = _gpu_em_any(env, shape, W, h, cb)
        np.testing.assert_array_equal(a, oracle.em_assign(f, W, h, cb))
        obj_e = oracle.em_objective(f, W, h, cb, a)
        assert obj_e <= last * (1 + 1e-6)
        cb = new
        last = oracle.em_objective(f, W, h, cb, a)
        assert last <= obj_e * (1 + 1e-6)
