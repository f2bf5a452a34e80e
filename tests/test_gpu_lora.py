"""GPU parity of y = W x + B (A x) (vq_gemv_lora, vq_gemv_lora_multi) against the oracle.

Tolerances as for the plain product: 2e-3 normwise with fp16 output (one rounding of the fp32
sum), 2e-5 with fp32 output (t = A x and the adapter term are accumulated in fp32 as well).
"""
import numpy as np
import pytest

import oracle
import workloads

pytestmark = pytest.mark.gpu

TOL_F16 = 2e-3
TOL_F32 = 2e-5


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2402_15319_amd as vq
    from paper_2402_15319_amd import device as vqdev
    assert torch.cuda.is_available()
    vq.lib()
    return torch, vq, vqdev


def _fmt(s):
    return oracle.VQFormat(s.out_features, s.in_features, s.k, s.index_bits, s.group_rows, s.group_cols, s.d)


def _adapter(s, rank, seed):
    """Seeded adapter: A fp16 [rank, in] ~ N(0, 1/sqrt(in)), B fp16 [out, rank] ~ N(0, 0.02 * 4): the
    adapter term is of the order of the base product, so a wrong adapter cannot hide."""
    rng = np.random.default_rng(seed ^ 0x10A)
    A = (rng.standard_normal((rank, s.in_features)) / np.sqrt(s.in_features)).astype(np.float16)
    B = (rng.standard_normal((s.out_features, rank)) * 0.08 * np.sqrt(s.in_features) / np.sqrt(max(rank, 1))).astype(np.float16)
    return A, B


def _pack(env, s, seed):
    torch, vq, vqdev = env
    desc = vqdev.desc_from_shape(s)
    f = _fmt(s)
    if s.block_norm:
        idx, q, scale, levels, codes = workloads.make_weights_bn(s, seed)
        tables = workloads.tables_bn_bytes(s, q, scale, levels, codes)
        idx_d, cb_d = vqdev.upload_and_pack(desc, idx, tables)
        q, scale, levels, codes = oracle.read_tables_bn(f, tables)
        W = oracle.apply_block_scales(f, oracle.decode_dense(f, idx, oracle.dequantise_codebooks(q, scale)), levels, codes)
        base = lambda x: W.view(np.float16).astype(np.float64) @ x.astype(np.float64)
        return desc, idx_d, cb_d, base
    if s.int8_tables:
        idx, q, scale = workloads.make_weights_i8(s, seed)
        tables = workloads.tables_i8_bytes(s, q, scale)
        idx_d, cb_d = vqdev.upload_and_pack(desc, idx, tables)
        cb = oracle.dequantise_codebooks(*oracle.read_tables_i8(f, tables))
    else:
        idx, cb = workloads.make_weights(s, seed)
        idx_d, cb_d = vqdev.upload_and_pack(desc, idx, cb)
    return desc, idx_d, cb_d, (lambda x: oracle.gemv(f, idx, cb, x))


def _ref(base, x, A, B):
    """The oracle's y = W x + B (A x) from its own pieces (base(x) is oracle.gemv or the dense product
    of the block-normalised W): the same sum oracle.gemv_lora forms."""
    x64 = x.astype(np.float64)
    return base(x) + B.astype(np.float64) @ (A.astype(np.float64) @ x64)


V = workloads.VQShape
# every representation the adapter entry points take, on shapes that reach the one-chunk, the
# multi-chunk and (32,776+ rows) the persistent streaming kernel
CASES = [
    (V(256, 256, 16, 4), 16), (V(40, 768, 16, 4), 8), (V(24, 2816, 16, 4), 64), (V(264, 1024, 16, 4), 24),
    (V(72, 1280, 256, 8), 16), (V(16, 256 * 43, 256, 8), 32),
    (V(96, 2816, 64, 6, 32, 256, 2, True), 16), (V(40, 768, 16, 4, 8, 256, 2, True), 40),
    (V(40, 256 * 5, 16, 4, 4, 256, 2, True), 24), (V(32776, 768, 16, 4, 4, 256, 2, True), 8),   # k = 16, int8 tables, 4-row groups
    (V(40, 256 * 5, 32, 5, 8, 256, 2, True), 24), (V(32776, 768, 32, 5, 8, 256, 2, True), 8),   # k = 32, 5-bit indices
    (V(72, 1280, 16, 4, 8, 256, 1), 16), (V(96, 768, 8, 3, 32, 256, 1, True), 16), (V(40, 1280, 4, 2, 1, 256, 1, True), 56),
    (V(96, 768, 64, 6, 32, 256, 2, True, True), 16), (V(40, 256 * 5, 16, 4, 8, 256, 2, True, True), 24),
    (V(48, 256 * 5, 8, 3, 16, 256, 1, True, True), 24), (V(32800, 768, 8, 3, 32, 256, 1, True, True), 8),  # d = 1, k = 8, block scales
    (V(256, 256 * 5, 256, 8, 128, 256, 4, True, True), 16), (V(128, 768, 256, 8, 64, 256, 2, True, True), 40),  # tall groups, block scales
    (V(128, 768, 256, 8, 64, 256, 4), 32),                                                            # d = 4, fp16 tables
    (V(128, 768, 256, 8, 64, 256, 4, True), 16), (V(512, 256 * 5, 256, 8, 256, 256, 4, True), 64),    # d = 4
    (V(256, 1280, 256, 8, 128, 256, 2, True), 24), (V(64, 256 * 3, 256, 8, 64, 256, 2, True), 8),      # k = 256, int8 tables
    (V(32776, 768, 16, 4), 16), (V(32776, 2816, 16, 4), 64), (V(33000, 1280, 256, 8), 8),
    (V(32800, 1280, 64, 6, 32, 256, 2, True), 32), (V(32800, 768, 64, 6, 32, 256, 2, True, True), 16),
    (V(32776, 768, 16, 4, 8, 256, 1), 48),
]


@pytest.mark.parametrize("f32", [False, True], ids=["y16", "y32"])
@pytest.mark.parametrize("case", CASES, ids=lambda c: f"{c[0]}-r{c[1]}")
def test_gemv_lora(env, case, f32):
    torch, vq, vqdev = env
    s, rank = case
    seed = 8000 + s.out_features + s.in_features + s.k + rank
    desc, idx_d, cb_d, base = _pack(env, s, seed)
    x = workloads.make_x(s.in_features, seed)
    A, B = _adapter(s, rank, seed)
    n = s.out_features
    y = torch.full((n + 64,), 12352.0, dtype=torch.float32 if f32 else torch.float16, device="cuda:0")
    ws = torch.full((64 + 16,), float("nan"), dtype=torch.float32, device="cuda:0")     # canary behind the 64 slots
    vq.vq_gemv_lora(desc, idx_d, cb_d, vqdev.to_device_bytes(x), vqdev.to_device_bytes(A), vqdev.to_device_bytes(B),
                    rank, ws, y, vq.VQ_F32 if f32 else vq.VQ_F16, workspace_bytes=256)
    torch.cuda.synchronize()
    out = y.cpu().numpy().astype(np.float64)
    assert np.all(out[n:] == 12352.0), "wrote past the end of y"
    assert np.all(np.isnan(ws.cpu().numpy()[rank:])), "wrote workspace slots beyond the rank"
    ref = _ref(base, x, A, B)
    plain = base(x)
    assert oracle.normwise_rel_err(ref, plain) > 0.1          # the adapter matters in this test
    assert oracle.normwise_rel_err(out[:n], ref) <= (TOL_F32 if f32 else TOL_F16)


def test_gemv_lora_matches_oracle_gemv_lora_directly(env):
    """One case through oracle.gemv_lora itself (the pinned function), fp32 output."""
    torch, vq, vqdev = env
    s = V(264, 1024, 16, 4)
    idx, cb = workloads.make_weights(s, 81)
    x = workloads.make_x(1024, 81)
    A, B = _adapter(s, 16, 81)
    desc = vqdev.desc_from_shape(s)
    idx_d, cb_d = vqdev.upload_and_pack(desc, idx, cb)
    y = torch.zeros(264, dtype=torch.float32, device="cuda:0")
    ws = torch.zeros(64, dtype=torch.float32, device="cuda:0")
    vq.vq_gemv_lora(desc, idx_d, cb_d, vqdev.to_device_bytes(x), vqdev.to_device_bytes(A), vqdev.to_device_bytes(B), 16, ws, y, vq.VQ_F32)
    torch.cuda.synchronize()
    assert oracle.normwise_rel_err(y.cpu().numpy(), oracle.gemv_lora(_fmt(s), idx, cb, x, A, B)) <= TOL_F32
    # t = A x is what the first kernel left in the workspace
    t = A.astype(np.float64) @ x.astype(np.float64)
    assert oracle.normwise_rel_err(ws.cpu().numpy()[:16], t) <= TOL_F32


def test_rank_zero_is_the_plain_product_bit_for_bit(env):
    torch, vq, vqdev = env
    s = V(264, 1024, 16, 4)
    desc, idx_d, cb_d, base = _pack(env, s, 82)
    x_d = vqdev.to_device_bytes(workloads.make_x(1024, 82))
    y0 = torch.zeros(264, dtype=torch.float16, device="cuda:0")
    y1 = torch.ones(264, dtype=torch.float16, device="cuda:0")
    ws = torch.zeros(64, dtype=torch.float32, device="cuda:0")
    vq.vq_gemv(desc, idx_d, cb_d, x_d, y0)
    vq.vq_gemv_lora(desc, idx_d, cb_d, x_d, None, None, 0, ws, y1)
    torch.cuda.synchronize()
    assert torch.equal(y0, y1)


@pytest.mark.parametrize("f32", [False, True], ids=["y16", "y32"])
def test_gemv_lora_multi_llama_layer(env, f32):
    """The 7 matrices of a decoder layer in one call (the streaming kernel), adapters of rank 16 on the
    attention projections, rank 32 on down_proj and none on gate/up (rank 0), every row checked."""
    torch, vq, vqdev = env
    descs, idxs, cbs, xs, ys, As, Bs, ranks, refs = [], [], [], [], [], [], [], [], []
    for m, (name, key) in enumerate(workloads.LLAMA7B_LAYER):
        s = workloads.CONFIGS[key]
        seed = workloads.seed_for(key, 1, m)
        desc, idx_d, cb_d, base = _pack(env, s, seed)
        x = workloads.make_x(s.in_features, seed)
        rank = {"gate_proj": 0, "up_proj": 0, "down_proj": 32}.get(name, 16)
        A, B = _adapter(s, max(rank, 8), seed)
        descs.append(desc); idxs.append(idx_d); cbs.append(cb_d); xs.append(vqdev.to_device_bytes(x))
        ys.append(torch.full((s.out_features,), float("nan"), dtype=torch.float32 if f32 else torch.float16, device="cuda:0"))
        As.append(vqdev.to_device_bytes(A) if rank else None)
        Bs.append(vqdev.to_device_bytes(B) if rank else None)
        ranks.append(rank)
        refs.append(_ref(base, x, A, B) if rank else base(x))
    ws = torch.zeros(vq.vq_lora_workspace_bytes(7) // 4, dtype=torch.float32, device="cuda:0")
    vq.vq_gemv_lora_multi(vq.GemvMultiArgs(descs, idxs, cbs, xs, ys), As, Bs, ranks, ws, vq.VQ_F32 if f32 else vq.VQ_F16)
    torch.cuda.synchronize()
    for i, ref in enumerate(refs):
        y = ys[i].cpu().numpy().astype(np.float64)
        assert not np.isnan(y).any(), i
        assert oracle.normwise_rel_err(y, ref) <= (TOL_F32 if f32 else TOL_F16), i
        for r0 in range(0, len(y), 512):          # per block of 512 rows too
            assert oracle.normwise_rel_err(y[r0:r0 + 512], ref[r0:r0 + 512]) <= (TOL_F32 if f32 else TOL_F16), (i, r0)


def test_gemv_lora_multi_more_than_one_launch(env):
    """300 small products (two launches of the problem table), ranks cycling through 0, 8, ..., 64."""
    torch, vq, vqdev = env
    shapes = [V(64, 512, 16, 4), V(176, 512, 16, 4), V(64, 1280, 16, 4), V(8, 256, 16, 4)] * 75
    descs, idxs, cbs, xs, ys, As, Bs, ranks, refs = [], [], [], [], [], [], [], [], []
    for i, s in enumerate(shapes):
        desc, idx_d, cb_d, base = _pack(env, s, 8300 + i)
        x = workloads.make_x(s.in_features, 8300 + i)
        rank = 8 * (i % 9)
        A, B = _adapter(s, max(rank, 8), 8300 + i)
        descs.append(desc); idxs.append(idx_d); cbs.append(cb_d); xs.append(vqdev.to_device_bytes(x))
        ys.append(torch.zeros(s.out_features, dtype=torch.float32, device="cuda:0"))
        As.append(vqdev.to_device_bytes(A) if rank else None)
        Bs.append(vqdev.to_device_bytes(B) if rank else None)
        ranks.append(rank)
        refs.append(_ref(base, x, A, B) if rank else base(x))
    ws = torch.zeros(vq.vq_lora_workspace_bytes(300) // 4, dtype=torch.float32, device="cuda:0")
    vq.vq_gemv_lora_multi(vq.GemvMultiArgs(descs, idxs, cbs, xs, ys), As, Bs, ranks, ws, vq.VQ_F32)
    torch.cuda.synchronize()
    for i, ref in enumerate(refs):
        assert oracle.normwise_rel_err(ys[i].cpu().numpy(), ref) <= TOL_F32, i


@pytest.mark.parametrize("d", [4, 2], ids=["d4", "k256_int8_tables"])
def test_gemv_lora_multi_wide_group_formats(env, d):
    """The formats whose tables are shared by 64 to 256 rows (kernels of their own: a workgroup per 64
    rows): five matrices of mixed group heights and widths in one call, ranks 0, 8, 24, 40, 64."""
    torch, vq, vqdev = env
    shapes = [V(256, 768, 256, 8, 64, 256, d, True), V(256, 256 * 5, 256, 8, 128, 256, d, True),
              V(512, 512, 256, 8, 256, 256, d, True), V(64, 256, 256, 8, 64, 256, d, True),
              V(1024, 1280, 256, 8, 256, 256, d, True)]
    descs, idxs, cbs, xs, ys, As, Bs, ranks, refs = [], [], [], [], [], [], [], [], []
    for i, (s, rank) in enumerate(zip(shapes, (0, 8, 24, 40, 64))):
        desc, idx_d, cb_d, base = _pack(env, s, 8800 + 10 * d + i)
        x = workloads.make_x(s.in_features, 8800 + i)
        A, B = _adapter(s, max(rank, 8), 8800 + i)
        descs.append(desc); idxs.append(idx_d); cbs.append(cb_d); xs.append(vqdev.to_device_bytes(x))
        ys.append(torch.full((s.out_features,), float("nan"), dtype=torch.float32, device="cuda:0"))
        As.append(vqdev.to_device_bytes(A) if rank else None)
        Bs.append(vqdev.to_device_bytes(B) if rank else None)
        ranks.append(rank)
        refs.append(_ref(base, x, A, B) if rank else base(x))
    ws = torch.zeros(vq.vq_lora_workspace_bytes(len(shapes)) // 4, dtype=torch.float32, device="cuda:0")
    vq.vq_gemv_lora_multi(vq.GemvMultiArgs(descs, idxs, cbs, xs, ys), As, Bs, ranks, ws, vq.VQ_F32)
    torch.cuda.synchronize()
    for i, ref in enumerate(refs):
        y = ys[i].cpu().numpy().astype(np.float64)
        assert not np.isnan(y).any(), i
        assert oracle.normwise_rel_err(y, ref) <= TOL_F32, i


def test_lora_replays_in_a_hip_graph(env):
    """Both launches of the adapter path captured in a HIP graph; three replays with eager work
    between them reproduce the eager result bit for bit."""
    torch, vq, vqdev = env
    s = V(32776, 768, 16, 4)
    desc, idx_d, cb_d, base = _pack(env, s, 84)
    x = workloads.make_x(768, 84)
    A, B = _adapter(s, 16, 84)
    x_d, A_d, B_d = vqdev.to_device_bytes(x), vqdev.to_device_bytes(A), vqdev.to_device_bytes(B)
    ws = torch.zeros(64, dtype=torch.float32, device="cuda:0")
    y_e = torch.zeros(s.out_features, dtype=torch.float16, device="cuda:0")
    vq.vq_gemv_lora(desc, idx_d, cb_d, x_d, A_d, B_d, 16, ws, y_e)
    torch.cuda.synchronize()
    assert oracle.normwise_rel_err(y_e.cpu().numpy(), _ref(base, x, A, B)) <= TOL_F16
    y_g = torch.zeros_like(y_e)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        vq.vq_gemv_lora(desc, idx_d, cb_d, x_d, A_d, B_d, 16, ws, y_g)
    for _ in range(3):
        y_g.fill_(3); ws.fill_(9)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(y_g, y_e)
