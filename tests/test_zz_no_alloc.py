"""vq_gemv_lora_multi_static (the entry point that allocates nothing: t = A x lives in a static
device array) against vq_gemv_lora_multi (caller workspace), through the C ABI: two calls in a
row, the second with a smaller input, each bit-identical to the existing entry point and within
tolerance of the oracle."""
import ctypes

import numpy as np
import pytest

import oracle
import workloads

pytestmark = pytest.mark.gpu


def test_static_scratch_entry_point_matches_the_workspace_one():
    import torch
    import paper_2402_15319_amd as vq
    from paper_2402_15319_amd import device as vqdev
    assert torch.cuda.is_available()
    L = vq.lib()
    V = workloads.VQShape
    dev = "cuda:0"

    def problem_set(shapes, ranks, seed0):
        items = []
        for i, (s, rank) in enumerate(zip(shapes, ranks)):
            seed = seed0 + i
            idx, cb = workloads.make_weights(s, seed)
            x = workloads.make_x(s.in_features, seed)
            rng = np.random.default_rng(seed)
            A = (rng.standard_normal((max(rank, 8), s.in_features)) / np.sqrt(s.in_features)).astype(np.float16)
            B = (rng.standard_normal((s.out_features, max(rank, 8))) * 0.5).astype(np.float16)
            desc = vqdev.desc_from_shape(s)
            idx_d, cb_d = vqdev.upload_and_pack(desc, idx, cb)
            f = oracle.VQFormat(s.out_features, s.in_features, s.k, s.index_bits)
            ref = oracle.gemv_lora(f, idx, cb, x, A[:rank], B[:, :rank]) if rank else oracle.gemv(f, idx, cb, x)
            # adapters are stored with exactly `rank` rows / columns
            A_d = vqdev.to_device_bytes(np.ascontiguousarray(A[:rank])) if rank else None
            B_d = vqdev.to_device_bytes(np.ascontiguousarray(B[:, :rank])) if rank else None
            items.append((desc, idx_d, cb_d, vqdev.to_device_bytes(x), A_d, B_d, rank, ref, s))
        return items

    def run(items, static):
        n = len(items)
        ys = [torch.full((it[8].out_features,), float("nan"), dtype=torch.float32, device=dev) for it in items]
        descs = (vq.VQDesc * n)(*[it[0] for it in items])
        arr = ctypes.c_void_p * n
        idx = arr(*[it[1].data_ptr() for it in items]); cb = arr(*[it[2].data_ptr() for it in items])
        xs = arr(*[it[3].data_ptr() for it in items]); yp = arr(*[y.data_ptr() for y in ys])
        lora = (vq.VQLoraDesc * n)(*[vq.VQLoraDesc(it[4].data_ptr() if it[6] else 0, it[5].data_ptr() if it[6] else 0,
                                                  it[6], 0) for it in items])
        stream = torch.cuda.current_stream().cuda_stream
        if static:
            st = L.vq_gemv_lora_multi_static(n, descs, idx, cb, xs, lora, yp, vq.VQ_F32, stream)
        else:
            ws = torch.zeros(64 * n, dtype=torch.float32, device=dev)
            st = L.vq_gemv_lora_multi(n, descs, idx, cb, xs, lora, ws.data_ptr(), 256 * n, yp, vq.VQ_F32, stream)
        assert st == 0, vq.vq_status_string(st)
        torch.cuda.synchronize()
        return [y.cpu().numpy() for y in ys]

    # first call: a layer-sized launch (streaming kernel), ranks 64 / 16 / 0 / 32
    big = problem_set([V(4096, 4096, 16, 4), V(4096, 4096, 16, 4), V(11008, 4096, 16, 4), V(4096, 11008, 16, 4),
                       V(16384, 4096, 16, 4)], [64, 16, 0, 32, 8], 9100)
    # second call: fewer and smaller products (split-K kernel), lower ranks: stale t of the first
    # call is still in the array and must not be read
    small = problem_set([V(264, 1024, 16, 4), V(40, 768, 16, 4)], [16, 8], 9200)
    for items in (big, small):
        got_static = run(items, True)
        got_ws = run(items, False)
        for a, b, it in zip(got_static, got_ws, items):
            np.testing.assert_array_equal(a.view(np.uint32), b.view(np.uint32))       # bit for bit
            assert oracle.normwise_rel_err(a, it[7]) <= 2e-5
    # sizes beyond the static array are refused with a clear status, before anything is launched
    n = 257
    st = L.vq_gemv_lora_multi_static(n, None, None, None, None, None, None, vq.VQ_F32, 0)
    assert st == -6 and "out of range" in vq.vq_status_string(st)
