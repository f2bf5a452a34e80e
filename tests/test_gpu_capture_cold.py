"""The first vq_gemv of a process may be issued while its stream is being captured into a HIP graph.

The streaming kernel's grid size comes from an occupancy query that the library makes (and
caches) on first use; the query enqueues nothing, so a cold first call under capture must work
and replay correctly.  Runs in a fresh child process, because every other test of the session
has long since filled that cache in this one.
"""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

CHILD = r"""
import sys
import numpy as np
import torch
import oracle, workloads
import paper_2402_15319_amd as vq
from paper_2402_15319_amd import device as vqdev

s = workloads.VQShape(32776, 768, 16, 4)            # 4,097 row-blocks: the persistent streaming kernel
idx, cb = workloads.make_weights(s, 31)
x = workloads.make_x(s.in_features, 31)
desc = vqdev.desc_from_shape(s)
idx_d, cb_d = vqdev.upload_and_pack(desc, idx, cb)   # pack kernels only: no GEMV has run yet
x_d = vqdev.to_device_bytes(x)
y = torch.zeros(s.out_features, dtype=torch.float32, device="cuda:0")
torch.cuda.synchronize()
print("capturing the first vq_gemv of this process", flush=True)
g = torch.cuda.CUDAGraph()
with torch.cuda.graph(g):
    vq.vq_gemv(desc, idx_d, cb_d, x_d, y, vq.VQ_F32)
ref = oracle.gemv(oracle.VQFormat(s.out_features, s.in_features, 16, 4), idx, cb, x)
for replay in range(3):
    y.fill_(7)
    torch.cuda.synchronize()
    g.replay()
    torch.cuda.synchronize()
    err = oracle.normwise_rel_err(y.cpu().numpy(), ref)
    print(f"replay {replay}: normwise rel err {err:.2e}", flush=True)
    assert err <= 2e-5, err
y2 = torch.zeros_like(y)
vq.vq_gemv(desc, idx_d, cb_d, x_d, y2, vq.VQ_F32)   # eager, after the capture: same bits
torch.cuda.synchronize()
assert torch.equal(y, y2)
print("ok", flush=True)
"""


def test_first_gemv_of_a_process_under_stream_capture():
    env = dict(os.environ, PYTHONPATH=ROOT + os.pathsep + os.environ.get("PYTHONPATH", ""))
    res = subprocess.run([sys.executable, "-u", "-c", CHILD], cwd=ROOT, env=env, capture_output=True,
                         text=True, timeout=300)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-4000:]
    assert res.stdout.strip().endswith("ok")
