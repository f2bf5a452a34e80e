"""Device-memory plumbing around the binding (torch is used for allocation only)."""
from __future__ import annotations

import numpy as np
import torch

from . import VQDesc, VQ_F16, VQ_I8, VQ_I8_BN, make_desc, vq_layout_bytes, vq_pack_layout


def desc_from_shape(s) -> VQDesc:
    """VQDesc from any object with out_features/in_features/k/index_bits/group_* /d fields."""
    dtype = VQ_F16
    if getattr(s, "int8_tables", False):
        dtype = VQ_I8_BN if getattr(s, "block_norm", False) else VQ_I8
    return make_desc(s.out_features, s.in_features, s.k, s.index_bits,
                     s.group_rows, s.group_cols, s.d, dtype)


def to_device_bytes(a: np.ndarray, device="cuda:0") -> torch.Tensor:
    """Host array -> uint8 device tensor holding the same bytes."""
    flat = np.ascontiguousarray(a).view(np.uint8).reshape(-1)
    return torch.from_numpy(flat.copy()).to(device)


def upload_and_pack(desc: VQDesc, idx_canon: np.ndarray, cb_canon: np.ndarray,
                    device="cuda:0"):
    """Canonical host arrays -> (idx_dev, cb_dev) device-layout tensors via vq_pack_layout."""
    idx_c = to_device_bytes(idx_canon, device)
    cb_c = to_device_bytes(cb_canon, device)
    ib, cbb = vq_layout_bytes(desc)
    idx_d = torch.empty(ib, dtype=torch.uint8, device=device)
    cb_d = torch.empty(cbb, dtype=torch.uint8, device=device)
    vq_pack_layout(desc, idx_c, cb_c, idx_d, cb_d)
    torch.cuda.synchronize()
    return idx_d, cb_d
