"""Device-memory plumbing around the binding (torch is used for allocation only)."""
from __future__ import annotations

import numpy as np
import torch

from . import VQDesc, VQ_F16, VQ_I8, VQ_I8_BN, make_desc, vq_canonical_bytes, vq_layout_bytes, vq_pack_layout


def desc_from_shape(s) -> VQDesc:
    """VQDesc from any object with out_features/in_features/k/index_bits/group_* /d fields."""
    dtype = VQ_F16
    if getattr(s, "int8_tables", False):
        dtype = VQ_I8_BN if getattr(s, "block_norm", False) else VQ_I8
    return make_desc(s.out_features, s.in_features, s.k, s.index_bits,
                     s.group_rows, s.group_cols, s.d, dtype)


def canonical_tables_i8(desc: VQDesc, q: np.ndarray, scale: np.ndarray) -> np.ndarray:
    """Canonical table buffer of the VQ_I8 representation: the int8 tables q[g, k, d],
    zero-padded to a multiple of 16 bytes, then the fp16 scales scale[g] (byte copy only)."""
    assert q.dtype == np.int8 and scale.dtype == np.float16
    _, cb_bytes = vq_canonical_bytes(desc)
    buf = np.zeros(cb_bytes, dtype=np.uint8)
    qb = np.ascontiguousarray(q).view(np.uint8).reshape(-1)
    sb = np.ascontiguousarray(scale).view(np.uint8).reshape(-1)
    buf[:qb.size] = qb
    off = (qb.size + 15) // 16 * 16
    assert off + sb.size == cb_bytes
    buf[off:] = sb
    return buf


def canonical_tables_bn(desc: VQDesc, q: np.ndarray, scale: np.ndarray, levels: np.ndarray,
                        codes: np.ndarray) -> np.ndarray:
    """Canonical table buffer of the VQ_I8_BN representation: q and scale as for VQ_I8, each
    padded to 16 bytes, then the fp16 levels[g, 16], then the 4-bit block codes codes[out, in/32]
    two per byte, even block in the low nibble (byte copies and nibble packing only)."""
    assert q.dtype == np.int8 and scale.dtype == np.float16 and levels.dtype == np.float16
    assert codes.dtype == np.uint8 and codes.shape[1] % 2 == 0
    _, cb_bytes = vq_canonical_bytes(desc)
    buf = np.zeros(cb_bytes, dtype=np.uint8)
    off = 0
    for part in (q, scale):
        b = np.ascontiguousarray(part).view(np.uint8).reshape(-1)
        buf[off:off + b.size] = b
        off = (off + b.size + 15) // 16 * 16
    lb = np.ascontiguousarray(levels).view(np.uint8).reshape(-1)
    buf[off:off + lb.size] = lb
    off += lb.size
    packed = (codes[:, 0::2] | (codes[:, 1::2] << 4)).astype(np.uint8).reshape(-1)
    assert off + packed.size == cb_bytes
    buf[off:] = packed
    return buf


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
