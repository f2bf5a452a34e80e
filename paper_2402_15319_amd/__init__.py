"""Python binding of libvq (MI355X / gfx950 vector-quantised GEMV library).

Argument marshalling only: every step of the path runs in the HIP kernels behind
the C ABI declared in include/vq.h.  Tensors are used for device memory and
streams, nothing else.  There is no CPU fallback: if the shared library is not
built, importing the binding's functions raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Sequence

__all__ = [
    "VQDesc", "VQError", "VQ_F16", "VQ_F32", "VQ_I8", "VQ_I8_BN", "lib", "lib_path", "make_desc",
    "vq_status_string", "vq_version", "vq_canonical_bytes", "vq_layout_bytes",
    "vq_pack_layout", "vq_gemv", "vq_gemv_multi", "GemvMultiArgs", "VQLoraDesc", "vq_lora_workspace_bytes", "vq_gemv_lora",
    "vq_gemv_lora_multi", "vq_gemv_lora_multi_static", "vq_gemm_batched", "vq_decode_dense", "vq_em_assign", "vq_em_update",
]

VQ_F16 = 1
VQ_F32 = 2
VQ_I8 = 3      # codebook_dtype: int8 lookup tables with one fp16 scale per group
VQ_I8_BN = 4   # the same plus blockwise normalisation (16 levels per group, a 4-bit code per 32 weights)

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libvq.so")
_lib = None


class VQDesc(ctypes.Structure):
    """Mirror of `vq_desc` (include/vq.h)."""
    _fields_ = [
        ("out_features", ctypes.c_int32), ("in_features", ctypes.c_int32),
        ("group_rows", ctypes.c_int32), ("group_cols", ctypes.c_int32),
        ("d", ctypes.c_int32), ("k", ctypes.c_int32),
        ("index_bits", ctypes.c_int32), ("codebook_dtype", ctypes.c_int32),
    ]


class VQLoraDesc(ctypes.Structure):
    """Mirror of `vq_lora_desc` (include/vq.h)."""
    _fields_ = [("A_f16", ctypes.c_void_p), ("B_f16", ctypes.c_void_p),
                ("rank", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class VQError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {vq_status_string(status)} ({status})")


def lib_path() -> str:
    return _LIB_PATH


def lib() -> ctypes.CDLL:
    """Loads libvq.so (built in-tree by `python -m paper_2402_15319_amd.build`)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(
                f"{_LIB_PATH} is not built; run `python -m paper_2402_15319_amd.build` "
                "(there is no fallback path)")
        L = ctypes.CDLL(_LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int, ctypes.POINTER(ctypes.c_size_t)
        dp = ctypes.POINTER(VQDesc)
        L.vq_status_string.restype = ctypes.c_char_p
        L.vq_status_string.argtypes = [i32]
        L.vq_version.restype = i32
        L.vq_version.argtypes = []
        for name in ("vq_canonical_bytes", "vq_layout_bytes"):
            getattr(L, name).restype = i32
            getattr(L, name).argtypes = [dp, sz, sz]
        L.vq_pack_layout.restype = i32
        L.vq_pack_layout.argtypes = [dp, vp, vp, vp, vp, vp]
        L.vq_gemv.restype = i32
        L.vq_gemv.argtypes = [dp, vp, vp, vp, vp, i32, vp]
        L.vq_gemv_multi.restype = i32
        L.vq_gemv_multi.argtypes = [i32, dp, ctypes.POINTER(vp), ctypes.POINTER(vp),
                                    ctypes.POINTER(vp), ctypes.POINTER(vp), i32, vp]
        L.vq_lora_workspace_bytes.restype = i32
        L.vq_lora_workspace_bytes.argtypes = [i32, sz]
        L.vq_gemv_lora.restype = i32
        L.vq_gemv_lora.argtypes = [dp, vp, vp, vp, vp, vp, i32, vp, ctypes.c_size_t, vp, i32, vp]
        L.vq_gemv_lora_multi.restype = i32
        L.vq_gemv_lora_multi.argtypes = [i32, dp, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp),
                                         ctypes.POINTER(VQLoraDesc), vp, ctypes.c_size_t, ctypes.POINTER(vp), i32, vp]
        L.vq_gemv_lora_multi_static.restype = i32
        L.vq_gemv_lora_multi_static.argtypes = [i32, dp, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp),
                                                ctypes.POINTER(VQLoraDesc), ctypes.POINTER(vp), i32, vp]
        L.vq_gemm_batched.restype = i32
        L.vq_gemm_batched.argtypes = [dp, vp, vp, vp, i32, i32, vp, i32, i32, vp]
        L.vq_decode_dense.restype = i32
        L.vq_decode_dense.argtypes = [dp, vp, vp, vp, vp]
        L.vq_em_assign.restype = i32
        L.vq_em_assign.argtypes = [dp, vp, vp, vp, vp, vp]
        L.vq_em_update.restype = i32
        L.vq_em_update.argtypes = [dp, vp, vp, vp, vp, vp]
        _lib = L
    return _lib


def make_desc(out_features: int, in_features: int, k: int, index_bits: int,
              group_rows: int = 8, group_cols: int = 256, d: int = 2,
              codebook_dtype: int = VQ_F16) -> VQDesc:
    return VQDesc(out_features, in_features, group_rows, group_cols, d, k, index_bits,
                  codebook_dtype)


def _ptr(t) -> int:
    """Device/host address of a tensor, or an int passed through (0 = NULL)."""
    if t is None:
        return 0
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> int:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _check(status: int, where: str) -> None:
    if status != 0:
        raise VQError(status, where)


def vq_status_string(status: int) -> str:
    return lib().vq_status_string(status).decode()


def vq_version() -> int:
    return lib().vq_version()


def vq_canonical_bytes(desc: VQDesc) -> tuple[int, int]:
    a, b = ctypes.c_size_t(0), ctypes.c_size_t(0)
    _check(lib().vq_canonical_bytes(ctypes.byref(desc), ctypes.byref(a), ctypes.byref(b)),
           "vq_canonical_bytes")
    return a.value, b.value


def vq_layout_bytes(desc: VQDesc) -> tuple[int, int]:
    a, b = ctypes.c_size_t(0), ctypes.c_size_t(0)
    _check(lib().vq_layout_bytes(ctypes.byref(desc), ctypes.byref(a), ctypes.byref(b)),
           "vq_layout_bytes")
    return a.value, b.value


def vq_pack_layout(desc: VQDesc, idx_canon, cb_canon, idx_dev, cb_dev, stream=None) -> None:
    _check(lib().vq_pack_layout(ctypes.byref(desc), _ptr(idx_canon), _ptr(cb_canon),
                                _ptr(idx_dev), _ptr(cb_dev), _stream(stream)), "vq_pack_layout")


def vq_gemv(desc: VQDesc, idx_dev, cb_dev, x, y, y_dtype: int = VQ_F16, stream=None) -> None:
    _check(lib().vq_gemv(ctypes.byref(desc), _ptr(idx_dev), _ptr(cb_dev), _ptr(x), _ptr(y),
                         y_dtype, _stream(stream)), "vq_gemv")


class GemvMultiArgs:
    """Pre-marshalled argument arrays for vq_gemv_multi (build once, call many times).  Keeps a
    reference to every tensor it was given, so the device memory behind the stored addresses
    lives as long as this object."""

    def __init__(self, descs: Sequence[VQDesc], idx_dev, cb_dev, xs, ys):
        n = len(descs)
        if not (len(idx_dev) == len(cb_dev) == len(xs) == len(ys) == n):
            raise ValueError("vq_gemv_multi: argument lists differ in length")
        self.count = n
        self.descs = (VQDesc * n)(*descs)
        arr = ctypes.c_void_p * n
        self.idx = arr(*[_ptr(t) for t in idx_dev])
        self.cb = arr(*[_ptr(t) for t in cb_dev])
        self.x = arr(*[_ptr(t) for t in xs])
        self.y = arr(*[_ptr(t) for t in ys])
        self._keep = (list(idx_dev), list(cb_dev), list(xs), list(ys))


def vq_gemv_multi(args_or_descs, idx_dev=None, cb_dev=None, xs=None, ys=None,
                  y_dtype: int = VQ_F16, stream=None) -> None:
    a = args_or_descs if isinstance(args_or_descs, GemvMultiArgs) else \
        GemvMultiArgs(args_or_descs, idx_dev, cb_dev, xs, ys)
    _check(lib().vq_gemv_multi(a.count, a.descs, a.idx, a.cb, a.x, a.y, y_dtype,
                               _stream(stream)), "vq_gemv_multi")


def vq_lora_workspace_bytes(count: int) -> int:
    a = ctypes.c_size_t(0)
    _check(lib().vq_lora_workspace_bytes(count, ctypes.byref(a)), "vq_lora_workspace_bytes")
    return a.value


def vq_gemv_lora(desc: VQDesc, idx_dev, cb_dev, x, A, B, rank: int, workspace, y,
                 y_dtype: int = VQ_F16, stream=None, workspace_bytes: int | None = None) -> None:
    nb = workspace.numel() * workspace.element_size() if workspace_bytes is None else workspace_bytes
    _check(lib().vq_gemv_lora(ctypes.byref(desc), _ptr(idx_dev), _ptr(cb_dev), _ptr(x), _ptr(A), _ptr(B), rank,
                              _ptr(workspace), nb, _ptr(y), y_dtype, _stream(stream)), "vq_gemv_lora")


def vq_gemv_lora_multi(args: GemvMultiArgs, As, Bs, ranks: Sequence[int], workspace,
                       y_dtype: int = VQ_F16, stream=None, workspace_bytes: int | None = None) -> None:
    """args as for vq_gemv_multi; As/Bs/ranks: one adapter per product (rank 0 = none)."""
    n = args.count
    if not (len(As) == len(Bs) == len(ranks) == n):
        raise ValueError("vq_gemv_lora_multi: argument lists differ in length")
    lora = (VQLoraDesc * n)(*[VQLoraDesc(_ptr(a), _ptr(b), r, 0) for a, b, r in zip(As, Bs, ranks)])
    nb = workspace.numel() * workspace.element_size() if workspace_bytes is None else workspace_bytes
    _check(lib().vq_gemv_lora_multi(n, args.descs, args.idx, args.cb, args.x, lora, _ptr(workspace), nb,
                                    args.y, y_dtype, _stream(stream)), "vq_gemv_lora_multi")


def vq_gemv_lora_multi_static(args: GemvMultiArgs, As, Bs, ranks: Sequence[int],
                              y_dtype: int = VQ_F16, stream=None) -> None:
    """vq_gemv_lora_multi without a workspace (at most 256 products; allocates nothing)."""
    n = args.count
    if not (len(As) == len(Bs) == len(ranks) == n):
        raise ValueError("vq_gemv_lora_multi_static: argument lists differ in length")
    lora = (VQLoraDesc * n)(*[VQLoraDesc(_ptr(a), _ptr(b), r, 0) for a, b, r in zip(As, Bs, ranks)])
    _check(lib().vq_gemv_lora_multi_static(n, args.descs, args.idx, args.cb, args.x, lora, args.y, y_dtype,
                                           _stream(stream)), "vq_gemv_lora_multi_static")


def vq_gemm_batched(desc: VQDesc, idx_dev, cb_dev, X, B: int, ldx: int, Y, ldy: int,
                    y_dtype: int = VQ_F16, stream=None) -> None:
    _check(lib().vq_gemm_batched(ctypes.byref(desc), _ptr(idx_dev), _ptr(cb_dev), _ptr(X), B, ldx,
                                 _ptr(Y), ldy, y_dtype, _stream(stream)), "vq_gemm_batched")


def vq_decode_dense(desc: VQDesc, idx_dev, cb_dev, W, stream=None) -> None:
    _check(lib().vq_decode_dense(ctypes.byref(desc), _ptr(idx_dev), _ptr(cb_dev), _ptr(W),
                                 _stream(stream)), "vq_decode_dense")


def vq_em_assign(desc: VQDesc, W_f32, hdiag_f32, cb_f32, assign_u8, stream=None) -> None:
    _check(lib().vq_em_assign(ctypes.byref(desc), _ptr(W_f32), _ptr(hdiag_f32), _ptr(cb_f32),
                              _ptr(assign_u8), _stream(stream)), "vq_em_assign")


def vq_em_update(desc: VQDesc, W_f32, hdiag_f32, assign_u8, cb_f32_out, stream=None) -> None:
    _check(lib().vq_em_update(ctypes.byref(desc), _ptr(W_f32), _ptr(hdiag_f32), _ptr(assign_u8),
                              _ptr(cb_f32_out), _stream(stream)), "vq_em_update")
