"""Thin ctypes binding of libzipserv_hip.so: argument marshalling only.

Every step of the path (packing, decoding, the GEMM) runs inside the library; there is no
Python or CPU fallback.  If the shared library is missing and cannot be built the import
of any entry point raises.  PyTorch is used by callers for device memory and streams; the
functions here accept anything with ``data_ptr()`` (torch tensors) or raw integer addresses.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from . import build as _build

ZS_OK = 0
_STATUS = {0: "ZS_OK", -1: "ZS_ERR_ARG", -2: "ZS_ERR_SHAPE", -3: "ZS_ERR_SIZE", -4: "ZS_ERR_FORMAT",
           -5: "ZS_ERR_HIP", -6: "ZS_ERR_CONFIG"}

EXPORTS = ["zs_encode_bound", "zs_encode", "zs_encode_device", "zs_desc_validate", "zs_decompress", "zs_gemm_workspace", "zs_gemm",
           "zs_gemm_ex", "zs_gemm_workspace_ex", "zs_gemm_config_name", "zs_gemm_num_configs",
           "zs_gemm_pick_config", "zs_gemm_noalloc", "zs_gemm_bf16", "zs_dense_gemm", "zs_dense_gemm_algos", "zs_linear",
           "zs_linear_path", "zs_linear_workspace", "zs_compute_units", "zs_strerror", "zs_version",
           "zs_variant_bound", "zs_variant_encode", "zs_variant_validate", "zs_variant_decompress"]


class ZsError(RuntimeError):
    def __init__(self, fn: str, status: int):
        self.status = status
        msg = lib().zs_strerror(status).decode() if _lib is not None else ""
        super().__init__(f"{fn} failed: {_STATUS.get(status, status)} ({msg})")


class ZsDesc(ctypes.Structure):
    """Mirror of ``zs_desc`` in include/zipserv.h."""
    _fields_ = [
        ("magic", ctypes.c_uint32), ("version", ctypes.c_uint32),
        ("N", ctypes.c_int64), ("K", ctypes.c_int64),
        ("base_exp", ctypes.c_int32), ("tile_cfg", ctypes.c_uint32),
        ("n_high", ctypes.c_uint64), ("n_fallback", ctypes.c_uint64),
        ("off_bitmaps", ctypes.c_uint64), ("off_offsets", ctypes.c_uint64),
        ("off_H", ctypes.c_uint64), ("off_L", ctypes.c_uint64),
        ("h_bytes", ctypes.c_uint64), ("l_bytes", ctypes.c_uint64),
        ("total_bytes", ctypes.c_uint64),
        ("max_h_units", ctypes.c_uint32), ("max_l_units", ctypes.c_uint32),
    ]


class ZsVariantDesc(ctypes.Structure):
    """Mirror of ``zs_variant_desc`` in include/zipserv.h."""
    _fields_ = [
        ("magic", ctypes.c_uint32), ("version", ctypes.c_uint32),
        ("n_planes", ctypes.c_int32), ("base_mode", ctypes.c_int32),
        ("dense_h", ctypes.c_int32), ("reserved", ctypes.c_int32),
        ("N", ctypes.c_int64), ("K", ctypes.c_int64),
        ("n_high", ctypes.c_uint64), ("n_fallback", ctypes.c_uint64),
        ("off_planes", ctypes.c_uint64), ("off_offsets", ctypes.c_uint64), ("off_bases", ctypes.c_uint64),
        ("off_H", ctypes.c_uint64), ("off_L", ctypes.c_uint64),
        ("h_bytes", ctypes.c_uint64), ("l_bytes", ctypes.c_uint64),
        ("total_bytes", ctypes.c_uint64),
    ]


ZS_BASE_MATRIX, ZS_BASE_TILE, ZS_BASE_ROW = 0, 1, 2

_lib = None


def lib() -> ctypes.CDLL:
    """Loads the built library; builds it first only when none exists."""
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path):
            path = _build.build()
        L = ctypes.CDLL(path)
        vp, i64, sz, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_size_t, ctypes.c_int
        dp = ctypes.POINTER(ZsDesc)
        L.zs_encode_bound.argtypes, L.zs_encode_bound.restype = [i64, i64], sz
        L.zs_encode.argtypes, L.zs_encode.restype = [vp, i64, i64, i64, vp, sz, dp, ci], ci
        L.zs_encode_device.argtypes, L.zs_encode_device.restype = [vp, i64, i64, i64, vp, sz, dp, vp, sz, vp], ci
        L.zs_desc_validate.argtypes, L.zs_desc_validate.restype = [dp], ci
        L.zs_decompress.argtypes, L.zs_decompress.restype = [dp, vp, vp, i64, vp], ci
        L.zs_gemm_workspace.argtypes, L.zs_gemm_workspace.restype = [dp, i64], sz
        L.zs_gemm_workspace_ex.argtypes, L.zs_gemm_workspace_ex.restype = [dp, i64, ci], sz
        L.zs_gemm.argtypes, L.zs_gemm.restype = [dp, vp, vp, i64, vp, i64, i64, vp, sz, vp], ci
        L.zs_gemm_ex.argtypes, L.zs_gemm_ex.restype = [dp, vp, vp, i64, vp, i64, i64, vp, sz, vp, ci], ci
        L.zs_gemm_bf16.argtypes, L.zs_gemm_bf16.restype = [dp, vp, vp, i64, vp, i64, i64, vp, sz, vp], ci
        L.zs_gemm_noalloc.argtypes, L.zs_gemm_noalloc.restype = [dp, vp, vp, i64, vp, i64, i64, vp], ci
        L.zs_dense_gemm.argtypes = [vp, i64, vp, i64, vp, i64, i64, i64, i64, vp, sz, vp, ci]
        L.zs_dense_gemm.restype = ci
        L.zs_dense_gemm_algos.argtypes, L.zs_dense_gemm_algos.restype = [i64, i64, i64, i64, i64, i64, sz], ci
        L.zs_linear.argtypes, L.zs_linear.restype = [dp, vp, vp, i64, vp, i64, i64, vp, sz, vp], ci
        L.zs_linear_path.argtypes, L.zs_linear_path.restype = [dp, i64], ci
        L.zs_linear_workspace.argtypes, L.zs_linear_workspace.restype = [dp, i64], sz
        L.zs_compute_units.argtypes, L.zs_compute_units.restype = [], ci
        L.zs_gemm_config_name.argtypes, L.zs_gemm_config_name.restype = [ci], ctypes.c_char_p
        L.zs_gemm_num_configs.argtypes, L.zs_gemm_num_configs.restype = [], ci
        L.zs_gemm_pick_config.argtypes, L.zs_gemm_pick_config.restype = [dp, i64], ci
        L.zs_strerror.argtypes, L.zs_strerror.restype = [ci], ctypes.c_char_p
        L.zs_version.argtypes, L.zs_version.restype = [], ci
        vdp = ctypes.POINTER(ZsVariantDesc)
        L.zs_variant_bound.argtypes, L.zs_variant_bound.restype = [i64, i64, ci, ci, ci], sz
        L.zs_variant_encode.argtypes, L.zs_variant_encode.restype = [vp, i64, i64, i64, ci, ci, ci, vp, sz, vdp, ci], ci
        L.zs_variant_validate.argtypes, L.zs_variant_validate.restype = [vdp], ci
        L.zs_variant_decompress.argtypes, L.zs_variant_decompress.restype = [vdp, vp, vp, i64, vp], ci
        _lib = L
    return _lib


def _ptr(x) -> ctypes.c_void_p:
    if x is None:
        return ctypes.c_void_p(0)
    if hasattr(x, "data_ptr"):
        return ctypes.c_void_p(x.data_ptr())
    if isinstance(x, np.ndarray):
        return ctypes.c_void_p(x.ctypes.data)
    return ctypes.c_void_p(int(x))


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(getattr(stream, "cuda_stream", stream))


def _check(fn: str, rc: int) -> None:
    if rc != ZS_OK:
        raise ZsError(fn, rc)


def aligned_empty(nbytes: int, align: int = 256) -> np.ndarray:
    raw = np.empty(nbytes + align, dtype=np.uint8)
    off = (-raw.ctypes.data) % align
    return raw[off:off + nbytes]


def zs_encode_bound(N: int, K: int) -> int:
    return int(lib().zs_encode_bound(N, K))


def zs_encode(W: np.ndarray, threads: int = 0) -> tuple[np.ndarray, ZsDesc]:
    """Packs a [N, K] uint16 (BF16 bit patterns) host matrix.  Returns (blob, desc); the blob
    is a 256-byte-aligned uint8 array trimmed to ``desc.total_bytes``."""
    if W.dtype != np.uint16 or W.ndim != 2 or W.strides[1] != 2:
        raise TypeError("W must be a 2-D uint16 array with unit column stride")
    N, K = W.shape
    cap = zs_encode_bound(N, K)
    if cap == 0:
        raise ZsError("zs_encode_bound", -2)
    blob = aligned_empty(cap)
    desc = ZsDesc()
    _check("zs_encode", lib().zs_encode(_ptr(W), N, K, W.strides[0] // 2, _ptr(blob), cap, ctypes.byref(desc), threads))
    return blob[:desc.total_bytes], desc


ZS_ENCODE_WORKSPACE_BYTES = 4096


def zs_encode_device(W_dev, N: int, K: int, blob_dev, blob_cap: int, workspace_dev, ldw: int | None = None,
                     stream=None) -> ZsDesc:
    """Packs a [N, K] BF16 matrix that lies in device memory into blob_dev; returns the descriptor."""
    desc = ZsDesc()
    _check("zs_encode_device", lib().zs_encode_device(_ptr(W_dev), N, K, K if ldw is None else ldw, _ptr(blob_dev), blob_cap,
                                                       ctypes.byref(desc), _ptr(workspace_dev), ZS_ENCODE_WORKSPACE_BYTES,
                                                       _stream(stream)))
    return desc


def zs_desc_validate(desc: ZsDesc) -> int:
    return int(lib().zs_desc_validate(ctypes.byref(desc)))


def zs_decompress(desc: ZsDesc, blob_dev, W_out_dev, ldw: int | None = None, stream=None) -> None:
    _check("zs_decompress", lib().zs_decompress(ctypes.byref(desc), _ptr(blob_dev), _ptr(W_out_dev),
                                                  desc.K if ldw is None else ldw, _stream(stream)))


def zs_variant_bound(N: int, K: int, n_planes: int, base_mode: int, dense_h: int) -> int:
    return int(lib().zs_variant_bound(N, K, n_planes, base_mode, dense_h))


def zs_variant_encode(W: np.ndarray, n_planes: int, base_mode: int, dense_h: int, threads: int = 0) -> tuple[np.ndarray, ZsVariantDesc]:
    """Packs a host matrix in a format variant; returns (blob trimmed to total_bytes, descriptor)."""
    if W.dtype != np.uint16 or W.ndim != 2 or W.strides[1] != 2:
        raise TypeError("W must be a 2-D uint16 array with unit column stride")
    N, K = W.shape
    cap = zs_variant_bound(N, K, n_planes, base_mode, dense_h)
    if cap == 0:
        raise ZsError("zs_variant_bound", -2)
    blob = aligned_empty(cap)
    desc = ZsVariantDesc()
    _check("zs_variant_encode", lib().zs_variant_encode(_ptr(W), N, K, W.strides[0] // 2, n_planes, base_mode, dense_h,
                                                         _ptr(blob), cap, ctypes.byref(desc), threads))
    return blob[:desc.total_bytes], desc


def zs_variant_validate(desc: ZsVariantDesc) -> int:
    return int(lib().zs_variant_validate(ctypes.byref(desc)))


def zs_variant_decompress(desc: ZsVariantDesc, blob_dev, W_out_dev, ldw: int | None = None, stream=None) -> None:
    _check("zs_variant_decompress", lib().zs_variant_decompress(ctypes.byref(desc), _ptr(blob_dev), _ptr(W_out_dev),
                                                                 desc.K if ldw is None else ldw, _stream(stream)))


def zs_gemm_workspace(desc: ZsDesc, M: int, config: int = 0) -> int:
    return int(lib().zs_gemm_workspace_ex(ctypes.byref(desc), M, config))


def zs_gemm(desc: ZsDesc, blob_dev, A_dev, C_dev, M: int, lda: int | None = None, ldc: int | None = None,
            workspace_dev=None, workspace_bytes: int = 0, stream=None, config: int = 0) -> None:
    """C = A decode(W)^T.  workspace_dev is optional scratch of zs_gemm_workspace() bytes that the
    caller zero-fills once (torch.zeros) and may then reuse for every call on the same stream."""
    _check("zs_gemm", lib().zs_gemm_ex(ctypes.byref(desc), _ptr(blob_dev), _ptr(A_dev),
                                        desc.K if lda is None else lda, _ptr(C_dev),
                                        desc.N if ldc is None else ldc, M, _ptr(workspace_dev),
                                        workspace_bytes, _stream(stream), config))


def zs_gemm_bf16(desc: ZsDesc, blob_dev, A_dev, C_dev, M: int, lda: int | None = None, ldc: int | None = None,
                 workspace_dev=None, workspace_bytes: int = 0, stream=None) -> None:
    """C (BF16 bit patterns) = bf16(A decode(W)^T); the scratch workspace is required (see zs_gemm)."""
    _check("zs_gemm_bf16", lib().zs_gemm_bf16(ctypes.byref(desc), _ptr(blob_dev), _ptr(A_dev),
                                               desc.K if lda is None else lda, _ptr(C_dev),
                                               desc.N if ldc is None else ldc, M, _ptr(workspace_dev),
                                               workspace_bytes, _stream(stream)))


def zs_gemm_noalloc(desc: ZsDesc, blob_dev, A_dev, C_dev, M: int, lda: int | None = None, ldc: int | None = None,
                    stream=None) -> None:
    """zs_gemm for callers that cannot allocate: its scratch is a device array inside the library."""
    _check("zs_gemm_noalloc", lib().zs_gemm_noalloc(ctypes.byref(desc), _ptr(blob_dev), _ptr(A_dev),
                                                    desc.K if lda is None else lda, _ptr(C_dev),
                                                    desc.N if ldc is None else ldc, M, _stream(stream)))


ZS_PATH_FUSED, ZS_PATH_DECOUPLED = 0, 1
ZS_DENSE_WORKSPACE_BYTES = 32 << 20


def zs_dense_gemm(A_dev, W_dev, C_dev, M: int, N: int, K: int, lda: int | None = None, ldw: int | None = None,
                  ldc: int | None = None, workspace_dev=None, workspace_bytes: int = 0, stream=None, algo: int = 0) -> None:
    """C[M,N] (FP32) = A[M,K] W[N,K]^T on uncompressed BF16 weights through hipBLASLt."""
    _check("zs_dense_gemm", lib().zs_dense_gemm(_ptr(A_dev), K if lda is None else lda, _ptr(W_dev),
                                                  K if ldw is None else ldw, _ptr(C_dev), N if ldc is None else ldc,
                                                  M, N, K, _ptr(workspace_dev), workspace_bytes, _stream(stream), algo))


def zs_dense_gemm_algos(M: int, N: int, K: int, workspace_bytes: int = 0) -> int:
    n = int(lib().zs_dense_gemm_algos(M, N, K, K, K, N, workspace_bytes))
    _check("zs_dense_gemm_algos", min(n, 0))
    return n


def zs_linear_path(desc: ZsDesc, M: int) -> int:
    return int(lib().zs_linear_path(ctypes.byref(desc), M))


def zs_linear_workspace(desc: ZsDesc, M: int) -> int:
    return int(lib().zs_linear_workspace(ctypes.byref(desc), M))


def zs_linear(desc: ZsDesc, blob_dev, A_dev, C_dev, M: int, lda: int | None = None, ldc: int | None = None,
              workspace_dev=None, workspace_bytes: int = 0, stream=None) -> None:
    """Stage-aware C = A decode(W)^T: fused ZipGEMM for few tokens, zs_decompress + dense GEMM for many."""
    _check("zs_linear", lib().zs_linear(ctypes.byref(desc), _ptr(blob_dev), _ptr(A_dev), desc.K if lda is None else lda,
                                          _ptr(C_dev), desc.N if ldc is None else ldc, M, _ptr(workspace_dev),
                                          workspace_bytes, _stream(stream)))


def zs_gemm_configs() -> dict[int, str]:
    L = lib()
    return {i: L.zs_gemm_config_name(i).decode() for i in range(1, L.zs_gemm_num_configs() + 1)}


def zs_gemm_pick_config(desc: ZsDesc, M: int) -> int:
    return int(lib().zs_gemm_pick_config(ctypes.byref(desc), M))
