"""CPU oracle for the ZipServ hot path -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper over ``zs_oracle.c`` (plain scalar C, compiled with gcc).  Only
``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py``
may import this package; the product (``paper_2603_17435_amd``) never does, and this
package never imports the product.

What it computes, with the passages of the paper it follows (ZipServ, ASPLOS'26):

* ``exponent_histogram``, ``select_window``  -- Algorithm 1, phase I.
* ``encode``                                 -- Algorithm 1, phase II; Section 4.2 layout.
* ``decode`` (popcount form), ``decode_walk``-- Algorithm 2 / a cursor-walking cross-check.
* ``tile_index``                             -- the index arithmetic of Algorithm 2.
* ``average_bits3``                          -- Section 4.2, AverageBits(n) at n = 3.
* ``gemm``                                   -- Section 2.1, C = A W^T, double accumulation.
* ``gaussian_exponent_pmf``                  -- Appendix A, erf closed form.

Pins (see tests/test_oracle_pins.py): bitwise round trip on all 65536 BF16 patterns,
the worked example of Section 4.3.2, brute-force window search, cursor-walk decoder,
the AverageBits closed form against the measured array sizes, the Appendix-A erf law
on Gaussian samples, numpy float64 matmul and one-hot activations for the GEMM.
No function here is "parity unpinned".

``oracle.variants`` (numpy, its own pins in tests/test_variants_oracle.py) writes the same
encoding out for codeword lengths 2 and 4, for windows per BlockTile or per BlockTile row, and
with a dense H array.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "zs_oracle.c")
_LIB = os.path.join(_HERE, "libzs_oracle.so")


def build(force: bool = False) -> str:
    """Compile zs_oracle.c with gcc (a second or two).  Returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.run(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
             "-o", tmp, _SRC, "-lm"],
            check=True,
        )
        os.replace(tmp, _LIB)
    return _LIB


class _Info(ctypes.Structure):
    _fields_ = [
        ("N", ctypes.c_int64), ("K", ctypes.c_int64),
        ("window_start", ctypes.c_int32), ("base_exp", ctypes.c_int32),
        ("n_bt", ctypes.c_uint64), ("n_high", ctypes.c_uint64), ("n_fallback", ctypes.c_uint64),
        ("h_bytes", ctypes.c_uint64), ("l_bytes", ctypes.c_uint64),
    ]


_lib = None


def _L():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32
        lib.zso_exponent_histogram.argtypes = [vp, i64, i64, i64, vp]
        lib.zso_exponent_histogram.restype = None
        lib.zso_select_window.argtypes = [vp, vp]
        lib.zso_select_window.restype = ctypes.c_int
        lib.zso_average_bits3.argtypes = [vp, ctypes.c_int]
        lib.zso_average_bits3.restype = ctypes.c_double
        lib.zso_encode_sizes.argtypes = [vp, i64, i64, i64, ctypes.POINTER(_Info)]
        lib.zso_encode_sizes.restype = ctypes.c_int
        lib.zso_encode.argtypes = [vp, i64, i64, i64, ctypes.POINTER(_Info), vp, vp, vp, vp, vp]
        lib.zso_encode.restype = ctypes.c_int
        for name in ("zso_decode_popc", "zso_decode_walk"):
            fn = getattr(lib, name)
            fn.argtypes = [vp, vp, vp, vp, vp, i32, i64, i64, vp, i64]
            fn.restype = ctypes.c_int
        lib.zso_tile_index.argtypes = [ctypes.c_uint64, ctypes.c_int, ctypes.POINTER(ctypes.c_int)]
        lib.zso_tile_index.restype = ctypes.c_int
        lib.zso_gemm_rows.argtypes = [vp, i64, vp, i64, i64, i64, vp, i64, vp, vp, i64, ctypes.c_int]
        lib.zso_gemm_rows.restype = None
        lib.zso_max_threads.argtypes = []
        lib.zso_max_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _p(a: np.ndarray):
    return ctypes.c_void_p(a.ctypes.data)


def _as_u16_matrix(W) -> np.ndarray:
    W = np.ascontiguousarray(W)
    if W.dtype != np.uint16 or W.ndim != 2:
        raise TypeError("expected a 2-D uint16 array of BF16 bit patterns")
    return W


@dataclass
class Encoded:
    """The TCA-TBE arrays of one weight matrix (Section 4.2)."""
    N: int
    K: int
    base_exp: int        # one per matrix; window is base_exp+1 .. base_exp+7
    window_start: int
    planes: np.ndarray   # uint64 [n_fragtiles, 3]: bit-planes 1..3 of every FragTile
    H: np.ndarray        # uint8: PackedSignMantissa, per-BlockTile segments padded to 16 B
    L: np.ndarray        # uint16: FullValue fallbacks, per-BlockTile segments padded to 16 B
    offH: np.ndarray     # uint32 [n_bt + 1], 16-byte units
    offL: np.ndarray     # uint32 [n_bt + 1], 16-byte units
    n_high: int
    n_fallback: int

    @property
    def payload_bits(self) -> int:
        """Bits the format itself needs: planes + H + L, without padding/offsets."""
        return 3 * self.N * self.K + 8 * self.n_high + 16 * self.n_fallback

    @property
    def stored_bytes(self) -> int:
        return self.planes.nbytes + self.H.nbytes + self.L.nbytes + self.offH.nbytes + self.offL.nbytes


def exponent_histogram(W) -> np.ndarray:
    W = _as_u16_matrix(W)
    hist = np.zeros(256, dtype=np.uint64)
    _L().zso_exponent_histogram(_p(W), W.shape[0], W.shape[1], W.shape[1], _p(hist))
    return hist


def select_window(hist) -> tuple[int, int]:
    """(start of the best 7-wide window, its coverage).  base_exp = start - 1."""
    hist = np.ascontiguousarray(hist, dtype=np.uint64)
    cov = ctypes.c_uint64(0)
    s = _L().zso_select_window(_p(hist), ctypes.byref(cov))
    return int(s), int(cov.value)


def average_bits3(hist, window_start: int) -> float:
    hist = np.ascontiguousarray(hist, dtype=np.uint64)
    return float(_L().zso_average_bits3(_p(hist), int(window_start)))


def encode(W) -> Encoded:
    W = _as_u16_matrix(W)
    N, K = W.shape
    info = _Info()
    rc = _L().zso_encode_sizes(_p(W), N, K, K, ctypes.byref(info))
    if rc != 0:
        raise ValueError(f"zso_encode_sizes failed: {rc}")
    n_bt = int(info.n_bt)
    planes = np.zeros((n_bt * 64, 3), dtype=np.uint64)
    H = np.zeros(int(info.h_bytes), dtype=np.uint8)
    L = np.zeros(int(info.l_bytes) // 2, dtype=np.uint16)
    offH = np.zeros(n_bt + 1, dtype=np.uint32)
    offL = np.zeros(n_bt + 1, dtype=np.uint32)
    rc = _L().zso_encode(_p(W), N, K, K, ctypes.byref(info), _p(planes), _p(H), _p(L), _p(offH), _p(offL))
    if rc != 0:
        raise ValueError(f"zso_encode failed: {rc}")
    return Encoded(N, K, int(info.base_exp), int(info.window_start), planes, H, L, offH, offL,
                   int(info.n_high), int(info.n_fallback))


def _decode(fn_name: str, enc: Encoded) -> np.ndarray:
    out = np.zeros((enc.N, enc.K), dtype=np.uint16)
    rc = getattr(_L(), fn_name)(_p(enc.planes), _p(enc.H), _p(enc.L), _p(enc.offH), _p(enc.offL),
                                enc.base_exp, enc.N, enc.K, _p(out), enc.K)
    if rc != 0:
        raise ValueError(f"{fn_name} failed: {rc}")
    return out


def decode(enc: Encoded) -> np.ndarray:
    """Algorithm 2 (masked-popcount addressing)."""
    return _decode("zso_decode_popc", enc)


def decode_walk(enc: Encoded) -> np.ndarray:
    """Cursor-walking decoder, independent of the popcount arithmetic."""
    return _decode("zso_decode_walk", enc)


def tile_index(M: int, p: int) -> tuple[bool, int]:
    idx = ctypes.c_int(0)
    is_high = _L().zso_tile_index(ctypes.c_uint64(M), int(p), ctypes.byref(idx))
    return bool(is_high), int(idx.value)


def max_threads() -> int:
    return int(_L().zso_max_threads())


def gemm(A, W, rows=None, threads: int = 1) -> tuple[np.ndarray, np.ndarray]:
    """C[m, j] = sum_k A[m,k] * W[rows[j], k] (double, ascending k) and S = sum |.|.

    ``A`` [M, K] and ``W`` [N, K] are uint16 BF16 bit patterns; ``rows`` selects rows of
    W (all rows when None).  Returns (C, S), both float64 [M, len(rows)]."""
    A = _as_u16_matrix(A)
    W = _as_u16_matrix(W)
    M, K = A.shape
    if W.shape[1] != K:
        raise ValueError("inner dimensions differ")
    if rows is None:
        n_rows, rows_p = W.shape[0], ctypes.c_void_p(0)
    else:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        if rows.size and (rows.min() < 0 or rows.max() >= W.shape[0]):
            raise ValueError("row index out of range")
        n_rows, rows_p = rows.size, _p(rows)
    C = np.zeros((M, n_rows), dtype=np.float64)
    S = np.zeros((M, n_rows), dtype=np.float64)
    _L().zso_gemm_rows(_p(A), K, _p(W), K, M, K, rows_p, n_rows, _p(C), _p(S), n_rows, int(threads))
    return C, S


def gaussian_exponent_pmf(sigma: float) -> np.ndarray:
    """Appendix A: P(E = x + 127) = erf(2^(x+1) / (sigma sqrt 2)) - erf(2^x / (sigma sqrt 2))
    for the normal exponents E = 1..254 (index = E).  Rounding to BF16 is ignored, as in
    the paper's derivation."""
    pmf = np.zeros(256, dtype=np.float64)
    for E in range(1, 255):
        x = E - 127
        pmf[E] = math.erf(2.0 ** (x + 1) / (sigma * math.sqrt(2.0))) - math.erf(2.0 ** x / (sigma * math.sqrt(2.0)))
    return pmf
