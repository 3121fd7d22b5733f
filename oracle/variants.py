"""CPU oracle for the format variants of TCA-TBE -- TEST INFRASTRUCTURE ONLY.

Plain numpy / Python, one FragTile at a time; slow on purpose.  Only ``tests/`` and the
checking legs of ``bench.py`` may import it; the product never does, and this module imports
nothing of the product.

The paper fixes the codeword length at n = 3 after comparing it with n = 2 and n = 4
(Section 4.2, "The Choice of Codeword Length": AverageBits(n) = r_n (n + 8) + (1 - r_n)(n + 16),
r_n = share of the weights whose exponent is one of the 2^n - 1 covered values).  This module
writes the same encoding out for any n in {2, 3, 4}:

* n bit-planes per 8 x 8 FragTile; the codeword of element p is bit p of plane 1 (LSB) ..
  plane n (MSB); codeword c in 1 .. 2^n - 1 stands for exponent base_exp + c, codeword 0 for a
  fallback (Section 4.2, Algorithm 1 phase II, with 7 replaced by 2^n - 1);
* the window is the run of 2^n - 1 consecutive exponents that covers most elements, the
  smallest start winning a tie (Algorithm 1 phase I; contiguity: Appendix A);
* ``base``: "matrix" = one window per matrix (the paper's); "tile" = one per 64 x 64 BlockTile;
  "row" = one per row of a BlockTile (64 elements).  The finer two are NOT in the paper: an
  extension for matrices whose blocks or rows differ in scale;
* ``dense_h``: every element owns a sign+mantissa byte at a fixed place (64 per FragTile, the
  byte of a fallback element is zero), only fallbacks go to L.  NOT in the paper either: it
  trades 8 (1 - r) more bits per element for a decoder that needs no prefix count on the common
  path.

Element order inside a BlockTile: TensorCoreTile tt = 0..7 (rows 16 (tt % 4), columns
32 (tt / 4)), FragTile ft = 0..7 inside it (rows + 8 (ft % 2), columns + 8 (ft / 2)), element
p = 8 r + c inside the FragTile -- the same nesting as the n = 3 format, so that the n = 3,
per-matrix, sparse-H variant is that format array for array.

Pins (tests/test_variants_oracle.py): bitwise round trip over all 65536 BF16 patterns for all
eighteen variants; the (3, per-matrix, sparse) variant equals the arrays of the C oracle's
``encode``; measured payload bits equal AverageBits(n) evaluated at the measured r_n; r_n on
Gaussian samples equals the Appendix-A erf law summed over the window; the three averages the
paper prints are mutually consistent under the formula; finer windows never cover fewer
elements than coarser ones; brute-force window search.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np

BT = 64  # BlockTile edge


def window_width(n: int) -> int:
    if n not in (2, 3, 4):
        raise ValueError("codeword length must be 2, 3 or 4")
    return (1 << n) - 1


def average_bits(n: int, r: float) -> float:
    """Section 4.2: expected bits per element at codeword length n and coverage r."""
    return r * (n + 8) + (1.0 - r) * (n + 16)


def select_window(hist, n: int) -> tuple[int, int]:
    """(start, coverage) of the best run of 2^n - 1 consecutive exponents; smallest start on ties."""
    hist = np.asarray(hist, dtype=np.int64)
    w = window_width(n)
    best_start, best_cov = 0, -1
    for s in range(0, 256 - w + 1):
        cov = int(hist[s:s + w].sum())
        if cov > best_cov:
            best_start, best_cov = s, cov
    return best_start, best_cov


def fragtile_origin(tt: int, ft: int) -> tuple[int, int]:
    return 16 * (tt % 4) + 8 * (ft % 2), 32 * (tt // 4) + 8 * (ft // 2)


@dataclass
class VariantEncoded:
    N: int
    K: int
    n: int
    base: str            # "matrix", "tile" or "row"
    dense_h: bool
    win_lo: np.ndarray   # uint8 [n_bt, 64]: first exponent (base_exp + 1) of the window of each BlockTile row
    planes: np.ndarray   # uint64 [n_bt * 64, n]
    H: np.ndarray        # uint8, per-BlockTile segments padded to 16 bytes
    L: np.ndarray        # uint16, per-BlockTile segments padded to 16 bytes
    offH: np.ndarray     # uint32 [n_bt + 1], 16-byte units
    offL: np.ndarray     # uint32 [n_bt + 1], 16-byte units
    n_high: int
    n_fallback: int

    @property
    def payload_bits(self) -> int:
        """Bits of planes + H + L without padding, offsets or window bytes."""
        h = self.N * self.K if self.dense_h else self.n_high
        return self.n * self.N * self.K + 8 * h + 16 * self.n_fallback


def _exponents(W: np.ndarray) -> np.ndarray:
    return (W >> 7) & 0xFF


BASES = ("matrix", "tile", "row")


def encode(W: np.ndarray, n: int = 3, base: str = "matrix", dense_h: bool = False) -> VariantEncoded:
    W = np.ascontiguousarray(W)
    if W.dtype != np.uint16 or W.ndim != 2:
        raise TypeError("expected a 2-D uint16 array of BF16 bit patterns")
    N, K = W.shape
    if N <= 0 or K <= 0 or N % BT or K % BT:
        raise ValueError("N and K must be positive multiples of 64")
    if base not in BASES:
        raise ValueError("base must be one of " + ", ".join(BASES))
    width = window_width(n)
    n_bt = (N // BT) * (K // BT)
    if base == "matrix":
        start, _ = select_window(np.bincount(_exponents(W).ravel(), minlength=256), n)
    planes = np.zeros((n_bt * 64, n), dtype=np.uint64)
    win_lo = np.zeros((n_bt, BT), dtype=np.uint8)
    offH = np.zeros(n_bt + 1, dtype=np.uint32)
    offL = np.zeros(n_bt + 1, dtype=np.uint32)
    h_parts, l_parts = [], []
    n_high = 0
    for bt in range(n_bt):
        strip, kb = divmod(bt, K // BT)
        tile = W[strip * BT:(strip + 1) * BT, kb * BT:(kb + 1) * BT]
        if base == "tile":
            start, _ = select_window(np.bincount(_exponents(tile).ravel(), minlength=256), n)
        for row in range(BT):
            win_lo[bt, row] = start if base != "row" else select_window(
                np.bincount(_exponents(tile[row]), minlength=256), n)[0]
        h_seg, l_seg = [], []
        for tt in range(8):
            for ft in range(8):
                r0, c0 = fragtile_origin(tt, ft)
                frag = tile[r0:r0 + 8, c0:c0 + 8].ravel()  # p = 8 r + c
                for p in range(64):
                    w = int(frag[p])
                    d = ((w >> 7) & 0xFF) - int(win_lo[bt, r0 + p // 8])
                    if 0 <= d < width:
                        code = d + 1
                        for i in range(n):
                            if (code >> i) & 1:
                                planes[bt * 64 + tt * 8 + ft, i] |= np.uint64(1) << np.uint64(p)
                        h_seg.append(((w >> 8) & 0x80) | (w & 0x7F))
                    else:
                        l_seg.append(w)
                        if dense_h:
                            h_seg.append(0)
        n_high += BT * BT - len(l_seg)
        h_seg += [0] * (-len(h_seg) % 16)
        l_seg += [0] * (-len(l_seg) % 8)
        offH[bt + 1] = offH[bt] + len(h_seg) // 16
        offL[bt + 1] = offL[bt] + len(l_seg) // 8
        h_parts.append(np.array(h_seg, dtype=np.uint8))
        l_parts.append(np.array(l_seg, dtype=np.uint16))
    H = np.concatenate(h_parts) if h_parts else np.zeros(0, np.uint8)
    L = np.concatenate(l_parts) if l_parts else np.zeros(0, np.uint16)
    return VariantEncoded(N, K, n, base, dense_h, win_lo, planes, H, L, offH, offL,
                          n_high, N * K - n_high)


def decode(enc: VariantEncoded) -> np.ndarray:
    """Algorithm 2 with n planes: walk every FragTile in element order, taking the next H byte
    for a non-zero codeword and the next L halfword for a zero one."""
    out = np.zeros((enc.N, enc.K), dtype=np.uint16)
    for bt in range(enc.offH.size - 1):
        strip, kb = divmod(bt, enc.K // BT)
        h = int(enc.offH[bt]) * 16
        l = int(enc.offL[bt]) * 8
        for tt in range(8):
            for ft in range(8):
                r0, c0 = fragtile_origin(tt, ft)
                f = bt * 64 + tt * 8 + ft
                for p in range(64):
                    code = 0
                    for i in range(enc.n):
                        code |= ((int(enc.planes[f, i]) >> p) & 1) << i
                    if code:
                        b = int(enc.H[h])
                        base_exp = int(enc.win_lo[bt, r0 + p // 8]) - 1
                        w = ((b & 0x80) << 8) | ((base_exp + code) << 7) | (b & 0x7F)
                        h += 1
                    else:
                        w = int(enc.L[l])
                        l += 1
                        if enc.dense_h:
                            h += 1
                    out[strip * BT + r0 + p // 8, kb * BT + c0 + p % 8] = w
    return out


def gaussian_window_coverage(sigma: float, n: int) -> tuple[int, float]:
    """Appendix A: the exponent law of N(0, sigma^2), summed over its best window of 2^n - 1
    values.  Returns (window start, coverage)."""
    pmf = np.zeros(256)
    for E in range(1, 255):
        x = E - 127
        pmf[E] = math.erf(2.0 ** (x + 1) / (sigma * math.sqrt(2.0))) - math.erf(2.0 ** x / (sigma * math.sqrt(2.0)))
    w = window_width(n)
    sums = [pmf[s:s + w].sum() for s in range(256 - w + 1)]
    s = int(np.argmax(sums))
    return s, float(sums[s])
