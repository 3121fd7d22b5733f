"""Seeded synthetic inputs for the ZipGEMM path.

This module holds no arithmetic of the method itself: it only draws numbers and rounds
them to BF16.  Both the tests (which feed the CPU oracle and the HIP library the same
arrays) and bench.py use it.  Real model weights are not available offline, so the
layer *shapes* of the paper's kernel benchmark (Section 6.1, LLaMA-3.1 family) are kept
and the value distributions are stand-ins: the zero-mean Gaussian of Appendix A and a set
of adversarial laws that stress the fallback path.

All generators are numpy ``Generator(PCG64(seed))``; FP32 -> BF16 is round-to-nearest-even.
Seed convention: ``1000 * config_id + 10 * matrix_index + variant``.
"""
from __future__ import annotations

import numpy as np

# (name, N = out features, K = hidden) -- LLaMA-3.1-8B / 70B linear layers.
LLAMA3_8B_LAYERS = [("qkv", 6144, 4096), ("o", 4096, 4096), ("gate_up", 28672, 4096), ("down", 4096, 14336)]
LLAMA3_70B_LAYERS = [("qkv", 10240, 8192), ("o", 8192, 8192), ("gate_up", 57344, 8192), ("down", 8192, 28672)]
# the seven projections of one 8B decoder layer, stored separately
LLAMA3_8B_PROJECTIONS = [("q", 4096, 4096), ("k", 1024, 4096), ("v", 1024, 4096), ("o", 4096, 4096),
                         ("gate", 14336, 4096), ("up", 14336, 4096), ("down", 4096, 14336)]

SPECIAL_PATTERNS = {
    "pos_zero": [0x0000], "neg_zero": [0x8000],
    "subnormal": [0x0001, 0x007F, 0x8001, 0x807F],
    "inf": [0x7F80, 0xFF80],
    "nan": [0x7FC0, 0x7F81, 0xFFFF],
}


def seed_for(config_id: int, matrix_index: int = 0, variant: int = 0) -> int:
    return 1000 * config_id + 10 * matrix_index + variant


def f32_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 -> BF16 bit patterns (uint16), round to nearest even; NaN stays NaN."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    with np.errstate(over="ignore"):  # the sum wraps only for NaN patterns, which are replaced below
        r = bits + np.uint32(0x7FFF)
        r += (bits >> np.uint32(16)) & np.uint32(1)
    rounded = (r >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        rounded[nan] = ((bits[nan] >> 16) | 0x0040).astype(np.uint16)
    return rounded


def bf16_to_f32(u: np.ndarray) -> np.ndarray:
    """BF16 bit patterns (uint16) -> float32, exact."""
    return (np.ascontiguousarray(u, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def _rows_chunked(N: int, K: int, fn, chunk_elems: int = 1 << 24) -> np.ndarray:
    out = np.empty((N, K), dtype=np.uint16)
    rows = max(1, chunk_elems // K)
    for r0 in range(0, N, rows):
        r1 = min(N, r0 + rows)
        out[r0:r1] = f32_to_bf16(fn(r0, r1))
    return out


def gaussian_weights(N: int, K: int, seed: int, sigma: float = 0.02) -> np.ndarray:
    """i.i.d. N(0, sigma^2), the Appendix-A model."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return _rows_chunked(N, K, lambda r0, r1: rng.standard_normal((r1 - r0, K), dtype=np.float32) * np.float32(sigma))


def student_t_weights(N: int, K: int, seed: int, nu: float = 3.0, scale: float = 0.02) -> np.ndarray:
    """Heavy tails: Student-t(nu) * scale."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return _rows_chunked(N, K, lambda r0, r1: (rng.standard_t(nu, (r1 - r0, K)) * scale).astype(np.float32))


def outlier_weights(N: int, K: int, seed: int, sigma: float = 0.02, frac: float = 1e-3, gain: float = 50.0) -> np.ndarray:
    """N(0, sigma^2) with a fraction ``frac`` of entries multiplied by ``gain``."""
    rng = np.random.Generator(np.random.PCG64(seed))

    def fn(r0, r1):
        x = rng.standard_normal((r1 - r0, K), dtype=np.float32) * np.float32(sigma)
        hit = rng.random((r1 - r0, K), dtype=np.float32) < frac
        x[hit] *= np.float32(gain)
        return x

    return _rows_chunked(N, K, fn)


def rowscale_weights(N: int, K: int, seed: int, sigma: float = 0.02, lo: float = 1e-3, hi: float = 1.0) -> np.ndarray:
    """Every row has its own scale, log-uniform in [lo, hi]: spreads the exponents over
    about ten binades, so roughly a third of the elements miss the 7-exponent window."""
    rng = np.random.Generator(np.random.PCG64(seed))
    scales = np.exp(rng.uniform(np.log(lo), np.log(hi), N)).astype(np.float32)
    return _rows_chunked(N, K, lambda r0, r1: rng.standard_normal((r1 - r0, K), dtype=np.float32)
                         * np.float32(sigma) * scales[r0:r1, None])


def special_weights(N: int, K: int, seed: int, sigma: float = 0.02, per_pattern: int = 64,
                    finite_only: bool = False) -> np.ndarray:
    """N(0, sigma^2) with injected +-0, subnormals, +-Inf and NaNs (>= ``per_pattern`` of
    each bit pattern at seeded positions), one whole 8x8 tile of each class, and one
    64x64 block made entirely of out-of-window values.  ``finite_only`` leaves Inf/NaN
    out so that a numeric GEMM check is meaningful."""
    W = gaussian_weights(N, K, seed, sigma)
    rng = np.random.Generator(np.random.PCG64(seed + 7))
    classes = [c for c in SPECIAL_PATTERNS if not (finite_only and c in ("inf", "nan"))]
    for c in classes:
        for pat in SPECIAL_PATTERNS[c]:
            idx = rng.integers(0, N * K, per_pattern)
            W.reshape(-1)[idx] = pat
    # one aligned 8x8 tile per class
    for i, c in enumerate(classes):
        pats = SPECIAL_PATTERNS[c]
        n0 = 8 * int(rng.integers(0, N // 8))
        k0 = 8 * int(rng.integers(0, K // 8))
        W[n0:n0 + 8, k0:k0 + 8] = np.array(pats, dtype=np.uint16)[np.arange(64).reshape(8, 8) % len(pats)]
    # one aligned 64x64 block with exponents far outside any plausible window
    n0 = 64 * int(rng.integers(0, N // 64))
    k0 = 64 * int(rng.integers(0, K // 64))
    big = rng.standard_normal((64, 64), dtype=np.float32) * np.float32(3.0e4)
    W[n0:n0 + 64, k0:k0 + 64] = f32_to_bf16(big)
    return W


def activations(M: int, K: int, seed: int) -> np.ndarray:
    """BF16 N(0, 1) activations [M, K]."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return f32_to_bf16(rng.standard_normal((M, K), dtype=np.float32))


WEIGHT_KINDS = {
    "gauss": gaussian_weights,
    "student_t": student_t_weights,
    "outliers": outlier_weights,
    "rowscale": rowscale_weights,
    "specials": special_weights,
}


def make_weights(kind: str, N: int, K: int, seed: int, **kw) -> np.ndarray:
    return WEIGHT_KINDS[kind](N, K, seed, **kw)
