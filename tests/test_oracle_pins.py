"""Pins for the CPU oracle: every check binds the oracle to something other than itself
(a value the paper prints, a closed form, an invariant, a library routine, brute force)."""
import math

import numpy as np
import pytest

import oracle
from paper_2603_17435_amd import inputs
from util import read_golden, storage_order_view


def bf16_fields(W):
    return (W >> 15) & 1, (W >> 7) & 0xFF, W & 0x7F


# --------------------------------------------------------------------------- losslessness
def test_roundtrip_all_65536_patterns():
    """Section 1 / 4: 'bit-exact'.  Every BF16 bit pattern, +-0, subnormals, Inf, NaN payloads."""
    W = np.arange(65536, dtype=np.uint16).reshape(256, 256)
    for perm_seed in (None, 3):
        X = W.copy()
        if perm_seed is not None:
            X = np.random.default_rng(perm_seed).permutation(X.reshape(-1)).reshape(256, 256)
        enc = oracle.encode(X)
        assert np.array_equal(oracle.decode(enc), X)
        assert np.array_equal(oracle.decode_walk(enc), X)
        assert enc.n_high + enc.n_fallback == X.size


@pytest.mark.parametrize("kind", ["all_high", "all_fallback", "alternating", "fb_first", "fb_last"])
def test_roundtrip_degenerate_tiles(kind):
    rng = np.random.default_rng(11)
    # background pins the window at exponents 120..126
    W = (rng.integers(120, 127, (64, 128)).astype(np.uint16) << 7) | rng.integers(0, 128, (64, 128)).astype(np.uint16)
    W |= (rng.integers(0, 2, W.shape).astype(np.uint16) << 15)
    out_of_window = np.uint16((40 << 7) | 0x55)
    tile = W[8:16, 32:40]
    if kind == "all_fallback":
        tile[:] = out_of_window
    elif kind == "alternating":
        tile[:, ::2] = out_of_window
    elif kind == "fb_first":
        tile[0, 0] = out_of_window
    elif kind == "fb_last":
        tile[7, 7] = out_of_window
    enc = oracle.encode(W)
    assert enc.window_start == 120 and enc.base_exp == 119
    assert np.array_equal(oracle.decode(enc), W)
    assert np.array_equal(oracle.decode_walk(enc), W)
    expected_fb = {"all_high": 0, "all_fallback": 64, "alternating": 32, "fb_first": 1, "fb_last": 1}[kind]
    assert enc.n_fallback == expected_fb


def test_popcount_decoder_equals_walk_decoder_bruteforce():
    """Random 64x64 blocks with a wide exponent spread (many fallbacks)."""
    rng = np.random.default_rng(5)
    for trial in range(20):
        W = rng.integers(0, 65536, (64, 64)).astype(np.uint16)
        if trial % 2:
            e = rng.integers(110, 122, (64, 64)).astype(np.uint16)
            W = (W & 0x807F) | (e << 7)
        enc = oracle.encode(W)
        a, b = oracle.decode(enc), oracle.decode_walk(enc)
        assert np.array_equal(a, W) and np.array_equal(b, W)


# --------------------------------------------------------------------------- worked example
def test_paper_worked_example():
    g = read_golden("worked_example.txt")
    bit_hi, bit_fb = int(g["bit_high"]), int(g["bit_fallback"])
    assert bit_hi == 2 * int(g["thread_high"]) and bit_fb == 2 * int(g["thread_fallback"])
    base, code, expo = int(g["base_exp"]), int(g["code"]), int(g["exponent"])
    assert int(g["code_bits"], 2) == code and base + code == expo

    # index arithmetic on an arbitrary indicator that satisfies the two printed facts
    rng = np.random.default_rng(38)
    for _ in range(50):
        M = int(rng.integers(0, 2**63)) | (1 << bit_hi)
        M &= ~(1 << bit_fb)
        ones_below = bin(M & ((1 << bit_hi) - 1)).count("1")          # ones in bits [0, 37]
        zeros_below = bit_fb - bin(M & ((1 << bit_fb) - 1)).count("1")  # zeros in bits [0, 11]
        assert oracle.tile_index(M, bit_hi) == (True, ones_below)
        assert oracle.tile_index(M, bit_fb) == (False, zeros_below)

    # a real tile: window 116..122 (base 115); element 38 has exponent 120, element 12 is out of window
    W = (rng.integers(116, 123, (64, 64)).astype(np.uint16) << 7) | rng.integers(0, 128, (64, 64)).astype(np.uint16)
    r_hi, c_hi = divmod(bit_hi, 8)
    r_fb, c_fb = divmod(bit_fb, 8)
    W[r_hi, c_hi] = (1 << 15) | (expo << 7) | 0x2A
    W[r_fb, c_fb] = (90 << 7) | 0x11
    enc = oracle.encode(W)
    assert enc.base_exp == base
    b1, b2, b3 = (int(x) for x in enc.planes[0])        # FragTile 0 = rows 0..7, cols 0..7
    assert ((b3 >> bit_hi) & 1, (b2 >> bit_hi) & 1, (b1 >> bit_hi) & 1) == (1, 0, 1)
    assert ((b1 | b2 | b3) >> bit_fb) & 1 == 0
    M = b1 | b2 | b3
    is_high, idx = oracle.tile_index(M, bit_hi)
    assert is_high and enc.H[idx] == 0x80 | 0x2A           # sign << 7 | mantissa
    is_high, idx = oracle.tile_index(M, bit_fb)
    assert (not is_high) and enc.L[idx] == W[r_fb, c_fb]
    assert np.array_equal(oracle.decode(enc), W)


# --------------------------------------------------------------------------- window selection
def test_window_selection_bruteforce_and_ties():
    rng = np.random.default_rng(2)
    for trial in range(200):
        hist = np.zeros(256, dtype=np.uint64)
        if trial % 3 == 0:
            hist[:] = rng.integers(0, 5, 256)                 # many ties
        elif trial % 3 == 1:
            c = rng.integers(0, 256)
            for e in range(256):
                hist[e] = int(1000 * math.exp(-0.5 * ((e - c) / 2.0) ** 2))
        else:
            hist[rng.integers(0, 256, 10)] = rng.integers(1, 1000, 10)
        sums = np.array([int(hist[s:s + 7].sum()) for s in range(250)])
        s_ref = int(np.argmax(sums))                           # first maximum
        s, cov = oracle.select_window(hist)
        assert (s, cov) == (s_ref, int(sums[s_ref]))


def test_window_edges():
    hist = np.zeros(256, dtype=np.uint64)
    hist[0] = 10                                               # zeros / subnormals only
    assert oracle.select_window(hist)[0] == 0
    W = np.zeros((64, 64), dtype=np.uint16)
    W[::2] = 0x8000
    enc = oracle.encode(W)
    assert enc.base_exp == -1 and enc.n_fallback == 0
    assert np.array_equal(oracle.decode(enc), W)
    hist[:] = 0
    hist[255] = 7
    s, cov = oracle.select_window(hist)
    assert s == 249 and cov == 7
    W = np.full((64, 64), 0x7F80, dtype=np.uint16)             # +Inf everywhere
    enc = oracle.encode(W)
    assert enc.base_exp == 248 and enc.n_fallback == 0 and np.array_equal(oracle.decode(enc), W)


def test_window_equals_top7_when_contiguous():
    """Section 3.1 / Appendix A, theorem 2: for a unimodal histogram the seven most
    frequent exponents are contiguous and are exactly the best window."""
    for seed, sigma in ((0, 0.02), (1, 0.015), (2, 0.3)):
        W = inputs.gaussian_weights(256, 1024, seed, sigma)
        hist = oracle.exponent_histogram(W)
        top7 = np.sort(np.argsort(hist.astype(np.int64))[-7:])
        assert np.array_equal(np.diff(top7), np.ones(6, dtype=top7.dtype))
        assert oracle.select_window(hist)[0] == int(top7[0])


# --------------------------------------------------------------------------- format / layout
def test_histogram_matches_numpy():
    W = np.random.default_rng(9).integers(0, 65536, (128, 192)).astype(np.uint16)
    ref = np.bincount(((W >> 7) & 0xFF).reshape(-1), minlength=256).astype(np.uint64)
    assert np.array_equal(oracle.exponent_histogram(W), ref)


def test_arrays_follow_documented_layout():
    """Planes, H, L and offsets recomputed with numpy from the documented element order."""
    W = inputs.rowscale_weights(128, 192, 77)
    enc = oracle.encode(W)
    s = enc.window_start
    v = storage_order_view(W).astype(np.int64)               # [bt, tt, ft, p]
    sign, expo, mant = bf16_fields(v)
    high = (expo >= s) & (expo <= s + 6)
    code = np.where(high, expo - enc.base_exp, 0)
    assert code.max() <= 7 and (code[high] >= 1).all()
    weights = (np.uint64(1) << np.arange(64, dtype=np.uint64))
    for j in range(3):
        plane = (((code >> j) & 1).astype(np.uint64) * weights).sum(axis=-1, dtype=np.uint64)
        assert np.array_equal(plane.reshape(-1), enc.planes[:, j])
    n_bt = v.shape[0]
    assert enc.offH.shape == (n_bt + 1,) and enc.offH[0] == 0 and enc.offL[0] == 0
    for bt in range(n_bt):
        hb = high[bt].reshape(-1)
        h_ref = ((sign[bt].reshape(-1)[hb] << 7) | mant[bt].reshape(-1)[hb]).astype(np.uint8)
        l_ref = v[bt].reshape(-1)[~hb].astype(np.uint16)
        h0, h1 = 16 * int(enc.offH[bt]), 16 * int(enc.offH[bt + 1])
        l0, l1 = 8 * int(enc.offL[bt]), 8 * int(enc.offL[bt + 1])
        assert h1 - h0 == -(-h_ref.size // 16) * 16 and l1 - l0 == -(-l_ref.size // 8) * 8
        assert np.array_equal(enc.H[h0:h0 + h_ref.size], h_ref) and not enc.H[h0 + h_ref.size:h1].any()
        assert np.array_equal(enc.L[l0:l0 + l_ref.size], l_ref) and not enc.L[l0 + l_ref.size:l1].any()
    assert 16 * int(enc.offH[-1]) == enc.H.size and 8 * int(enc.offL[-1]) == enc.L.size


# --------------------------------------------------------------------------- storage cost
def test_average_bits_closed_form_and_paper_value():
    g = read_golden("paper_numbers.txt")
    r = float(g["average_bits3_r"])
    hist = np.zeros(256, dtype=np.uint64)
    hist[100:107] = [960_000 // 7 + (1 if i < 960_000 % 7 else 0) for i in range(7)]
    hist[200] = 40_000
    assert abs(oracle.average_bits3(hist, 100) - (r * 11 + (1 - r) * 19)) < 1e-9
    assert round(oracle.average_bits3(hist, 100), 1) == float(g["average_bits3"])
    assert abs(16 / (8 + 2.6) - float(g["ideal_cr"])) < 0.005

    for kind, seed in (("gauss", 1), ("student_t", 2), ("rowscale", 3)):
        W = inputs.make_weights(kind, 256, 512, seed)
        enc = oracle.encode(W)
        hist = oracle.exponent_histogram(W)
        r3 = enc.n_high / W.size
        assert abs(oracle.average_bits3(hist, enc.window_start) - (19 - 8 * r3)) < 1e-12
        assert enc.payload_bits == round(W.size * (19 - 8 * r3))
        n_bt = W.size // 4096
        overhead = enc.stored_bytes * 8 - enc.payload_bits
        assert 8 * 8 * (n_bt + 1) <= overhead <= 8 * (8 * (n_bt + 1) + 30 * n_bt)


def test_gaussian_exponent_law():
    """Appendix A: P(E) = erf(2^(x+1)/(sigma sqrt2)) - erf(2^x/(sigma sqrt2))."""
    for sigma, seed in ((0.02, 10), (0.015, 11)):
        pmf = oracle.gaussian_exponent_pmf(sigma)
        assert abs(pmf.sum() - 1.0) < 1e-6
        sums = np.array([pmf[s:s + 7].sum() for s in range(250)])
        s_theory = int(np.argmax(sums))
        W = inputs.gaussian_weights(2048, 2048, seed, sigma)
        hist = oracle.exponent_histogram(W)
        s, cov = oracle.select_window(hist)
        assert s == s_theory == 116
        r = cov / W.size
        assert abs(r - sums[s_theory]) < 2e-3
        emp = hist / W.size
        assert np.abs(emp - pmf).max() < 4e-3                  # BF16 rounding moves a sliver upward
    assert abs(oracle.gaussian_exponent_pmf(0.02)[116:123].sum() - 0.97874) < 2e-5


# --------------------------------------------------------------------------- GEMM
def test_gemm_against_numpy_float64():
    rng = np.random.default_rng(4)
    W = inputs.gaussian_weights(192, 320, 21)
    A = inputs.activations(5, 320, 22)
    C, S = oracle.gemm(A, W)
    Af, Wf = inputs.bf16_to_f32(A).astype(np.float64), inputs.bf16_to_f32(W).astype(np.float64)
    assert np.allclose(C, Af @ Wf.T, rtol=1e-13, atol=1e-15)
    assert np.allclose(S, np.abs(Af) @ np.abs(Wf).T, rtol=1e-13, atol=1e-15)
    rows = rng.integers(0, 192, 17)
    C2, S2 = oracle.gemm(A, W, rows=rows, threads=3)
    assert np.array_equal(C2, C[:, rows]) and np.array_equal(S2, S[:, rows])
    # not symmetric in its operands: a transposed W would fail this
    assert C.shape == (5, 192)


def test_gemm_one_hot_reads_out_weights():
    W = np.random.default_rng(6).integers(0, 0x7F00, (64, 64)).astype(np.uint16)  # finite, positive
    A = np.zeros((64, 64), dtype=np.uint16)
    A[np.arange(64), np.arange(64)] = 0x3F80                                        # 1.0
    C, S = oracle.gemm(A, W)
    assert np.array_equal(C, inputs.bf16_to_f32(W).astype(np.float64).T)
    assert np.array_equal(S, C)


def test_gemm_non_finite_propagation():
    W = inputs.gaussian_weights(64, 64, 1)
    A = inputs.activations(2, 64, 2)
    W[3, 5] = 0x7F80   # +Inf
    W[4, 6] = 0x7FC0   # NaN
    W[5, 0] = 0x7F80
    W[5, 1] = 0xFF80   # +Inf and -Inf in one row
    A[:, 0] = 0x3F80
    A[:, 1] = 0x3F80
    C, _ = oracle.gemm(A, W)
    assert np.isinf(C[:, 3]).all() and np.isnan(C[:, 4]).all() and np.isnan(C[:, 5]).all()
    assert np.isfinite(np.delete(C, [3, 4, 5], axis=1)).all()


def test_compute_intensity_model_reproduces_the_paper():
    """Section 3.3: for a 4096 x 4096 weight the decoupled pipeline loses 62.3 / 62.2 / 62.0 /
    61.7 % of the plain GEMM's compute intensity at batch 8 / 16 / 32 / 64 (CR = 1.51).  The byte
    formulas are the ones bench.py reports against."""
    import bench
    g = read_golden("paper_numbers.txt")
    cr = float(g["ideal_cr"])
    for batch, want in zip(g["ci_batches"], g["ci_degradation_pct"]):
        got = bench.ci_degradation_pct(int(batch), 4096, 4096, cr)
        # one printed decimal, and the paper's own figures follow from its rounded coefficient
        # 2.66 (the exact 1 / CR + 2 is 2.662): together under 0.1 point; a wrong or missing
        # term of the byte model moves the figure by whole points
        assert abs(got - float(want)) < 0.1, (batch, got, want)
    # Section 3.3: the fused design's compute intensity is about 50 % above the plain GEMM's
    M, N, K = 32, 4096, 4096
    gain = bench.dense_gemm_bytes(M, N, K) / bench.fused_bytes(M, N, K, cr) - 1.0
    assert 0.45 < gain < 0.52
