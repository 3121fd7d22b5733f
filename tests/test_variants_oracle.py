"""Pins for the format-variant oracle (codeword lengths 2 / 3 / 4, windows per matrix /
BlockTile / BlockTile row, dense H): each check binds it to something other than itself."""
import itertools

import numpy as np
import pytest

import oracle
from oracle import variants as ov
from paper_2603_17435_amd import inputs
from util import read_golden, storage_order_view

ALL = list(itertools.product((2, 3, 4), ov.BASES, (False, True)))  # (n, base, dense_h)


@pytest.mark.parametrize("n,base,dense_h", ALL)
def test_roundtrip_all_65536_patterns(n, base, dense_h):
    """Lossless for every BF16 bit pattern, in sorted order (windows differ per BlockTile) and
    shuffled (every BlockTile sees every exponent)."""
    W = np.arange(65536, dtype=np.uint16).reshape(256, 256)
    for X in (W, np.random.default_rng(7).permutation(W.reshape(-1)).reshape(256, 256)):
        enc = ov.encode(X, n, base, dense_h)
        assert np.array_equal(ov.decode(enc), X)
        assert enc.n_high + enc.n_fallback == X.size


def test_three_planes_per_matrix_is_the_paper_format():
    """n = 3 with one window per matrix and sparse H is Section 4.2's format: array for array
    what the C oracle (a separate implementation) produces."""
    for kind, seed in (("gauss", 3), ("rowscale", 4), ("specials", 5)):
        W = inputs.make_weights(kind, 128, 192, seed)
        a, b = oracle.encode(W), ov.encode(W, 3, "matrix", False)
        assert (b.win_lo == a.window_start).all()
        assert np.array_equal(a.planes, b.planes)
        assert np.array_equal(a.H, b.H) and np.array_equal(a.L, b.L)
        assert np.array_equal(a.offH, b.offH) and np.array_equal(a.offL, b.offL)
        assert (a.n_high, a.n_fallback) == (b.n_high, b.n_fallback)


@pytest.mark.parametrize("n", (2, 3, 4))
def test_element_order_and_codewords_against_reshapes(n):
    """The documented nesting, written with numpy reshapes only, fixes where every H byte and
    every plane bit sits."""
    W = inputs.gaussian_weights(128, 128, 9)
    view = storage_order_view(W)                      # [bt, tt, ft, p]
    rows = storage_order_view(np.tile(np.arange(128, dtype=np.uint16)[:, None] % 64, (1, 128)))  # BlockTile row of every element
    for base, dense_h in (("matrix", False), ("tile", True), ("row", False)):
        enc = ov.encode(W, n, base, dense_h)
        for bt in range(4):
            elems = view[bt].reshape(-1).astype(np.int64)
            lo = enc.win_lo[bt].astype(np.int64)[rows[bt].reshape(-1)]
            d = ((elems >> 7) & 0xFF) - lo
            inside = (d >= 0) & (d < (1 << n) - 1)
            hb = ((elems >> 8) & 0x80) | (elems & 0x7F)
            h0 = int(enc.offH[bt]) * 16
            if dense_h:
                assert np.array_equal(enc.H[h0:h0 + 4096], np.where(inside, hb, 0))
            else:
                assert np.array_equal(enc.H[h0:h0 + inside.sum()], hb[inside])
            l0 = int(enc.offL[bt]) * 8
            assert np.array_equal(enc.L[l0:l0 + (~inside).sum()], elems[~inside])
            code = np.where(inside, d + 1, 0).reshape(64, 64)          # [fragtile, p]
            for i in range(n):
                bits = ((code >> i) & 1).astype(np.uint64)
                words = (bits << np.arange(64, dtype=np.uint64)[None, :]).sum(axis=1, dtype=np.uint64)
                assert np.array_equal(enc.planes[bt * 64:(bt + 1) * 64, i], words)


@pytest.mark.parametrize("n", (2, 3, 4))
def test_window_is_the_best_run_and_payload_follows_average_bits(n):
    """Coverage = the best sliding-window sum of the histogram (numpy's convolution, first
    maximum); payload bits = AverageBits(n) at that coverage, times the element count."""
    for kind, seed in (("gauss", 1), ("student_t", 2), ("rowscale", 3)):
        W = inputs.make_weights(kind, 128, 256, seed)
        hist = np.bincount(((W >> 7) & 0xFF).ravel(), minlength=256)
        sums = np.convolve(hist, np.ones((1 << n) - 1, dtype=np.int64), mode="valid")
        enc = ov.encode(W, n, "matrix", False)
        assert (enc.win_lo == int(np.argmax(sums))).all() and enc.n_high == int(sums.max())
        r = enc.n_high / W.size
        assert abs(enc.payload_bits - ov.average_bits(n, r) * W.size) < 1e-6 * W.size
        dense = ov.encode(W, n, "matrix", True)
        assert dense.payload_bits == enc.payload_bits + 8 * enc.n_fallback
        assert dense.H.size == W.size and np.array_equal(dense.L, enc.L)


def test_average_bits_against_the_paper():
    """Section 4.2: 11.3 bits at r3 = 0.96; the 2-bit and 4-bit figures (12.4, 12.1) imply
    coverages through the same formula, which must be proportions and must grow with n."""
    g = read_golden("paper_numbers.txt")
    assert abs(ov.average_bits(3, float(g["average_bits3_r"])) - float(g["average_bits3"])) < 0.05
    r2 = (2 + 16 - float(g["average_bits2"])) / 8
    r3 = (3 + 16 - float(g["average_bits3"])) / 8
    r4 = (4 + 16 - float(g["average_bits4"])) / 8
    assert 0 < r2 < r3 < r4 < 1
    for n, r in ((2, r2), (3, r3), (4, r4)):
        assert abs(ov.average_bits(n, r) - float(g[f"average_bits{n}"])) < 1e-9
    # limits: everything covered costs n + 8 bits, nothing covered n + 16
    assert ov.average_bits(3, 1.0) == 11 and ov.average_bits(3, 0.0) == 19


def test_gaussian_coverage_follows_the_erf_law_and_three_bits_win():
    """Appendix A summed over the window, against samples; and with those coverages the
    3-bit codeword is the cheapest of the three (Section 4.2's conclusion)."""
    W = inputs.gaussian_weights(1024, 1024, 12, 0.02)
    cost = {}
    for n in (2, 3, 4):
        s, r_theory = ov.gaussian_window_coverage(0.02, n)
        enc_start, cov = ov.select_window(np.bincount(((W >> 7) & 0xFF).ravel(), minlength=256), n)
        assert enc_start == s
        assert abs(cov / W.size - r_theory) < 3e-3          # sampling + BF16 rounding
        cost[n] = ov.average_bits(n, r_theory)
    assert abs(ov.gaussian_window_coverage(0.02, 3)[1] - 0.97874) < 2e-5
    assert cost[3] < cost[4] < cost[2]
    assert abs(cost[3] - 11.17) < 0.01


def test_finer_windows_cover_at_least_as_much():
    """A window chosen for a part is optimal for that part, so per BlockTile it never covers
    fewer of the tile's elements than the matrix-wide window, and per row never fewer than per
    tile; on row-scaled weights only the per-row windows recover the Gaussian coverage."""
    def fallbacks_per_tile(enc):  # zero codewords, counted from the planes
        any_plane = np.bitwise_or.reduce(enc.planes, axis=1).reshape(-1, 64)
        return 4096 - np.array([[bin(int(x)).count("1") for x in row] for row in any_plane]).sum(axis=1)

    for kind, seed in (("gauss", 21), ("rowscale", 22)):
        W = inputs.make_weights(kind, 256, 128, seed)
        for n in (2, 3, 4):
            fb = [fallbacks_per_tile(ov.encode(W, n, base, False)) for base in ov.BASES]
            assert (fb[1] <= fb[0]).all() and (fb[2] <= fb[1]).all()
            assert fb[0].sum() == ov.encode(W, n, "matrix", False).n_fallback
    W = inputs.make_weights("rowscale", 256, 128, 22)
    r = {base: ov.encode(W, 3, base, False).n_high / W.size for base in ov.BASES}
    assert r["matrix"] < 0.8 and r["tile"] < 0.8 and r["row"] > 0.97


def test_select_window_brute_force():
    rng = np.random.default_rng(3)
    for _ in range(20):
        hist = rng.integers(0, 50, 256)
        for n in (2, 3, 4):
            w = (1 << n) - 1
            best = max(range(256 - w + 1), key=lambda s: (hist[s:s + w].sum(), -s))
            assert ov.select_window(hist, n) == (best, int(hist[best:best + w].sum()))
