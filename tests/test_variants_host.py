"""Host packer of the format variants against the variant oracle, array for array (CPU)."""
import itertools

import numpy as np
import pytest

from oracle import variants as ov
from paper_2603_17435_amd import binding, inputs

MODES = {"matrix": binding.ZS_BASE_MATRIX, "tile": binding.ZS_BASE_TILE, "row": binding.ZS_BASE_ROW}
ALL = list(itertools.product((2, 3, 4), ov.BASES, (0, 1)))


def sections(blob, d):
    n_bt = (d.N // 64) * (d.K // 64)
    planes = blob[d.off_planes:d.off_planes + n_bt * 64 * 8 * d.n_planes].view(np.uint64).reshape(n_bt * 64, d.n_planes)
    offs = blob[d.off_offsets:d.off_offsets + (n_bt + 1) * 8].view(np.uint32).reshape(n_bt + 1, 2)
    per_bt = 64 if d.base_mode == binding.ZS_BASE_ROW else 1
    bases = blob[d.off_bases:d.off_bases + n_bt * per_bt].reshape(n_bt, per_bt)
    H = blob[d.off_H:d.off_H + d.h_bytes]
    L = blob[d.off_L:d.off_L + d.l_bytes].view(np.uint16)
    return planes, offs, bases, H, L


@pytest.mark.parametrize("n,base,dense", ALL)
def test_variant_packer_equals_oracle(n, base, dense):
    for kind, shape, seed in (("gauss", (128, 192), 1), ("rowscale", (64, 256), 2), ("specials", (128, 64), 3)):
        W = inputs.make_weights(kind, *shape, seed)
        enc = ov.encode(W, n, base, bool(dense))
        blob, d = binding.zs_variant_encode(W, n, MODES[base], dense, threads=3)
        assert binding.zs_variant_validate(d) == 0 and d.total_bytes == blob.size
        planes, offs, bases, H, L = sections(blob, d)
        assert np.array_equal(planes, enc.planes)
        assert np.array_equal(offs[:, 0], enc.offH) and np.array_equal(offs[:, 1], enc.offL)
        assert np.array_equal(np.broadcast_to(bases, enc.win_lo.shape), enc.win_lo)
        assert np.array_equal(H, enc.H) and np.array_equal(L, enc.L)
        assert (d.n_high, d.n_fallback) == (enc.n_high, enc.n_fallback)


def test_three_planes_per_matrix_holds_the_main_format_sections():
    W = inputs.gaussian_weights(192, 128, 5)
    blob, d = binding.zs_encode(W)
    vblob, vd = binding.zs_variant_encode(W, 3, binding.ZS_BASE_MATRIX, 0)
    n_bt = 6
    assert np.array_equal(blob[d.off_bitmaps:d.off_bitmaps + n_bt * 1536], vblob[vd.off_planes:vd.off_planes + n_bt * 1536])
    assert np.array_equal(blob[d.off_offsets:d.off_offsets + (n_bt + 1) * 8], vblob[vd.off_offsets:vd.off_offsets + (n_bt + 1) * 8])
    assert np.array_equal(blob[d.off_H:d.off_H + d.h_bytes], vblob[vd.off_H:vd.off_H + vd.h_bytes])
    assert np.array_equal(blob[d.off_L:d.off_L + d.l_bytes], vblob[vd.off_L:vd.off_L + vd.l_bytes])
    assert (vblob[vd.off_bases:vd.off_bases + n_bt] == d.base_exp + 1).all()


def test_variant_packer_threads_stride_and_errors():
    W = inputs.make_weights("student_t", 128, 128, 9)
    ref, d0 = binding.zs_variant_encode(W, 4, binding.ZS_BASE_ROW, 1, threads=1)
    for t in (2, 5):
        b, d = binding.zs_variant_encode(W, 4, binding.ZS_BASE_ROW, 1, threads=t)
        assert np.array_equal(b, ref)
    padded = np.zeros((128, 160), dtype=np.uint16)
    padded[:, :128] = W
    b, _ = binding.zs_variant_encode(padded[:, :128], 4, binding.ZS_BASE_ROW, 1)
    assert np.array_equal(b, ref)
    assert binding.zs_variant_bound(128, 128, 5, 0, 0) == 0 and binding.zs_variant_bound(128, 128, 3, 3, 0) == 0
    assert binding.zs_variant_bound(100, 128, 3, 0, 0) == 0
    with pytest.raises(binding.ZsError):
        binding.zs_variant_encode(W[:100], 3, 0, 0)
    bad = binding.ZsVariantDesc.from_buffer_copy(d0)
    bad.n_planes = 7
    assert binding.zs_variant_validate(bad) == -6
    bad = binding.ZsVariantDesc.from_buffer_copy(d0)
    bad.off_L = bad.off_H
    assert binding.zs_variant_validate(bad) == -4


def test_variant_sizes_follow_average_bits():
    """Blob size = elements x AverageBits(n) / 8 at the measured coverage, plus the documented
    overheads (8 bytes of offsets and the window bytes per BlockTile, padding below 31 bytes per
    BlockTile, section alignment)."""
    W = inputs.gaussian_weights(256, 256, 4)
    n_bt = 16
    for n, base, dense in ALL:
        blob, d = binding.zs_variant_encode(W, n, MODES[base], dense)
        r = d.n_high / W.size
        payload = ov.average_bits(n, r) * W.size / 8 + (d.n_fallback if dense else 0)
        overhead = blob.size - payload
        fixed = 8 * (n_bt + 1) + n_bt * (64 if base == "row" else 1)
        assert fixed <= overhead <= fixed + 31 * n_bt + 5 * 256
