"""GPU parity of the format variants: zs_variant_decompress (through the C ABI) against the
variant oracle and the original matrix, bit for bit, for every codeword length, window
granularity and H layout."""
import itertools

import numpy as np
import pytest

from oracle import variants as ov
from paper_2603_17435_amd import binding, inputs

pytestmark = pytest.mark.gpu

MODES = {"matrix": binding.ZS_BASE_MATRIX, "tile": binding.ZS_BASE_TILE, "row": binding.ZS_BASE_ROW}
ALL = list(itertools.product((2, 3, 4), ov.BASES, (0, 1)))


def gpu_variant_decompress(W, n, base, dense, ldw=None):
    import torch
    blob, d = binding.zs_variant_encode(W, n, MODES[base], dense)
    dev = torch.from_numpy(np.ascontiguousarray(blob)).cuda()
    assert dev.data_ptr() % 256 == 0
    ld = d.K if ldw is None else ldw
    out = torch.full((d.N, ld), 0x5A5A, dtype=torch.int16, device="cuda")
    binding.zs_variant_decompress(d, dev, out, ldw=ld)
    torch.cuda.synchronize()
    return out.cpu().numpy().view(np.uint16), d


@pytest.mark.parametrize("n,base,dense", ALL)
def test_variant_decompress_bit_exact(n, base, dense):
    for kind, N, K in (("gauss", 192, 320), ("rowscale", 128, 192), ("specials", 256, 128)):
        W = inputs.make_weights(kind, N, K, seed=inputs.seed_for(3, 1, n))
        out, d = gpu_variant_decompress(W, n, base, dense)
        assert np.array_equal(out, W)
    # against the oracle's decoder on its own arrays (one case per variant keeps the CPU time low)
    W = inputs.make_weights("student_t", 64, 128, seed=11)
    out, _ = gpu_variant_decompress(W, n, base, dense)
    assert np.array_equal(out, ov.decode(ov.encode(W, n, base, bool(dense))))


@pytest.mark.parametrize("n", (2, 3, 4))
def test_variant_decompress_all_bit_patterns_and_row_stride(n):
    sorted_W = np.arange(65536, dtype=np.uint16).reshape(256, 256)
    shuffled = np.random.default_rng(n).permutation(sorted_W.reshape(-1)).reshape(256, 256)
    for W in (sorted_W, shuffled):
        for base, dense in itertools.product(ov.BASES, (0, 1)):
            out, _ = gpu_variant_decompress(W, n, base, dense)
            assert np.array_equal(out, W)
    out, _ = gpu_variant_decompress(shuffled, n, "row", 0, ldw=256 + 24)
    assert np.array_equal(out[:, :256], shuffled)
    assert (out[:, 256:] == 0x5A5A).all()  # nothing written beyond K


def test_variant_decompress_degenerate_and_errors():
    import torch
    zeros = np.zeros((64, 128), dtype=np.uint16)                  # every element in the window at exponent 0
    wide = (np.arange(64 * 128, dtype=np.uint32) % 251 * 257 % 65536).astype(np.uint16).reshape(64, 128)  # mostly fallbacks
    for W in (zeros, wide):
        for n, base, dense in ALL:
            out, _ = gpu_variant_decompress(W, n, base, dense)
            assert np.array_equal(out, W)
    blob, d = binding.zs_variant_encode(zeros, 3, 0, 0)
    dev = torch.from_numpy(np.ascontiguousarray(blob)).cuda()
    out = torch.zeros((64, 128), dtype=torch.int16, device="cuda")
    with pytest.raises(binding.ZsError):
        binding.zs_variant_decompress(d, dev, out, ldw=100)        # ldw < K
    with pytest.raises(binding.ZsError):
        binding.zs_variant_decompress(d, dev[16:], out)            # blob not 256-byte aligned
    bad = binding.ZsVariantDesc.from_buffer_copy(d)
    bad.n_planes = 5
    with pytest.raises(binding.ZsError):
        binding.zs_variant_decompress(bad, dev, out)
    torch.cuda.synchronize()


@pytest.mark.parametrize("n,base,dense", [(2, "matrix", 0), (3, "row", 0), (4, "tile", 1)])
def test_variant_decompress_full_size(n, base, dense):
    """The GateUp shape of the benchmark (28672 x 4096, 7168 workgroups): the whole matrix bit
    for bit.  Lossless decoding has a plain definition -- the matrix itself -- so no oracle pass
    over 117 M elements is needed; the packer it inverts is pinned to the oracle at small sizes."""
    import torch
    W = inputs.make_weights("rowscale" if base == "row" else "gauss", 28672, 4096, seed=inputs.seed_for(1, 2, n))
    blob, d = binding.zs_variant_encode(W, n, MODES[base], dense)
    dev = torch.from_numpy(np.ascontiguousarray(blob)).cuda()
    out = torch.full((d.N, d.K), 0x5A5A, dtype=torch.int16, device="cuda")
    binding.zs_variant_decompress(d, dev, out)
    torch.cuda.synchronize()
    assert torch.equal(out, torch.from_numpy(W.view(np.int16)).cuda())
