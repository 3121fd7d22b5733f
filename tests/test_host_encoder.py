"""CPU-side checks of the product: the C ABI loads and exports what include/zipserv.h
declares, and the host packer writes byte for byte what the oracle's encoder defines."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
from paper_2603_17435_amd import binding, inputs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def sections(blob, d):
    n_bt = (d.N // 64) * (d.K // 64)
    planes = blob[d.off_bitmaps:d.off_bitmaps + n_bt * 1536].view(np.uint64).reshape(-1, 3)
    offs = blob[d.off_offsets:d.off_offsets + (n_bt + 1) * 8].view(np.uint32).reshape(-1, 2)
    H = blob[d.off_H:d.off_H + d.h_bytes]
    L = blob[d.off_L:d.off_L + d.l_bytes].view(np.uint16)
    return planes, offs, H, L


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "zipserv.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(zs_[a-z_0-9]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    L = binding.lib()
    for name in declared:
        assert getattr(L, name) is not None
    assert L.zs_version() >= 1
    assert ctypes.sizeof(binding.ZsDesc) == 112


@pytest.mark.parametrize("kind,N,K", [("gauss", 128, 256), ("rowscale", 192, 128), ("specials", 256, 256),
                                       ("student_t", 64, 64), ("outliers", 128, 128)])
def test_blob_equals_oracle_encoding(kind, N, K):
    W = inputs.make_weights(kind, N, K, seed=31)
    enc = oracle.encode(W)
    for threads in (1, 5):
        blob, d = binding.zs_encode(W, threads=threads)
        assert binding.zs_desc_validate(d) == 0
        assert (d.N, d.K, d.base_exp, d.n_high, d.n_fallback) == (N, K, enc.base_exp, enc.n_high, enc.n_fallback)
        planes, offs, H, L = sections(blob, d)
        assert np.array_equal(planes, enc.planes)
        assert np.array_equal(offs[:, 0], enc.offH) and np.array_equal(offs[:, 1], enc.offL)
        assert np.array_equal(H, enc.H) and np.array_equal(L, enc.L)
        assert d.total_bytes == blob.size and blob.ctypes.data % 256 == 0
        assert d.max_h_units == np.diff(enc.offH.astype(np.int64)).max()
        assert d.max_l_units == np.diff(enc.offL.astype(np.int64)).max()
        # the oracle's decoder reads the product's blob back to the original bits
        enc2 = oracle.Encoded(N, K, d.base_exp, d.base_exp + 1, np.ascontiguousarray(planes), np.ascontiguousarray(H),
                              np.ascontiguousarray(L), np.ascontiguousarray(offs[:, 0]), np.ascontiguousarray(offs[:, 1]),
                              d.n_high, d.n_fallback)
        assert np.array_equal(oracle.decode(enc2), W)


def test_all_bit_patterns_blob():
    W = np.random.default_rng(1).permutation(np.arange(65536, dtype=np.uint16)).reshape(256, 256)
    blob, d = binding.zs_encode(W)
    enc = oracle.encode(W)
    planes, offs, H, L = sections(blob, d)
    assert np.array_equal(planes, enc.planes) and np.array_equal(H, enc.H) and np.array_equal(L, enc.L)


def test_strided_input_and_errors():
    big = inputs.gaussian_weights(128, 256, 5)
    view = big[:, :128]                                   # ldw = 256 > K = 128
    blob, d = binding.zs_encode(view)
    blob2, d2 = binding.zs_encode(np.ascontiguousarray(view))
    assert np.array_equal(blob, blob2)
    L = binding.lib()
    assert L.zs_encode_bound(100, 64) == 0 and L.zs_encode_bound(64, 0) == 0
    desc = binding.ZsDesc()
    W = np.zeros((64, 64), dtype=np.uint16)
    buf = binding.aligned_empty(64)
    assert L.zs_encode(W.ctypes.data, 64, 64, 64, buf.ctypes.data, 64, ctypes.byref(desc), 1) == -3   # ZS_ERR_SIZE
    assert L.zs_encode(W.ctypes.data, 60, 64, 64, buf.ctypes.data, 64, ctypes.byref(desc), 1) == -2   # ZS_ERR_SHAPE
    assert L.zs_encode(None, 64, 64, 64, buf.ctypes.data, 64, ctypes.byref(desc), 1) == -1            # ZS_ERR_ARG
    bad = binding.ZsDesc()
    assert binding.zs_desc_validate(bad) == -4
    d.n_high += 1
    assert binding.zs_desc_validate(d) == -4
    assert L.zs_strerror(-2).decode().startswith("unsupported shape")


def test_config_table():
    cfgs = binding.zs_gemm_configs()
    assert len(cfgs) == binding.lib().zs_gemm_num_configs() >= 3
    assert binding.lib().zs_gemm_config_name(0) is None
    _, d = binding.zs_encode(np.zeros((64, 64), dtype=np.uint16))
    assert binding.zs_gemm_pick_config(d, 1) in cfgs and binding.zs_gemm_pick_config(d, 32) in cfgs


def test_stage_aware_dispatch_rule():
    """Section 4.4's dispatch as zs_linear_path answers it (host logic; 256 compute units assumed
    without a device): fused kernels for few tokens, the decoupled pipeline beyond a crossover
    that comes earlier on layers with few BlockTiles per compute unit."""
    assert binding.lib().zs_compute_units() >= 1
    _, small = binding.zs_encode(np.zeros((4096, 4096), dtype=np.uint16))      # 16 BlockTiles per unit
    _, large = binding.zs_encode(np.zeros((4096, 14336), dtype=np.uint16))     # 56
    F, D = binding.ZS_PATH_FUSED, binding.ZS_PATH_DECOUPLED
    assert [binding.zs_linear_path(small, M) for M in (1, 32, 127, 128, 4096)] == [F, F, F, D, D]
    assert [binding.zs_linear_path(large, M) for M in (1, 128, 256, 257, 4096)] == [F, F, F, D, D]
    assert binding.zs_linear_path(small, 0) == -1
    assert binding.zs_linear_workspace(small, 16) == binding.zs_gemm_workspace(small, 16)
    assert binding.zs_linear_workspace(small, 512) == 4096 * 4096 * 2 + binding.ZS_DENSE_WORKSPACE_BYTES
