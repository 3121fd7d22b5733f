"""Helpers for the GPU parity tests: device buffers via PyTorch, comparison rules."""
import numpy as np
import torch

import oracle
from paper_2603_17435_amd import binding


def upload_blob(blob: np.ndarray) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(blob)).cuda()
    assert t.data_ptr() % 256 == 0
    return t


_SCRATCH = None


def scratch(d, M: int, config: int = 0):
    """One zero-filled scratch buffer shared by every zs_gemm call of the test session: the
    library promises to leave its counters at zero, so a call that did not would break the
    calls after it."""
    global _SCRATCH
    need = binding.zs_gemm_workspace(d, M, config)
    if _SCRATCH is None or _SCRATCH.numel() < need:
        _SCRATCH = torch.zeros(max(need, 1 << 22), dtype=torch.uint8, device="cuda")
    return _SCRATCH, _SCRATCH.numel()


def gpu_decompress(W: np.ndarray) -> np.ndarray:
    blob, d = binding.zs_encode(W)
    dev = upload_blob(blob)
    out = torch.empty((d.N, d.K), dtype=torch.int16, device="cuda")
    out.fill_(0x5A5A)
    binding.zs_decompress(d, dev, out)
    torch.cuda.synchronize()
    return out.cpu().numpy().view(np.uint16)


def gpu_gemm(W: np.ndarray, A: np.ndarray, config: int = 0, encoded=None) -> np.ndarray:
    blob, d = encoded if encoded is not None else binding.zs_encode(W)
    dev = upload_blob(blob)
    M = A.shape[0]
    a = torch.from_numpy(A.view(np.int16)).cuda()
    c = torch.full((M, d.N), float("nan"), dtype=torch.float32, device="cuda")
    ws, ws_bytes = scratch(d, M, config)
    binding.zs_gemm(d, dev, a, c, M, workspace_dev=ws, workspace_bytes=ws_bytes, config=config)
    torch.cuda.synchronize()
    return c.cpu().numpy()


def gpu_gemm_resident(d, dev: torch.Tensor, A: np.ndarray, config: int = 0) -> np.ndarray:
    """zs_gemm on a blob that is already on the device (one upload, several M)."""
    M = A.shape[0]
    a = torch.from_numpy(A.view(np.int16)).cuda()
    c = torch.full((M, d.N), float("nan"), dtype=torch.float32, device="cuda")
    ws, ws_bytes = scratch(d, M, config)
    binding.zs_gemm(d, dev, a, c, M, workspace_dev=ws, workspace_bytes=ws_bytes, config=config)
    torch.cuda.synchronize()
    return c.cpu().numpy()


def assert_gemm_matches(C_gpu: np.ndarray, C_ref: np.ndarray, S: np.ndarray):
    """|C_gpu - C_ref| <= 1e-3 * sum_k |a_k w_k| + 1e-6 per element where the reference is
    finite; where it is not, the classes must agree (NaN <-> NaN, +-Inf same sign)."""
    finite = np.isfinite(C_ref) & np.isfinite(S)
    diff = np.abs(C_gpu.astype(np.float64) - C_ref)
    bound = 1e-3 * S + 1e-6
    bad = finite & ~(diff <= bound)
    assert not bad.any(), (f"{bad.sum()} elements out of tolerance; worst ratio "
                           f"{np.nanmax(np.where(finite, diff / bound, 0)):.3g} at {np.argwhere(bad)[:4].tolist()}")
    nan_ref = np.isnan(C_ref) | (np.isnan(S) & ~np.isinf(C_ref))
    assert np.isnan(C_gpu[nan_ref]).all()
    inf_ref = np.isinf(C_ref)
    assert np.array_equal(C_gpu[inf_ref], C_ref[inf_ref].astype(np.float32))


def check_gemm(W, A, config=0, rows=None, threads=8):
    C_gpu = gpu_gemm(W, A, config)
    W_dec = oracle.decode(oracle.encode(W))          # the oracle GEMM consumes oracle-decoded weights
    assert np.array_equal(W_dec, W)
    C_ref, S = oracle.gemm(A, W_dec, rows=rows, threads=threads)
    if rows is not None:
        C_gpu = C_gpu[:, rows]
    assert_gemm_matches(C_gpu, C_ref, S)
    return C_gpu
