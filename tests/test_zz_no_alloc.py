"""GPU test of zs_gemm_noalloc, the ZipGEMM entry point whose scratch buffer is a device array
inside the library (for callers that cannot allocate).  Its output is compared with zs_gemm's
(caller-provided scratch) on the same inputs to the parity bar |diff| <= 1e-3 * sum|a w| + 1e-6,
and with the CPU oracle, on two calls in a row, the second on a smaller input: the array keeps
what the first call left."""
import numpy as np
import pytest

import oracle
from paper_2603_17435_amd import binding, inputs

pytestmark = pytest.mark.gpu


def run_pair(gu, N, K, M, seed):
    import torch
    W = inputs.gaussian_weights(N, K, seed)
    A = inputs.activations(M, K, seed + 1)
    blob, d = binding.zs_encode(W)
    dev = gu.upload_blob(blob)
    a = torch.from_numpy(A.view(np.int16)).cuda()
    c_new = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    binding.zs_gemm_noalloc(d, dev, a, c_new, M)
    torch.cuda.synchronize()
    c_old = gu.gpu_gemm_resident(d, dev, A)
    C_ref, S = oracle.gemm(A, oracle.decode(oracle.encode(W)), threads=8)
    bound = 1e-3 * S + 1e-6
    got = c_new.cpu().numpy().astype(np.float64)
    assert (np.abs(got - c_old.astype(np.float64)) <= bound).all(), "differs from zs_gemm beyond the parity bar"
    gu.assert_gemm_matches(c_new.cpu().numpy(), C_ref, S)


@pytest.mark.parametrize("M_first,M_second", [(16, 5), (32, 1), (64, 40)])
def test_noalloc_matches_zs_gemm_twice(M_first, M_second):
    import gpu_util as gu
    # 1024 x 1280: 320 BlockTiles over 256 workgroups, so most strips are shared between
    # workgroups and go through the scratch array; the second call is smaller in N, K and M
    run_pair(gu, 1024, 1280, M_first, seed=71)
    run_pair(gu, 384, 704, M_second, seed=73)


def test_noalloc_wider_than_the_scratch_kernel():
    """M > 64 runs the producer / consumer kernel, which needs no scratch: still no allocation."""
    import gpu_util as gu
    run_pair(gu, 256, 512, 100, seed=75)
    run_pair(gu, 128, 256, 3, seed=77)


def test_noalloc_rejects_bad_arguments():
    import torch
    W = inputs.gaussian_weights(64, 64, 1)
    blob, d = binding.zs_encode(W)
    dev = torch.from_numpy(blob).cuda()
    a = torch.zeros((4, 64), dtype=torch.int16, device="cuda")
    c = torch.zeros((4, 64), dtype=torch.float32, device="cuda")
    with pytest.raises(binding.ZsError):
        binding.zs_gemm_noalloc(d, dev, a, c, 0)
    with pytest.raises(binding.ZsError):
        binding.zs_gemm_noalloc(d, dev, None, c, 4)
