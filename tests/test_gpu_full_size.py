"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration
bench.py times (zs_gemm's automatic choice).  Per matrix: the decoded weights are compared
bit for bit over the whole matrix; the GEMM is compared with the oracle on every output
element for M <= 8 and, beyond, on sampled output features (every strip position class: first,
last, random) and sampled tokens that include the edges of the 64-token panels.  Inputs are
the seeded synthetic generators."""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_17435_amd import binding, inputs

pytestmark = pytest.mark.gpu

LLAMA3_8B = [("qkv", 6144, 4096), ("o", 4096, 4096), ("gate_up", 28672, 4096), ("down", 4096, 14336)]
LLAMA3_70B = [("qkv", 10240, 8192), ("o", 8192, 8192), ("gate_up", 57344, 8192), ("down", 8192, 28672)]
# the seven projections of one LLaMA-3-8B layer (grouped-query attention: 8 KV heads of 128)
LLAMA3_8B_PROJ = [("q", 4096, 4096), ("k", 1024, 4096), ("v", 1024, 4096), ("o", 4096, 4096),
                  ("gate", 14336, 4096), ("up", 14336, 4096), ("down", 4096, 14336)]


@pytest.fixture(scope="module")
def gu():
    import gpu_util
    return gpu_util


def sample_rows(N: int, seed: int, n: int = 96) -> np.ndarray:
    rng = np.random.default_rng(seed)
    fixed = np.array([0, 1, 63, 64, N - 65, N - 64, N - 1])
    return np.unique(np.concatenate([fixed, rng.choice(N, n, replace=False)]))


def sample_tokens(M: int, seed: int, n: int = 24) -> np.ndarray:
    if M <= 128:
        return np.arange(M)
    rng = np.random.default_rng(seed)
    fixed = np.array([0, 15, 16, 63, 64, 65, M - 65, M - 64, M - 1])
    return np.unique(np.concatenate([fixed, rng.choice(M, n, replace=False)]))


def run_matrix(gu, W: np.ndarray, Ms, seed: int):
    N, K = W.shape
    W_dec = oracle.decode(oracle.encode(W))  # the oracle GEMM consumes oracle-decoded weights
    assert np.array_equal(W_dec, W)
    blob, d = binding.zs_encode(W)
    dev = gu.upload_blob(blob)
    out = torch.full((N, K), 0x5A5A, dtype=torch.int16, device="cuda")
    binding.zs_decompress(d, dev, out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy().view(np.uint16), W_dec)
    del out
    rows = sample_rows(N, seed)
    for M in Ms:
        A = inputs.activations(M, K, seed + M)
        C = gu.gpu_gemm_resident(d, dev, A)
        if M <= 8:  # every output element
            C_ref, S = oracle.gemm(A, W_dec, threads=8)
            gu.assert_gemm_matches(C, C_ref, S)
            continue
        tok = sample_tokens(M, seed + 7 * M)
        C_ref, S = oracle.gemm(np.ascontiguousarray(A[tok]), W_dec, rows=rows, threads=8)
        gu.assert_gemm_matches(C[np.ix_(tok, rows)], C_ref, S)


@pytest.mark.parametrize("layer", range(4))
def test_llama3_8b_layers(gu, layer):
    name, N, K = LLAMA3_8B[layer]
    run_matrix(gu, inputs.gaussian_weights(N, K, inputs.seed_for(2, layer)), (1, 8, 32, 128), inputs.seed_for(2, layer, 1))


@pytest.mark.parametrize("N", [4096, 28672])
@pytest.mark.parametrize("kind", ["student_t", "outliers", "rowscale", "specials"])
def test_adversarial_full_size(gu, kind, N):
    seed = inputs.seed_for(3, N // 4096, ["student_t", "outliers", "rowscale", "specials"].index(kind))
    run_matrix(gu, inputs.make_weights(kind, N, 4096, seed=seed), (1, 16), seed + 1)


@pytest.mark.parametrize("layer", range(4))
def test_llama3_70b_layers(gu, layer):
    name, N, K = LLAMA3_70B[layer]
    run_matrix(gu, inputs.gaussian_weights(N, K, inputs.seed_for(4, layer), sigma=0.015), (1, 8, 64, 256),
               inputs.seed_for(4, layer, 1))


@pytest.mark.parametrize("layer", [2, 3])
def test_prefill_regime(gu, layer):
    name, N, K = LLAMA3_8B[layer]
    run_matrix(gu, inputs.gaussian_weights(N, K, inputs.seed_for(5, layer)), (1024, 2048, 4096), inputs.seed_for(5, layer, 1))


@pytest.mark.parametrize("layer", [2, 3])
def test_prefill_regime_stage_aware(gu, layer):
    """zs_linear on the prefill shapes: the decoupled path (zs_decompress + dense GEMM) at its real size."""
    name, N, K = LLAMA3_8B[layer]
    W = inputs.gaussian_weights(N, K, inputs.seed_for(5, layer))
    blob, d = binding.zs_encode(W)
    dev = gu.upload_blob(blob)
    rows = sample_rows(N, 7)
    ws = torch.empty(binding.zs_linear_workspace(d, 4096), dtype=torch.uint8, device="cuda")
    for M in (1024, 4096):
        assert binding.zs_linear_path(d, M) == binding.ZS_PATH_DECOUPLED
        A = inputs.activations(M, K, inputs.seed_for(5, layer, 1) + M)
        a = torch.from_numpy(A.view(np.int16)).cuda()
        c = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
        binding.zs_linear(d, dev, a, c, M, workspace_dev=ws, workspace_bytes=ws.numel())
        torch.cuda.synchronize()
        tok = sample_tokens(M, 11 * M)
        C_ref, S = oracle.gemm(np.ascontiguousarray(A[tok]), W, rows=rows, threads=8)
        gu.assert_gemm_matches(c.cpu().numpy()[np.ix_(tok, rows)], C_ref, S)


@pytest.mark.parametrize("name,N,K", [LLAMA3_8B[2], LLAMA3_8B[3]])
def test_encode_device_full_size(gu, name, N, K):
    """The GPU-side packer at benchmark size: blob and descriptor equal to the host packer's."""
    W = inputs.gaussian_weights(N, K, inputs.seed_for(2, 7))
    blob, d = binding.zs_encode(W)
    w_dev = torch.from_numpy(W.view(np.int16)).cuda()
    cap = binding.zs_encode_bound(N, K)
    out = torch.empty(cap, dtype=torch.uint8, device="cuda")
    ws = torch.empty(binding.ZS_ENCODE_WORKSPACE_BYTES, dtype=torch.uint8, device="cuda")
    d_dev = binding.zs_encode_device(w_dev, N, K, out, cap, ws)
    torch.cuda.synchronize()
    assert all(getattr(d_dev, f) == getattr(d, f) for f, _ in binding.ZsDesc._fields_)
    assert torch.equal(out[:d.total_bytes].cpu(), torch.from_numpy(blob))


def test_lm_head_shape(gu):
    """The LM head of the 8B family (128256 x 4096; Section 6.1 lists it among the benchmarked layers)."""
    run_matrix(gu, inputs.gaussian_weights(128256, 4096, inputs.seed_for(2, 4)), (1, 8, 32), inputs.seed_for(2, 4, 1))


@pytest.mark.parametrize("layer", range(32))
def test_decode_step_sweep_layer(gu, layer):
    """The 32 layers of the decode-step sweep (all seven projections, distinct seeds).  Every matrix
    is decompressed on the GPU and compared bit for bit with the weights it was packed from; on the
    first and the last layer the oracle decodes too and checks the GEMM at M = 16 (the other
    layers differ from them by their seeds only)."""
    for i, (name, N, K) in enumerate(LLAMA3_8B_PROJ):
        W = inputs.gaussian_weights(N, K, inputs.seed_for(5, 100 + 7 * layer + i))
        if layer in (0, 31):
            run_matrix(gu, W, (16,), inputs.seed_for(5, 100 + 7 * layer + i, 1))
            continue
        blob, d = binding.zs_encode(W)
        dev = gu.upload_blob(blob)
        out = torch.full((N, K), 0x5A5A, dtype=torch.int16, device="cuda")
        binding.zs_decompress(d, dev, out)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy().view(np.uint16), W)


@pytest.mark.parametrize("layer", [1, 2])
def test_bf16_output_full_size(gu, layer):
    """zs_gemm_bf16 at benchmark size (O: every strip shared by four workgroups; GateUp): sampled output
    features, all tokens, against the oracle with the BF16-output bound of the small-size test."""
    name, N, K = LLAMA3_8B[layer]
    W = inputs.gaussian_weights(N, K, inputs.seed_for(2, layer))
    blob, d = binding.zs_encode(W)
    dev = gu.upload_blob(blob)
    rows = sample_rows(N, 21 + layer)
    for M in (8, 32, 64):
        A = inputs.activations(M, K, inputs.seed_for(2, layer, 2) + M)
        a = torch.from_numpy(A.view(np.int16)).cuda()
        need = binding.zs_gemm_workspace(d, M)
        ws = torch.zeros(max(need, 256), dtype=torch.uint8, device="cuda")
        c = torch.full((M, N), 0x7FC1, dtype=torch.int16, device="cuda")
        binding.zs_gemm_bf16(d, dev, a, c, M, workspace_dev=ws, workspace_bytes=ws.numel())
        torch.cuda.synchronize()
        got = inputs.bf16_to_f32(c.cpu().numpy().view(np.uint16)[:, rows]).astype(np.float64)
        C_ref, S = oracle.gemm(A, W, rows=rows, threads=8)
        assert (np.abs(got - C_ref) <= 1e-3 * S + 1e-6 + 2.0 ** -8 * np.abs(C_ref)).all()
        assert not ws.cpu().numpy().any()
