"""The GEMM entry points under HIP graph capture: they launch kernels only (no memset nodes, no
allocation, no synchronisation), so a captured step can be replayed.  Every replay is checked
against the eager result, with eager work and synchronisations between the replays."""
import numpy as np
import pytest

import oracle
from paper_2603_17435_amd import binding, inputs

pytestmark = pytest.mark.gpu


def test_gemm_entry_points_replay_from_a_graph():
    import torch
    import gpu_util as gu
    N, K, M = 1024, 1280, 24          # 320 BlockTiles over 256 workgroups: most strips are shared
    W = inputs.gaussian_weights(N, K, 91)
    A1, A2 = inputs.activations(M, K, 92), inputs.activations(M, K, 93)
    blob, d = binding.zs_encode(W)
    dev = gu.upload_blob(blob)
    a = torch.from_numpy(A1.view(np.int16)).cuda()
    need = binding.zs_gemm_workspace(d, M)
    ws = torch.zeros(max(need, 256), dtype=torch.uint8, device="cuda")
    c_ws = torch.empty((M, N), dtype=torch.float32, device="cuda")
    c_na = torch.empty((M, N), dtype=torch.float32, device="cuda")
    c_16 = torch.empty((M, N), dtype=torch.int16, device="cuda")

    def step():
        binding.zs_gemm(d, dev, a, c_ws, M, workspace_dev=ws, workspace_bytes=ws.numel())
        binding.zs_gemm_noalloc(d, dev, a, c_na, M)
        binding.zs_gemm_bf16(d, dev, a, c_16, M, workspace_dev=ws, workspace_bytes=ws.numel())

    refs = {}
    for name, Ax in (("a1", A1), ("a2", A2)):
        refs[name] = oracle.gemm(Ax, W, threads=8)
    step()                               # eager once: attribute caches, symbol lookup
    torch.cuda.synchronize()
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(graph, stream=stream):
            step()
    torch.cuda.synchronize()
    for rep, name in enumerate(("a1", "a2", "a1", "a2")):
        a.copy_(torch.from_numpy((A1 if name == "a1" else A2).view(np.int16)).cuda())  # eager work between replays
        for c in (c_ws, c_na):
            c.fill_(float("nan"))
        c_16.fill_(0x7FC1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        C_ref, S = refs[name]
        gu.assert_gemm_matches(c_ws.cpu().numpy(), C_ref, S)
        gu.assert_gemm_matches(c_na.cpu().numpy(), C_ref, S)
        got16 = inputs.bf16_to_f32(c_16.cpu().numpy().view(np.uint16)).astype(np.float64)
        assert (np.abs(got16 - C_ref) <= 1e-3 * S + 1e-6 + 2.0 ** -8 * np.abs(C_ref)).all()
        assert not ws.cpu().numpy().any()
