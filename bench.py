#!/usr/bin/env python3
"""ZipGEMM benchmark on one MI355X.

Default run (the driver's contract): one JSON line.  A "step" is one pass of the hot path
over one batch: ``zs_gemm`` on the four LLaMA-3-8B-shaped linear layers (QKV 6144x4096,
O 4096x4096, GateUp 28672x4096, Down 4096x14336; weights N(0, 0.02) packed with
``zs_encode``) at M tokens (default 32).  Inputs are resident in HBM before the timed
region.  Weights rotate over several distinct copies so that more than 512 MB is touched
between two uses of the same bytes (the 256 MB Infinity Cache cannot serve them).

``value`` = compressed-byte throughput of the whole step: (blob + 2MK + 4MN) summed over the
layers / time, in GB/s.  ``roofline`` = the dominant launch (GateUp) against the 8 TB/s HBM
peak, timed live with events on the launch stream.  ``cpu_baseline`` = the CPU oracle
(scalar decode + double-accumulation GEMM) on a bounded sample of the same workload.

``--table PATH`` additionally writes per-(layer, M) rows with an uncompressed BF16 GEMM
(torch.matmul, i.e. hipBLASLt/rocBLAS) and the decompress-then-GEMM pipeline beside ZipGEMM.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--m", type=int, default=32, help="tokens per step")
    ap.add_argument("--copies", type=int, default=0, help="rotating weight copies (0 = enough for > 512 MB)")
    ap.add_argument("--config", type=int, default=0, help="force a zs_gemm configuration id")
    ap.add_argument("--table", type=str, default="", help="write the per-(layer, M) comparison table here")
    ap.add_argument("--table-m", type=str, default="1,8,32,128")
    ap.add_argument("--family", type=str, default="8b", choices=["8b", "70b"])
    ap.add_argument("--layers", type=str, default="", help="comma list of layer names to keep (profiling aid)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three 1 GiB device-to-device copies (reference for the HBM byte counters)")
    return ap.parse_args()


class Layer:
    """One packed weight matrix resident on the GPU, in `copies` distinct instances."""

    def __init__(self, name, N, K, seed, copies, sigma=0.02, keep_dense=False):
        import torch
        from paper_2603_17435_amd import binding, inputs
        self.name, self.N, self.K = name, N, K
        self.blobs, self.dense = [], []
        for c in range(copies):
            W = inputs.gaussian_weights(N, K, seed + c, sigma)
            blob, d = binding.zs_encode(W)
            self.desc = d if c == 0 else self.desc
            self.descs = getattr(self, "descs", []) + [d]
            self.blobs.append(torch.from_numpy(blob).cuda())
            if keep_dense:
                self.dense.append(torch.from_numpy(W.view(np.int16)).cuda().view(torch.bfloat16))
            if c == 0:
                self.W0 = W
        self.blob_bytes = int(np.mean([d.total_bytes for d in self.descs]))
        self.r = float(np.mean([d.n_high / (N * K) for d in self.descs]))

    def bytes_per_call(self, M):
        return self.blob_bytes + 2 * M * self.K + 4 * M * self.N

    def flops_per_call(self, M):
        return 2.0 * M * self.N * self.K


def time_calls(fn, steps, warmup):
    """Runs fn(i) warmup + steps times on the current stream; returns ms per call (events)."""
    import torch
    for i in range(warmup):
        fn(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(steps):
        fn(warmup + i)
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    return e0.elapsed_time(e1) / steps, wall_ms / steps


def cpu_baseline(M):
    """The CPU oracle on a bounded sample of the step: decode of a whole 4096 x 4096 layer plus
    the double-accumulation GEMM on it, single thread; reported in compressed GB/s."""
    import oracle
    from paper_2603_17435_amd import inputs
    N, K = 4096, 4096
    W = inputs.gaussian_weights(N, K, inputs.seed_for(2, 1))
    A = inputs.activations(M, K, inputs.seed_for(2, 1, 1))
    enc = oracle.encode(W)
    t0 = time.perf_counter()
    Wd = oracle.decode(enc)
    C, S = oracle.gemm(A, Wd, threads=1)
    dt = time.perf_counter() - t0
    nbytes = enc.stored_bytes + 2 * M * K + 4 * M * N
    return {"value": nbytes / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"O-projection 4096x4096 at M={M}: scalar decode + double GEMM, {dt:.2f} s, "
                      f"{2.0 * M * N * K / dt / 1e9:.2f} GFLOP/s"}


def recorded_traffic(layer, M):
    """HBM bytes per launch of the dominant kernel, as measured offline with rocprofv3 --pmc
    FETCH_SIZE / WRITE_SIZE and written to profiles/ (None when no record matches)."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{layer}_m{M}.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch"):
                return int(float(line.split()[1]))
    except OSError:
        pass
    return None


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (--gpus must be 1).", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2603_17435_amd import binding, inputs

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    M = args.m
    shapes = inputs.LLAMA3_8B_LAYERS if args.family == "8b" else inputs.LLAMA3_70B_LAYERS
    if args.layers:
        shapes = [sh for sh in shapes if sh[0] in args.layers.split(",")]
    sigma = 0.02 if args.family == "8b" else 0.015
    cfg_id = 2 if args.family == "8b" else 4
    raw_bytes = sum(2 * N * K for _, N, K in shapes)
    copies = args.copies or max(2, int(np.ceil(512e6 / (0.7 * raw_bytes))) + 1)
    layers = [Layer(name, N, K, inputs.seed_for(cfg_id, i), copies, sigma, keep_dense=bool(args.table))
              for i, (name, N, K) in enumerate(shapes)]

    Kmax = max(L.K for L in layers)
    acts = {L.K: torch.from_numpy(inputs.activations(M, L.K, inputs.seed_for(cfg_id, 9, M)).view(np.int16)).cuda()
            for L in layers}
    outs = {L.name: torch.empty((M, L.N), dtype=torch.float32, device="cuda") for L in layers}
    ws_bytes = max(binding.zs_gemm_workspace(L.desc, M, args.config) for L in layers)
    ws = torch.zeros(max(ws_bytes, 256), dtype=torch.uint8, device="cuda")  # zs_gemm wants it zero-filled once

    def step(i):
        c = i % copies
        for L in layers:
            binding.zs_gemm(L.descs[c], L.blobs[c], acts[L.K], outs[L.name], M, workspace_dev=ws,
                            workspace_bytes=ws_bytes, config=args.config)

    ms_step, wall_ms = time_calls(step, args.steps, args.warmup)
    step_bytes = sum(L.bytes_per_call(M) for L in layers)
    step_flops = sum(L.flops_per_call(M) for L in layers)
    gbps = step_bytes / (ms_step * 1e-3) / 1e9
    tflops = step_flops / (ms_step * 1e-3) / 1e12

    # dominant launch: the largest layer, timed alone on the same stream
    big = max(layers, key=lambda L: L.blob_bytes)

    def big_call(i):
        c = i % copies
        binding.zs_gemm(big.descs[c], big.blobs[c], acts[big.K], outs[big.name], M, workspace_dev=ws,
                        workspace_bytes=ws_bytes, config=args.config)

    ms_big, _ = time_calls(big_call, args.steps, args.warmup)
    achieved = big.bytes_per_call(M) / (ms_big * 1e-3) / 1e9
    per_layer = {}
    for L in layers:
        def one(i, L=L):
            c = i % copies
            binding.zs_gemm(L.descs[c], L.blobs[c], acts[L.K], outs[L.name], M, workspace_dev=ws,
                            workspace_bytes=ws_bytes, config=args.config)
        ms, _ = time_calls(one, max(20, args.steps // 2), 5)
        per_layer[L.name] = {"us": round(ms * 1e3, 2), "GBps": round(L.bytes_per_call(M) / ms / 1e6, 1),
                             "TFLOPs": round(L.flops_per_call(M) / ms / 1e9, 2),
                             "hbm_frac": round(L.bytes_per_call(M) / ms / 1e6 / HBM_PEAK_GBPS, 4)}

    result = {
        "metric": "ZipGEMM compressed GB/s (fused TCA-TBE decode + BF16 GEMM)",
        "value": round(gbps, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"LLaMA-3-{args.family.upper()}-shaped linear layers "
                               f"({', '.join(f'{n} {N}x{K}' for n, N, K in shapes)}), N(0,{sigma}) weights, M={M}, "
                               f"cold weights ({copies} rotating copies)",
                   "M": M, "gemm_config": args.config, "fraction_in_window": round(float(np.mean([L.r for L in layers])), 5)},
        "tflops": round(tflops, 3), "hbm_frac_step": round(gbps / HBM_PEAK_GBPS, 4),
        "mfma_frac_step": round(tflops / MFMA_BF16_PEAK_TFLOPS, 5), "wall_ms_per_step": round(wall_ms, 5),
        "per_layer": per_layer,
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": recorded_traffic(big.name, M),
                     "kernel": f"zs_gemm on {big.name} {big.N}x{big.K}, M={M}",
                     "bytes_per_launch": big.bytes_per_call(M), "us_per_launch": round(ms_big * 1e3, 2)},
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(M)

    if args.copy_calibration:
        x = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        y = torch.empty_like(x)
        for _ in range(3):
            y.copy_(x)
        torch.cuda.synchronize()
    if args.table:
        write_table(args, layers, copies, cfg_id)
    print(json.dumps(result))


def write_table(args, layers, copies, cfg_id):
    """Per-(layer, M): ZipGEMM vs uncompressed BF16 GEMM (torch.matmul) vs decompress + GEMM."""
    import torch
    from paper_2603_17435_amd import binding, inputs
    rows = []
    for L in layers:
        for M in [int(x) for x in args.table_m.split(",")]:
            A = torch.from_numpy(inputs.activations(M, L.K, inputs.seed_for(cfg_id, 9, M)).view(np.int16)).cuda()
            Ab = A.view(torch.bfloat16)
            C = torch.empty((M, L.N), dtype=torch.float32, device="cuda")
            scratch = torch.empty((L.N, L.K), dtype=torch.int16, device="cuda")
            ws_bytes = binding.zs_gemm_workspace(L.desc, M, args.config)
            ws = torch.zeros(max(ws_bytes, 256), dtype=torch.uint8, device="cuda")  # zs_gemm wants it zero-filled once
            steps = 200 if M <= 256 else 30

            def zip_(i):
                c = i % copies
                binding.zs_gemm(L.descs[c], L.blobs[c], A, C, M, workspace_dev=ws, workspace_bytes=ws_bytes,
                                config=args.config)

            def dense(i):
                torch.matmul(Ab, L.dense[i % copies].t())

            def decoupled(i):
                c = i % copies
                binding.zs_decompress(L.descs[c], L.blobs[c], scratch)
                torch.matmul(Ab, scratch.view(torch.bfloat16).t())

            def decomp_only(i):
                c = i % copies
                binding.zs_decompress(L.descs[c], L.blobs[c], scratch)

            t_zip, _ = time_calls(zip_, steps, 10)
            t_dense, _ = time_calls(dense, steps, 10)
            t_dec, _ = time_calls(decoupled, steps, 10)
            t_dco, _ = time_calls(decomp_only, steps, 10)
            rows.append({"layer": L.name, "N": L.N, "K": L.K, "M": M,
                         "zip_us": t_zip * 1e3, "dense_us": t_dense * 1e3, "decoupled_us": t_dec * 1e3,
                         "decompress_us": t_dco * 1e3,
                         "zip_GBps": L.bytes_per_call(M) / t_zip / 1e6,
                         "zip_hbm_frac": L.bytes_per_call(M) / t_zip / 1e6 / HBM_PEAK_GBPS,
                         "zip_TFLOPs": L.flops_per_call(M) / t_zip / 1e9,
                         "zip_mfma_frac": L.flops_per_call(M) / t_zip / 1e9 / MFMA_BF16_PEAK_TFLOPS,
                         "dense_GBps": (2 * L.N * L.K + 2 * M * L.K + 2 * M * L.N) / t_dense / 1e6,
                         "speedup_vs_dense": t_dense / t_zip,
                         "decompress_GBps": (L.blob_bytes + 2 * L.N * L.K) / t_dco / 1e6})
    os.makedirs(os.path.dirname(os.path.abspath(args.table)), exist_ok=True)
    with open(args.table, "w") as f:
        f.write("| layer | N x K | M | ZipGEMM us | GB/s (% of 8 TB/s) | TFLOP/s (% of 2.5 PF) | dense BF16 us | "
                "zip vs dense | decompress+GEMM us | decompress us (GB/s) |\n|---|---|---|---|---|---|---|---|---|---|\n")
        for r in rows:
            f.write(f"| {r['layer']} | {r['N']}x{r['K']} | {r['M']} | {r['zip_us']:.1f} | {r['zip_GBps']:.0f} "
                    f"({100 * r['zip_hbm_frac']:.1f}%) | {r['zip_TFLOPs']:.2f} ({100 * r['zip_mfma_frac']:.2f}%) | "
                    f"{r['dense_us']:.1f} | {r['speedup_vs_dense']:.2f}x | {r['decoupled_us']:.1f} | "
                    f"{r['decompress_us']:.1f} ({r['decompress_GBps']:.0f}) |\n")
        f.write("\n" + json.dumps(rows) + "\n")


if __name__ == "__main__":
    main()
