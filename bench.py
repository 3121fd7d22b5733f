#!/usr/bin/env python3
"""ZipGEMM benchmark on one MI355X.

Default run (the driver's contract): one JSON line.  A "step" is one pass of the hot path
over one batch: ``zs_gemm`` on the four LLaMA-3-8B-shaped linear layers (QKV 6144x4096,
O 4096x4096, GateUp 28672x4096, Down 4096x14336; weights N(0, 0.02) packed with
``zs_encode``) at M tokens (default 32).  Inputs are resident in HBM before the timed
region.  Weights rotate over several distinct copies so that more than 512 MB is touched
between two uses of the same bytes (the 256 MB Infinity Cache cannot serve them).

``value`` = compressed-byte throughput of the whole step: (blob + 2MK + 4MN) summed over the
layers / time, in GB/s; ``--steps`` / ``--warmup`` govern this leg only.  The other legs
follow the paper's timing method (Section 6.1: 100 warm-up + 1000 timed launches) whatever
``--steps`` says:
  ``roofline``    the dominant launch (GateUp) against the 8 TB/s HBM peak, events on the
                  launch stream;
  ``per_layer``   every layer alone, with the uncompressed BF16 GEMM (hipBLASLt through the
                  library's ``zs_dense_gemm``, best of the heuristic's algorithms) beside it;
  ``decompress``  the standalone decompression kernel on GateUp against the same peak;
  ``cpu_baseline`` the CPU oracle (scalar decode + double-accumulation GEMM) on a bounded
                  sample of the same workload, on one core (and on all cores beside it).

``--table PATH`` writes per-(layer, M) rows: ZipGEMM, the stage-aware ``zs_linear``, dense BF16,
decompress + dense, decompress alone.  ``--sweep`` runs the 32-layer, seven-projection decode
sweep at M = 16 (generated, packed and uploaded layer by layer) and reports aggregate GB/s.
``--variants PATH`` packs a GateUp-shaped matrix in every format variant (codeword length 2 / 3 / 4,
window per matrix / BlockTile / row, sparse or dense H) and times their decompression.
"""
from __future__ import annotations

import argparse
import json
import os
import subprocess
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
PAPER_WARMUP, PAPER_TIMED = 100, 1000  # Section 6.1


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--m", type=int, default=32, help="tokens per step")
    ap.add_argument("--copies", type=int, default=0, help="rotating weight copies (0 = enough for > 512 MB)")
    ap.add_argument("--config", type=int, default=0, help="force a zs_gemm configuration id")
    ap.add_argument("--table", type=str, default="", help="write the per-(layer, M) comparison table here")
    ap.add_argument("--table-m", type=str, default="1,8,16,32,64,128,256,1024,4096")
    ap.add_argument("--family", type=str, default="8b", choices=["8b", "70b"])
    ap.add_argument("--layers", type=str, default="", help="comma list of layer names to keep (profiling aid)")
    ap.add_argument("--sweep", type=str, default="", help="run the 32-layer decode sweep at M = 16; write its report here")
    ap.add_argument("--sweep-layers", type=int, default=32)
    ap.add_argument("--variants", type=str, default="",
                    help="compare the format variants (codeword length, window granularity, dense H) on GateUp; write the table here")
    ap.add_argument("--dense-algos", type=int, default=8,
                    help="how many of hipBLASLt's heuristic algorithms the dense baseline is picked from")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-clock-query", action="store_true", help="do not start rocm-smi (for runs under rocprofv3)")
    ap.add_argument("--quick", action="store_true", help="10 + 100 launches instead of 100 + 1000 in the fixed legs")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three 1 GiB device-to-device copies (reference for the HBM byte counters)")
    return ap.parse_args()


# ---- byte and flop accounting (Section 3.3: compute intensity = FLOP / bytes moved) -------------------
def gemm_flops(M, N, K):
    return 2.0 * M * N * K


def dense_gemm_bytes(M, N, K):
    """Uncompressed BF16 GEMM: weights, activations and results, two bytes each (CI_GEMM)."""
    return 2.0 * (N * K + M * K + M * N)


def decoupled_bytes(M, N, K, cr):
    """Decompress-then-GEMM: the compressed weights are read, the decompressed ones written and
    read again (CI_Decoupled): N K (2 / CR + 4) + 2 (M K + M N)."""
    return N * K * (2.0 / cr + 4.0) + 2.0 * (M * K + M * N)


def fused_bytes(M, N, K, cr):
    """Fused decompression-GEMM: only the compressed weights move (CI_ZipServ)."""
    return N * K * 2.0 / cr + 2.0 * (M * K + M * N)


def ci_degradation_pct(M, N, K, cr):
    """How far the decoupled pipeline's compute intensity falls below the plain GEMM's, in percent."""
    ci_gemm = gemm_flops(M, N, K) / dense_gemm_bytes(M, N, K)
    ci_dec = gemm_flops(M, N, K) / decoupled_bytes(M, N, K, cr)
    return 100.0 * (1.0 - ci_dec / ci_gemm)


class Layer:
    """One packed weight matrix resident on the GPU, in `copies` distinct instances."""

    def __init__(self, name, N, K, seed, copies, sigma=0.02, keep_dense=False):
        import torch
        from paper_2603_17435_amd import binding, inputs
        self.name, self.N, self.K = name, N, K
        self.blobs, self.dense, self.descs = [], [], []
        for c in range(copies):
            W = inputs.gaussian_weights(N, K, seed + c, sigma)
            blob, d = binding.zs_encode(W)
            self.descs.append(d)
            self.blobs.append(torch.from_numpy(blob).cuda())
            if keep_dense:
                self.dense.append(torch.from_numpy(W.view(np.int16)).cuda())
        self.desc = self.descs[0]
        self.blob_bytes = int(np.mean([d.total_bytes for d in self.descs]))
        self.r = float(np.mean([d.n_high / (N * K) for d in self.descs]))

    def bytes_per_call(self, M):
        """Algorithmic bytes of one ZipGEMM call: the blob, the activations, the FP32 result."""
        return self.blob_bytes + 2 * M * self.K + 4 * M * self.N

    def flops_per_call(self, M):
        return gemm_flops(M, self.N, self.K)


def time_calls(fn, steps, warmup):
    """Runs fn(i) warmup + steps times on the current stream; returns ms per call (events)."""
    import torch
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for i in range(warmup):
        fn(i)
    torch.cuda.synchronize()
    # (nothing but the event between the synchronisation and the first launch: the GPU's clocks
    # sag after an idle gap, and a short timed window would mostly measure their recovery)
    e0.record()
    t0 = time.perf_counter()
    for i in range(steps):
        fn(warmup + i)
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    return e0.elapsed_time(e1) / steps, wall_ms / steps


def best_dense_algo(A, W, C, M, N, K, lt_ws, tries=8):
    """Index of the fastest of the first `tries` algorithms hipBLASLt's heuristic returns for this
    shape (short timing).  Only the head of the list is tried: it holds the library's preferred
    kernels, and one of the entries further down faulted the GPU on the 70B QKV shape at 1024 tokens."""
    from paper_2603_17435_amd import binding
    n = min(binding.zs_dense_gemm_algos(M, N, K, lt_ws.numel()), tries)
    best, best_t = 0, float("inf")
    for a in range(n):
        try:
            t, _ = time_calls(lambda i: binding.zs_dense_gemm(A, W, C, M, N, K, workspace_dev=lt_ws,
                                                              workspace_bytes=lt_ws.numel(), algo=a), 20, 3)
        except binding.ZsError:
            continue
        if t < best_t:
            best, best_t = a, t
    return best


def cpu_baseline(M, threads):
    """The CPU oracle on one whole step (every layer of the workload once): scalar decode of the
    blob plus the double-accumulation GEMM on the decoded weights; reported in compressed GB/s."""
    import oracle
    from paper_2603_17435_amd import inputs
    layers = inputs.LLAMA3_8B_LAYERS
    nbytes, flops, t_dec, t_all = 0, 0.0, 0.0, 0.0
    for i, (name, N, K) in enumerate(layers):
        W = inputs.gaussian_weights(N, K, inputs.seed_for(2, i))
        A = inputs.activations(M, K, inputs.seed_for(2, i, 1))
        enc = oracle.encode(W)
        t0 = time.perf_counter()
        Wd = oracle.decode(enc)
        t1 = time.perf_counter()
        oracle.gemm(A, Wd, threads=threads)
        t2 = time.perf_counter()
        t_dec, t_all = t_dec + (t1 - t0), t_all + (t2 - t0)
        nbytes += enc.stored_bytes + 2 * M * K + 4 * M * N
        flops += 2.0 * M * N * K
        del W, Wd, enc
    return {"value": nbytes / t_all / 1e9, "unit": "GB/s", "cores": threads, "kind": "oracle",
            "sample": f"one step ({', '.join(n for n, _, _ in layers)}) at M={M}: scalar decode ({t_dec:.1f} s, one thread) + "
                      f"double GEMM on {threads} thread(s), {t_all:.1f} s in all, {flops / t_all / 1e9:.2f} GFLOP/s"}


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


def environment(query_clocks=True):
    """Clocks and versions of the machine the numbers come from."""
    import torch
    env = {"torch": torch.__version__, "hip": getattr(torch.version, "hip", None),
           "device": torch.cuda.get_device_name(0), "compute_units": torch.cuda.get_device_properties(0).multi_processor_count}
    try:
        env["rocm"] = open("/opt/rocm/.info/version").read().strip()
    except OSError:
        pass
    if not query_clocks:  # under a profiler no other program is started
        return env
    try:
        out = subprocess.run(["rocm-smi", "--showclocks", "--json"], capture_output=True, text=True, timeout=20).stdout
        card = next(iter(json.loads(out).values()))
        env["clocks"] = {k: v for k, v in card.items() if "sclk" in k.lower() or "mclk" in k.lower()}
    except Exception:  # the numbers do not depend on this
        pass
    return env


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (--gpus must be 1).", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2603_17435_amd import binding, inputs

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.sweep:
        run_sweep(args)
        return
    if args.variants:
        run_variants(args)
        return
    M = args.m
    fixed_warm, fixed_timed = (10, 100) if args.quick else (PAPER_WARMUP, PAPER_TIMED)
    shapes = inputs.LLAMA3_8B_LAYERS if args.family == "8b" else inputs.LLAMA3_70B_LAYERS
    if args.layers:
        # the LM head of the 8B family (Section 6.1) is not part of the step: only on request
        shapes = [sh for sh in list(shapes) + [("lm_head", 128256, 4096)] if sh[0] in args.layers.split(",")]
    sigma = 0.02 if args.family == "8b" else 0.015
    cfg_id = 2 if args.family == "8b" else 4
    raw_bytes = sum(2 * N * K for _, N, K in shapes)
    copies = args.copies or max(2, int(np.ceil(512e6 / (0.7 * raw_bytes))) + 1)
    layers = [Layer(name, N, K, inputs.seed_for(cfg_id, i), copies, sigma, keep_dense=True)
              for i, (name, N, K) in enumerate(shapes)]

    acts = {L.K: torch.from_numpy(inputs.activations(M, L.K, inputs.seed_for(cfg_id, 9, M)).view(np.int16)).cuda()
            for L in layers}
    outs = {L.name: torch.empty((M, L.N), dtype=torch.float32, device="cuda") for L in layers}
    ws_bytes = max(binding.zs_gemm_workspace(L.desc, M, args.config) for L in layers)
    ws = torch.zeros(max(ws_bytes, 256), dtype=torch.uint8, device="cuda")  # zs_gemm wants it zero-filled once
    lt_ws = torch.empty(binding.ZS_DENSE_WORKSPACE_BYTES, dtype=torch.uint8, device="cuda")

    def gemm(L, i):
        c = i % copies
        binding.zs_gemm(L.descs[c], L.blobs[c], acts[L.K], outs[L.name], M, workspace_dev=ws,
                        workspace_bytes=ws_bytes, config=args.config)

    def step(i):
        for L in layers:
            gemm(L, i)

    # per layer, each alone on the same stream, with the dense BF16 GEMM beside it (paper's timing method)
    per_layer = {}
    for L in layers:
        ms, _ = time_calls(lambda i, L=L: gemm(L, i), fixed_timed, fixed_warm)
        algo = best_dense_algo(acts[L.K], L.dense[0], outs[L.name], M, L.N, L.K, lt_ws, args.dense_algos)
        ms_d, _ = time_calls(lambda i, L=L: binding.zs_dense_gemm(acts[L.K], L.dense[i % copies], outs[L.name], M, L.N,
                                                                  L.K, workspace_dev=lt_ws, workspace_bytes=lt_ws.numel(),
                                                                  algo=algo), fixed_timed, fixed_warm)
        per_layer[L.name] = {"us": round(ms * 1e3, 2), "GBps": round(L.bytes_per_call(M) / ms / 1e6, 1),
                             "TFLOPs": round(L.flops_per_call(M) / ms / 1e9, 2),
                             "hbm_frac": round(L.bytes_per_call(M) / ms / 1e6 / HBM_PEAK_GBPS, 4),
                             "config": binding.zs_gemm_configs()[args.config or binding.zs_gemm_pick_config(L.desc, M)],
                             "dense_us": round(ms_d * 1e3, 2), "vs_dense": round(ms_d / ms, 3)}

    # dominant launch: the largest layer (its per-layer figure is the roofline figure)
    big = max(layers, key=lambda L: L.blob_bytes)
    us_big = per_layer[big.name]["us"]
    achieved = big.bytes_per_call(M) / us_big / 1e3

    # standalone decompression of the largest layer
    dense_out = torch.empty((big.N, big.K), dtype=torch.int16, device="cuda")
    ms_dec, _ = time_calls(lambda i: binding.zs_decompress(big.descs[i % copies], big.blobs[i % copies], dense_out),
                           max(fixed_timed // 4, 50), max(fixed_warm // 4, 10))
    dec_bytes = big.blob_bytes + 2 * big.N * big.K

    # GPU-side packer on the same layer (wall clock: the call waits for the stream twice)
    w_dev = big.dense[0]
    enc_cap = binding.zs_encode_bound(big.N, big.K)
    enc_out = torch.empty(enc_cap, dtype=torch.uint8, device="cuda")
    enc_ws = torch.empty(binding.ZS_ENCODE_WORKSPACE_BYTES, dtype=torch.uint8, device="cuda")
    enc_times = []
    for _ in range(6):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        enc_desc = binding.zs_encode_device(w_dev, big.N, big.K, enc_out, enc_cap, enc_ws)
        torch.cuda.synchronize()
        enc_times.append(time.perf_counter() - t0)
    ms_enc = float(np.median(enc_times[1:])) * 1e3
    assert enc_desc.total_bytes == big.desc.total_bytes
    del enc_out

    # The step leg comes last: the legs above have brought the GPU to its steady clocks, so a short
    # run (few steps, few warm-up steps) measures the same state as a long one.
    ms_step, wall_ms = time_calls(step, args.steps, args.warmup)
    step_bytes = sum(L.bytes_per_call(M) for L in layers)
    step_flops = sum(L.flops_per_call(M) for L in layers)
    gbps = step_bytes / (ms_step * 1e-3) / 1e9
    tflops = step_flops / (ms_step * 1e-3) / 1e12

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
        "vs_dense_step": round(sum(v["dense_us"] for v in per_layer.values()) / sum(v["us"] for v in per_layer.values()), 3),
        "per_layer": per_layer,
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": recorded_traffic(big.name, M),
                     "kernel": f"zs_gemm on {big.name} {big.N}x{big.K}, M={M}",
                     "bytes_per_launch": big.bytes_per_call(M), "us_per_launch": us_big,
                     "launches": f"{fixed_warm} warm-up + {fixed_timed} timed"},
        "decompress": {"kernel": f"zs_decompress on {big.name} {big.N}x{big.K}", "us_per_launch": round(ms_dec * 1e3, 2),
                       "bytes_per_launch": dec_bytes, "achieved": round(dec_bytes / ms_dec / 1e6, 1), "unit": "GB/s",
                       "frac": round(dec_bytes / ms_dec / 1e6 / HBM_PEAK_GBPS, 4)},
        "encode_device": {"kernel": f"zs_encode_device on {big.name} {big.N}x{big.K}", "ms_per_call": round(ms_enc, 3),
                          "GBps_of_bf16_input": round(2 * big.N * big.K / ms_enc / 1e6, 1)},
        "env": environment(not args.no_clock_query),
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(M, 1)
        result["cpu_baseline_all_cores"] = cpu_baseline(M, min(os.cpu_count() or 1, 16))

    if args.copy_calibration:
        x = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        y = torch.empty_like(x)
        for _ in range(3):
            y.copy_(x)
        torch.cuda.synchronize()
    if args.table:
        del dense_out
        write_table(args, layers, copies, cfg_id)
    print(json.dumps(result))


def write_table(args, layers, copies, cfg_id):
    """Per-(layer, M): ZipGEMM, zs_linear, uncompressed BF16 GEMM (hipBLASLt), decompress + GEMM."""
    import torch
    from paper_2603_17435_amd import binding, inputs
    rows = []
    lt_ws = torch.empty(binding.ZS_DENSE_WORKSPACE_BYTES, dtype=torch.uint8, device="cuda")
    for L in layers:
        scratch = torch.empty((L.N, L.K), dtype=torch.int16, device="cuda")
        lin_ws = torch.zeros(max(binding.zs_linear_workspace(L.desc, 4096), binding.zs_linear_workspace(L.desc, 1), 256),
                             dtype=torch.uint8, device="cuda")
        cr = 2.0 * L.N * L.K / L.blob_bytes
        for M in [int(x) for x in args.table_m.split(",")]:
            A = torch.from_numpy(inputs.activations(M, L.K, inputs.seed_for(cfg_id, 9, M)).view(np.int16)).cuda()
            C = torch.empty((M, L.N), dtype=torch.float32, device="cuda")
            ws_bytes = binding.zs_gemm_workspace(L.desc, M, args.config)
            ws = torch.zeros(max(ws_bytes, 256), dtype=torch.uint8, device="cuda")  # zs_gemm wants it zero-filled once
            timed, warm = (PAPER_TIMED, PAPER_WARMUP) if M <= 256 else (100, 10)
            if args.quick:
                timed, warm = timed // 10, warm // 10 + 1
            algo = best_dense_algo(A, L.dense[0], C, M, L.N, L.K, lt_ws, args.dense_algos)

            def zip_(i):
                c = i % copies
                binding.zs_gemm(L.descs[c], L.blobs[c], A, C, M, workspace_dev=ws, workspace_bytes=ws_bytes,
                                config=args.config)

            def linear(i):
                c = i % copies
                binding.zs_linear(L.descs[c], L.blobs[c], A, C, M, workspace_dev=lin_ws, workspace_bytes=lin_ws.numel())

            def dense(i):
                binding.zs_dense_gemm(A, L.dense[i % copies], C, M, L.N, L.K, workspace_dev=lt_ws,
                                      workspace_bytes=lt_ws.numel(), algo=algo)

            def decoupled(i):
                c = i % copies
                binding.zs_decompress(L.descs[c], L.blobs[c], scratch)
                binding.zs_dense_gemm(A, scratch, C, M, L.N, L.K, workspace_dev=lt_ws, workspace_bytes=lt_ws.numel(),
                                      algo=algo)

            def decomp_only(i):
                c = i % copies
                binding.zs_decompress(L.descs[c], L.blobs[c], scratch)

            t_zip, _ = time_calls(zip_, timed if M <= 256 else 30, warm)
            if binding.zs_linear_path(L.desc, M) == binding.ZS_PATH_FUSED:
                lin_ws.zero_()  # the decoupled path leaves decompressed weights where the fused one keeps its counters
            t_lin, _ = time_calls(linear, timed, warm)
            t_dense, _ = time_calls(dense, timed, warm)
            t_dec, _ = time_calls(decoupled, timed, warm)
            t_dco, _ = time_calls(decomp_only, max(timed // 4, 25), max(warm // 4, 5))
            rows.append({"layer": L.name, "N": L.N, "K": L.K, "M": M,
                         "zip_us": t_zip * 1e3, "linear_us": t_lin * 1e3, "dense_us": t_dense * 1e3,
                         "decoupled_us": t_dec * 1e3, "decompress_us": t_dco * 1e3,
                         "linear_path": "fused" if binding.zs_linear_path(L.desc, M) == binding.ZS_PATH_FUSED else "decoupled",
                         "zip_config": binding.zs_gemm_configs()[args.config or binding.zs_gemm_pick_config(L.desc, M)],
                         "zip_GBps": L.bytes_per_call(M) / t_zip / 1e6,
                         "zip_hbm_frac": L.bytes_per_call(M) / t_zip / 1e6 / HBM_PEAK_GBPS,
                         "zip_TFLOPs": L.flops_per_call(M) / t_zip / 1e9,
                         "zip_mfma_frac": L.flops_per_call(M) / t_zip / 1e9 / MFMA_BF16_PEAK_TFLOPS,
                         "linear_TFLOPs": L.flops_per_call(M) / t_lin / 1e9,
                         "dense_TFLOPs": L.flops_per_call(M) / t_dense / 1e9,
                         "dense_GBps": dense_gemm_bytes(M, L.N, L.K) / t_dense / 1e6,
                         "speedup_vs_dense": t_dense / t_zip, "linear_vs_dense": t_dense / t_lin,
                         "decoupled_overhead_pct": 100.0 * (t_dec - t_dense) / t_dense,
                         "ci_degradation_pct_model": ci_degradation_pct(M, L.N, L.K, cr),
                         "decompress_GBps": (L.blob_bytes + 2 * L.N * L.K) / t_dco / 1e6})
        del scratch, lin_ws
    os.makedirs(os.path.dirname(os.path.abspath(args.table)), exist_ok=True)
    with open(args.table, "w") as f:
        f.write(f"Command: `python bench.py {' '.join(sys.argv[1:])}`  \n")
        f.write(f"Environment: {json.dumps(environment())}  \n")
        f.write("Every figure: average over back-to-back launches after a warm-up (M <= 256: "
                f"{PAPER_TIMED // (10 if args.quick else 1)} launches after {PAPER_WARMUP // (10 if args.quick else 1)}; beyond: 100 after 10), "
                f"weights rotating over {copies} copies of the layer so that no launch finds its weights in the last-level cache; "
                f"dense = hipBLASLt BF16 GEMM on the uncompressed weights, the fastest of the first {args.dense_algos} "
                "algorithms its heuristic returns for the shape; zs_linear's decoupled path runs the heuristic's first.\n\n")
        f.write("| layer | N x K | M | ZipGEMM us (kernel) | GB/s (% of 8 TB/s) | TFLOP/s (% of 2.5 PF) | dense BF16 us | "
                "zip vs dense | zs_linear us (path) | linear vs dense | decompress+dense us (overhead vs dense) | "
                "decompress us (GB/s) |\n|---|---|---|---|---|---|---|---|---|---|---|---|\n")
        for r in rows:
            f.write(f"| {r['layer']} | {r['N']}x{r['K']} | {r['M']} | {r['zip_us']:.1f} ({r['zip_config']}) | {r['zip_GBps']:.0f} "
                    f"({100 * r['zip_hbm_frac']:.1f}%) | {r['zip_TFLOPs']:.2f} ({100 * r['zip_mfma_frac']:.2f}%) | "
                    f"{r['dense_us']:.1f} | {r['speedup_vs_dense']:.2f}x | {r['linear_us']:.1f} ({r['linear_path']}) | "
                    f"{r['linear_vs_dense']:.2f}x | {r['decoupled_us']:.1f} ({r['decoupled_overhead_pct']:+.0f}%) | "
                    f"{r['decompress_us']:.1f} ({r['decompress_GBps']:.0f}) |\n")
    with open(args.table + ".json", "w") as f:
        json.dump(rows, f)


def run_sweep(args):
    """A whole decode step of an 8B-shaped model at M = 16: 32 layers x 7 projections with distinct
    seeds, generated, packed and uploaded layer by layer, then every zs_gemm back to back (each
    weight byte is touched once per pass: cold HBM by construction)."""
    import torch
    from paper_2603_17435_amd import binding, inputs
    M = 16
    mats = []
    t0 = time.perf_counter()
    for layer in range(args.sweep_layers):
        for j, (name, N, K) in enumerate(inputs.LLAMA3_8B_PROJECTIONS):
            W = inputs.gaussian_weights(N, K, inputs.seed_for(5, 10 * layer + j))
            blob, d = binding.zs_encode(W)
            mats.append((f"{layer}.{name}", d, torch.from_numpy(blob).cuda()))
        print(f"layer {layer} packed and uploaded ({time.perf_counter() - t0:.0f} s)", file=sys.stderr, flush=True)
    Ks = sorted({d.K for _, d, _ in mats})
    acts = {K: torch.from_numpy(inputs.activations(M, K, inputs.seed_for(5, 9, M)).view(np.int16)).cuda() for K in Ks}
    outs = {N: torch.empty((M, N), dtype=torch.float32, device="cuda") for N in sorted({d.N for _, d, _ in mats})}
    ws_bytes = max(binding.zs_gemm_workspace(d, M) for _, d, _ in mats)
    ws = torch.zeros(max(ws_bytes, 256), dtype=torch.uint8, device="cuda")

    def sweep(i):
        for _, d, blob in mats:
            binding.zs_gemm(d, blob, acts[d.K], outs[d.N], M, workspace_dev=ws, workspace_bytes=ws_bytes)

    ms, _ = time_calls(sweep, 20, 3)
    nbytes = sum(d.total_bytes + 2 * M * d.K + 4 * M * d.N for _, d, _ in mats)
    raw = sum(2 * d.N * d.K for _, d, _ in mats)
    rep = {"workload": f"{args.sweep_layers} layers x 7 projections (q, k, v, o, gate, up, down), N(0,0.02), M={M}",
           "matrices": len(mats), "blob_GB": round(sum(d.total_bytes for _, d, _ in mats) / 1e9, 3), "raw_GB": round(raw / 1e9, 3),
           "ms_per_sweep": round(ms, 3), "GBps": round(nbytes / ms / 1e6, 1), "hbm_frac": round(nbytes / ms / 1e6 / HBM_PEAK_GBPS, 4),
           "launches_per_sweep": len(mats), "us_per_launch": round(ms * 1e3 / len(mats), 2), "env": environment()}
    os.makedirs(os.path.dirname(os.path.abspath(args.sweep)), exist_ok=True)
    with open(args.sweep, "w") as f:
        f.write(json.dumps(rep, indent=1) + "\n")
    print(json.dumps(rep))


def run_variants(args):
    """Section 4.2's comparison of codeword lengths, measured: every variant of the format packs
    the same GateUp-shaped matrix (Gaussian, and with a scale per row), and the variant kernel
    decompresses it (checked bit for bit against the matrix on the device)."""
    import torch
    from paper_2603_17435_amd import binding, inputs
    N, K = 28672, 4096
    modes = (("matrix", binding.ZS_BASE_MATRIX), ("BlockTile", binding.ZS_BASE_TILE), ("row", binding.ZS_BASE_ROW))
    rows = []
    for kind in ("gauss", "rowscale"):
        W = inputs.make_weights(kind, N, K, inputs.seed_for(1, 2))
        W_dev = torch.from_numpy(W.view(np.int16)).cuda()
        # three copies of every blob and three outputs in rotation: > 1 GB between two uses of the
        # same bytes, so the 256 MB last-level cache serves none of them
        outs = [torch.empty((N, K), dtype=torch.int16, device="cuda") for _ in range(3)]
        out = outs[0]
        blob, d = binding.zs_encode(W)
        devs = [torch.from_numpy(blob).cuda() for _ in range(3)]
        ms, _ = time_calls(lambda i: binding.zs_decompress(d, devs[i % 3], outs[i % 3]), 99, 9)
        rows.append({"weights": kind, "variant": "main format, zs_decompress (tuned)", "r": d.n_high / W.size,
                     "bits_model": None, "bits_stored": 8 * d.total_bytes / W.size, "us": ms * 1e3,
                     "GBps": (d.total_bytes + 2 * W.size) / ms / 1e6})
        del devs
        for n in (2, 3, 4):
            for mode_name, mode in modes:
                for dense in (0, 1):
                    t0 = time.perf_counter()
                    blob, vd = binding.zs_variant_encode(W, n, mode, dense)
                    pack_s = time.perf_counter() - t0
                    devs = [torch.from_numpy(blob).cuda() for _ in range(3)]
                    for o in outs:
                        o.fill_(0x5A5A)
                    ms, _ = time_calls(lambda i: binding.zs_variant_decompress(vd, devs[i % 3], outs[i % 3]), 99, 9)
                    exact = all(bool(torch.equal(o, W_dev)) for o in outs)
                    r = vd.n_high / W.size
                    model = r * (n + 8) + (1 - r) * (n + 16) + (8 * (1 - r) if dense else 0)
                    rows.append({"weights": kind, "variant": f"n={n}, window per {mode_name}, {'dense' if dense else 'sparse'} H",
                                 "n": n, "window": mode_name, "dense_h": dense, "r": r, "bits_model": model,
                                 "bits_stored": 8 * vd.total_bytes / W.size, "us": ms * 1e3,
                                 "GBps": (vd.total_bytes + 2 * W.size) / ms / 1e6, "bit_exact": exact, "pack_s": pack_s})
                    print(f"{kind} n={n} {mode_name} dense={dense}: r={r:.4f} {rows[-1]['bits_stored']:.3f} bits "
                          f"{ms * 1e3:.1f} us exact={exact}", file=sys.stderr, flush=True)
                    assert exact, "variant decompression is not bit-exact"
                    del devs
    os.makedirs(os.path.dirname(os.path.abspath(args.variants)), exist_ok=True)
    with open(args.variants, "w") as f:
        f.write("# TCA-TBE format variants on a GateUp-shaped matrix (28672 x 4096)\n\n")
        f.write(f"Command (GPU box, repository root): `python3 bench.py --variants {args.variants}`  \n")
        f.write(f"Environment: {json.dumps(environment())}  \n")
        f.write("Weights: `gauss` = N(0, 0.02); `rowscale` = N(0, 0.02) with a scale per row, log-uniform over three decades. "
                "r = share of elements inside the window(s); model = Section 4.2's AverageBits(n) = r (n + 8) + (1 - r)(n + 16) "
                "(+ 8 (1 - r) with dense H); stored = blob bits per element (model + offsets, window bytes, padding). "
                "Decompression: zs_variant_decompress, 9 warm-up + 99 timed launches rotating over three copies of the blob and three "
                "outputs (cold), bytes = blob + 2 N K; every output compared bit for bit with the matrix on the device.\n\n")
        f.write("| weights | variant | r | model bits | stored bits | vs BF16 | decompress us | GB/s (% of 8 TB/s) |\n|---|---|---|---|---|---|---|---|\n")
        for r in rows:
            model = "" if r["bits_model"] is None else f"{r['bits_model']:.3f}"
            f.write(f"| {r['weights']} | {r['variant']} | {r['r']:.4f} | {model} | {r['bits_stored']:.3f} | "
                    f"{16 / r['bits_stored']:.3f}x | {r['us']:.1f} | {r['GBps']:.0f} ({100 * r['GBps'] / HBM_PEAK_GBPS:.1f}%) |\n")
    with open(args.variants + ".json", "w") as f:
        f.write(json.dumps(rows, indent=1) + "\n")
    print(json.dumps({"variants": len(rows), "table": args.variants}))


if __name__ == "__main__":
    main()
