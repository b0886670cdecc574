"""Benchmark of the SR-quantized linear hot path on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic input: for each of the
two GPT-2-small MLP linears (d=768, d_ff=3072) at 8192 tokens, the five per-tensor absmax
scales, the five SR quantizations (int8 forward, E5M2 backward) and the three products
Y = Q(A)Q(W)^T, dA = Q(dY)Q(W), dW = Q(dY)^T Q(A).  Inputs are resident in HBM before the
timed region.  Prints ONE JSON line; extra keys carry the standalone-quantizer sweep
(2^28 fp32 elements -> int8 / int4 / E4M3 / E5M2), the kernel rooflines and the CPU oracle
timed on the host cores.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = {"int8": 5000.0, "fp8": 5000.0, "bf16": 2500.0}
TOKENS = 8192
FWD_KIND, BWD_KIND = "int8", "e5m2"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-quantizer-sweep", action="store_true")
    return ap.parse_args()


class Layer:
    """One linear's tensors, scales, quantizers, outputs and workspaces, all preallocated."""

    def __init__(self, L, synth, torch, name, M, N, K, seed, f8_flag):
        dev = "cuda:0"
        self.name, self.M, self.N, self.K = name, M, N, K
        self.A = synth.gaussian_torch((M, K), 1.0, seed, dev)
        self.W = synth.gaussian_torch((N, K), 0.02, seed + 1, dev)
        self.dY = synth.gaussian_torch((M, N), 1e-3, seed + 2, dev)
        kinds = {"A_fwd": L.INT8, "W_fwd": L.INT8, "A_bwd": L.E5M2, "W_bwd": L.E5M2, "dY_bwd": L.E5M2}
        src = {"A": self.A, "W": self.W, "dY": self.dY}
        self.scales = torch.empty(5, dtype=torch.float32, device=dev)
        self.q, self.src_of = {}, {}
        off = 0
        for i, (qn, kind) in enumerate(kinds.items()):
            t = src[qn.split("_")[0]]
            self.q[qn] = L.Quant(kind, self.scales[i:i + 1], seed=seed, counter_offset=off,
                                 flags=f8_flag if kind in (L.E4M3, L.E5M2) else 0)
            self.src_of[qn] = (t, kind, self.scales[i:i + 1])
            off += (t.numel() + 7) // 8
        self.Y = torch.empty((M, N), dtype=torch.float32, device=dev)
        self.dA = torch.empty((M, K), dtype=torch.float32, device=dev)
        self.dW = torch.empty((N, K), dtype=torch.float32, device=dev)
        need = max(L.sr_linear_workspace_bytes(op, M, N, K) for op in (L.OP_FWD, L.OP_BWD))
        self.ws = torch.empty(need, dtype=torch.uint8, device=dev)
        self.absmax = L.AbsmaxBatch([(t, kind, s) for t, kind, s in self.src_of.values()])

    def step(self, L):
        # a0: five scales (three passes: A and W feed two formats each); a1-a5: forward, then the
        # backward pass with one Q(dY) for both products
        self.absmax.run()
        L.sr_linear_fwd(self.A, self.W, self.q["A_fwd"], self.q["W_fwd"], out=self.Y, workspace=self.ws)
        L.sr_linear_bwd(self.dY, self.W, self.A, self.q["dY_bwd"], self.q["W_bwd"], self.q["A_bwd"],
                        out_dA=self.dA, out_dW=self.dW, workspace=self.ws)

    def flops(self):
        return 6.0 * self.M * self.N * self.K


def time_steps(torch, fn, steps, warmup):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def event_ms(torch, fn, reps, warmup=3):
    """Average duration of fn's launches on the current stream, by HIP events."""
    for _ in range(warmup):
        fn()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / reps


def quantizer_sweep(L, synth, torch, reps):
    """Standalone SR quantize of 2^28 fp32 values ~N(0,1) with 1% outliers ~N(0,50)."""
    n = 1 << 28
    x = synth.outlier_tensor_torch(n, 1234, "cuda:0")
    out = torch.empty(n, dtype=torch.uint8, device="cuda:0")
    res = {}
    for kind in (L.INT8, L.INT4, L.E4M3, L.E5M2):
        s = L.sr_absmax_scale(x, kind)
        q = L.Quant(kind, s, seed=42, counter_offset=1 << 40)
        ms = event_ms(torch, lambda: L.sr_quantize(x, q, out=out), reps)
        nbytes = 4 * n + (n // 2 if kind == L.INT4 else n)
        gbs = nbytes / (ms * 1e-3) / 1e9
        res[L.KIND_NAMES[kind]] = {"ms": round(ms, 4), "GB/s": round(gbs, 1), "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4)}
    ms = event_ms(torch, lambda: L.sr_absmax_scale(x, L.INT8, out=s), reps)
    res["absmax"] = {"ms": round(ms, 4), "GB/s": round(4 * n / (ms * 1e-3) / 1e9, 1),
                     "frac_of_hbm_peak": round(4 * n / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
    del x, out
    torch.cuda.empty_cache()
    return res


def gemm_rooflines(L, torch, layers, reps):
    """The product kernels alone (operands already quantized), by HIP events: per pipeline the
    average launch duration over the six products of one step and the MFMA rate it reaches."""
    out = {}
    for pipe, kind, flag, peak in (("int8", L.INT8, 0, MFMA_PEAK_TFLOPS["int8"]),
                                   ("fp8", L.E5M2, 1, MFMA_PEAK_TFLOPS["fp8"])):
        calls, flops = [], 0.0
        for ly in layers:
            for (P, Q, R) in ((ly.M, ly.N, ly.K), (ly.M, ly.K, ly.N), (ly.N, ly.K, ly.M)):
                X = torch.randint(0, 120, (P, R), dtype=torch.uint8, device="cuda:0")
                Z = torch.randint(0, 120, (Q, R), dtype=torch.uint8, device="cuda:0")
                o = torch.empty((P, Q), dtype=torch.float32, device="cuda:0")
                need = L.sr_gemm_workspace_bytes(P, Q, R)
                ws = torch.empty(max(need, 1), dtype=torch.uint8, device="cuda:0")
                calls.append((X, Z, o, ws))
                flops += 2.0 * P * Q * R

        def run():
            for X, Z, o, ws in calls:
                L.sr_gemm_codes(X, kind, Z, kind, out=o, workspace=ws)
        ms = event_ms(torch, run, reps)
        out[pipe] = {"ms_six_products": round(ms, 4), "TFLOP/s": round(flops / (ms * 1e-3) / 1e12, 1),
                     "frac_of_peak": round(flops / (ms * 1e-3) / 1e12 / peak, 4)}
    return out


def cpu_baseline(layers_shape):
    """The CPU oracle on a bounded sample of the same workload: the five quantizations of a
    512-token slab of fc1 and the three products on sampled output entries."""
    import numpy as np

    import oracle
    from paper_2511_00874_amd import synth
    name, N, K = layers_shape[0]
    M = 512
    A, W, dY = synth.single_layer(M, N, K, seed=0, std_dy=1e-3)
    t0 = time.perf_counter()
    q = {}
    off = 0
    for qn, x, kind in (("A_fwd", A, oracle.INT8), ("W_fwd", W, oracle.INT8), ("A_bwd", A, oracle.E5M2),
                        ("W_bwd", W, oracle.E5M2), ("dY_bwd", dY, oracle.E5M2)):
        q[qn] = oracle.Quant(kind, oracle.absmax_scale(x, kind), 0, off)
        off += (x.size + 7) // 8
    rng = np.random.default_rng(0)
    n_out = 1 << 16
    flops = 0.0
    oracle.linear_fwd(A, W, q["A_fwd"], q["W_fwd"], at=rng.integers(0, M * N, n_out).astype(np.uint64))
    flops += 2.0 * n_out * K
    oracle.linear_bwd_data(dY, W, q["dY_bwd"], q["W_bwd"], at=rng.integers(0, M * K, n_out).astype(np.uint64))
    flops += 2.0 * n_out * N
    oracle.linear_bwd_weight(dY, A, q["dY_bwd"], q["A_bwd"], at=rng.integers(0, N * K, n_out).astype(np.uint64))
    flops += 2.0 * n_out * M
    dt = time.perf_counter() - t0
    return {"value": round(flops / dt / 1e12, 6), "unit": "TFLOP/s", "cores": oracle.threads(), "kind": "oracle",
            "sample": f"fc1 slab of {M} tokens: 5 absmax + 5 quantizations in full, 3 x {n_out} sampled "
                      f"output entries of Y/dA/dW; {dt:.1f} s of wall time"}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import torch

    from paper_2511_00874_amd import lib as L
    from paper_2511_00874_amd import synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU (there is no CPU path)", file=sys.stderr)
        sys.exit(2)

    shapes = synth.GPT2_SMALL_MLP
    result = {}
    for label, flag in (("exact", 0), ("f8_pipeline", L.FLAG_F8_PIPELINE)):
        layers = [Layer(L, synth, torch, nm, TOKENS, N, K, 100 + 10 * i, flag) for i, (nm, N, K) in enumerate(shapes)]

        def step():
            for ly in layers:
                ly.step(L)
        sec = time_steps(torch, step, args.steps, args.warmup)
        flops = sum(ly.flops() for ly in layers)
        result[label] = (sec, flops / sec / 1e12)
        if label == "f8_pipeline":
            rl = gemm_rooflines(L, torch, layers, max(5, args.steps // 5))
            # the bf16 pipeline products of the default path, through the linear entry points' own
            # kernels: time one backward product pair minus nothing -- reported from the profile
        del layers
        torch.cuda.empty_cache()

    sec, tflops = result["exact"]
    line = {
        "metric": "SR-quantized linear fwd+bwd TFLOP/s",
        "value": round(tflops, 2),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(sec * 1e3, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int8 fwd (i32 acc) / e5m2 bwd as bf16 (f32 acc)",
        "data": "synthetic",
        "config": {"workload": "configs[2]: GPT-2-small MLP linears fc1 (3072x768) + fc2 (768x3072), "
                               "8192 tokens, fp32 in/out, int8 SR forward, E5M2 SR backward, "
                               "5 absmax + 5 quantizers + 3 products per layer",
                   "tokens": TOKENS, "flop_per_step": 2 * 6.0 * TOKENS * 768 * 3072},
        "frac_of_8bit_mfma_peak": round(tflops / MFMA_PEAK_TFLOPS["int8"], 4),
        "f8_pipeline": {"value": round(result["f8_pipeline"][1], 2), "unit": "TFLOP/s",
                        "ms_per_step": round(result["f8_pipeline"][0] * 1e3, 4),
                        "frac_of_8bit_mfma_peak": round(result["f8_pipeline"][1] / MFMA_PEAK_TFLOPS["fp8"], 4),
                        "note": "backward products on the fp8 matrix pipeline (hardware-truncated group sums)"},
        "product_kernels": rl,
    }
    dom = rl["int8"]
    line["roofline"] = {"bound": "mfma", "kernel": "gemm_nt_kernel<I8Mma> (six products of one step)",
                        "achieved": dom["TFLOP/s"], "peak": MFMA_PEAK_TFLOPS["int8"], "unit": "TFLOP/s",
                        "frac": dom["frac_of_peak"], "traffic": None}
    if not args.no_quantizer_sweep:
        qs = quantizer_sweep(L, synth, torch, max(5, args.steps // 5))
        line["sr_quantize"] = qs
        line["roofline_quantizer"] = {"bound": "hbm", "kernel": "quantize_flat_kernel<INT8,F32,SR> on 2^28 elements",
                                      "achieved": qs["int8"]["GB/s"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                      "frac": qs["int8"]["frac_of_hbm_peak"], "traffic": None}
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(shapes)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
