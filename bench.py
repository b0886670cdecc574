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
# HBM bytes per launch from rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled by what the same counters
# read for a plain copy of known size (profiles/bench_hbm_traffic.txt): mean over the three
# launches per step of the bf16 128 x 128 product kernel, and the int8 quantizer on 2^28 elements
# mean over the three launches of that kernel in a step: fc2's input gradient (8192 x 3072 out,
# contraction 768) and the two weight gradients (2.36 M outputs, contraction 8192), one-byte operands
ALGORITHMIC_F16_PRODUCT_128 = ((8192 * 768 + 3072 * 768 + 4 * 8192 * 3072) + 2 * (3072 * 8192 + 768 * 8192 + 4 * 3072 * 768)) / 3
# measured HBM bytes of the same three launches, slice sums included (rocprofv3 FETCH_SIZE / WRITE_SIZE)
TRAFFIC_F16_PRODUCT_128 = (2 * (52.7 + 27.0 + 27.0 + 9.0) + (24.2 + 96.2)) / 3 * 2**20
TRAFFIC_QUANTIZE_INT8_2P28 = (1024.0 + 256.0) * 2**20
MFMA_PEAK_TFLOPS = {"int8": 5000.0, "fp8": 5000.0, "bf16": 2500.0, "fp16": 2500.0}
TOKENS = 8192
FWD_KIND, BWD_KIND = "int8", "e5m2"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-quantizer-sweep", action="store_true")
    ap.add_argument("--train-step", action="store_true",
                    help="also time whole training steps of the small decoder at batch 8, 32 and 128")
    ap.add_argument("--llama-sweep", action="store_true",
                    help="also time the Llama-1B-shaped linears (bf16 weights, 4-bit output gradient, 8-bit "
                         "elsewhere) at 4096, 16384 and 65536 tokens, with the error of dW for a 4-bit against "
                         "an 8-bit output gradient")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB -> 1 GiB device copy (known HBM traffic, to scale "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


class Layer:
    """One linear's tensors, scales, quantizers, outputs and workspaces, all preallocated."""

    def __init__(self, L, synth, torch, name, M, N, K, seed, f8_flag, kinds=None, w_bf16=False):
        dev = "cuda:0"
        self.name, self.M, self.N, self.K = name, M, N, K
        self.A = synth.gaussian_torch((M, K), 1.0, seed, dev)
        self.W = synth.gaussian_torch((N, K), 0.02, seed + 1, dev)
        if w_bf16:
            self.W = self.W.to(torch.bfloat16)
        self.dY = synth.gaussian_torch((M, N), 1e-3, seed + 2, dev)
        kinds = kinds or {"A_fwd": L.INT8, "W_fwd": L.INT8, "A_bwd": L.E5M2, "W_bwd": L.E5M2, "dY_bwd": L.E5M2}
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
        # backward pass with one Q(dY) for both products.  (The variant that saves the backward
        # codes of A and W during the forward pass, sr_linear_fwd_stash, moves fewer bytes but is
        # no faster here: its forward quantizer does two quantizations per element loaded and its
        # products read operands that have left the last-level cache.  It is there to save memory.)
        self.absmax.run()
        self.forward(L)
        self.backward(L)

    def forward(self, L):
        L.sr_linear_fwd(self.A, self.W, self.q["A_fwd"], self.q["W_fwd"], out=self.Y, workspace=self.ws)

    def backward(self, L):
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


def event_ms(torch, fn, reps, warmup=3, warm_ms=30.0):
    """Average duration of fn's launches on the current stream, by HIP events.  Warm-up runs
    until `warm_ms` of GPU time has passed: after an idle gap the clocks take a while to ramp."""
    w0, w1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    w0.record()
    done = 0
    while True:
        for _ in range(warmup):
            fn()
        done += warmup
        w1.record()
        w1.synchronize()
        if w0.elapsed_time(w1) >= warm_ms or done > 10000:
            break
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
    # the weight update of Eq. 10 on 2^28 bfloat16 weights: 2 + 4 bytes read, 2 written per element
    w = (torch.randn(n, device="cuda:0") * 0.02).to(torch.bfloat16)
    g = torch.randn(n, device="cuda:0") * 1e-3
    ms = event_ms(torch, lambda: L.sr_update_bf16(w, g, 1e-3, seed=7, counter_offset=1 << 41), reps)
    res["update_bf16"] = {"ms": round(ms, 4), "GB/s": round(8 * n / (ms * 1e-3) / 1e9, 1),
                          "frac_of_hbm_peak": round(8 * n / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
    del w, g
    torch.cuda.empty_cache()
    return res


def train_step_times(torch, steps=3):
    """Whole training step of the 12-layer decoder (d = 768, 12 heads, vocabulary 32000, 1024
    tokens per sequence, random weights and token ids): forward, backward and the updates, every
    linear through the SR-quantized path, weights in bfloat16 updated by Eq. 10.  Also the
    weight-only objective of Sec. 3.2 (int8 weights, binary32 activations and gradients) at the
    smallest batch."""
    from paper_2511_00874_amd import train
    out = {}
    for label, weight_only, batches in (("five_quantizers", False, ((8, 1), (32, 1), (128, 4))),
                                        ("weight_only", True, ((8, 1),))):
        model = train.Decoder(weight_only=weight_only)
        out["model"] = ("decoder 12 x 768, 12 heads, vocab 32000, seq 1024; %.1f M weights in SR linears"
                        % (sum(m.in_features * m.out_features for m in model.sr_linears()) / 1e6))
        res = {}
        for b, micro in batches:
            ids = torch.randint(0, 32000, (b, 1024), device="cuda:0")
            tgt = torch.roll(ids, -1, 1)
            train.train_step(model, ids, tgt, 1e-3, micro)
            sec = time_steps(torch, lambda: train.train_step(model, ids, tgt, 1e-3, micro), steps, 0)
            res["b%d" % b] = {"ms_per_step": round(sec * 1e3, 2), "micro_batches": micro,
                              "sr_linear_TFLOP/s": round(train.flops_per_token(model) * b * 1024 / sec / 1e12, 1)}
        out[label] = res
        del model
        torch.cuda.empty_cache()
    return out


def llama_sweep(L, synth, torch):
    """Config 4: the Llama-1B-shaped linears, weights held in bfloat16, the output gradient on the
    4-bit integer grid and the other four quantizers on the 8-bit one, whole layer step (scales,
    quantizers, three products) by HIP events.  Per token count also the batch-for-bits figure of
    Sec. 4.2 on the 2048 x 2048 layer: rms error of the mean gradient dW / T against the product
    of the unquantized tensors (binary64 on the device, 256 rows of dW), with a 4-bit and with an
    8-bit output gradient: it falls like 1 / sqrt(T) and scales with the step of the format."""
    out = {}
    i8 = {"A_fwd": L.INT8, "W_fwd": L.INT8, "A_bwd": L.INT8, "W_bwd": L.INT8}
    for T in (4096, 16384, 65536):
        row = {}
        for name, N, K in (("qkvo", 2048, 2048), ("gate_up", 5632, 2048), ("down", 2048, 5632)):
            ly = Layer(L, synth, torch, name, T, N, K, 7, 0, kinds=dict(i8, dY_bwd=L.INT4), w_bf16=True)
            ms = event_ms(torch, lambda: ly.step(L), 10)
            row[name] = {"us": round(ms * 1e3, 1), "TFLOP/s": round(ly.flops() / ms / 1e9, 1)}
            if name == "qkvo":
                exact = ly.dY[:, :256].double().t() @ ly.A.double()
                ref = float(T)
                err = {"int4": float((ly.dW[:256].double() - exact).pow(2).mean().sqrt()) / ref}
                l8 = Layer(L, synth, torch, name, T, N, K, 7, 0, kinds=dict(i8, dY_bwd=L.INT8), w_bf16=True)
                l8.step(L)
                err["int8"] = float((l8.dW[:256].double() - exact).pow(2).mean().sqrt()) / ref
                row["rms_error_of_dW_over_T"] = {k: float("%.3g" % v) for k, v in err.items()}
                del l8, exact
            del ly
            torch.cuda.empty_cache()
        out["T%d" % T] = row
    return out


def product_kernel_rooflines(L, torch, layers, reps):
    """The product kernels alone, operands already quantized, timed by HIP events on the stream
    they are launched on: the f16 pipeline fed from E5M2 codes (backward products of the default
    path), the int8 pipeline (forward products) and the fp8 pipeline (backward products with the
    flag set), each over the same shapes the step launches them on."""
    dev = "cuda:0"
    out = {}

    def codes(P, R):
        return torch.randint(0, 120, (P, R), dtype=torch.uint8, device=dev)

    fwd_shapes = [(ly.M, ly.N, ly.K) for ly in layers]
    bwd_shapes = [s for ly in layers for s in ((ly.M, ly.K, ly.N), (ly.N, ly.K, ly.M))]
    # the backward products that run the 128 x 128-tile instantiation (the 8192 x 768 output of
    # fc1's input gradient takes the 128 x 192 one): fc2's input gradient and both weight gradients
    bwd128 = [s for s in bwd_shapes if not (s[0] == TOKENS and s[1] == 768)]
    for name, shapes, make, call, need_fn, peak, kernel in (
            ("f16", bwd128, codes, lambda X, Z, o, ws: L.sr_gemm_e5m2(X, Z, out=o, workspace=ws),
             L.raw.sr_gemm_e5m2_workspace_bytes, MFMA_PEAK_TFLOPS["fp16"], "gemm_nt_kernel<E5M2F16Mma, 128, 128, 2, 2, 2>"),
            ("int8", fwd_shapes, codes, lambda X, Z, o, ws: L.sr_gemm_codes(X, L.INT8, Z, L.INT8, out=o, workspace=ws),
             L.raw.sr_gemm_workspace_bytes, MFMA_PEAK_TFLOPS["int8"], "gemm_nt_kernel<I8Mma, 128, ...>"),
            ("fp8", bwd_shapes, codes, lambda X, Z, o, ws: L.sr_gemm_codes(X, L.E5M2, Z, L.E5M2, out=o, workspace=ws),
             L.raw.sr_gemm_workspace_bytes, MFMA_PEAK_TFLOPS["fp8"], "gemm_nt_kernel<F8Mma<1,1>, 128, ...>")):
        calls, flops = [], 0.0
        for (P, Q, R) in shapes:
            need = need_fn(P, Q, R)
            calls.append((make(P, R), make(Q, R), torch.empty((P, Q), dtype=torch.float32, device=dev),
                          torch.empty(max(need, 16), dtype=torch.uint8, device=dev)))
            flops += 2.0 * P * Q * R

        def run():
            for X, Z, o, ws in calls:
                call(X, Z, o, ws)
        ms = event_ms(torch, run, reps) / len(calls)
        fl = flops / len(calls)
        tf = fl / (ms * 1e-3) / 1e12
        out[name] = {"kernel": kernel, "launches": len(calls), "avg_launch_us": round(ms * 1e3, 2),
                     "flop_per_launch": fl, "TFLOP/s": round(tf, 1), "peak": peak, "frac": round(tf / peak, 4)}
        del calls
    torch.cuda.empty_cache()
    return out


def phase_times(L, torch, layers, reps):
    """Entry-point level split of one step, by HIP events."""
    def absmax():
        for ly in layers:
            ly.absmax.run()

    def fwd():
        for ly in layers:
            ly.forward(L)

    def bwd():
        for ly in layers:
            ly.backward(L)
    res = {n: round(event_ms(torch, f, reps) * 1e3, 1) for n, f in (("absmax_us", absmax), ("fwd_us", fwd), ("bwd_us", bwd))}
    nbytes = sum(4 * (ly.A.numel() + ly.W.numel() + ly.dY.numel()) for ly in layers)
    res["absmax_GB/s"] = round(nbytes / (res["absmax_us"] * 1e-6) / 1e9, 1)
    return res


def cpu_baseline(layers_shape):
    """The CPU oracle, as it stands, on a bounded sample of the same workload: the five absmax
    scales and five quantizations of fc1 in full (8192 tokens) and the three products on 2^20
    sampled output entries each."""
    import numpy as np

    import oracle
    from paper_2511_00874_amd import synth
    name, N, K = layers_shape[0]
    M = TOKENS
    A, W, dY = synth.single_layer(M, N, K, seed=0, std_dy=1e-3)
    t0 = time.perf_counter()
    q = {}
    off = 0
    for qn, x, kind in (("A_fwd", A, oracle.INT8), ("W_fwd", W, oracle.INT8), ("A_bwd", A, oracle.E5M2),
                        ("W_bwd", W, oracle.E5M2), ("dY_bwd", dY, oracle.E5M2)):
        q[qn] = oracle.Quant(kind, oracle.absmax_scale(x, kind), 0, off)
        off += (x.size + 7) // 8
    rng = np.random.default_rng(0)
    n_out = 1 << 20
    flops = 0.0
    oracle.linear_fwd(A, W, q["A_fwd"], q["W_fwd"], at=rng.integers(0, M * N, n_out).astype(np.uint64))
    flops += 2.0 * n_out * K
    oracle.linear_bwd_data(dY, W, q["dY_bwd"], q["W_bwd"], at=rng.integers(0, M * K, n_out).astype(np.uint64))
    flops += 2.0 * n_out * N
    oracle.linear_bwd_weight(dY, A, q["dY_bwd"], q["A_bwd"], at=rng.integers(0, N * K, n_out).astype(np.uint64))
    flops += 2.0 * n_out * M
    dt = time.perf_counter() - t0
    return {"value": round(flops / dt / 1e12, 6), "unit": "TFLOP/s", "cores": oracle.threads(), "kind": "oracle",
            "sample": f"fc1 at {M} tokens: 5 absmax + 5 quantizations of the full tensors (each product re-quantizes "
                      f"its operands, as Alg. 1/2 state), then 3 x {n_out} sampled entries of Y/dA/dW; "
                      f"{flops / 1e9:.1f} GFLOP of products in {dt:.1f} s wall"}


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
    result, phases, rl = {}, None, None
    for label, flag in (("exact", 0), ("f8_pipeline", L.FLAG_F8_PIPELINE)):
        layers = [Layer(L, synth, torch, nm, TOKENS, N, K, 100 + 10 * i, flag) for i, (nm, N, K) in enumerate(shapes)]

        def step():
            for ly in layers:
                ly.step(L)
        sec = time_steps(torch, step, args.steps, args.warmup)
        flops = sum(ly.flops() for ly in layers)
        result[label] = (sec, flops / sec / 1e12)
        if label == "exact":
            # the same steps with the scales taken as given (they are inputs of the entry points)
            def step_given_scales():
                for ly in layers:
                    ly.forward(L)
                    ly.backward(L)
            sec_gs = time_steps(torch, step_given_scales, args.steps, args.warmup)
            result["given_scales"] = (sec_gs, flops / sec_gs / 1e12)
            reps = max(5, args.steps // 2)
            phases = phase_times(L, torch, layers, reps)
            rl = product_kernel_rooflines(L, torch, layers, reps)
        del layers
        torch.cuda.empty_cache()

    sec, tflops = result["exact"]
    io_bytes = sum(4.0 * (3 * TOKENS * K + 3 * N * K + 2 * TOKENS * N) for _, N, K in shapes)
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
        "dtype": "int8 (i32 acc) forward; e5m2 codes widened to f16 on the f16 pipeline (f32 acc) backward",
        "data": "synthetic",
        "config": {"workload": "configs[2]: GPT-2-small MLP linears fc1 (3072x768) + fc2 (768x3072), "
                               "8192 tokens, fp32 in/out, int8 SR forward, E5M2 SR backward; per layer "
                               "5 absmax scales, 5 quantizers, 3 products",
                   "tokens": TOKENS, "flop_per_step": 2 * 6.0 * TOKENS * 768 * 3072,
                   "min_hbm_bytes_per_step": io_bytes},
        "frac_of_8bit_mfma_peak": round(tflops / MFMA_PEAK_TFLOPS["int8"], 4),
        # the path's own ceiling: fp32 tensors in and out once per quantizer pass at HBM peak
        "composite_ceiling_TFLOP/s": round(2 * 6.0 * TOKENS * 768 * 3072 / (io_bytes / (HBM_PEAK_GBS * 1e9)) / 1e12, 1),
        "phases": phases,
        "scales_given": {"value": round(result["given_scales"][1], 2), "unit": "TFLOP/s",
                         "ms_per_step": round(result["given_scales"][0] * 1e3, 4),
                         "note": "forward + backward entry points only (five quantizers, three products per "
                                 "layer), the absmax passes left out: the scale is an input of the entry points"},
        "f8_pipeline": {"value": round(result["f8_pipeline"][1], 2), "unit": "TFLOP/s",
                        "ms_per_step": round(result["f8_pipeline"][0] * 1e3, 4),
                        "frac_of_8bit_mfma_peak": round(result["f8_pipeline"][1] / MFMA_PEAK_TFLOPS["fp8"], 4),
                        "note": "backward products on the fp8 matrix pipeline (hardware-truncated group sums, "
                                "SRQ_FLAG_F8_PIPELINE)"},
        "product_kernels": rl,
    }
    dom = rl["f16"]
    line["roofline"] = {"bound": "mfma", "kernel": dom["kernel"], "achieved": dom["TFLOP/s"], "peak": dom["peak"],
                        "unit": "TFLOP/s", "frac": dom["frac"], "traffic": round(TRAFFIC_F16_PRODUCT_128),
                        "note": "dominant kernel of the step by time (3 of its 6 products); 38.65 GFLOP per launch "
                                "over the mean event-timed launch, which for the two weight-gradient launches "
                                "includes the kernel that sums the three contraction slices; algorithmic bytes "
                                "per launch %.1fe6 (operands once, result once), traffic = measured HBM bytes"
                                % (ALGORITHMIC_F16_PRODUCT_128 / 1e6)}
    if not args.no_quantizer_sweep:
        qs = quantizer_sweep(L, synth, torch, max(5, args.steps // 5))
        line["sr_quantize"] = qs
        line["roofline_quantizer"] = {"bound": "hbm", "kernel": "quantize_flat_f32_kernel<INT8, SR, byte> on 2^28 elements (5 B per element)",
                                      "achieved": qs["int8"]["GB/s"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                      "frac": qs["int8"]["frac_of_hbm_peak"], "traffic": round(TRAFFIC_QUANTIZE_INT8_2P28)}
    if args.train_step:
        line["train_step"] = train_step_times(torch)
    if args.llama_sweep:
        line["llama_linears"] = llama_sweep(L, synth, torch)
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(shapes)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
