"""Benchmark of the SR-quantized linear hot path on one MI355X.

Headline workload: the seven linears of one Llama-1B-shaped decoder layer (q, k, v, o:
2048 x 2048; gate, up: 5632 x 2048; down: 2048 x 5632) at 65536 tokens, master weights in
bfloat16, the output gradient on the 4-bit integer grid and the other four quantizers on the
8-bit one.  One step = one pass of the whole hot path over that batch: per linear the five
per-tensor absmax scales, the five SR quantizations and the three products
Y = Q(A)Q(W)^T, dA = Q(dY)Q(W), dW = Q(dY)^T Q(A).  Inputs are resident in HBM before the
timed region.  Prints ONE JSON line; extra keys carry the token sweep (4096 / 16384 tokens),
the GPT-2-small MLP workload (int8 forward, E5M2 backward; also replayed from a HIP graph),
the standalone-quantizer sweep (2^28 fp32 elements -> int8 / int4 / E4M3 / E5M2), whole
training steps of the small decoder, the kernel rooflines and the CPU oracle timed on the host.
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
MFMA_PEAK_TFLOPS = {"int8": 5000.0, "fp8": 5000.0, "bf16": 2500.0, "fp16": 2500.0}
TOKENS = 65536
GPT2_TOKENS = 8192
# Bytes moved behind the L2 per launch of the dominant kernel (int8 product, 256 x 256 tiles) on the nine
# products of the headline workload, slice sums included: rocprofv3 FETCH_SIZE + WRITE_SIZE scaled by
# what the same counters read for a plain copy of known size (profiles/product_int8_llama_hbm_traffic.txt)
TRAFFIC_I8_PRODUCT_LLAMA = 1393623303
TRAFFIC_QUANTIZE_INT8_2P28 = (1024.0 + 256.0) * 2**20


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="headline step and its roofline only (for profiling runs)")
    ap.add_argument("--only", default="", help="run only this section (profiling runs): step, gpt2, products, fused, quantizer")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB -> 1 GiB device copy (known HBM traffic, to scale "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


class Layer:
    """One linear's tensors, scales, quantizers, outputs and workspaces, all preallocated."""

    def __init__(self, L, synth, torch, name, M, N, K, seed, f8_flag=0, kinds=None, w_bf16=False, counters_dev=False,
                 stash=False):
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
        offs = []
        off = 0
        for qn in kinds:
            offs.append(off)
            off += (src[qn.split("_")[0]].numel() + 7) // 8
        # stream positions on the device: a captured step is replayed with fresh thresholds by
        # advancing these words (one add kernel per step)
        self.counters = torch.tensor(offs, dtype=torch.int64, device=dev) if counters_dev else None
        self.advance = off
        for i, (qn, kind) in enumerate(kinds.items()):
            t = src[qn.split("_")[0]]
            self.q[qn] = L.Quant(kind, self.scales[i:i + 1], seed=seed,
                                 counter_offset=self.counters[i:i + 1] if counters_dev else offs[i],
                                 flags=f8_flag if kind in (L.E4M3, L.E5M2) else 0)
            self.src_of[qn] = (t, kind, self.scales[i:i + 1])
        self.Y = torch.empty((M, N), dtype=torch.float32, device=dev)
        self.dA = torch.empty((M, K), dtype=torch.float32, device=dev)
        self.dW = torch.empty((N, K), dtype=torch.float32, device=dev)
        # forward and backward operands in workspaces of their own: the backward operands of a layer can
        # then be rounded while its forward product still reads the forward ones
        # `stash`: the forward pass also rounds A and W with the backward quantizers (one read of each feeds
        # both of its quantizers) and keeps those codes for the backward pass, which then reads only dY
        self.stash = torch.empty(L.sr_linear_stash_bytes(M, N, K), dtype=torch.uint8, device=dev) if stash else None
        op_f, op_b = (L.OP_FWD_STASH, L.OP_BWD_STASHED) if stash else (L.OP_FWD, L.OP_BWD)
        self.ws = torch.empty(L.sr_linear_workspace_bytes(op_f, M, N, K), dtype=torch.uint8, device=dev)
        self.ws_bwd = torch.empty(L.sr_linear_workspace_bytes(op_b, M, N, K), dtype=torch.uint8, device=dev)
        self.absmax = L.AbsmaxBatch([(t, kind, s) for t, kind, s in self.src_of.values()])

    def step(self, L):
        # a0: five scales (three passes: A and W feed two formats each); a1-a5: forward, then the
        # backward pass with one Q(dY) for both products
        self.absmax.run()
        self.forward(L)
        self.backward(L)
        if self.counters is not None:
            self.counters.add_(self.advance)

    def forward(self, L):
        if self.stash is not None:
            return self.forward_phase(L, L.PHASE_BOTH)
        L.sr_linear_fwd(self.A, self.W, self.q["A_fwd"], self.q["W_fwd"], out=self.Y, workspace=self.ws)

    def backward(self, L, phase=None):
        q = self.q
        if self.stash is not None:
            L.sr_linear_bwd_stashed(self.dY, self.stash, self.K, q["dY_bwd"], q["W_bwd"], q["A_bwd"], out_dA=self.dA,
                                    out_dW=self.dW, workspace=self.ws_bwd, phase=phase or L.PHASE_BOTH)
        else:
            L.sr_linear_bwd(self.dY, self.W, self.A, q["dY_bwd"], q["W_bwd"], q["A_bwd"],
                            out_dA=self.dA, out_dW=self.dW, workspace=self.ws_bwd, phase=phase)

    def forward_phase(self, L, phase):
        q = self.q
        if self.stash is not None:
            L.sr_linear_fwd_stash(self.A, self.W, q["A_fwd"], q["W_fwd"], q["A_bwd"], q["W_bwd"], stash=self.stash,
                                  out=self.Y, workspace=self.ws, phase=phase)
        else:
            L.sr_linear_fwd(self.A, self.W, q["A_fwd"], q["W_fwd"], out=self.Y, workspace=self.ws, phase=phase)

    def flops(self):
        return 6.0 * self.M * self.N * self.K

    def min_hbm_bytes(self):
        """Every fp32 / bf16 tensor in once per pass over it (absmax, forward quantizers, backward quantizers;
        with the stash the forward pass over A and W serves their backward quantizers too), every result out once."""
        ew = self.W.element_size()
        passes = 2.0 if self.stash is not None else 3.0
        return (4.0 * passes * self.M * self.K + ew * passes * self.N * self.K + 4.0 * 2 * self.M * self.N
                + 4.0 * (self.M * self.N + self.M * self.K + self.N * self.K))


class TwoStreamStep:
    """One step over several independent linears with the memory-bound half of the path (absmax, operand
    quantizers) on one stream and the products on another: the quantizer and absmax kernels of the next
    linears run on the CUs beside the product kernel of the current one (its two waves per SIMD leave
    registers and LDS for one more wave), instead of each kernel waiting for the one before.  Every
    launch of the single-stream step is made, with the same arguments; events carry the dependencies
    (scales -> quantizers -> products), and both streams join the caller's stream at the end."""

    def __init__(self, torch, L, layers):
        self.torch, self.L, self.layers = torch, L, layers
        self.mem, self.mat = torch.cuda.Stream(), torch.cuda.Stream()
        self.ev = [(torch.cuda.Event(), torch.cuda.Event()) for _ in layers]

    def __call__(self):
        torch, L = self.torch, self.L
        cur = torch.cuda.current_stream()
        self.mem.wait_stream(cur)
        self.mat.wait_stream(cur)
        for ly, (ev_f, ev_b) in zip(self.layers, self.ev):
            with torch.cuda.stream(self.mem):
                ly.absmax.run()
                ly.forward_phase(L, L.PHASE_QUANTIZE)
                ev_f.record()
                ly.backward(L, L.PHASE_QUANTIZE)
                ev_b.record()
            with torch.cuda.stream(self.mat):
                self.mat.wait_event(ev_f)
                ly.forward_phase(L, L.PHASE_PRODUCT)
                self.mat.wait_event(ev_b)
                ly.backward(L, L.PHASE_PRODUCT)
        cur.wait_stream(self.mem)
        cur.wait_stream(self.mat)


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


LLAMA_KINDS = ("A_fwd", "W_fwd", "A_bwd", "W_bwd")


def llama_layers(L, synth, torch, T, shapes, seed0=7):
    kinds = {k: L.INT8 for k in LLAMA_KINDS}
    kinds["dY_bwd"] = L.INT4
    return [Layer(L, synth, torch, nm, T, N, K, seed0 + 10 * i, kinds=kinds, w_bf16=True, stash=True)
            for i, (nm, N, K) in enumerate(shapes)]


def llama_products_roofline(L, synth, torch, reps):
    """The dominant kernel of the headline step alone: the nine product launches of the three distinct
    layer shapes at 65536 tokens -- forward product, weight-gradient product, input-gradient product
    (which also carries the sum of the weight gradient's contraction slices) -- as the step issues
    them (product halves of the stash pair), from the operands the step's quantizers wrote: int8
    codes, the 4-bit output gradient two values per byte.  Timed by HIP events on the launch stream."""
    T = TOKENS
    shapes = [synth.LLAMA_1B_LINEARS[i] for i in (0, 4, 6)]
    layers = llama_layers(L, synth, torch, T, shapes)
    flops = alg_bytes = 0.0
    for ly in layers:
        ly.absmax.run()
        ly.forward_phase(L, L.PHASE_QUANTIZE)
        ly.backward(L, L.PHASE_QUANTIZE)
        M, N, K = ly.M, ly.N, ly.K
        flops += 6.0 * M * N * K
        # operands once (Q(dY) at half a byte per element) + the fp32 result once, per product
        alg_bytes += (M * K + N * K + 4.0 * M * N) + (M * N / 2 + K * N + 4.0 * M * K) + (N * M / 2 + K * M + 4.0 * N * K)
    torch.cuda.synchronize()

    def run():
        for ly in layers:
            ly.forward_phase(L, L.PHASE_PRODUCT)
            ly.backward(L, L.PHASE_PRODUCT)
    launches = 3 * len(layers)
    ms = event_ms(torch, run, reps) / launches
    fl = flops / launches
    tf = fl / (ms * 1e-3) / 1e12
    del layers
    torch.cuda.empty_cache()
    return {"bound": "mfma", "kernel": "gemm_nt_persist_kernel<I8Mma, *> (int8 codes, 4-bit X two per byte in the backward "
                                       "products, int32 accumulators, 256 x 256 tiles on workgroups that stay)",
            "achieved": round(tf, 1), "peak": MFMA_PEAK_TFLOPS["int8"], "unit": "TFLOP/s",
            "frac": round(tf / MFMA_PEAK_TFLOPS["int8"], 4), "traffic": TRAFFIC_I8_PRODUCT_LLAMA,
            "launches": launches, "avg_launch_us": round(ms * 1e3, 2), "flop_per_launch": fl,
            "algorithmic_bytes_per_launch": alg_bytes / launches,
            "note": "mean over the nine product launches (Y, dW, dA of the 2048x2048, 5632x2048 and 2048x5632 layers at "
                    "65536 tokens) as the step issues them, on the operands its quantizers wrote; algorithmic bytes = "
                    "both operands once + the fp32 result once; the input-gradient launches carry the sum of the "
                    "weight gradient's contraction slices"}


def fused_prologue(L, synth, torch, reps):
    """Forward product with the SR quantizers inside the product kernel (sr_linear_fwd_fused: source
    tensors -> Eq. 1 -> LDS codes -> MFMA) against the quantize-once form (sr_linear_fwd with
    SRQ_FLAG_QUANTIZE_ONCE: one launch writes the codes, a second multiplies), int8, scales given:
    the small single layer, where the call selects the fused form, and the GPT-2 fc1 product, where
    every element would be rounded again by 24 (A) or 64 (W) tiles."""
    dev = "cuda:0"
    out = {}
    for name, (M, N, K) in (("single_layer_64x128x128", (64, 128, 128)), ("mid_128x128x768", (128, 128, 768)),
                            ("gpt2_fc1_8192x3072x768", (8192, 3072, 768))):
        A = synth.gaussian_torch((M, K), 1.0, 1, dev)
        W = synth.gaussian_torch((N, K), 0.02, 2, dev)
        sc = torch.empty(2, dtype=torch.float32, device=dev)
        L.sr_absmax_scale(A, L.INT8, out=sc[0:1])
        L.sr_absmax_scale(W, L.INT8, out=sc[1:2])
        qA, qW = L.Quant(L.INT8, sc[0:1], 0, 0), L.Quant(L.INT8, sc[1:2], 0, 1 << 24)
        qA_once = L.Quant(L.INT8, sc[0:1], 0, 0, flags=L.FLAG_QUANTIZE_ONCE)
        Y = torch.empty((M, N), dtype=torch.float32, device=dev)
        ws = torch.empty(L.sr_linear_workspace_bytes(L.OP_FWD, M, N, K) + 256, dtype=torch.uint8, device=dev)
        once = event_ms(torch, lambda: L.sr_linear_fwd(A, W, qA_once, qW, out=Y, workspace=ws), reps, warm_ms=5.0)
        fused = event_ms(torch, lambda: L.sr_linear_fwd_fused(A, W, qA, qW, out=Y), reps, warm_ms=5.0)
        out[name] = {"quantize_once_us": round(once * 1e3, 1), "fused_us": round(fused * 1e3, 1)}
    return out


def vendor_int8_context(torch, reps):
    """Context, not a target: the int8 x int8 -> int32 product of the ROCm BLAS library (through
    torch._int_mm) on the three forward-product shapes of the headline step, same box, same run."""
    dev = "cuda:0"
    out = {}
    for (P, Q, R) in ((TOKENS, 2048, 2048), (TOKENS, 5632, 2048), (TOKENS, 2048, 5632)):
        X = torch.randint(-127, 128, (P, R), dtype=torch.int8, device=dev)
        Zt = torch.randint(-127, 128, (Q, R), dtype=torch.int8, device=dev).t()
        try:
            ms = event_ms(torch, lambda: torch._int_mm(X, Zt), reps)
            out["%dx%dx%d" % (P, Q, R)] = {"us": round(ms * 1e3, 1), "TOP/s": round(2.0 * P * Q * R / ms / 1e9, 1)}
        except Exception as e:  # the routine is optional in a torch build
            out["%dx%dx%d" % (P, Q, R)] = {"error": repr(e)[:120]}
        del X, Zt
    torch.cuda.empty_cache()
    return out


def token_sweep(L, synth, torch):
    """The same linears at 4096 and 16384 tokens (whole layer step by HIP events) and, per token
    count incl. 65536, the batch-for-bits figure of Sec. 4.2 on the 2048 x 2048 layer: rms error of
    the mean gradient dW / T against the product of the unquantized tensors (binary64 on the device,
    256 rows of dW) with a 4-bit and with an 8-bit output gradient: it falls like 1 / sqrt(T) and
    scales with the step of the format."""
    out = {}
    shapes = (("qkvo", 2048, 2048), ("gate_up", 5632, 2048), ("down", 2048, 5632))
    for T in (4096, 16384, 65536):
        row = {}
        for name, N, K in shapes:
            if T == TOKENS and name != "qkvo":
                continue  # timed by the headline step
            ly = llama_layers(L, synth, torch, T, [(name, N, K)])[0]
            ms = event_ms(torch, lambda: ly.step(L), 10)
            row[name] = {"us": round(ms * 1e3, 1), "TFLOP/s": round(ly.flops() / ms / 1e9, 1)}
            if name == "qkvo":
                exact = ly.dY[:, :256].double().t() @ ly.A.double()
                err = {"int4": float((ly.dW[:256].double() - exact).pow(2).mean().sqrt()) / T}
                kinds8 = {k: L.INT8 for k in LLAMA_KINDS + ("dY_bwd",)}
                l8 = Layer(L, synth, torch, name, T, N, K, 7, kinds=kinds8, w_bf16=True)
                l8.step(L)
                err["int8"] = float((l8.dW[:256].double() - exact).pow(2).mean().sqrt()) / T
                row["rms_error_of_dW_over_T"] = {k: float("%.3g" % v) for k, v in err.items()}
                del l8, exact
            del ly
            torch.cuda.empty_cache()
        out["T%d" % T] = row
    return out


def gpt2_mlp(L, synth, torch, steps, warmup):
    """The GPT-2-small MLP linears (fc1 3072 x 768, fc2 768 x 3072) at 8192 tokens, int8 forward and
    E5M2 backward quantizers: step time from direct launches, the same step replayed from a HIP
    graph (stream positions on the device, advanced inside the graph), the entry-point split, and
    the product kernels alone."""
    shapes = synth.GPT2_SMALL_MLP
    res = {"workload": "fc1 (3072x768) + fc2 (768x3072), 8192 tokens, fp32 in/out, int8 SR forward, E5M2 SR backward"}
    flops = 2 * 6.0 * GPT2_TOKENS * 768 * 3072
    io_bytes = sum(4.0 * (3 * GPT2_TOKENS * K + 3 * N * K + 2 * GPT2_TOKENS * N) for _, N, K in shapes)
    res["flop_per_step"], res["min_hbm_bytes_per_step"] = flops, io_bytes
    res["composite_ceiling_TFLOP/s"] = round(flops / (io_bytes / (HBM_PEAK_GBS * 1e9)) / 1e12, 1)
    for label, flag in (("exact", 0), ("f8_pipeline", L.FLAG_F8_PIPELINE)):
        layers = [Layer(L, synth, torch, nm, GPT2_TOKENS, N, K, 100 + 10 * i, flag, stash=True) for i, (nm, N, K) in enumerate(shapes)]

        def step():
            for ly in layers:
                ly.step(L)
        sec = time_steps(torch, step, steps, warmup)
        res[label] = {"ms_per_step": round(sec * 1e3, 4), "TFLOP/s": round(flops / sec / 1e12, 1)}
        if label == "exact":
            def step_given_scales():
                for ly in layers:
                    ly.forward(L)
                    ly.backward(L)
            sec_gs = time_steps(torch, step_given_scales, steps, warmup)
            res["scales_given"] = {"ms_per_step": round(sec_gs * 1e3, 4), "TFLOP/s": round(flops / sec_gs / 1e12, 1)}
            # the same step recorded once and replayed: one graph launch per step instead of 14
            glayers = [Layer(L, synth, torch, nm, GPT2_TOKENS, N, K, 100 + 10 * i, flag, counters_dev=True, stash=True)
                       for i, (nm, N, K) in enumerate(shapes)]

            def gstep():
                for ly in glayers:
                    ly.step(L)
            g = torch.cuda.CUDAGraph()
            s = torch.cuda.Stream()
            s.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(s):
                gstep()
                torch.cuda.synchronize()
                g.capture_begin()
                gstep()
                g.capture_end()
            torch.cuda.synchronize()
            sec_g = time_steps(torch, g.replay, steps, warmup)
            res["graph"] = {"ms_per_step": round(sec_g * 1e3, 4), "TFLOP/s": round(flops / sec_g / 1e12, 1),
                            "note": "HIP graph of the whole step; stream positions live on the device and are "
                                    "advanced inside the graph, so every replay draws fresh thresholds"}
            del g, glayers
            res["phases"] = phase_times(L, torch, layers, max(5, steps // 2))
            res["product_kernels"] = gpt2_product_kernels(L, torch, layers, max(5, steps // 2))
        del layers
        torch.cuda.empty_cache()
    return res


def gpt2_product_kernels(L, torch, layers, reps):
    """The product kernels alone on the GPT-2 shapes, operands already quantized: the f16 pipeline
    fed from E5M2 codes (backward products), the int8 pipeline (forward products), the fp8
    pipeline (backward products with the flag set)."""
    dev = "cuda:0"
    out = {}

    def codes(P, R):
        return torch.randint(0, 120, (P, R), dtype=torch.uint8, device=dev)

    fwd_shapes = [(ly.M, ly.N, ly.K) for ly in layers]
    bwd_shapes = [s for ly in layers for s in ((ly.M, ly.K, ly.N), (ly.N, ly.K, ly.M))]
    for name, shapes, call, need_fn, peak in (
            ("f16", bwd_shapes, lambda X, Z, o, ws: L.sr_gemm_e5m2(X, Z, out=o, workspace=ws),
             L.raw.sr_gemm_e5m2_workspace_bytes, MFMA_PEAK_TFLOPS["fp16"]),
            ("int8", fwd_shapes, lambda X, Z, o, ws: L.sr_gemm_codes(X, L.INT8, Z, L.INT8, out=o, workspace=ws),
             L.raw.sr_gemm_workspace_bytes, MFMA_PEAK_TFLOPS["int8"]),
            ("fp8", bwd_shapes, lambda X, Z, o, ws: L.sr_gemm_codes(X, L.E5M2, Z, L.E5M2, out=o, workspace=ws),
             L.raw.sr_gemm_workspace_bytes, MFMA_PEAK_TFLOPS["fp8"])):
        calls, flops = [], 0.0
        for (P, Q, R) in shapes:
            need = need_fn(P, Q, R)
            calls.append((codes(P, R), codes(Q, R), torch.empty((P, Q), dtype=torch.float32, device=dev),
                          torch.empty(max(need, 16), dtype=torch.uint8, device=dev)))
            flops += 2.0 * P * Q * R

        def run():
            for X, Z, o, ws in calls:
                call(X, Z, o, ws)
        ms = event_ms(torch, run, reps) / len(calls)
        fl = flops / len(calls)
        tf = fl / (ms * 1e-3) / 1e12
        out[name] = {"launches": len(calls), "avg_launch_us": round(ms * 1e3, 2), "flop_per_launch": fl,
                     "TFLOP/s": round(tf, 1), "peak": peak, "frac": round(tf / peak, 4)}
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
    nbytes = sum(ly.A.numel() * ly.A.element_size() + ly.W.numel() * ly.W.element_size() + 4 * ly.dY.numel()
                 for ly in layers)
    res["absmax_GB/s"] = round(nbytes / (res["absmax_us"] * 1e-6) / 1e9, 1)
    return res


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


def train_step_times(torch, steps=2):
    """Whole training step of the 12-layer decoder (d = 768, 12 heads, vocabulary 32000, 1024
    tokens per sequence, random weights and token ids): forward, backward and the updates, every
    linear through the SR-quantized path (int8 forward, E5M2 backward quantizers), weights in
    bfloat16 updated by Eq. 10; batch 8, 32 and 128 (the last as 4 micro-batches of 32)."""
    from paper_2511_00874_amd import train
    model = train.Decoder()
    out = {"model": "decoder 12 x 768, 12 heads, vocab 32000, seq 1024; %.1f M weights in SR linears"
                    % (sum(m.in_features * m.out_features for m in model.sr_linears()) / 1e6)}
    for b, micro in ((8, 1), (32, 1), (128, 4)):
        ids = torch.randint(0, 32000, (b, 1024), device="cuda:0")
        tgt = torch.roll(ids, -1, 1)
        train.train_step(model, ids, tgt, 1e-3, micro)
        sec = time_steps(torch, lambda: train.train_step(model, ids, tgt, 1e-3, micro), steps, 0)
        out["b%d" % b] = {"ms_per_step": round(sec * 1e3, 2), "micro_batches": micro,
                          "sr_linear_TFLOP/s": round(train.flops_per_token(model) * b * 1024 / sec / 1e12, 1)}
    del model
    torch.cuda.empty_cache()
    return out


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline():
    """The CPU oracle, as it stands, on a bounded sample of the headline workload: the 2048 x 2048
    linear with bfloat16 weights, 8-bit quantizers and a 4-bit output gradient; per run the five
    absmax scales, the quantizations Alg. 1 / Alg. 2 state (each product quantizes its two
    operands) of the full tensors at `T` tokens, then `n_out` sampled entries of each of Y, dA, dW.
    Once on all host threads and once, on a smaller sample, on a single thread."""
    import numpy as np

    import oracle
    from paper_2511_00874_amd import synth
    N = K = 2048

    def run(T, n_out):
        A, W, dY = synth.single_layer(T, N, K, seed=0, std_dy=1e-3)
        Wb = synth.to_bf16_bits(W)
        t0 = time.perf_counter()
        q, off = {}, 0
        for qn, x, kind in (("A_fwd", A, oracle.INT8), ("W_fwd", Wb, oracle.INT8), ("A_bwd", A, oracle.INT8),
                            ("W_bwd", Wb, oracle.INT8), ("dY_bwd", dY, oracle.INT4)):
            q[qn] = oracle.Quant(kind, oracle.absmax_scale(x, kind), 0, off)
            off += (x.size + 7) // 8
        rng = np.random.default_rng(0)
        oracle.linear_fwd(A, Wb, q["A_fwd"], q["W_fwd"], at=rng.integers(0, T * N, n_out).astype(np.uint64))
        oracle.linear_bwd_data(dY, Wb, q["dY_bwd"], q["W_bwd"], at=rng.integers(0, T * K, n_out).astype(np.uint64))
        oracle.linear_bwd_weight(dY, A, q["dY_bwd"], q["A_bwd"], at=rng.integers(0, N * K, n_out).astype(np.uint64))
        dt = time.perf_counter() - t0
        flops = 2.0 * n_out * (K + N + T)
        return flops / dt / 1e12, dt, flops

    threads = oracle.threads()
    v_all, dt_all, fl_all = run(16384, 1 << 21)
    oracle.set_threads(1)
    v_one, dt_one, fl_one = run(1024, 1 << 18)
    oracle.set_threads(threads)
    return {"value": round(v_all, 6), "unit": "TFLOP/s", "cores": threads, "kind": "oracle", "cpu_model": cpu_model(),
            "sample": f"2048x2048 linear (bf16 W, int8 quantizers, int4 dY) at 16384 tokens: 5 absmax + the 6 "
                      f"quantizations of the full tensors, then 3 x {1 << 21} sampled entries of Y/dA/dW; "
                      f"{fl_all / 1e9:.1f} GFLOP of products in {dt_all:.1f} s wall",
            "single_thread": {"value": round(v_one, 6), "unit": "TFLOP/s", "cores": 1,
                              "sample": f"the same at 1024 tokens with 3 x {1 << 18} sampled entries; "
                                        f"{fl_one / 1e9:.1f} GFLOP of products in {dt_one:.1f} s wall"}}


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

    def calibrate_copy():
        # a plain device copy of 2^28 floats: 1 GiB read, 1 GiB written
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    if args.only:
        if args.only == "gpt2":
            out = {"gpt2_mlp": gpt2_mlp(L, synth, torch, args.steps, args.warmup)}
        elif args.only == "fused":
            out = {"fused_prologue": fused_prologue(L, synth, torch, 50)}
        elif args.only == "quantizer":
            out = {"sr_quantize": quantizer_sweep(L, synth, torch, max(5, args.steps // 5))}
        elif args.only == "products":
            out = {"roofline": llama_products_roofline(L, synth, torch, max(5, args.steps // 2))}
        elif args.only == "step":
            # the headline step alone: warm-up + steps on two streams, then the same in one stream
            layers = llama_layers(L, synth, torch, TOKENS, synth.LLAMA_1B_LINEARS)
            two = TwoStreamStep(torch, L, layers)

            def one():
                for ly in layers:
                    ly.step(L)
            flops = sum(ly.flops() for ly in layers)
            out = {}
            for name, fn in (("two_streams", two), ("single_stream", one)):
                sec = time_steps(torch, fn, args.steps, args.warmup)
                out[name] = {"ms_per_step": round(sec * 1e3, 4), "TFLOP/s": round(flops / sec / 1e12, 1)}
        else:
            print("unknown section " + args.only, file=sys.stderr)
            sys.exit(2)
        if args.calibrate_copy:
            calibrate_copy()
        print(json.dumps(out))
        return

    layers = llama_layers(L, synth, torch, TOKENS, synth.LLAMA_1B_LINEARS)

    def step_one_stream():
        for ly in layers:
            ly.step(L)
    # the step: every launch of the seven linears, the memory-bound half on one stream and the products
    # on another (same launches, same arguments, same results as in a single stream)
    step = TwoStreamStep(torch, L, layers)
    sec = time_steps(torch, step, args.steps, args.warmup)
    sec_one = time_steps(torch, step_one_stream, args.steps, args.warmup)
    flops = sum(ly.flops() for ly in layers)
    io_bytes = sum(ly.min_hbm_bytes() for ly in layers)
    tflops = flops / sec / 1e12
    per_shape = {}
    for name, idx in (("qkvo_2048x2048", 0), ("gate_up_5632x2048", 4), ("down_2048x5632", 6)):
        ms = event_ms(torch, lambda: layers[idx].step(L), 5)
        per_shape[name] = {"us": round(ms * 1e3, 1), "TFLOP/s": round(layers[idx].flops() / ms / 1e9, 1)}
    phases = phase_times(L, torch, layers, 5)
    del layers
    torch.cuda.empty_cache()

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
        "dtype": "int8 (int4 values for dY), int32 accumulators",
        "data": "synthetic",
        "config": {"workload": "configs[3] at 65536 tokens: the seven linears of one Llama-1B-shaped decoder layer "
                               "(q, k, v, o 2048x2048; gate, up 5632x2048; down 2048x5632), bf16 master weights, "
                               "fp32 activations and gradients in and out, int4 SR on the output gradient and int8 SR "
                               "on the other four quantizers; per linear 5 absmax scales, 5 quantizers, 3 products",
                   "tokens": TOKENS, "flop_per_step": flops, "min_hbm_bytes_per_step": io_bytes},
        "frac_of_8bit_mfma_peak": round(tflops / MFMA_PEAK_TFLOPS["int8"], 4),
        # the path's own ceiling: every tensor in once per quantizer pass and every result out once
        # at HBM peak, or the 8-bit MFMA peak, whichever is lower
        "composite_ceiling_TFLOP/s": round(min(MFMA_PEAK_TFLOPS["int8"],
                                               flops / (io_bytes / (HBM_PEAK_GBS * 1e9)) / 1e12), 1),
        "streams": "2: absmax and operand quantizers on one stream, products on the other (events carry the "
                   "dependencies); the kernels of the two streams share the CUs",
        "single_stream": {"ms_per_step": round(sec_one * 1e3, 4), "TFLOP/s": round(flops / sec_one / 1e12, 1)},
        "per_shape": per_shape,
        "phases": phases,
    }
    line["roofline"] = llama_products_roofline(L, synth, torch, max(5, args.steps // 2))
    if not args.no_extras:
        line["token_sweep"] = token_sweep(L, synth, torch)
        line["gpt2_mlp"] = gpt2_mlp(L, synth, torch, args.steps, args.warmup)
        qs = quantizer_sweep(L, synth, torch, max(5, args.steps // 5))
        line["sr_quantize"] = qs
        line["roofline_quantizer"] = {"bound": "hbm", "kernel": "quantize_flat_f32_kernel<INT8, SR, byte> on 2^28 elements (5 B per element)",
                                      "achieved": qs["int8"]["GB/s"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                      "frac": qs["int8"]["frac_of_hbm_peak"], "traffic": round(TRAFFIC_QUANTIZE_INT8_2P28)}
        line["fused_prologue"] = fused_prologue(L, synth, torch, 50)
        line["vendor_int8_gemm_context"] = vendor_int8_context(torch, 5)
        line["train_step"] = train_step_times(torch)
    if args.calibrate_copy:
        calibrate_copy()
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline()
    print(json.dumps(line))


if __name__ == "__main__":
    main()
