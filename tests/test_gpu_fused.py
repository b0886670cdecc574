"""GPU parity of the forward product with the quantizers inside it (sr_linear_fwd_fused): against the
oracle, and against the quantize-once path (sr_linear_fwd), whose codes it must reproduce."""
import numpy as np
import pytest
import torch

import oracle
from paper_2511_00874_amd import lib as L
from paper_2511_00874_amd import synth
from gpu_util import check_product, host_src, say, to_dev

pytestmark = pytest.mark.gpu


def _pair(A, W, kA, kW, seed, mode=L.SR, offs=(0, 1 << 20)):
    out = []
    for t, kind, off in ((A, kA, offs[0]), (W, kW, offs[1])):
        scale = oracle.absmax_scale(host_src(t), kind)
        out.append((L.Quant(kind, scale, seed, off, round_mode=mode), oracle.Quant(kind, scale, seed, off, round_mode=mode)))
    return out


def _check(A, W, qA, qW, sample=None, exact=True):
    M, N = A.shape[0], W.shape[0]
    got_t = L.sr_linear_fwd_fused(A, W, qA[0], qW[0])
    # the quantize-once form, also for the small layers that sr_linear_fwd would round in the product
    keep = L.Quant(qA[0].kind, qA[0].scale, qA[0].seed, qA[0].counter_offset, qA[0].round_mode, L.FLAG_QUANTIZE_ONCE)
    once = L.sr_linear_fwd(A, W, keep, qW[0])
    assert torch.equal(once, L.sr_linear_fwd(A, W, qA[0], qW[0]))   # whichever form that call takes
    got = got_t.cpu().numpy().reshape(-1)
    if sample is None:
        ref, ab = oracle.linear_fwd(host_src(A), host_src(W), qA[1], qW[1], want_abs=True)
        pick = slice(None)
    else:
        rng = np.random.default_rng(7)
        idx = np.concatenate([rng.integers(0, M * N, size=sample).astype(np.uint64),
                              np.array([0, N - 1, (M - 1) * N, M * N - 1], dtype=np.uint64)])
        ref, ab = oracle.linear_fwd(host_src(A), host_src(W), qA[1], qW[1], want_abs=True, at=idx)
        pick = idx.astype(np.int64)
    check_product(got[pick], ref, ab, "fused vs oracle")
    if exact:
        # integer codes, int32 sums, one scaling: equal to the quantize-once path bit for bit, which
        # is to say every code rounded inside the product equals the one sr_quantize writes
        assert torch.equal(got_t, once)
    else:
        assert float((got_t - once).abs().max()) <= 1e-5 * float(once.abs().max())


def test_single_layer_int8():
    # the small CPU-checkable layer: 64 x 128 activations, 128 x 128 weights, seed 0
    A, W, _ = synth.single_layer()
    A, W = to_dev(A), to_dev(W)
    qA, qW = _pair(A, W, L.INT8, L.INT8, seed=0, offs=(0, 1024))
    _check(A, W, qA, qW)
    # int32 accumulators themselves: with unit scales the result is the integer product of the codes
    one = (L.Quant(L.INT8, 1.0, 0, 0), L.Quant(L.INT8, 1.0, 0, 1024))
    Ai, Wi = (A * 40).contiguous(), (W * 2000).contiguous()
    got = L.sr_linear_fwd_fused(Ai, Wi, *one).cpu().numpy()
    cA = oracle.quantize(host_src(Ai), L.INT8, 1.0, 0, 0).view(np.int8).astype(np.int64)
    cW = oracle.quantize(host_src(Wi), L.INT8, 1.0, 0, 1024).view(np.int8).astype(np.int64)
    assert np.array_equal(got.astype(np.int64), cA @ cW.T)


@pytest.mark.parametrize("kA,kW,exact", [(L.INT8, L.INT8, True), (L.INT4, L.INT8, True), (L.INT8, L.INT4, True),
                                         (L.E5M2, L.E5M2, False)])
@pytest.mark.parametrize("mode", [L.SR, L.RTN])
@pytest.mark.parametrize("w_bf16", [False, True])
def test_ragged_shapes_formats_sources(kA, kW, exact, mode, w_bf16):
    # several 64-wide tiles with ragged edges in both output dimensions, a contraction that ends inside
    # a 128-byte stage, binary32 and bfloat16 sources, both rounding modes
    M, N, K = 272, 144, 208
    say("fused", L.KIND_NAMES[kA], L.KIND_NAMES[kW], mode, w_bf16)
    A, W, _ = synth.single_layer(M, N, K, 3)
    A, W = to_dev(A), to_dev(W, w_bf16)
    qA, qW = _pair(A, W, kA, kW, seed=5, mode=mode)
    _check(A, W, qA, qW, exact=exact)


def test_specials_and_saturation_go_through_the_same_rule():
    # NaN / Inf / values beyond the scale inside a tile: same codes as the standalone quantizer
    M, N, K = 64, 64, 128
    A, W, _ = synth.single_layer(M, N, K, 11)
    A[3, 5], A[10, 100], A[63, 127], A[0, 0] = np.inf, -np.inf, 1e30, -0.0
    A, W = to_dev(A), to_dev(W)
    qA = (L.Quant(L.INT8, 0.01, 9, 0), oracle.Quant(L.INT8, 0.01, 9, 0))
    qW = (L.Quant(L.INT8, 0.001, 9, 4096), oracle.Quant(L.INT8, 0.001, 9, 4096))
    assert torch.equal(L.sr_linear_fwd_fused(A, W, qA[0], qW[0]), L.sr_linear_fwd(A, W, qA[0], qW[0]))
    ref = oracle.linear_fwd(host_src(A), host_src(W), qA[1], qW[1])
    assert np.array_equal(L.sr_linear_fwd_fused(A, W, qA[0], qW[0]).cpu().numpy(), ref.astype(np.float32))


def test_many_tiles_large_tile_kernel_sampled():
    # more than 1024 tiles of 64 x 64: the 128 x 128 form, ragged in both dimensions
    M, N, K = 2320, 2064, 144
    A, W, _ = synth.single_layer(M, N, K, 13)
    A, W = to_dev(A), to_dev(W, True)
    qA, qW = _pair(A, W, L.INT8, L.INT8, seed=2)
    _check(A, W, qA, qW, sample=20000)


def test_device_resident_scale_and_counter():
    # scales and stream positions read on the device, as a captured step passes them
    M, N, K = 64, 128, 128
    A, W, _ = synth.single_layer()
    A, W = to_dev(A), to_dev(W)
    sc = torch.tensor([oracle.absmax_scale(host_src(A), L.INT8), oracle.absmax_scale(host_src(W), L.INT8)],
                      dtype=torch.float32, device=A.device)
    ctr = torch.tensor([77, 5000], dtype=torch.int64, device=A.device)
    qA = L.Quant(L.INT8, sc[0:1], 4, ctr[0:1])
    qW = L.Quant(L.INT8, sc[1:2], 4, ctr[1:2])
    got = L.sr_linear_fwd_fused(A, W, qA, qW)
    ref = L.sr_linear_fwd_fused(A, W, L.Quant(L.INT8, float(sc[0]), 4, 77), L.Quant(L.INT8, float(sc[1]), 4, 5000))
    assert torch.equal(got, ref)
    assert torch.equal(got, L.sr_linear_fwd(A, W, qA, qW))


def test_unsupported_pairs_are_refused():
    A, W, _ = synth.single_layer()
    A, W = to_dev(A), to_dev(W)
    for kA, kW in ((L.E4M3, L.E4M3), (L.INT8, L.E5M2), (L.E5M2, L.E4M3)):
        with pytest.raises(L.SrqError) as e:
            L.sr_linear_fwd_fused(A, W, L.Quant(kA, 1.0), L.Quant(kW, 1.0))
        assert e.value.status == -6


# ---- the two halves of the linear calls as calls of their own (sr_linear_fwd_phase / sr_linear_bwd_phase) ----

@pytest.mark.parametrize("kinds", [(L.INT8, L.INT8, L.INT4), (L.E5M2, L.E5M2, L.E5M2), (L.E4M3, L.E4M3, L.E5M2)])
def test_phase_calls_equal_the_whole_call(kinds):
    # quantize half on one stream, product half on another, ordered by an event: same results bit for bit
    kA, kW, kdY = kinds
    M, N, K = 528, 272, 400
    A, W, dY = synth.single_layer(M, N, K, 31, std_dy=1e-3)
    A, W, dY = to_dev(A), to_dev(W, True), to_dev(dY)
    q = {}
    off = 0
    for name, t, kind in (("A_fwd", A, kA), ("W_fwd", W, kW), ("dY", dY, kdY), ("W_bwd", W, kW), ("A_bwd", A, kA)):
        q[name] = L.Quant(kind, oracle.absmax_scale(host_src(t), kind), 8, off)
        off += (t.numel() + 7) // 8
    Y = L.sr_linear_fwd(A, W, q["A_fwd"], q["W_fwd"])
    dA, dW = L.sr_linear_bwd(dY, W, A, q["dY"], q["W_bwd"], q["A_bwd"])
    ws_f = torch.empty(L.sr_linear_workspace_bytes(L.OP_FWD, M, N, K), dtype=torch.uint8, device=A.device)
    ws_b = torch.empty(L.sr_linear_workspace_bytes(L.OP_BWD, M, N, K), dtype=torch.uint8, device=A.device)
    Y2, dA2, dW2 = torch.zeros_like(Y), torch.zeros_like(dA), torch.full_like(dW, 1.0)
    mem, mat = torch.cuda.Stream(), torch.cuda.Stream()
    ev_f, ev_b = torch.cuda.Event(), torch.cuda.Event()
    cur = torch.cuda.current_stream()
    mem.wait_stream(cur)
    mat.wait_stream(cur)
    with torch.cuda.stream(mem):
        L.sr_linear_fwd(A, W, q["A_fwd"], q["W_fwd"], out=Y2, workspace=ws_f, phase=L.PHASE_QUANTIZE)
        ev_f.record()
        L.sr_linear_bwd(dY, W, A, q["dY"], q["W_bwd"], q["A_bwd"], out_dA=dA2, out_dW=dW2, workspace=ws_b,
                        phase=L.PHASE_QUANTIZE)
        ev_b.record()
    with torch.cuda.stream(mat):
        mat.wait_event(ev_f)
        L.sr_linear_fwd(A, W, q["A_fwd"], q["W_fwd"], out=Y2, workspace=ws_f, phase=L.PHASE_PRODUCT)
        mat.wait_event(ev_b)
        L.sr_linear_bwd(dY, W, A, q["dY"], q["W_bwd"], q["A_bwd"], out_dA=dA2, out_dW=dW2, workspace=ws_b,
                        phase=L.PHASE_PRODUCT)
    cur.wait_stream(mem)
    cur.wait_stream(mat)
    torch.cuda.synchronize()
    assert torch.equal(Y, Y2) and torch.equal(dA, dA2) and torch.equal(dW, dW2)
    # the product half accumulates onto dW with beta = 1 as the whole call does
    L.sr_linear_bwd(dY, W, A, q["dY"], q["W_bwd"], q["A_bwd"], out_dA=dA2, out_dW=dW2, beta=1.0, workspace=ws_b,
                    phase=L.PHASE_PRODUCT)
    assert torch.equal(dW2, dW + dW)
    # PHASE_BOTH through the phase entry point; an unknown phase; the weight-only objective
    Y3 = torch.zeros_like(Y)
    L.sr_linear_fwd(A, W, q["A_fwd"], q["W_fwd"], out=Y3, workspace=ws_f, phase=L.PHASE_BOTH)
    assert torch.equal(Y, Y3)
    with pytest.raises(L.SrqError) as e:
        L.sr_linear_fwd(A, W, q["A_fwd"], q["W_fwd"], out=Y3, workspace=ws_f, phase=7)
    assert e.value.status == -3
    with pytest.raises(L.SrqError) as e:
        L.sr_linear_fwd(A, W, L.Quant(L.NONE, 1.0), q["W_fwd"], out=Y3, workspace=ws_f, phase=L.PHASE_PRODUCT)
    assert e.value.status == -6


@pytest.mark.parametrize("kinds", [(L.INT8, L.INT4), (L.E5M2, L.E5M2), (L.E4M3, L.E5M2)])
def test_phase_calls_with_the_stash_equal_the_whole_calls(kinds):
    # forward that also rounds the backward operands of A and W (read once), backward from that stash: in
    # halves on two streams, against sr_linear_fwd / sr_linear_bwd with the same five quantizers
    kb, kdY = kinds
    M, N, K = 528, 272, 400
    A, W, dY = synth.single_layer(M, N, K, 37, std_dy=1e-3)
    A, W, dY = to_dev(A), to_dev(W, True), to_dev(dY)
    q, off = {}, 0
    for name, t, kind in (("A_fwd", A, L.INT8), ("W_fwd", W, L.INT8), ("dY", dY, kdY), ("W_bwd", W, kb), ("A_bwd", A, kb)):
        q[name] = L.Quant(kind, oracle.absmax_scale(host_src(t), kind), 12, off)
        off += (t.numel() + 7) // 8
    Y = L.sr_linear_fwd(A, W, q["A_fwd"], q["W_fwd"])
    dA, dW = L.sr_linear_bwd(dY, W, A, q["dY"], q["W_bwd"], q["A_bwd"])
    dev = A.device
    stash = torch.empty(L.sr_linear_stash_bytes(M, N, K), dtype=torch.uint8, device=dev)
    ws_f = torch.empty(L.sr_linear_workspace_bytes(L.OP_FWD_STASH, M, N, K), dtype=torch.uint8, device=dev)
    ws_b = torch.empty(L.sr_linear_workspace_bytes(L.OP_BWD_STASHED, M, N, K), dtype=torch.uint8, device=dev)
    Y2, dA2, dW2 = torch.zeros_like(Y), torch.zeros_like(dA), torch.full_like(dW, 1.0)
    fwd = dict(stash=stash, out=Y2, workspace=ws_f)
    bwd = dict(out_dA=dA2, out_dW=dW2, workspace=ws_b)
    mem, mat = torch.cuda.Stream(), torch.cuda.Stream()
    ev_f, ev_b = torch.cuda.Event(), torch.cuda.Event()
    cur = torch.cuda.current_stream()
    mem.wait_stream(cur)
    mat.wait_stream(cur)
    with torch.cuda.stream(mem):
        L.sr_linear_fwd_stash(A, W, q["A_fwd"], q["W_fwd"], q["A_bwd"], q["W_bwd"], phase=L.PHASE_QUANTIZE, **fwd)
        ev_f.record()
        L.sr_linear_bwd_stashed(dY, stash, K, q["dY"], q["W_bwd"], q["A_bwd"], phase=L.PHASE_QUANTIZE, **bwd)
        ev_b.record()
    with torch.cuda.stream(mat):
        mat.wait_event(ev_f)
        L.sr_linear_fwd_stash(A, W, q["A_fwd"], q["W_fwd"], q["A_bwd"], q["W_bwd"], phase=L.PHASE_PRODUCT, **fwd)
        mat.wait_event(ev_b)
        L.sr_linear_bwd_stashed(dY, stash, K, q["dY"], q["W_bwd"], q["A_bwd"], phase=L.PHASE_PRODUCT, **bwd)
    cur.wait_stream(mem)
    cur.wait_stream(mat)
    torch.cuda.synchronize()
    assert torch.equal(Y, Y2) and torch.equal(dA, dA2) and torch.equal(dW, dW2)
    L.sr_linear_bwd_stashed(dY, stash, K, q["dY"], q["W_bwd"], q["A_bwd"], beta=1.0, phase=L.PHASE_PRODUCT, **bwd)
    assert torch.equal(dW2, dW + dW)
    with pytest.raises(L.SrqError) as e:
        L.sr_linear_bwd_stashed(dY, stash, K, q["dY"], q["W_bwd"], q["A_bwd"], phase=0, **bwd)
    assert e.value.status == -3
    with pytest.raises(L.SrqError) as e:
        L.sr_linear_fwd_stash(A, W, q["A_fwd"], q["W_fwd"], q["A_bwd"], q["W_bwd"], phase=4, **fwd)
    assert e.value.status == -3
