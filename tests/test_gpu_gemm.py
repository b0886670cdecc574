"""GPU parity of the code-matrix product and the three linear entry points against the oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2511_00874_amd import lib as L
from paper_2511_00874_amd import synth
from gpu_util import (DEV, check_product, check_product_f8_pipeline, group_max_sum, host_src, say,
                      to_dev)

pytestmark = pytest.mark.gpu

PAIRS = [(L.INT8, L.INT8), (L.INT4, L.INT8), (L.E4M3, L.E4M3), (L.E4M3, L.E5M2), (L.E5M2, L.E4M3),
         (L.E5M2, L.E5M2), (L.E4M2, L.E5M2), (L.E4M0, L.E4M1)]


def _rand_codes(shape, kind, seed):
    rng = np.random.default_rng(seed)
    if kind == L.INT8:
        return rng.integers(-127, 128, size=shape).astype(np.int8).view(np.uint8)
    if kind == L.INT4:
        return rng.integers(-7, 8, size=shape).astype(np.int8).view(np.uint8)
    c = rng.integers(0, 256, size=shape).astype(np.uint8)
    c &= {L.E4M2: 0xFE, L.E4M1: 0xFC, L.E4M0: 0xF8}.get(kind, 0xFF)   # sub-grids of E4M3: low fraction bits zero
    bad = ~np.isfinite(oracle.decode_array(kind, c))   # NaN / Inf codes never come out of the quantizer
    c[bad] = 0x30
    return c


# shapes chosen to hit: the 64-tile kernel with ragged edges; a contraction that is not a
# multiple of the 128-byte stage; the 128-tile kernel; the split contraction
SHAPES = [(64, 128, 128), (70, 90, 48), (33, 1, 16), (200, 136, 272), (1040, 1100, 400), (256, 192, 8192)]


@pytest.mark.parametrize("kx,kz", PAIRS)
@pytest.mark.parametrize("P,Q,R", SHAPES)
def test_gemm_codes_matches_oracle(kx, kz, P, Q, R):
    say("gemm", L.KIND_NAMES[kx], L.KIND_NAMES[kz], P, Q, R)
    X, Z = _rand_codes((P, R), kx, 1), _rand_codes((Q, R), kz, 2)
    got = L.sr_gemm_codes(to_dev(X), kx, to_dev(Z), kz, alpha=0.25).cpu().numpy()
    ref, ab = oracle.gemm_fwd(X, kx, 0.5, Z, kz, 0.5, want_abs=True)
    if kx in (L.INT8, L.INT4):
        assert np.array_equal(got, ref)     # int32 accumulation is exact, 0.25 scaling too
    elif P * Q * R <= 200 * 136 * 272:
        # one-byte float codes run on the fp8 pipeline: hardware-truncated group sums
        gms = group_max_sum(oracle.decode_array(kx, X), oracle.decode_array(kz, Z), 0.25)
        check_product_f8_pipeline(got, ref, gms, ab, (kx, kz, P, Q, R))
    else:
        assert np.abs(got - ref).max() <= 7 * 2.0**-13 * ab.max()


def test_gemm_large_tiles_sampled():
    # enough tiles for the 256 x 256 kernel; checked on sampled entries
    P, Q, R = 4096, 3840, 384
    rng = np.random.default_rng(0)
    idx = rng.integers(0, P * Q, size=20000).astype(np.uint64)
    edge = np.array([0, Q - 1, (P - 1) * Q, P * Q - 1, 255 * Q + 255, 256 * Q + 256], dtype=np.uint64)
    idx = np.concatenate([idx, edge])
    for kx, kz in ((L.INT8, L.INT8), (L.E5M2, L.E4M3)):
        say("gemm-large", L.KIND_NAMES[kx], L.KIND_NAMES[kz])
        X, Z = _rand_codes((P, R), kx, 3), _rand_codes((Q, R), kz, 4)
        got = L.sr_gemm_codes(to_dev(X), kx, to_dev(Z), kz).cpu().numpy().reshape(-1)[idx.astype(np.int64)]
        ref, ab = oracle.gemm_fwd(X, kx, 1.0, Z, kz, 1.0, want_abs=True, at=idx)
        if kx == L.INT8:
            assert np.array_equal(got, ref)
        else:
            assert np.all(np.abs(got - ref) <= 7 * 2.0**-13 * ab)


def test_gemm_bf16_exact_products_binary32_sums():
    # bfloat16 operands holding 8-bit float grid values: the exact path of the linear entry points
    P, Q, R = 200, 136, 272
    X, Z = _rand_codes((P, R), L.E4M3, 7), _rand_codes((Q, R), L.E5M2, 8)
    Xv, Zv = oracle.decode_array(L.E4M3, X), oracle.decode_array(L.E5M2, Z)
    got = L.sr_gemm_bf16(torch.from_numpy(Xv).to(DEV).to(torch.bfloat16), torch.from_numpy(Zv).to(DEV).to(torch.bfloat16),
                         alpha=0.25).cpu().numpy()
    ref, ab = oracle.gemm_fwd(X, L.E4M3, 0.5, Z, L.E5M2, 0.5, want_abs=True)
    check_product(got, ref, ab)


@pytest.mark.parametrize("P,Q,R", [(200, 136, 272), (70, 90, 48), (33, 1, 16), (1040, 1100, 400), (256, 192, 8192)])
def test_gemm_e5m2_from_codes_is_exact_like_the_bf16_form(P, Q, R):
    # every finite E5M2 code, subnormals included: the codes widened in registers must give what
    # the same values give as bfloat16 operands (same exact products; the binary32 sums may
    # differ in the last bits, the two pipelines group the contraction differently)
    say("gemm e5m2 codes", P, Q, R)
    X, Z = _rand_codes((P, R), L.E5M2, 17), _rand_codes((Q, R), L.E5M2, 18)
    X[0, :16] = [0x00, 0x01, 0x02, 0x03, 0x04, 0x7B, 0xFB, 0x80, 0x81, 0x83, 0x84, 0x3C, 0xBC, 0x7A, 0x05, 0x40]
    got = L.sr_gemm_e5m2(to_dev(X), to_dev(Z), alpha=0.25).cpu().numpy()
    ref, ab = oracle.gemm_fwd(X, L.E5M2, 0.5, Z, L.E5M2, 0.5, want_abs=True)
    check_product(got, ref, ab)
    Xv, Zv = oracle.decode_array(L.E5M2, X), oracle.decode_array(L.E5M2, Z)
    same = L.sr_gemm_bf16(torch.from_numpy(Xv).to(DEV).to(torch.bfloat16), torch.from_numpy(Zv).to(DEV).to(torch.bfloat16),
                          alpha=0.25).cpu().numpy()
    assert np.all(np.abs(got - same) <= 2e-6 * ab)


def test_fp8_pipeline_aligns_groups_of_eight_products_to_14_bits():
    # What the hardware does, pinned: in E4M3, 256 * 256 = 2^16 next to 1 * 1 inside one run of 8
    # contraction indices loses the 1 (bits below 2^(16-13) are dropped); in the next run of 8 it
    # is kept.  Operands widened to bfloat16 multiply exactly either way.
    big, one = 0x78, 0x38   # E4M3 codes of 256 and 1
    for pos, want_fp8 in ((1, 65536.0), (7, 65536.0), (8, 65537.0), (15, 65537.0)):
        X = np.zeros((16, 16), dtype=np.uint8)
        X[0, 0], X[0, pos] = big, one
        got = L.sr_gemm_codes(to_dev(X), L.E4M3, to_dev(X), L.E4M3).cpu().numpy()[0, 0]
        assert got == want_fp8, (pos, got)
        Xv = torch.from_numpy(oracle.decode_array(L.E4M3, X)).to(DEV).to(torch.bfloat16)
        assert L.sr_gemm_bf16(Xv, Xv).cpu().numpy()[0, 0] == 65537.0
    # 2^16 + 2^3 is the smallest kept companion: 14 bits
    X = np.zeros((16, 16), dtype=np.uint8)
    X[0, 0], X[0, 1] = big, 0x50   # 8 = 2^3
    Z = X.copy()
    Z[0, 1] = one
    assert L.sr_gemm_codes(to_dev(X), L.E4M3, to_dev(Z), L.E4M3).cpu().numpy()[0, 0] == 65544.0
    X[0, 1] = 0x48                 # 4 = 2^2: dropped
    assert L.sr_gemm_codes(to_dev(X), L.E4M3, to_dev(Z), L.E4M3).cpu().numpy()[0, 0] == 65536.0


def test_gemm_accumulate_beta_one():
    P, Q, R = 96, 80, 256
    X, Z = _rand_codes((P, R), L.INT8, 5), _rand_codes((Q, R), L.INT8, 6)
    out = torch.full((P, Q), 3.0, device=DEV)
    L.sr_gemm_codes(to_dev(X), L.INT8, to_dev(Z), L.INT8, out=out, beta=1.0)
    ref = oracle.gemm_fwd(X, L.INT8, 1.0, Z, L.INT8, 1.0)
    assert np.array_equal(out.cpu().numpy(), ref + np.float32(3.0))


# ---- the linear entry points -----------------------------------------------------------------

def _quants(kinds, tensors, seed, flags=0):
    """Five quantizers with absmax scales and running block offsets; returns (lib, oracle) pairs."""
    out, off = {}, 0
    for name, kind in kinds.items():
        t = tensors[name.split("_")[0]]
        scale = oracle.absmax_scale(host_src(t), kind)
        out[name] = (L.Quant(kind, scale, seed, off, flags=flags), oracle.Quant(kind, scale, seed, off))
        off += (t.numel() + 7) // 8
    return out


def _layer(M, N, K, seed, std_dy=1.0, w_bf16=False):
    A, W, dY = synth.single_layer(M, N, K, seed, std_dy=std_dy)
    return {"A": to_dev(A), "W": to_dev(W, w_bf16), "dY": to_dev(dY)}


def _run_layer(t, q, sample=None, beta_check=False, f8_pipeline=False):
    M, K = t["A"].shape
    N = t["W"].shape[0]
    hA, hW, hdY = host_src(t["A"]), host_src(t["W"]), host_src(t["dY"])
    for name, fn, ofn, args, oargs, size in (
            ("fwd", L.sr_linear_fwd, oracle.linear_fwd, (t["A"], t["W"], q["A_fwd"][0], q["W_fwd"][0]),
             (hA, hW, q["A_fwd"][1], q["W_fwd"][1]), M * N),
            ("bwd_data", L.sr_linear_bwd_data, oracle.linear_bwd_data,
             (t["dY"], t["W"], q["dY_bwd"][0], q["W_bwd"][0]), (hdY, hW, q["dY_bwd"][1], q["W_bwd"][1]), M * K),
            ("bwd_weight", L.sr_linear_bwd_weight, oracle.linear_bwd_weight,
             (t["dY"], t["A"], q["dY_bwd"][0], q["A_bwd"][0]), (hdY, hA, q["dY_bwd"][1], q["A_bwd"][1]), N * K)):
        say("linear", name, M, N, K)
        got = fn(*args).cpu().numpy().reshape(-1)
        if sample is None:
            ref, ab = ofn(*oargs, want_abs=True)
        else:
            idx = np.random.default_rng(1).integers(0, size, size=sample).astype(np.uint64)
            got = got[idx.astype(np.int64)]
            ref, ab = ofn(*oargs, want_abs=True, at=idx)
        if f8_pipeline:
            # bound of the fp8 pipeline, with sum_g max_g <= sum |x z|
            ref, ab = ref.reshape(-1).astype(np.float64), ab.reshape(-1).astype(np.float64)
            assert np.all(np.abs(got - ref) <= (7 * 2.0**-13 + 1e-6) * ab), name
            rel_rms = np.sqrt(((got - ref) ** 2).mean() / (ref ** 2).mean())
            say("   fp8 pipeline rms relative error", rel_rms)
            assert rel_rms < 1e-4
        else:
            check_product(got, ref, ab, name)
    # the fused backward pass gives the very same dA and dW (one Q(dY), Alg. 2)
    fl = 0 if not f8_pipeline else L.FLAG_F8_PIPELINE
    dA1 = L.sr_linear_bwd_data(t["dY"], t["W"], q["dY_bwd"][0], q["W_bwd"][0])
    dW1 = L.sr_linear_bwd_weight(t["dY"], t["A"], q["dY_bwd"][0], q["A_bwd"][0])
    dA2, dW2 = L.sr_linear_bwd(t["dY"], t["W"], t["A"], q["dY_bwd"][0], q["W_bwd"][0], q["A_bwd"][0])
    bk = [q[n][0].kind for n in ("dY_bwd", "W_bwd", "A_bwd")]
    if bk[0] == L.E5M2 and (bk[1] == L.E5M2) != (bk[2] == L.E5M2) and not f8_pipeline:
        # one product is E5M2 x E5M2 (from codes when called alone), the other is not: the fused call
        # stores Q(dY) once, as bfloat16, for both -- same exact products, other order of sums
        for a, b in ((dA1, dA2), (dW1, dW2)):
            assert float((a - b).abs().max()) <= 1e-5 * float(a.abs().max())
    else:
        assert torch.equal(dA1, dA2) and torch.equal(dW1, dW2), "fused backward differs"
    if beta_check:
        acc = dW2.clone()
        L.sr_linear_bwd(t["dY"], t["W"], t["A"], q["dY_bwd"][0], q["W_bwd"][0], q["A_bwd"][0], out_dW=acc, beta=1.0)
        assert torch.equal(acc, dW2 + dW2)
    # the pass that saves the backward operands of A and W as codes during the forward pass gives
    # the very same Y, dA and dW (integer forward formats only)
    if q["A_fwd"][0].kind in (L.INT8, L.INT4) and q["W_fwd"][0].kind in (L.INT8, L.INT4):
        Y1 = L.sr_linear_fwd(t["A"], t["W"], q["A_fwd"][0], q["W_fwd"][0])
        Y3, stash = L.sr_linear_fwd_stash(t["A"], t["W"], q["A_fwd"][0], q["W_fwd"][0], q["A_bwd"][0], q["W_bwd"][0])
        dA3, dW3 = L.sr_linear_bwd_stashed(t["dY"], stash, K, q["dY_bwd"][0], q["W_bwd"][0], q["A_bwd"][0])
        assert torch.equal(Y1, Y3), "forward with stash differs"
        assert torch.equal(dA2, dA3) and torch.equal(dW2, dW3), "backward from the stash differs"
        if beta_check:
            acc = dW3.clone()
            L.sr_linear_bwd_stashed(t["dY"], stash, K, q["dY_bwd"][0], q["W_bwd"][0], q["A_bwd"][0], out_dW=acc, beta=1.0)
            assert torch.equal(acc, dW3 + dW3)
    if beta_check:
        base = L.sr_linear_bwd_weight(t["dY"], t["A"], q["dY_bwd"][0], q["A_bwd"][0])
        acc = base.clone()
        L.sr_linear_bwd_weight(t["dY"], t["A"], q["dY_bwd"][0], q["A_bwd"][0], out=acc, beta=1.0)
        assert torch.equal(acc, base + base)


ALL_INT8 = {"A_fwd": L.INT8, "W_fwd": L.INT8, "A_bwd": L.INT8, "W_bwd": L.INT8, "dY_bwd": L.INT8}


def test_single_layer_int8_all_five_quantizers():
    # the small CPU-checkable layer: 64 x 128 activations, 128 x 128 weights, seed 0
    t = _layer(64, 128, 128, 0)
    _run_layer(t, _quants(ALL_INT8, t, seed=0), beta_check=True)


@pytest.mark.parametrize("kinds", [
    {"A_fwd": L.INT8, "W_fwd": L.INT8, "A_bwd": L.E5M2, "W_bwd": L.E5M2, "dY_bwd": L.E5M2},
    {"A_fwd": L.E4M3, "W_fwd": L.E4M3, "A_bwd": L.E4M3, "W_bwd": L.E4M3, "dY_bwd": L.E5M2},
    {"A_fwd": L.INT8, "W_fwd": L.INT4, "A_bwd": L.INT8, "W_bwd": L.INT8, "dY_bwd": L.INT4},
    {"A_fwd": L.E4M2, "W_fwd": L.E4M2, "A_bwd": L.E4M1, "W_bwd": L.E4M1, "dY_bwd": L.E4M0},
    {"A_fwd": L.INT4, "W_fwd": L.INT8, "A_bwd": L.E4M3, "W_bwd": L.E4M2, "dY_bwd": L.E5M2},
    {"A_fwd": L.INT8, "W_fwd": L.INT8, "A_bwd": L.E4M3, "W_bwd": L.E5M2, "dY_bwd": L.E5M2},
])
def test_ragged_layer_mixed_formats(kinds):
    t = _layer(272, 144, 208, 3, std_dy=1e-3, w_bf16=True)
    _run_layer(t, _quants(kinds, t, seed=5), beta_check=True)


def test_gpt2_mlp_shapes_int8_forward_e5m2_backward():
    # GPT-2-small MLP linears at 8192 tokens; checked on sampled output entries
    kinds = {"A_fwd": L.INT8, "W_fwd": L.INT8, "A_bwd": L.E5M2, "W_bwd": L.E5M2, "dY_bwd": L.E5M2}
    for name, N, K in synth.GPT2_SMALL_MLP:
        t = _layer(8192, N, K, 10, std_dy=1e-3)
        _run_layer(t, _quants(kinds, t, seed=1), sample=65536)


def test_llama_shapes_int4_gradient_bf16_weights():
    # Llama-1B-shaped linears at 4096 tokens: q-projection in full, the MLP ones sampled
    kinds = {"A_fwd": L.INT8, "W_fwd": L.INT8, "A_bwd": L.INT8, "W_bwd": L.INT8, "dY_bwd": L.INT4}
    t = _layer(4096, 2048, 2048, 20, std_dy=1e-3, w_bf16=True)
    _run_layer(t, _quants(kinds, t, seed=2))
    for N, K in ((5632, 2048), (2048, 5632)):
        t = _layer(4096, N, K, 21, std_dy=1e-3, w_bf16=True)
        _run_layer(t, _quants(kinds, t, seed=2), sample=65536)


def _two_stream_stash_step(t, q):
    """The benchmark's launch configuration: the stash pair in halves, the quantizing halves on one stream and
    the products on another, events between them; returns Y, dA, dW."""
    M, K = t["A"].shape
    N = t["W"].shape[0]
    dev = t["A"].device
    stash = torch.empty(L.sr_linear_stash_bytes(M, N, K), dtype=torch.uint8, device=dev)
    ws_f = torch.empty(L.sr_linear_workspace_bytes(L.OP_FWD_STASH, M, N, K), dtype=torch.uint8, device=dev)
    ws_b = torch.empty(L.sr_linear_workspace_bytes(L.OP_BWD_STASHED, M, N, K), dtype=torch.uint8, device=dev)
    Y = torch.zeros((M, N), dtype=torch.float32, device=dev)
    dA = torch.zeros((M, K), dtype=torch.float32, device=dev)
    dW = torch.zeros((N, K), dtype=torch.float32, device=dev)
    fa = (t["A"], t["W"], q["A_fwd"][0], q["W_fwd"][0], q["A_bwd"][0], q["W_bwd"][0])
    fk = dict(stash=stash, out=Y, workspace=ws_f)
    ba = (t["dY"], stash, K, q["dY_bwd"][0], q["W_bwd"][0], q["A_bwd"][0])
    bk = dict(out_dA=dA, out_dW=dW, workspace=ws_b)
    mem, mat = torch.cuda.Stream(), torch.cuda.Stream()
    ev_f, ev_b = torch.cuda.Event(), torch.cuda.Event()
    cur = torch.cuda.current_stream()
    mem.wait_stream(cur)
    mat.wait_stream(cur)
    with torch.cuda.stream(mem):
        L.sr_linear_fwd_stash(*fa, phase=L.PHASE_QUANTIZE, **fk)
        ev_f.record()
        L.sr_linear_bwd_stashed(*ba, phase=L.PHASE_QUANTIZE, **bk)
        ev_b.record()
    with torch.cuda.stream(mat):
        mat.wait_event(ev_f)
        L.sr_linear_fwd_stash(*fa, phase=L.PHASE_PRODUCT, **fk)
        mat.wait_event(ev_b)
        L.sr_linear_bwd_stashed(*ba, phase=L.PHASE_PRODUCT, **bk)
    cur.wait_stream(mem)
    cur.wait_stream(mat)
    torch.cuda.synchronize()
    return Y, dA, dW


def test_llama_projection_at_65536_tokens_sampled():
    # the largest token count of the sweep: 2^27-element activations and gradients, 256 x 256 tiles
    # for Y and dA, a 65536-long contraction for dW (int32 sums stay exact below 133143)
    kinds = {"A_fwd": L.INT8, "W_fwd": L.INT8, "A_bwd": L.INT8, "W_bwd": L.INT8, "dY_bwd": L.INT4}
    t = _layer(65536, 2048, 2048, 22, std_dy=1e-3, w_bf16=True)
    q = _quants(kinds, t, seed=3)
    _run_layer(t, q, sample=16384)
    # the same layer as the benchmark launches it (two streams, stash pair in halves): the results just
    # checked against the oracle, bit for bit
    Y, dA, dW = _two_stream_stash_step(t, q)
    assert torch.equal(Y, L.sr_linear_fwd(t["A"], t["W"], q["A_fwd"][0], q["W_fwd"][0]))
    dA0, dW0 = L.sr_linear_bwd(t["dY"], t["W"], t["A"], q["dY_bwd"][0], q["W_bwd"][0], q["A_bwd"][0])
    assert torch.equal(dA, dA0) and torch.equal(dW, dW0)
    del Y, dA, dW, dA0, dW0
    # and the middle one with the two MLP shapes
    for N, K in ((5632, 2048), (2048, 5632)):
        t = _layer(16384, N, K, 23, std_dy=1e-3, w_bf16=True)
        _run_layer(t, _quants(kinds, t, seed=4), sample=16384)


def test_llama_mlp_shapes_at_65536_tokens_sampled():
    # the benchmark's largest products: gate / up (5632 x 2048) and down (2048 x 5632) at 65536 tokens
    kinds = {"A_fwd": L.INT8, "W_fwd": L.INT8, "A_bwd": L.INT8, "W_bwd": L.INT8, "dY_bwd": L.INT4}
    for N, K in ((5632, 2048), (2048, 5632)):
        t = _layer(65536, N, K, 24, std_dy=1e-3, w_bf16=True)
        _run_layer(t, _quants(kinds, t, seed=6), sample=8192)
        del t
        torch.cuda.empty_cache()


def test_decoder_lm_head_shape_sampled():
    # the widest linear of the 12-layer decoder (vocabulary 32000, d = 768) at 8 x 1024 tokens, in the
    # formats of its training step
    kinds = {"A_fwd": L.INT8, "W_fwd": L.INT8, "A_bwd": L.E5M2, "W_bwd": L.E5M2, "dY_bwd": L.E5M2}
    t = _layer(8192, 32000, 768, 25, std_dy=1e-3, w_bf16=True)
    _run_layer(t, _quants(kinds, t, seed=7), sample=16384)


def test_fp8_pipeline_flag_same_codes_hardware_rounding():
    # the fp8 matrix pipeline: same quantized operands, products within the hardware's bound
    kinds = {"A_fwd": L.E4M3, "W_fwd": L.E4M3, "A_bwd": L.E5M2, "W_bwd": L.E5M2, "dY_bwd": L.E5M2}
    t = _layer(272, 144, 208, 3, std_dy=1e-3)
    _run_layer(t, _quants(kinds, t, seed=5, flags=L.FLAG_F8_PIPELINE), f8_pipeline=True)
    t = _layer(2048, 768, 512, 4, std_dy=1e-3)
    _run_layer(t, _quants(kinds, t, seed=6, flags=L.FLAG_F8_PIPELINE), sample=20000, f8_pipeline=True)


# Shapes that take the 256 x 256 tiles on workgroups that stay: ragged in both output dimensions
# and in the contraction; more tiles than CUs (every workgroup walks several, the last ones fewer);
# a contraction of one stage and of two (ring buffer parity at the tile change); a long contraction
# cut into slices (partial tiles, ragged last slice).
PERSIST_SHAPES = [(4104, 2056, 2064), (8200, 4104, 400), (8200, 4104, 144), (6160, 4104, 1040), (2056, 1032, 32784)]


def _exact_on_device(X, Z, scale):
    """Exact product of two int8 code matrices, in binary64 on the device (|sum| < 2^53)."""
    return (X.view(torch.int8).double() @ Z.view(torch.int8).double().t()) * scale


@pytest.mark.parametrize("P,Q,R", PERSIST_SHAPES)
def test_large_tile_kernel_full_output_int8(P, Q, R):
    say("gemm 256-tile int8", P, Q, R)
    X, Z = _rand_codes((P, R), L.INT8, 5), _rand_codes((Q, R), L.INT4, 6)
    Xd, Zd = to_dev(X), to_dev(Z)
    got = L.sr_gemm_codes(Xd, L.INT8, Zd, L.INT4, alpha=0.5)
    # every entry, against the exact integer product (no tile missing, none written twice wrongly)
    assert torch.equal(got.double(), _exact_on_device(Xd, Zd, 0.5))
    # and sampled entries against the oracle, edges of the tile grid included
    rng = np.random.default_rng(1)
    idx = np.concatenate([rng.integers(0, P * Q, size=4096).astype(np.uint64),
                          np.array([0, Q - 1, (P - 1) * Q, P * Q - 1, 255 * Q + 255, 256 * Q + 256], dtype=np.uint64)])
    ref = oracle.gemm_fwd(X, L.INT8, 1.0, Z, L.INT4, 0.5, at=idx)
    assert np.array_equal(got.cpu().numpy().reshape(-1)[idx.astype(np.int64)], ref)
    # beta = 1 adds to what is there
    again = L.sr_gemm_codes(Xd, L.INT8, Zd, L.INT4, alpha=0.5, out=got.clone(), beta=1.0)
    assert torch.equal(again.double(), 2 * _exact_on_device(Xd, Zd, 0.5))


@pytest.mark.parametrize("P,Q,R", [(4104, 2056, 2064), (2056, 1032, 32784)])
def test_large_tile_kernel_float_pipelines(P, Q, R):
    say("gemm 256-tile e5m2", P, Q, R)
    X, Z = _rand_codes((P, R), L.E5M2, 27), _rand_codes((Q, R), L.E5M2, 28)
    Xd, Zd = to_dev(X), to_dev(Z)
    rng = np.random.default_rng(2)
    idx = np.concatenate([rng.integers(0, P * Q, size=4096).astype(np.uint64),
                          np.array([0, Q - 1, (P - 1) * Q, P * Q - 1], dtype=np.uint64)])
    ref, ab = oracle.gemm_fwd(X, L.E5M2, 0.5, Z, L.E5M2, 0.5, want_abs=True, at=idx)
    pick = idx.astype(np.int64)
    got = L.sr_gemm_e5m2(Xd, Zd, alpha=0.25).cpu().numpy().reshape(-1)[pick]      # f16 pipeline from codes
    check_product(got, ref, ab, "e5m2 codes")
    Xv = torch.from_numpy(oracle.decode_array(L.E5M2, X)).to(DEV).to(torch.bfloat16)
    Zv = torch.from_numpy(oracle.decode_array(L.E5M2, Z)).to(DEV).to(torch.bfloat16)
    got = L.sr_gemm_bf16(Xv, Zv, alpha=0.25).cpu().numpy().reshape(-1)[pick]       # bf16 pipeline
    check_product(got, ref, ab, "bf16 values")
    got = L.sr_gemm_codes(Xd, L.E5M2, Zd, L.E5M2, alpha=0.25).cpu().numpy().reshape(-1)[pick]  # fp8 pipeline
    assert np.all(np.abs(got - ref) <= 7 * 2.0**-13 * ab)
