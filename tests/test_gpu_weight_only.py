"""The weight-only objective (Sec. 3.2: quantized weights, full-precision activations and
gradients) through the C ABI against the oracle's binary64 definition: Y = A Q(W)^T and
dA = dY Q(W), every weight format, binary32 and bfloat16 row operands."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import DEV, KINDS, check_product, host_src, say
from paper_2511_00874_amd import lib as L
from paper_2511_00874_amd import synth

pytestmark = pytest.mark.gpu

NOQ = L.Quant(L.NONE, 1.0)


def _case(M, N, K, kind, bf16_rows, bf16_w, seed):
    A = synth.gaussian_torch((M, K), 1.0, seed, DEV)
    dY = synth.gaussian_torch((M, N), 1e-3, seed + 1, DEV)
    W = synth.gaussian_torch((N, K), 0.02, seed + 2, DEV)
    if bf16_rows:
        A, dY = A.to(torch.bfloat16), dY.to(torch.bfloat16)
    if bf16_w:
        W = W.to(torch.bfloat16)
    sW = float(L.sr_absmax_scale(W, kind).cpu()[0])
    return A, dY, W, sW


@pytest.mark.parametrize("bf16_rows", [False, True])
@pytest.mark.parametrize("kind", KINDS)
def test_forward_and_input_gradient_match_the_definition(kind, bf16_rows):
    # ragged: edge tiles in both output dimensions, contraction tails (208 = 128 + 80)
    M, N, K = 272, 144, 208
    A, dY, W, sW = _case(M, N, K, kind, bf16_rows, bf16_w=(kind == L.INT4), seed=50 + kind)
    qW = L.Quant(kind, sW, seed=9, counter_offset=77)
    oq = oracle.Quant(kind, sW, seed=9, counter_offset=77)
    say("weight-only", L.KIND_NAMES[kind], "bf16 rows" if bf16_rows else "fp32 rows", M, N, K)
    Y = L.sr_linear_fwd(A, W, NOQ, qW).cpu().numpy()
    ref, ab = oracle.linear_fwd_weight_only(host_src(A), host_src(W), oq, want_abs=True)
    check_product(Y, ref, ab, "Y")
    dA = L.sr_linear_bwd_data(dY, W, NOQ, qW).cpu().numpy()
    ref, ab = oracle.linear_bwd_data_weight_only(host_src(dY), host_src(W), oq, want_abs=True)
    check_product(dA, ref, ab, "dA")


def test_binary32_operand_is_split_exactly():
    # integers up to 2^24 - 1 need all 24 significand bits: with W = identity (on the int8 grid
    # at scale 1) the product returns A itself, bit for bit, only if the three planes sum to it
    M, K = 64, 64
    g = torch.Generator(device=DEV).manual_seed(3)
    A = torch.randint(-(1 << 24) + 1, 1 << 24, (M, K), device=DEV, generator=g).float()
    A[0, :8] = torch.tensor([0.0, -0.0, 1.0, 2.0 ** -126, 16777215.0, -16777215.0, 3.0e38, 1.0 + 2.0 ** -23], device=DEV)
    W = torch.eye(K, device=DEV)
    Y = L.sr_linear_fwd(A, W, NOQ, L.Quant(L.INT8, 1.0, seed=1))
    bad = (Y != A).nonzero().cpu().numpy()
    say("mismatches", [(int(i), int(j), float(A[i, j]), float(Y[i, j])) for i, j in bad[:10]])
    assert torch.equal(Y, A)
    # the stated limit: the bf16 matrix pipeline takes subnormal numbers as zero
    A[0, 3] = 2.0 ** -140
    Y = L.sr_linear_fwd(A, W, NOQ, L.Quant(L.INT8, 1.0, seed=1))
    assert float(Y[0, 3]) == 0.0 and torch.equal(Y[1:], A[1:])


def test_long_contraction_is_split_and_accumulated():
    # few tiles, long contraction: the three plane products each run in slices and accumulate
    M, N, K = 128, 128, 16384
    A, dY, W, sW = _case(M, N, K, L.E5M2, False, False, seed=70)
    qW, oq = L.Quant(L.E5M2, sW, seed=2), oracle.Quant(L.E5M2, sW, seed=2)
    Y = L.sr_linear_fwd(A, W, NOQ, qW).cpu().numpy()
    ref, ab = oracle.linear_fwd_weight_only(host_src(A), host_src(W), oq, want_abs=True)
    check_product(Y, ref, ab, "Y")


def test_gpt2_mlp_shape_int8_weights():
    M, N, K = 8192, 3072, 768
    A, dY, W, sW = _case(M, N, K, L.INT8, False, False, seed=80)
    qW, oq = L.Quant(L.INT8, sW, seed=4, counter_offset=5), oracle.Quant(L.INT8, sW, seed=4, counter_offset=5)
    Y = L.sr_linear_fwd(A, W, NOQ, qW).cpu().numpy()
    ref, ab = oracle.linear_fwd_weight_only(host_src(A), host_src(W), oq, want_abs=True)
    check_product(Y, ref, ab, "Y")
    dA = L.sr_linear_bwd_data(dY, W, NOQ, qW).cpu().numpy()
    ref, ab = oracle.linear_bwd_data_weight_only(host_src(dY), host_src(W), oq, want_abs=True)
    check_product(dA, ref, ab, "dA")


def test_where_the_identity_quantizer_is_not_accepted():
    A = torch.zeros((16, 16), device=DEV)
    q8 = L.Quant(L.INT8, 1.0)
    with pytest.raises(RuntimeError):
        L.sr_linear_fwd(A, A, q8, NOQ)            # W must be quantized
    with pytest.raises(RuntimeError):
        L.sr_linear_bwd_weight(A, A, NOQ, q8)     # no quantized operand: not this library's product
    with pytest.raises(RuntimeError):
        L.sr_quantize(A, NOQ)
