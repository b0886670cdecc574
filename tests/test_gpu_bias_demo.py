"""Stochastic rounding against round-to-nearest on the GPU path (Sec. 2.2.1, Sec. 3.2, Lemma 3):
nearest rounding has a systematic error that averaging over a mini-batch cannot remove, the
error of stochastic rounding has zero mean and its contribution to the weight gradient shrinks
with the batch size.  Synthetic inputs only; the checks are statistical properties with
explicit standard-error margins."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import DEV, say
from paper_2511_00874_amd import lib as L
from paper_2511_00874_amd import synth

pytestmark = pytest.mark.gpu


def test_rounding_error_has_zero_mean_under_sr_and_not_under_rtn():
    # the outlier-heavy tensor: with absmax scaling almost every value lies within half a step
    # of zero, which nearest rounding maps to zero
    n = 1 << 22
    x = synth.outlier_tensor_torch(n, 99, DEV)
    for kind in (L.INT4, L.INT8):
        s = L.sr_absmax_scale(x, kind)
        scale = float(s.cpu()[0])
        xs = x.cpu().numpy().astype(np.float64)
        err = {}
        for mode in (L.SR, L.RTN):
            q = L.Quant(L.INT8 if kind == L.INT8 else L.INT4, s, seed=5, counter_offset=0, round_mode=mode)
            codes = L.sr_quantize(x, q).cpu().numpy()
            if kind == L.INT4:
                codes = oracle.unpack_int4(codes)
            val = codes.view(np.int8).astype(np.float64) * scale
            # error along the sign of x: shrinkage toward zero shows up as a negative mean
            err[mode] = (val - xs) * np.sign(xs)
        se = scale / np.sqrt(n)  # per-element error is below one step
        say(L.KIND_NAMES[kind], "step", scale, "mean signed error SR", err[L.SR].mean(), "RTN", err[L.RTN].mean(), "s.e.<", se)
        assert abs(err[L.SR].mean()) < 5 * se
        assert err[L.RTN].mean() < -20 * se


def test_weight_gradient_error_shrinks_with_batch_only_under_sr():
    # dW / b = (1/b) sum_j dy_j a_j^T.  Every a, dy is an integer uniform on -3..3 plus 0.3 of a
    # step (Delta = 1).  Nearest rounding drops the 0.3 from every sample alike: the error of an
    # entry is -(0.3 i + 0.3 j + 0.09) per sample, mean -0.09 whatever b, variance 0.09 * 8 / b.
    # Stochastic rounding adds independent zero-mean errors e with variance 0.3 * 0.7 = 0.21:
    # the error of an entry is mean_j(dy e_a + a e_dy + e_a e_dy), variance
    # (2 * 0.21 * E[x^2] + 0.21^2) / b with E[x^2] = 4 + 0.09 (the batch-size law of Lemma 3).
    K, N = 64, 32
    rms = {L.SR: [], L.RTN: []}
    sizes = (256, 1024, 4096, 16384)
    for b in sizes:
        g = torch.Generator(device=DEV).manual_seed(b)
        A = torch.randint(-3, 4, (b, K), device=DEV, generator=g).float() + 0.3
        dY = torch.randint(-3, 4, (b, N), device=DEV, generator=g).float() + 0.3
        exact = (dY.double().T @ A.double()) / b
        for mode in (L.SR, L.RTN):
            qdy = L.Quant(L.INT8, 1.0, seed=17, counter_offset=0, round_mode=mode)
            qa = L.Quant(L.INT8, 1.0, seed=17, counter_offset=1 << 30, round_mode=mode)
            dW = L.sr_linear_bwd_weight(dY, A, qdy, qa).double() / b
            rms[mode].append(float(torch.sqrt(torch.mean((dW - exact) ** 2))))
    say("rms error of an entry of dW/b  SR", rms[L.SR], " RTN", rms[L.RTN])
    for b, sr, rtn in zip(sizes, rms[L.SR], rms[L.RTN]):
        assert abs(sr / np.sqrt((2 * 0.21 * 4.09 + 0.21 ** 2) / b) - 1) < 0.1
        assert abs(rtn / np.sqrt(0.09 ** 2 + 0.72 / b) - 1) < 0.1
    assert rms[L.RTN][-1] > 8 * rms[L.SR][-1]


def test_batch_size_pays_for_bits():
    # Remark after Lemma 3 (Sec. 4.2): the stochastic-rounding part of the gradient variance goes
    # like Delta^2 / b, so a format with one bit less (Delta doubled) needs four times the batch,
    # and a 4-bit output gradient next to 8-bit activations is dominated by the 4-bit operand.
    # a, dy uniform on [-1, 1): fractions are uniform, E[p (1 - p)] = 1/6, E[x^2] = 1/3, and the
    # error of an entry of dW / b has variance
    #   (Da^2 / 6 * E[dy^2] + Ddy^2 / 6 * E[a^2] + Da^2 Ddy^2 / 36) / b.
    K, N = 64, 32

    def rms_error(b, kind_dy, step_dy, step_a):
        g = torch.Generator(device=DEV).manual_seed(1000 + b)
        A = torch.rand((b, K), device=DEV, generator=g) * 2 - 1
        dY = torch.rand((b, N), device=DEV, generator=g) * 2 - 1
        exact = (dY.double().T @ A.double()) / b
        qdy = L.Quant(kind_dy, step_dy, seed=23, counter_offset=0)
        qa = L.Quant(L.INT8, step_a, seed=23, counter_offset=1 << 30)
        dW = L.sr_linear_bwd_weight(dY, A, qdy, qa).double() / b
        return float(torch.sqrt(torch.mean((dW - exact) ** 2)))

    def closed_form(b, step_dy, step_a):
        return np.sqrt((step_a ** 2 / 6 / 3 + step_dy ** 2 / 6 / 3 + step_a ** 2 * step_dy ** 2 / 36) / b)

    d8, d4 = 1.0 / 127, 1.0 / 7
    got = {}
    for b in (1024, 4096, 16384):
        got[b] = (rms_error(b, L.INT8, d8, d8), rms_error(b, L.INT8, 2 * d8, 2 * d8), rms_error(b, L.INT4, d4, d8))
        say("b", b, "rms error of dW/b: int8", got[b][0], "one bit less", got[b][1], "int4 dY", got[b][2])
        assert abs(got[b][0] / closed_form(b, d8, d8) - 1) < 0.1
        assert abs(got[b][1] / closed_form(b, 2 * d8, 2 * d8) - 1) < 0.1
        assert abs(got[b][2] / closed_form(b, d4, d8) - 1) < 0.1
    # one bit less at four times the batch: the same error
    assert abs(got[4096][1] / got[1024][0] - 1) < 0.1 and abs(got[16384][1] / got[4096][0] - 1) < 0.1
    # the 4-bit gradient costs (127 / 7)^2 / 2 = 165 times the variance of the all-8-bit layer
    assert abs(got[4096][2] / got[4096][0] / np.sqrt(((127 / 7) ** 2 + 1) / 2) - 1) < 0.1
