"""Pins for the oracle's quantized matrix products (CPU only)."""
import numpy as np
import pytest

import oracle
from oracle import E4M3, E5M2, INT4, INT8
from paper_2511_00874_amd import synth


def _codes(shape, kind, seed):
    x = synth.gaussian(shape, 1.0, seed)
    s = oracle.absmax_scale(x, kind)
    return oracle.quantize(x, kind, s, seed, 0), s


PAIRS = [(INT8, INT8), (INT4, INT8), (E4M3, E4M3), (E5M2, E4M3), (E5M2, E5M2)]


@pytest.mark.parametrize("kx,kz", PAIRS)
def test_products_equal_fp64_matmul_of_dequantized_codes(kx, kz):
    # Sec. 2.2.2: low-precision multiply + high-precision accumulate == exact product of
    # the two quantized matrices
    M, N, K = 13, 11, 37
    Ac, sA = _codes((M, K), kx, 1)
    Wc, sW = _codes((N, K), kz, 2)
    dYc, sdY = _codes((M, N), kx, 3)
    Av, Wv, dYv = (oracle.decode_array(k, c) for k, c in ((kx, Ac), (kz, Wc), (kx, dYc)))

    def chk(got, ref, s1, s2):
        want = (np.float64(np.float32(s1) * np.float32(s2)) * ref).astype(np.float32)
        assert np.array_equal(got, want)

    chk(oracle.gemm_fwd(Ac, kx, sA, Wc, kz, sW), Av @ Wv.T, sA, sW)                 # Alg. 1
    chk(oracle.gemm_bwd_data(dYc, kx, sdY, Wc, kz, sW), dYv @ Wv, sdY, sW)           # Alg. 2
    Ac2, sA2 = _codes((M, K), kz, 4)
    chk(oracle.gemm_bwd_weight(dYc, kx, sdY, Ac2, kz, sA2),
        dYv.T @ oracle.decode_array(kz, Ac2), sdY, sA2)                              # Alg. 2


def test_integer_products_are_exact_integers():
    M, N, K = 9, 7, 300
    rng = np.random.default_rng(0)
    Ac = rng.integers(-127, 128, size=(M, K)).astype(np.int8)
    Wc = rng.integers(-127, 128, size=(N, K)).astype(np.int8)
    Y = oracle.gemm_fwd(Ac.view(np.uint8), INT8, 1.0, Wc.view(np.uint8), INT8, 1.0)
    assert np.array_equal(Y.astype(np.int64), Ac.astype(np.int64) @ Wc.astype(np.int64).T)
    # worst case magnitude stays exact
    Ac[:] = -127
    Wc[:] = 127
    Y = oracle.gemm_fwd(Ac.view(np.uint8), INT8, 1.0, Wc.view(np.uint8), INT8, 1.0)
    assert np.all(Y == np.float32(-127 * 127 * K))


def test_backward_products_are_transposed_forward_products():
    M, N, K = 10, 6, 14
    dYc, sdY = _codes((M, N), E5M2, 5)
    Wc, sW = _codes((N, K), E5M2, 6)
    Ac, sA = _codes((M, K), E5M2, 7)
    # dA = dY W = dY (W^T)^T ; dW = dY^T A = dY^T (A^T)^T
    assert np.array_equal(oracle.gemm_bwd_data(dYc, E5M2, sdY, Wc, E5M2, sW),
                          oracle.gemm_fwd(dYc, E5M2, sdY, Wc.T.copy(), E5M2, sW))
    assert np.array_equal(oracle.gemm_bwd_weight(dYc, E5M2, sdY, Ac, E5M2, sA),
                          oracle.gemm_fwd(dYc.T.copy(), E5M2, sdY, Ac.T.copy(), E5M2, sA))


def test_sampled_entries_equal_full_products_and_abs_sums():
    M, N, K = 12, 9, 21
    Ac, sA = _codes((M, K), INT8, 1)
    Wc, sW = _codes((N, K), INT8, 2)
    dYc, sdY = _codes((M, N), INT4, 3)
    rng = np.random.default_rng(0)
    for fn, args, size in (
            (oracle.gemm_fwd, (Ac, INT8, sA, Wc, INT8, sW), M * N),
            (oracle.gemm_bwd_data, (dYc, INT4, sdY, Wc, INT8, sW), M * K),
            (oracle.gemm_bwd_weight, (dYc, INT4, sdY, Ac, INT8, sA), N * K)):
        full, ab = fn(*args, want_abs=True)
        idx = rng.integers(0, size, size=40)
        part, pab = fn(*args, want_abs=True, at=idx)
        assert np.array_equal(part, full.reshape(-1)[idx])
        assert np.array_equal(pab, ab.reshape(-1)[idx])
        assert np.all(ab >= np.abs(full))


def test_algorithms_compose_quantizers_and_product():
    # Alg. 1 / Alg. 2 on the small layer: equal to quantizing by hand and multiplying
    A, W, dY = synth.single_layer()
    q = {n: oracle.Quant(INT8, oracle.absmax_scale(x, INT8), seed=0, counter_offset=off)
         for n, x, off in (("A_fwd", A, 0), ("W_fwd", W, 1024), ("A_bwd", A, 3072),
                           ("W_bwd", W, 4096), ("dY_bwd", dY, 6144))}
    Y = oracle.linear_fwd(A, W, q["A_fwd"], q["W_fwd"])
    Av = oracle.decode_array(INT8, q["A_fwd"](A)) * q["A_fwd"].scale
    Wv = oracle.decode_array(INT8, q["W_fwd"](W)) * q["W_fwd"].scale
    np.testing.assert_allclose(Y, Av @ Wv.T, rtol=2e-7, atol=0)
    # the quantized product approximates the real one (Sec. 2.2.2: AB ~ Ahat Bhat)
    rel = np.abs(Y - A @ W.T).max() / np.abs(A @ W.T).max()
    assert rel < 0.05
    dA = oracle.linear_bwd_data(dY, W, q["dY_bwd"], q["W_bwd"])
    dW = oracle.linear_bwd_weight(dY, A, q["dY_bwd"], q["A_bwd"])
    assert np.abs(dA - dY @ W).max() / np.abs(dY @ W).max() < 0.05
    assert np.abs(dW - dY.T @ A).max() / np.abs(dY.T @ A).max() < 0.05
    # the five quantizers use distinct thresholds: A's forward and backward codes differ
    assert not np.array_equal(q["A_fwd"](A), q["A_bwd"](A))


def _sr_moments(x, kind, scale):
    """mean (= t) and Bernoulli variance of one SR-quantized element, in real units."""
    t = (x * np.float32(1.0 / np.float32(scale))).astype(np.float64)
    p = t - np.floor(t)
    return t * scale, p * (1 - p) * scale * scale


@pytest.mark.parametrize("kdY", [INT8, INT4])
def test_weight_gradient_is_unbiased_with_the_variance_of_lemma_3(kdY):
    # proof of Lemma 3: per term Var = X^2 s_Y^2 + Y^2 s_X^2 + s_X^2 s_Y^2, terms independent,
    # so Var[dW_nk] = sum_m (A_mk^2 s_dY^2 + dY_mn^2 s_A^2 + s_A^2 s_dY^2)
    M, N, K, seeds = 48, 8, 8, 1500
    A, _, dY = synth.single_layer(M=M, N=N, K=K, seed=11)
    sA, sdY = oracle.absmax_scale(A, INT8), oracle.absmax_scale(dY, kdY)
    Am, Av = _sr_moments(A, INT8, sA)
    Ym, Yv = _sr_moments(dY, kdY, sdY)
    want_mean = Ym.T @ Am
    want_var = Yv.T @ (Am**2) + (Ym**2).T @ Av + Yv.T @ Av
    acc = np.zeros((N, K))
    acc2 = np.zeros((N, K))
    for s in range(seeds):
        dW = oracle.linear_bwd_weight(dY, A, oracle.Quant(kdY, sdY, s, 0),
                                      oracle.Quant(INT8, sA, s, 1000)).astype(np.float64)
        acc += dW
        acc2 += dW * dW
    mean = acc / seeds
    var = acc2 / seeds - mean**2
    z = (mean - want_mean) / np.sqrt(want_var / seeds)
    assert np.abs(z).max() < 5
    assert abs(var.sum() / want_var.sum() - 1) < 0.05


def test_fewer_gradient_bits_raise_variance_by_the_square_of_the_step_ratio():
    # Lemma 3: T^Q scales with Delta^2 (4x per bit).  Both operands int4 vs both int8: the two
    # leading terms scale by (Delta_4/Delta_8)^2 = (127/7)^2, the product term is small
    M, N, K, seeds = 48, 8, 8, 500
    A, _, dY = synth.single_layer(M=M, N=N, K=K, seed=11)
    tot = {}
    for kind in (INT8, INT4):
        sdY, sA = oracle.absmax_scale(dY, kind), oracle.absmax_scale(A, kind)
        vals = np.stack([oracle.linear_bwd_weight(dY, A, oracle.Quant(kind, sdY, s, 0),
                                                  oracle.Quant(kind, sA, s, 1000)).astype(np.float64)
                         for s in range(seeds)])
        tot[kind] = vals.var(axis=0).sum()
    ratio = tot[INT4] / tot[INT8]
    assert 0.7 * (127 / 7) ** 2 < ratio < 1.4 * (127 / 7) ** 2


def test_variance_of_mean_gradient_decays_as_one_over_b():
    # Lemma 3: with the 1/b normalisation the SR variance of dW is proportional to 1/b
    N, K, seeds = 4, 4, 600
    out = {}
    for b in (16, 64):
        A, _, dY = synth.single_layer(M=b, N=N, K=K, seed=3)
        # fixed scales so that both batch sizes share one grid
        sA, sdY = 4.0 / 127, 4.0 / 7
        vals = np.stack([oracle.linear_bwd_weight(dY, A, oracle.Quant(INT4, sdY, s, 0),
                                                  oracle.Quant(INT8, sA, s, 500)).astype(np.float64) / b
                         for s in range(seeds)])
        out[b] = vals.var(axis=0).mean()
    assert 2.8 < out[16] / out[64] < 5.6  # 4 within sampling error
