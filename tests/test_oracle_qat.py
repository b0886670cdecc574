"""Pins for the oracle's composition of the Sec. 3.3 estimator (Fig. 3): one quantized weight
copy shared by the two passes, SR on the saved activation and the output gradient, and the
unbiasedness statement of Eq. 6-7 checked by averaging over thresholds."""
import numpy as np

import oracle
from oracle import INT8, E5M2


def _data(M=12, N=10, K=16, seed=0):
    rng = np.random.default_rng(seed)
    A = rng.standard_normal((M, K)).astype(np.float32)
    W = (0.02 * rng.standard_normal((N, K))).astype(np.float32)
    dY = (1e-3 * rng.standard_normal((M, N))).astype(np.float32)
    return A, W, dY


def _q(x, kind, seed, off):
    return oracle.Quant(kind, oracle.absmax_scale(x, kind), seed, off)


def test_both_passes_use_the_same_quantized_weights():
    # written out with numpy on the dequantized codes: the W_hat inside Y and the one inside dA
    # are the same matrix
    for kind in (INT8, E5M2):
        A, W, dY = _data()
        qW, qA, qdY = _q(W, kind, 3, 0), _q(A, kind, 3, 100), _q(dY, kind, 3, 200)
        Y, dA, dW = oracle.qat_pass(A, W, dY, qW, qA, qdY)
        What = oracle.decode_array(kind, qW(W)).astype(np.float64) * qW.scale
        dYhat = oracle.decode_array(kind, qdY(dY)).astype(np.float64) * qdY.scale
        Ahat = oracle.decode_array(kind, qA(A)).astype(np.float64) * qA.scale
        assert np.allclose(Y, A.astype(np.float64) @ What.T, rtol=1e-6, atol=1e-12)
        assert np.allclose(dA, dYhat @ What, rtol=1e-6, atol=1e-15)
        assert np.allclose(dW, dYhat.T @ Ahat, rtol=1e-6, atol=1e-15)
        # a different position for the backward weights would give another W_hat: the sharing is
        # a property of (seed, offset), not of the data
        other = oracle.Quant(kind, qW.scale, 3, 999)
        assert not np.array_equal(other(W), qW(W))


def test_backward_estimator_is_unbiased_given_the_weights():
    # Eq. 6-7: over the thresholds of A and dY (W_hat held fixed) the means of dA and dW are the
    # gradients at the quantized weights, dY W_hat and dY^T A
    A, W, dY = _data(M=8, N=6, K=8, seed=1)
    kind = INT8
    qW = _q(W, kind, 1, 0)
    sA, sdY = oracle.absmax_scale(A, kind), oracle.absmax_scale(dY, kind)
    S = 3000
    sum_dA = np.zeros((8, 8)); sum_dW = np.zeros((6, 8)); sq_dW = np.zeros((6, 8)); sq_dA = np.zeros((8, 8))
    for s in range(S):
        _, dA, dW = oracle.qat_pass(A, W, dY, qW, oracle.Quant(kind, sA, 1000 + s, 50), oracle.Quant(kind, sdY, 1000 + s, 90))
        sum_dA += dA; sum_dW += dW; sq_dA += dA.astype(np.float64) ** 2; sq_dW += dW.astype(np.float64) ** 2
    What = oracle.decode_array(kind, qW(W)).astype(np.float64) * qW.scale
    for mean, sq, exact in ((sum_dA / S, sq_dA / S, dY.astype(np.float64) @ What),
                            (sum_dW / S, sq_dW / S, dY.astype(np.float64).T @ A.astype(np.float64))):
        se = np.sqrt(np.maximum(sq - mean ** 2, 0) / S) + 1e-12 * np.abs(exact).max()
        assert np.all(np.abs(mean - exact) <= 5 * se + 2.0 ** -17 * np.abs(exact).max())
