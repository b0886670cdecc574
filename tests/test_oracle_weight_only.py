"""Pins for the oracle's weight-only products (Sec. 3.2, the objective with quantized weights and
full-precision activations): special cases that reduce to the already pinned code products, a
brute-force loop with the indices written out, and the adjoint identity between the two."""
import numpy as np
import pytest

import oracle

KINDS = [oracle.INT8, oracle.INT4, oracle.E4M3, oracle.E5M2, oracle.E4M1]


def _w(n, k, seed):
    return (np.random.default_rng(seed).standard_normal((n, k)) * 0.02).astype(np.float32)


@pytest.mark.parametrize("kind", KINDS)
def test_integer_activations_reduce_to_the_product_of_codes(kind):
    # small integers are int8 codes at scale 1: the weight-only product must equal the code product
    rng = np.random.default_rng(1)
    M, N, K = 7, 5, 24
    W = _w(N, K, 2)
    qW = oracle.Quant(kind, oracle.absmax_scale(W, kind), seed=3, counter_offset=11)
    if kind in (oracle.INT8, oracle.INT4):
        A = rng.integers(-127, 128, (M, K)).astype(np.float32)
        Ac, kA = A.astype(np.int8).view(np.uint8), oracle.INT8
        dY = rng.integers(-127, 128, (M, N)).astype(np.float32)
        dYc = dY.astype(np.int8).view(np.uint8)
    else:
        # values on the E5M2 grid pass through the E5M2 quantizer at scale 1 unchanged
        grid = np.array([0.0, 0.5, -0.75, 1.0, -1.25, 1.5, 2.0, -3.0, 4.0, 0.375], dtype=np.float32)
        A = grid[rng.integers(0, grid.size, (M, K))]
        dY = grid[rng.integers(0, grid.size, (M, N))]
        Ac, kA = oracle.quantize(A, oracle.E5M2, 1.0, 0, 0), oracle.E5M2
        dYc = oracle.quantize(dY, oracle.E5M2, 1.0, 0, 0)
        assert np.array_equal(oracle.decode_array(oracle.E5M2, Ac), A.astype(np.float64))
    Wc = qW(W)
    np.testing.assert_array_equal(oracle.linear_fwd_weight_only(A, W, qW), oracle.gemm_fwd(Ac, kA, 1.0, Wc, kind, qW.scale))
    np.testing.assert_array_equal(oracle.linear_bwd_data_weight_only(dY, W, qW),
                                  oracle.gemm_bwd_data(dYc, kA, 1.0, Wc, kind, qW.scale))


@pytest.mark.parametrize("kind", [oracle.INT8, oracle.E4M3])
def test_against_loops_with_the_indices_written_out(kind):
    rng = np.random.default_rng(4)
    M, N, K = 3, 4, 5
    A = rng.standard_normal((M, K)).astype(np.float32)
    dY = rng.standard_normal((M, N)).astype(np.float32)
    W = _w(N, K, 5)
    qW = oracle.Quant(kind, oracle.absmax_scale(W, kind), seed=6)
    Wc = qW(W)
    Y, Yabs = oracle.linear_fwd_weight_only(A, W, qW, want_abs=True)
    dA = oracle.linear_bwd_data_weight_only(dY, W, qW)
    s = float(np.float32(qW.scale))
    for m in range(M):
        for n in range(N):
            acc = sum(float(A[m, k]) * oracle.decode(kind, int(Wc[n, k])) for k in range(K))
            aacc = sum(abs(float(A[m, k]) * oracle.decode(kind, int(Wc[n, k]))) for k in range(K))
            assert Y[m, n] == np.float32(s * acc)
            assert Yabs[m, n] == pytest.approx(s * aacc, rel=1e-6)
        for k in range(K):
            acc = sum(float(dY[m, n]) * oracle.decode(kind, int(Wc[n, k])) for n in range(N))
            assert dA[m, k] == np.float32(s * acc)


def test_identity_activations_return_the_dequantized_weights():
    W = _w(6, 6, 7)
    qW = oracle.Quant(oracle.E5M2, oracle.absmax_scale(W, oracle.E5M2), seed=8)
    What = oracle.decode_array(oracle.E5M2, qW(W)) * np.float64(np.float32(qW.scale))
    eye = np.eye(6, dtype=np.float32)
    np.testing.assert_array_equal(oracle.linear_fwd_weight_only(eye, W, qW), What.T.astype(np.float32))
    np.testing.assert_array_equal(oracle.linear_bwd_data_weight_only(eye, W, qW), What.astype(np.float32))


def test_forward_and_input_gradient_are_adjoint():
    # <dY, A What^T> = <dY What, A>; with small-integer A, dY and int4 weights at a power-of-two
    # scale every number involved is an exact binary32 integer multiple, so equality is exact
    rng = np.random.default_rng(9)
    M, N, K = 6, 8, 16
    A = rng.integers(-7, 8, (M, K)).astype(np.float32)
    dY = rng.integers(-7, 8, (M, N)).astype(np.float32)
    W = rng.integers(-7, 8, (N, K)).astype(np.float32) * 0.25
    qW = oracle.Quant(oracle.INT4, 0.25, seed=10)
    assert np.array_equal(oracle.decode_array(oracle.INT4, qW(W)) * 0.25, W.astype(np.float64))
    Y = oracle.linear_fwd_weight_only(A, W, qW).astype(np.float64)
    dA = oracle.linear_bwd_data_weight_only(dY, W, qW).astype(np.float64)
    assert np.sum(dY * Y) == np.sum(dA * A)
    # and it is the full-precision product, since W passed through the quantizer unchanged
    np.testing.assert_array_equal(Y, A.astype(np.float64) @ W.astype(np.float64).T)


def test_bfloat16_sources_are_widened_exactly():
    rng = np.random.default_rng(11)
    A32 = rng.standard_normal((5, 8)).astype(np.float32)
    bits = (A32.view(np.uint32) >> 16).astype(np.uint16)          # truncate to bfloat16
    A_as_f32 = (bits.astype(np.uint32) << 16).view(np.float32)
    W = _w(4, 8, 12)
    qW = oracle.Quant(oracle.INT8, oracle.absmax_scale(W, oracle.INT8), seed=13)
    np.testing.assert_array_equal(oracle.linear_fwd_weight_only(bits, W, qW), oracle.linear_fwd_weight_only(A_as_f32, W, qW))
