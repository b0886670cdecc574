"""ctypes + numpy face of the CPU oracle in srq_oracle.c.

TEST INFRASTRUCTURE.  Only tests/, the smoke check and the benchmark's
CPU-baseline leg import this package; the product package never does, and this
package never imports the product.  The arithmetic lives in the C file; this
module marshals numpy arrays and composes the oracle's own functions in the
order of Alg. 1 and Alg. 2.  The one exception are the products of the
weight-only objective at the end, which are their definition written as numpy
binary64 matrix products.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

NONE, INT8, INT4, E4M3, E5M2, E4M2, E4M1, E4M0 = 0, 1, 2, 3, 4, 5, 6, 7
SR, RTN = 0, 1
F32, BF16 = 0, 1
KIND_NAMES = {INT8: "int8", INT4: "int4", E4M3: "e4m3", E5M2: "e5m2", E4M2: "e4m2", E4M1: "e4m1", E4M0: "e4m0"}

_lib = C.CDLL(_build.build(force=False))

_u8p = C.POINTER(C.c_uint8)
_f32p = C.POINTER(C.c_float)
_u32p = C.POINTER(C.c_uint32)
_u64p = C.POINTER(C.c_uint64)

_lib.srq_oracle_threads.restype = C.c_int
_lib.srq_oracle_set_threads.argtypes = [C.c_int]
_lib.srq_oracle_Q.restype = C.c_double
_lib.srq_oracle_Q.argtypes = [C.c_double, C.c_double, C.c_double]
_lib.srq_oracle_philox4x32_10.argtypes = [_u32p, _u32p, _u32p]
_lib.srq_oracle_r16.restype = C.c_uint32
_lib.srq_oracle_r16.argtypes = [C.c_uint64, C.c_uint64, C.c_uint64]
_lib.srq_oracle_eps_from_r16.restype = C.c_float
_lib.srq_oracle_eps_from_r16.argtypes = [C.c_uint32]
_lib.srq_oracle_qmax.restype = C.c_float
_lib.srq_oracle_qmax.argtypes = [C.c_int]
_lib.srq_oracle_decode.restype = C.c_double
_lib.srq_oracle_decode.argtypes = [C.c_int, C.c_uint8]
_lib.srq_oracle_quantize_one.restype = C.c_uint8
_lib.srq_oracle_quantize_one.argtypes = [C.c_float, C.c_float, C.c_int, C.c_float]
_lib.srq_oracle_quantize.argtypes = [_u8p, C.c_void_p, C.c_int, C.c_size_t, C.c_int, C.c_int,
                                     C.c_float, C.c_uint64, C.c_uint64]
_lib.srq_oracle_sr_bf16_one.restype = C.c_uint16
_lib.srq_oracle_sr_bf16_one.argtypes = [C.c_float, C.c_float]
_lib.srq_oracle_update_bf16.argtypes = [C.POINTER(C.c_uint16), _f32p, C.c_float, C.c_size_t, C.c_int,
                                        C.c_uint64, C.c_uint64]
_lib.srq_oracle_pack_int4.argtypes = [_u8p, _u8p, C.c_size_t]
_lib.srq_oracle_unpack_int4.argtypes = [_u8p, _u8p, C.c_size_t]
_lib.srq_oracle_absmax_scale.restype = C.c_float
_lib.srq_oracle_absmax_scale.argtypes = [C.c_void_p, C.c_int, C.c_size_t, C.c_int]
_gemm_args = [_f32p, _f32p, _u8p, C.c_int, C.c_float, _u8p, C.c_int, C.c_float,
              C.c_size_t, C.c_size_t, C.c_size_t]
_gemm_at_args = [_f32p, _f32p, _u64p, C.c_size_t] + _gemm_args[2:]
for _n in ("fwd", "bwd_data", "bwd_weight"):
    getattr(_lib, "srq_oracle_" + _n).argtypes = _gemm_args
    getattr(_lib, "srq_oracle_" + _n + "_at").argtypes = _gemm_at_args


def threads() -> int:
    return _lib.srq_oracle_threads()


def set_threads(n: int) -> None:
    _lib.srq_oracle_set_threads(int(n))


def Q(x: float, delta: float, eps: float) -> float:
    """Threshold quantization function, Eq. 1, in binary64."""
    return _lib.srq_oracle_Q(x, delta, eps)


def philox4x32_10(ctr, key):
    c = (C.c_uint32 * 4)(*[int(v) & 0xFFFFFFFF for v in ctr])
    k = (C.c_uint32 * 2)(*[int(v) & 0xFFFFFFFF for v in key])
    o = (C.c_uint32 * 4)()
    _lib.srq_oracle_philox4x32_10(c, k, o)
    return [int(v) for v in o]


def r16(seed: int, counter_offset: int, i: int) -> int:
    return _lib.srq_oracle_r16(seed & (2**64 - 1), counter_offset & (2**64 - 1), i)


def eps_from_r16(r: int) -> float:
    return _lib.srq_oracle_eps_from_r16(r)


def qmax(kind: int) -> float:
    return _lib.srq_oracle_qmax(kind)


def decode(kind: int, code: int) -> float:
    return _lib.srq_oracle_decode(kind, code & 0xFF)


def decode_array(kind: int, codes: np.ndarray) -> np.ndarray:
    """Values (grid units, float64) of an array of unpacked codes."""
    table = np.array([decode(kind, c) for c in range(256)], dtype=np.float64)
    return table[np.asarray(codes, dtype=np.uint8)]


def quantize_one(x: float, inv: float, kind: int, eps: float) -> int:
    return _lib.srq_oracle_quantize_one(x, inv, kind, eps)


def sr_bf16_one(u: float, eps: float) -> int:
    """Eq. 1 on the bfloat16 grid: bit pattern of Q(u, eps)."""
    return _lib.srq_oracle_sr_bf16_one(u, eps)


def update_bf16(w_bits: np.ndarray, g: np.ndarray, eta: float, seed: int, counter_offset: int,
                round_mode: int = SR) -> np.ndarray:
    """Eq. 10: bfloat16 bit patterns of Q_SR(w - eta * g); w_bits is uint16, g float32."""
    w = np.ascontiguousarray(w_bits, dtype=np.uint16).copy()
    g = np.ascontiguousarray(g, dtype=np.float32)
    assert w.size == g.size
    _lib.srq_oracle_update_bf16(w.ctypes.data_as(C.POINTER(C.c_uint16)), g.ctypes.data_as(_f32p),
                                float(eta), w.size, round_mode, seed, counter_offset)
    return w


def _src(x: np.ndarray):
    x = np.ascontiguousarray(x)
    if x.dtype == np.float32:
        return x, F32
    if x.dtype == np.uint16:  # raw bfloat16 bit patterns
        return x, BF16
    raise TypeError("source must be float32, or uint16 holding bfloat16 bits")


def quantize(x: np.ndarray, kind: int, scale: float, seed: int, counter_offset: int,
             round_mode: int = SR) -> np.ndarray:
    """Unpacked codes (uint8, same shape as x; int4 sign-extended in the byte)."""
    x, dt = _src(x)
    codes = np.empty(x.shape, dtype=np.uint8)
    _lib.srq_oracle_quantize(codes.ctypes.data_as(_u8p), x.ctypes.data, dt, x.size, kind,
                             round_mode, np.float32(scale), seed & (2**64 - 1),
                             counter_offset & (2**64 - 1))
    return codes


def pack_int4(codes: np.ndarray) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    assert codes.size % 2 == 0
    out = np.empty(codes.size // 2, dtype=np.uint8)
    _lib.srq_oracle_pack_int4(out.ctypes.data_as(_u8p), codes.ctypes.data_as(_u8p), codes.size)
    return out


def unpack_int4(packed: np.ndarray) -> np.ndarray:
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    out = np.empty(packed.size * 2, dtype=np.uint8)
    _lib.srq_oracle_unpack_int4(out.ctypes.data_as(_u8p), packed.ctypes.data_as(_u8p), out.size)
    return out


def absmax_scale(x: np.ndarray, kind: int) -> float:
    x, dt = _src(x)
    return float(_lib.srq_oracle_absmax_scale(x.ctypes.data, dt, x.size, kind))


def _gemm(name, out_shape, X, kX, sX, Z, kZ, sZ, M, N, K, want_abs, at=None):
    X = np.ascontiguousarray(X, dtype=np.uint8)
    Z = np.ascontiguousarray(Z, dtype=np.uint8)
    if at is None:
        out = np.empty(out_shape, dtype=np.float32)
        ab = np.empty(out_shape, dtype=np.float32) if want_abs else None
        getattr(_lib, "srq_oracle_" + name)(
            out.ctypes.data_as(_f32p), ab.ctypes.data_as(_f32p) if want_abs else None,
            X.ctypes.data_as(_u8p), kX, np.float32(sX), Z.ctypes.data_as(_u8p), kZ,
            np.float32(sZ), M, N, K)
    else:
        at = np.ascontiguousarray(at, dtype=np.uint64)
        out = np.empty(at.size, dtype=np.float32)
        ab = np.empty(at.size, dtype=np.float32) if want_abs else None
        getattr(_lib, "srq_oracle_" + name + "_at")(
            out.ctypes.data_as(_f32p), ab.ctypes.data_as(_f32p) if want_abs else None,
            at.ctypes.data_as(_u64p), at.size,
            X.ctypes.data_as(_u8p), kX, np.float32(sX), Z.ctypes.data_as(_u8p), kZ,
            np.float32(sZ), M, N, K)
    return (out, ab) if want_abs else out


def gemm_fwd(Ac, kA, sA, Wc, kW, sW, want_abs=False, at=None):
    """Y = Ahat What^T from unpacked codes Ac (M,K), Wc (N,K).  Alg. 1."""
    M, K = Ac.shape
    N = Wc.shape[0]
    assert Wc.shape[1] == K
    return _gemm("fwd", (M, N), Ac, kA, sA, Wc, kW, sW, M, N, K, want_abs, at)


def gemm_bwd_data(dYc, kdY, sdY, Wc, kW, sW, want_abs=False, at=None):
    """dA = dYhat What from unpacked codes dYc (M,N), Wc (N,K).  Alg. 2."""
    M, N = dYc.shape
    K = Wc.shape[1]
    assert Wc.shape[0] == N
    return _gemm("bwd_data", (M, K), dYc, kdY, sdY, Wc, kW, sW, M, N, K, want_abs, at)


def gemm_bwd_weight(dYc, kdY, sdY, Ac, kA, sA, want_abs=False, at=None):
    """dW = dYhat^T Ahat from unpacked codes dYc (M,N), Ac (M,K).  Alg. 2."""
    M, N = dYc.shape
    K = Ac.shape[1]
    assert Ac.shape[0] == M
    return _gemm("bwd_weight", (N, K), dYc, kdY, sdY, Ac, kA, sA, M, N, K, want_abs, at)


class Quant:
    """One quantizer = (Delta, eps) of the paper: format, scale, RNG position."""

    def __init__(self, kind, scale, seed=0, counter_offset=0, round_mode=SR):
        self.kind, self.scale, self.seed = kind, float(np.float32(scale)), seed
        self.counter_offset, self.round_mode = counter_offset, round_mode

    def __call__(self, x):
        return quantize(x, self.kind, self.scale, self.seed, self.counter_offset, self.round_mode)


def linear_fwd(A, W, qA: Quant, qW: Quant, **kw):
    """Alg. 1: quantize A and W, multiply."""
    return gemm_fwd(qA(A), qA.kind, qA.scale, qW(W), qW.kind, qW.scale, **kw)


def linear_bwd_data(dY, W, qdY: Quant, qW: Quant, **kw):
    """Alg. 2, input-gradient product."""
    return gemm_bwd_data(qdY(dY), qdY.kind, qdY.scale, qW(W), qW.kind, qW.scale, **kw)


def linear_bwd_weight(dY, A, qdY: Quant, qA: Quant, **kw):
    """Alg. 2, weight-gradient product."""
    return gemm_bwd_weight(qdY(dY), qdY.kind, qdY.scale, qA(A), qA.kind, qA.scale, **kw)


# ---- weight-only quantization (Sec. 3.2: the objective with quantized weights and full-precision
# activations; Fig. 3).  Only W goes through Q; the other operand enters the product as it is.
# Plain definition: a binary64 matrix product of the operand with the dequantized codes (a
# binary32 number times a grid value is exact in binary64, and the sums of at most 2^17 such
# products lose less than 1e-11 relatively), then one rounding of scale * sum to binary32.
def _values64(x: np.ndarray) -> np.ndarray:
    x, dt = _src(x)
    if dt == BF16:
        return (x.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return x.astype(np.float64)


def _weight_only(X64, Wv64, scale, want_abs):
    s = np.float64(np.float32(scale))
    out = (s * (X64 @ Wv64)).astype(np.float32)
    if want_abs:
        return out, (s * (np.abs(X64) @ np.abs(Wv64))).astype(np.float32)
    return out


def linear_fwd_weight_only(A, W, qW: Quant, want_abs=False):
    """Y (M,N) = A What^T with A (M,K) unquantized and W (N,K) quantized by qW."""
    What = decode_array(qW.kind, qW(W)).astype(np.float64)
    return _weight_only(_values64(A), What.T, qW.scale, want_abs)


def linear_bwd_data_weight_only(dY, W, qW: Quant, want_abs=False):
    """dA (M,K) = dY What with dY (M,N) unquantized and W (N,K) quantized by qW (the same
    quantizer as in the forward pass gives the same What: one weight copy per mini-batch)."""
    What = decode_array(qW.kind, qW(W)).astype(np.float64)
    return _weight_only(_values64(dY), What, qW.scale, want_abs)


# ---- the estimator for the quantization-aware objective (Sec. 3.3, Fig. 3).  The forward pass
# multiplies the unquantized activation by What = Q(W; eps_W); the backward pass uses that SAME
# What (the weight thresholds carry no pass index: one copy per mini-batch) and stochastically
# rounds the saved activation and the output gradient.  A composition of the functions above.
def qat_pass(A, W, dY, qW: Quant, qA_bwd: Quant, qdY_bwd: Quant, want_abs=False):
    """(Y, dA, dW) with Y = A What^T, dA = dYhat What, dW = dYhat^T Ahat."""
    Y = linear_fwd_weight_only(A, W, qW, want_abs=want_abs)
    dA = linear_bwd_data(dY, W, qdY_bwd, qW, want_abs=want_abs)
    dW = linear_bwd_weight(dY, A, qdY_bwd, qA_bwd, want_abs=want_abs)
    return Y, dA, dW
