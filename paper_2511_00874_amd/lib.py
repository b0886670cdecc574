"""Thin ctypes binding over libsrq.so: same names as include/srq.h, argument marshalling only.

PyTorch is used for device memory and streams; every step of the path runs in the HIP
kernels.  There is no fallback: if the library is not built this module raises on import.
"""
import ctypes as C
import os

import torch  # first: its HIP runtime must be the one the library binds to

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libsrq.so")

OK = 0
F32, BF16 = 0, 1
NONE, INT8, INT4, E4M3, E5M2, E4M2, E4M1, E4M0 = 0, 1, 2, 3, 4, 5, 6, 7
SR, RTN = 0, 1
OP_FWD, OP_BWD_DATA, OP_BWD_WEIGHT, OP_BWD, OP_FWD_STASH, OP_BWD_STASHED = 0, 1, 2, 3, 4, 5
OP_FWD_WEIGHT_ONLY, OP_BWD_DATA_WEIGHT_ONLY = 6, 7
FLAG_F8_PIPELINE, FLAG_COUNTER_DEV, FLAG_QUANTIZE_ONCE = 1, 2, 4
PHASE_QUANTIZE, PHASE_PRODUCT, PHASE_BOTH = 1, 2, 3
KIND_NAMES = {INT8: "int8", INT4: "int4", E4M3: "e4m3", E5M2: "e5m2", E4M2: "e4m2", E4M1: "e4m1", E4M0: "e4m0"}
QMAX = {INT8: 127.0, INT4: 7.0, E4M3: 448.0, E5M2: 57344.0, E4M2: 448.0, E4M1: 384.0, E4M0: 256.0}


class srq_quant(C.Structure):
    _fields_ = [("kind", C.c_int32), ("round", C.c_int32), ("scale", C.c_float),
                ("flags", C.c_uint32), ("scale_dev", C.c_void_p), ("seed", C.c_uint64),
                ("counter_offset", C.c_uint64)]


class srq_absmax_req(C.Structure):
    _fields_ = [("x", C.c_void_p), ("dtype", C.c_int32), ("kind", C.c_int32), ("n", C.c_size_t),
                ("scale_out_dev", C.c_void_p)]


if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python -m paper_2511_00874_amd.build` "
        "(there is no CPU fallback)")
_lib = C.CDLL(LIB_PATH)

_vp, _sz, _qp = C.c_void_p, C.c_size_t, C.POINTER(srq_quant)
_lib.sr_absmax_scale.argtypes = [_vp, _vp, C.c_int, _sz, C.c_int, _vp]
_lib.sr_absmax_scales.argtypes = [C.POINTER(srq_absmax_req), C.c_int, _vp, _sz, _vp]
_lib.sr_absmax_workspace_bytes.argtypes = [C.POINTER(srq_absmax_req), C.c_int]
_lib.sr_absmax_workspace_bytes.restype = _sz
_lib.sr_quantize.argtypes = [_vp, _vp, C.c_int, _sz, _sz, C.c_int, _qp, _vp]
_lib.sr_gemm_codes.argtypes = [_vp, _vp, C.c_int, _vp, C.c_int, _sz, _sz, _sz, C.c_float, C.c_float,
                               _vp, _sz, _vp]
_lib.sr_gemm_workspace_bytes.argtypes = [_sz, _sz, _sz]
_lib.sr_gemm_workspace_bytes.restype = _sz
_lib.sr_gemm_bf16.argtypes = [_vp, _vp, _vp, _sz, _sz, _sz, C.c_float, C.c_float, _vp, _sz, _vp]
_lib.sr_gemm_bf16_workspace_bytes.argtypes = [_sz, _sz, _sz]
_lib.sr_gemm_bf16_workspace_bytes.restype = _sz
_lib.sr_gemm_e5m2.argtypes = _lib.sr_gemm_bf16.argtypes
_lib.sr_gemm_e5m2_workspace_bytes.argtypes = [_sz, _sz, _sz]
_lib.sr_gemm_e5m2_workspace_bytes.restype = _sz
_lib.sr_linear_fwd.argtypes = [_vp, _vp, C.c_int, _vp, C.c_int, _sz, _sz, _sz, _qp, _qp, _vp, _sz, _vp]
_lib.sr_linear_bwd_data.argtypes = _lib.sr_linear_fwd.argtypes
_lib.sr_linear_fwd_static.argtypes = [_vp, _vp, C.c_int, _vp, C.c_int, _sz, _sz, _sz, _qp, _qp, _vp]
_lib.sr_linear_fwd_fused.argtypes = _lib.sr_linear_fwd_static.argtypes
_lib.sr_linear_fwd_phase.argtypes = [_vp, _vp, C.c_int, _vp, C.c_int, _sz, _sz, _sz, _qp, _qp, _vp, _sz, C.c_int, _vp]
_lib.sr_linear_fwd_static_limit.argtypes = []
_lib.sr_linear_fwd_static_limit.restype = _sz
_lib.sr_linear_bwd_weight.argtypes = [_vp, _vp, C.c_int, _vp, C.c_int, _sz, _sz, _sz, _qp, _qp,
                                      C.c_float, _vp, _sz, _vp]
_lib.sr_linear_bwd.argtypes = [_vp, _vp, _vp, C.c_int, _vp, C.c_int, _vp, C.c_int, _sz, _sz, _sz, _qp, _qp, _qp,
                               C.c_float, _vp, _sz, _vp]
_lib.sr_linear_bwd_phase.argtypes = [_vp, _vp, _vp, C.c_int, _vp, C.c_int, _vp, C.c_int, _sz, _sz, _sz, _qp, _qp, _qp,
                                     C.c_float, _vp, _sz, C.c_int, _vp]
_lib.sr_linear_workspace_bytes.argtypes = [C.c_int, _sz, _sz, _sz]
_lib.sr_linear_workspace_bytes.restype = _sz
_lib.sr_linear_stash_bytes.argtypes = [_sz, _sz, _sz]
_lib.sr_linear_stash_bytes.restype = _sz
_lib.sr_linear_fwd_stash.argtypes = [_vp, _vp, C.c_int, _vp, C.c_int, _sz, _sz, _sz, _qp, _qp, _qp, _qp, _vp, _sz, _vp, _sz, _vp]
_lib.sr_linear_bwd_stashed.argtypes = [_vp, _vp, _vp, C.c_int, _sz, _sz, _sz, _qp, _qp, _qp, _vp, _sz, C.c_float, _vp, _sz, _vp]
_lib.sr_linear_fwd_stash_phase.argtypes = [_vp, _vp, C.c_int, _vp, C.c_int, _sz, _sz, _sz, _qp, _qp, _qp, _qp, _vp, _sz, _vp, _sz,
                                           C.c_int, _vp]
_lib.sr_linear_bwd_stashed_phase.argtypes = [_vp, _vp, _vp, C.c_int, _sz, _sz, _sz, _qp, _qp, _qp, _vp, _sz, C.c_float, _vp, _sz,
                                             C.c_int, _vp]
_lib.sr_update_bf16.argtypes = [_vp, _vp, C.c_float, _sz, C.c_int, C.c_uint64, C.c_uint64, _vp]
_lib.sr_status_string.argtypes = [C.c_int]
_lib.sr_status_string.restype = C.c_char_p
for _n in ("sr_linear_fwd_static", "sr_linear_fwd_fused", "sr_linear_fwd_phase", "sr_linear_bwd_phase", "sr_absmax_scale", "sr_absmax_scales", "sr_quantize", "sr_gemm_codes", "sr_gemm_bf16", "sr_gemm_e5m2", "sr_linear_fwd", "sr_linear_bwd_data",
           "sr_linear_bwd_weight", "sr_linear_bwd", "sr_update_bf16", "sr_linear_fwd_stash", "sr_linear_bwd_stashed",
           "sr_linear_fwd_stash_phase", "sr_linear_bwd_stashed_phase"):
    getattr(_lib, _n).restype = C.c_int

EXPORTS = ["sr_absmax_scale", "sr_absmax_scales", "sr_absmax_workspace_bytes", "sr_quantize", "sr_gemm_codes", "sr_gemm_workspace_bytes", "sr_gemm_bf16", "sr_gemm_bf16_workspace_bytes", "sr_gemm_e5m2", "sr_gemm_e5m2_workspace_bytes",
           "sr_linear_fwd", "sr_linear_bwd_data", "sr_linear_bwd_weight", "sr_linear_bwd",
           "sr_linear_workspace_bytes", "sr_linear_stash_bytes", "sr_linear_fwd_stash", "sr_linear_bwd_stashed",
           "sr_update_bf16", "sr_status_string", "sr_linear_fwd_static", "sr_linear_fwd_static_limit",
           "sr_linear_fwd_fused", "sr_linear_fwd_phase", "sr_linear_bwd_phase", "sr_linear_fwd_stash_phase",
           "sr_linear_bwd_stashed_phase"]

raw = _lib  # the C entry points themselves, for tests of the error paths


class SrqError(RuntimeError):
    def __init__(self, status):
        self.status = status
        super().__init__(f"srq status {status}: {_lib.sr_status_string(status).decode()}")


def _check(status):
    if status != OK:
        raise SrqError(status)


def status_string(status):
    return _lib.sr_status_string(status).decode()


def _dtype(t):
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError("source tensors must be float32 or bfloat16")


def _dev(t):
    if not t.is_cuda:
        raise RuntimeError("srq needs device tensors: there is no CPU path")
    if not t.is_contiguous():
        raise ValueError("tensors must be dense row-major")
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


class Quant:
    """One quantizer (Delta, eps): format, per-tensor scale (float or 1-element device tensor),
    rounding mode and position in the Philox stream."""

    def __init__(self, kind, scale, seed=0, counter_offset=0, round_mode=SR, flags=0):
        self.kind, self.scale, self.seed = kind, scale, seed
        self.counter_offset, self.round_mode, self.flags = counter_offset, round_mode, flags

    def c(self):
        q = srq_quant()
        q.kind, q.round, q.flags = self.kind, self.round_mode, self.flags
        if isinstance(self.scale, torch.Tensor):
            q.scale, q.scale_dev = 0.0, _dev(self.scale)
        else:
            q.scale, q.scale_dev = float(self.scale), None
        q.seed = self.seed & (2**64 - 1)
        if isinstance(self.counter_offset, torch.Tensor):
            # a 1-element int64 device tensor: the kernels read the offset when they run
            assert self.counter_offset.dtype == torch.int64 and self.counter_offset.numel() == 1
            q.flags |= FLAG_COUNTER_DEV
            q.counter_offset = _dev(self.counter_offset)
        else:
            q.counter_offset = self.counter_offset & (2**64 - 1)
        return q


def sr_absmax_scale(x, kind, out=None):
    """Device tensor holding max|x| / Qmax(kind) (1 if x is all zero)."""
    if out is None:
        out = torch.empty(1, dtype=torch.float32, device=x.device)
    _check(_lib.sr_absmax_scale(_dev(out), _dev(x), _dtype(x), x.numel(), kind, _stream()))
    return out


class AbsmaxBatch:
    """Prepared sr_absmax_scales call: requests [(tensor, kind, out 1-element tensor)], marshalled once."""

    def __init__(self, requests):
        self.keep = requests
        self.count = len(requests)
        self.reqs = (srq_absmax_req * self.count)()
        for r, (x, kind, out) in zip(self.reqs, requests):
            r.x, r.dtype, r.kind, r.n, r.scale_out_dev = _dev(x), _dtype(x), kind, x.numel(), _dev(out)
        need = _lib.sr_absmax_workspace_bytes(self.reqs, self.count)
        self.ws = torch.empty(max(need, 4), dtype=torch.uint8, device=requests[0][0].device)

    def run(self):
        _check(_lib.sr_absmax_scales(self.reqs, self.count, _dev(self.ws), self.ws.numel(), _stream()))


def sr_absmax_scales(requests):
    """requests: [(tensor, kind, out 1-element device tensor)]; all scales in two launches."""
    AbsmaxBatch(requests).run()


def sr_linear_stash_bytes(M, N, K):
    return _lib.sr_linear_stash_bytes(M, N, K)


def sr_linear_fwd_stash(A, W, qA, qW, qA_bwd, qW_bwd, stash=None, out=None, workspace=None, phase=PHASE_BOTH):
    """Alg. 1 that also saves Q(A; qA_bwd)^T and Q(W; qW_bwd)^T in code form: returns (Y, stash).
    `phase`: the quantizer launch, the product, or both (the halves take the same out, stash, workspace)."""
    M, K = A.shape
    N = W.shape[0]
    if out is None:
        out = torch.empty((M, N), dtype=torch.float32, device=A.device)
    if stash is None:
        stash = torch.empty(sr_linear_stash_bytes(M, N, K), dtype=torch.uint8, device=A.device)
    ws = _ws(OP_FWD_STASH, M, N, K, workspace, A.device)
    _check(_lib.sr_linear_fwd_stash_phase(_dev(out), _dev(A), _dtype(A), _dev(W), _dtype(W), M, N, K, C.byref(qA.c()),
                                          C.byref(qW.c()), C.byref(qA_bwd.c()), C.byref(qW_bwd.c()), _dev(stash),
                                          stash.numel(), _dev(ws), ws.numel(), phase, _stream()))
    return out, stash


def sr_linear_bwd_stashed(dY, stash, K, qdY, qW, qA, out_dA=None, out_dW=None, beta=0.0, workspace=None,
                          phase=PHASE_BOTH):
    """Alg. 2 from the stash of sr_linear_fwd_stash: (dA, dW); only dY is read.  `phase` as above."""
    M, N = dY.shape
    if out_dA is None:
        out_dA = torch.empty((M, K), dtype=torch.float32, device=dY.device)
    if out_dW is None:
        out_dW = torch.empty((N, K), dtype=torch.float32, device=dY.device)
    ws = _ws(OP_BWD_STASHED, M, N, K, workspace, dY.device)
    _check(_lib.sr_linear_bwd_stashed_phase(_dev(out_dA), _dev(out_dW), _dev(dY), _dtype(dY), M, N, K, C.byref(qdY.c()),
                                            C.byref(qW.c()), C.byref(qA.c()), _dev(stash), stash.numel(), beta, _dev(ws),
                                            ws.numel(), phase, _stream()))
    return out_dA, out_dW


def sr_update_bf16(w, g, eta, seed=0, counter_offset=0, round_mode=SR):
    """Eq. 10 in place: w (bfloat16 tensor) <- Q(w - eta * g), g float32 of the same size."""
    assert w.dtype == torch.bfloat16 and g.dtype == torch.float32 and w.numel() == g.numel()
    assert w.is_contiguous() and g.is_contiguous()
    _check(_lib.sr_update_bf16(_dev(w), _dev(g), float(eta), w.numel(), round_mode, seed, counter_offset, _stream()))
    return w


def sr_quantize(x, q, transpose_out=False, out=None):
    """Codes of x (2-D, or 1-D treated as one row): uint8, packed two per byte for INT4."""
    rows, cols = (1, x.numel()) if x.dim() == 1 else x.shape
    n = rows * cols
    nbytes = n // 2 if q.kind == INT4 else n
    if out is None:
        out = torch.empty(max(nbytes, 1), dtype=torch.uint8, device=x.device)[:nbytes]
    _check(_lib.sr_quantize(_dev(out), _dev(x), _dtype(x), rows, cols, int(bool(transpose_out)),
                            C.byref(q.c()), _stream()))
    return out


def sr_gemm_workspace_bytes(P, Q, R):
    return _lib.sr_gemm_workspace_bytes(P, Q, R)


def sr_gemm_codes(X, kindX, Z, kindZ, alpha=1.0, out=None, beta=0.0, workspace=None):
    """out (P,Q) = alpha * X (P,R) . Z (Q,R)^T on codes, one byte per element."""
    P, R = X.shape
    Q = Z.shape[0]
    if out is None:
        out = torch.empty((P, Q), dtype=torch.float32, device=X.device)
    need = sr_gemm_workspace_bytes(P, Q, R)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=X.device)
    _check(_lib.sr_gemm_codes(_dev(out), _dev(X), kindX, _dev(Z), kindZ, P, Q, R, alpha, beta,
                              _dev(workspace) if workspace is not None else None,
                              workspace.numel() if workspace is not None else 0, _stream()))
    return out


def sr_gemm_bf16(X, Z, alpha=1.0, out=None, beta=0.0, workspace=None):
    """out (P,Q) = alpha * X (P,R) . Z (Q,R)^T for bfloat16 operands."""
    P, R = X.shape
    Q = Z.shape[0]
    if out is None:
        out = torch.empty((P, Q), dtype=torch.float32, device=X.device)
    need = _lib.sr_gemm_bf16_workspace_bytes(P, Q, R)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=X.device)
    _check(_lib.sr_gemm_bf16(_dev(out), _dev(X), _dev(Z), P, Q, R, alpha, beta,
                             _dev(workspace) if workspace is not None else None,
                             workspace.numel() if workspace is not None else 0, _stream()))
    return out


def sr_gemm_e5m2(X, Z, alpha=1.0, beta=0.0, out=None, workspace=None):
    """out (P,Q) = alpha * X Z^T for uint8 matrices of E5M2 codes: exact products, binary32 sums."""
    P, R = X.shape
    Q = Z.shape[0]
    if out is None:
        out = torch.empty((P, Q), dtype=torch.float32, device=X.device)
    need = _lib.sr_gemm_e5m2_workspace_bytes(P, Q, R)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=X.device)
    _check(_lib.sr_gemm_e5m2(_dev(out), _dev(X), _dev(Z), P, Q, R, alpha, beta,
                             _dev(workspace) if workspace is not None else None,
                             workspace.numel() if workspace is not None else 0, _stream()))
    return out


def sr_linear_workspace_bytes(op, M, N, K):
    return _lib.sr_linear_workspace_bytes(op, M, N, K)


def _ws(op, M, N, K, workspace, device):
    need = sr_linear_workspace_bytes(op, M, N, K)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=device)
    return workspace


def sr_linear_fwd(A, W, qA, qW, out=None, workspace=None, phase=None):
    """Alg. 1: Y (M,N) = Q(A) Q(W)^T, A (M,K), W (N,K).  qA = Quant(NONE, 1.0): A as it is
    (weight-only objective, Sec. 3.2).  phase = PHASE_QUANTIZE / PHASE_PRODUCT: one half of the call
    (sr_linear_fwd_phase); `out` and `workspace` are then required."""
    M, K = A.shape
    N = W.shape[0]
    if phase is not None:
        _check(_lib.sr_linear_fwd_phase(_dev(out), _dev(A), _dtype(A), _dev(W), _dtype(W), M, N, K, C.byref(qA.c()),
                                        C.byref(qW.c()), _dev(workspace), workspace.numel(), phase, _stream()))
        return out
    if out is None:
        out = torch.empty((M, N), dtype=torch.float32, device=A.device)
    ws = _ws(OP_FWD_WEIGHT_ONLY if qA.kind == NONE else OP_FWD, M, N, K, workspace, A.device)
    _check(_lib.sr_linear_fwd(_dev(out), _dev(A), _dtype(A), _dev(W), _dtype(W), M, N, K,
                              C.byref(qA.c()), C.byref(qW.c()), _dev(ws), ws.numel(), _stream()))
    return out


def sr_linear_fwd_static(A, W, qA, qW, out):
    """sr_linear_fwd with the library's static scratch array as workspace; `out` is required (this
    call is for callers that may not allocate)."""
    M, K = A.shape
    N = W.shape[0]
    _check(_lib.sr_linear_fwd_static(_dev(out), _dev(A), _dtype(A), _dev(W), _dtype(W), M, N, K,
                                     C.byref(qA.c()), C.byref(qW.c()), _stream()))
    return out


def sr_linear_fwd_fused(A, W, qA, qW, out=None):
    """Alg. 1 with the quantizers inside the product kernel (no workspace, no codes in memory)."""
    M, K = A.shape
    N = W.shape[0]
    if out is None:
        out = torch.empty((M, N), dtype=torch.float32, device=A.device)
    _check(_lib.sr_linear_fwd_fused(_dev(out), _dev(A), _dtype(A), _dev(W), _dtype(W), M, N, K,
                                    C.byref(qA.c()), C.byref(qW.c()), _stream()))
    return out


def sr_linear_bwd_data(dY, W, qdY, qW, out=None, workspace=None):
    """Alg. 2: dA (M,K) = Q(dY) Q(W), dY (M,N), W (N,K).  qdY = Quant(NONE, 1.0): dY as it is."""
    M, N = dY.shape
    K = W.shape[1]
    if out is None:
        out = torch.empty((M, K), dtype=torch.float32, device=dY.device)
    ws = _ws(OP_BWD_DATA_WEIGHT_ONLY if qdY.kind == NONE else OP_BWD_DATA, M, N, K, workspace, dY.device)
    _check(_lib.sr_linear_bwd_data(_dev(out), _dev(dY), _dtype(dY), _dev(W), _dtype(W), M, N, K,
                                   C.byref(qdY.c()), C.byref(qW.c()), _dev(ws), ws.numel(), _stream()))
    return out


def sr_linear_bwd_weight(dY, A, qdY, qA, out=None, beta=0.0, workspace=None):
    """Alg. 2: dW (N,K) = beta * dW + Q(dY)^T Q(A), dY (M,N), A (M,K)."""
    M, N = dY.shape
    K = A.shape[1]
    if out is None:
        out = torch.empty((N, K), dtype=torch.float32, device=dY.device)
    ws = _ws(OP_BWD_WEIGHT, M, N, K, workspace, dY.device)
    _check(_lib.sr_linear_bwd_weight(_dev(out), _dev(dY), _dtype(dY), _dev(A), _dtype(A), M, N, K,
                                     C.byref(qdY.c()), C.byref(qA.c()), beta, _dev(ws), ws.numel(),
                                     _stream()))
    return out


def sr_linear_bwd(dY, W, A, qdY, qW, qA, out_dA=None, out_dW=None, beta=0.0, workspace=None, phase=None):
    """Alg. 2 in one call: (dA, dW), with dY read and quantized once.  phase = PHASE_QUANTIZE /
    PHASE_PRODUCT: one half of the call (sr_linear_bwd_phase); outputs and workspace are then required."""
    M, N = dY.shape
    K = W.shape[1]
    if phase is not None:
        _check(_lib.sr_linear_bwd_phase(_dev(out_dA), _dev(out_dW), _dev(dY), _dtype(dY), _dev(W), _dtype(W), _dev(A),
                                        _dtype(A), M, N, K, C.byref(qdY.c()), C.byref(qW.c()), C.byref(qA.c()), beta,
                                        _dev(workspace), workspace.numel(), phase, _stream()))
        return out_dA, out_dW
    if out_dA is None:
        out_dA = torch.empty((M, K), dtype=torch.float32, device=dY.device)
    if out_dW is None:
        out_dW = torch.empty((N, K), dtype=torch.float32, device=dY.device)
    ws = _ws(OP_BWD, M, N, K, workspace, dY.device)
    _check(_lib.sr_linear_bwd(_dev(out_dA), _dev(out_dW), _dev(dY), _dtype(dY), _dev(W), _dtype(W), _dev(A),
                              _dtype(A), M, N, K, C.byref(qdY.c()), C.byref(qW.c()), C.byref(qA.c()), beta,
                              _dev(ws), ws.numel(), _stream()))
    return out_dA, out_dW
