// C ABI: argument checks and the composition of quantizer and product launches that makes
// up Alg. 1 (forward) and Alg. 2 (backward).  Nothing here computes; every step of the path
// runs in the kernels of srq_quantize.hip and srq_gemm.hip.
#include <cmath>

#include "srq_internal.hpp"

using namespace srq;

namespace {

constexpr size_t WS_ALIGN = 256;
size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bool kind_ok(int k) { return k == SRQ_INT8 || k == SRQ_INT4 || k == SRQ_E4M3 || k == SRQ_E5M2; }
bool dtype_ok(int d) { return d == SRQ_F32 || d == SRQ_BF16; }

int check_quant(const srq_quant* q) {
  if (!q) return SRQ_ERR_NULL;
  if (q->kind == SRQ_NONE) return SRQ_ERR_UNSUPPORTED;  // Delta = 0 (identity) has no code form
  if (!kind_ok(q->kind)) return SRQ_ERR_FORMAT;
  if (q->round != SRQ_SR && q->round != SRQ_RTN) return SRQ_ERR_FORMAT;
  if (q->flags & ~(uint32_t)SRQ_FLAG_F8_PIPELINE) return SRQ_ERR_FORMAT;
  if (!q->scale_dev) {
    const float s = q->scale;
    if (!(s > 0.0f) || !std::isfinite(s) || !std::isfinite(1.0f / s)) return SRQ_ERR_FORMAT;
  }
  return SRQ_OK;
}

QuantArgs make_args(const srq_quant* q, int dtype, int store) {
  QuantArgs a;
  a.kind = q->kind; a.round = q->round; a.dtype = dtype; a.store = store;
  a.scale = q->scale; a.scale_dev = q->scale_dev;
  a.seed = q->seed; a.counter_offset = q->counter_offset;
  return a;
}

bool fits_u32(size_t v) { return v <= 0xFFFFFFFFull; }

// Both operands of a product must be integer codes or both 8-bit float codes.
int check_pair(int kx, int kz) {
  if (kind_is_int(kx) && kind_is_int(kz)) return SRQ_OK;
  if (kind_is_f8(kx) && kind_is_f8(kz)) return SRQ_OK;
  return SRQ_ERR_UNSUPPORTED;
}

// Matrix pipeline for a product of two quantized operands; -1 if the two disagree.
int pick_pipe(const srq_quant* qx, const srq_quant* qz) {
  if (kind_is_int(qx->kind)) return PIPE_I8;
  const bool fx = qx->flags & SRQ_FLAG_F8_PIPELINE, fz = qz->flags & SRQ_FLAG_F8_PIPELINE;
  if (fx != fz) return -1;
  return fx ? PIPE_F8 : PIPE_BF16;
}

// int32 accumulation is exact while R * 127^2 < 2^31
bool int_contraction_ok(int kx, size_t R) { return !kind_is_int(kx) || R * 16129ull < (1ull << 31); }

struct LinearLayout {
  size_t x_bytes, z_bytes, gemm_bytes, total;
};

// Workspace: [codes of the row operand | codes of the column operand | split partials]
LinearLayout linear_layout(size_t P, size_t Q, size_t R, int pipe) {
  LinearLayout l;
  const size_t es = pipe == PIPE_BF16 ? 2 : 1;
  l.x_bytes = align_up(P * R * es, WS_ALIGN);
  l.z_bytes = align_up(Q * R * es, WS_ALIGN);
  l.gemm_bytes = align_up(gemm_workspace_bytes(P, Q, R, pipe), WS_ALIGN);
  l.total = l.x_bytes + l.z_bytes + l.gemm_bytes;
  return l;
}

// One product of Alg. 1 / Alg. 2: quantize both operands into the workspace with the
// contraction index contiguous, then multiply the codes.
//   out (P x Q) = Q(x)[P x R] . Q(z)[Q x R]^T,  x given as xr x xc (transposed if x_tr), same for z
int run_linear(float* out, const void* x, int dtx, size_t xr, size_t xc, int x_tr, const srq_quant* qx,
               const void* z, int dtz, size_t zr, size_t zc, int z_tr, const srq_quant* qz, size_t P,
               size_t Q, size_t R, float beta, void* workspace, size_t workspace_bytes, void* stream) {
  if (!out || !x || !z) return SRQ_ERR_NULL;
  int st = check_quant(qx);
  if (st != SRQ_OK) return st;
  st = check_quant(qz);
  if (st != SRQ_OK) return st;
  if (!dtype_ok(dtx) || !dtype_ok(dtz)) return SRQ_ERR_FORMAT;
  if (P == 0 || Q == 0 || R == 0) return SRQ_ERR_SHAPE;
  if (!fits_u32(P) || !fits_u32(Q) || !fits_u32(R)) return SRQ_ERR_SHAPE;
  if ((P % 16) || (Q % 16) || (R % 16)) return SRQ_ERR_ALIGN;
  if (!aligned16(out) || !aligned16(x) || !aligned16(z)) return SRQ_ERR_ALIGN;
  if (beta != 0.0f && beta != 1.0f) return SRQ_ERR_UNSUPPORTED;
  st = check_pair(qx->kind, qz->kind);
  if (st != SRQ_OK) return st;
  if (!int_contraction_ok(qx->kind, R)) return SRQ_ERR_UNSUPPORTED;
  const int pipe = pick_pipe(qx, qz);
  if (pipe < 0) return SRQ_ERR_UNSUPPORTED;
  if (!gemm_operands_addressable(P, Q, R, pipe)) return SRQ_ERR_UNSUPPORTED;
  const int store = pipe == PIPE_BF16 ? STORE_BF16 : STORE_BYTE;
  const LinearLayout l = linear_layout(P, Q, R, pipe);
  if (!workspace || workspace_bytes < l.total || (reinterpret_cast<uintptr_t>(workspace) & 255u))
    return SRQ_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  uint8_t* xcodes = static_cast<uint8_t*>(workspace);
  uint8_t* zcodes = xcodes + l.x_bytes;
  void* gws = zcodes + l.z_bytes;
  if (launch_quantize(xcodes, x, xr, xc, x_tr, make_args(qx, dtx, store), s) != hipSuccess)
    return SRQ_ERR_HIP;
  if (launch_quantize(zcodes, z, zr, zc, z_tr, make_args(qz, dtz, store), s) != hipSuccess)
    return SRQ_ERR_HIP;
  GemmScale sc{1.0f, qx->scale, qz->scale, qx->scale_dev, qz->scale_dev};
  if (launch_gemm_codes(out, xcodes, qx->kind, zcodes, qz->kind, P, Q, R, R * (pipe == PIPE_BF16 ? 2 : 1), pipe, sc,
                        beta == 1.0f, gws, s) !=
      hipSuccess)
    return SRQ_ERR_HIP;
  return SRQ_OK;
}

}  // namespace

extern "C" {

int sr_absmax_scale(float* scale_out_dev, const void* x, int dtype, size_t n, int kind, void* stream) {
  if (!scale_out_dev || (!x && n > 0)) return SRQ_ERR_NULL;
  if (!kind_ok(kind) || !dtype_ok(dtype)) return SRQ_ERR_FORMAT;
  if (!aligned16(x)) return SRQ_ERR_ALIGN;
  return launch_absmax_scale(scale_out_dev, x, dtype, n, kind, static_cast<hipStream_t>(stream)) == hipSuccess
             ? SRQ_OK
             : SRQ_ERR_HIP;
}

int sr_quantize(void* codes, const void* x, int dtype, size_t rows, size_t cols, int transpose_out,
                const srq_quant* q, void* stream) {
  const int st = check_quant(q);
  if (st != SRQ_OK) return st;
  if (!dtype_ok(dtype)) return SRQ_ERR_FORMAT;
  if (rows != 0 && cols > SIZE_MAX / rows) return SRQ_ERR_SHAPE;
  const size_t n = rows * cols;
  if (n == 0) return SRQ_OK;
  if (!codes || !x) return SRQ_ERR_NULL;
  if (!aligned16(x) || !aligned16(codes)) return SRQ_ERR_ALIGN;
  if (transpose_out != 0 && transpose_out != 1) return SRQ_ERR_FORMAT;
  if (q->kind == SRQ_INT4 && (n % 2)) return SRQ_ERR_ALIGN;
  if (transpose_out) {
    if (!fits_u32(rows) || !fits_u32(cols)) return SRQ_ERR_SHAPE;
    if (cols % 8) return SRQ_ERR_ALIGN;
    if (q->kind == SRQ_INT4 && (rows % 2)) return SRQ_ERR_ALIGN;
  }
  const int store = q->kind == SRQ_INT4 ? STORE_NIBBLE : STORE_BYTE;
  return launch_quantize(codes, x, rows, cols, transpose_out, make_args(q, dtype, store),
                         static_cast<hipStream_t>(stream)) == hipSuccess
             ? SRQ_OK
             : SRQ_ERR_HIP;
}

size_t sr_gemm_workspace_bytes(size_t P, size_t Q, size_t R) {
  if (P == 0 || Q == 0 || R == 0) return 0;
  return gemm_workspace_bytes(P, Q, R, PIPE_I8);  // same plan for both one-byte pipelines
}

int sr_gemm_codes(float* out, const void* X, int kindX, const void* Z, int kindZ, size_t P, size_t Q,
                  size_t R, float alpha, float beta, void* workspace, size_t workspace_bytes,
                  void* stream) {
  if (!out || !X || !Z) return SRQ_ERR_NULL;
  if (!kind_ok(kindX) || !kind_ok(kindZ)) return SRQ_ERR_FORMAT;
  if (P == 0 || Q == 0 || R == 0) return SRQ_ERR_SHAPE;
  if (!fits_u32(P) || !fits_u32(Q) || !fits_u32(R)) return SRQ_ERR_SHAPE;
  if (R % 16) return SRQ_ERR_ALIGN;
  if (!aligned16(out) || !aligned16(X) || !aligned16(Z)) return SRQ_ERR_ALIGN;
  if (beta != 0.0f && beta != 1.0f) return SRQ_ERR_UNSUPPORTED;
  const int st = check_pair(kindX, kindZ);
  if (st != SRQ_OK) return st;
  if (!int_contraction_ok(kindX, R)) return SRQ_ERR_UNSUPPORTED;
  const int pipe = kind_is_int(kindX) ? PIPE_I8 : PIPE_F8;
  if (!gemm_operands_addressable(P, Q, R, pipe)) return SRQ_ERR_UNSUPPORTED;
  const size_t need = gemm_workspace_bytes(P, Q, R, pipe);
  if (need > 0 && (!workspace || workspace_bytes < need || !aligned16(workspace))) return SRQ_ERR_WORKSPACE;
  GemmScale sc{alpha, 1.0f, 1.0f, nullptr, nullptr};
  return launch_gemm_codes(out, static_cast<const uint8_t*>(X), kindX, static_cast<const uint8_t*>(Z), kindZ,
                           P, Q, R, R, pipe, sc, beta == 1.0f, workspace, static_cast<hipStream_t>(stream)) == hipSuccess
             ? SRQ_OK
             : SRQ_ERR_HIP;
}

size_t sr_linear_workspace_bytes(int op, size_t M, size_t N, size_t K) {
  if (M == 0 || N == 0 || K == 0) return 0;
  // sized for the widest operand storage (two bytes per element), so that one buffer serves
  // every format
  auto widest = [](size_t P, size_t Q, size_t R) {
    const size_t a = linear_layout(P, Q, R, PIPE_BF16).total, b = linear_layout(P, Q, R, PIPE_I8).total;
    return a > b ? a : b;
  };
  switch (op) {
    case SRQ_OP_FWD: return widest(M, N, K);         // Y  (M x N), contraction K
    case SRQ_OP_BWD_DATA: return widest(M, K, N);    // dA (M x K), contraction N
    case SRQ_OP_BWD_WEIGHT: return widest(N, K, M);  // dW (N x K), contraction M
    default: return 0;
  }
}

// Alg. 1: Y = Ahat What^T.  A (M x K) and W (N x K) already have K contiguous.
int sr_linear_fwd(float* Y, const void* A, int dtypeA, const void* W, int dtypeW, size_t M, size_t N,
                  size_t K, const srq_quant* qA_fwd, const srq_quant* qW_fwd, void* workspace,
                  size_t workspace_bytes, void* stream) {
  return run_linear(Y, A, dtypeA, M, K, 0, qA_fwd, W, dtypeW, N, K, 0, qW_fwd, M, N, K, 0.0f, workspace,
                    workspace_bytes, stream);
}

// Alg. 2: dA = dYhat What.  Contraction over N: dY (M x N) as is, W (N x K) written as K x N.
int sr_linear_bwd_data(float* dA, const void* dY, int dtypedY, const void* W, int dtypeW, size_t M,
                       size_t N, size_t K, const srq_quant* qdY_bwd, const srq_quant* qW_bwd,
                       void* workspace, size_t workspace_bytes, void* stream) {
  return run_linear(dA, dY, dtypedY, M, N, 0, qdY_bwd, W, dtypeW, N, K, 1, qW_bwd, M, K, N, 0.0f,
                    workspace, workspace_bytes, stream);
}

// Alg. 2: dW = dYhat^T Ahat.  Contraction over M: dY written as N x M, A written as K x M.
int sr_linear_bwd_weight(float* dW, const void* dY, int dtypedY, const void* A, int dtypeA, size_t M,
                         size_t N, size_t K, const srq_quant* qdY_bwd, const srq_quant* qA_bwd, float beta,
                         void* workspace, size_t workspace_bytes, void* stream) {
  return run_linear(dW, dY, dtypedY, M, N, 1, qdY_bwd, A, dtypeA, M, K, 1, qA_bwd, N, K, M, beta,
                    workspace, workspace_bytes, stream);
}

const char* sr_status_string(int status) {
  switch (status) {
    case SRQ_OK: return "ok";
    case SRQ_ERR_NULL: return "null pointer";
    case SRQ_ERR_SHAPE: return "bad shape";
    case SRQ_ERR_FORMAT: return "bad format, rounding mode, dtype or scale";
    case SRQ_ERR_ALIGN: return "pointer or dimension not aligned";
    case SRQ_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case SRQ_ERR_UNSUPPORTED: return "unsupported combination";
    case SRQ_ERR_HIP: return "HIP launch error";
    default: return "unknown status";
  }
}

}  // extern "C"
