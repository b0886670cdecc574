// C ABI: argument checks and the composition of quantizer and product launches that makes
// up Alg. 1 (forward) and Alg. 2 (backward).  Nothing here computes; every step of the path
// runs in the kernels of srq_quantize.hip and srq_gemm.hip.
#include <cmath>
#include <mutex>

#include "srq_internal.hpp"

using namespace srq;

// Device memory of the allocation-free entry point (sr_linear_fwd_static): the workspace that
// sr_linear_fwd takes from its caller, as a file-scope array.  Every GPU the library runs on
// holds its own copy at its own address until the process ends.  In host code this name is only
// a handle for hipGetSymbolAddress; kernels and copies get the address that call returns.
static __device__ __align__(256) unsigned char scratch[SRQ_STATIC_SCRATCH_BYTES];

namespace {

constexpr size_t WS_ALIGN = 256;
size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bool kind_ok(int k) { return k >= SRQ_INT8 && k <= SRQ_E4M0; }
bool dtype_ok(int d) { return d == SRQ_F32 || d == SRQ_BF16; }

int check_quant(const srq_quant* q) {
  if (!q) return SRQ_ERR_NULL;
  if (q->kind == SRQ_NONE) return SRQ_ERR_UNSUPPORTED;  // Delta = 0 (identity) has no code form
  if (!kind_ok(q->kind)) return SRQ_ERR_FORMAT;
  if (q->round != SRQ_SR && q->round != SRQ_RTN) return SRQ_ERR_FORMAT;
  if (q->flags & ~(uint32_t)(SRQ_FLAG_F8_PIPELINE | SRQ_FLAG_COUNTER_DEV | SRQ_FLAG_QUANTIZE_ONCE)) return SRQ_ERR_FORMAT;
  if ((q->flags & SRQ_FLAG_COUNTER_DEV) && (q->counter_offset == 0 || (q->counter_offset & 7u))) return SRQ_ERR_ALIGN;
  if (!q->scale_dev) {
    const float s = q->scale;
    if (!(s >= 0x1p-100f) || !std::isfinite(s)) return SRQ_ERR_FORMAT;  // the kernels use (1/s) * 2^16
  }
  return SRQ_OK;
}

// With SRQ_FLAG_COUNTER_DEV the counter_offset field holds the device address of the counter.
uint64_t counter_host(const srq_quant* q) { return (q->flags & SRQ_FLAG_COUNTER_DEV) ? 0ull : q->counter_offset; }
const uint64_t* counter_dev(const srq_quant* q) {
  return (q->flags & SRQ_FLAG_COUNTER_DEV) ? reinterpret_cast<const uint64_t*>(static_cast<uintptr_t>(q->counter_offset))
                                           : nullptr;
}

QuantArgs make_args(const srq_quant* q, int dtype, int store) {
  QuantArgs a;
  a.kind = q->kind; a.round = q->round; a.dtype = dtype; a.store = store;
  a.scale = q->scale; a.scale_dev = q->scale_dev;
  a.seed = q->seed;
  a.counter_offset = counter_host(q); a.counter_dev = counter_dev(q);
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
  if (fx) return PIPE_F8;
  // exact pipelines: E5M2 x E5M2 multiplies straight from the one-byte codes; anything with an
  // E4M3-family operand goes through the bfloat16 form
  return qx->kind == SRQ_E5M2 && qz->kind == SRQ_E5M2 ? PIPE_F16C : PIPE_BF16;
}

// int32 accumulation is exact while R * 127^2 < 2^31
bool int_contraction_ok(int kx, size_t R) { return !kind_is_int(kx) || R * 16129ull < (1ull << 31); }

QuantJob make_job(const srq_quant* q, const void* x, int dtype, size_t rows, size_t cols, int transpose,
                  int store, uint8_t* out, uint8_t* out2) {
  QuantJob j;
  j.x = x; j.out = out; j.out2 = out2;
  j.rows = (uint32_t)rows; j.cols = (uint32_t)cols;
  j.kind = q->kind; j.round = q->round; j.dtype = dtype; j.store = store; j.transpose = transpose;
  j.scale = q->scale; j.scale_dev = q->scale_dev;
  j.seed = q->seed;
  j.counter_offset = counter_host(q); j.counter_dev = counter_dev(q);
  j.kind2 = 0; j.round2 = SRQ_SR; j.scale2 = 1.0f; j.scale_dev2 = nullptr; j.seed2 = j.counter_offset2 = 0;
  j.counter_dev2 = nullptr;
  j.pack_t = j.pack_2 = 0;
  j.first_block = j.nblocks = 0;
  return j;
}

// A transposing job that also writes, in the source layout, the byte codes of a second
// (integer) quantizer of the same tensor.
QuantJob make_dual_job(const srq_quant* q, const srq_quant* q2, const void* x, int dtype, size_t rows, size_t cols,
                       int store, uint8_t* out_t, uint8_t* out2) {
  QuantJob j = make_job(q, x, dtype, rows, cols, 1, store, out_t, out2);
  j.kind2 = q2->kind; j.round2 = q2->round; j.scale2 = q2->scale; j.scale_dev2 = q2->scale_dev;
  j.seed2 = q2->seed;
  j.counter_offset2 = counter_host(q2); j.counter_dev2 = counter_dev(q2);
  return j;
}

// Checks shared by the linear entry points for one operand.
int check_operand(const void* x, int dtype, const srq_quant* q) {
  if (!x) return SRQ_ERR_NULL;
  const int st = check_quant(q);
  if (st != SRQ_OK) return st;
  if (!dtype_ok(dtype)) return SRQ_ERR_FORMAT;
  if (!aligned16(x)) return SRQ_ERR_ALIGN;
  return SRQ_OK;
}

int check_dims(size_t M, size_t N, size_t K) {
  if (M == 0 || N == 0 || K == 0) return SRQ_ERR_SHAPE;
  if (!fits_u32(M) || !fits_u32(N) || !fits_u32(K)) return SRQ_ERR_SHAPE;
  if ((M % 16) || (N % 16) || (K % 16)) return SRQ_ERR_ALIGN;
  return SRQ_OK;
}

// One product out (P x Q) = X (P x R) . Z (Q x R)^T of quantized operands: pipeline, element
// size and the pieces of workspace it uses.
struct ProductPlan {
  int pipe;
  size_t es, x_bytes, z_bytes, gemm_bytes;
};

// from_codes = false: an operand shared with another product is stored as bfloat16 there, so
// this product may not use the pipeline that reads one-byte E5M2 codes.
int plan_product(ProductPlan& pp, const srq_quant* qx, const srq_quant* qz, size_t P, size_t Q, size_t R,
                 bool from_codes = true) {
  int st = check_pair(qx->kind, qz->kind);
  if (st != SRQ_OK) return st;
  if (!int_contraction_ok(qx->kind, R)) return SRQ_ERR_UNSUPPORTED;
  pp.pipe = pick_pipe(qx, qz);
  if (pp.pipe < 0) return SRQ_ERR_UNSUPPORTED;
  if (pp.pipe == PIPE_F16C && !from_codes) pp.pipe = PIPE_BF16;
  if (!gemm_operands_addressable(P, Q, R, pp.pipe)) return SRQ_ERR_UNSUPPORTED;
  pp.es = pp.pipe == PIPE_BF16 ? 2 : 1;
  pp.x_bytes = align_up(P * R * pp.es, WS_ALIGN);
  pp.z_bytes = align_up(Q * R * pp.es, WS_ALIGN);
  pp.gemm_bytes = align_up(gemm_workspace_bytes(P, Q, R, pp.pipe), WS_ALIGN);
  return SRQ_OK;
}

// upper bound over the pipelines, for the workspace queries
size_t product_bytes_max(size_t P, size_t Q, size_t R) {
  size_t best = 0;
  for (int pipe : {PIPE_I8, PIPE_BF16}) {
    const size_t es = pipe == PIPE_BF16 ? 2 : 1;
    const size_t t = align_up(P * R * es, WS_ALIGN) + align_up(Q * R * es, WS_ALIGN) +
                     align_up(gemm_workspace_bytes(P, Q, R, pipe), WS_ALIGN);
    if (t > best) best = t;
  }
  return best;
}

bool workspace_ok(const void* ws, size_t have, size_t need) {
  return ws && have >= need && (reinterpret_cast<uintptr_t>(ws) & 255u) == 0;
}

int launch_product(float* out, const uint8_t* xc, const srq_quant* qx, const uint8_t* zc, const srq_quant* qz,
                   size_t P, size_t Q, size_t R, const ProductPlan& pp, float beta, void* gws, hipStream_t s,
                   const SliceSum* carry = nullptr, SliceSum* defer = nullptr, bool x_packed = false) {
  // packed 4-bit X: the kernel multiplies 16 * value, the factor goes into alpha (a power of two: exact)
  GemmScale sc{x_packed ? 0.0625f : 1.0f, qx->scale, qz->scale, qx->scale_dev, qz->scale_dev};
  return launch_gemm_codes(out, xc, qx->kind, zc, qz->kind, P, Q, R, R * pp.es, pp.pipe, sc, beta == 1.0f, gws,
                           s, carry, defer, x_packed) == hipSuccess
             ? SRQ_OK
             : SRQ_ERR_HIP;
}

// The two products of Alg. 2 after their operands are quantized.  The weight gradient goes first
// and leaves the sum of its contraction slices to the launch of the input gradient, whose last
// workgroups do it (same arithmetic as in a launch of its own, one launch fewer, and the
// memory-bound sum runs beside the matrix work).
int launch_backward_products(float* dA, float* dW, const uint8_t* dy_rm, const uint8_t* w_t, const uint8_t* dy_t,
                             const uint8_t* a_t, const srq_quant* qdY, const srq_quant* qW, const srq_quant* qA,
                             size_t M, size_t N, size_t K, const ProductPlan& pd, const ProductPlan& pw, float beta,
                             void* gws_d, void* gws_w, hipStream_t s, bool packed_rm = false,
                             bool packed_t = false) {
  SliceSum sum_w{};
  int st = launch_product(dW, dy_t, qdY, a_t, qA, N, K, M, pw, beta, gws_w, s, nullptr, &sum_w, packed_t);
  if (st != SRQ_OK) return st;
  st = launch_product(dA, dy_rm, qdY, w_t, qW, M, K, N, pd, 0.0f, gws_d, s, &sum_w, nullptr, packed_rm);
  // the weight gradient is already enqueued: if the launch that was to carry its slice sum
  // failed, finish it in a launch of its own so that dW is whole whatever happens to dA
  if (st != SRQ_OK) (void)launch_slice_sum(sum_w, s);
  return st;
}

// A 4-bit output gradient from a binary32 source is written two values per byte for the products that
// take it so (the int8 pipeline on 256 x 256 tiles): half the bytes written, and read, of the
// operand every backward product shares.  rm: the copy in the source layout (X of dA, M x N);
// t: the transposed copy (X of dW, N x M).
struct PackedDy {
  bool rm, t;
};
PackedDy packed_dy(const srq_quant* qdY, int dtypedY, const ProductPlan& pd, const ProductPlan& pw, size_t M, size_t N,
                   size_t K) {
  const bool nib = dtypedY == SRQ_F32 && qdY->kind == SRQ_INT4 && pd.pipe == PIPE_I8 && pw.pipe == PIPE_I8;
  return PackedDy{nib && gemm_takes_packed_x(M, K, N, PIPE_I8), nib && gemm_takes_packed_x(N, K, M, PIPE_I8)};
}

// One product of Alg. 1 / Alg. 2: quantize both operands into the workspace (one launch) with
// the contraction index contiguous, then multiply.
//   out (P x Q) = Q(x)[P x R] . Q(z)[Q x R]^T,  x given as xr x xc (transposed if x_tr), same for z
int run_linear(float* out, const void* x, int dtx, size_t xr, size_t xc, int x_tr, const srq_quant* qx,
               const void* z, int dtz, size_t zr, size_t zc, int z_tr, const srq_quant* qz, size_t P,
               size_t Q, size_t R, float beta, void* workspace, size_t workspace_bytes, void* stream,
               int phase = SRQ_PHASE_BOTH) {
  if (!out) return SRQ_ERR_NULL;
  if (phase < SRQ_PHASE_QUANTIZE || phase > SRQ_PHASE_BOTH) return SRQ_ERR_FORMAT;
  int st = check_operand(x, dtx, qx);
  if (st != SRQ_OK) return st;
  st = check_operand(z, dtz, qz);
  if (st != SRQ_OK) return st;
  st = check_dims(P, Q, R);
  if (st != SRQ_OK) return st;
  if (!aligned16(out)) return SRQ_ERR_ALIGN;
  if (beta != 0.0f && beta != 1.0f) return SRQ_ERR_UNSUPPORTED;
  ProductPlan pp;
  st = plan_product(pp, qx, qz, P, Q, R);
  if (st != SRQ_OK) return st;
  if (!workspace_ok(workspace, workspace_bytes, pp.x_bytes + pp.z_bytes + pp.gemm_bytes)) return SRQ_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  // An output of at most four 64 x 64 tiles over a short contraction: every element is used by one
  // or two tiles, and rounding it inside the product (no codes in memory, one launch instead of
  // two) is the faster form -- measured 9.6 against 14.2 us on the 64 x 128 x 128 layer, but 27
  // against 14 us already at 128 x 128 x 768.  Integer pairs only: their results are the same bit
  // for bit in both forms.
  if (phase == SRQ_PHASE_BOTH && !x_tr && !z_tr && beta == 0.0f && pp.pipe == PIPE_I8 &&
      ((P + 63) / 64) * ((Q + 63) / 64) <= 4 && R <= 256 && !((qx->flags | qz->flags) & SRQ_FLAG_QUANTIZE_ONCE))
    return launch_fused_fwd(out, x, make_args(qx, dtx, STORE_BYTE), z, make_args(qz, dtz, STORE_BYTE), P, Q, R, s) == hipSuccess
               ? SRQ_OK
               : SRQ_ERR_HIP;
  uint8_t* xcodes = static_cast<uint8_t*>(workspace);
  uint8_t* zcodes = xcodes + pp.x_bytes;
  void* gws = zcodes + pp.z_bytes;
  const int store = pp.pipe == PIPE_BF16 ? STORE_BF16 : STORE_BYTE;
  QuantJobs jobs;
  jobs.njobs = 2;
  jobs.job[0] = make_job(qx, x, dtx, xr, xc, x_tr, store, xcodes, nullptr);
  jobs.job[1] = make_job(qz, z, dtz, zr, zc, z_tr, store, zcodes, nullptr);
  if ((phase & SRQ_PHASE_QUANTIZE) && launch_quantize_jobs(jobs, s) != hipSuccess) return SRQ_ERR_HIP;
  if (!(phase & SRQ_PHASE_PRODUCT)) return SRQ_OK;
  return launch_product(out, xcodes, qx, zcodes, qz, P, Q, R, pp, beta, gws, s);
}

// Products of the weight-only objective (Sec. 3.2): out (P x Q) = x . Q(w)^T with the row operand
// x (P x R, R contiguous, binary32 or bfloat16) taken as it is.  The bf16 matrix pipeline multiplies
// exactly: w is written as the bfloat16 numbers of its grid values (R contiguous); a bfloat16 x is
// used in place; a binary32 x becomes three bfloat16 planes that sum to it, side by side in each
// row, multiplied in one launch over the contraction 3 R against [w | w | w], so the planes are
// added inside the binary32 accumulators.
struct WeightOnlyPlan {
  int planes;  // 1: x is bfloat16 already; 3: binary32
  size_t x_bytes, zcodes_bytes, z_bytes, z3_bytes, gemm_bytes;
};
WeightOnlyPlan plan_weight_only(int dtx, int kind_w, size_t P, size_t Q, size_t R) {
  WeightOnlyPlan wp;
  wp.planes = dtx == SRQ_F32 ? 3 : 1;
  wp.x_bytes = wp.planes == 3 ? align_up(3 * P * R * 2, WS_ALIGN) : 0;
  wp.zcodes_bytes = kind_is_int(kind_w) ? align_up(Q * R, WS_ALIGN) : 0;
  wp.z_bytes = align_up(Q * R * 2, WS_ALIGN);
  wp.z3_bytes = wp.planes == 3 ? align_up(3 * Q * R * 2, WS_ALIGN) : 0;
  wp.gemm_bytes = align_up(gemm_workspace_bytes(P, Q, wp.planes * R, PIPE_BF16), WS_ALIGN);
  return wp;
}
size_t weight_only_total(const WeightOnlyPlan& wp) {
  return wp.x_bytes + wp.zcodes_bytes + wp.z_bytes + wp.z3_bytes + wp.gemm_bytes;
}
size_t weight_only_bytes_max(size_t P, size_t Q, size_t R) {
  const size_t a = weight_only_total(plan_weight_only(SRQ_F32, SRQ_INT8, P, Q, R));
  const size_t b = weight_only_total(plan_weight_only(SRQ_BF16, SRQ_INT8, P, Q, R));
  return a > b ? a : b;
}

int run_weight_only(float* out, const void* x, int dtx, const void* w, int dtw, size_t wr, size_t wc, int w_tr,
                    const srq_quant* qw, size_t P, size_t Q, size_t R, void* workspace, size_t workspace_bytes,
                    void* stream) {
  if (!out || !x) return SRQ_ERR_NULL;
  if (!dtype_ok(dtx)) return SRQ_ERR_FORMAT;
  int st = check_operand(w, dtw, qw);
  if (st != SRQ_OK) return st;
  st = check_dims(P, Q, R);
  if (st != SRQ_OK) return st;
  if (!aligned16(out) || !aligned16(x)) return SRQ_ERR_ALIGN;
  const WeightOnlyPlan wp = plan_weight_only(dtx, qw->kind, P, Q, R);
  const size_t R3 = (size_t)wp.planes * R;  // contraction length of the launch
  if (!fits_u32(R3) || !gemm_operands_addressable(P, Q, R3, PIPE_BF16)) return SRQ_ERR_UNSUPPORTED;
  if (!workspace_ok(workspace, workspace_bytes, weight_only_total(wp))) return SRQ_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  uint8_t* xplanes = static_cast<uint8_t*>(workspace);
  uint8_t* zcodes = xplanes + wp.x_bytes;
  uint8_t* zvals = zcodes + wp.zcodes_bytes;
  uint8_t* z3 = zvals + wp.z_bytes;
  void* gws = z3 + wp.z3_bytes;
  const bool w_int = kind_is_int(qw->kind);
  QuantJobs jobs;
  jobs.njobs = 1;
  jobs.job[0] = make_job(qw, w, dtw, wr, wc, w_tr, w_int ? STORE_BYTE : STORE_BF16, w_int ? zcodes : zvals, nullptr);
  if (launch_quantize_jobs(jobs, s) != hipSuccess) return SRQ_ERR_HIP;
  if (w_int && launch_int_codes_to_bf16(reinterpret_cast<uint16_t*>(zvals), zcodes, Q * R, s) != hipSuccess)
    return SRQ_ERR_HIP;
  const uint8_t* xop = static_cast<const uint8_t*>(x);
  const uint8_t* zop = zvals;
  if (wp.planes == 3) {
    if (launch_split3(reinterpret_cast<uint16_t*>(xplanes), static_cast<const float*>(x), P, R, s) != hipSuccess ||
        launch_repeat3(reinterpret_cast<uint16_t*>(z3), reinterpret_cast<const uint16_t*>(zvals), Q, R, s) != hipSuccess)
      return SRQ_ERR_HIP;
    xop = xplanes;
    zop = z3;
  }
  const GemmScale sc{1.0f, 1.0f, qw->scale, nullptr, qw->scale_dev};
  return launch_gemm_codes(out, xop, SRQ_E5M2, zop, SRQ_E5M2, P, Q, R3, 2 * R3, PIPE_BF16, sc, false, gws, s) == hipSuccess
             ? SRQ_OK
             : SRQ_ERR_HIP;
}

bool is_none(const srq_quant* q) { return q && q->kind == SRQ_NONE; }

// Address of `scratch` on the current device, looked up once per device (with that device
// current) and kept.  Returns nullptr if the runtime refuses.
constexpr int MAX_DEVICES = 64;
void* static_scratch_ptr() {
  static std::mutex lock;
  static void* ptr[MAX_DEVICES] = {};
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return nullptr;
  std::lock_guard<std::mutex> guard(lock);
  if (!ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    ptr[dev] = p;
  }
  return ptr[dev];
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

static int build_absmax_batch(AbsmaxBatch& b, const srq_absmax_req* reqs, int count) {
  if (!reqs) return SRQ_ERR_NULL;
  if (count < 1 || count > ABSMAX_MAX) return SRQ_ERR_SHAPE;
  b.ntensors = 0;
  b.nouts = count;
  for (int i = 0; i < count; ++i) {
    const srq_absmax_req& r = reqs[i];
    if (!r.scale_out_dev || (!r.x && r.n > 0)) return SRQ_ERR_NULL;
    if (!kind_ok(r.kind) || !dtype_ok(r.dtype)) return SRQ_ERR_FORMAT;
    if (!aligned16(r.x)) return SRQ_ERR_ALIGN;
    int t = -1;
    for (int j = 0; j < b.ntensors; ++j)
      if (b.x[j] == r.x && b.n[j] == r.n && b.dtype[j] == r.dtype) t = j;
    if (t < 0) {
      t = b.ntensors++;
      b.x[t] = r.x; b.n[t] = r.n; b.dtype[t] = r.dtype;
    }
    b.out_tensor[i] = t; b.out_kind[i] = r.kind; b.out[i] = r.scale_out_dev;
  }
  return SRQ_OK;
}

size_t sr_absmax_workspace_bytes(const srq_absmax_req* reqs, int count) {
  AbsmaxBatch b;
  if (build_absmax_batch(b, reqs, count) != SRQ_OK) return 0;
  return absmax_batch_plan(b) * sizeof(uint32_t);
}

int sr_absmax_scales(const srq_absmax_req* reqs, int count, void* workspace, size_t workspace_bytes,
                     void* stream) {
  AbsmaxBatch b;
  const int st = build_absmax_batch(b, reqs, count);
  if (st != SRQ_OK) return st;
  const size_t need = absmax_batch_plan(b) * sizeof(uint32_t);
  if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 3u)) return SRQ_ERR_WORKSPACE;
  b.partial = static_cast<uint32_t*>(workspace);
  return launch_absmax_batch(b, static_cast<hipStream_t>(stream)) == hipSuccess ? SRQ_OK : SRQ_ERR_HIP;
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

size_t sr_gemm_bf16_workspace_bytes(size_t P, size_t Q, size_t R) {
  if (P == 0 || Q == 0 || R == 0) return 0;
  return gemm_workspace_bytes(P, Q, R, PIPE_BF16);
}

int sr_gemm_bf16(float* out, const void* X, const void* Z, size_t P, size_t Q, size_t R, float alpha, float beta,
                 void* workspace, size_t workspace_bytes, void* stream) {
  if (!out || !X || !Z) return SRQ_ERR_NULL;
  if (P == 0 || Q == 0 || R == 0) return SRQ_ERR_SHAPE;
  if (!fits_u32(P) || !fits_u32(Q) || !fits_u32(R)) return SRQ_ERR_SHAPE;
  if (R % 8) return SRQ_ERR_ALIGN;
  if (!aligned16(out) || !aligned16(X) || !aligned16(Z)) return SRQ_ERR_ALIGN;
  if (beta != 0.0f && beta != 1.0f) return SRQ_ERR_UNSUPPORTED;
  if (!gemm_operands_addressable(P, Q, R, PIPE_BF16)) return SRQ_ERR_UNSUPPORTED;
  const size_t need = gemm_workspace_bytes(P, Q, R, PIPE_BF16);
  if (need > 0 && (!workspace || workspace_bytes < need || !aligned16(workspace))) return SRQ_ERR_WORKSPACE;
  GemmScale sc{alpha, 1.0f, 1.0f, nullptr, nullptr};
  return launch_gemm_codes(out, static_cast<const uint8_t*>(X), SRQ_E5M2, static_cast<const uint8_t*>(Z), SRQ_E5M2,
                           P, Q, R, 2 * R, PIPE_BF16, sc, beta == 1.0f, workspace,
                           static_cast<hipStream_t>(stream)) == hipSuccess
             ? SRQ_OK
             : SRQ_ERR_HIP;
}

size_t sr_gemm_e5m2_workspace_bytes(size_t P, size_t Q, size_t R) {
  if (P == 0 || Q == 0 || R == 0) return 0;
  return gemm_workspace_bytes(P, Q, R, PIPE_F16C);
}

int sr_gemm_e5m2(float* out, const void* X, const void* Z, size_t P, size_t Q, size_t R, float alpha, float beta,
                 void* workspace, size_t workspace_bytes, void* stream) {
  if (!out || !X || !Z) return SRQ_ERR_NULL;
  if (P == 0 || Q == 0 || R == 0) return SRQ_ERR_SHAPE;
  if (!fits_u32(P) || !fits_u32(Q) || !fits_u32(R)) return SRQ_ERR_SHAPE;
  if (R % 16) return SRQ_ERR_ALIGN;
  if (!aligned16(out) || !aligned16(X) || !aligned16(Z)) return SRQ_ERR_ALIGN;
  if (beta != 0.0f && beta != 1.0f) return SRQ_ERR_UNSUPPORTED;
  if (!gemm_operands_addressable(P, Q, R, PIPE_F16C)) return SRQ_ERR_UNSUPPORTED;
  const size_t need = gemm_workspace_bytes(P, Q, R, PIPE_F16C);
  if (need > 0 && (!workspace || workspace_bytes < need || !aligned16(workspace))) return SRQ_ERR_WORKSPACE;
  GemmScale sc{alpha, 1.0f, 1.0f, nullptr, nullptr};
  return launch_gemm_codes(out, static_cast<const uint8_t*>(X), SRQ_E5M2, static_cast<const uint8_t*>(Z), SRQ_E5M2,
                           P, Q, R, R, PIPE_F16C, sc, beta == 1.0f, workspace,
                           static_cast<hipStream_t>(stream)) == hipSuccess
             ? SRQ_OK
             : SRQ_ERR_HIP;
}

size_t sr_linear_workspace_bytes(int op, size_t M, size_t N, size_t K) {
  if (M == 0 || N == 0 || K == 0) return 0;
  // sized for the widest operand storage (two bytes per element), so one buffer serves every format
  switch (op) {
    case SRQ_OP_FWD: return product_bytes_max(M, N, K);         // Y  (M x N), contraction K
    case SRQ_OP_BWD_DATA: return product_bytes_max(M, K, N);    // dA (M x K), contraction N
    case SRQ_OP_BWD_WEIGHT: return product_bytes_max(N, K, M);  // dW (N x K), contraction M
    case SRQ_OP_BWD:                                            // both; dY is held in both layouts
      return product_bytes_max(M, K, N) + product_bytes_max(N, K, M);
    case SRQ_OP_FWD_STASH: return product_bytes_max(M, N, K);
    case SRQ_OP_BWD_STASHED:                                    // dY in both layouts + the two products' scratch
      return 2 * align_up(2 * M * N, WS_ALIGN) + align_up(gemm_workspace_bytes(M, K, N, PIPE_BF16), WS_ALIGN) +
             align_up(gemm_workspace_bytes(N, K, M, PIPE_BF16), WS_ALIGN) +
             align_up(gemm_workspace_bytes(M, K, N, PIPE_I8), WS_ALIGN) +
             align_up(gemm_workspace_bytes(N, K, M, PIPE_I8), WS_ALIGN);
    case SRQ_OP_FWD_WEIGHT_ONLY: return weight_only_bytes_max(M, N, K);
    case SRQ_OP_BWD_DATA_WEIGHT_ONLY: return weight_only_bytes_max(M, K, N);
    default: return 0;
  }
}

// Alg. 1: Y = Ahat What^T.  A (M x K) and W (N x K) already have K contiguous.
int sr_linear_fwd(float* Y, const void* A, int dtypeA, const void* W, int dtypeW, size_t M, size_t N,
                  size_t K, const srq_quant* qA_fwd, const srq_quant* qW_fwd, void* workspace,
                  size_t workspace_bytes, void* stream) {
  if (is_none(qA_fwd))  // weight-only objective: A enters as it is
    return run_weight_only(Y, A, dtypeA, W, dtypeW, N, K, 0, qW_fwd, M, N, K, workspace, workspace_bytes, stream);
  return run_linear(Y, A, dtypeA, M, K, 0, qA_fwd, W, dtypeW, N, K, 0, qW_fwd, M, N, K, 0.0f, workspace,
                    workspace_bytes, stream);
}

// Alg. 1 in two halves: the quantizer launch, the product launch, or both.
int sr_linear_fwd_phase(float* Y, const void* A, int dtypeA, const void* W, int dtypeW, size_t M, size_t N,
                        size_t K, const srq_quant* qA_fwd, const srq_quant* qW_fwd, void* workspace,
                        size_t workspace_bytes, int phase, void* stream) {
  if (is_none(qA_fwd)) return SRQ_ERR_UNSUPPORTED;
  return run_linear(Y, A, dtypeA, M, K, 0, qA_fwd, W, dtypeW, N, K, 0, qW_fwd, M, N, K, 0.0f, workspace,
                    workspace_bytes, stream, phase);
}

int sr_linear_fwd_fused(float* Y, const void* A, int dtypeA, const void* W, int dtypeW, size_t M, size_t N,
                        size_t K, const srq_quant* qA_fwd, const srq_quant* qW_fwd, void* stream) {
  if (!Y) return SRQ_ERR_NULL;
  int st = check_operand(A, dtypeA, qA_fwd);
  if (st != SRQ_OK) return st;
  st = check_operand(W, dtypeW, qW_fwd);
  if (st != SRQ_OK) return st;
  st = check_dims(M, N, K);
  if (st != SRQ_OK) return st;
  if (!aligned16(Y)) return SRQ_ERR_ALIGN;
  if (!fused_pair_supported(qA_fwd->kind, qW_fwd->kind)) return SRQ_ERR_UNSUPPORTED;
  if (!int_contraction_ok(qA_fwd->kind, K)) return SRQ_ERR_UNSUPPORTED;
  if (((M + 127) / 128) * ((N + 127) / 128) > 0x7FFFFFFFull) return SRQ_ERR_UNSUPPORTED;  // one workgroup per tile
  return launch_fused_fwd(Y, A, make_args(qA_fwd, dtypeA, STORE_BYTE), W, make_args(qW_fwd, dtypeW, STORE_BYTE), M, N,
                          K, static_cast<hipStream_t>(stream)) == hipSuccess
             ? SRQ_OK
             : SRQ_ERR_HIP;
}

// Alg. 1 for callers that may not allocate: the workspace is the library's static device array.
size_t sr_linear_fwd_static_limit(void) { return SRQ_STATIC_SCRATCH_BYTES; }

int sr_linear_fwd_static(float* Y, const void* A, int dtypeA, const void* W, int dtypeW, size_t M, size_t N,
                         size_t K, const srq_quant* qA_fwd, const srq_quant* qW_fwd, void* stream) {
  // what sr_linear_fwd would ask of its caller for this call; beyond the array: refuse
  const size_t need = sr_linear_workspace_bytes(is_none(qA_fwd) ? SRQ_OP_FWD_WEIGHT_ONLY : SRQ_OP_FWD, M, N, K);
  if (need > SRQ_STATIC_SCRATCH_BYTES) return SRQ_ERR_STATIC_LIMIT;
  void* ws = static_scratch_ptr();
  if (!ws) return SRQ_ERR_HIP;
  // every byte of the workspace that the product reads is written by this call's quantizer
  // launch first (operand codes; slice partials by the product itself), so the array needs no
  // clearing between calls
  return sr_linear_fwd(Y, A, dtypeA, W, dtypeW, M, N, K, qA_fwd, qW_fwd, ws, SRQ_STATIC_SCRATCH_BYTES, stream);
}

// Alg. 2: dA = dYhat What.  Contraction over N: dY (M x N) as is, W (N x K) written as K x N.
int sr_linear_bwd_data(float* dA, const void* dY, int dtypedY, const void* W, int dtypeW, size_t M,
                       size_t N, size_t K, const srq_quant* qdY_bwd, const srq_quant* qW_bwd,
                       void* workspace, size_t workspace_bytes, void* stream) {
  if (is_none(qdY_bwd))  // weight-only objective: dY enters as it is
    return run_weight_only(dA, dY, dtypedY, W, dtypeW, N, K, 1, qW_bwd, M, K, N, workspace, workspace_bytes, stream);
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

// Alg. 2 in one call: the output gradient is read and quantized once (one Q(dY), as the
// algorithm has it) and written in both layouts; W and A are quantized in the same launch.
int sr_linear_bwd(float* dA, float* dW, const void* dY, int dtypedY, const void* W, int dtypeW, const void* A,
                  int dtypeA, size_t M, size_t N, size_t K, const srq_quant* qdY_bwd, const srq_quant* qW_bwd,
                  const srq_quant* qA_bwd, float beta, void* workspace, size_t workspace_bytes, void* stream) {
  return sr_linear_bwd_phase(dA, dW, dY, dtypedY, W, dtypeW, A, dtypeA, M, N, K, qdY_bwd, qW_bwd, qA_bwd, beta,
                             workspace, workspace_bytes, SRQ_PHASE_BOTH, stream);
}

int sr_linear_bwd_phase(float* dA, float* dW, const void* dY, int dtypedY, const void* W, int dtypeW, const void* A,
                        int dtypeA, size_t M, size_t N, size_t K, const srq_quant* qdY_bwd, const srq_quant* qW_bwd,
                        const srq_quant* qA_bwd, float beta, void* workspace, size_t workspace_bytes, int phase,
                        void* stream) {
  if (!dA || !dW) return SRQ_ERR_NULL;
  if (phase < SRQ_PHASE_QUANTIZE || phase > SRQ_PHASE_BOTH) return SRQ_ERR_FORMAT;
  int st = check_operand(dY, dtypedY, qdY_bwd);
  if (st != SRQ_OK) return st;
  st = check_operand(W, dtypeW, qW_bwd);
  if (st != SRQ_OK) return st;
  st = check_operand(A, dtypeA, qA_bwd);
  if (st != SRQ_OK) return st;
  st = check_dims(M, N, K);
  if (st != SRQ_OK) return st;
  if (!aligned16(dA) || !aligned16(dW)) return SRQ_ERR_ALIGN;
  if (beta != 0.0f && beta != 1.0f) return SRQ_ERR_UNSUPPORTED;
  ProductPlan pd, pw;  // dA = dY (M x N) . Wt (K x N)^T ;  dW = dYt (N x M) . At (K x M)^T
  // Q(dY) is stored once for both products: one-byte codes only if all three formats are E5M2
  const bool codes = qW_bwd->kind == SRQ_E5M2 && qA_bwd->kind == SRQ_E5M2;
  st = plan_product(pd, qdY_bwd, qW_bwd, M, K, N, codes);
  if (st != SRQ_OK) return st;
  st = plan_product(pw, qdY_bwd, qA_bwd, N, K, M, codes);
  if (st != SRQ_OK) return st;
  if (pd.pipe != pw.pipe) return SRQ_ERR_UNSUPPORTED;  // one stored form of Q(dY) serves both products
  const size_t need = pd.x_bytes + pd.z_bytes + pd.gemm_bytes + pw.x_bytes + pw.z_bytes + pw.gemm_bytes;
  if (!workspace_ok(workspace, workspace_bytes, need)) return SRQ_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  uint8_t* dy_rm = static_cast<uint8_t*>(workspace);  // M x N
  uint8_t* w_t = dy_rm + pd.x_bytes;                  // K x N
  uint8_t* gws_d = w_t + pd.z_bytes;
  uint8_t* dy_t = gws_d + pd.gemm_bytes;              // N x M
  uint8_t* a_t = dy_t + pw.x_bytes;                   // K x M
  uint8_t* gws_w = a_t + pw.z_bytes;
  const int store = pd.pipe == PIPE_BF16 ? STORE_BF16 : STORE_BYTE;
  QuantJobs jobs;
  jobs.njobs = 3;
  jobs.job[0] = make_job(qdY_bwd, dY, dtypedY, M, N, 1, store, dy_t, dy_rm);
  const PackedDy pk = packed_dy(qdY_bwd, dtypedY, pd, pw, M, N, K);
  jobs.job[0].pack_2 = pk.rm;
  jobs.job[0].pack_t = pk.t;
  jobs.job[1] = make_job(qW_bwd, W, dtypeW, N, K, 1, store, w_t, nullptr);
  jobs.job[2] = make_job(qA_bwd, A, dtypeA, M, K, 1, store, a_t, nullptr);
  if ((phase & SRQ_PHASE_QUANTIZE) && launch_quantize_jobs(jobs, s) != hipSuccess) return SRQ_ERR_HIP;
  if (!(phase & SRQ_PHASE_PRODUCT)) return SRQ_OK;
  return launch_backward_products(dA, dW, dy_rm, w_t, dy_t, a_t, qdY_bwd, qW_bwd, qA_bwd, M, N, K, pd, pw, beta, gws_d,
                                  gws_w, s, pk.rm, pk.t);
}

// Eq. 10 with bfloat16 weights.
int sr_update_bf16(void* w_bf16, const float* g, float eta, size_t n, int round_mode, uint64_t seed,
                   uint64_t counter_offset, void* stream) {
  if (n == 0) return SRQ_OK;
  if (!w_bf16 || !g) return SRQ_ERR_NULL;
  if (round_mode != SRQ_SR && round_mode != SRQ_RTN) return SRQ_ERR_FORMAT;
  if (!(eta == eta) || std::isinf(eta)) return SRQ_ERR_FORMAT;
  if (!aligned16(w_bf16) || !aligned16(g)) return SRQ_ERR_ALIGN;
  return launch_update_bf16(static_cast<uint16_t*>(w_bf16), g, eta, n, round_mode, seed, counter_offset,
                            static_cast<hipStream_t>(stream)) == hipSuccess
             ? SRQ_OK
             : SRQ_ERR_HIP;
}

size_t sr_linear_stash_bytes(size_t M, size_t N, size_t K) {
  return align_up(2 * K * M, WS_ALIGN) + align_up(2 * K * N, WS_ALIGN);
}

// Alg. 1 that also leaves behind what Alg. 2 needs of A and W: one pass over A and one over W
// feed the forward quantizers (row-major byte codes, into the workspace) and the backward
// quantizers (transposed, in the form the backward products read, into the stash).
int sr_linear_fwd_stash(float* Y, const void* A, int dtypeA, const void* W, int dtypeW, size_t M, size_t N,
                        size_t K, const srq_quant* qA_fwd, const srq_quant* qW_fwd, const srq_quant* qA_bwd,
                        const srq_quant* qW_bwd, void* stash, size_t stash_bytes, void* workspace,
                        size_t workspace_bytes, void* stream) {
  return sr_linear_fwd_stash_phase(Y, A, dtypeA, W, dtypeW, M, N, K, qA_fwd, qW_fwd, qA_bwd, qW_bwd, stash, stash_bytes,
                                   workspace, workspace_bytes, SRQ_PHASE_BOTH, stream);
}

int sr_linear_fwd_stash_phase(float* Y, const void* A, int dtypeA, const void* W, int dtypeW, size_t M, size_t N,
                              size_t K, const srq_quant* qA_fwd, const srq_quant* qW_fwd, const srq_quant* qA_bwd,
                              const srq_quant* qW_bwd, void* stash, size_t stash_bytes, void* workspace,
                              size_t workspace_bytes, int phase, void* stream) {
  if (!Y) return SRQ_ERR_NULL;
  if (phase < SRQ_PHASE_QUANTIZE || phase > SRQ_PHASE_BOTH) return SRQ_ERR_FORMAT;
  int st = check_operand(A, dtypeA, qA_fwd);
  if (st != SRQ_OK) return st;
  st = check_operand(W, dtypeW, qW_fwd);
  if (st != SRQ_OK) return st;
  if ((st = check_quant(qA_bwd)) != SRQ_OK || (st = check_quant(qW_bwd)) != SRQ_OK) return st;
  st = check_dims(M, N, K);
  if (st != SRQ_OK) return st;
  if (!aligned16(Y)) return SRQ_ERR_ALIGN;
  // the rider quantizer is the integer one
  if (!kind_is_int(qA_fwd->kind) || !kind_is_int(qW_fwd->kind)) return SRQ_ERR_UNSUPPORTED;
  ProductPlan pf;
  st = plan_product(pf, qA_fwd, qW_fwd, M, N, K);
  if (st != SRQ_OK) return st;
  // the stored form of the backward operands: the pipeline their products with dY will use
  if (check_pair(qA_bwd->kind, qW_bwd->kind) != SRQ_OK) return SRQ_ERR_UNSUPPORTED;
  const int stash_pipe = pick_pipe(qA_bwd, qW_bwd);
  if (stash_pipe < 0) return SRQ_ERR_UNSUPPORTED;
  if (!workspace_ok(workspace, workspace_bytes, pf.x_bytes + pf.z_bytes + pf.gemm_bytes)) return SRQ_ERR_WORKSPACE;
  if (!workspace_ok(stash, stash_bytes, sr_linear_stash_bytes(M, N, K))) return SRQ_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  uint8_t* a_codes = static_cast<uint8_t*>(workspace);
  uint8_t* w_codes = a_codes + pf.x_bytes;
  void* gws = w_codes + pf.z_bytes;
  uint8_t* a_t = static_cast<uint8_t*>(stash);
  uint8_t* w_t = a_t + align_up(2 * K * M, WS_ALIGN);
  const int store = stash_pipe == PIPE_BF16 ? STORE_BF16 : STORE_BYTE;
  QuantJobs jobs;
  jobs.njobs = 2;
  jobs.job[0] = make_dual_job(qA_bwd, qA_fwd, A, dtypeA, M, K, store, a_t, a_codes);
  jobs.job[1] = make_dual_job(qW_bwd, qW_fwd, W, dtypeW, N, K, store, w_t, w_codes);
  if ((phase & SRQ_PHASE_QUANTIZE) && launch_quantize_jobs(jobs, s) != hipSuccess) return SRQ_ERR_HIP;
  if (!(phase & SRQ_PHASE_PRODUCT)) return SRQ_OK;
  return launch_product(Y, a_codes, qA_fwd, w_codes, qW_fwd, M, N, K, pf, 0.0f, gws, s);
}

// Alg. 2 from the stash of sr_linear_fwd_stash: only dY is read and quantized here.
int sr_linear_bwd_stashed(float* dA, float* dW, const void* dY, int dtypedY, size_t M, size_t N, size_t K,
                          const srq_quant* qdY_bwd, const srq_quant* qW_bwd, const srq_quant* qA_bwd,
                          const void* stash, size_t stash_bytes, float beta, void* workspace,
                          size_t workspace_bytes, void* stream) {
  return sr_linear_bwd_stashed_phase(dA, dW, dY, dtypedY, M, N, K, qdY_bwd, qW_bwd, qA_bwd, stash, stash_bytes, beta,
                                     workspace, workspace_bytes, SRQ_PHASE_BOTH, stream);
}

int sr_linear_bwd_stashed_phase(float* dA, float* dW, const void* dY, int dtypedY, size_t M, size_t N, size_t K,
                                const srq_quant* qdY_bwd, const srq_quant* qW_bwd, const srq_quant* qA_bwd,
                                const void* stash, size_t stash_bytes, float beta, void* workspace,
                                size_t workspace_bytes, int phase, void* stream) {
  if (!dA || !dW) return SRQ_ERR_NULL;
  if (phase < SRQ_PHASE_QUANTIZE || phase > SRQ_PHASE_BOTH) return SRQ_ERR_FORMAT;
  int st = check_operand(dY, dtypedY, qdY_bwd);
  if (st != SRQ_OK) return st;
  if ((st = check_quant(qA_bwd)) != SRQ_OK || (st = check_quant(qW_bwd)) != SRQ_OK) return st;
  st = check_dims(M, N, K);
  if (st != SRQ_OK) return st;
  if (!aligned16(dA) || !aligned16(dW)) return SRQ_ERR_ALIGN;
  if (beta != 0.0f && beta != 1.0f) return SRQ_ERR_UNSUPPORTED;
  ProductPlan pd, pw;
  // all three operands in one stored form, the one the stash was written in (one-byte codes
  // when A and W are both E5M2, which then needs an E5M2 dY as well)
  if (check_pair(qA_bwd->kind, qW_bwd->kind) != SRQ_OK) return SRQ_ERR_UNSUPPORTED;
  const int stash_pipe = pick_pipe(qA_bwd, qW_bwd);
  st = plan_product(pd, qdY_bwd, qW_bwd, M, K, N, stash_pipe == PIPE_F16C);
  if (st != SRQ_OK) return st;
  st = plan_product(pw, qdY_bwd, qA_bwd, N, K, M, stash_pipe == PIPE_F16C);
  if (st != SRQ_OK) return st;
  if (pd.pipe != pw.pipe || pd.pipe != stash_pipe) return SRQ_ERR_UNSUPPORTED;
  const size_t need = pd.x_bytes + pd.gemm_bytes + pw.x_bytes + pw.gemm_bytes;
  if (!workspace_ok(workspace, workspace_bytes, need)) return SRQ_ERR_WORKSPACE;
  if (!workspace_ok(stash, stash_bytes, sr_linear_stash_bytes(M, N, K))) return SRQ_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  uint8_t* dy_rm = static_cast<uint8_t*>(workspace);  // M x N
  uint8_t* gws_d = dy_rm + pd.x_bytes;
  uint8_t* dy_t = gws_d + pd.gemm_bytes;              // N x M
  uint8_t* gws_w = dy_t + pw.x_bytes;
  const uint8_t* a_t = static_cast<const uint8_t*>(stash);
  const uint8_t* w_t = a_t + align_up(2 * K * M, WS_ALIGN);
  const int store = pd.pipe == PIPE_BF16 ? STORE_BF16 : STORE_BYTE;
  QuantJobs jobs;
  jobs.njobs = 1;
  jobs.job[0] = make_job(qdY_bwd, dY, dtypedY, M, N, 1, store, dy_t, dy_rm);
  const PackedDy pk = packed_dy(qdY_bwd, dtypedY, pd, pw, M, N, K);
  jobs.job[0].pack_2 = pk.rm;
  jobs.job[0].pack_t = pk.t;
  if ((phase & SRQ_PHASE_QUANTIZE) && launch_quantize_jobs(jobs, s) != hipSuccess) return SRQ_ERR_HIP;
  if (!(phase & SRQ_PHASE_PRODUCT)) return SRQ_OK;
  return launch_backward_products(dA, dW, dy_rm, w_t, dy_t, a_t, qdY_bwd, qW_bwd, qA_bwd, M, N, K, pd, pw, beta, gws_d,
                                  gws_w, s, pk.rm, pk.t);
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
    case SRQ_ERR_STATIC_LIMIT: return "problem needs more scratch than the static array of sr_linear_fwd_static holds";
    default: return "unknown status";
  }
}

}  // extern "C"
