/*
 * srq.h -- C ABI of the stochastic-rounding quantized linear layer for AMD MI355X (gfx950).
 *
 * The library implements the quantized linear layer of mixed-precision SGD with
 * stochastic rounding: the threshold quantizer of Def. 1 (Eq. 1) applied element-wise
 * with independent thresholds (Def. 3), and the forward / backward products of Alg. 1 and
 * Alg. 2, in which the two operands of every product are quantized first and the product
 * is then taken exactly with high-precision accumulation (Sec. 2.2.2).  One layer has five
 * quantizers (A and W in the forward pass; A, W and the output gradient in the backward
 * pass, Sec. 3); each is described by one `srq_quant`.
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller.  The library never
 *     allocates, frees or keeps them.  Tensors are dense row-major.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work; they never synchronise.
 *   - The return value is the only error channel.  Argument errors are found before anything is
 *     launched.  SRQ_ERR_HIP (the runtime refused a launch) can come after earlier launches of
 *     the same call were enqueued; the outputs are then unspecified.
 *   - Entry points may be called from several host threads at once; the library keeps no
 *     state between calls (beyond a one-time launch configuration per kernel).  Calls that
 *     share a workspace must be ordered by the caller (same stream, or events).
 *   - Layer shapes follow torch.nn.Linear: A is M x K (tokens x in), W is N x K (out x in),
 *     Y and dY are M x N, dA is M x K, dW is N x K.  (The paper writes A_out = A W with W
 *     as in x out; that W is the transpose of this one.)
 *   - The codes produced for a tensor depend only on (data, source dtype, scale, format,
 *     rounding mode, seed, counter_offset): never on the entry point, the output layout,
 *     tile shapes or launch order.  Thresholds are fixed by (seed, counter_offset, element
 *     index), which is what makes the passes deterministic for fixed thresholds (note under
 *     Alg. 1).
 *
 * The quantizer, per element i (row-major index) of a tensor:
 *     inv  = fl32(1 / scale)
 *     t    = clamp(fl32(x_i * inv), -Qmax, +Qmax)                  grid coordinate
 *     D    = 1 for integer formats; for the 8-bit floats the spacing of the format's grid
 *            at t: 2^(max(floor(log2|t|), emin) - m)
 *     y    = t / D;  q = floor(y) if y - floor(y) < eps_i else floor(y) + 1       (Eq. 1)
 *     code = encoding of q * D;   represented value = q * D * scale
 *     eps_i = (r16 + 1/2) / 65536 for stochastic rounding, 1/2 for round-to-nearest (Def. 2),
 *     r16 = 16-bit slice (i mod 8) of Philox4x32-10(counter = (counter_offset + i / 8) as
 *           (lo, hi, 0, 0), key = (seed lo, seed hi)), low half of output word 0 first.
 *     inv and t are single IEEE binary32 operations (no fused multiply-add); from t on, Eq. 1
 *     is evaluated exactly (t / D, floor, fractional part, comparison with eps).
 *     NaN input gives code 0 (integers) or 0x7F (floats); +-Inf saturates to +-Qmax.
 */
#ifndef SRQ_H
#define SRQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SRQ_OK = 0,
  SRQ_ERR_NULL = -1,        /* a required pointer is NULL                                  */
  SRQ_ERR_SHAPE = -2,       /* a dimension is zero where it may not be, or overflows        */
  SRQ_ERR_FORMAT = -3,      /* unknown kind / rounding / dtype, or a bad host-side scale    */
  SRQ_ERR_ALIGN = -4,       /* pointer or dimension not aligned as the entry point requires */
  SRQ_ERR_WORKSPACE = -5,   /* workspace NULL or smaller than sr_linear_workspace_bytes     */
  SRQ_ERR_UNSUPPORTED = -6, /* valid but not implemented (e.g. int x float operand pair)    */
  SRQ_ERR_HIP = -7,         /* the HIP runtime reported an error at launch                  */
  SRQ_ERR_STATIC_LIMIT = -8 /* sr_linear_fwd_static: the call needs more scratch than the   */
                            /* library's static array holds (SRQ_STATIC_SCRATCH_BYTES)      */
} srq_status;

typedef enum { SRQ_F32 = 0, SRQ_BF16 = 1 } srq_dtype; /* dtype of a source tensor */

/* Target grid.  INT8: two's complement, [-127,127].  INT4: [-7,7], two per byte, element 2k
 * in bits 3:0 and 2k+1 in bits 7:4 of byte k (pairs run along the contiguous dimension of
 * the output).  E4M3 / E5M2: OCP 8-bit floats (bias 7 / 15, subnormals, max 448 / 57344;
 * never Inf, NaN only from NaN input).  Any zero result is stored as +0.
 * SRQ_NONE (Delta = 0, the identity of Def. 1) has no code form.  It is accepted in one place:
 * as the quantizer of the row operand of sr_linear_fwd (A) and sr_linear_bwd_data (dY), for
 * the objective with quantized weights and full-precision activations (Sec. 3.2); the other
 * fields of that srq_quant are then ignored.  Everywhere else it is SRQ_ERR_UNSUPPORTED. */
typedef enum {
  SRQ_NONE = 0, SRQ_INT8 = 1, SRQ_INT4 = 2, SRQ_E4M3 = 3, SRQ_E5M2 = 4,
  /* The 4-exponent-bit formats of the paper's experiments (Sec. 5) with 2 / 1 / 0 fraction bits.
   * The paper does not give their bias or subnormal rule; here they are the sub-grids of E4M3
   * with the same exponent range (subnormals at the spacing of the smallest normal binade),
   * Qmax 448 / 384 / 256, and their codes are the E4M3 codes of the same values (low 1 / 2 / 3
   * fraction bits zero), so that products treat them as E4M3. */
  SRQ_E4M2 = 5, SRQ_E4M1 = 6, SRQ_E4M0 = 7
} srq_kind;

typedef enum { SRQ_SR = 0, SRQ_RTN = 1 } srq_round; /* Def. 3 / Def. 2 */

/* One quantizer: the pair (Delta, eps) of the paper for one tensor. */
typedef struct {
  int32_t kind;            /* srq_kind                                                       */
  int32_t round;           /* srq_round                                                      */
  float scale;             /* Delta: finite, at least 2^-100 (1/scale * 2^16 stays finite)   */
  uint32_t flags;          /* 0, or a combination of the SRQ_FLAG_* bits below                */
  const float* scale_dev;  /* if not NULL: device pointer to the scale, read by the kernels  */
                           /* instead of `scale` (no host check is then possible)            */
  uint64_t seed;           /* Philox key                                                     */
  uint64_t counter_offset; /* first Philox block of this tensor; a tensor of n elements uses */
                           /* blocks [counter_offset, counter_offset + ceil(n/8))            */
} srq_quant;

/* How the linear entry points multiply two operands on 8-bit float grids (E4M3 / E5M2 and the
 * sub-grids of E4M3).
 * Default (flag clear): products are exact and sums are accumulated in binary32, so the result
 * equals the exact product of the quantized matrices (Sec. 2.2.2) to binary32 rounding.  Two
 * E5M2 operands are multiplied from their one-byte codes, widened to binary16 inside the kernel
 * (an E5M2 code is the high byte of the binary16 number of the same value), on the f16 matrix
 * pipeline.  For any other pair the quantizer writes each grid value as a bfloat16 number
 * (every E4M3 / E5M2 value is one) and the product runs on the bf16 matrix pipeline.  The two
 * pipelines group the contraction differently, so their binary32 sums can differ in the last
 * bits.
 * With SRQ_FLAG_F8_PIPELINE set on BOTH operands' quantizers the one-byte codes go to the fp8
 * matrix pipeline at twice the rate.  That hardware adds the products of each run of 8
 * consecutive contraction indices after aligning them to the largest one and truncating to 14
 * bits, so a product more than 2^13 times smaller than its group's largest loses low bits:
 * |error| <= 7 * 2^-13 * sum over groups of the group's largest |product| (plus binary32
 * rounding).  Integer formats ignore the flag: their products are exact in int32. */
enum { SRQ_FLAG_F8_PIPELINE = 1,
       /* counter_offset holds, instead of the offset itself, the device address (8-byte aligned, not
        * NULL) of a uint64 that holds it: the kernels read it when they run.  A launch recorded in a
        * HIP graph can then be replayed with fresh thresholds by updating that word on the device
        * between replays (by ceil(n/8) per tensor, as the host would advance the offset). */
       SRQ_FLAG_COUNTER_DEV = 2,
       /* on either quantizer of sr_linear_fwd: keep the quantize-once form (operands rounded into the
        * workspace by one launch, multiplied by a second) also where the call would round them inside
        * the product kernel; the results are the same, the flag exists so that the two forms can be
        * timed against each other.  Ignored everywhere else. */
       SRQ_FLAG_QUANTIZE_ONCE = 4 };

enum { SRQ_OP_FWD = 0, SRQ_OP_BWD_DATA = 1, SRQ_OP_BWD_WEIGHT = 2, SRQ_OP_BWD = 3, SRQ_OP_FWD_STASH = 4,
       SRQ_OP_BWD_STASHED = 5, SRQ_OP_FWD_WEIGHT_ONLY = 6, SRQ_OP_BWD_DATA_WEIGHT_ONLY = 7 };

/* Per-tensor scale for absmax scaling (a choice of Delta; the paper leaves Delta open):
 * *scale_out_dev = max|x_i| / Qmax(kind) over the finite elements, or 1 if that is zero, and
 * never below 2^-100, the smallest step the quantizer takes (a tensor of vanishing values is
 * then quantized on that grid, mostly to zero, instead of being saturated).
 * x: device, n elements of `dtype`, 16-byte aligned.  n may be 0 (result 1). */
int sr_absmax_scale(float* scale_out_dev, const void* x, int dtype, size_t n, int kind,
                    void* stream);

/* The same for several tensors at once (at most 8 requests), in two launches however many
 * there are.  Requests naming the same (x, n, dtype) share one pass over the tensor, so the
 * scales of A for its forward and backward quantizers cost one read of A.
 * workspace: device scratch of sr_absmax_workspace_bytes(reqs, count) bytes, 4-byte aligned;
 * it needs no initialisation.  reqs is host memory, read before the call returns. */
typedef struct {
  const void* x;        /* device, 16-byte aligned                  */
  int32_t dtype;        /* srq_dtype                                */
  int32_t kind;         /* srq_kind whose Qmax divides the maximum  */
  size_t n;             /* elements                                 */
  float* scale_out_dev; /* device, one float                        */
} srq_absmax_req;
int sr_absmax_scales(const srq_absmax_req* reqs, int count, void* workspace, size_t workspace_bytes,
                     void* stream);
size_t sr_absmax_workspace_bytes(const srq_absmax_req* reqs, int count);

/* Element-wise quantization of a rows x cols tensor (Def. 1-3).
 * codes: device output.  transpose_out = 0: same layout as x (rows x cols); 1: cols x rows.
 *        One byte per element, or one byte per two elements for SRQ_INT4.
 * x: device, 16-byte aligned.  Requirements: transpose_out = 0: any rows, cols (an odd
 * element count with SRQ_INT4 is SRQ_ERR_ALIGN); transpose_out = 1: cols % 8 == 0, and rows
 * even for SRQ_INT4.  rows * cols == 0 is a no-op. */
int sr_quantize(void* codes, const void* x, int dtype, size_t rows, size_t cols,
                int transpose_out, const srq_quant* q, void* stream);

/* Exact product of two code matrices with high-precision accumulation (Sec. 2.2.2):
 * out[p][q] = alpha * sum_r val(X[p][r]) * val(Z[q][r]) + beta * out[p][q].
 * X: P x R codes, Z: Q x R codes, one byte per element, R contiguous, both device and
 * 16-byte aligned; R % 16 == 0.  kinds: both integer (INT8; INT4 values held one per byte)
 * or both 8-bit float.  Integer pairs accumulate in int32 (exact while R * 127^2 < 2^31);
 * float pairs run on the fp8 matrix pipeline (see SRQ_FLAG_F8_PIPELINE for its rounding).
 * beta must be 0 or 1.
 * workspace: device scratch of at least sr_gemm_workspace_bytes(P, Q, R) bytes (may be
 * NULL when that is 0). */
int sr_gemm_codes(float* out, const void* X, int kindX, const void* Z, int kindZ, size_t P,
                  size_t Q, size_t R, float alpha, float beta, void* workspace,
                  size_t workspace_bytes, void* stream);
size_t sr_gemm_workspace_bytes(size_t P, size_t Q, size_t R);

/* The same product for operands held as bfloat16 values (the form in which the linear entry
 * points store E4M3 / E5M2 operands by default): X is P x R, Z is Q x R bfloat16, R % 8 == 0.
 * Products are exact and sums binary32, on the bf16 matrix pipeline. */
int sr_gemm_bf16(float* out, const void* X, const void* Z, size_t P, size_t Q, size_t R, float alpha,
                 float beta, void* workspace, size_t workspace_bytes, void* stream);
size_t sr_gemm_bf16_workspace_bytes(size_t P, size_t Q, size_t R);

/* The same product for two matrices of E5M2 codes, computed exactly as on the bf16 pipeline
 * (exact products, binary32 sums) but from the one-byte codes: an E5M2 code is the high byte of
 * the binary16 number of the same value, so the kernel widens the operands in registers and
 * multiplies on the f16 matrix pipeline.  This is how the linear entry points multiply when both
 * operands are E5M2 and SRQ_FLAG_F8_PIPELINE is clear.  X is P x R, Z is Q x R, R % 16 == 0. */
int sr_gemm_e5m2(float* out, const void* X, const void* Z, size_t P, size_t Q, size_t R, float alpha,
                 float beta, void* workspace, size_t workspace_bytes, void* stream);
size_t sr_gemm_e5m2_workspace_bytes(size_t P, size_t Q, size_t R);

/* Forward pass, Alg. 1:  Y = Q(A; qA_fwd) Q(W; qW_fwd)^T.
 * M, N, K multiples of 16.  workspace: sr_linear_workspace_bytes(SRQ_OP_FWD, M, N, K).
 * The operands are quantized once into the workspace and multiplied from there -- except for an
 * integer pair with an output of at most four 64 x 64 tiles and K <= 256, which is rounded inside
 * the product kernel (as sr_linear_fwd_fused; same result bit for bit, workspace untouched).
 * Weight-only objective (Sec. 3.2): with qA_fwd->kind == SRQ_NONE, Y = A Q(W; qW_fwd)^T with A
 * as it is: every product a * w_hat is exact and the sums are accumulated in binary32 (a
 * bfloat16 A is multiplied in place on the bf16 matrix pipeline, a binary32 A as three bfloat16
 * planes that sum to it; a non-finite element of A makes its row of Y NaN; that pipeline takes
 * subnormal numbers as zero, so parts of A below 2^-126 do not contribute).  W may use any
 * format.  workspace: sr_linear_workspace_bytes(SRQ_OP_FWD_WEIGHT_ONLY, M, N, K). */
int sr_linear_fwd(float* Y, const void* A, int dtypeA, const void* W, int dtypeW, size_t M,
                  size_t N, size_t K, const srq_quant* qA_fwd, const srq_quant* qW_fwd,
                  void* workspace, size_t workspace_bytes, void* stream);

/* The two halves of sr_linear_fwd and of sr_linear_bwd as calls of their own, for callers that run the
 * memory-bound half of one layer (rounding the operands into the workspace: SRQ_PHASE_QUANTIZE) beside
 * the matrix half of another (the products from the workspace: SRQ_PHASE_PRODUCT) on two streams; the
 * quantizer kernels fit into the registers and LDS the product kernels leave free on a CU.  Arguments as
 * for the whole call, plus `phase`; the two calls of a pair take the same arguments and workspace, the
 * caller orders them (same stream, or an event) and keeps the workspace untouched in between.
 * SRQ_PHASE_BOTH is the whole call, except that sr_linear_fwd_phase always rounds into the workspace
 * (never inside the product kernel).  The results equal those of the whole call bit for bit.  The
 * product half does not read A, W or dY (the pointers are still checked).  Not available for the
 * weight-only objective (SRQ_NONE: SRQ_ERR_UNSUPPORTED); an unknown phase is SRQ_ERR_FORMAT. */
enum { SRQ_PHASE_QUANTIZE = 1, SRQ_PHASE_PRODUCT = 2, SRQ_PHASE_BOTH = 3 };
int sr_linear_fwd_phase(float* Y, const void* A, int dtypeA, const void* W, int dtypeW, size_t M,
                        size_t N, size_t K, const srq_quant* qA_fwd, const srq_quant* qW_fwd,
                        void* workspace, size_t workspace_bytes, int phase, void* stream);
int sr_linear_bwd_phase(float* dA, float* dW, const void* dY, int dtypedY, const void* W, int dtypeW,
                        const void* A, int dtypeA, size_t M, size_t N, size_t K,
                        const srq_quant* qdY_bwd, const srq_quant* qW_bwd, const srq_quant* qA_bwd,
                        float beta, void* workspace, size_t workspace_bytes, int phase, void* stream);

/* Alg. 1 with both quantizers inside the product kernel: every workgroup reads its tiles of A and
 * W in their source precision, applies Eq. 1 (the thresholds of an element are fixed by its
 * index, so the codes are the ones sr_quantize gives) and multiplies from LDS; no quantized
 * operand is written to memory and no workspace is needed.  An element is rounded again by every
 * output tile that uses it, so the call is meant for outputs of a few tiles (small M and N);
 * on large shapes it is many times slower than sr_linear_fwd and exists there to be measured.
 * Formats: qA_fwd and qW_fwd both integer (results equal to sr_linear_fwd bit for bit: the int32
 * sums are exact), or both SRQ_E5M2 (exact products, binary32 sums; SRQ_FLAG_F8_PIPELINE is
 * ignored); any other pair, and SRQ_NONE, is SRQ_ERR_UNSUPPORTED.  M, N, K multiples of 16. */
int sr_linear_fwd_fused(float* Y, const void* A, int dtypeA, const void* W, int dtypeW, size_t M,
                        size_t N, size_t K, const srq_quant* qA_fwd, const srq_quant* qW_fwd,
                        void* stream);

/* sr_linear_fwd for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * same kernels, same results bit for bit as sr_linear_fwd (it is that call); the scratch (quantized operands,
 * slice partials) is a static device array of SRQ_STATIC_SCRATCH_BYTES inside the library, one
 * copy per GPU, held until the process ends.  The call allocates nothing (no hipMalloc / hipFree,
 * no allocating runtime or library routine); the array's address is looked up once per device on
 * the first call there.  A call that would need a larger workspace than the array
 * (sr_linear_workspace_bytes(SRQ_OP_FWD or SRQ_OP_FWD_WEIGHT_ONLY, M, N, K) > the limit) returns
 * SRQ_ERR_STATIC_LIMIT and launches nothing; all other errors as sr_linear_fwd.
 * All calls on one GPU share that GPU's array, which keeps the previous call's contents (nothing
 * in it needs clearing: a call writes every byte it later reads).  Calls that overlap on one GPU
 * -- different streams without ordering, or several host threads -- race on it: order them. */
#define SRQ_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
size_t sr_linear_fwd_static_limit(void);
int sr_linear_fwd_static(float* Y, const void* A, int dtypeA, const void* W, int dtypeW, size_t M,
                         size_t N, size_t K, const srq_quant* qA_fwd, const srq_quant* qW_fwd,
                         void* stream);

/* Backward pass, Alg. 2, input gradient:  dA = Q(dY; qdY_bwd) Q(W; qW_bwd).
 * Weight-only objective: with qdY_bwd->kind == SRQ_NONE, dA = dY Q(W; qW_bwd), computed as in
 * sr_linear_fwd; the qW of the forward pass gives the same quantized weights (one copy per
 * mini-batch).  workspace: sr_linear_workspace_bytes(SRQ_OP_BWD_DATA_WEIGHT_ONLY, M, N, K).
 * (The weight gradient of that objective, dY^T A, has no quantized operand and is not part of
 * this library.) */
int sr_linear_bwd_data(float* dA, const void* dY, int dtypedY, const void* W, int dtypeW,
                       size_t M, size_t N, size_t K, const srq_quant* qdY_bwd,
                       const srq_quant* qW_bwd, void* workspace, size_t workspace_bytes,
                       void* stream);

/* Backward pass, Alg. 2, weight gradient:  dW = beta * dW + Q(dY; qdY_bwd)^T Q(A; qA_bwd).
 * The same qdY_bwd as in sr_linear_bwd_data gives the same quantized gradient, as Alg. 2
 * uses one.  beta = 1 accumulates micro-batches (Sec. 6.1); beta must be 0 or 1. */
int sr_linear_bwd_weight(float* dW, const void* dY, int dtypedY, const void* A, int dtypeA,
                         size_t M, size_t N, size_t K, const srq_quant* qdY_bwd,
                         const srq_quant* qA_bwd, float beta, void* workspace,
                         size_t workspace_bytes, void* stream);

/* The whole backward pass of Alg. 2 in one call: dA and dW as the two entry points above
 * would give them with the same quantizers, but the output gradient is read and quantized once
 * and all three operands are quantized in one launch.  The results are equal bit for bit
 * whenever the two products use the same pipeline in both forms of the call (always, except
 * when exactly one of W, A shares the E5M2 format with dY: the stored Q(dY) then has to serve
 * both products as bfloat16, and the E5M2 x E5M2 product differs from the separate call in the
 * order of its binary32 sums).  The form in which the workspace holds the quantized operands is
 * the library's own (a 4-bit Q(dY) of a binary32 dY, for one, is kept two values per byte for the
 * products that run on 256 x 256 tiles; the results are those of one byte per value bit for bit).
 * workspace: sr_linear_workspace_bytes(SRQ_OP_BWD, M, N, K). */
int sr_linear_bwd(float* dA, float* dW, const void* dY, int dtypedY, const void* W, int dtypeW,
                  const void* A, int dtypeA, size_t M, size_t N, size_t K, const srq_quant* qdY_bwd,
                  const srq_quant* qW_bwd, const srq_quant* qA_bwd, float beta, void* workspace,
                  size_t workspace_bytes, void* stream);

/* Alg. 1 and Alg. 2 with the backward operands of A and W saved in code form by the forward
 * pass ("saved for backward" as codes): A and W are read once per step instead of twice, and the
 * caller need not keep A in binary32 for the backward pass.
 *
 * sr_linear_fwd_stash computes Y exactly as sr_linear_fwd(.., qA_fwd, qW_fwd) does and, in the
 * same pass over A and W, writes Q(A; qA_bwd)^T and Q(W; qW_bwd)^T -- the very codes
 * sr_linear_bwd would produce -- into `stash` (device, 256-byte aligned, at least
 * sr_linear_stash_bytes(M, N, K) bytes, owned by the caller, opaque).  qA_fwd and qW_fwd must be
 * integer formats (else SRQ_ERR_UNSUPPORTED); qA_bwd and qW_bwd any pair a product accepts.
 * sr_linear_bwd_stashed then gives dA and dW bit for bit as sr_linear_bwd would with the same
 * three backward quantizers, reading only dY; qA_bwd and qW_bwd must be the ones the stash was
 * written with (their scales multiply the results; their formats select the product pipeline).
 * workspace: sr_linear_workspace_bytes(SRQ_OP_FWD_STASH / SRQ_OP_BWD_STASHED, M, N, K).
 * Errors as for sr_linear_fwd / sr_linear_bwd; a stash that is NULL, misaligned or too small is
 * SRQ_ERR_WORKSPACE. */
size_t sr_linear_stash_bytes(size_t M, size_t N, size_t K);
int sr_linear_fwd_stash(float* Y, const void* A, int dtypeA, const void* W, int dtypeW, size_t M, size_t N,
                        size_t K, const srq_quant* qA_fwd, const srq_quant* qW_fwd, const srq_quant* qA_bwd,
                        const srq_quant* qW_bwd, void* stash, size_t stash_bytes, void* workspace,
                        size_t workspace_bytes, void* stream);
int sr_linear_bwd_stashed(float* dA, float* dW, const void* dY, int dtypedY, size_t M, size_t N, size_t K,
                          const srq_quant* qdY_bwd, const srq_quant* qW_bwd, const srq_quant* qA_bwd,
                          const void* stash, size_t stash_bytes, float beta, void* workspace,
                          size_t workspace_bytes, void* stream);
/* The same two calls in halves (`phase` as for sr_linear_fwd_phase: the quantizer launch into the
 * workspace and the stash, or the products from them, or both); the two calls of a pair take the
 * same arguments, workspace and stash, and the caller orders them. */
int sr_linear_fwd_stash_phase(float* Y, const void* A, int dtypeA, const void* W, int dtypeW, size_t M, size_t N,
                              size_t K, const srq_quant* qA_fwd, const srq_quant* qW_fwd,
                              const srq_quant* qA_bwd, const srq_quant* qW_bwd, void* stash, size_t stash_bytes,
                              void* workspace, size_t workspace_bytes, int phase, void* stream);
int sr_linear_bwd_stashed_phase(float* dA, float* dW, const void* dY, int dtypedY, size_t M, size_t N, size_t K,
                                const srq_quant* qdY_bwd, const srq_quant* qW_bwd, const srq_quant* qA_bwd,
                                const void* stash, size_t stash_bytes, float beta, void* workspace,
                                size_t workspace_bytes, int phase, void* stream);

/* Weight update of Eq. 10 with the weights stored in bfloat16, in place:
 *     w[i] <- Q(w[i] - eta * g[i]),   i in [0, n)
 * Q is the threshold quantizer of Eq. 1 on the bfloat16 grid (8 exponent bits, 7 fraction
 * bits; subnormals kept), stochastic (round_mode = SRQ_SR: the threshold of element i comes
 * from 16-bit slice i of the Philox stream (seed, counter_offset), as in sr_quantize) or
 * nearest with ties toward +inf (SRQ_RTN).  u = w - eta * g is formed in binary32 with one
 * rounding per operation, clamped to the largest finite bfloat16; NaN gives 0x7FC0; a zero
 * result is +0.  With g = 0 the weights come back unchanged (-0 becomes +0).
 * w_bf16: device, n bfloat16 values, read and written; g: device, n floats; both 16-byte
 * aligned.  eta: host value, finite.  n = 0 is a no-op.  The stream advances by ceil(n / 8)
 * blocks. */
int sr_update_bf16(void* w_bf16, const float* g, float eta, size_t n, int round_mode, uint64_t seed,
                   uint64_t counter_offset, void* stream);

/* Bytes of device scratch the linear entry points need (quantized operands in the layout
 * the product wants, plus split partial sums), for any format.  op: SRQ_OP_*. */
size_t sr_linear_workspace_bytes(int op, size_t M, size_t N, size_t K);

const char* sr_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* SRQ_H */
