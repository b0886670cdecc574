// Launchers shared between the translation units of the library (host side).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/srq.h"

namespace srq {

// How a quantize launch stores its codes.
enum StoreMode {
  STORE_BYTE = 0,   // one byte per element (INT4 values sign-extended to the byte)
  STORE_NIBBLE = 1, // INT4 only: two elements per byte along the output's contiguous dim
  STORE_BF16 = 2    // E4M3 / E5M2 only: the grid value itself as bfloat16 (two bytes per element)
};

struct QuantArgs {
  int kind, round, dtype, store;
  float scale;
  const float* scale_dev;
  uint64_t seed, counter_offset;
  const uint64_t* counter_dev;  // if not null: its value is added to counter_offset on the device
};

// codes: rows x cols (transpose_out = 0) or cols x rows (1).  Shapes already validated.
hipError_t launch_quantize(void* codes, const void* x, size_t rows, size_t cols, int transpose_out,
                           const QuantArgs& a, hipStream_t stream);

// Several quantizations in one launch (the operands of a product; in the fused backward pass
// the output gradient in both layouts).
constexpr int QUANT_JOBS_MAX = 3;
struct QuantJob {
  const void* x;
  uint8_t* out;    // rows x cols codes, or cols x rows when transpose
  uint8_t* out2;   // transpose only: optional extra rows x cols output, else nullptr:
                   //   kind2 == 0: the same codes again, in the source layout
                   //   kind2 == SRQ_INT8 / SRQ_INT4: the byte codes of a second, integer quantizer of the
                   //   same tensor (its own scale, rounding mode and stream position), source layout
  uint32_t rows, cols;
  int kind, round, dtype, store, transpose;
  float scale;
  const float* scale_dev;
  uint64_t seed, counter_offset;
  const uint64_t* counter_dev;   // if not null: its value is added to counter_offset on the device
  int kind2, round2;
  float scale2;
  const float* scale_dev2;
  uint64_t seed2, counter_offset2;
  const uint64_t* counter_dev2;
  // SRQ_INT4 from a binary32 source, transposing jobs: write the transposed output (pack_t) or the
  // same-codes output in the source layout (pack_2, kind2 == 0) two values per byte, in the form
  // gemm_takes_packed_x describes (runs of 16 along rows, respectively along columns)
  int pack_t, pack_2;
  uint32_t first_block, nblocks;  // filled by the launcher
};
struct QuantJobs {
  int njobs;
  QuantJob job[QUANT_JOBS_MAX];
};
hipError_t launch_quantize_jobs(QuantJobs& jobs, hipStream_t stream);

// Several per-tensor scales in two launches: up to ABSMAX_MAX distinct tensors and
// ABSMAX_MAX scales (a tensor may feed several formats).
constexpr int ABSMAX_MAX = 8;
struct AbsmaxBatch {
  int ntensors, nouts;
  const void* x[ABSMAX_MAX];
  size_t n[ABSMAX_MAX];
  int dtype[ABSMAX_MAX];
  uint32_t first_block[ABSMAX_MAX], nblocks[ABSMAX_MAX];
  int out_tensor[ABSMAX_MAX], out_kind[ABSMAX_MAX];
  float out_qmax[ABSMAX_MAX];
  float* out[ABSMAX_MAX];
  uint32_t* partial;  // one word per launched block
};
size_t absmax_batch_plan(AbsmaxBatch& b);  // fills first_block / nblocks, returns the block count
hipError_t launch_absmax_batch(AbsmaxBatch& b, hipStream_t stream);

// Eq. 10 on bfloat16 weights, in place: w[i] <- Q(w[i] - eta * g[i]); element i takes slice i of
// the Philox stream that starts counter_offset blocks in.
hipError_t launch_update_bf16(uint16_t* w, const float* g, float eta, size_t n, int round, uint64_t seed,
                              uint64_t counter_offset, hipStream_t stream);

// Weight-only objective (Sec. 3.2).  split3: x (rows x cols binary32, cols % 8 == 0) as rows x 3 cols
// bfloat16, row m = [p0 | p1 | p2] with p0 + p1 + p2 = x row m exactly.  repeat3: rows x cols bfloat16
// -> rows x 3 cols, each row three times over.  Integer codes (n bytes, n % 8 == 0) -> bfloat16 values.
hipError_t launch_split3(uint16_t* out, const float* x, size_t rows, size_t cols, hipStream_t stream);
hipError_t launch_repeat3(uint16_t* out, const uint16_t* in, size_t rows, size_t cols, hipStream_t stream);
hipError_t launch_int_codes_to_bf16(uint16_t* out, const uint8_t* codes, size_t n, hipStream_t stream);

hipError_t launch_absmax_scale(float* scale_out_dev, const void* x, int dtype, size_t n, int kind,
                               hipStream_t stream);

// out[P][Q] = alpha_scale * sum_r X[p][r] Z[q][r] (+ out if accumulate); alpha_scale =
// alpha * (*sx_dev or sx) * (*sz_dev or sz), computed on the device in binary32.
struct GemmScale {
  float alpha;
  float sx, sz;
  const float* sx_dev;
  const float* sz_dev;
};
// Which matrix pipeline multiplies the operands.
enum Pipe {
  PIPE_I8 = 0,   // int8 codes, int32 accumulators (exact)
  PIPE_F8 = 1,   // E4M3 / E5M2 codes on the fp8 pipeline (hardware aligns groups of 8 products)
  PIPE_BF16 = 2, // E4M3 / E5M2 grid values widened to bfloat16: exact products, binary32 sums
  PIPE_F16C = 3  // E5M2 codes (both operands), widened to binary16 inside the kernel: the same arithmetic
                 // as PIPE_BF16 from one byte per element
};
// R is the contraction length in elements; operand rows hold R bytes (PIPE_I8, PIPE_F8) or
// 2 R bytes (PIPE_BF16).
size_t gemm_workspace_bytes(size_t P, size_t Q, size_t R, int pipe);
// operand matrices must stay below 2 GiB (32-bit buffer offsets with an out-of-range sentinel)
bool gemm_operands_addressable(size_t P, size_t Q, size_t R, int pipe);
// pitch: bytes between consecutive operand rows (both operands), >= the row length.
// The sum of the contraction slices of a product (fixed order, then scale): run by the product's
// own launcher, or left to the caller (`defer`) who hands it to a LATER product launch (`carry`)
// whose last workgroups then do it -- memory-bound work beside the tiles of an unrelated product
// instead of a launch of its own.  total == 0: nothing to sum.
struct SliceSum {
  const uint32_t* partial;  // nsplit x total raw accumulators
  float* out;
  uint32_t nsplit;
  size_t total;
  GemmScale s;
  int accumulate, is_int;
};
hipError_t launch_gemm_codes(float* out, const uint8_t* X, int kindX, const uint8_t* Z, int kindZ,
                             size_t P, size_t Q, size_t R, size_t pitch, int pipe, const GemmScale& s,
                             bool accumulate, void* workspace, hipStream_t stream,
                             const SliceSum* carry = nullptr, SliceSum* defer = nullptr, bool x_packed = false);
// x_packed: X holds 4-bit integers two per byte -- byte j of every 8 holds elements j (low nibble)
// and j + 8 (high nibble) of a run of 16 along the contraction -- in rows of pitch / 2 bytes, and
// s.alpha carries a factor 1/16 (the kernel multiplies 16 * value).  Only where
// gemm_takes_packed_x says so: the int8 pipeline on the 256 x 256 tiles.
bool gemm_takes_packed_x(size_t P, size_t Q, size_t R, int pipe);
// a deferred slice sum that found no later launch to ride on
hipError_t launch_slice_sum(const SliceSum& r, hipStream_t stream);

// Alg. 1 with the quantizers inside the product kernel (srq_fused.hip): out (P x Q) =
// Q(x)[P x R] . Q(z)[Q x R]^T from the source tensors, no codes in memory.  Formats: both integer,
// or both E5M2.
bool fused_pair_supported(int kind_x, int kind_z);
hipError_t launch_fused_fwd(float* out, const void* x, const QuantArgs& qx, const void* z, const QuantArgs& qz,
                            size_t P, size_t Q, size_t R, hipStream_t stream);

inline bool kind_is_int(int k) { return k == SRQ_INT8 || k == SRQ_INT4; }
// 8-bit float codes: E4M3, E5M2 and the sub-grids of E4M3 (stored as E4M3 codes)
inline bool kind_is_f8(int k) { return k >= SRQ_E4M3 && k <= SRQ_E4M0; }

}  // namespace srq
