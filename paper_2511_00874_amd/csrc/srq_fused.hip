// Forward product with the quantizers inside it (the data flow of Alg. 1 taken literally):
//
//   Y[m][n] = s_A s_W * sum_k Q(A)[m][k] * Q(W)[n][k]
//
// Each workgroup reads its tiles of A and W in their source precision, applies Eq. 1 to every
// element (Def. 1 - 3; the threshold of an element is fixed by its index in the tensor, so the
// codes are those sr_quantize writes), puts the one-byte codes into LDS in the layout the MFMA
// operand reads want, and multiplies from there.  No code ever reaches global memory.
//
// The price is that an element is rounded again by every tile that uses it: A once per tile
// column, W once per tile row.  One Philox block and eight passes through Eq. 1 are about 200
// vector operations for eight elements, against the 32 x 32 x 32 MFMA those eight codes share
// with 2040 others, so the kernel is bound by the vector ALU as soon as the output has more than
// a few tiles.  It pays where the tensors are used once or twice and the contraction is short -- an
// output of a few tiles, where it also saves a launch -- and that is where sr_linear_fwd selects
// it; sr_linear_fwd_fused runs it on any shape so that the crossover can be measured.
#include "srq_device.hpp"
#include "srq_internal.hpp"
#include "srq_mma.hpp"

namespace srq {
namespace {

using namespace mma;

struct FusedOperand {
  const void* x;  // rows x R, R contiguous
  uint32_t rows;
  int dtype, kind, round;
  float scale;
  const float* scale_dev;
  uint64_t seed, counter_offset;
  const uint64_t* counter_dev;
};
struct FusedParams {
  float* out;  // P x Q
  FusedOperand X, Z;
  uint32_t P, Q, R;
};

// Quantize ROWS x 128 elements of `op` (tile rows from row0, contraction bytes from k0) into an
// LDS tile of 128-byte rows.  A thread takes groups of 8 consecutive elements of one row: one
// Philox block each, the block sr_quantize uses for the same elements.
template <int KIND, int ROWS>
__device__ __forceinline__ void stage_codes(uint8_t* tile, const FusedOperand& op, const InvScale& s, uint64_t block0,
                                            uint32_t row0, uint32_t k0, uint32_t R) {
  const uint32_t key0 = (uint32_t)op.seed, key1 = (uint32_t)(op.seed >> 32);
  const size_t n = (size_t)op.rows * R;
  for (uint32_t g = threadIdx.x; g < ROWS * 16u; g += 256u) {
    const uint32_t r = g >> 4, kg = g & 15u;
    const uint32_t row = row0 + r, k = k0 + kg * 8u;
    uint32_t c[8] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};  // beyond the tensor: zeros
    if (row < op.rows && k < R) {
      const size_t group = ((size_t)row * R + k) >> 3;  // R % 16 == 0: a group never leaves its row
      float v[8];
      if (op.dtype == SRQ_F32) load_group<SRQ_F32>(v, op.x, group, n);
      else load_group<SRQ_BF16>(v, op.x, group, n);
      if (op.round == SRQ_SR) quantize_group<KIND, SRQ_SR, false>(c, v, s, block0 + group, key0, key1);
      else quantize_group<KIND, SRQ_RTN, false>(c, v, s, block0 + group, key0, key1);
    }
    const uint32_t lo[4] = {c[0], c[1], c[2], c[3]}, hi[4] = {c[4], c[5], c[6], c[7]};
    const u32x2 w = {pack4_bytes(lo), pack4_bytes(hi)};
    *reinterpret_cast<u32x2*>(tile + r * BK + (swizzled_chunk(r, kg >> 1) << 4) + (kg & 1u) * 8u) = w;
  }
}

// KIND: SRQ_INTX (int8 / int4 values as bytes, int8 pipeline) or SRQ_E5M2 (codes, f16 pipeline).
// 256 threads: 2 x 2 waves, wave tile BM/2 x BN/2.
template <class MMA, int KIND, int BM, int BN>
__global__ __launch_bounds__(256) void fused_fwd_kernel(FusedParams f) {
  __shared__ __attribute__((aligned(1024))) uint8_t lds[(BM + BN) * BK];
  constexpr int WTM = BM / 2, WTN = BN / 2, TM = WTM / 32, TN = WTN / 32;
  using acc_t = typename MMA::acc_t;
  using frag_t = typename MMA::frag_t;
  using raw_t = typename MMA::raw_t;
  static_assert(sizeof(raw_t) == 16 && MMA::KSTEP == 32, "one 16-byte chunk per lane and MFMA step");
  constexpr int KSUB = BK / MMA::KSTEP;

  const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
  const uint32_t wp = wave >> 1, wq = wave & 1u;
  const uint32_t tiles_q = (f.Q + BN - 1) / BN;
  const uint32_t p0 = (blockIdx.x / tiles_q) * BM, q0 = (blockIdx.x % tiles_q) * BN;

  const InvScale sx = inv_scale(f.X.scale, f.X.scale_dev, f.X.kind);
  const InvScale sz = inv_scale(f.Z.scale, f.Z.scale_dev, f.Z.kind);
  const uint64_t bx = first_block(f.X.counter_offset, f.X.counter_dev);
  const uint64_t bz = first_block(f.Z.counter_offset, f.Z.counter_dev);

  // operand reads as in the product kernels: lane (row = lane % 32, kgroup = lane / 32)
  const uint32_t swz = ((lane >> 1) & 7u) ^ (lane >> 5);
  acc_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

  for (uint32_t k0 = 0; k0 < f.R; k0 += BK) {
    if (k0) __syncthreads();  // every wave has multiplied the stage before
    stage_codes<KIND, BM>(lds, f.X, sx, bx, p0, k0, f.R);
    stage_codes<KIND, BN>(lds + BM * BK, f.Z, sz, bz, q0, k0, f.R);
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < KSUB; ++ks) {
      frag_t xe[TM], ze[TN];
      const uint32_t chunk = (swz ^ (uint32_t)(2 * ks)) << 4;
#pragma unroll
      for (int i = 0; i < TM; ++i)
        xe[i] = MMA::expand(*reinterpret_cast<const raw_t*>(lds + (wp * WTM + i * 32 + (lane & 31u)) * BK + chunk));
#pragma unroll
      for (int j = 0; j < TN; ++j)
        ze[j] = MMA::expand(*reinterpret_cast<const raw_t*>(lds + BM * BK + (wq * WTN + j * 32 + (lane & 31u)) * BK + chunk));
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = MMA::mma(ze[j], xe[i], acc[i][j]);  // MFMA rows: q, columns: p
    }
  }

  // MFMA result register r of lane l: q = 8 (r / 4) + 4 (l / 32) + r % 4, p = l % 32
  const float sxv = f.X.scale_dev ? *f.X.scale_dev : f.X.scale, szv = f.Z.scale_dev ? *f.Z.scale_dev : f.Z.scale;
  const float s = __fmul_rn(1.0f, __fmul_rn(sxv, szv));
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const uint32_t p = p0 + wp * WTM + i * 32 + (lane & 31u);
#pragma unroll
      for (int gq = 0; gq < 4; ++gq) {
        const uint32_t q = q0 + wq * WTN + j * 32 + 8 * gq + 4 * (lane >> 5);
        if (p < f.P && q < f.Q) {  // Q % 16 == 0: the four entries are inside together
          v4f v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = __fmul_rn(MMA::to_f32(acc[i][j][4 * gq + e]), s);
          *reinterpret_cast<v4f*>(f.out + (size_t)p * f.Q + q) = v;
        }
      }
    }
}

FusedOperand make_operand(const void* x, size_t rows, const QuantArgs& a) {
  FusedOperand o;
  o.x = x; o.rows = (uint32_t)rows;
  o.dtype = a.dtype; o.kind = a.kind; o.round = a.round;
  o.scale = a.scale; o.scale_dev = a.scale_dev;
  o.seed = a.seed; o.counter_offset = a.counter_offset; o.counter_dev = a.counter_dev;
  return o;
}

template <class MMA, int KIND>
hipError_t launch_fused(const FusedParams& f, bool large_tiles, hipStream_t stream) {
  if (large_tiles) {
    const uint32_t blocks = ((f.P + 127) / 128) * ((f.Q + 127) / 128);
    fused_fwd_kernel<MMA, KIND, 128, 128><<<blocks, 256, 0, stream>>>(f);
  } else {
    const uint32_t blocks = ((f.P + 63) / 64) * ((f.Q + 63) / 64);
    fused_fwd_kernel<MMA, KIND, 64, 64><<<blocks, 256, 0, stream>>>(f);
  }
  return hipGetLastError();
}

}  // namespace

bool fused_pair_supported(int kind_x, int kind_z) {
  return (kind_is_int(kind_x) && kind_is_int(kind_z)) || (kind_x == SRQ_E5M2 && kind_z == SRQ_E5M2);
}

hipError_t launch_fused_fwd(float* out, const void* x, const QuantArgs& qx, const void* z, const QuantArgs& qz,
                            size_t P, size_t Q, size_t R, hipStream_t stream) {
  FusedParams f;
  f.out = out;
  f.X = make_operand(x, P, qx);
  f.Z = make_operand(z, Q, qz);
  f.P = (uint32_t)P; f.Q = (uint32_t)Q; f.R = (uint32_t)R;
  // 64 x 64 tiles while they still give every CU a workgroup; 128 x 128 beyond (half the re-rounding)
  const bool large = ((P + 63) / 64) * ((Q + 63) / 64) > 1024;
  if (kind_is_int(qx.kind)) return launch_fused<I8Mma, SRQ_INTX>(f, large, stream);
  return launch_fused<E5M2F16Mma, SRQ_E5M2>(f, large, stream);
}

}  // namespace srq
