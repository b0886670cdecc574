// Operands of the weight-only objective (Sec. 3.2: quantized weights, activations and gradients
// in full precision) in the form the bf16 matrix pipeline multiplies exactly: a binary32 operand
// as three bfloat16 planes whose sum is the operand, laid side by side along the contraction
// (row m = [p0 row | p1 row | p2 row]) so that one product over the tripled contraction, against
// the weights repeated three times, adds the planes inside the accumulators; integer codes as
// the bfloat16 numbers of their values.  HBM-bound element-wise kernels.
#include "srq_internal.hpp"

namespace srq {
namespace {

constexpr int WBLOCK = 256;
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// x = p0 + p1 + p2 exactly, each pi a bfloat16 number: p0 is x cut to its top 8 significand
// bits, p1 the remainder cut the same way, p2 what is then left (binary32 has 24 bits; both
// subtractions are exact).  A non-finite x gives a NaN plane.
__device__ __forceinline__ void split3(float x, uint32_t& b0, uint32_t& b1, uint32_t& b2) {
  const uint32_t u0 = __float_as_uint(x) & 0xFFFF0000u;
  const float r1 = __fsub_rn(x, __uint_as_float(u0));
  const uint32_t u1 = __float_as_uint(r1) & 0xFFFF0000u;
  const float r2 = __fsub_rn(r1, __uint_as_float(u1));
  b0 = u0 >> 16;
  b1 = u1 >> 16;
  b2 = __float_as_uint(r2) >> 16;
}

// out: rows x (3 * cols) bfloat16; n4 = rows * cols / 4 quads, row_quads = cols / 4
__global__ __launch_bounds__(WBLOCK) void split3_kernel(uint16_t* __restrict__ out, const float* __restrict__ x,
                                                        size_t n4, uint32_t row_quads) {
  const f32x4* src = reinterpret_cast<const f32x4*>(x);
  u32x2* dst = reinterpret_cast<u32x2*>(out);
  for (size_t i = (size_t)blockIdx.x * WBLOCK + threadIdx.x; i < n4; i += (size_t)gridDim.x * WBLOCK) {
    const size_t row = i / row_quads;
    u32x2* p0 = dst + row * 2 * row_quads + i;  // = (row * 3) * row_quads + (i - row * row_quads)
    u32x2* p1 = p0 + row_quads;
    u32x2* p2 = p1 + row_quads;
    const f32x4 v = __builtin_nontemporal_load(src + i);
    uint32_t a[4], b[4], c[4];
    split3(v.x, a[0], b[0], c[0]);
    split3(v.y, a[1], b[1], c[1]);
    split3(v.z, a[2], b[2], c[2]);
    split3(v.w, a[3], b[3], c[3]);
    *p0 = u32x2{a[0] | (a[1] << 16), a[2] | (a[3] << 16)};
    *p1 = u32x2{b[0] | (b[1] << 16), b[2] | (b[3] << 16)};
    *p2 = u32x2{c[0] | (c[1] << 16), c[2] | (c[3] << 16)};
  }
}

// out (rows x 3 cols) = [in row | in row | in row], 16-byte chunks of 8 bfloat16; n8 = rows * cols / 8
__global__ __launch_bounds__(WBLOCK) void repeat3_kernel(uint16_t* __restrict__ out, const uint16_t* __restrict__ in,
                                                         size_t n8, uint32_t row_chunks) {
  const u32x4* src = reinterpret_cast<const u32x4*>(in);
  u32x4* dst = reinterpret_cast<u32x4*>(out);
  for (size_t i = (size_t)blockIdx.x * WBLOCK + threadIdx.x; i < n8; i += (size_t)gridDim.x * WBLOCK) {
    const size_t row = i / row_chunks;
    const u32x4 v = src[i];
    u32x4* p = dst + row * 2 * row_chunks + i;
    p[0] = v;
    p[row_chunks] = v;
    p[2 * (size_t)row_chunks] = v;
  }
}

// Integer codes (one value per byte, two's complement, |v| <= 127) -> bfloat16 numbers; n8 = n / 8
__global__ __launch_bounds__(WBLOCK) void int_codes_to_bf16_kernel(uint16_t* __restrict__ out,
                                                                   const uint8_t* __restrict__ codes, size_t n8) {
  const u32x2* src = reinterpret_cast<const u32x2*>(codes);
  u32x4* dst = reinterpret_cast<u32x4*>(out);
  for (size_t i = (size_t)blockIdx.x * WBLOCK + threadIdx.x; i < n8; i += (size_t)gridDim.x * WBLOCK) {
    const u32x2 w = src[i];
    uint32_t h[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int v = (int)(int8_t)((e < 4 ? w.x : w.y) >> (8 * (e & 3)));
      h[e] = __float_as_uint((float)v) >> 16;  // exact: at most 7 significant bits
    }
    dst[i] = u32x4{h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
  }
}

unsigned grid_for_items(size_t items) {
  size_t blocks = (items + WBLOCK - 1) / WBLOCK;
  if (blocks < 1) blocks = 1;
  if (blocks > 65536) blocks = 65536;
  return (unsigned)blocks;
}

}  // namespace

hipError_t launch_split3(uint16_t* out, const float* x, size_t rows, size_t cols, hipStream_t stream) {
  const size_t n4 = rows * cols / 4;
  split3_kernel<<<grid_for_items(n4), WBLOCK, 0, stream>>>(out, x, n4, (uint32_t)(cols / 4));
  return hipGetLastError();
}

hipError_t launch_repeat3(uint16_t* out, const uint16_t* in, size_t rows, size_t cols, hipStream_t stream) {
  const size_t n8 = rows * cols / 8;
  repeat3_kernel<<<grid_for_items(n8), WBLOCK, 0, stream>>>(out, in, n8, (uint32_t)(cols / 8));
  return hipGetLastError();
}

hipError_t launch_int_codes_to_bf16(uint16_t* out, const uint8_t* codes, size_t n, hipStream_t stream) {
  int_codes_to_bf16_kernel<<<grid_for_items(n / 8), WBLOCK, 0, stream>>>(out, codes, n / 8);
  return hipGetLastError();
}

}  // namespace srq
