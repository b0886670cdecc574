// Matrix-pipeline adapters shared by the product kernels: what a lane reads from LDS for one
// contraction sub-step, how that becomes MFMA operands, and the MFMA itself (gfx950).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace srq {
namespace mma {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) void lds_void;

constexpr int BK = 128;  // bytes of contraction per LDS stage

// raw_t: what a lane reads from LDS for one contraction sub-step (a multiple of 16 bytes);
// frag_t: what the MFMA(s) of that sub-step consume; expand() turns one into the other.
struct I8Mma {
  using acc_t = v16i;
  using raw_t = v4i;
  using frag_t = v4i;
  static constexpr bool WIDENS = false;
  static __device__ __forceinline__ frag_t expand(raw_t r) { return r; }
  static constexpr int KSTEP = 32;  // contraction bytes per MFMA
  static __device__ __forceinline__ acc_t mma(frag_t a, frag_t b, acc_t c) {
    return __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ float to_f32(int v) { return (float)v; }
  static __device__ __forceinline__ int from_bits(uint32_t b) { return (int)b; }
  static __device__ __forceinline__ uint32_t bits(int v) { return (uint32_t)v; }
};

// bfloat16 operands (the 8-bit float grid values widened by the quantizer): products are exact
// and the accumulation is a true binary32 one, unlike the fp8 pipeline, which aligns the
// eight products of a group to 14 bits before adding them.
struct BF16Mma {
  using acc_t = v16f;
  using raw_t = v4i;
  using frag_t = v4i;  // 8 bfloat16
  static constexpr bool WIDENS = false;
  static __device__ __forceinline__ frag_t expand(raw_t r) { return r; }
  static constexpr int KSTEP = 32;  // bytes: 16 elements per MFMA
  static __device__ __forceinline__ acc_t mma(frag_t a, frag_t b, acc_t c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, b), c,
                                                   0, 0, 0);
  }
  static __device__ __forceinline__ float to_f32(float v) { return v; }
  static __device__ __forceinline__ float from_bits(uint32_t b) { return __uint_as_float(b); }
  static __device__ __forceinline__ uint32_t bits(float v) { return __float_as_uint(v); }
};

// FA / FB: format select of the first / second MFMA operand, 0 = E4M3, 1 = E5M2
template <int FA, int FB>
struct F8Mma {
  using acc_t = v16f;
  using raw_t = v8i;
  using frag_t = v8i;
  static constexpr bool WIDENS = false;
  static __device__ __forceinline__ frag_t expand(raw_t r) { return r; }
  static constexpr int KSTEP = 64;
  static __device__ __forceinline__ acc_t mma(frag_t a, frag_t b, acc_t c) {
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, FA, FB, 0, 0, 0, 0);
  }
  static __device__ __forceinline__ float to_f32(float v) { return v; }
  static __device__ __forceinline__ float from_bits(uint32_t b) { return __uint_as_float(b); }
  static __device__ __forceinline__ uint32_t bits(float v) { return __float_as_uint(v); }
};

// E5M2 codes on the f16 pipeline.  E5M2 is binary16 cut to its high byte, so (code << 8) is the
// binary16 number of the same value (subnormals included; the MFMA honours binary16 subnormals).
// A lane reads 16 codes per sub-step and widens them with four byte permutes into two operands
// of 8 halves: one sub-step is two MFMAs of depth 16.  Products are exact (6-bit significands),
// sums binary32, as on the bf16 pipeline, with half the operand bytes through LDS.
struct E5M2F16Mma {
  using acc_t = v16f;
  using raw_t = v4i;   // 16 codes
  using frag_t = v8i;  // 16 halves: codes 0..7, then 8..15
  static constexpr bool WIDENS = true;
  static constexpr int MFMA_PER_MMA = 2, VALU_PER_EXPAND = 8;
  static constexpr int KSTEP = 32;  // 32 codes (two lane groups of 16) per sub-step
  static __device__ __forceinline__ frag_t expand(raw_t r) {
    frag_t f;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const uint32_t d = (uint32_t)r[c];
      f[(c >> 1) * 4 + (c & 1) * 2 + 0] = (int)__builtin_amdgcn_perm(d, d, 0x010c000cu);  // codes 0,1 -> high bytes
      f[(c >> 1) * 4 + (c & 1) * 2 + 1] = (int)__builtin_amdgcn_perm(d, d, 0x030c020cu);  // codes 2,3
    }
    return f;
  }
  static __device__ __forceinline__ acc_t mma(frag_t a, frag_t b, acc_t c) {
    const v4i a0 = {a[0], a[1], a[2], a[3]}, a1 = {a[4], a[5], a[6], a[7]};
    const v4i b0 = {b[0], b[1], b[2], b[3]}, b1 = {b[4], b[5], b[6], b[7]};
    c = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, a0), __builtin_bit_cast(v8h, b0), c, 0, 0, 0);
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, a1), __builtin_bit_cast(v8h, b1), c, 0, 0, 0);
  }
  static __device__ __forceinline__ float to_f32(float v) { return v; }
  static __device__ __forceinline__ float from_bits(uint32_t b) { return __uint_as_float(b); }
  static __device__ __forceinline__ uint32_t bits(float v) { return __float_as_uint(v); }
};

// Operand tiles in LDS: rows of 128 bytes of the contraction, the 16-byte chunk c of row r stored
// at chunk c ^ ((r >> 1) & 7).  The LDS has 64 banks (256 bytes per cycle) and serves a
// ds_read_b128 sixteen lanes at a time: sixteen consecutive rows reading the same logical chunk
// then touch sixteen different 16-byte slots (two rows per 256 bytes, eight swizzle values per
// row parity), i.e. no bank conflicts.
__device__ __forceinline__ uint32_t swizzled_chunk(uint32_t row, uint32_t chunk) { return chunk ^ ((row >> 1) & 7u); }

}  // namespace mma
}  // namespace srq
