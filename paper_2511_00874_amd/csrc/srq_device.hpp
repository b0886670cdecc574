// Device-side building blocks of the SR quantizer: the counter-based random bits and the
// per-element threshold quantizer (Def. 1 / Eq. 1, Def. 2, Def. 3) on the four target grids.
// gfx950 only.  Every floating-point step that decides a code is one IEEE binary32
// operation; the translation unit is built with -ffp-contract=off and the rounding-explicit
// intrinsics are used so that no multiply-add fusion can change a decision.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/srq.h"

namespace srq {

// ---- Philox4x32-10 (Salmon et al., SC'11), counter (block_lo, block_hi, 0, 0) ----------
// The key schedule is wave-uniform, so it lives in scalar registers; only the two 32x32->64
// multiplies and the xors per round are vector work.
__device__ __forceinline__ void philox_block(uint64_t block, uint32_t k0, uint32_t k1,
                                             uint32_t (&w)[4]) {
  uint32_t c0 = (uint32_t)block, c1 = (uint32_t)(block >> 32), c2 = 0u, c3 = 0u;
#pragma unroll
  for (int round = 0; round < 10; ++round) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    c1 = (uint32_t)p1;
    c3 = (uint32_t)p0;
    c0 = n0;
    c2 = n2;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  w[0] = c0; w[1] = c1; w[2] = c2; w[3] = c3;
}

// 16-bit slice j (0..7) of a block: low half of word 0 first.
__device__ __forceinline__ uint32_t r16_of(const uint32_t (&w)[4], int j) {
  return (w[j >> 1] >> (16 * (j & 1))) & 0xFFFFu;
}

// Threshold in (0,1): (r16 + 1/2) / 65536, exact in binary32.
__device__ __forceinline__ float eps_of(uint32_t r16) {
  return __builtin_fmaf((float)r16, 0x1p-16f, 0x1p-17f);
}

template <int KIND> struct Grid;
template <> struct Grid<SRQ_INT8> { static constexpr bool is_float = false; static constexpr float qmax = 127.0f; };
template <> struct Grid<SRQ_INT4> { static constexpr bool is_float = false; static constexpr float qmax = 7.0f; };
template <> struct Grid<SRQ_E4M3> {
  static constexpr bool is_float = true; static constexpr float qmax = 448.0f;
  static constexpr int mbits = 3, emin = -6;
};
template <> struct Grid<SRQ_E5M2> {
  static constexpr bool is_float = true; static constexpr float qmax = 57344.0f;
  static constexpr int mbits = 2, emin = -14;
};

// One element through Eq. 1 on grid KIND.  Returns the code in the low 8 bits (integers:
// two's complement byte; INT4 values are in [-7,7], sign-extended to the byte).  With
// AS_BF16 (8-bit float grids only) it returns instead the bfloat16 bit pattern of the grid
// point q * D itself -- every E4M3 / E5M2 value is a normal bfloat16 number -- which is what
// the exact (bf16 matrix pipeline) product consumes.
template <int KIND, bool AS_BF16 = false>
__device__ __forceinline__ uint32_t quantize_elem(float x, float inv, float eps) {
  using G = Grid<KIND>;
  float t = __fmul_rn(x, inv);                          // grid coordinate
  t = __builtin_amdgcn_fmed3f(t, -G::qmax, G::qmax);    // saturate (NaN fixed up below)
  uint32_t code;
  if constexpr (!G::is_float) {
    static_assert(!AS_BF16, "integer grids are stored as bytes");
    const float fl = __builtin_floorf(t);
    const float frac = __fsub_rn(t, fl);
    const int q = (int)fl + (frac >= eps ? 1 : 0);      // Eq. 1: down iff frac < eps
    code = (uint32_t)q & 0xFFu;
    if (x != x) code = 0u;
  } else {
    // spacing of the grid at t: D = 2^(e - m), e = max(floor(log2|t|), emin)
    const uint32_t a = __float_as_uint(t) & 0x7FFFFFFFu;
    const int eb = max((int)(a >> 23), G::emin + 127);  // biased e (0 and subnormals clamp)
    const float inv_d = __uint_as_float((uint32_t)(254 + G::mbits - eb) << 23);  // 2^(m - e)
    const float y = __fmul_rn(t, inv_d);                // exact: power-of-two scaling
    const float fl = __builtin_floorf(y);
    const float frac = __fsub_rn(y, fl);
    const int q = (int)fl + (frac >= eps ? 1 : 0);      // |q| in [0, 2^(m+1)]
    if constexpr (AS_BF16) {
      const float d = __uint_as_float((uint32_t)(eb - G::mbits) << 23);  // D = 2^(e - m)
      code = __float_as_uint(__fmul_rn((float)q, d)) >> 16;             // exact, <= 4 significant bits
      if (x != x) code = 0x7FC0u;
    } else {
      // sign | ((e - emin) << m) + |q| : covers subnormals (field 0), normals (the hidden one
      // of |q| bumps the field) and the carry into the next binade
      const uint32_t mag = ((uint32_t)(eb - (G::emin + 127)) << G::mbits) + (uint32_t)abs(q);
      code = mag | (q < 0 ? 0x80u : 0u);
      if (x != x) code = 0x7Fu;
    }
  }
  return code;
}

__device__ __forceinline__ float bf16_to_f32(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

// 1 / scale, correctly rounded, from a host value or a device-resident one.
__device__ __forceinline__ float inv_scale(float scale, const float* scale_dev) {
  const float s = scale_dev ? *scale_dev : scale;
  return __fdiv_rn(1.0f, s);
}

// ---- groups of 8 consecutive elements (one Philox block) -----------------------------------
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Load the 8 elements of group g (element index 8g..8g+7) as binary32; lanes beyond n read 0.
template <int SRC>
__device__ __forceinline__ void load_group(float (&v)[8], const void* x, size_t g, size_t n) {
  const size_t base = g * 8;
  if (base + 8 <= n) {
    if constexpr (SRC == SRQ_F32) {
      const f32x4* p = reinterpret_cast<const f32x4*>(static_cast<const float*>(x) + base);
      const f32x4 a = __builtin_nontemporal_load(p);
      const f32x4 b = __builtin_nontemporal_load(p + 1);
      v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
      v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    } else {
      const u32x4 a = __builtin_nontemporal_load(
          reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(x) + base));
      v[0] = bf16_to_f32(a.x & 0xFFFFu); v[1] = bf16_to_f32(a.x >> 16);
      v[2] = bf16_to_f32(a.y & 0xFFFFu); v[3] = bf16_to_f32(a.y >> 16);
      v[4] = bf16_to_f32(a.z & 0xFFFFu); v[5] = bf16_to_f32(a.z >> 16);
      v[6] = bf16_to_f32(a.w & 0xFFFFu); v[7] = bf16_to_f32(a.w >> 16);
    }
  } else {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float e = 0.0f;
      if (base + j < n) {
        if constexpr (SRC == SRQ_F32) e = static_cast<const float*>(x)[base + j];
        else e = bf16_to_f32(static_cast<const uint16_t*>(x)[base + j]);
      }
      v[j] = e;
    }
  }
}

// Quantize one group; c[j] = code byte of element j.
template <int KIND, int ROUND, bool AS_BF16>
__device__ __forceinline__ void quantize_group(uint32_t (&c)[8], const float (&v)[8], float inv,
                                               uint64_t block, uint32_t k0, uint32_t k1) {
  if constexpr (ROUND == SRQ_SR) {
    uint32_t w[4];
    philox_block(block, k0, k1, w);
#pragma unroll
    for (int j = 0; j < 8; ++j) c[j] = quantize_elem<KIND, AS_BF16>(v[j], inv, eps_of(r16_of(w, j)));
  } else {
#pragma unroll
    for (int j = 0; j < 8; ++j) c[j] = quantize_elem<KIND, AS_BF16>(v[j], inv, 0.5f);  // Def. 2
  }
}

}  // namespace srq
