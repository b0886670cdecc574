// Device-side building blocks of the SR quantizer: the counter-based random bits and the
// per-element threshold quantizer (Def. 1 / Eq. 1, Def. 2, Def. 3) on the four target grids.
// gfx950 only.
//
// Arithmetic.  The grid coordinate t = fl32(x * inv) is one binary32 multiply.  From there
// Eq. 1 is evaluated EXACTLY, in 16.16 fixed point: with y = t / D (a power-of-two scaling),
//     threshold eps = (r + 1/2) / 2^16,   y = f + frac,  f = floor(y)
//     round up  <=>  frac >= eps  <=>  frac * 2^16 >= r + 1/2  <=>  r < floor(frac * 2^16 + 1/2)
// and since floor(y * 2^16 + 1/2) = f * 2^16 + floor(frac * 2^16 + 1/2) =: U,
//     q = floor((U + 65535 - r) / 2^16)        (the carry out of the low 16 bits is "up").
// U is one v_cvt_rpi_i32_f32 (floor(x + 1/2), exact, saturating) of y * 2^16, which is itself
// exact.  Round-to-nearest (eps = 1/2) is  q = floor((floor(y * 2^16) + 32768) / 2^16).
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
    const uint32_t n0 = __builtin_amdgcn_bitop3_b32((uint32_t)(p1 >> 32), c1, k0, 0x96);  // three-way xor
    const uint32_t n2 = __builtin_amdgcn_bitop3_b32((uint32_t)(p0 >> 32), c3, k1, 0x96);
    c1 = (uint32_t)p1;
    c3 = (uint32_t)p0;
    c0 = n0;
    c2 = n2;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  w[0] = c0; w[1] = c1; w[2] = c2; w[3] = c3;
}

// floor(x + 1/2) and floor(x) as int32: exact, saturating (NaN gives INT_MAX)
__device__ __forceinline__ int cvt_rpi(float x) {
  int r;
  asm("v_cvt_rpi_i32_f32 %0, %1" : "=v"(r) : "v"(x));
  return r;
}
__device__ __forceinline__ int cvt_flr(float x) {
  int r;
  asm("v_cvt_flr_i32_f32 %0, %1" : "=v"(r) : "v"(x));
  return r;
}

// What is added to U before the shift: 65535 - r16 for stochastic rounding (r16 the element's
// 16 random bits), 32768 for round-to-nearest.
constexpr uint32_t RTN_ADDEND = 32768u;

// The four addends of two output words of a Philox block (elements 4h .. 4h+3 of a group,
// low half of the first word first).
__device__ __forceinline__ void sr_addends(uint32_t w0, uint32_t w1, uint32_t (&add)[4]) {
  const uint32_t n0 = ~w0, n1 = ~w1;  // 65535 - r in each half
  add[0] = n0 & 0xFFFFu; add[1] = n0 >> 16; add[2] = n1 & 0xFFFFu; add[3] = n1 >> 16;
}

template <int KIND> struct Grid;
template <> struct Grid<SRQ_INT8> { static constexpr bool is_float = false; static constexpr int qmax = 127; };
template <> struct Grid<SRQ_INT4> { static constexpr bool is_float = false; static constexpr int qmax = 7; };
template <> struct Grid<SRQ_E4M3> {
  static constexpr bool is_float = true; static constexpr float qmax = 448.0f;
  static constexpr int mbits = 3, emin = -6;
};
template <> struct Grid<SRQ_E5M2> {
  static constexpr bool is_float = true; static constexpr float qmax = 57344.0f;
  static constexpr int mbits = 2, emin = -14;
};
// E4M2 / E4M1 / E4M0: sub-grids of E4M3 whose fraction width and Qmax are run-time values (one
// instantiation serves the three); codes are written as E4M3 codes.
constexpr int SRQ_E4MX = 100;
template <> struct Grid<SRQ_E4MX> {
  static constexpr bool is_float = true; static constexpr float qmax = 0.0f;  // unused: InvScale::sub_qmax
  static constexpr int mbits = 0, emin = -6;                                  // mbits unused: InvScale::sub_m
};
__host__ __device__ constexpr bool kind_is_e4mx(int kind) { return kind >= SRQ_E4M2 && kind <= SRQ_E4M0; }
// INT8 / INT4 with the clamp as a run-time value (one instantiation serves both): used where a
// second, integer quantizer rides along with another format's pass over the same tensor.
constexpr int SRQ_INTX = 101;
template <> struct Grid<SRQ_INTX> { static constexpr bool is_float = false; static constexpr int qmax = 0; };  // InvScale::sub_qi

// Per-tensor constants of the multiply that produces the grid coordinate.
struct InvScale {
  float inv;    // fl32(1 / scale)
  float inv16;  // inv * 2^16 (exact): fl32(x * inv16) = fl32(x * inv) * 2^16
  int sub_m;        // SRQ_E4MX only: fraction bits (2, 1, 0)
  float sub_qmax;   // SRQ_E4MX only: 448, 384, 256
  int sub_qi;       // SRQ_INTX only: Qmax * 2^16 (127 or 7)
};

// One element through Eq. 1 on grid KIND.  Returns the code in the low 8 bits (integers:
// two's complement byte; INT4 values are in [-7,7], sign-extended to the byte).  With
// AS_BF16 (8-bit float grids only) it returns instead the bfloat16 bit pattern of the grid
// point q * D itself -- every E4M3 / E5M2 value is a normal bfloat16 number -- which is what
// the exact (bf16 matrix pipeline) product consumes.
// FIX_NAN = false leaves the NaN rule to the caller (quantize_quad applies it per quad).
// Integer codes come back sign-extended to 32 bits: take the low byte (or nibble).
template <int KIND, int ROUND, bool AS_BF16 = false, bool FIX_NAN = true>
__device__ __forceinline__ uint32_t quantize_elem(float x, const InvScale& s, uint32_t addend) {
  using G = Grid<KIND>;
  uint32_t code;
  if constexpr (!G::is_float) {
    static_assert(!AS_BF16, "integer grids are stored as bytes");
    const int QI = KIND == SRQ_INTX ? s.sub_qi : (G::qmax << 16);
    const float y16 = __fmul_rn(x, s.inv16);                            // t * 2^16, D = 1
    int u = ROUND == SRQ_SR ? cvt_rpi(y16) : cvt_flr(y16);              // saturating
    u = min(max(u, -QI), QI);                                           // clamp t to +-Qmax
    const int q = (u + (int)addend) >> 16;
    code = (uint32_t)q;
    if (FIX_NAN && x != x) code = 0u;
  } else {
    const int m = KIND == SRQ_E4MX ? s.sub_m : G::mbits;
    const float qm = KIND == SRQ_E4MX ? s.sub_qmax : G::qmax;
    float t = __fmul_rn(x, s.inv);                                      // grid coordinate
    t = __builtin_amdgcn_fmed3f(t, -qm, qm);                            // saturate (NaN fixed up below)
    // spacing of the grid at t: D = 2^(e - m), e = max(floor(log2|t|), emin)
    const uint32_t a = __float_as_uint(t) & 0x7FFFFFFFu;
    const int eb = max((int)(a >> 23), G::emin + 127);                  // biased e (0 and subnormals clamp)
    const float up16 = __uint_as_float((uint32_t)(270 + m - eb) << 23);  // 2^(16 + m - e)
    const float y16 = __fmul_rn(t, up16);                               // (t / D) * 2^16, exact
    const int u = ROUND == SRQ_SR ? cvt_rpi(y16) : cvt_flr(y16);
    const int q = (u + (int)addend) >> 16;                              // |q| in [0, 2^(m+1)]
    if constexpr (AS_BF16) {
      const float d = __uint_as_float((uint32_t)(eb - m) << 23);        // D = 2^(e - m)
      code = __float_as_uint(__fmul_rn((float)q, d)) >> 16;             // exact, <= 4 significant bits
      if (FIX_NAN && x != x) code = 0x7FC0u;
    } else {
      // sign | ((e - emin) << m) + |q| : covers subnormals (field 0), normals (the hidden one
      // of |q| bumps the field) and the carry into the next binade
      uint32_t mag = ((uint32_t)(eb - (G::emin + 127)) << m) + (uint32_t)abs(q);
      if constexpr (KIND == SRQ_E4MX) mag <<= 3 - m;                    // the E4M3 code of the same value
      code = mag | (q < 0 ? 0x80u : 0u);
      if (FIX_NAN && x != x) code = 0x7Fu;
    }
  }
  return code;
}

// Four elements.  The NaN rule is tested for the quad as a whole (two unordered compares)
// and applied element-wise only on the rare lanes where it fires.
template <int KIND, int ROUND, bool AS_BF16>
__device__ __forceinline__ void quantize_quad(uint32_t (&c)[4], float x0, float x1, float x2, float x3,
                                              const InvScale& s, const uint32_t (&add)[4]) {
  c[0] = quantize_elem<KIND, ROUND, AS_BF16, false>(x0, s, add[0]);
  c[1] = quantize_elem<KIND, ROUND, AS_BF16, false>(x1, s, add[1]);
  c[2] = quantize_elem<KIND, ROUND, AS_BF16, false>(x2, s, add[2]);
  c[3] = quantize_elem<KIND, ROUND, AS_BF16, false>(x3, s, add[3]);
  if (__builtin_isunordered(x0, x1) || __builtin_isunordered(x2, x3)) {
    constexpr uint32_t NAN_CODE = !Grid<KIND>::is_float ? 0u : AS_BF16 ? 0x7FC0u : 0x7Fu;
    if (x0 != x0) c[0] = NAN_CODE;
    if (x1 != x1) c[1] = NAN_CODE;
    if (x2 != x2) c[2] = NAN_CODE;
    if (x3 != x3) c[3] = NAN_CODE;
  }
}

// low bytes of four codes -> one word (c0 in bits 7:0); upper bits of the inputs are ignored
__device__ __forceinline__ uint32_t pack4_bytes(const uint32_t (&c)[4]) {
  const uint32_t lo = __builtin_amdgcn_perm(c[1], c[0], 0x0c0c0400u);
  const uint32_t hi = __builtin_amdgcn_perm(c[3], c[2], 0x0c0c0400u);
  return __builtin_amdgcn_perm(hi, lo, 0x05040100u);
}
// low nibbles of four codes -> 16 bits (c0 in bits 3:0)
__device__ __forceinline__ uint32_t pack4_nibbles(const uint32_t (&c)[4]) {
  return (c[0] & 0xFu) | ((c[1] & 0xFu) << 4) | ((c[2] & 0xFu) << 8) | ((c[3] & 0xFu) << 12);
}

__device__ __forceinline__ float bf16_to_f32(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

// 1 / scale, correctly rounded, from a host value or a device-resident one.
// `kind` is the srq_kind of the tensor (it fills the run-time grid parameters of SRQ_E4MX).
__device__ __forceinline__ InvScale inv_scale(float scale, const float* scale_dev, int kind) {
  const float sc = scale_dev ? *scale_dev : scale;
  InvScale s;
  s.inv = __fdiv_rn(1.0f, sc);
  s.inv16 = __fmul_rn(s.inv, 65536.0f);
  s.sub_m = SRQ_E4M0 - kind;  // E4M2 -> 2, E4M1 -> 1, E4M0 -> 0
  s.sub_qmax = kind == SRQ_E4M2 ? 448.0f : kind == SRQ_E4M1 ? 384.0f : 256.0f;
  s.sub_qi = (kind == SRQ_INT4 ? 7 : 127) << 16;
  return s;
}

// First Philox block of a tensor: a host value, plus the value of a device-resident counter if
// one is given (so that a captured launch can be replayed with fresh thresholds).
__device__ __forceinline__ uint64_t first_block(uint64_t counter_offset, const uint64_t* counter_dev) {
  return counter_offset + (counter_dev ? *counter_dev : 0ull);
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

// Quantize one group; c[j] = code of element j (integer codes sign-extended: use the low byte).
template <int KIND, int ROUND, bool AS_BF16>
__device__ __forceinline__ void quantize_group(uint32_t (&c)[8], const float (&v)[8], const InvScale& s,
                                               uint64_t block, uint32_t k0, uint32_t k1) {
  uint32_t add[8];
  if constexpr (ROUND == SRQ_SR) {
    uint32_t w[4];
    philox_block(block, k0, k1, w);
    uint32_t lo[4], hi[4];
    sr_addends(w[0], w[1], lo);
    sr_addends(w[2], w[3], hi);
#pragma unroll
    for (int j = 0; j < 4; ++j) { add[j] = lo[j]; add[4 + j] = hi[j]; }
  } else {
#pragma unroll
    for (int j = 0; j < 8; ++j) add[j] = RTN_ADDEND;  // Def. 2
  }
  uint32_t lo4[4], hi4[4];
  const uint32_t addlo[4] = {add[0], add[1], add[2], add[3]}, addhi[4] = {add[4], add[5], add[6], add[7]};
  quantize_quad<KIND, ROUND, AS_BF16>(lo4, v[0], v[1], v[2], v[3], s, addlo);
  quantize_quad<KIND, ROUND, AS_BF16>(hi4, v[4], v[5], v[6], v[7], s, addhi);
#pragma unroll
  for (int j = 0; j < 4; ++j) { c[j] = lo4[j]; c[4 + j] = hi4[j]; }
}

// ---- one wave, 512 consecutive binary32 elements, fully coalesced ---------------------------
// Lane L loads elements 4L..4L+3 of the chunk and 256+4L..256+4L+3: two 16-byte loads, each a
// contiguous kilobyte across the wave.  A lane therefore holds one half of Philox group L/2 and
// one half of group 32 + L/2.  The even lane of a pair draws the block of the first group, the
// odd lane the block of the second, and they trade the two words the other needs through a
// quad permute: one Philox block per 8 elements, as in the layout-free definition.
constexpr int CHUNK = 512;

// store modes: 0 one byte per element, 1 nibbles, 2 bfloat16 (values as in StoreMode)
// Stores that write through the L2 (system-scope cache policy) without the streaming hint: the
// line does not stay dirty in the L2 (nothing left to flush when the kernel ends) but is still
// allocated in the last-level cache for the kernel that reads it next.
__device__ __forceinline__ void store_through16(void* p, const u32x4& v) {
  asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1" : : "v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void store_through8(void* p, const u32x2& v) {
  asm volatile("global_store_dwordx2 %0, %1, off sc0 sc1" : : "v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void store_through4(void* p, uint32_t v) {
  asm volatile("global_store_dword %0, %1, off sc0 sc1" : : "v"(p), "v"(v) : "memory");
}

template <int KIND, int ROUND, int STORE>
__device__ __forceinline__ void quantize_chunk_f32(uint8_t* __restrict__ out, const float* __restrict__ x,
                                                   size_t chunk, uint32_t lane, const InvScale& s, uint32_t k0,
                                                   uint32_t k1, uint64_t counter_offset) {
  constexpr bool AS_BF16 = STORE == 2;
  const size_t e0 = chunk * CHUNK + 4 * lane;  // first element of this lane's first quad
  const f32x4 a = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(x + e0));
  const f32x4 b = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(x + e0 + 256));
  uint32_t addA[4], addB[4];
  if constexpr (ROUND == SRQ_SR) {
    const bool odd = lane & 1u;
    uint32_t w[4];
    philox_block(counter_offset + chunk * (CHUNK / 8) + (odd ? 32u : 0u) + (lane >> 1), k0, k1, w);
    // Even lane: its first quad is the first half of its own block (words 0,1), its second quad
    // the first half of the odd neighbour's block.  Odd lane: first quad = second half (words
    // 2,3) of the even neighbour's block, second quad = second half of its own.
    const uint32_t nb0 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w[0], 0xB1, 0xF, 0xF, true);  // lane ^ 1
    const uint32_t nb1 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w[1], 0xB1, 0xF, 0xF, true);
    const uint32_t nb2 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w[2], 0xB1, 0xF, 0xF, true);
    const uint32_t nb3 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w[3], 0xB1, 0xF, 0xF, true);
    sr_addends(odd ? nb2 : w[0], odd ? nb3 : w[1], addA);
    sr_addends(odd ? w[2] : nb0, odd ? w[3] : nb1, addB);
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j) addA[j] = addB[j] = RTN_ADDEND;  // Def. 2
  }
  uint32_t ca[4], cb[4];
  quantize_quad<KIND, ROUND, AS_BF16>(ca, a.x, a.y, a.z, a.w, s, addA);
  quantize_quad<KIND, ROUND, AS_BF16>(cb, b.x, b.y, b.z, b.w, s, addB);
  if constexpr (STORE == 1) {
    uint16_t* o = reinterpret_cast<uint16_t*>(out + e0 / 2);
    o[0] = (uint16_t)pack4_nibbles(ca);
    o[64] = (uint16_t)pack4_nibbles(cb);
  } else if constexpr (STORE == 2) {
    u32x2* o = reinterpret_cast<u32x2*>(reinterpret_cast<uint16_t*>(out) + e0);
    const u32x2 va = {ca[0] | (ca[1] << 16), ca[2] | (ca[3] << 16)}, vb = {cb[0] | (cb[1] << 16), cb[2] | (cb[3] << 16)};
    __builtin_nontemporal_store(va, o);
    __builtin_nontemporal_store(vb, o + 64);
  } else {
    uint32_t* o = reinterpret_cast<uint32_t*>(out + e0);
    __builtin_nontemporal_store(pack4_bytes(ca), o);
    __builtin_nontemporal_store(pack4_bytes(cb), o + 64);
  }
}

}  // namespace srq
