// Weight update of Eq. 10 with the weights kept in bfloat16:  w <- Q_SR(w - eta * g), Q on the
// bfloat16 grid (8 exponent bits, 7 fraction bits).  gfx950 only.
//
// Arithmetic.  u = fl32(w - fl32(eta * g)): two binary32 roundings, no fused multiply-add.
// binary32 has exactly 16 fraction bits beyond bfloat16, and the threshold of Eq. 1 is
// eps = (r + 1/2) / 2^16 with r the element's 16 random bits, so on the sign-magnitude bit
// pattern of u (L = its low 16 bits):
//     u > 0: round up (away from zero)  <=>  L / 2^16 >= eps      <=>  L + (65535 - r) >= 2^16
//     u < 0: round down (away from zero) <=> 1 - L / 2^16 < eps   <=>  L + r >= 2^16
// i.e. one integer add and a shift; the carry walks into the exponent when the rounding
// crosses a binade, and subnormals need no special case.  |u| is clamped to the largest finite
// bfloat16 first, NaN gives 0x7FC0, a zero result is +0.  Round-to-nearest (eps = 1/2, ties
// toward +inf) adds 0x8000 for u > 0 and 0x7FFF for u < 0.
// Memory-bound: 2 + 4 bytes read and 2 written per element.
#include "srq_device.hpp"
#include "srq_internal.hpp"

namespace srq {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int UBLOCK = 256;

// addend: 65535 - r (stochastic rounding) or 0x8000 (nearest), as the quantizers use it
template <int ROUND>
__device__ __forceinline__ uint32_t update_elem(uint32_t w_bits, float g, float eta, uint32_t addend) {
  const float u = __fsub_rn(__uint_as_float(w_bits << 16), __fmul_rn(eta, g));
  const uint32_t bits = __float_as_uint(u);
  const uint32_t sign = bits & 0x80000000u;
  uint32_t mag = bits & 0x7FFFFFFFu;
  if (mag > 0x7F800000u) return 0x7FC0u;       // NaN
  mag = min(mag, 0x7F7F0000u);                 // saturate (covers +-Inf)
  uint32_t add;
  if (ROUND == SRQ_SR) add = sign ? 65535u - addend : addend;
  else add = sign ? 0x7FFFu : 0x8000u;
  const uint32_t r = (mag + add) >> 16;
  return r ? (r | (sign >> 16)) : 0u;
}

template <int ROUND>
__device__ __forceinline__ uint32_t update_pair(uint32_t w2, float g0, float g1, float eta, uint32_t a0, uint32_t a1) {
  return update_elem<ROUND>(w2 & 0xFFFFu, g0, eta, a0) | (update_elem<ROUND>(w2 >> 16, g1, eta, a1) << 16);
}

// Whole chunks of 512 elements, one per wave and iteration: lane L holds elements 4L..4L+3 and
// 256+4L..256+4L+3 of the chunk (coalesced 16-byte gradient loads, 8-byte weight accesses); a
// pair of lanes shares two Philox blocks, each lane draws one and they trade two words.
template <int ROUND>
__global__ __launch_bounds__(UBLOCK) void update_bf16_kernel(uint16_t* __restrict__ w, const float* __restrict__ g,
                                                             float eta, size_t n, uint32_t k0, uint32_t k1,
                                                             uint64_t counter_offset) {
  const size_t nchunks = n / CHUNK, waves = (size_t)gridDim.x * (UBLOCK / 64);
  const uint32_t lane = threadIdx.x & 63u;
  const bool odd = lane & 1u;
  for (size_t c = (size_t)blockIdx.x * (UBLOCK / 64) + (threadIdx.x >> 6); c < nchunks; c += waves) {
    const size_t e0 = c * CHUNK + 4 * lane;
    const f32x4 ga = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(g + e0));
    const f32x4 gb = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(g + e0 + 256));
    u32x2* wa = reinterpret_cast<u32x2*>(w + e0);
    u32x2* wb = reinterpret_cast<u32x2*>(w + e0 + 256);
    const u32x2 va = *wa, vb = *wb;
    uint32_t addA[4], addB[4];
    if (ROUND == SRQ_SR) {
      uint32_t x[4];
      philox_block(counter_offset + c * (CHUNK / 8) + (odd ? 32u : 0u) + (lane >> 1), k0, k1, x);
      const uint32_t nb0 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x[0], 0xB1, 0xF, 0xF, true);  // lane ^ 1
      const uint32_t nb1 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x[1], 0xB1, 0xF, 0xF, true);
      const uint32_t nb2 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x[2], 0xB1, 0xF, 0xF, true);
      const uint32_t nb3 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x[3], 0xB1, 0xF, 0xF, true);
      sr_addends(odd ? nb2 : x[0], odd ? nb3 : x[1], addA);
      sr_addends(odd ? x[2] : nb0, odd ? x[3] : nb1, addB);
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) addA[j] = addB[j] = RTN_ADDEND;
    }
    *wa = u32x2{update_pair<ROUND>(va.x, ga.x, ga.y, eta, addA[0], addA[1]),
                update_pair<ROUND>(va.y, ga.z, ga.w, eta, addA[2], addA[3])};
    *wb = u32x2{update_pair<ROUND>(vb.x, gb.x, gb.y, eta, addB[0], addB[1]),
                update_pair<ROUND>(vb.y, gb.z, gb.w, eta, addB[2], addB[3])};
  }
}

// The elements after the last whole chunk: one thread per group of 8 (one Philox block).
template <int ROUND>
__global__ __launch_bounds__(UBLOCK) void update_bf16_tail_kernel(uint16_t* __restrict__ w, const float* __restrict__ g,
                                                                  float eta, size_t first, size_t n, uint32_t k0,
                                                                  uint32_t k1, uint64_t counter_offset) {
  const size_t grp = first / 8 + (size_t)blockIdx.x * UBLOCK + threadIdx.x;
  if (grp * 8 >= n) return;
  uint32_t add[8];
  if (ROUND == SRQ_SR) {
    uint32_t x[4];
    philox_block(counter_offset + grp, k0, k1, x);
    uint32_t lo[4], hi[4];
    sr_addends(x[0], x[1], lo);
    sr_addends(x[2], x[3], hi);
#pragma unroll
    for (int j = 0; j < 4; ++j) { add[j] = lo[j]; add[4 + j] = hi[j]; }
  } else {
#pragma unroll
    for (int j = 0; j < 8; ++j) add[j] = RTN_ADDEND;
  }
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const size_t i = grp * 8 + j;
    if (i < n) w[i] = (uint16_t)update_elem<ROUND>(w[i], g[i], eta, add[j]);
  }
}

}  // namespace

hipError_t launch_update_bf16(uint16_t* w, const float* g, float eta, size_t n, int round, uint64_t seed,
                              uint64_t counter_offset, hipStream_t stream) {
  if (n == 0) return hipSuccess;
  const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
  const size_t nchunks = n / CHUNK, done = nchunks * CHUNK;
  if (nchunks) {
    size_t blocks = (nchunks + UBLOCK / 64 - 1) / (UBLOCK / 64);
    if (blocks > (1u << 20)) blocks = 1u << 20;
    if (round == SRQ_SR) update_bf16_kernel<SRQ_SR><<<(unsigned)blocks, UBLOCK, 0, stream>>>(w, g, eta, n, k0, k1, counter_offset);
    else update_bf16_kernel<SRQ_RTN><<<(unsigned)blocks, UBLOCK, 0, stream>>>(w, g, eta, n, k0, k1, counter_offset);
  }
  if (done < n) {
    const size_t groups = (n - done + 7) / 8;
    const unsigned blocks = (unsigned)((groups + UBLOCK - 1) / UBLOCK);
    if (round == SRQ_SR) update_bf16_tail_kernel<SRQ_SR><<<blocks, UBLOCK, 0, stream>>>(w, g, eta, done, n, k0, k1, counter_offset);
    else update_bf16_tail_kernel<SRQ_RTN><<<blocks, UBLOCK, 0, stream>>>(w, g, eta, done, n, k0, k1, counter_offset);
  }
  return hipGetLastError();
}

}  // namespace srq
