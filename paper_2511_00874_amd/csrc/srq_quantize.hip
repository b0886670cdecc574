// Tensor-level SR quantizer kernels (Def. 3: element-wise, independent thresholds) and the
// per-tensor absmax scale.  HBM-bound streaming kernels for gfx950: 128-bit loads, one
// Philox block per 8 consecutive elements, 64-bit (or 32-bit for nibbles) stores.
#include <type_traits>

#include "srq_device.hpp"
#include "srq_internal.hpp"

namespace srq {
namespace {

constexpr int QBLOCK = 256;

__device__ __forceinline__ uint32_t pack_bytes(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
  const uint32_t q[4] = {a, b, c, d};
  return pack4_bytes(q);
}
__device__ __forceinline__ uint32_t pack_nibbles(const uint32_t (&c)[8]) {
  uint32_t r = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) r |= (c[j] & 0xFu) << (4 * j);
  return r;
}

// ---- same-layout output -------------------------------------------------------------------
template <int KIND, int SRC, int ROUND, int STORE>
__global__ __launch_bounds__(QBLOCK) void quantize_flat_kernel(uint8_t* __restrict__ out,
                                                               const void* __restrict__ x, size_t n,
                                                               float scale, const float* scale_dev, int kind,
                                                               uint64_t seed, uint64_t counter_host,
                                                               const uint64_t* counter_dev) {
  const InvScale inv = inv_scale(scale, scale_dev, kind);
  const uint64_t counter_offset = first_block(counter_host, counter_dev);
  const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
  const size_t ngroups = (n + 7) / 8;
  const size_t stride = (size_t)gridDim.x * QBLOCK;
  for (size_t g = (size_t)blockIdx.x * QBLOCK + threadIdx.x; g < ngroups; g += stride) {
    float v[8];
    uint32_t c[8];
    load_group<SRC>(v, x, g, n);
    quantize_group<KIND, ROUND, STORE == STORE_BF16>(c, v, inv, counter_offset + g, k0, k1);
    const size_t base = g * 8;
    if constexpr (STORE == STORE_NIBBLE) {
      const uint32_t word = pack_nibbles(c);
      if (base + 8 <= n) {
        __builtin_nontemporal_store(word, reinterpret_cast<uint32_t*>(out + base / 2));
      } else {
        for (size_t j = 0; base + 2 * j < n; ++j) out[base / 2 + j] = (uint8_t)(word >> (8 * j));
      }
    } else if constexpr (STORE == STORE_BF16) {
      uint16_t* o16 = reinterpret_cast<uint16_t*>(out);
      if (base + 8 <= n) {
        u32x4 word = {c[0] | (c[1] << 16), c[2] | (c[3] << 16), c[4] | (c[5] << 16), c[6] | (c[7] << 16)};
        __builtin_nontemporal_store(word, reinterpret_cast<u32x4*>(o16 + base));
      } else {
#pragma unroll
        for (int j = 0; j < 8; ++j)
          if (base + j < n) o16[base + j] = (uint16_t)c[j];
      }
    } else {
      if (base + 8 <= n) {
        u32x2 word = {pack_bytes(c[0], c[1], c[2], c[3]), pack_bytes(c[4], c[5], c[6], c[7])};
        __builtin_nontemporal_store(word, reinterpret_cast<u32x2*>(out + base));
      } else {
#pragma unroll
        for (int j = 0; j < 8; ++j)
          if (base + j < n) out[base + j] = (uint8_t)c[j];
      }
    }
  }
}

// binary32 source, whole 512-element chunks: one chunk per wave, fully coalesced (see
// quantize_chunk_f32); the ragged remainder goes to quantize_flat_kernel
template <int KIND, int ROUND, int STORE>
__global__ __launch_bounds__(QBLOCK) void quantize_flat_f32_kernel(uint8_t* __restrict__ out,
                                                                   const float* __restrict__ x, size_t nchunks,
                                                                   float scale, const float* scale_dev, int kind,
                                                                   uint64_t seed, uint64_t counter_host,
                                                                   const uint64_t* counter_dev) {
  const InvScale inv = inv_scale(scale, scale_dev, kind);
  const uint64_t counter_offset = first_block(counter_host, counter_dev);
  const uint32_t lane = threadIdx.x & 63u;
  const size_t waves = (size_t)gridDim.x * (QBLOCK / 64);
  for (size_t c = (size_t)blockIdx.x * (QBLOCK / 64) + (threadIdx.x >> 6); c < nchunks; c += waves)
    quantize_chunk_f32<KIND, ROUND, STORE>(out, x, c, lane, inv, (uint32_t)seed, (uint32_t)(seed >> 32),
                                           counter_offset);
}

// ---- transposed output --------------------------------------------------------------------
// A block quantizes a TR x TC tile (thresholds keyed by the row-major SOURCE index, so the
// codes equal those of the same-layout kernel), turns it through LDS, and writes it as
// TC rows of TR contiguous codes.
constexpr int TR = 128, TC = 64;

template <int KIND, int SRC, int ROUND, int STORE>
__global__ __launch_bounds__(QBLOCK) void quantize_transpose_kernel(
    uint8_t* __restrict__ out, const void* __restrict__ x, uint32_t rows, uint32_t cols, float scale,
    const float* scale_dev, int kind, uint64_t seed, uint64_t counter_host, const uint64_t* counter_dev) {
  const uint64_t counter_offset = first_block(counter_host, counter_dev);
  // one tile element per code: a byte, or 16 bits when the grid values are stored as bfloat16
  using elem_t = typename std::conditional<STORE == STORE_BF16, uint16_t, uint8_t>::type;
  constexpr int ES = sizeof(elem_t);
  constexpr int PITCH = TR + 4 / ES;            // elements; keeps rows 4-byte aligned
  __shared__ __attribute__((aligned(16))) elem_t tile[TC * PITCH];
  const InvScale inv = inv_scale(scale, scale_dev, kind);
  const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
  const uint32_t r0 = blockIdx.y * TR, c0 = blockIdx.x * TC;
  const size_t n = (size_t)rows * cols;
#pragma unroll
  for (int it = 0; it < (TR * TC / 8) / QBLOCK; ++it) {
    const uint32_t id = it * QBLOCK + threadIdx.x;
    const uint32_t gc = id % (TC / 8), r = id / (TC / 8);
    const uint32_t row = r0 + r, col = c0 + gc * 8;
    uint32_t c[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (row < rows && col < cols) {  // cols % 8 == 0: a group never straddles the edge
      const size_t g = ((size_t)row * cols + col) / 8;
      float v[8];
      load_group<SRC>(v, x, g, n);
      quantize_group<KIND, ROUND, STORE == STORE_BF16>(c, v, inv, counter_offset + g, k0, k1);
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) tile[(gc * 8 + j) * PITCH + r] = (elem_t)c[j];
  }
  __syncthreads();
  // TC columns x (TR / 16) chunks of 16 source rows
#pragma unroll
  for (int it = 0; it < (TC * TR / 16) / QBLOCK; ++it) {
    const uint32_t id = it * QBLOCK + threadIdx.x;
    const uint32_t ch = id % (TR / 16), c = id / (TR / 16);
    const uint32_t col = c0 + c, row = r0 + ch * 16;
    if (col >= cols || row >= rows) continue;
    const uint32_t* src = reinterpret_cast<const uint32_t*>(&tile[c * PITCH + ch * 16]);
    uint32_t w[4 * ES];
#pragma unroll
    for (int i = 0; i < 4 * ES; ++i) w[i] = src[i];
    const bool whole = row + 16 <= rows && (rows % 16) == 0;  // 16 rows, aligned destination
    if constexpr (STORE == STORE_NIBBLE) {
      // pairs along the output's contiguous dimension (source rows); rows is even
      auto squeeze = [](uint32_t v) {  // 4 code bytes -> 4 nibbles (16 bits)
        return (v & 0xFu) | ((v >> 4) & 0xF0u) | ((v >> 8) & 0xF00u) | ((v >> 12) & 0xF000u);
      };
      const uint32_t lo = squeeze(w[0]) | (squeeze(w[1]) << 16), hi = squeeze(w[2]) | (squeeze(w[3]) << 16);
      uint8_t* dst = out + ((size_t)col * rows + row) / 2;
      if (whole) {
        *reinterpret_cast<u32x2*>(dst) = u32x2{lo, hi};
      } else {
        const uint64_t both = (uint64_t)lo | ((uint64_t)hi << 32);
        for (uint32_t j = 0; row + 2 * j < rows && j < 8; ++j) dst[j] = (uint8_t)(both >> (8 * j));
      }
    } else {
      elem_t* dst = reinterpret_cast<elem_t*>(out) + (size_t)col * rows + row;
      if (whole) {
#pragma unroll
        for (int i = 0; i < ES; ++i)
          reinterpret_cast<u32x4*>(dst)[i] = u32x4{w[4 * i], w[4 * i + 1], w[4 * i + 2], w[4 * i + 3]};
      } else {
        constexpr int PER = 4 / ES;  // elements per 32-bit word
        for (uint32_t j = 0; j < 16 && row + j < rows; ++j)
          dst[j] = (elem_t)(w[j / PER] >> (8 * ES * (j % PER)));
      }
    }
  }
}

// ---- absmax ---------------------------------------------------------------------------------
// max over the wave of non-negative bit patterns: DPP butterflies inside each row of 16
// lanes, then the four rows through scalar reads.
__device__ __forceinline__ uint32_t wave_umax(uint32_t v) {
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xF, 0xF, true));  // row_half_mirror
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xF, 0xF, true));  // row_mirror
  const uint32_t a = __builtin_amdgcn_readlane((int)v, 0), b = __builtin_amdgcn_readlane((int)v, 16);
  const uint32_t c = __builtin_amdgcn_readlane((int)v, 32), d = __builtin_amdgcn_readlane((int)v, 48);
  return max(max(a, b), max(c, d));
}

// |x| as bits, with Inf and NaN ignored (they do not take part in the scale).
__device__ __forceinline__ uint32_t abs_bits_finite(float f) {
  const uint32_t a = __float_as_uint(f) & 0x7FFFFFFFu;
  return a < 0x7F800000u ? a : 0u;
}

// max of the finite |x_i| bit patterns over the 16-byte pieces [g0, g1) of x (4 binary32 or 8
// bfloat16 elements each; the last piece of the tensor may be partial): thread t of nt, eight loads in
// flight per lane, the pieces of a workgroup contiguous in memory
template <int SRC>
__device__ __forceinline__ uint32_t absmax_pieces(const void* __restrict__ x, size_t n, size_t g0, size_t g1, uint32_t t,
                                                  uint32_t nt) {
  constexpr int PER = SRC == SRQ_F32 ? 4 : 8;
  uint32_t m = 0u;
  const size_t full = n / PER;  // pieces that lie wholly inside the tensor
  const size_t gf = g1 < full ? g1 : full;
  const u32x4* p = static_cast<const u32x4*>(x);
  auto fold = [&](const u32x4& a) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if constexpr (SRC == SRQ_F32) {
        m = max(m, abs_bits_finite(__uint_as_float(a[j])));
      } else {
        m = max(m, max(abs_bits_finite(bf16_to_f32(a[j] & 0xFFFFu)), abs_bits_finite(bf16_to_f32(a[j] >> 16))));
      }
    }
  };
  size_t i = g0 + t;
  for (; i + 7 * (size_t)nt < gf; i += 8 * (size_t)nt) {
    u32x4 a[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) a[j] = __builtin_nontemporal_load(p + i + j * (size_t)nt);
#pragma unroll
    for (int j = 0; j < 8; ++j) fold(a[j]);
  }
  for (; i + 3 * (size_t)nt < gf; i += 4 * (size_t)nt) {
    const u32x4 a = __builtin_nontemporal_load(p + i), b = __builtin_nontemporal_load(p + i + nt);
    const u32x4 c = __builtin_nontemporal_load(p + i + 2 * (size_t)nt), d = __builtin_nontemporal_load(p + i + 3 * (size_t)nt);
    fold(a); fold(b); fold(c); fold(d);
  }
  for (; i < gf; i += nt) fold(__builtin_nontemporal_load(p + i));
  if (g1 > full && t < n - full * PER) {  // the partial last piece, element by element
    const size_t e = full * PER + t;
    m = max(m, abs_bits_finite(SRC == SRQ_F32 ? static_cast<const float*>(x)[e]
                                              : bf16_to_f32(static_cast<const uint16_t*>(x)[e])));
  }
  return m;
}

// The smallest step the quantizer takes (2^16 / step must stay finite in binary32): the absmax
// scale of a tensor of vanishing values is floored here instead of saturating every element.
constexpr float MIN_SCALE = 0x1p-100f;

__global__ void absmax_init_kernel(uint32_t* acc) { *acc = 0u; }

template <int SRC>
__global__ __launch_bounds__(QBLOCK) void absmax_kernel(uint32_t* __restrict__ acc,
                                                        const void* __restrict__ x, size_t n) {
  // every workgroup one contiguous share of the tensor
  constexpr size_t PER = SRC == SRQ_F32 ? 4 : 8;
  const size_t pieces = (n + PER - 1) / PER, share = (pieces + gridDim.x - 1) / gridDim.x;
  const size_t g0 = (size_t)blockIdx.x * share, g1 = g0 + share < pieces ? g0 + share : pieces;
  uint32_t m = g0 < pieces ? absmax_pieces<SRC>(x, n, g0, g1, threadIdx.x, QBLOCK) : 0u;
  m = wave_umax(m);
  __shared__ uint32_t part[QBLOCK / 64];
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t b = part[0];
#pragma unroll
    for (int i = 1; i < QBLOCK / 64; ++i) b = max(b, part[i]);
    if (b != 0u) atomicMax(acc, b);  // bit patterns of non-negative floats order like the floats
  }
}

__global__ void absmax_finish_kernel(float* scale, float qmax) {
  const float amax = *scale;  // the accumulator holds the bits of max|x|
  *scale = amax == 0.0f ? 1.0f : fmaxf(__fdiv_rn(amax, qmax), MIN_SCALE);
}

// ---- several tensors, several scales, two launches -----------------------------------------
// Launch 1: every block reduces one contiguous slice of one tensor and writes its partial maximum
// to the workspace (plain stores: nothing to initialise).  Launch 2: one block per tensor folds
// that tensor's partials and writes the scales requested of it (several formats may share one
// tensor).
__global__ __launch_bounds__(QBLOCK) void absmax_multi_kernel(AbsmaxBatch b) {
  int t = 0;
#pragma unroll
  for (int i = 1; i < ABSMAX_MAX; ++i)
    if (i < b.ntensors && blockIdx.x >= b.first_block[i]) t = i;
  const uint32_t local = blockIdx.x - b.first_block[t], nblk = b.nblocks[t];
  const size_t n = b.n[t];
  const void* x = b.x[t];
  const size_t per = b.dtype[t] == SRQ_F32 ? 4 : 8;
  const size_t pieces = (n + per - 1) / per, share = (pieces + nblk - 1) / nblk;
  const size_t g0 = (size_t)local * share, g1 = g0 + share < pieces ? g0 + share : pieces;
  uint32_t m = 0u;
  if (g0 < pieces)
    m = b.dtype[t] == SRQ_F32 ? absmax_pieces<SRQ_F32>(x, n, g0, g1, threadIdx.x, QBLOCK)
                              : absmax_pieces<SRQ_BF16>(x, n, g0, g1, threadIdx.x, QBLOCK);
  m = wave_umax(m);
  __shared__ uint32_t part[QBLOCK / 64];
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t r = part[0];
#pragma unroll
    for (int i = 1; i < QBLOCK / 64; ++i) r = max(r, part[i]);
    b.partial[blockIdx.x] = r;
  }
}

// 256 threads (one wave per SIMD, 20 registers): small enough to start on a CU that a product kernel
// occupies, when the scales are computed on a second stream beside the products of another layer (a
// workgroup of 1024 threads waited there for a product launch to end, 200-700 us)
constexpr int FINISH_BLOCK = 256;
__global__ __launch_bounds__(FINISH_BLOCK) void absmax_multi_finish_kernel(AbsmaxBatch b) {
  __shared__ uint32_t part[FINISH_BLOCK / 64];
  const int t = blockIdx.x;  // one block per tensor
  const uint32_t* p = b.partial + b.first_block[t];
  const uint32_t nb = b.nblocks[t];
  uint32_t m = 0u;
  uint32_t i = threadIdx.x;
  for (; i + 3 * FINISH_BLOCK < nb; i += 4 * FINISH_BLOCK)
    m = max(max(m, max(p[i], p[i + FINISH_BLOCK])), max(p[i + 2 * FINISH_BLOCK], p[i + 3 * FINISH_BLOCK]));
  for (; i < nb; i += FINISH_BLOCK) m = max(m, p[i]);
  m = wave_umax(m);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = m;
  __syncthreads();
  if ((int)threadIdx.x < b.nouts && b.out_tensor[threadIdx.x] == t) {
    uint32_t r = part[0];
    for (int w = 1; w < FINISH_BLOCK / 64; ++w) r = max(r, part[w]);
    const float amax = __uint_as_float(r);
    *b.out[threadIdx.x] = amax == 0.0f ? 1.0f : fmaxf(__fdiv_rn(amax, b.out_qmax[threadIdx.x]), MIN_SCALE);
  }
}

int grid_for(size_t work_items, int per_block, int cap) {
  size_t blocks = (work_items + per_block - 1) / per_block;
  if (blocks < 1) blocks = 1;
  if (blocks > (size_t)cap) blocks = cap;
  return (int)blocks;
}

float qmax_of(int kind) {
  switch (kind) {
    case SRQ_INT8: return 127.0f;
    case SRQ_INT4: return 7.0f;
    case SRQ_E4M3: case SRQ_E4M2: return 448.0f;
    case SRQ_E4M1: return 384.0f;
    case SRQ_E4M0: return 256.0f;
    default: return 57344.0f;
  }
}

template <int KIND, int SRC, int ROUND, int STORE>
hipError_t launch_one(void* codes, const void* x, size_t rows, size_t cols, int transpose_out,
                      const QuantArgs& a, hipStream_t stream) {
  if (transpose_out) {
    dim3 grid((unsigned)((cols + TC - 1) / TC), (unsigned)((rows + TR - 1) / TR));
    quantize_transpose_kernel<KIND, SRC, ROUND, STORE><<<grid, QBLOCK, 0, stream>>>(
        static_cast<uint8_t*>(codes), x, (uint32_t)rows, (uint32_t)cols, a.scale, a.scale_dev, a.kind, a.seed,
        a.counter_offset, a.counter_dev);
  } else {
    const size_t n = rows * cols;
    size_t done = 0;  // elements handled by the coalesced chunk kernel
    if constexpr (SRC == SRQ_F32) {
      const size_t nchunks = n / CHUNK;
      if (nchunks > 0) {
        const int grid = grid_for(nchunks, QBLOCK / 64, 1 << 22);
        quantize_flat_f32_kernel<KIND, ROUND, STORE><<<grid, QBLOCK, 0, stream>>>(
            static_cast<uint8_t*>(codes), static_cast<const float*>(x), nchunks, a.scale, a.scale_dev, a.kind, a.seed,
            a.counter_offset, a.counter_dev);
        done = nchunks * CHUNK;
      }
    }
    if (done < n) {
      // remainder (or a bfloat16 source, whose groups are one 16-byte load each already)
      const size_t es = SRC == SRQ_F32 ? 4 : 2;
      const size_t out_bytes = STORE == STORE_NIBBLE ? done / 2 : STORE == STORE_BF16 ? done * 2 : done;
      const int grid = grid_for((n - done + 7) / 8, QBLOCK * 4, 1 << 20);
      quantize_flat_kernel<KIND, SRC, ROUND, STORE><<<grid, QBLOCK, 0, stream>>>(
          static_cast<uint8_t*>(codes) + out_bytes, static_cast<const uint8_t*>(x) + done * es, n - done, a.scale,
          a.scale_dev, a.kind, a.seed, a.counter_offset + done / 8, a.counter_dev);
    }
  }
  return hipGetLastError();
}

template <int KIND, int STORE>
hipError_t dispatch_src_round(void* codes, const void* x, size_t rows, size_t cols, int tr,
                              const QuantArgs& a, hipStream_t s) {
  if (a.dtype == SRQ_F32) {
    return a.round == SRQ_SR ? launch_one<KIND, SRQ_F32, SRQ_SR, STORE>(codes, x, rows, cols, tr, a, s)
                             : launch_one<KIND, SRQ_F32, SRQ_RTN, STORE>(codes, x, rows, cols, tr, a, s);
  }
  return a.round == SRQ_SR ? launch_one<KIND, SRQ_BF16, SRQ_SR, STORE>(codes, x, rows, cols, tr, a, s)
                           : launch_one<KIND, SRQ_BF16, SRQ_RTN, STORE>(codes, x, rows, cols, tr, a, s);
}

}  // namespace

hipError_t launch_quantize(void* codes, const void* x, size_t rows, size_t cols, int transpose_out,
                           const QuantArgs& a, hipStream_t stream) {
  if (rows * cols == 0) return hipSuccess;
  switch (a.kind) {
    case SRQ_INT8: return dispatch_src_round<SRQ_INT8, STORE_BYTE>(codes, x, rows, cols, transpose_out, a, stream);
    case SRQ_INT4:
      return a.store == STORE_NIBBLE
                 ? dispatch_src_round<SRQ_INT4, STORE_NIBBLE>(codes, x, rows, cols, transpose_out, a, stream)
                 : dispatch_src_round<SRQ_INT4, STORE_BYTE>(codes, x, rows, cols, transpose_out, a, stream);
    case SRQ_E4M3:
      return a.store == STORE_BF16
                 ? dispatch_src_round<SRQ_E4M3, STORE_BF16>(codes, x, rows, cols, transpose_out, a, stream)
                 : dispatch_src_round<SRQ_E4M3, STORE_BYTE>(codes, x, rows, cols, transpose_out, a, stream);
    case SRQ_E5M2:
      return a.store == STORE_BF16
                 ? dispatch_src_round<SRQ_E5M2, STORE_BF16>(codes, x, rows, cols, transpose_out, a, stream)
                 : dispatch_src_round<SRQ_E5M2, STORE_BYTE>(codes, x, rows, cols, transpose_out, a, stream);
    case SRQ_E4M2: case SRQ_E4M1: case SRQ_E4M0:
      return a.store == STORE_BF16
                 ? dispatch_src_round<SRQ_E4MX, STORE_BF16>(codes, x, rows, cols, transpose_out, a, stream)
                 : dispatch_src_round<SRQ_E4MX, STORE_BYTE>(codes, x, rows, cols, transpose_out, a, stream);
    default: return hipErrorInvalidValue;
  }
}

size_t absmax_batch_plan(AbsmaxBatch& b) {
  // sixteen 16-byte loads per lane (64 KiB per workgroup: measured best between 16 and 128 KiB),
  // at most 32768 workgroups in all; at least one per tensor
  size_t total_groups = 0;
  for (int t = 0; t < b.ntensors; ++t) total_groups += (b.n[t] + 7) / 8;
  uint32_t first = 0;
  for (int t = 0; t < b.ntensors; ++t) {
    const size_t groups = (b.n[t] + 7) / 8;
    size_t nb = (groups + QBLOCK * 8 - 1) / (QBLOCK * 8);
    const size_t share = total_groups ? (32768 * groups + total_groups - 1) / total_groups : 1;
    if (nb > share) nb = share;
    if (nb < 1) nb = 1;
    b.first_block[t] = first;
    b.nblocks[t] = (uint32_t)nb;
    first += (uint32_t)nb;
  }
  return first;
}

hipError_t launch_absmax_batch(AbsmaxBatch& b, hipStream_t stream) {
  const size_t blocks = absmax_batch_plan(b);
  for (int i = 0; i < b.nouts; ++i) b.out_qmax[i] = qmax_of(b.out_kind[i]);
  absmax_multi_kernel<<<(unsigned)blocks, QBLOCK, 0, stream>>>(b);
  absmax_multi_finish_kernel<<<b.ntensors, FINISH_BLOCK, 0, stream>>>(b);
  return hipGetLastError();
}

hipError_t launch_absmax_scale(float* scale_out_dev, const void* x, int dtype, size_t n, int kind,
                               hipStream_t stream) {
  uint32_t* acc = reinterpret_cast<uint32_t*>(scale_out_dev);
  absmax_init_kernel<<<1, 1, 0, stream>>>(acc);
  if (n > 0) {
    const int grid = grid_for((n + 7) / 8, QBLOCK * 4, 2048);  // one atomic per workgroup: keep them few
    if (dtype == SRQ_F32) absmax_kernel<SRQ_F32><<<grid, QBLOCK, 0, stream>>>(acc, x, n);
    else absmax_kernel<SRQ_BF16><<<grid, QBLOCK, 0, stream>>>(acc, x, n);
  }
  absmax_finish_kernel<<<1, 1, 0, stream>>>(scale_out_dev, qmax_of(kind));
  return hipGetLastError();
}

}  // namespace srq
