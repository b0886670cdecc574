// Product of two code matrices on the gfx950 matrix cores (Sec. 2.2.2: low-precision
// multiplies, high-precision accumulation == exact product of the quantized matrices).
//
//   out[p][q] = s * sum_r val(X[p][r]) * val(Z[q][r])        X: P x R, Z: Q x R, R contiguous
//
// All three products of Alg. 1 / Alg. 2 have this form once the quantizer has written the
// codes with the contraction index contiguous.  Integer codes use v_mfma_i32_32x32x32_i8
// (int32 accumulators, exact), 8-bit float codes use v_mfma_f32_32x32x64_f8f6f4 with the
// per-operand format select (binary32 accumulators).
//
// Tiling: a workgroup of 4 waves owns a BM x BN output tile; each wave owns a
// (BM/2) x (BN/2) sub-tile built from 32x32 MFMA tiles.  The contraction runs in steps of
// BK = 128 bytes: global -> registers (prefetched one step ahead) -> LDS (two buffers, rows of
// 128 bytes with the 16-byte chunks XOR-swizzled by row so that the MFMA operand reads are
// bank-conflict free) -> MFMA.
#include "srq_internal.hpp"

namespace srq {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

constexpr int BK = 128;       // bytes of contraction per LDS stage
constexpr int NTHREADS = 256; // 4 waves, 2 x 2

struct I8Mma {
  using acc_t = v16i;
  using frag_t = v4i;
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
  using frag_t = v4i;  // 8 bfloat16
  static constexpr int KSTEP = 32;  // bytes: 16 elements per MFMA
  static __device__ __forceinline__ acc_t mma(frag_t a, frag_t b, acc_t c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, b), c,
                                                   0, 0, 0);
  }
  static __device__ __forceinline__ float to_f32(float v) { return v; }
  static __device__ __forceinline__ float from_bits(uint32_t b) { return __uint_as_float(b); }
  static __device__ __forceinline__ uint32_t bits(float v) { return __float_as_uint(v); }
};

// FX / FZ: 0 = E4M3, 1 = E5M2 (the instruction's format selects)
template <int FX, int FZ>
struct F8Mma {
  using acc_t = v16f;
  using frag_t = v8i;
  static constexpr int KSTEP = 64;
  static __device__ __forceinline__ acc_t mma(frag_t a, frag_t b, acc_t c) {
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, FX, FZ, 0, 0, 0, 0);
  }
  static __device__ __forceinline__ float to_f32(float v) { return v; }
  static __device__ __forceinline__ float from_bits(uint32_t b) { return __uint_as_float(b); }
  static __device__ __forceinline__ uint32_t bits(float v) { return __float_as_uint(v); }
};

// byte offset of 16-byte chunk `chunk` (0..7) of tile row `row` in an LDS stage
__device__ __forceinline__ uint32_t lds_off(uint32_t row, uint32_t chunk) {
  return row * BK + ((chunk ^ (row & 7u)) << 4);
}

struct GemmParams {
  float* out;            // P x Q (final) -- or partial sums when nsplit > 1
  uint32_t* partial;     // nsplit x P x Q raw accumulators (nsplit > 1)
  const uint8_t* X;
  const uint8_t* Z;
  uint32_t P, Q, R;      // R: bytes per operand row (contraction length x element size)
  uint32_t k_per_split;  // bytes of R per z-slice, multiple of BK
  uint32_t nsplit;
  float alpha, sx, sz;
  const float* sx_dev;
  const float* sz_dev;
  int accumulate;
};

__device__ __forceinline__ float total_scale(const GemmParams& g) {
  const float sx = g.sx_dev ? *g.sx_dev : g.sx;
  const float sz = g.sz_dev ? *g.sz_dev : g.sz;
  return __fmul_rn(g.alpha, __fmul_rn(sx, sz));
}

template <class MMA, int BM, int BN>
__global__ __launch_bounds__(NTHREADS) void gemm_nt_kernel(GemmParams g) {
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  constexpr int WTM = BM / 2, WTN = BN / 2;  // wave tile
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int STAGE = (BM + BN) * BK;
  constexpr int XLOADS = BM * (BK / 16) / NTHREADS;  // 16-byte loads per thread per stage
  constexpr int ZLOADS = BN * (BK / 16) / NTHREADS;
  using acc_t = typename MMA::acc_t;
  using frag_t = typename MMA::frag_t;
  constexpr int FRAG_CHUNKS = sizeof(frag_t) / 16;  // 16-byte chunks per lane per MFMA
  constexpr int KSUB = BK / MMA::KSTEP;

  const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
  const uint32_t wm = wave >> 1, wn = wave & 1u;
  const uint32_t p0 = blockIdx.y * BM, q0 = blockIdx.x * BN;
  const uint32_t kbeg = blockIdx.z * g.k_per_split;
  const uint32_t kend = min(g.R, kbeg + g.k_per_split);
  const int ktiles = (int)((kend - kbeg + BK - 1) / BK);

  v4i xreg[XLOADS], zreg[ZLOADS];

  auto load_global = [&](int kt) {
    const uint32_t k0 = kbeg + kt * BK;
#pragma unroll
    for (int i = 0; i < XLOADS; ++i) {
      const uint32_t id = i * NTHREADS + tid, row = id >> 3, chunk = id & 7u;
      const uint32_t p = p0 + row, k = k0 + chunk * 16;
      v4i v = {0, 0, 0, 0};
      if (p < g.P && k < kend) v = *reinterpret_cast<const v4i*>(g.X + (size_t)p * g.R + k);
      xreg[i] = v;
    }
#pragma unroll
    for (int i = 0; i < ZLOADS; ++i) {
      const uint32_t id = i * NTHREADS + tid, row = id >> 3, chunk = id & 7u;
      const uint32_t q = q0 + row, k = k0 + chunk * 16;
      v4i v = {0, 0, 0, 0};
      if (q < g.Q && k < kend) v = *reinterpret_cast<const v4i*>(g.Z + (size_t)q * g.R + k);
      zreg[i] = v;
    }
  };
  auto store_lds = [&](int buf) {
    uint8_t* xs = lds + buf * STAGE;
    uint8_t* zs = xs + BM * BK;
#pragma unroll
    for (int i = 0; i < XLOADS; ++i) {
      const uint32_t id = i * NTHREADS + tid;
      *reinterpret_cast<v4i*>(xs + lds_off(id >> 3, id & 7u)) = xreg[i];
    }
#pragma unroll
    for (int i = 0; i < ZLOADS; ++i) {
      const uint32_t id = i * NTHREADS + tid;
      *reinterpret_cast<v4i*>(zs + lds_off(id >> 3, id & 7u)) = zreg[i];
    }
  };
  auto load_frag = [&](const uint8_t* base, uint32_t row, int ks) {
    // lane (row, kgroup = lane / 32) takes FRAG_CHUNKS consecutive chunks of the row
    frag_t f;
    const uint32_t c0 = ks * (2 * FRAG_CHUNKS) + (lane >> 5) * FRAG_CHUNKS;
#pragma unroll
    for (int c = 0; c < FRAG_CHUNKS; ++c) {
      const v4i part = *reinterpret_cast<const v4i*>(base + lds_off(row, c0 + c));
      f[4 * c + 0] = part[0]; f[4 * c + 1] = part[1]; f[4 * c + 2] = part[2]; f[4 * c + 3] = part[3];
    }
    return f;
  };

  acc_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

  if (ktiles > 0) {
    load_global(0);
    store_lds(0);
  }
  __syncthreads();
  for (int kt = 0; kt < ktiles; ++kt) {
    const int buf = kt & 1;
    const bool more = kt + 1 < ktiles;
    if (more) load_global(kt + 1);
    const uint8_t* xs = lds + buf * STAGE;
    const uint8_t* zs = xs + BM * BK;
#pragma unroll
    for (int ks = 0; ks < KSUB; ++ks) {
      frag_t xf[TM], zf[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) xf[i] = load_frag(xs, wm * WTM + i * 32 + (lane & 31u), ks);
#pragma unroll
      for (int j = 0; j < TN; ++j) zf[j] = load_frag(zs, wn * WTN + j * 32 + (lane & 31u), ks);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = MMA::mma(xf[i], zf[j], acc[i][j]);
    }
    if (more) store_lds(buf ^ 1);
    __syncthreads();
  }

  // epilogue: accumulator register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, col l%32
  const float s = total_scale(g);
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const uint32_t q = q0 + wn * WTN + j * 32 + (lane & 31u);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const uint32_t p = p0 + wm * WTM + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (p < g.P && q < g.Q) {
          const size_t idx = (size_t)p * g.Q + q;
          if (g.nsplit > 1) {
            g.partial[(size_t)blockIdx.z * g.P * g.Q + idx] = MMA::bits(acc[i][j][r]);
          } else {
            float v = __fmul_rn(MMA::to_f32(acc[i][j][r]), s);
            if (g.accumulate) v = __fadd_rn(v, g.out[idx]);
            g.out[idx] = v;
          }
        }
      }
    }
}

// Fixed-order sum of the split partials (deterministic), then scale.
template <class MMA>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(GemmParams g) {
  const size_t total = (size_t)g.P * g.Q;
  const float s = total_scale(g);
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
    auto a = MMA::from_bits(g.partial[i]);
    for (uint32_t z = 1; z < g.nsplit; ++z) a += MMA::from_bits(g.partial[z * total + i]);
    float v = __fmul_rn(MMA::to_f32(a), s);
    if (g.accumulate) v = __fadd_rn(v, g.out[i]);
    g.out[i] = v;
  }
}

struct Plan {
  int bm, bn;
  uint32_t nsplit, k_per_split;
};

constexpr int NUM_CU = 256;

Plan make_plan(size_t P, size_t Q, size_t R) {
  Plan pl;
  auto tiles = [&](int bm, int bn) { return ((P + bm - 1) / bm) * ((Q + bn - 1) / bn); };
  if (tiles(256, 256) >= (size_t)NUM_CU * 3 / 4) { pl.bm = 256; pl.bn = 256; }
  else if (tiles(128, 128) >= (size_t)NUM_CU / 2) { pl.bm = 128; pl.bn = 128; }
  else { pl.bm = 64; pl.bn = 64; }
  const size_t t = tiles(pl.bm, pl.bn);
  const size_t ksteps = (R + BK - 1) / BK;
  size_t nsplit = 1;
  if (t < (size_t)NUM_CU && ksteps >= 16) {
    nsplit = (2 * NUM_CU + t - 1) / t;           // aim at two workgroups per CU
    const size_t max_split = ksteps / 8;         // keep >= 8 stages per slice
    if (nsplit > max_split) nsplit = max_split;
    if (nsplit > 64) nsplit = 64;
    if (nsplit < 1) nsplit = 1;
  }
  const size_t steps_per = (ksteps + nsplit - 1) / nsplit;
  pl.k_per_split = (uint32_t)(steps_per * BK);
  pl.nsplit = (uint32_t)((ksteps + steps_per - 1) / steps_per);
  return pl;
}

template <class MMA, int BM, int BN>
hipError_t launch_tile(const GemmParams& g, hipStream_t stream) {
  constexpr int LDS_BYTES = 2 * (BM + BN) * BK;
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_nt_kernel<MMA, BM, BN>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
    if (e != hipSuccess) return e;
    configured = true;
  }
  dim3 grid((g.Q + BN - 1) / BN, (g.P + BM - 1) / BM, g.nsplit);
  gemm_nt_kernel<MMA, BM, BN><<<grid, NTHREADS, LDS_BYTES, stream>>>(g);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (g.nsplit > 1) {
    const size_t total = (size_t)g.P * g.Q;
    size_t blocks = (total + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    splitk_reduce_kernel<MMA><<<(unsigned)blocks, 256, 0, stream>>>(g);
    e = hipGetLastError();
  }
  return e;
}

template <class MMA>
hipError_t launch_mma(const GemmParams& g, const Plan& pl, hipStream_t stream) {
  if (pl.bm == 256) return launch_tile<MMA, 256, 256>(g, stream);
  if (pl.bm == 128) return launch_tile<MMA, 128, 128>(g, stream);
  return launch_tile<MMA, 64, 64>(g, stream);
}

}  // namespace

size_t gemm_workspace_bytes(size_t P, size_t Q, size_t R, int pipe) {
  const Plan pl = make_plan(P, Q, pipe == PIPE_BF16 ? 2 * R : R);
  return pl.nsplit > 1 ? (size_t)pl.nsplit * P * Q * sizeof(uint32_t) : 0;
}

hipError_t launch_gemm_codes(float* out, const uint8_t* X, int kindX, const uint8_t* Z, int kindZ,
                             size_t P, size_t Q, size_t R, int pipe, const GemmScale& s, bool accumulate,
                             void* workspace, hipStream_t stream) {
  const size_t row_bytes = pipe == PIPE_BF16 ? 2 * R : R;
  const Plan pl = make_plan(P, Q, row_bytes);
  GemmParams g;
  g.out = out;
  g.partial = static_cast<uint32_t*>(workspace);
  g.X = X; g.Z = Z;
  g.P = (uint32_t)P; g.Q = (uint32_t)Q; g.R = (uint32_t)row_bytes;
  g.k_per_split = pl.k_per_split;
  g.nsplit = pl.nsplit;
  g.alpha = s.alpha; g.sx = s.sx; g.sz = s.sz; g.sx_dev = s.sx_dev; g.sz_dev = s.sz_dev;
  g.accumulate = accumulate ? 1 : 0;
  if (pipe == PIPE_I8) return launch_mma<I8Mma>(g, pl, stream);
  if (pipe == PIPE_BF16) return launch_mma<BF16Mma>(g, pl, stream);
  const int fx = kindX == SRQ_E5M2, fz = kindZ == SRQ_E5M2;
  if (!fx && !fz) return launch_mma<F8Mma<0, 0>>(g, pl, stream);
  if (!fx && fz) return launch_mma<F8Mma<0, 1>>(g, pl, stream);
  if (fx && !fz) return launch_mma<F8Mma<1, 0>>(g, pl, stream);
  return launch_mma<F8Mma<1, 1>>(g, pl, stream);
}

}  // namespace srq
