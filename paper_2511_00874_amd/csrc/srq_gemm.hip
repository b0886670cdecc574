// Product of two code matrices on the gfx950 matrix cores (Sec. 2.2.2: low-precision
// multiplies, high-precision accumulation == exact product of the quantized matrices).
//
//   out[p][q] = s * sum_r val(X[p][r]) * val(Z[q][r])        X: P x R, Z: Q x R, R contiguous
//
// All three products of Alg. 1 / Alg. 2 have this form once the quantizer has written the
// operands with the contraction index contiguous.  Four matrix pipelines:
//   int8 codes          v_mfma_i32_32x32x32_i8        int32 accumulators, exact
//   E4M3/E5M2 as bf16   v_mfma_f32_32x32x16_bf16      exact products, binary32 sums
//   E5M2 codes as f16   v_mfma_f32_32x32x16_f16       the same, from one-byte codes: an E5M2 code is the
//                                                     high byte of the binary16 number of the same value,
//                                                     so the operands are widened in registers
//   E4M3/E5M2 codes     v_mfma_f32_32x32x64_f8f6f4    fp8 pipeline (aligns groups of 8 products)
//
// Kernel shape.  A workgroup owns a BM x BN output tile, its waves a WGM x WGN grid of
// sub-tiles made of 32x32 MFMA tiles.  The contraction advances BK = 128 bytes per stage.
// Operand tiles go from global memory straight into LDS (buffer_load ... lds, 16 bytes per
// lane, no registers in between) through a ring of STAGES buffers, so the loads of the next
// stages are in flight while the current one is multiplied; out-of-range rows and the tail of
// the contraction come back as zeros from the buffer bounds check.  LDS rows are 128 bytes
// with the 16-byte chunks XOR-swizzled by (row mod 8): the DMA writes 8 full rows per wave
// instruction and the MFMA operand reads (ds_read_b128, one row per lane) spread over all
// banks.  The product is computed transposed inside the wave (Z rows as the first MFMA
// operand) so that each lane ends up with 4 consecutive q of one p: 16-byte output stores.
#include <type_traits>

#include "srq_internal.hpp"
#include "srq_mma.hpp"

namespace srq {
namespace {

using namespace mma;
typedef int v2i __attribute__((ext_vector_type(2)));

struct GemmParams {
  float* out;            // P x Q (final) -- or partial sums when nsplit > 1
  uint32_t* partial;     // nsplit x P x Q raw accumulators (nsplit > 1)
  const uint8_t* X;
  const uint8_t* Z;
  uint32_t P, Q, R;      // R: bytes per operand row (contraction length x element size)
  uint32_t pitch;        // bytes between operand rows (>= R, multiple of 16)
  uint32_t pitch_x;      // the same for X when its rows hold two 4-bit values per byte (else = pitch)
  uint32_t k_per_split;  // bytes of R per z-slice, multiple of BK
  uint32_t nsplit;
  uint32_t tiles_p, tiles_q;
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

// Fixed-order sum of the slice partials of a product (deterministic), then scale: workgroup
// `block` of `nblocks`.  Integer partials are summed in int32, the others in binary32.
template <bool IS_INT>
__device__ __forceinline__ void slice_sum(const SliceSum& r, uint32_t block, uint32_t nblocks) {
  const float sx = r.s.sx_dev ? *r.s.sx_dev : r.s.sx, sz = r.s.sz_dev ? *r.s.sz_dev : r.s.sz;
  const float s = __fmul_rn(r.s.alpha, __fmul_rn(sx, sz));
  auto value = [&](uint32_t bits) {
    if constexpr (IS_INT) return (int)bits; else return __uint_as_float(bits);
  };
  const size_t nthreads = (size_t)nblocks * blockDim.x, tid = (size_t)block * blockDim.x + threadIdx.x;
  if ((r.total & 3u) == 0) {
    const size_t total4 = r.total / 4;
    const v4u* part = reinterpret_cast<const v4u*>(r.partial);
    v4f* out = reinterpret_cast<v4f*>(r.out);
    for (size_t i = tid; i < total4; i += nthreads) {
      const v4u p0 = part[i];
      auto a0 = value(p0[0]), a1 = value(p0[1]), a2 = value(p0[2]), a3 = value(p0[3]);
      for (uint32_t z = 1; z < r.nsplit; ++z) {
        const v4u p = part[z * total4 + i];
        a0 += value(p[0]); a1 += value(p[1]); a2 += value(p[2]); a3 += value(p[3]);
      }
      v4f v = {__fmul_rn((float)a0, s), __fmul_rn((float)a1, s), __fmul_rn((float)a2, s), __fmul_rn((float)a3, s)};
      if (r.accumulate) {
        const v4f o = out[i];
        v = v4f{__fadd_rn(v[0], o[0]), __fadd_rn(v[1], o[1]), __fadd_rn(v[2], o[2]), __fadd_rn(v[3], o[3])};
      }
      out[i] = v;
    }
  } else {
    for (size_t i = tid; i < r.total; i += nthreads) {
      auto a = value(r.partial[i]);
      for (uint32_t z = 1; z < r.nsplit; ++z) a += value(r.partial[z * r.total + i]);
      float v = __fmul_rn((float)a, s);
      if (r.accumulate) v = __fadd_rn(v, r.out[i]);
      r.out[i] = v;
    }
  }
}

constexpr uint32_t OOB = 0x80000000u;  // beyond any operand (operands are < 2 GiB): loads as zero

// s_waitcnt vmcnt(n) alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14, others left at max)
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 0xF) | (0x7 << 4) | (0xF << 8) | ((N >> 4) << 14));
}

// One wave-level LDS DMA: 64 lanes x 16 bytes from buffer `rsrc` at byte offset `voff` (per
// lane; out of range reads as zero) to LDS address `lds_addr` + lane * 16.  Written as inline
// assembly so that the compiler does not serialise the ring of stages behind vmcnt(0): the
// kernel counts outstanding DMAs itself (wait_vmcnt).
// M0 (the LDS base of the DMA) is written inside the asm.  It is a reserved register: the compiler
// neither allocates it nor honours it in a clobber list, and it writes M0 itself only for
// constructs this file does not contain (dynamic register indexing, messages, GWS, LDS-direct
// reads).  In the assembly generated for this file every write of m0 is the one below.
__device__ __forceinline__ void lds_dma16(__amdgpu_buffer_rsrc_t rsrc, uint32_t lds_addr, uint32_t voff) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
               :
               : "s"(lds_addr), "v"(voff), "s"(rsrc)
               : "memory");
}

// Besides its tiles a launch can carry the slice sum of an EARLIER product (`rider`, complete when
// this launch starts): memory-bound work that runs beside the matrix work, in the resident slots
// the tiles leave free and in the tail of the launch, instead of in a launch of its own.
// Workgroups [0, gemm_blocks) multiply, the rest sum.  (Measured against this: the rider groups
// spread through the launch, every fourth group of 8 -- slower.)
template <class MMA, int BM, int BN, int WGM, int WGN, int STAGES>
__global__ __launch_bounds__(WGM* WGN * 64) void gemm_nt_kernel(GemmParams g, SliceSum rider, uint32_t gemm_blocks) {
  extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
  if (blockIdx.x >= gemm_blocks) {
    if (rider.is_int) slice_sum<true>(rider, blockIdx.x - gemm_blocks, gridDim.x - gemm_blocks);
    else slice_sum<false>(rider, blockIdx.x - gemm_blocks, gridDim.x - gemm_blocks);
    return;
  }
  constexpr int NW = WGM * WGN;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;  // wave tile (p x q)
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int STAGE = (BM + BN) * BK;
  constexpr int XL = BM / 8 / NW, ZL = BN / 8 / NW;  // wave-level DMA instructions per stage
  constexpr int LPW = XL + ZL;
  static_assert(XL * 8 * NW == BM && ZL * 8 * NW == BN, "tile rows must split over the waves");
  static_assert((STAGES - 2) * LPW <= 63 && STAGES >= 2, "vmcnt range");
  using acc_t = typename MMA::acc_t;
  using frag_t = typename MMA::frag_t;
  using raw_t = typename MMA::raw_t;
  constexpr int FC = sizeof(raw_t) / 16;  // 16-byte chunks a lane reads per sub-step
  constexpr int KSUB = BK / MMA::KSTEP;

  const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
  const uint32_t wave_u = __builtin_amdgcn_readfirstlane(wave);  // the same, known to be uniform
  const uint32_t wp = wave / WGN, wq = wave % WGN;
  const uint32_t lds_base = (uint32_t)(size_t)(lds_void*)lds;
  // Workgroup -> tile.  Consecutive workgroup ids are dealt round-robin to the 8 XCDs, each
  // with its own L2.  XCD x takes the contiguous range [x * chunk, (x+1) * chunk) of a tile
  // order that walks bands of GROUP tile rows column by column: the workgroups resident on one
  // XCD at a time (one or two per CU, 32 CUs) then cover a compact block of about GROUP x GROUP
  // tiles, and share GROUP X row panels and as many Z row panels in that L2 instead of one X
  // panel and a whole row of Z panels.
  // With the contraction cut into slices the order is slice-major (all tiles of slice 0, then
  // slice 1, ...): an XCD then works mostly inside one slice, i.e. on one range of the
  // contraction of a few panels, instead of on every slice of its tiles.
  constexpr uint32_t GROUP = 8;
  const uint32_t ntiles = g.tiles_p * g.tiles_q, nwork = ntiles * g.nsplit, chunk = (nwork + 7u) >> 3;
  const uint32_t work = (blockIdx.x & 7u) * chunk + (blockIdx.x >> 3);
  if (work >= nwork) return;  // padding of the last XCD's range (whole workgroup leaves)
  const uint32_t slice = work / ntiles, tile = work - slice * ntiles;
  const uint32_t band = tile / (GROUP * g.tiles_q), band_p = band * GROUP;
  const uint32_t band_rows = min(GROUP, g.tiles_p - band_p), in_band = tile - band * GROUP * g.tiles_q;
  const uint32_t tp = band_p + in_band % band_rows, tq = in_band / band_rows;
  const uint32_t p0 = tp * BM, q0 = tq * BN;
  const uint32_t kbeg = slice * g.k_per_split;
  const uint32_t kend = min(g.R, kbeg + g.k_per_split);
  const int ktiles = (int)((kend - kbeg + BK - 1) / BK);

  const __amdgpu_buffer_rsrc_t xrsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(g.X), 0, (int)(g.P * g.pitch), 0x00020000);
  const __amdgpu_buffer_rsrc_t zrsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(g.Z), 0, (int)(g.Q * g.pitch), 0x00020000);

  // LDS layout of a stage: tile row r at r * 128, its logical 16-byte chunk c at physical
  // chunk c ^ ((r >> 1) & 7).  The LDS has 64 banks (256 bytes per cycle) and serves a
  // ds_read_b128 sixteen lanes at a time: sixteen consecutive rows reading the same logical
  // chunk then touch sixteen different 16-byte slots (two rows per 256 bytes, eight swizzle
  // values per row parity), i.e. no bank conflicts.
  // DMA addressing: a wave instruction fills 8 tile rows (1 KiB of LDS, lane L at L*16); lane L
  // fetches row L/8 and the logical chunk whose physical slot is L%8.  (r >> 1) & 7 depends on
  // the parity of the 8-row block, hence two per-lane offsets.
  static_assert(XL % 2 == 0 && ZL % 2 == 0, "row blocks of a wave must start at an even block");
  const uint32_t lrow = lane >> 3;
  const uint32_t lchunk0 = (lane & 7u) ^ (lane >> 4), lchunk1 = lchunk0 ^ 4u;  // even / odd row block
  const uint32_t xvoff = (p0 + wave * XL * 8 + lrow) * g.pitch + kbeg;
  const uint32_t zvoff = (q0 + wave * ZL * 8 + lrow) * g.pitch + kbeg;

  auto issue = [&](int kt, int buf) {
    const uint32_t koff = (uint32_t)kt * BK;
    // beyond the contraction the lane loads zeros (offset past the buffer)
    const uint32_t kc0 = koff + lchunk0 * 16, kc1 = koff + lchunk1 * 16;
    const bool live0 = kbeg + kc0 < kend, live1 = kbeg + kc1 < kend;
    const uint32_t xs = lds_base + buf * STAGE + wave_u * XL * 1024;
    const uint32_t zs = lds_base + buf * STAGE + BM * BK + wave_u * ZL * 1024;
#pragma unroll
    for (int i = 0; i < XL; ++i)
      lds_dma16(xrsrc, xs + i * 1024,
                (i & 1) ? (live1 ? xvoff + kc1 + i * 8 * g.pitch : OOB) : (live0 ? xvoff + kc0 + i * 8 * g.pitch : OOB));
#pragma unroll
    for (int i = 0; i < ZL; ++i)
      lds_dma16(zrsrc, zs + i * 1024,
                (i & 1) ? (live1 ? zvoff + kc1 + i * 8 * g.pitch : OOB) : (live0 ? zvoff + kc0 + i * 8 * g.pitch : OOB));
  };

  // operand reads: lane (row = lane % 32, kgroup = lane / 32) takes FC chunks per MFMA;
  // physical chunk = logical ^ ((row >> 1) & 7), and logical = t | kgroup * FC with t a constant
  const uint32_t swz = ((lane >> 1) & 7u) ^ ((lane >> 5) * FC);
  uint32_t xoff[KSUB * FC], zoff[KSUB * FC];
#pragma unroll
  for (int t = 0; t < KSUB * FC; ++t) {
    const uint32_t tt = (t / FC) * 2 * FC + (t % FC);
    xoff[t] = (wp * WTM + (lane & 31u)) * BK + ((swz ^ tt) << 4);
    zoff[t] = BM * BK + (wq * WTN + (lane & 31u)) * BK + ((swz ^ tt) << 4);
  }
  auto load_frag = [&](const uint8_t* stage, const uint32_t (&off)[KSUB * FC], int sub, int ks) {
    raw_t f;
#pragma unroll
    for (int c = 0; c < FC; ++c) {
      const v4i part = *reinterpret_cast<const v4i*>(stage + off[ks * FC + c] + sub * 32 * BK);
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

#pragma unroll
  for (int s = 0; s < STAGES - 1; ++s) issue(s, s);  // stages past the end load zeros

  // one stage: the fragments of the sub-steps up to PF ahead are fetched before sub-step ks is
  // multiplied; the scheduling barriers pin that order (the LDS latency then hides behind the
  // MFMAs) and bound the number of live fragments (registers)
  constexpr int PF = KSUB > 2 ? 2 : 1;
  auto compute = [&](int buf) {
    const uint8_t* stage = lds + buf * STAGE;
    raw_t xf[PF + 1][TM], zf[PF + 1][TN];
    auto fetch = [&](int ks) {
#pragma unroll
      for (int i = 0; i < TM; ++i) xf[ks % (PF + 1)][i] = load_frag(stage, xoff, i, ks);
#pragma unroll
      for (int j = 0; j < TN; ++j) zf[ks % (PF + 1)][j] = load_frag(stage, zoff, j, ks);
    };
#pragma unroll
    for (int ks = 0; ks < PF && ks < KSUB; ++ks) fetch(ks);
    // the interleaved widening below keeps two widened operand sets live: it fits the register
    // file of the 4-wave workgroups (two of them per CU), not of the 8-wave 256 x 256 one
    constexpr bool INTERLEAVE = MMA::WIDENS && NW <= 4;
    if constexpr (!INTERLEAVE) {
#pragma unroll
      for (int ks = 0; ks < KSUB; ++ks) {
        if (ks + PF < KSUB) fetch(ks + PF);
        __builtin_amdgcn_sched_barrier(0);
        frag_t xe[TM], ze[TN];  // (a plain copy unless the pipeline widens its operands)
#pragma unroll
        for (int i = 0; i < TM; ++i) xe[i] = MMA::expand(xf[ks % (PF + 1)][i]);
#pragma unroll
        for (int j = 0; j < TN; ++j) ze[j] = MMA::expand(zf[ks % (PF + 1)][j]);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j) acc[i][j] = MMA::mma(ze[j], xe[i], acc[i][j]);  // MFMA rows: q, columns: p
        __builtin_amdgcn_sched_barrier(0);
      }
    } else {
      // Operands are widened in registers (VALU) before they are multiplied.  A wave issues in
      // order, so widening a whole sub-step and then multiplying it would leave the matrix pipe
      // idle during the widening: instead the operands of sub-step ks + 1 are widened while the
      // MFMAs of sub-step ks are issued, a few VALU operations after each MFMA (the scheduling
      // groups below pin that interleaving).
      frag_t xe[2][TM], ze[2][TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) xe[0][i] = MMA::expand(xf[0][i]);
#pragma unroll
      for (int j = 0; j < TN; ++j) ze[0][j] = MMA::expand(zf[0][j]);
#pragma unroll
      for (int ks = 0; ks < KSUB; ++ks) {
        if (ks + PF < KSUB) fetch(ks + PF);
        __builtin_amdgcn_sched_barrier(0);
        if (ks + 1 < KSUB) {
#pragma unroll
          for (int i = 0; i < TM; ++i) xe[(ks + 1) & 1][i] = MMA::expand(xf[(ks + 1) % (PF + 1)][i]);
#pragma unroll
          for (int j = 0; j < TN; ++j) ze[(ks + 1) & 1][j] = MMA::expand(zf[(ks + 1) % (PF + 1)][j]);
        }
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j) acc[i][j] = MMA::mma(ze[ks & 1][j], xe[ks & 1][i], acc[i][j]);
        constexpr int N_MFMA = TM * TN * MMA::MFMA_PER_MMA;
        constexpr int N_VALU = (TM + TN) * MMA::VALU_PER_EXPAND;
        constexpr int PER = (N_VALU + N_MFMA - 1) / N_MFMA;
#pragma unroll
        for (int m = 0; m < N_MFMA; ++m) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);    // one MFMA
          __builtin_amdgcn_sched_group_barrier(0x002, PER, 0);  // then up to PER VALU operations
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };

  // ring of STAGES buffers, one barrier per stage: after the barrier of step kt every wave has
  // finished step kt-1, whose buffer is the one refilled now
  for (int kt0 = 0; kt0 < ktiles; kt0 += STAGES) {
#pragma unroll
    for (int s = 0; s < STAGES; ++s) {
      const int kt = kt0 + s;
      if (kt < ktiles) {
        wait_vmcnt<(STAGES - 2) * LPW>();
        __syncthreads();
        issue(kt + STAGES - 1, (s + STAGES - 1) % STAGES);
        compute(s);
      }
    }
  }

  // epilogue.  MFMA result register r of lane l: MFMA row 8*(r/4) + 4*(l/32) + r%4 (a q),
  // MFMA column l%32 (a p).  Each wave turns its tile through its own piece of LDS, one band
  // of 32 p-rows at a time, so that every global store instruction writes whole rows of the
  // band: WTN * 4 contiguous bytes per row.
  constexpr int EP_PITCH = WTN + 4;                   // floats; +4 staggers the banks
  constexpr int EP_WAVE = 32 * EP_PITCH * 4;          // bytes per wave
  static_assert(NW * EP_WAVE <= STAGES * STAGE, "epilogue staging must fit in the operand ring");
  constexpr int CPR = WTN / 4;                        // 16-byte chunks per band row
  constexpr int EP_ITERS = 32 * CPR / 64;
  wait_vmcnt<0>();   // the zero-filled stages issued past the end must have landed too
  __syncthreads();
  uint32_t* ep = reinterpret_cast<uint32_t*>(lds + wave * EP_WAVE);
  const float s = total_scale(g);
  const bool q_vec = (g.Q & 3u) == 0;
  const uint32_t qw0 = q0 + wq * WTN;
  uint32_t* const pbase = g.nsplit > 1 ? g.partial + (size_t)slice * g.P * g.Q : nullptr;
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int gq = 0; gq < 4; ++gq)
        *reinterpret_cast<v4u*>(ep + (lane & 31u) * EP_PITCH + j * 32 + 8 * gq + 4 * (lane >> 5)) =
            v4u{MMA::bits(acc[i][j][4 * gq]), MMA::bits(acc[i][j][4 * gq + 1]), MMA::bits(acc[i][j][4 * gq + 2]),
                MMA::bits(acc[i][j][4 * gq + 3])};
    const uint32_t pb = p0 + wp * WTM + i * 32;
#pragma unroll
    for (int it = 0; it < EP_ITERS; ++it) {
      const uint32_t id = it * 64 + lane, row = id / CPR, c = id % CPR;
      const uint32_t p = pb + row, q = qw0 + c * 4;
      const v4u raw = *reinterpret_cast<const v4u*>(ep + row * EP_PITCH + c * 4);
      if (p >= g.P || q >= g.Q) continue;
      const size_t idx = (size_t)p * g.Q + q;
      if (pbase) {
        if (q_vec) {
          // write-through: nothing of the partial tile stays dirty in the L2 when the kernel
          // ends, and the reduction launched next still finds it in the last-level cache
          asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1" : : "v"(pbase + idx), "v"(raw) : "memory");
        } else {
          for (int e = 0; e < 4 && q + e < g.Q; ++e) pbase[idx + e] = raw[e];
        }
      } else {
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = __fmul_rn(MMA::to_f32(MMA::from_bits(raw[e])), s);
        float* dst = g.out + idx;
        if (q_vec) {
          if (g.accumulate) {
            const v4f o = *reinterpret_cast<const v4f*>(dst);
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = __fadd_rn(v[e], o[e]);
          }
          // the result is not read again by this kernel: a streaming store keeps it from pushing
          // operand panels out of the L2
          __builtin_nontemporal_store(v4f{v[0], v[1], v[2], v[3]}, reinterpret_cast<v4f*>(dst));
        } else {
          for (int e = 0; e < 4 && q + e < g.Q; ++e) dst[e] = g.accumulate ? __fadd_rn(v[e], dst[e]) : v[e];
        }
      }
    }
  }
}

// ---- 256 x 256 tiles, workgroups that stay -------------------------------------------------------
// One workgroup per CU walks a list of tiles.  What that buys over one workgroup per tile:
//   - the operand loads of the next tile's first stage are issued during the last stage of the
//     current tile and land while its result is written, so no tile starts with an empty ring;
//   - the result stores of tile i drain while tile i + 1 is multiplied.
// The second point needs care on this chip: loads and stores of a wave share ONE in-order counter
// (vmcnt), so a wave that has result stores in flight cannot wait for a later operand load without
// waiting for those stores as well.  Waves 0-3 ("loaders") issue every operand DMA of the
// workgroup and are the only ones that wait on the counter; all eight multiply (wave tile
// 128 x 64) and every wave writes out its own part of a finished tile, band by band through its own
// piece of the staging area, without a barrier.  The loaders' one wait that can meet stores still
// in flight is the first of the next tile, and it costs less than what it replaced: a form in
// which only waves 4-7 stored -- the others handing them their bands through LDS and two barriers
// per band -- kept the loaders' counter exact and was 1.5 % slower on the Llama-shaped products.
// The ring has two stages of 64 KiB.  Stages are numbered through the whole tile list (`gs`): the
// loaders issue stage gs + 1 -- the next stage of this tile, or the first of the next tile -- at
// the barrier of stage gs, into the buffer that stage gs - 1 has just left.  When a tile is done,
// the buffer of its last stage is the staging area of the epilogue (the other one is receiving the
// next tile's first stage); it is handed back to the ring by the barrier of the next stage.
// Every loop bound below is uniform over the workgroup, so all waves meet at every barrier.
// The lane index again, as a value the optimiser cannot see through.  Address arithmetic that is
// derived from it inside a loop is recomputed there (a few VALU operations) instead of being
// hoisted out of the loop and held in registers across it: in the kernel below the accumulators and
// operand fragments leave no room for that.
__device__ __forceinline__ uint32_t opaque(uint32_t v) {
  asm volatile("" : "+v"(v));
  return v;
}

struct TileItem {
  uint32_t valid, p0, q0, slice, kbeg, kend;
};

// XP: the X operand holds 4-bit integers, two per byte ("packed": byte j of every 8 holds elements j
// and j + 8 of a run of 16 along the contraction, low and high nibble).  Its rows take 64 bytes of
// a stage, half the DMA instructions, and half the LDS bytes per fragment; a fragment is widened in
// registers to the bytes 16 * value (shift / mask: the nibble's sign bit becomes the byte's), so
// the accumulators hold 16 times the sums and the caller passes alpha / 16 -- powers of two, the
// results are bit for bit those of the one-byte form.
template <class MMA, bool XP>
__global__ __launch_bounds__(512) void gemm_nt_persist_kernel(GemmParams g, SliceSum rider) {
  extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
  constexpr int BM = 256, BN = 256, WGN = 4, NW = 8, NLOAD = 4;
  constexpr int WTM = 128, WTN = 64, TM = WTM / 32, TN = WTN / 32;
  constexpr int STAGE = (BM + BN) * BK;
  // DMA instructions per loader wave and stage (an instruction covers 8 rows of 128 bytes, or 16 packed rows of 64)
  constexpr int XL = XP ? BM / 16 / NLOAD : BM / 8 / NLOAD, ZL = BN / 8 / NLOAD;
  static_assert(XL % 2 == 0 && ZL % 2 == 0, "row blocks of a wave must start at an even block");
  static_assert(XL + ZL <= 63, "vmcnt range");
  using acc_t = typename MMA::acc_t;
  using frag_t = typename MMA::frag_t;
  using raw_t = typename MMA::raw_t;
  constexpr int FC = sizeof(raw_t) / 16;
  constexpr int KSUB = BK / MMA::KSTEP;
  static_assert(!XP || (FC == 1 && sizeof(frag_t) == 16 && MMA::KSTEP == 32), "packed X: the int8 pipeline only");

  const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
  const uint32_t wave_u = __builtin_amdgcn_readfirstlane(wave);
  const bool loader = wave_u < NLOAD;
  const uint32_t wp = wave / WGN, wq = wave % WGN;
  const uint32_t lds_base = (uint32_t)(size_t)(lds_void*)lds;

  // Tile list of this workgroup.  As in gemm_nt_kernel, XCD x (workgroup ids = x mod 8) owns the
  // contiguous range [x * chunk, (x + 1) * chunk) of the banded, slice-major tile order; its
  // workgroups (slots) walk that range side by side, so the tiles in flight on one XCD at any time
  // are neighbours and share operand panels in that L2.
  constexpr uint32_t GROUP = 8;
  const uint32_t ntiles = g.tiles_p * g.tiles_q, nwork = ntiles * g.nsplit, chunk = (nwork + 7u) >> 3;
  const uint32_t xcd = blockIdx.x & 7u, slot = blockIdx.x >> 3, nslots = gridDim.x >> 3;
  const uint32_t range_end = min(nwork, (xcd + 1) * chunk);
  auto item_at = [&](uint32_t n) {
    TileItem it;
    const uint32_t work = xcd * chunk + slot + n * nslots;
    it.valid = work < range_end ? 1u : 0u;
    const uint32_t w = it.valid ? work : 0u;
    const uint32_t slice = w / ntiles, tile = w - slice * ntiles;
    const uint32_t band = tile / (GROUP * g.tiles_q), band_p = band * GROUP;
    const uint32_t band_rows = min(GROUP, g.tiles_p - band_p), in_band = tile - band * GROUP * g.tiles_q;
    it.p0 = (band_p + in_band % band_rows) * BM;
    it.q0 = (in_band / band_rows) * BN;
    it.slice = slice;
    it.kbeg = slice * g.k_per_split;
    it.kend = min(g.R, it.kbeg + g.k_per_split);
    return it;
  };

  const __amdgpu_buffer_rsrc_t xrsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(g.X), 0, (int)(g.P * g.pitch_x), 0x00020000);
  const __amdgpu_buffer_rsrc_t zrsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(g.Z), 0, (int)(g.Q * g.pitch), 0x00020000);

  // DMA addressing (LDS layout of a stage as in gemm_nt_kernel: 128-byte rows, 16-byte chunk c of
  // row r at chunk c ^ ((r >> 1) & 7)); loader wave w fills tile rows [64 w, 64 w + 64) of X and of Z
  auto issue = [&](const TileItem& it, int kt, uint32_t buf) {
    const uint32_t ln = opaque(lane);
    const uint32_t lrow = ln >> 3;
    const uint32_t lchunk0 = (ln & 7u) ^ (ln >> 4), lchunk1 = lchunk0 ^ 4u;
    const uint32_t xvoff = (it.p0 + wave * XL * 8 + lrow) * g.pitch + it.kbeg;
    const uint32_t zvoff = (it.q0 + wave * ZL * 8 + lrow) * g.pitch + it.kbeg;
    const uint32_t koff = (uint32_t)kt * BK;
    const uint32_t kc0 = koff + lchunk0 * 16, kc1 = koff + lchunk1 * 16;
    const bool live0 = it.kbeg + kc0 < it.kend, live1 = it.kbeg + kc1 < it.kend;
    const uint32_t xs = lds_base + buf * STAGE + wave_u * XL * 1024;
    const uint32_t zs = lds_base + buf * STAGE + BM * BK + wave_u * ZL * 1024;
    if constexpr (XP) {
      // packed rows: 64 bytes of a row per stage, 16 rows per instruction; lane L fetches row L / 4
      // and the logical 16-byte chunk whose physical slot is L % 4 (chunk c of row r is stored at
      // chunk c ^ ((r >> 2) & 3)); a chunk holds 32 elements of the contraction
      const uint32_t pchunk = (ln & 3u) ^ ((ln >> 4) & 3u);
      const uint32_t xvp = (it.p0 + wave * XL * 16 + (ln >> 2)) * g.pitch_x + ((it.kbeg + koff) >> 1) + pchunk * 16;
      const bool livep = it.kbeg + koff + pchunk * 32 < it.kend;
#pragma unroll
      for (int i = 0; i < XL; ++i) lds_dma16(xrsrc, xs + i * 1024, livep ? xvp + i * 16 * g.pitch_x : OOB);
    } else {
#pragma unroll
      for (int i = 0; i < XL; ++i)
        lds_dma16(xrsrc, xs + i * 1024,
                  (i & 1) ? (live1 ? xvoff + kc1 + i * 8 * g.pitch : OOB) : (live0 ? xvoff + kc0 + i * 8 * g.pitch : OOB));
    }
#pragma unroll
    for (int i = 0; i < ZL; ++i)
      lds_dma16(zrsrc, zs + i * 1024,
                (i & 1) ? (live1 ? zvoff + kc1 + i * 8 * g.pitch : OOB) : (live0 ? zvoff + kc0 + i * 8 * g.pitch : OOB));
  };

  const uint32_t swz = ((lane >> 1) & 7u) ^ ((lane >> 5) * FC);
  uint32_t xoff[KSUB * FC], zoff[KSUB * FC];
#pragma unroll
  for (int t = 0; t < KSUB * FC; ++t) {
    const uint32_t tt = (t / FC) * 2 * FC + (t % FC);
    xoff[t] = (wp * WTM + (lane & 31u)) * BK + ((swz ^ tt) << 4);
    zoff[t] = BM * BK + (wq * WTN + (lane & 31u)) * BK + ((swz ^ tt) << 4);
  }
  // packed X: 8 bytes per lane and MFMA (16 elements), row pitch 64, chunk ks of row r at ks ^ ((r >> 2) & 3)
  uint32_t xoffp[KSUB];
#pragma unroll
  for (int ks = 0; ks < KSUB; ++ks)
    xoffp[ks] = (wp * WTM + (lane & 31u)) * 64u + ((((uint32_t)ks ^ (lane >> 2)) & 3u) << 4) + 8u * (lane >> 5);
  auto load_frag = [&](const uint8_t* stage, const uint32_t (&off)[KSUB * FC], int sub, int ks) {
    raw_t f;
#pragma unroll
    for (int c = 0; c < FC; ++c) {
      const v4i part = *reinterpret_cast<const v4i*>(stage + off[ks * FC + c] + sub * 32 * BK);
      f[4 * c + 0] = part[0]; f[4 * c + 1] = part[1]; f[4 * c + 2] = part[2]; f[4 * c + 3] = part[3];
    }
    return f;
  };

  acc_t acc[TM][TN];
    // fragments are read one sub-step ahead (two, as in gemm_nt_kernel, is no faster here and costs 24
  // registers): at 219 VGPRs two waves of this kernel leave a SIMD 64 registers, enough for one wave
  // of the quantizer or absmax kernels, so a memory-bound launch on another stream runs BESIDE this
  // kernel on the same CUs instead of behind it
  constexpr int PF = 1;
  auto compute = [&](uint32_t buf) {
    const uint8_t* stage = lds + buf * STAGE;
    typename std::conditional<XP, v2i, raw_t>::type xf[PF + 1][TM];
    raw_t zf[PF + 1][TN];
    auto fetch = [&](int ks) {
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        if constexpr (XP) xf[ks % (PF + 1)][i] = *reinterpret_cast<const v2i*>(stage + xoffp[ks] + i * 32 * 64);
        else xf[ks % (PF + 1)][i] = load_frag(stage, xoff, i, ks);
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) zf[ks % (PF + 1)][j] = load_frag(stage, zoff, j, ks);
    };
#pragma unroll
    for (int ks = 0; ks < PF && ks < KSUB; ++ks) fetch(ks);
#pragma unroll
    for (int ks = 0; ks < KSUB; ++ks) {
      if (ks + PF < KSUB) fetch(ks + PF);
      __builtin_amdgcn_sched_barrier(0);
      frag_t xe[TM], ze[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        if constexpr (XP) {
          // byte j of the 8 holds elements j (low nibble) and j + 8 (high nibble): four words of 16 * value
          const v2i x = xf[ks % (PF + 1)][i];
          const int hi = (int)0xF0F0F0F0u;
          xe[i] = frag_t{(x[0] << 4) & hi, (x[1] << 4) & hi, x[0] & hi, x[1] & hi};
        } else {
          xe[i] = MMA::expand(xf[ks % (PF + 1)][i]);
        }
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) ze[j] = MMA::expand(zf[ks % (PF + 1)][j]);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = MMA::mma(ze[j], xe[i], acc[i][j]);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // Epilogue staging: every wave owns 8 KiB, a band of 32 p-rows x 64 q as rows of 256 bytes
  // (16 chunks of 16 bytes); chunk c of row r is stored at chunk c ^ (r & 15), so that the
  // sixteen lanes an LDS instruction serves together -- sixteen rows with one chunk index when
  // the MFMA registers are written, sixteen chunks of one row when the rows are read back --
  // always fall on sixteen different 16-byte slots of the 64 banks.
  constexpr int EP_WAVE = 32 * WTN * 4;
  static_assert(NW * EP_WAVE <= STAGE, "epilogue staging must fit in one ring buffer");
  const float s = total_scale(g);
  const bool q_vec = (g.Q & 3u) == 0;

  TileItem cur = item_at(0);
  uint32_t n_item = 0, gs = 0;
  if (cur.valid) {
    if (loader) issue(cur, 0, 0);
    while (true) {
      const TileItem nxt = item_at(++n_item);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;
      const int ktiles = (int)((cur.kend - cur.kbeg + BK - 1) / BK);
      for (int kt = 0; kt < ktiles; ++kt) {
        if (loader) wait_vmcnt<0>();  // stage gs has landed (the only DMAs in flight)
        __syncthreads();              // ... for every wave; and every wave has left stage gs - 1
        if (loader) {
          if (kt + 1 < ktiles) issue(cur, kt + 1, (gs + 1) & 1u);
          else if (nxt.valid) issue(nxt, 0, (gs + 1) & 1u);
        }
        compute(gs & 1u);
        ++gs;
      }
      __syncthreads();  // the buffer of the last stage is free: it stages the result
      uint8_t* const stg = lds + ((gs - 1) & 1u) * STAGE;
      uint32_t* const pbase = g.nsplit > 1 ? g.partial + (size_t)cur.slice * g.P * g.Q : nullptr;
      // whole tile inside the output, rows 16-byte aligned, nothing to add to: plain row stores
      const bool fast = q_vec && !g.accumulate && cur.p0 + BM <= g.P && cur.q0 + BN <= g.Q;
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        // MFMA result register r of lane l: q = 8 (r / 4) + 4 (l / 32) + r % 4, p = l % 32.
        // Final results are converted and scaled here, by the wave that computed them (all eight
        // share that work); partial results of a slice go out as raw accumulator bits.
        const uint32_t le = opaque(lane);
        uint8_t* const mine = stg + wave_u * EP_WAVE + (le & 31u) * (WTN * 4);
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int gq = 0; gq < 4; ++gq) {
            const uint32_t c = j * 8 + 2 * gq + (le >> 5);
            v4u w;
#pragma unroll
            for (int e = 0; e < 4; ++e)
              w[e] = pbase ? MMA::bits(acc[i][j][4 * gq + e])
                           : __float_as_uint(__fmul_rn(MMA::to_f32(acc[i][j][4 * gq + e]), s));
            *reinterpret_cast<v4u*>(mine + ((c ^ (le & 15u)) << 4)) = w;
          }
        // the wave reads back what it has just written (its LDS instructions complete in order) and
        // writes whole rows of its band
        __builtin_amdgcn_wave_barrier();
        {
          {
            const uint32_t src = wave_u;
            const uint32_t pb = cur.p0 + (src / WGN) * WTM + i * 32, qw0 = cur.q0 + (src % WGN) * WTN;
            const uint8_t* const band = stg + src * EP_WAVE;
            const uint32_t ls = opaque(lane);
            const uint32_t r4 = ls >> 4, c = ls & 15u;
            if (fast) {
              // EB row reads in flight, then EB stores of four whole 256-byte rows each
              constexpr int EB = FC > 1 ? 4 : 8;  // (the pipeline with 32-byte fragments has fewer registers to spare)
              uint32_t* const dst0 = (pbase ? pbase : reinterpret_cast<uint32_t*>(g.out)) +
                                     (size_t)(pb + r4) * g.Q + qw0 + c * 4;
#pragma unroll
              for (int it0 = 0; it0 < 8; it0 += EB) {
                v4u raw[EB];
#pragma unroll
                for (int it = 0; it < EB; ++it) {
                  const uint32_t row = (it0 + it) * 4 + r4;
                  raw[it] = *reinterpret_cast<const v4u*>(band + row * (WTN * 4) + ((c ^ (row & 15u)) << 4));
                }
#pragma unroll
                for (int it = 0; it < EB; ++it) {
                  uint32_t* const dst = dst0 + (size_t)(it0 + it) * 4 * g.Q;
                  if (pbase) {
                    // write-through: the partial tile does not stay dirty in the L2, and the sum
                    // that reads it next still finds it in the last-level cache
                    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1" : : "v"(dst), "v"(raw[it]) : "memory");
                  } else {
                    // not read again by this kernel: a streaming store keeps it from pushing
                    // operand panels out of the L2
                    __builtin_nontemporal_store(raw[it], reinterpret_cast<v4u*>(dst));
                  }
                }
              }
            } else {
#pragma unroll 2
              for (int it = 0; it < 8; ++it) {
                const uint32_t row = it * 4 + r4;
                const v4u raw = *reinterpret_cast<const v4u*>(band + row * (WTN * 4) + ((c ^ (row & 15u)) << 4));
                const uint32_t p = pb + row, q = qw0 + c * 4;
                if (p >= g.P || q >= g.Q) continue;
                const size_t idx = (size_t)p * g.Q + q;
                if (pbase) {
                  if (q_vec) {
                    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1" : : "v"(pbase + idx), "v"(raw) : "memory");
                  } else {
                    for (int e = 0; e < 4 && q + e < g.Q; ++e) pbase[idx + e] = raw[e];
                  }
                } else {
                  float v[4];
#pragma unroll
                  for (int e = 0; e < 4; ++e) v[e] = __uint_as_float(raw[e]);
                  float* dst = g.out + idx;
                  if (q_vec) {
                    if (g.accumulate) {
                      const v4f o = *reinterpret_cast<const v4f*>(dst);
#pragma unroll
                      for (int e = 0; e < 4; ++e) v[e] = __fadd_rn(v[e], o[e]);
                    }
                    __builtin_nontemporal_store(v4f{v[0], v[1], v[2], v[3]}, reinterpret_cast<v4f*>(dst));
                  } else {
                    for (int e = 0; e < 4 && q + e < g.Q; ++e) dst[e] = g.accumulate ? __fadd_rn(v[e], dst[e]) : v[e];
                  }
                }
              }
            }
          }
        }
      }
      if (!nxt.valid) break;
      cur = nxt;
    }
  }
  // the slice sum of an earlier product, if this launch carries one: every workgroup takes a share
  // once its tiles are done
  if (rider.total > 0) {
    if (rider.is_int) slice_sum<true>(rider, blockIdx.x, gridDim.x);
    else slice_sum<false>(rider, blockIdx.x, gridDim.x);
  }
}

// The slice sum in a launch of its own.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(SliceSum r) {
  if (r.is_int) slice_sum<true>(r, blockIdx.x, gridDim.x);
  else slice_sum<false>(r, blockIdx.x, gridDim.x);
}

struct Plan {
  int tile;  // 0: 256x256, 1: 128x128, 2: 64x64, 3: 128x192
  int bm, bn;
  uint32_t nsplit, k_per_split;
};

constexpr int NUM_CU = 256;

// Tile shape and number of contraction slices by a cost model (seconds, for ranking only):
//   time = rounds x (stages per item + fixed per-item stages) x operations per stage / rate
//          + the pass over the partial results that every extra slice adds.
// `rate` is what a CU sustains with that tile shape once its slots are full (measured, int8: the
// other pipelines scale alike): 256 x 256 tiles on workgroups that stay run one per CU and hide
// most of a tile's start and end; the 128-row tiles run two workgroups per CU (one alone gets
// about 0.85 of the CU's rate); 64 x 64 is for problems too small for anything else.
struct TileKind {
  int tile, bm, bn, per_cu;
  double rate_chip;   // operations per second over the whole chip, slots full
  double fixed;       // start + end of an item, in stages
};
constexpr TileKind TILE_KINDS[] = {
    {0, 256, 256, 1, 2.1e15, 6.0},
    {1, 128, 128, 2, 1.45e15, 3.0},
    {3, 128, 192, 2, 1.5e15, 3.0},
    {2, 64, 64, 4, 0.5e15, 4.0},
};
constexpr double PARTIAL_BYTES_PER_SECOND = 4.0e12;  // partial tiles out and back in

Plan make_plan(size_t P, size_t Q, size_t row_bytes) {
  const size_t ksteps = (row_bytes + BK - 1) / BK;
  Plan best{};
  double best_time = 0.0;
  bool have = false;
  for (const TileKind& k : TILE_KINDS) {
    const size_t t = ((P + k.bm - 1) / k.bm) * ((Q + k.bn - 1) / k.bn);
    // slices only for long contractions (at least 8 stages each), at most 64
    size_t max_split = ksteps >= 16 ? ksteps / 8 : 1;
    if (max_split > 64) max_split = 64;
    const double ops_stage = 2.0 * k.bm * k.bn * BK;
    const double rate_cu = k.rate_chip / NUM_CU;
    for (size_t n = 1; n <= max_split; ++n) {
      const size_t items = t * n, slots = (size_t)NUM_CU * k.per_cu;
      const size_t rounds = (items + slots - 1) / slots;
      const size_t stages = (ksteps + n - 1) / n;
      // a workgroup's share of its CU: alone, or one of per_cu
      const double share = items <= (size_t)NUM_CU ? (k.per_cu > 1 ? 0.85 : 1.0) : 1.0 / k.per_cu;
      double time = (double)rounds * ((double)stages + k.fixed) * ops_stage / (rate_cu * share);
      if (n > 1) time += 2.0 * (double)n * (double)P * (double)Q * 4.0 / PARTIAL_BYTES_PER_SECOND;
      if (!have || time < best_time) {
        have = true;
        best_time = time;
        best.tile = k.tile; best.bm = k.bm; best.bn = k.bn;
        best.nsplit = (uint32_t)n;
      }
    }
  }
  const size_t steps_per = (ksteps + best.nsplit - 1) / best.nsplit;
  best.k_per_split = (uint32_t)(steps_per * BK);
  best.nsplit = (uint32_t)((ksteps + steps_per - 1) / steps_per);
  return best;
}

// What a launch is asked to do about slice sums: carry the one of an earlier product (`carry`,
// may be null or empty), and either run its own afterwards or hand it to the caller (`defer`).
struct SliceSumPlan {
  const SliceSum* carry;
  SliceSum* defer;
};

// per_thread elements per thread where the vector path applies (a launch of its own wants many
// small workgroups, riders few and fat ones: each holds a tile's slot), at most 4096 workgroups
uint32_t slice_sum_blocks(const SliceSum& r, uint32_t threads, uint32_t per_thread) {
  const size_t per_block = (size_t)threads * ((r.total & 3u) == 0 ? per_thread : 1);
  size_t blocks = (r.total + per_block - 1) / per_block;
  if (blocks > 4096) blocks = 4096;
  return (uint32_t)(blocks < 1 ? 1 : blocks);
}

template <class MMA, int BM, int BN, int WGM, int WGN, int STAGES>
hipError_t launch_tile(GemmParams g, const SliceSumPlan& ss, hipStream_t stream) {
  constexpr int LDS_BYTES = STAGES * (BM + BN) * BK;
  static_assert(LDS_BYTES <= 160 * 1024, "LDS");
  auto kern = &gemm_nt_kernel<MMA, BM, BN, WGM, WGN, STAGES>;
  // once per kernel (a function-local static: its initialisation is safe against concurrent
  // first calls from several host threads)
  static const hipError_t configured = hipFuncSetAttribute(
      reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
  if (configured != hipSuccess) return configured;
  g.tiles_p = (g.P + BM - 1) / BM;
  g.tiles_q = (g.Q + BN - 1) / BN;
  const uint32_t gemm_blocks = ((g.tiles_p * g.tiles_q * g.nsplit + 7) / 8) * 8;
  SliceSum carry{};
  uint32_t carry_blocks = 0;
  if (ss.carry && ss.carry->total > 0) {
    carry = *ss.carry;
    carry_blocks = slice_sum_blocks(carry, WGM * WGN * 64, 16);
  }
  kern<<<dim3(gemm_blocks + carry_blocks), WGM * WGN * 64, LDS_BYTES, stream>>>(g, carry, gemm_blocks);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  SliceSum own{};
  if (g.nsplit > 1) {
    own.partial = g.partial; own.out = g.out; own.nsplit = g.nsplit; own.total = (size_t)g.P * g.Q;
    own.s = GemmScale{g.alpha, g.sx, g.sz, g.sx_dev, g.sz_dev};
    own.accumulate = g.accumulate;
    own.is_int = std::is_same<typename MMA::acc_t, v16i>::value ? 1 : 0;
  }
  if (ss.defer) {
    *ss.defer = own;
  } else if (own.total > 0) {
    splitk_reduce_kernel<<<slice_sum_blocks(own, 256, 4), 256, 0, stream>>>(own);
    e = hipGetLastError();
  }
  return e;
}

// The 256 x 256 tiles on workgroups that stay (gemm_nt_persist_kernel): one workgroup per CU, or
// fewer if there is less work.
template <class MMA, bool XP = false>
hipError_t launch_persist(GemmParams g, const SliceSumPlan& ss, hipStream_t stream) {
  constexpr int LDS_BYTES = 2 * (256 + 256) * BK;
  auto kern = &gemm_nt_persist_kernel<MMA, XP>;
  static const hipError_t configured = hipFuncSetAttribute(
      reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
  if (configured != hipSuccess) return configured;
  g.tiles_p = (g.P + 255) / 256;
  g.tiles_q = (g.Q + 255) / 256;
  const uint32_t nwork = g.tiles_p * g.tiles_q * g.nsplit, chunk = (nwork + 7) / 8;
  const uint32_t slots = chunk < NUM_CU / 8 ? chunk : NUM_CU / 8;  // workgroups per XCD
  SliceSum carry{};
  if (ss.carry && ss.carry->total > 0) carry = *ss.carry;
  kern<<<dim3(8 * slots), 512, LDS_BYTES, stream>>>(g, carry);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  SliceSum own{};
  if (g.nsplit > 1) {
    own.partial = g.partial; own.out = g.out; own.nsplit = g.nsplit; own.total = (size_t)g.P * g.Q;
    own.s = GemmScale{g.alpha, g.sx, g.sz, g.sx_dev, g.sz_dev};
    own.accumulate = g.accumulate;
    own.is_int = std::is_same<typename MMA::acc_t, v16i>::value ? 1 : 0;
  }
  if (ss.defer) {
    *ss.defer = own;
  } else if (own.total > 0) {
    splitk_reduce_kernel<<<slice_sum_blocks(own, 256, 4), 256, 0, stream>>>(own);
    e = hipGetLastError();
  }
  return e;
}

template <class MMA>
hipError_t launch_mma(const GemmParams& g, const Plan& pl, const SliceSumPlan& ss, hipStream_t stream) {
  if (pl.tile == 0) return launch_persist<MMA>(g, ss, stream);                  // 8 waves of 128 x 64, persistent
  if (pl.tile == 1) return launch_tile<MMA, 128, 128, 2, 2, 2>(g, ss, stream);  // 4 waves of 64 x 64
  if (pl.tile == 3) return launch_tile<MMA, 128, 192, 2, 2, 2>(g, ss, stream);  // 4 waves of 64 x 96
  return launch_tile<MMA, 64, 64, 2, 2, 3>(g, ss, stream);
}

}  // namespace

size_t gemm_workspace_bytes(size_t P, size_t Q, size_t R, int pipe) {
  const Plan pl = make_plan(P, Q, pipe == PIPE_BF16 ? 2 * R : R);
  return pl.nsplit > 1 ? (size_t)pl.nsplit * P * Q * sizeof(uint32_t) : 0;
}

bool gemm_takes_packed_x(size_t P, size_t Q, size_t R, int pipe) {
  return pipe == PIPE_I8 && make_plan(P, Q, R).tile == 0;
}

bool gemm_operands_addressable(size_t P, size_t Q, size_t R, int pipe) {
  const size_t rb = pipe == PIPE_BF16 ? 2 * R : R;
  return (P + 256) * rb < (1ull << 31) && (Q + 256) * rb < (1ull << 31);
}

hipError_t launch_gemm_codes(float* out, const uint8_t* X, int kindX, const uint8_t* Z, int kindZ,
                             size_t P, size_t Q, size_t R, size_t pitch, int pipe, const GemmScale& s,
                             bool accumulate, void* workspace, hipStream_t stream, const SliceSum* carry,
                             SliceSum* defer, bool x_packed) {
  const SliceSumPlan ss{carry, defer};
  const size_t row_bytes = pipe == PIPE_BF16 ? 2 * R : R;
  const Plan pl = make_plan(P, Q, row_bytes);
  if (x_packed && !(pipe == PIPE_I8 && pl.tile == 0)) return hipErrorInvalidValue;  // see gemm_takes_packed_x
  GemmParams g;
  g.out = out;
  g.partial = static_cast<uint32_t*>(workspace);
  g.X = X; g.Z = Z;
  g.P = (uint32_t)P; g.Q = (uint32_t)Q; g.R = (uint32_t)row_bytes;
  g.pitch = (uint32_t)pitch;
  g.pitch_x = (uint32_t)(x_packed ? pitch / 2 : pitch);
  g.k_per_split = pl.k_per_split;
  g.nsplit = pl.nsplit;
  g.tiles_p = g.tiles_q = 0;
  g.alpha = s.alpha; g.sx = s.sx; g.sz = s.sz; g.sx_dev = s.sx_dev; g.sz_dev = s.sz_dev;
  g.accumulate = accumulate ? 1 : 0;
  if (x_packed) return launch_persist<I8Mma, true>(g, ss, stream);
  if (pipe == PIPE_I8) return launch_mma<I8Mma>(g, pl, ss, stream);
  if (pipe == PIPE_BF16) return launch_mma<BF16Mma>(g, pl, ss, stream);
  if (pipe == PIPE_F16C) return launch_mma<E5M2F16Mma>(g, pl, ss, stream);
  // the Z operand is the first MFMA operand, X the second
  const int fx = kindX == SRQ_E5M2, fz = kindZ == SRQ_E5M2;
  if (!fz && !fx) return launch_mma<F8Mma<0, 0>>(g, pl, ss, stream);
  if (!fz && fx) return launch_mma<F8Mma<0, 1>>(g, pl, ss, stream);
  if (fz && !fx) return launch_mma<F8Mma<1, 0>>(g, pl, ss, stream);
  return launch_mma<F8Mma<1, 1>>(g, pl, ss, stream);
}

hipError_t launch_slice_sum(const SliceSum& r, hipStream_t stream) {
  if (r.total == 0) return hipSuccess;
  splitk_reduce_kernel<<<slice_sum_blocks(r, 256, 4), 256, 0, stream>>>(r);
  return hipGetLastError();
}

}  // namespace srq
