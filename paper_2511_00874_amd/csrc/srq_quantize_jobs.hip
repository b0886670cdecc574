// Several tensor quantizations in ONE launch, for the linear entry points: the operands of a
// product (and, in the fused backward pass, the output gradient in both layouts at once) are
// independent element-wise jobs (Def. 3), so one grid serves them all and every tensor is
// read once.  A workgroup first finds its job, then runs the same-layout or the transposing
// path for that job's format; format, source dtype and rounding mode are uniform per
// workgroup, so the dispatch is scalar branches.
#include <cstddef>
#include <type_traits>

#include "srq_device.hpp"
#include "srq_internal.hpp"

namespace srq {
namespace {

constexpr int QBLOCK = 256;
constexpr int TC = 64;                  // transposing tile: tile_rows source rows x TC source columns
// Tile rows: 128, or 256 for one-byte codes of a tensor large enough to give every CU several such
// tiles (the same 16.6 KB of LDS as 128 rows of bfloat16 values).  A workgroup then writes 256 bytes
// of every transposed row (128 where two 4-bit values share a byte): whole cache lines.  Small
// tensors keep 128 rows: twice the workgroups (GPT-2 sizes lose 4 % of their step with 256).
__host__ __device__ inline int tile_rows(bool as_bf16, uint32_t rows, uint32_t cols) {
  return !as_bf16 && (size_t)((rows + 255u) / 256u) * ((cols + TC - 1) / TC) >= 2048u ? 256 : 128;
}
constexpr size_t STREAM_OUT_BYTES = 64u << 20;
constexpr int BAND_GROUP = 32;         // row bands whose tiles are walked together (tile order)
static_assert(BAND_GROUP % 8 == 0, "neighbouring column tiles of a band on one XCD");
constexpr int FLAT_GROUPS_PER_BLOCK = QBLOCK * 4;  // sixteen 512-element chunks: four per wave (measured best of 1, 2, 4, 8)

template <int KIND, bool AS_BF16>
__device__ __forceinline__ void job_quantize_group(uint32_t (&c)[8], const float (&v)[8], const InvScale& inv,
                                                   const QuantJob& j, uint64_t ctr, uint64_t g, uint32_t k0,
                                                   uint32_t k1) {
  if (j.round == SRQ_SR) quantize_group<KIND, SRQ_SR, AS_BF16>(c, v, inv, ctr + g, k0, k1);
  else quantize_group<KIND, SRQ_RTN, AS_BF16>(c, v, inv, 0, 0, 0);
}

__device__ __forceinline__ void job_load_group(float (&v)[8], const QuantJob& j, size_t g, size_t n) {
  if (j.dtype == SRQ_F32) load_group<SRQ_F32>(v, j.x, g, n);
  else load_group<SRQ_BF16>(v, j.x, g, n);
}

// 8 codes of one group to a row-major destination (elements base .. base+7, all in range)
template <bool AS_BF16>
__device__ __forceinline__ void store_group(uint8_t* out, size_t base, const uint32_t (&c)[8]) {
  if constexpr (AS_BF16) {
    u32x4 w = {c[0] | (c[1] << 16), c[2] | (c[3] << 16), c[4] | (c[5] << 16), c[6] | (c[7] << 16)};
    *reinterpret_cast<u32x4*>(reinterpret_cast<uint16_t*>(out) + base) = w;
  } else {
    const uint32_t lo[4] = {c[0], c[1], c[2], c[3]}, hi[4] = {c[4], c[5], c[6], c[7]};
    u32x2 w = {pack4_bytes(lo), pack4_bytes(hi)};
    *reinterpret_cast<u32x2*>(out + base) = w;
  }
}

// same layout as the source; rows * cols is a multiple of 8 for the linear entry points.
// binary32 sources go chunk-wise (one fully coalesced 512-element chunk per wave at a time),
// what is left over, and bfloat16 sources, group-wise.
template <int KIND, bool AS_BF16>
__device__ __forceinline__ void flat_path(const QuantJob& j, uint32_t local, uint32_t nblocks) {
  const InvScale inv = inv_scale(j.scale, j.scale_dev, j.kind);
  const uint64_t ctr = first_block(j.counter_offset, j.counter_dev);
  const uint32_t k0 = (uint32_t)j.seed, k1 = (uint32_t)(j.seed >> 32);
  const size_t n = (size_t)j.rows * j.cols, ngroups = n / 8;
  size_t first_group = 0;
  if (j.dtype == SRQ_F32) {
    const size_t nchunks = n / CHUNK, waves = (size_t)nblocks * (QBLOCK / 64);
    const float* x = static_cast<const float*>(j.x);
    for (size_t c = (size_t)local * (QBLOCK / 64) + (threadIdx.x >> 6); c < nchunks; c += waves) {
      if (j.round == SRQ_SR)
        quantize_chunk_f32<KIND, SRQ_SR, AS_BF16 ? 2 : 0>(j.out, x, c, threadIdx.x & 63u, inv, k0, k1, ctr);
      else
        quantize_chunk_f32<KIND, SRQ_RTN, AS_BF16 ? 2 : 0>(j.out, x, c, threadIdx.x & 63u, inv, k0, k1, ctr);
    }
    first_group = nchunks * (CHUNK / 8);
  }
  for (size_t g = first_group + (size_t)local * QBLOCK + threadIdx.x; g < ngroups; g += (size_t)nblocks * QBLOCK) {
    float v[8];
    uint32_t c[8];
    job_load_group(v, j, g, n);
    job_quantize_group<KIND, AS_BF16>(c, v, inv, j, ctr, g, k0, k1);
    store_group<AS_BF16>(j.out, g * 8, c);
  }
}

// transposed output (cols x rows), optionally a same-layout output as well (out2): the same
// codes, or those of a second (integer) quantizer of the same values
template <int KIND, bool AS_BF16, int TR>
__device__ __forceinline__ void transpose_path(const QuantJob& j, uint32_t local, uint8_t* smem) {
  using elem_t = typename std::conditional<AS_BF16, uint16_t, uint8_t>::type;
  constexpr int ES = sizeof(elem_t);
  constexpr int PITCH = TR + 4 / ES;
  elem_t* tile = reinterpret_cast<elem_t*>(smem);
  const InvScale inv = inv_scale(j.scale, j.scale_dev, j.kind);
  const InvScale inv2 = j.out2 && j.kind2 ? inv_scale(j.scale2, j.scale_dev2, j.kind2) : inv;
  const uint64_t ctr = first_block(j.counter_offset, j.counter_dev);
  const uint64_t ctr2 = j.out2 && j.kind2 ? first_block(j.counter_offset2, j.counter_dev2) : 0ull;
  const uint32_t k0 = (uint32_t)j.seed, k1 = (uint32_t)(j.seed >> 32);
  // Tile order: bands of TR source rows in groups of BAND_GROUP; inside a group the band index runs
  // fastest, then the column tile.  Workgroups that run together then write BAND_GROUP * TR
  // consecutive elements of every transposed row between them, and still read each source row in
  // neighbouring pieces.
  const uint32_t tiles_x = (j.cols + TC - 1) / TC, tiles_y = (j.rows + TR - 1) / TR;
  const uint32_t group = local / (BAND_GROUP * tiles_x), within = local % (BAND_GROUP * tiles_x);
  const uint32_t bands = min((uint32_t)BAND_GROUP, tiles_y - group * BAND_GROUP);
  const uint32_t r0 = (group * BAND_GROUP + within % bands) * TR, c0 = (within / bands) * TC;
  const uint32_t rows = j.rows, cols = j.cols;
  const size_t n = (size_t)rows * cols;
  if (j.dtype == SRQ_F32) {
    // 16 lanes x 16 bytes cover the 64 columns of one tile row: a wave loads 4 rows per
    // instruction, fully used lines.  A lane holds a quad (half a Philox group) of row rA and
    // one of row rA + 64; the even lane of a pair draws the block of the first group, the odd
    // lane the block of the second, and they trade two words (as in quantize_chunk_f32).
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const bool odd = lane & 1u;
    const uint32_t cq = (lane & 15u) * 4;                    // first column of the quad in the tile
    const float* x = static_cast<const float*>(j.x);
    // The output in the source layout leaves in pieces of 64 bytes of a row (32 where two values share a
    // byte): half cache lines, completed by the workgroup of the next column tile, which the tile
    // order puts on the same XCD (BAND_GROUP is a multiple of 8).  For a large tensor plain stores
    // let that L2 put the halves together and leave the codes where the product that reads them
    // next looks first (13.15 -> 13.02 ms per step of the Llama-shaped layer; streaming stores:
    // 13.36); small ones keep the write-through form (GPT-2 sizes: 4 us per step better).
    const bool big = (size_t)rows * cols > STREAM_OUT_BYTES;
    auto put4 = [&](void* p, uint32_t v) {
      if (big) *reinterpret_cast<uint32_t*>(p) = v;
      else store_through4(p, v);
    };
    auto put8 = [&](void* p, const u32x2& v) {
      if (big) *reinterpret_cast<u32x2*>(p) = v;
      else store_through8(p, v);
    };
#pragma unroll
    for (int it = 0; it < TR / 32; ++it) {
      const uint32_t rA = it * 16 + wave * 4 + (lane >> 4), rB = rA + TR / 2;
      const uint32_t col = c0 + cq;
      const bool okA = r0 + rA < rows && col < cols, okB = r0 + rB < rows && col < cols;
      const size_t eA = (size_t)(r0 + rA) * cols + col, eB = (size_t)(r0 + rB) * cols + col;
      f32x4 a = {0.f, 0.f, 0.f, 0.f}, b = {0.f, 0.f, 0.f, 0.f};
      if (okA) a = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(x + eA));
      if (okB) b = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(x + eB));
      uint32_t addA[4], addB[4];
      if (j.round == SRQ_SR) {
        uint32_t w[4];
        philox_block(ctr + (odd ? eB : eA) / 8, k0, k1, w);
        const uint32_t nb0 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w[0], 0xB1, 0xF, 0xF, true);
        const uint32_t nb1 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w[1], 0xB1, 0xF, 0xF, true);
        const uint32_t nb2 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w[2], 0xB1, 0xF, 0xF, true);
        const uint32_t nb3 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w[3], 0xB1, 0xF, 0xF, true);
        sr_addends(odd ? nb2 : w[0], odd ? nb3 : w[1], addA);
        sr_addends(odd ? w[2] : nb0, odd ? w[3] : nb1, addB);
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) addA[e] = addB[e] = RTN_ADDEND;
      }
      uint32_t ca[4], cb[4];
      if (j.round == SRQ_SR) {
        quantize_quad<KIND, SRQ_SR, AS_BF16>(ca, a.x, a.y, a.z, a.w, inv, addA);
        quantize_quad<KIND, SRQ_SR, AS_BF16>(cb, b.x, b.y, b.z, b.w, inv, addB);
      } else {
        quantize_quad<KIND, SRQ_RTN, AS_BF16>(ca, a.x, a.y, a.z, a.w, inv, addA);
        quantize_quad<KIND, SRQ_RTN, AS_BF16>(cb, b.x, b.y, b.z, b.w, inv, addB);
      }
      if (j.out2 && j.kind2 == 0) {
        if constexpr (AS_BF16) {
          uint16_t* o = reinterpret_cast<uint16_t*>(j.out2);
          if (okA) put8(o + eA, u32x2{ca[0] | (ca[1] << 16), ca[2] | (ca[3] << 16)});
          if (okB) put8(o + eB, u32x2{cb[0] | (cb[1] << 16), cb[2] | (cb[3] << 16)});
        } else if (KIND == SRQ_INT4 && j.pack_2) {
          // two values per byte: four lanes hold a run of 16 columns (cols % 16 == 0: whole runs);
          // byte j of its 8 takes element j in the low and element j + 8 in the high nibble, so the
          // lanes with elements 0-7 take the nibbles of the lane two further on and write 4 bytes each
          const uint32_t na = pack4_bytes(ca) & 0x0F0F0F0Fu, nb = pack4_bytes(cb) & 0x0F0F0F0Fu;
          const uint32_t pa = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)na, 0x4E, 0xF, 0xF, true);
          const uint32_t pb = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)nb, 0x4E, 0xF, 0xF, true);
          if (!(lane & 2u)) {
            if (okA) put4(j.out2 + (eA >> 1) + 2u * (lane & 1u), na | (pa << 4));
            if (okB) put4(j.out2 + (eB >> 1) + 2u * (lane & 1u), nb | (pb << 4));
          }
        } else {
          if (okA) put4(j.out2 + eA, pack4_bytes(ca));
          if (okB) put4(j.out2 + eB, pack4_bytes(cb));
        }
      } else if (j.out2) {
        // the second quantizer: its own thresholds (same pairing of lanes and Philox blocks)
        uint32_t add2A[4], add2B[4], da[4], db[4];
        if (j.round2 == SRQ_SR) {
          uint32_t w[4];
          philox_block(ctr2 + (odd ? eB : eA) / 8, (uint32_t)j.seed2, (uint32_t)(j.seed2 >> 32), w);
          const uint32_t nb0 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w[0], 0xB1, 0xF, 0xF, true);
          const uint32_t nb1 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w[1], 0xB1, 0xF, 0xF, true);
          const uint32_t nb2 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w[2], 0xB1, 0xF, 0xF, true);
          const uint32_t nb3 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w[3], 0xB1, 0xF, 0xF, true);
          sr_addends(odd ? nb2 : w[0], odd ? nb3 : w[1], add2A);
          sr_addends(odd ? w[2] : nb0, odd ? w[3] : nb1, add2B);
          quantize_quad<SRQ_INTX, SRQ_SR, false>(da, a.x, a.y, a.z, a.w, inv2, add2A);
          quantize_quad<SRQ_INTX, SRQ_SR, false>(db, b.x, b.y, b.z, b.w, inv2, add2B);
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) add2A[e] = add2B[e] = RTN_ADDEND;
          quantize_quad<SRQ_INTX, SRQ_RTN, false>(da, a.x, a.y, a.z, a.w, inv2, add2A);
          quantize_quad<SRQ_INTX, SRQ_RTN, false>(db, b.x, b.y, b.z, b.w, inv2, add2B);
        }
        if (okA) put4(j.out2 + eA, pack4_bytes(da));
        if (okB) put4(j.out2 + eB, pack4_bytes(db));
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        tile[(cq + e) * PITCH + rA] = (elem_t)(okA ? ca[e] : 0u);
        tile[(cq + e) * PITCH + rB] = (elem_t)(okB ? cb[e] : 0u);
      }
    }
  } else {
#pragma unroll
    for (int it = 0; it < (TR * TC / 8) / QBLOCK; ++it) {
      const uint32_t id = it * QBLOCK + threadIdx.x;
      const uint32_t gc = id % (TC / 8), r = id / (TC / 8);
      const uint32_t row = r0 + r, col = c0 + gc * 8;
      uint32_t c[8] = {0, 0, 0, 0, 0, 0, 0, 0};
      if (row < rows && col < cols) {
        const size_t g = ((size_t)row * cols + col) / 8;
        float v[8];
        job_load_group(v, j, g, n);
        job_quantize_group<KIND, AS_BF16>(c, v, inv, j, ctr, g, k0, k1);
        if (j.out2 && j.kind2 == 0) {
          store_group<AS_BF16>(j.out2, g * 8, c);
        } else if (j.out2) {
          uint32_t c2[8];
          if (j.round2 == SRQ_SR)
            quantize_group<SRQ_INTX, SRQ_SR, false>(c2, v, inv2, ctr2 + g, (uint32_t)j.seed2,
                                                    (uint32_t)(j.seed2 >> 32));
          else
            quantize_group<SRQ_INTX, SRQ_RTN, false>(c2, v, inv2, 0, 0, 0);
          store_group<false>(j.out2, g * 8, c2);
        }
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) tile[(gc * 8 + e) * PITCH + r] = (elem_t)c[e];
    }
  }
  // The transposed output of a large tensor goes out with streaming stores (it is far bigger than the
  // caches and the write-through form left the wide gradients at 1 TB/s: 65536 x 5632, 450 -> 355 us);
  // a small one with write-through stores, which leave it in the last-level cache for the product
  // that reads it next (GPT-2 sizes: a few us per step).
  const bool stream_out = (size_t)j.rows * j.cols * ES > STREAM_OUT_BYTES;
  __syncthreads();
#pragma unroll
  for (int it = 0; it < (TC * TR / 16) / QBLOCK; ++it) {
    const uint32_t id = it * QBLOCK + threadIdx.x;
    const uint32_t ch = id % (TR / 16), c = id / (TR / 16);
    const uint32_t col = c0 + c, row = r0 + ch * 16;
    if (col >= cols || row >= rows) continue;  // rows % 16 == 0 for the linear entry points
    const uint32_t* src = reinterpret_cast<const uint32_t*>(&tile[c * PITCH + ch * 16]);
    if (KIND == SRQ_INT4 && !AS_BF16 && j.pack_t) {
      // two values per byte along the transposed row: byte j of 8 = elements j and j + 8 of the 16
      const uint32_t m = 0x0F0F0F0Fu;
      const u32x2 w = {(src[0] & m) | ((src[2] & m) << 4), (src[1] & m) | ((src[3] & m) << 4)};
      uint8_t* const dst = j.out + (((size_t)col * rows + row) >> 1);
      if (stream_out) __builtin_nontemporal_store(w, reinterpret_cast<u32x2*>(dst));
      else store_through8(dst, w);
      continue;
    }
    elem_t* dst = reinterpret_cast<elem_t*>(j.out) + (size_t)col * rows + row;
#pragma unroll
    for (int i = 0; i < ES; ++i) {
      const u32x4 w = {src[4 * i], src[4 * i + 1], src[4 * i + 2], src[4 * i + 3]};
      if (stream_out) __builtin_nontemporal_store(w, reinterpret_cast<u32x4*>(dst) + i);
      else store_through16(reinterpret_cast<u32x4*>(dst) + i, w);
    }
  }
}

template <int KIND, bool AS_BF16>
__device__ __forceinline__ void run_job(const QuantJob& j, uint32_t local, uint8_t* smem) {
  if (j.transpose) {
    if constexpr (AS_BF16) {
      transpose_path<KIND, true, 128>(j, local, smem);
    } else {
      if (tile_rows(false, j.rows, j.cols) == 256) transpose_path<KIND, false, 256>(j, local, smem);
      else transpose_path<KIND, false, 128>(j, local, smem);
    }
  }
  else flat_path<KIND, AS_BF16>(j, local, j.nblocks);
}

__global__ __launch_bounds__(QBLOCK) void quantize_jobs_kernel(QuantJobs jobs) {
  __shared__ __attribute__((aligned(16))) uint8_t smem[TC * (128 + 2) * 2];
  static_assert(TC * (256 + 4) <= (int)sizeof(smem), "the tile of 256 rows of bytes fits as well");
  int ji = 0;
#pragma unroll
  for (int i = 1; i < QUANT_JOBS_MAX; ++i)
    if (i < jobs.njobs && blockIdx.x >= jobs.job[i].first_block) ji = i;
  // The job descriptor is workgroup-uniform.  Indexing the by-value argument with ji would make
  // the compiler copy the whole argument to per-lane scratch memory; instead the one descriptor
  // is read from the kernel-argument segment (constant address space, scalar loads), where the
  // explicit arguments start at offset 0.
  struct alignas(8) Raw { uint32_t w[sizeof(QuantJob) / 4]; } raw;
  static_assert(sizeof(QuantJob) % 4 == 0 && offsetof(QuantJobs, job) % 4 == 0, "descriptor is read word-wise");
  typedef __attribute__((address_space(4))) const uint32_t* kernarg_words;
  const kernarg_words kw = (kernarg_words)__builtin_amdgcn_kernarg_segment_ptr() +
                           (offsetof(QuantJobs, job) + (size_t)ji * sizeof(QuantJob)) / 4;
#pragma unroll
  for (unsigned k = 0; k < sizeof(QuantJob) / 4; ++k) raw.w[k] = kw[k];
  const QuantJob j = __builtin_bit_cast(QuantJob, raw);
  const uint32_t local = blockIdx.x - j.first_block;
  const bool bf = j.store == STORE_BF16;
  switch (j.kind) {
    case SRQ_INT8: run_job<SRQ_INT8, false>(j, local, smem); break;
    case SRQ_INT4: run_job<SRQ_INT4, false>(j, local, smem); break;
    case SRQ_E4M3:
      if (bf) run_job<SRQ_E4M3, true>(j, local, smem);
      else run_job<SRQ_E4M3, false>(j, local, smem);
      break;
    case SRQ_E5M2:
      if (bf) run_job<SRQ_E5M2, true>(j, local, smem);
      else run_job<SRQ_E5M2, false>(j, local, smem);
      break;
    default:  // E4M2 / E4M1 / E4M0
      if (bf) run_job<SRQ_E4MX, true>(j, local, smem);
      else run_job<SRQ_E4MX, false>(j, local, smem);
      break;
  }
}

}  // namespace

// Requirements (checked by the callers): rows % 16 == 0 and cols % 16 == 0 for every job,
// store is STORE_BYTE or STORE_BF16 (STORE_BF16 only with E4M3 / E5M2).
hipError_t launch_quantize_jobs(QuantJobs& jobs, hipStream_t stream) {
  uint32_t first = 0;
  for (int i = 0; i < jobs.njobs; ++i) {
    QuantJob& j = jobs.job[i];
    size_t nb;
    if (j.transpose) {
      const size_t tr = tile_rows(j.store == STORE_BF16, j.rows, j.cols);
      nb = (size_t)((j.cols + TC - 1) / TC) * ((j.rows + tr - 1) / tr);
    } else {
      const size_t groups = (size_t)j.rows * j.cols / 8;
      nb = (groups + FLAT_GROUPS_PER_BLOCK - 1) / FLAT_GROUPS_PER_BLOCK;
      if (nb > (1u << 20)) nb = 1u << 20;
    }
    j.first_block = first;
    j.nblocks = (uint32_t)nb;
    first += (uint32_t)nb;
  }
  if (first == 0) return hipSuccess;
  quantize_jobs_kernel<<<first, QBLOCK, 0, stream>>>(jobs);
  return hipGetLastError();
}

}  // namespace srq
