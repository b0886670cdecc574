/*
 * srq_oracle.c -- plain, slow CPU oracle for the stochastic-rounding quantized
 * linear layer.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It exists to check the GPU library; it is
 * not a fallback for it.  Only the test-suite, the smoke check and the
 * benchmark's CPU-baseline leg may load it.  It shares no source, header,
 * table or constant generator with the GPU code.
 *
 * What it computes (paper sections in brackets):
 *   - the threshold quantization function Q_Delta(x, eps)        [Def. 1, Eq. 1]
 *   - round-to-nearest  = Q_Delta(x, 1/2), ties toward +inf       [Def. 2]
 *   - stochastic rounding = Q_Delta(x, eps), eps ~ U, one
 *     independent threshold per matrix element                    [Def. 3]
 *   - the mixed-precision product: exact product of the two
 *     quantized matrices, accumulated in high precision           [Sec. 2.2.2]
 *   - forward  A_out = Q(A) Q(W)                                  [Alg. 1]
 *   - backward dA = Q(dA_out) Q(W)^T, dW = Q(A)^T Q(dA_out)       [Alg. 2]
 *   - the weight update w <- Q_SR(w - eta * g) onto the bfloat16
 *     grid                                                         [Eq. 10]
 *
 * Points the paper leaves open (how Delta is chosen, number formats, the
 * random number generator, saturation) are fixed as follows and are the same
 * on the GPU side by specification, not by shared code:
 *   - Delta of a tensor is a per-tensor fp32 `scale`; the grid coordinate is
 *     t = fl32(x * fl32(1/scale)), clamped to +-Qmax of the format.
 *   - integer formats are the uniform grid of Eq. 1 with Delta = 1 in t;
 *     8-bit floating formats use the local spacing D of the target grid at t
 *     (one power of two per binade, subnormals share the smallest normal
 *     binade's spacing), i.e. Eq. 1 with Delta = D.
 *   - eps for element i is built from 16 random bits r16:
 *     eps = (r16 + 1/2) / 65536, so eps lies strictly inside (0, 1) and a
 *     value already on the grid (frac = 0) is never moved.
 *   - the bits come from Philox4x32-10 (Salmon et al., SC'11): block number
 *     counter_offset + floor(i / 8), counter words (lo, hi, 0, 0), key
 *     (seed lo, seed hi); element i takes 16-bit slice i mod 8 of the four
 *     output words, low half of word 0 first.
 *   - the grid coordinate t = fl32(x * fl32(1/scale)) is IEEE binary32 (one
 *     rounding per operation, no fused multiply-add): that is the precision
 *     the inputs and the GPU kernels work in.  From t on, Eq. 1 is evaluated
 *     exactly: t / D, its floor, its fractional part and the comparison with
 *     eps are taken in binary64, where each of them is exact (t has 24
 *     significant bits and |t / D| < 2^8; the one case that rounds, a
 *     fractional part within 2^-53 of 1, lies above every threshold either
 *     way).  Matrix products are accumulated exactly (int64) or in binary64.
 *
 *   - the weight update of Eq. 10 takes u = fl32(w - fl32(eta * g)) (two
 *     binary32 roundings, no fused multiply-add), clamps it to the largest
 *     finite bfloat16 and applies Eq. 1 on the bfloat16 grid (8 exponent
 *     bits, 7 fraction bits, subnormals with the spacing of the smallest
 *     normal binade) with the same thresholds eps = (r16 + 1/2) / 65536: the
 *     16 random bits face exactly the 16 fraction bits binary32 has beyond
 *     bfloat16.  NaN gives 0x7FC0, a zero result is +0.
 *
 * Pins (see tests/test_oracle_*.py): Random123 known-answer vectors for
 * Philox; the worked 0.7 example of Sec. 2.2.1; the closed-form count of
 * thresholds that round up; pass-through of grid points; two-neighbour and
 * error bounds of Lemma 1's proof; unbiasedness and the Bernoulli variance;
 * torch's float8 dtypes for the 8-bit float grids; numpy fp64 matmul for the
 * products; the variance formula in the proof of Lemma 3; for the bfloat16
 * update: pass-through of bfloat16 values, the count of thresholds that round
 * away from zero (= the 16 dropped bits), exact unbiasedness over all 65536
 * thresholds, and torch's float32 -> bfloat16 conversion for eps = 1/2 away
 * from ties.
 * Parity unpinned by the paper: the encodings of NaN/Inf inputs, negative
 * zero and saturation -- these are pinned only by the rules stated here.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { KIND_NONE = 0, KIND_INT8 = 1, KIND_INT4 = 2, KIND_E4M3 = 3, KIND_E5M2 = 4,
       KIND_E4M2 = 5, KIND_E4M1 = 6, KIND_E4M0 = 7 };
enum { ROUND_SR = 0, ROUND_RTN = 1 };
enum { SRC_F32 = 0, SRC_BF16 = 1 };

int srq_oracle_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void srq_oracle_set_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

/* ------------------------------------------------------------------ */
/* Eq. 1 in binary64, exactly as printed: the generic definition.      */
/* ------------------------------------------------------------------ */
double srq_oracle_Q(double x, double delta, double eps) {
  if (delta == 0.0) return x; /* note under Eq. 1 */
  double y = x / delta;
  double fl = floor(y);
  if (y - fl < eps) return delta * fl;
  /* floor(y + 1) = floor(y) + 1; written this way because y + 1 itself can
   * round up to an integer in finite precision (y = -1e-20) */
  return delta * (fl + 1.0);
}

/* ------------------------------------------------------------------ */
/* Philox4x32-10.                                                       */
/* ------------------------------------------------------------------ */
void srq_oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    if (round > 0) {
      k0 += 0x9E3779B9u; /* golden ratio */
      k1 += 0xBB67AE85u; /* sqrt(3) - 1  */
    }
    uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
    uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
    uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
    uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
    uint32_t n0 = hi1 ^ c1 ^ k0;
    uint32_t n1 = lo1;
    uint32_t n2 = hi0 ^ c3 ^ k1;
    uint32_t n3 = lo0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* 16 random bits of element i of a tensor quantized with (seed, counter_offset). */
uint32_t srq_oracle_r16(uint64_t seed, uint64_t counter_offset, uint64_t i) {
  uint64_t block = counter_offset + (i >> 3); /* wraps mod 2^64 */
  uint32_t ctr[4] = {(uint32_t)block, (uint32_t)(block >> 32), 0u, 0u};
  uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  uint32_t w[4];
  srq_oracle_philox4x32_10(ctr, key, w);
  unsigned j = (unsigned)(i & 7u);
  return (w[j >> 1] >> (16u * (j & 1u))) & 0xFFFFu;
}

/* Threshold eps in (0,1) from 16 bits; exact in binary32. */
float srq_oracle_eps_from_r16(uint32_t r16) {
  return ((float)r16 + 0.5f) * (1.0f / 65536.0f);
}

/* ------------------------------------------------------------------ */
/* Formats.                                                             */
/* ------------------------------------------------------------------ */
/* E4M2 / E4M1 / E4M0 (the 4-exponent-bit formats of the paper's experiments, Sec. 5): the
 * paper does not state their bias or subnormal rule; they are read here as sub-grids of
 * E4M3 -- same exponent range (bias 7, subnormals at the spacing of the smallest normal
 * binade), 2 / 1 / 0 fraction bits -- and their codes are stored as the E4M3 code of the
 * same value (the low 1 / 2 / 3 fraction bits zero). */
static int kind_is_float(int kind) { return kind >= KIND_E4M3 && kind <= KIND_E4M0; }
static int kind_mbits(int kind) {
  switch (kind) {
    case KIND_E4M3: return 3;
    case KIND_E4M1: return 1;
    case KIND_E4M0: return 0;
    default: return 2; /* E5M2, E4M2 */
  }
}
static int kind_bias(int kind) { return kind == KIND_E5M2 ? 15 : 7; }
/* the format whose byte encoding the codes use */
static int kind_storage(int kind) { return kind >= KIND_E4M2 && kind <= KIND_E4M0 ? KIND_E4M3 : kind; }

float srq_oracle_qmax(int kind) {
  switch (kind) {
    case KIND_INT8: return 127.0f;
    case KIND_INT4: return 7.0f;
    case KIND_E4M3: return 448.0f;   /* 1.75 * 2^8  */
    case KIND_E5M2: return 57344.0f; /* 1.75 * 2^15 */
    case KIND_E4M2: return 448.0f;   /* 1.75 * 2^8: the E4M3 maximum has only two fraction bits set */
    case KIND_E4M1: return 384.0f;   /* 1.5  * 2^8  */
    case KIND_E4M0: return 256.0f;   /* 2^8         */
    default: return 0.0f;
  }
}

/* Value of a code, in grid units (multiply by scale for the real value).
 * Integer codes are two's complement (int4 codes are held sign-extended in a
 * byte when unpacked).  The 8-bit floats follow the OCP definitions: sign,
 * biased exponent, mantissa; exponent field 0 is subnormal; E4M3 has no
 * infinities and a single NaN mantissa pattern (all ones), E5M2 is IEEE-like. */
double srq_oracle_decode(int kind, uint8_t code) {
  if (!kind_is_float(kind)) return (double)(int8_t)code;
  kind = kind_storage(kind);
  int m = kind_mbits(kind), bias = kind_bias(kind);
  int sign = code >> 7;
  int efield = (code & 0x7F) >> m;
  int mant = code & ((1 << m) - 1);
  int emax_field = (1 << (7 - m)) - 1;
  double v;
  if (kind == KIND_E4M3) {
    if (efield == emax_field && mant == 7) return NAN;
  } else {
    if (efield == emax_field) return mant == 0 ? (sign ? -INFINITY : INFINITY) : NAN;
  }
  if (efield == 0)
    v = ldexp((double)mant / (double)(1 << m), 1 - bias);
  else
    v = ldexp(1.0 + (double)mant / (double)(1 << m), efield - bias);
  return sign ? -v : v;
}

/* Code of a value that is known to lie on the format's grid (finite). */
static uint8_t encode_on_grid(int kind, float v) {
  if (!kind_is_float(kind)) return (uint8_t)(int8_t)(int)v;
  if (v == 0.0f) return 0; /* +0 also for results that came from negatives */
  kind = kind_storage(kind);
  int m = kind_mbits(kind), bias = kind_bias(kind);
  int sign = v < 0.0f;
  float a = fabsf(v);
  int ex;
  (void)frexpf(a, &ex); /* a = fr * 2^ex, fr in [1/2, 1) */
  int e = ex - 1;       /* a = 1.xxx * 2^e                */
  int efield, mant;
  if (e < 1 - bias) {
    efield = 0;
    mant = (int)(a / ldexpf(1.0f, 1 - bias - m));
  } else {
    efield = e + bias;
    mant = (int)((a / ldexpf(1.0f, e) - 1.0f) * (float)(1 << m));
  }
  return (uint8_t)((sign << 7) | (efield << m) | mant);
}

/* One element: source value x (already widened to binary32), inv = fl32(1/scale),
 * threshold eps.  Returns the code byte (int4: sign-extended in the byte). */
uint8_t srq_oracle_quantize_one(float x, float inv, int kind, float eps) {
  if (isnan(x)) return kind_is_float(kind) ? 0x7F : 0;
  float qm = srq_oracle_qmax(kind);
  float t = x * inv; /* grid coordinate, one rounding */
  if (t > qm) t = qm;
  if (t < -qm) t = -qm;
  float D = 1.0f; /* spacing of the grid at t */
  if (kind_is_float(kind)) {
    int m = kind_mbits(kind), emin = 1 - kind_bias(kind);
    int e = emin;
    if (t != 0.0f) {
      int ex;
      (void)frexpf(fabsf(t), &ex);
      e = ex - 1; /* floor(log2 |t|) */
      if (e < emin) e = emin;
    }
    D = ldexpf(1.0f, e - m);
  }
  /* Eq. 1 with Delta = D, evaluated exactly (binary64) on the binary32 coordinate t */
  double y = (double)t / (double)D; /* exact: D is a power of two */
  double fl = floor(y);
  double frac = y - fl;
  double qd = (frac < (double)eps) ? fl : fl + 1.0; /* floor(y + 1) = floor(y) + 1 */
  float q = (float)qd;                              /* a small integer */
  return encode_on_grid(kind, q * D);
}

static float widen(const void* src, int src_dtype, size_t i) {
  if (src_dtype == SRC_BF16) {
    uint32_t bits = (uint32_t)((const uint16_t*)src)[i] << 16;
    float f;
    memcpy(&f, &bits, 4);
    return f;
  }
  return ((const float*)src)[i];
}

/* Tensor quantizer: codes[i] (one byte per element, unpacked) for i in [0, n). */
void srq_oracle_quantize(uint8_t* codes, const void* x, int src_dtype, size_t n, int kind,
                         int round_mode, float scale, uint64_t seed, uint64_t counter_offset) {
  float inv = 1.0f / scale;
#pragma omp parallel for schedule(static)
  for (long long i = 0; i < (long long)n; ++i) {
    float eps = 0.5f;
    if (round_mode == ROUND_SR)
      eps = srq_oracle_eps_from_r16(srq_oracle_r16(seed, counter_offset, (uint64_t)i));
    codes[i] = srq_oracle_quantize_one(widen(x, src_dtype, (size_t)i), inv, kind, eps);
  }
}

/* Eq. 1 on the bfloat16 grid for one binary32 value u and threshold eps; returns the
 * bfloat16 bit pattern. */
uint16_t srq_oracle_sr_bf16_one(float u, float eps) {
  if (isnan(u)) return 0x7FC0;
  const float bf16_max = 3.3895313892515355e38f; /* (2 - 2^-7) * 2^127 */
  if (u > bf16_max) u = bf16_max;
  if (u < -bf16_max) u = -bf16_max;
  int e = -126;
  if (u != 0.0f) {
    int ex;
    (void)frexpf(fabsf(u), &ex);
    e = ex - 1; /* floor(log2 |u|) */
    if (e < -126) e = -126;
  }
  double D = ldexp(1.0, e - 7); /* spacing of the bfloat16 grid at u */
  double y = (double)u / D;     /* exact; |y| < 2^8 */
  double fl = floor(y);
  double frac = y - fl;
  double qd = (frac < (double)eps) ? fl : fl + 1.0;
  float v = (float)(qd * D); /* on the bfloat16 grid, hence exact in binary32 */
  if (v == 0.0f) return 0;
  uint32_t bits;
  memcpy(&bits, &v, 4);
  return (uint16_t)(bits >> 16); /* the low 16 bits are zero */
}

/* Eq. 10 for a tensor: w[i] <- Q_SR(w[i] - eta * g[i]) on the bfloat16 grid, in place.
 * Element i uses the same 16-bit slice of the Philox stream as the quantizers. */
void srq_oracle_update_bf16(uint16_t* w, const float* g, float eta, size_t n, int round_mode,
                            uint64_t seed, uint64_t counter_offset) {
#pragma omp parallel for schedule(static)
  for (long long i = 0; i < (long long)n; ++i) {
    float eps = 0.5f;
    if (round_mode == ROUND_SR)
      eps = srq_oracle_eps_from_r16(srq_oracle_r16(seed, counter_offset, (uint64_t)i));
    float step = eta * g[i];                       /* one rounding */
    float u = widen(w, SRC_BF16, (size_t)i) - step; /* one rounding */
    w[i] = srq_oracle_sr_bf16_one(u, eps);
  }
}

/* int4 storage: element 2k in bits 3:0 and element 2k+1 in bits 7:4 of byte k;
 * n must be even. */
void srq_oracle_pack_int4(uint8_t* packed, const uint8_t* codes, size_t n) {
  for (size_t k = 0; k < n / 2; ++k)
    packed[k] = (uint8_t)((codes[2 * k] & 0xF) | ((codes[2 * k + 1] & 0xF) << 4));
}

void srq_oracle_unpack_int4(uint8_t* codes, const uint8_t* packed, size_t n) {
  for (size_t k = 0; k < n / 2; ++k) {
    int lo = packed[k] & 0xF, hi = packed[k] >> 4;
    codes[2 * k] = (uint8_t)(int8_t)(lo >= 8 ? lo - 16 : lo);
    codes[2 * k + 1] = (uint8_t)(int8_t)(hi >= 8 ? hi - 16 : hi);
  }
}

/* Per-tensor scale = max|x| / Qmax over the finite elements; 1 if that is 0.  The paper leaves
 * Delta open; this choice of it is floored at 2^-100, the smallest step the quantizer accepts
 * (below it 1 / Delta scaled by 2^16 leaves binary32): a tensor of vanishing values, such as an
 * underflowing gradient, is then quantized on the grid of step 2^-100 (to zeros, or to its
 * nearest neighbours), not saturated. */
float srq_oracle_absmax_scale(const void* x, int src_dtype, size_t n, int kind) {
  float amax = 0.0f;
  for (size_t i = 0; i < n; ++i) {
    float a = fabsf(widen(x, src_dtype, i));
    if (isfinite(a) && a > amax) amax = a;
  }
  if (amax == 0.0f) return 1.0f;
  float s = amax / srq_oracle_qmax(kind);
  return s < 0x1p-100f ? 0x1p-100f : s;
}

/* ------------------------------------------------------------------ */
/* Products of quantized matrices (Sec. 2.2.2, Alg. 1 and 2).          */
/* Codes are unpacked, row-major.  Integer pairs accumulate in int64,  */
/* anything else in binary64 (each product of two 8-bit floats is      */
/* exact there).  out = fl32( fl32(sx*sz) * sum ).  abs_out, when not   */
/* NULL, receives fl32(sx*sz) * sum |x z| for tolerance checks.        */
/* ------------------------------------------------------------------ */
static double dot_codes(const uint8_t* x, size_t sx, int kx, const uint8_t* z, size_t sz, int kz,
                        size_t len, double* abs_sum) {
  if (!kind_is_float(kx) && !kind_is_float(kz)) {
    int64_t acc = 0, aacc = 0;
    for (size_t r = 0; r < len; ++r) {
      int64_t p = (int64_t)(int8_t)x[r * sx] * (int64_t)(int8_t)z[r * sz];
      acc += p;
      aacc += p < 0 ? -p : p;
    }
    if (abs_sum) *abs_sum = (double)aacc;
    return (double)acc;
  }
  double acc = 0.0, aacc = 0.0;
  for (size_t r = 0; r < len; ++r) {
    double p = srq_oracle_decode(kx, x[r * sx]) * srq_oracle_decode(kz, z[r * sz]);
    acc += p;
    aacc += fabs(p);
  }
  if (abs_sum) *abs_sum = aacc;
  return acc;
}

static void store(float* out, float* abs_out, size_t idx, double s, double acc, double aacc) {
  out[idx] = (float)(s * acc);
  if (abs_out) abs_out[idx] = (float)(s * aacc);
}

/* Alg. 1:  Y[m][n] = sum_k Ahat[m][k] What[n][k]   (W held as out x in) */
void srq_oracle_fwd(float* Y, float* abs_out, const uint8_t* A, int kA, float sA, const uint8_t* W,
                    int kW, float sW, size_t M, size_t N, size_t K) {
  double s = (double)(sA * sW);
#pragma omp parallel for schedule(static)
  for (long long m = 0; m < (long long)M; ++m)
    for (size_t n = 0; n < N; ++n) {
      double aacc;
      double acc = dot_codes(A + (size_t)m * K, 1, kA, W + n * K, 1, kW, K, &aacc);
      store(Y, abs_out, (size_t)m * N + n, s, acc, aacc);
    }
}

/* Alg. 2:  dA[m][k] = sum_n dYhat[m][n] What[n][k] */
void srq_oracle_bwd_data(float* dA, float* abs_out, const uint8_t* dY, int kdY, float sdY,
                         const uint8_t* W, int kW, float sW, size_t M, size_t N, size_t K) {
  double s = (double)(sdY * sW);
#pragma omp parallel for schedule(static)
  for (long long m = 0; m < (long long)M; ++m)
    for (size_t k = 0; k < K; ++k) {
      double aacc;
      double acc = dot_codes(dY + (size_t)m * N, 1, kdY, W + k, K, kW, N, &aacc);
      store(dA, abs_out, (size_t)m * K + k, s, acc, aacc);
    }
}

/* Alg. 2:  dW[n][k] = sum_m dYhat[m][n] Ahat[m][k] */
void srq_oracle_bwd_weight(float* dW, float* abs_out, const uint8_t* dY, int kdY, float sdY,
                           const uint8_t* A, int kA, float sA, size_t M, size_t N, size_t K) {
  double s = (double)(sdY * sA);
#pragma omp parallel for schedule(static)
  for (long long n = 0; n < (long long)N; ++n)
    for (size_t k = 0; k < K; ++k) {
      double aacc;
      double acc = dot_codes(dY + (size_t)n, N, kdY, A + k, K, kA, M, &aacc);
      store(dW, abs_out, (size_t)n * K + k, s, acc, aacc);
    }
}

/* The same three products at a list of output positions (flat row-major
 * indices into the output), for shapes too large to compute in full. */
void srq_oracle_fwd_at(float* out, float* abs_out, const uint64_t* idx, size_t count,
                       const uint8_t* A, int kA, float sA, const uint8_t* W, int kW, float sW,
                       size_t M, size_t N, size_t K) {
  (void)M;
  double s = (double)(sA * sW);
#pragma omp parallel for schedule(static)
  for (long long j = 0; j < (long long)count; ++j) {
    size_t m = idx[j] / N, n = idx[j] % N;
    double aacc;
    double acc = dot_codes(A + m * K, 1, kA, W + n * K, 1, kW, K, &aacc);
    store(out, abs_out, (size_t)j, s, acc, aacc);
  }
}

void srq_oracle_bwd_data_at(float* out, float* abs_out, const uint64_t* idx, size_t count,
                            const uint8_t* dY, int kdY, float sdY, const uint8_t* W, int kW,
                            float sW, size_t M, size_t N, size_t K) {
  (void)M;
  double s = (double)(sdY * sW);
#pragma omp parallel for schedule(static)
  for (long long j = 0; j < (long long)count; ++j) {
    size_t m = idx[j] / K, k = idx[j] % K;
    double aacc;
    double acc = dot_codes(dY + m * N, 1, kdY, W + k, K, kW, N, &aacc);
    store(out, abs_out, (size_t)j, s, acc, aacc);
  }
}

void srq_oracle_bwd_weight_at(float* out, float* abs_out, const uint64_t* idx, size_t count,
                              const uint8_t* dY, int kdY, float sdY, const uint8_t* A, int kA,
                              float sA, size_t M, size_t N, size_t K) {
  double s = (double)(sdY * sA);
#pragma omp parallel for schedule(static)
  for (long long j = 0; j < (long long)count; ++j) {
    size_t n = idx[j] / K, k = idx[j] % K;
    double aacc;
    double acc = dot_codes(dY + n, N, kdY, A + k, K, kA, M, &aacc);
    store(out, abs_out, (size_t)j, s, acc, aacc);
  }
}
