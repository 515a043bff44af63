/*
 * CPU oracle for the QLoRA frozen-linear hot path -- see qlora_oracle.h.
 * TEST INFRASTRUCTURE ONLY: never linked into, imported by, or used as a
 * fallback for the HIP library.
 *
 * Build: g++ -O2 -std=c++17 -fopenmp -ffp-contract=off -shared -fPIC
 * (no -ffast-math, no -march flags: every operation below must be a plain
 * IEEE-754 binary32/binary64 operation).
 */
#include "qlora_oracle.h"

#include <cfloat>
#include <cmath>
#include <cstring>
#include <vector>
#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

/* ---- exactly rounded fp32 steps, evaluated through fp64 --------------------
 * For binary32 operands the fp64 result of one +, * or / rounded again to
 * binary32 equals the directly rounded binary32 result (53 >= 2*24 + 2). */
inline float fl32_mul(float a, float b) { return (float)((double)a * (double)b); }
inline float fl32_add(float a, float b) { return (float)((double)a + (double)b); }
inline float fl32_sub(float a, float b) { return (float)((double)a - (double)b); }
inline float fl32_div(float a, float b) { return (float)((double)a / (double)b); }

inline uint32_t f32_bits(float v) { uint32_t u; std::memcpy(&u, &v, 4); return u; }
inline float bits_f32(uint32_t u) { float v; std::memcpy(&v, &u, 4); return v; }
inline double bf16_to_f64(uint16_t b) { return (double)bits_f32((uint32_t)b << 16); }

/* Appendix E, index 0..15.  Each printed decimal is the shortest form of a
 * binary64 number that is exactly representable in binary32, so the
 * conversion to float loses nothing. */
const float kNF4[16] = {
    -1.0f,
    -0.6961928009986877f,
    -0.5250730514526367f,
    -0.39491748809814453f,
    -0.28444138169288635f,
    -0.18477343022823334f,
    -0.09105003625154495f,
    0.0f,
    0.07958029955625534f,
    0.16093020141124725f,
    0.24611230194568634f,
    0.33791524171829224f,
    0.44070982933044434f,
    0.5626170039176941f,
    0.7229568362236023f,
    1.0f,
};

/* value of an E4M3 magnitude code 0..0x7e: exponent field e, mantissa field m */
inline double e4m3_mag(int code7) {
  const int e = (code7 >> 3) & 15, m = code7 & 7;
  if (e == 0) return std::ldexp((double)m, -9);            /* subnormal: m/8 * 2^-6 */
  return std::ldexp(1.0 + (double)m / 8.0, e - 7);
}

}  // namespace

extern "C" {

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void oracle_nf4_table(float out[16]) {
  for (int i = 0; i < 16; ++i) out[i] = kNF4[i];
}

double oracle_normal_quantile(double p) {
  /* Phi(x) = erfc(-x / sqrt 2) / 2 is increasing; bisect Phi(x) = p. */
  if (!(p > 0.0 && p < 1.0)) return p <= 0.0 ? -HUGE_VAL : HUGE_VAL;
  double lo = -40.0, hi = 40.0;
  for (int it = 0; it < 200; ++it) {
    const double mid = 0.5 * (lo + hi);
    const double cdf = 0.5 * std::erfc(-mid / std::sqrt(2.0));
    if (cdf < p) lo = mid; else hi = mid;
  }
  return 0.5 * (lo + hi);
}

void oracle_nf4_derive(double p_max, double out[16]) {
  const double top = oracle_normal_quantile(p_max);
  /* negative half: 8 points, the first (p = 1/2) is the duplicate zero */
  for (int i = 1; i < 8; ++i) {
    const double p = 0.5 + (p_max - 0.5) * (double)i / 7.0;
    out[7 - i] = -oracle_normal_quantile(p) / top;
  }
  /* positive half: 9 points including the kept zero */
  for (int i = 0; i < 9; ++i) {
    const double p = 0.5 + (p_max - 0.5) * (double)i / 8.0;
    out[7 + i] = (i == 0) ? 0.0 : oracle_normal_quantile(p) / top;
  }
}

/* k-bit NormalFloat for k = 2, 3, 4 (Section 3, "4-bit NormalFloat Quantization": the construction is stated for
 * general k): 2^(k-1) evenly spaced probabilities from 1/2 to p_max give the negative side (the zero among them is
 * dropped), 2^(k-1) + 1 give the positive side, all quantiles divided by the top one: 2^k values with one exact zero.
 * The paper gives neither p_max nor a table for k != 4; the reading here is the tail mass that reproduces the printed
 * k = 4 table, written for general k:  1 - p_max = (1 / 2^(k+1) + 1 / (2^(k+1) - 2)) / 2.
 * out: the 2^k values ascending, then +1 repeated up to 16 entries (codes >= 2^k are never produced). */
int oracle_nfk_derive(int k, double out[16]) {
  if (!out) return -1;
  if (k < 2 || k > 4) return -2;
  const int n_neg = 1 << (k - 1), n_pos = n_neg + 1;
  const double two = (double)(1 << (k + 1));
  const double p_max = 1.0 - 0.5 * (1.0 / two + 1.0 / (two - 2.0));
  const double top = oracle_normal_quantile(p_max);
  for (int i = 1; i < n_neg; ++i) {
    const double p = 0.5 + (p_max - 0.5) * (double)i / (double)(n_neg - 1);
    out[n_neg - 1 - i] = -oracle_normal_quantile(p) / top;
  }
  for (int i = 0; i < n_pos; ++i) {
    const double p = 0.5 + (p_max - 0.5) * (double)i / (double)(n_pos - 1);
    out[n_neg - 1 + i] = (i == 0) ? 0.0 : oracle_normal_quantile(p) / top;
  }
  out[0] = -1.0;
  out[(1 << k) - 1] = 1.0;
  for (int i = 1 << k; i < 16; ++i) out[i] = 1.0;
  return 0;
}

/* Nearest value of a non-decreasing 16-entry table, the lower index on an exact tie:
 * the number of midpoints strictly below xhat. */
static int index_in(const float* table, float xhat) {
  int idx = 0;
  for (int j = 0; j < 15; ++j) {
    /* the midpoint of two binary32 numbers is exact in binary64 */
    const double mid = ((double)table[j] + (double)table[j + 1]) * 0.5;
    if ((double)xhat > mid) ++idx;
  }
  return idx;
}

int oracle_nf4_index(float xhat) { return index_in(kNF4, xhat); }

int oracle_index4(const float* table, float xhat) { return table ? index_in(table, xhat) : -1; }

/* The 4-bit data types the paper compares NF4 with (Section 4, the data-type table; Eq. 1 for the integer
 * type), as 16 values in [-1, 1] in ascending order.  The paper names the float formats and gives no value
 * table: each is enumerated here from its bit fields (sign, exponent, mantissa; exponent field 0 = subnormal,
 * no infinities or NaNs) and divided by its largest magnitude, which removes the exponent bias.  Both float
 * types have two zeros (entries 7 and 8); Int4 is round(7 x / absmax), 15 levels, entry 15 repeats the top. */
int oracle_codebook4(int kind, float out[16]) {
  if (!out) return -1;
  double mag[8];
  switch (kind) {
    case 0: for (int i = 0; i < 16; ++i) out[i] = kNF4[i]; return 0;
    case 1:                                            /* Float4 E2M1: e = 0: m/2;  e > 0: (1 + m/2) 2^(e-1) */
      for (int c = 0; c < 8; ++c) {
        const int e = c >> 1, m = c & 1;
        mag[c] = e == 0 ? 0.5 * m : std::ldexp(1.0 + 0.5 * m, e - 1);
      }
      break;
    case 2:                                            /* Float4 E3M0: e = 0: 0;  e > 0: 2^(e-1) */
      for (int c = 0; c < 8; ++c) mag[c] = c == 0 ? 0.0 : std::ldexp(1.0, c - 1);
      break;
    case 3:                                            /* Int4: j / 7, j = -7 .. 7 */
      for (int i = 0; i < 15; ++i) out[i] = (float)((double)(i - 7) / 7.0);
      out[15] = 1.0f;
      return 0;
    case 5: case 6: {                                  /* NF3, NF2: the derived quantiles, rounded once to fp32 */
      double d[16];
      if (oracle_nfk_derive(kind == 5 ? 3 : 2, d)) return -2;
      for (int i = 0; i < 16; ++i) out[i] = (float)d[i];
      return 0;
    }
    default: return -2;
  }
  for (int c = 0; c < 8; ++c) {
    const float v = (float)(mag[c] / mag[7]);
    out[8 + c] = v;
    out[7 - c] = -v;
  }
  out[7] = 0.0f;                                       /* the negative zero compares and multiplies as zero */
  return 0;
}

uint16_t oracle_bf16_rne(float v) {
  const uint32_t u = f32_bits(v);
  const uint32_t keep = u >> 16, rest = u & 0xffffu;
  uint32_t r = keep;
  if (rest > 0x8000u || (rest == 0x8000u && (keep & 1u))) r = keep + 1;  /* carry may bump the exponent */
  return (uint16_t)r;
}

float oracle_e4m3_value(uint8_t code) {
  const int mag = code & 0x7f;
  if (mag == 0x7f) return NAN;
  const double v = e4m3_mag(mag);
  return (float)((code & 0x80) ? -v : v);
}

float oracle_e4m3_unit(uint8_t code) {
  return fl32_div(oracle_e4m3_value(code), 448.0f);
}

uint8_t oracle_e4m3_encode(float z) {
  const double a = std::fabs((double)z);
  int best = 0;
  if (a >= 448.0) {
    best = 0x7e;                                   /* saturate */
  } else {
    double best_d = a;                             /* distance to code 0 */
    for (int c = 1; c <= 0x7e; ++c) {
      const double d = std::fabs(a - e4m3_mag(c));
      /* codes are in value order; on an exact tie keep the even one */
      if (d < best_d || (d == best_d && (c & 1) == 0)) { best_d = d; best = c; }
    }
  }
  if (best == 0) return 0;
  return (uint8_t)(best | (z < 0.0f ? 0x80 : 0));
}

/* ---- exact mean of n non-negative binary32 numbers -------------------------
 * Sum held as an unsigned big integer in units of 2^-149 (the binary32
 * subnormal spacing), then divided by n and rounded once to binary32. */
static float exact_mean_f32(const float* v, int64_t n) {
  const int L = 12;                                /* 384 bits >= 24 + 253 + 63 */
  uint32_t acc[L] = {0};
  for (int64_t i = 0; i < n; ++i) {
    const uint32_t u = f32_bits(v[i]) & 0x7fffffffu;
    uint32_t e = u >> 23;
    uint64_t m = u & 0x7fffffu;
    if (e == 0) e = 1; else m |= 0x800000u;
    const int sh = (int)e - 1;                     /* value = m * 2^(sh - 149) */
    const int limb = sh >> 5, off = sh & 31;
    uint64_t part = m << off;                      /* < 2^55 */
    uint64_t carry = 0;
    for (int k = limb; k < L; ++k) {
      const uint64_t t = (uint64_t)acc[k] + (part & 0xffffffffu) + carry;
      acc[k] = (uint32_t)t;
      carry = t >> 32;
      part >>= 32;
      if (part == 0 && carry == 0) break;
    }
  }
  /* long division by n (< 2^32 enforced by the caller) */
  uint32_t q[L];
  uint64_t rem = 0;
  for (int k = L - 1; k >= 0; --k) {
    const uint64_t cur = (rem << 32) | acc[k];
    q[k] = (uint32_t)(cur / (uint64_t)n);
    rem = cur % (uint64_t)n;
  }
  int top = -1;                                    /* index of the highest set bit of q */
  for (int k = L - 1; k >= 0 && top < 0; --k)
    if (q[k]) for (int b = 31; b >= 0; --b) if (q[k] >> b & 1u) { top = k * 32 + b; break; }
  auto bit = [&](int i) -> uint32_t { return i < 0 ? 0u : (q[i >> 5] >> (i & 31)) & 1u; };
  const int drop = top >= 24 ? top - 23 : 0;       /* low bits of q that do not fit in 24 */
  uint64_t kept = 0;
  for (int i = top; i >= drop; --i) kept = (kept << 1) | bit(i);
  /* discarded fraction = (low `drop` bits of q + rem/n) / 2^drop, compared with 1/2 */
  bool half, sticky;
  if (drop == 0) {
    half = 2 * rem >= (uint64_t)n;
    sticky = half ? (2 * rem > (uint64_t)n) : (rem != 0);
  } else {
    half = bit(drop - 1) != 0;
    sticky = rem != 0;
    for (int i = drop - 2; i >= 0 && !sticky; --i) sticky = bit(i) != 0;
  }
  if (half && (sticky || (kept & 1u))) ++kept;
  return (float)std::ldexp((double)kept, drop - 149);
}

static int quantize4(const float* table, const float* W, int64_t rows, int64_t cols,
                     int32_t blocksize, int32_t dq_blocksize,
                     uint8_t* packed, uint8_t* code, float* c1, float* mean,
                     float* c2_out) {
  if (!table || !W || !packed || !code || !c1 || !mean) return -1;
  if (rows <= 0 || cols <= 0 || blocksize <= 0 || dq_blocksize <= 0) return -2;
  const int64_t P = rows * cols;
  if (P % blocksize != 0 || P % 2 != 0) return -2;
  const int64_t n = P / blocksize;
  if (n >= ((int64_t)1 << 32)) return -2;
  for (int64_t i = 0; i < P; ++i) if (!std::isfinite(W[i])) return -3;

  std::vector<float> c2((size_t)n);
  std::vector<uint8_t> idx((size_t)P);
#pragma omp parallel for schedule(static)      /* blocks are independent */
  for (int64_t b = 0; b < n; ++b) {
    const float* w = W + b * blocksize;
    float amax = 0.0f;
    for (int i = 0; i < blocksize; ++i) amax = std::fmax(amax, std::fabs(w[i]));
    c2[(size_t)b] = amax;
    const float rc = (amax < FLT_MIN) ? 0.0f : fl32_div(1.0f, amax);   /* Eq. 1: c = range / absmax, range 1 */
    for (int i = 0; i < blocksize; ++i)
      idx[(size_t)(b * blocksize + i)] = (uint8_t)index_in(table, fl32_mul(w[i], rc));
  }
  for (int64_t i = 0; i < P / 2; ++i)
    packed[i] = (uint8_t)(idx[(size_t)(2 * i)] | (idx[(size_t)(2 * i + 1)] << 4));

  /* Double Quantization: the fp32 constants of the first step are the input */
  const float mu = exact_mean_f32(c2.data(), n);
  *mean = mu;
  const int64_t n1 = (n + dq_blocksize - 1) / dq_blocksize;
  for (int64_t B = 0; B < n1; ++B) {
    const int64_t lo = B * dq_blocksize;
    const int64_t hi = (lo + dq_blocksize < n) ? lo + dq_blocksize : n;
    float amax = 0.0f;
    for (int64_t b = lo; b < hi; ++b) amax = std::fmax(amax, std::fabs(fl32_sub(c2[(size_t)b], mu)));
    c1[B] = amax;
    float rc1 = (amax < FLT_MIN) ? 0.0f : fl32_div(448.0f, amax);
    if (!std::isfinite(rc1)) rc1 = 0.0f;
    for (int64_t b = lo; b < hi; ++b)
      code[b] = oracle_e4m3_encode(fl32_mul(fl32_sub(c2[(size_t)b], mu), rc1));
  }
  if (c2_out) std::memcpy(c2_out, c2.data(), (size_t)n * sizeof(float));
  return 0;
}

int oracle_nf4_quantize(const float* W, int64_t rows, int64_t cols,
                        int32_t blocksize, int32_t dq_blocksize,
                        uint8_t* packed, uint8_t* code, float* c1, float* mean,
                        float* c2_out) {
  return quantize4(kNF4, W, rows, cols, blocksize, dq_blocksize, packed, code, c1, mean, c2_out);
}

int oracle_quantize4(const float* table, const float* W, int64_t rows, int64_t cols,
                     int32_t blocksize, int32_t dq_blocksize,
                     uint8_t* packed, uint8_t* code, float* c1, float* mean,
                     float* c2_out) {
  return quantize4(table, W, rows, cols, blocksize, dq_blocksize, packed, code, c1, mean, c2_out);
}

static int dequant4(const float* table, const uint8_t* packed, const uint8_t* code, const float* c1,
                    float mean, int64_t rows, int64_t cols,
                    int32_t blocksize, int32_t dq_blocksize,
                    uint16_t* W_bf16, float* c2hat_out) {
  if (!table || !packed || !code || !c1 || !W_bf16) return -1;
  if (rows <= 0 || cols <= 0 || blocksize <= 0 || dq_blocksize <= 0) return -2;
  const int64_t P = rows * cols;
  if (P % blocksize != 0 || P % 2 != 0) return -2;
  const int64_t n = P / blocksize;
#pragma omp parallel for schedule(static)      /* blocks are independent */
  for (int64_t b = 0; b < n; ++b) {
    const float inner = fl32_mul(oracle_e4m3_unit(code[b]), c1[b / dq_blocksize]);   /* dequant(c1, c2) */
    const float c2hat = fl32_add(inner, mean);
    if (c2hat_out) c2hat_out[b] = c2hat;
    for (int i = 0; i < blocksize; ++i) {
      const int64_t e = b * blocksize + i;
      const int id = (packed[e >> 1] >> ((e & 1) * 4)) & 15;
      W_bf16[e] = oracle_bf16_rne(fl32_mul(table[id], c2hat));                         /* dequant(c2, W) */
    }
  }
  return 0;
}

/* ---- 8-bit integers: Eq. 1 and Eq. 2 as printed ------------------------------
 * Eq. 1:  X^Int8 = round(127 / absmax(X) * X) = round(c * X), per block of `blocksize` elements, with
 *         c = fl32(127 / absmax) (0 for an all-zero or subnormal block, or when the quotient overflows) and
 *         round = to nearest, ties to even, of the fp32 product fl32(c * x); the result lies in [-127, 127].
 * The constants absmax then go through Double Quantization exactly as for the 4-bit types (dq_blocksize = 0:
 * they are kept as fp32).
 * Eq. 2:  dequant(c, X^Int8) = X^Int8 / c = X^Int8 * absmax / 127, evaluated as
 *         w = bf16_rne(fl32(q * fl32(c2hat / 127))),  c2hat the (de-double-quantised) absmax of the block. */
static void dq_constants(const std::vector<float>& c2, int64_t n, int32_t dq_blocksize, uint8_t* code, float* c1,
                         float* mean) {
  const float mu = exact_mean_f32(c2.data(), n);
  *mean = mu;
  const int64_t n1 = (n + dq_blocksize - 1) / dq_blocksize;
  for (int64_t B = 0; B < n1; ++B) {
    const int64_t lo = B * dq_blocksize;
    const int64_t hi = (lo + dq_blocksize < n) ? lo + dq_blocksize : n;
    float amax = 0.0f;
    for (int64_t b = lo; b < hi; ++b) amax = std::fmax(amax, std::fabs(fl32_sub(c2[(size_t)b], mu)));
    c1[B] = amax;
    float rc1 = (amax < FLT_MIN) ? 0.0f : fl32_div(448.0f, amax);
    if (!std::isfinite(rc1)) rc1 = 0.0f;
    for (int64_t b = lo; b < hi; ++b)
      code[b] = oracle_e4m3_encode(fl32_mul(fl32_sub(c2[(size_t)b], mu), rc1));
  }
}

int oracle_quantize_int8(const float* W, int64_t rows, int64_t cols, int32_t blocksize, int32_t dq_blocksize,
                         int8_t* q8, uint8_t* code, float* c1, float* mean, float* c2_out) {
  if (!W || !q8 || !c2_out) return -1;
  if (dq_blocksize != 0 && (!code || !c1 || !mean)) return -1;
  if (rows <= 0 || cols <= 0 || blocksize <= 0 || dq_blocksize < 0) return -2;
  const int64_t P = rows * cols;
  if (P % blocksize != 0) return -2;
  const int64_t n = P / blocksize;
  for (int64_t i = 0; i < P; ++i) if (!std::isfinite(W[i])) return -3;
  std::vector<float> c2((size_t)n);
#pragma omp parallel for schedule(static)
  for (int64_t b = 0; b < n; ++b) {
    const float* w = W + b * blocksize;
    float amax = 0.0f;
    for (int i = 0; i < blocksize; ++i) amax = std::fmax(amax, std::fabs(w[i]));
    c2[(size_t)b] = amax;
    float c = (amax < FLT_MIN) ? 0.0f : fl32_div(127.0f, amax);
    if (!std::isfinite(c)) c = 0.0f;
    for (int i = 0; i < blocksize; ++i) {
      double v = std::nearbyint((double)fl32_mul(c, w[i]));    /* default rounding mode: ties to even */
      if (v > 127.0) v = 127.0;
      if (v < -127.0) v = -127.0;
      q8[b * blocksize + i] = (int8_t)v;
    }
  }
  std::memcpy(c2_out, c2.data(), (size_t)n * sizeof(float));
  if (dq_blocksize != 0) dq_constants(c2, n, dq_blocksize, code, c1, mean);
  return 0;
}

/* c2hat: the n reconstructed constants (oracle_nf4_dequant's c2hat_out, or c2 itself without Double Quantization) */
int oracle_dequant_int8(const int8_t* q8, const float* c2hat, int64_t rows, int64_t cols, int32_t blocksize,
                        uint16_t* W_bf16) {
  if (!q8 || !c2hat || !W_bf16) return -1;
  if (rows <= 0 || cols <= 0 || blocksize <= 0) return -2;
  const int64_t P = rows * cols;
  if (P % blocksize != 0) return -2;
#pragma omp parallel for schedule(static)
  for (int64_t e = 0; e < P; ++e) {
    const float step = fl32_div(c2hat[e / blocksize], 127.0f);
    W_bf16[e] = oracle_bf16_rne(fl32_mul((float)q8[e], step));
  }
  return 0;
}

/* the reconstructed constants alone: c2hat[b] = fl32(fl32(unit(code[b]) * c1[b / dq_blocksize]) + mean) */
int oracle_dq_constants(const uint8_t* code, const float* c1, float mean, int64_t n, int32_t dq_blocksize,
                        float* c2hat) {
  if (!code || !c1 || !c2hat) return -1;
  if (n <= 0 || dq_blocksize <= 0) return -2;
  for (int64_t b = 0; b < n; ++b)
    c2hat[b] = fl32_add(fl32_mul(oracle_e4m3_unit(code[b]), c1[b / dq_blocksize]), mean);
  return 0;
}

/* Without Double Quantization (Section 3: the constants then cost 32/64 = 0.5 bit per parameter): the fp32
 * constants c2 are used as they are, w_i = bf16_rne(fl32(table[idx_i] * c2[i / blocksize])). */
int oracle_dequant4_nodq(const float* table, const uint8_t* packed, const float* c2,
                         int64_t rows, int64_t cols, int32_t blocksize, uint16_t* W_bf16) {
  if (!table || !packed || !c2 || !W_bf16) return -1;
  if (rows <= 0 || cols <= 0 || blocksize <= 0) return -2;
  const int64_t P = rows * cols;
  if (P % blocksize != 0 || P % 2 != 0) return -2;
#pragma omp parallel for schedule(static)
  for (int64_t e = 0; e < P; ++e) {
    const int id = (packed[e >> 1] >> ((e & 1) * 4)) & 15;
    W_bf16[e] = oracle_bf16_rne(fl32_mul(table[id], c2[e / blocksize]));
  }
  return 0;
}

int oracle_nf4_dequant(const uint8_t* packed, const uint8_t* code, const float* c1,
                       float mean, int64_t rows, int64_t cols,
                       int32_t blocksize, int32_t dq_blocksize,
                       uint16_t* W_bf16, float* c2hat_out) {
  return dequant4(kNF4, packed, code, c1, mean, rows, cols, blocksize, dq_blocksize, W_bf16, c2hat_out);
}

int oracle_dequant4(const float* table, const uint8_t* packed, const uint8_t* code, const float* c1,
                    float mean, int64_t rows, int64_t cols,
                    int32_t blocksize, int32_t dq_blocksize,
                    uint16_t* W_bf16, float* c2hat_out) {
  return dequant4(table, packed, code, c1, mean, rows, cols, blocksize, dq_blocksize, W_bf16, c2hat_out);
}

/* ---- Eq. 5 / Eq. 3 and the backward products, fp64 triple loops ----------- */

static int check_lin(const void* a, const void* b, const void* out, int64_t M, int64_t h,
                     int64_t o, int64_t r, const uint16_t* L1, const uint16_t* L2) {
  if (!a || !b || !out) return -1;
  if (M <= 0 || h <= 0 || o <= 0 || r < 0) return -2;
  if (r > 0 && (!L1 || !L2)) return -1;
  return 0;
}

int oracle_linear_fwd(const uint16_t* X, const uint16_t* What,
                      const uint16_t* L1, const uint16_t* L2, double s,
                      int64_t M, int64_t h, int64_t o, int64_t r,
                      const int64_t* row_sel, int64_t n_sel, const double* D, double* Y) {
  if (int e = check_lin(X, What, Y, M, h, o, r, L1, L2)) return e;
  if (!row_sel) n_sel = M;
  for (int64_t i = 0; i < n_sel; ++i) { const int64_t m = row_sel ? row_sel[i] : i; if (m < 0 || m >= M) return -2; }
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t i = 0; i < n_sel; ++i) {
    const int64_t m = row_sel ? row_sel[i] : i;
    double* y = Y + i * o;
    for (int64_t n = 0; n < o; ++n) y[n] = 0.0;
    for (int64_t k = 0; k < h; ++k) {                       /* X What */
      const double x = bf16_to_f64(X[m * h + k]);
      const uint16_t* w = What + k * o;
      for (int64_t n = 0; n < o; ++n) y[n] += x * bf16_to_f64(w[n]);
    }
    std::vector<double> t((size_t)r, 0.0);                  /* T = (D o X) L1 */
    for (int64_t k = 0; k < h; ++k) {
      const double x = bf16_to_f64(X[m * h + k]) * (D ? D[m * h + k] : 1.0);
      for (int64_t j = 0; j < r; ++j) t[(size_t)j] += x * bf16_to_f64(L1[k * r + j]);
    }
    for (int64_t n = 0; n < o; ++n) {                       /* + s (T L2) */
      double acc = 0.0;
      for (int64_t j = 0; j < r; ++j) acc += t[(size_t)j] * bf16_to_f64(L2[j * o + n]);
      y[n] += s * acc;
    }
  }
  return 0;
}

int oracle_linear_fwd_cols(const uint16_t* X, const uint16_t* What,
                           const uint16_t* L1, const uint16_t* L2, double s,
                           int64_t M, int64_t h, int64_t o, int64_t r,
                           const int64_t* col_sel, int64_t n_sel, double* Y) {
  if (int e = check_lin(X, What, Y, M, h, o, r, L1, L2)) return e;
  if (!col_sel || n_sel <= 0) return -1;
  for (int64_t c = 0; c < n_sel; ++c) if (col_sel[c] < 0 || col_sel[c] >= o) return -2;
#pragma omp parallel for schedule(dynamic, 16)
  for (int64_t m = 0; m < M; ++m) {
    std::vector<double> t((size_t)r, 0.0);
    for (int64_t k = 0; k < h; ++k) {
      const double x = bf16_to_f64(X[m * h + k]);
      for (int64_t j = 0; j < r; ++j) t[(size_t)j] += x * bf16_to_f64(L1[k * r + j]);
    }
    for (int64_t c = 0; c < n_sel; ++c) {
      const int64_t n = col_sel[c];
      double acc = 0.0;
      for (int64_t k = 0; k < h; ++k) acc += bf16_to_f64(X[m * h + k]) * bf16_to_f64(What[k * o + n]);
      double lora = 0.0;
      for (int64_t j = 0; j < r; ++j) lora += t[(size_t)j] * bf16_to_f64(L2[j * o + n]);
      Y[m * n_sel + c] = acc + s * lora;
    }
  }
  return 0;
}

int oracle_linear_bwd_dx(const uint16_t* dY, const uint16_t* What,
                         const uint16_t* L1, const uint16_t* L2, double s,
                         int64_t M, int64_t h, int64_t o, int64_t r,
                         const int64_t* row_sel, int64_t n_sel, const double* D, double* dX) {
  if (int e = check_lin(dY, What, dX, M, h, o, r, L1, L2)) return e;
  if (!row_sel) n_sel = M;
  for (int64_t i = 0; i < n_sel; ++i) { const int64_t m = row_sel ? row_sel[i] : i; if (m < 0 || m >= M) return -2; }
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t i = 0; i < n_sel; ++i) {
    const int64_t m = row_sel ? row_sel[i] : i;
    const uint16_t* g = dY + m * o;
    std::vector<double> u((size_t)r, 0.0);                  /* U = dY L2^T */
    for (int64_t j = 0; j < r; ++j) {
      double acc = 0.0;
      for (int64_t n = 0; n < o; ++n) acc += bf16_to_f64(g[n]) * bf16_to_f64(L2[j * o + n]);
      u[(size_t)j] = acc;
    }
    for (int64_t k = 0; k < h; ++k) {
      const uint16_t* w = What + k * o;
      double acc = 0.0;                                     /* dY What^T */
      for (int64_t n = 0; n < o; ++n) acc += bf16_to_f64(g[n]) * bf16_to_f64(w[n]);
      double lora = 0.0;                                    /* U L1^T */
      for (int64_t j = 0; j < r; ++j) lora += u[(size_t)j] * bf16_to_f64(L1[k * r + j]);
      dX[i * h + k] = acc + s * (D ? D[m * h + k] : 1.0) * lora;   /* the branch saw D o X */
    }
  }
  return 0;
}

int oracle_linear_bwd_dx_cols(const uint16_t* dY, const uint16_t* What,
                              const uint16_t* L1, const uint16_t* L2, double s,
                              int64_t M, int64_t h, int64_t o, int64_t r,
                              const int64_t* col_sel, int64_t n_sel, double* dX) {
  if (int e = check_lin(dY, What, dX, M, h, o, r, L1, L2)) return e;
  if (!col_sel || n_sel <= 0) return -1;
  for (int64_t c = 0; c < n_sel; ++c) if (col_sel[c] < 0 || col_sel[c] >= h) return -2;
#pragma omp parallel for schedule(dynamic, 16)
  for (int64_t m = 0; m < M; ++m) {
    const uint16_t* g = dY + m * o;
    std::vector<double> u((size_t)r, 0.0);
    for (int64_t j = 0; j < r; ++j) {
      double acc = 0.0;
      for (int64_t n = 0; n < o; ++n) acc += bf16_to_f64(g[n]) * bf16_to_f64(L2[j * o + n]);
      u[(size_t)j] = acc;
    }
    for (int64_t c = 0; c < n_sel; ++c) {
      const int64_t k = col_sel[c];
      const uint16_t* w = What + k * o;
      double acc = 0.0;
      for (int64_t n = 0; n < o; ++n) acc += bf16_to_f64(g[n]) * bf16_to_f64(w[n]);
      double lora = 0.0;
      for (int64_t j = 0; j < r; ++j) lora += u[(size_t)j] * bf16_to_f64(L1[k * r + j]);
      dX[m * n_sel + c] = acc + s * lora;
    }
  }
  return 0;
}

int oracle_linear_bwd_dl(const uint16_t* dY, const uint16_t* X,
                         const uint16_t* L1, const uint16_t* L2, double s,
                         int64_t M, int64_t h, int64_t o, int64_t r,
                         const double* D, double* dL1, double* dL2) {
  if (!dY || !X || !L1 || !L2 || !dL1 || !dL2) return -1;
  if (M <= 0 || h <= 0 || o <= 0 || r <= 0) return -2;
  std::vector<double> U((size_t)(M * r)), T((size_t)(M * r));
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m) {
    for (int64_t j = 0; j < r; ++j) {                       /* U = dY L2^T */
      double acc = 0.0;
      for (int64_t n = 0; n < o; ++n) acc += bf16_to_f64(dY[m * o + n]) * bf16_to_f64(L2[j * o + n]);
      U[(size_t)(m * r + j)] = acc;
    }
    for (int64_t j = 0; j < r; ++j) T[(size_t)(m * r + j)] = 0.0;
    for (int64_t k = 0; k < h; ++k) {                       /* T = (D o X) L1 */
      const double x = bf16_to_f64(X[m * h + k]) * (D ? D[m * h + k] : 1.0);
      for (int64_t j = 0; j < r; ++j) T[(size_t)(m * r + j)] += x * bf16_to_f64(L1[k * r + j]);
    }
  }
#pragma omp parallel for schedule(static)
  for (int64_t k = 0; k < h; ++k) {                         /* dL1 = s (D o X)^T U */
    std::vector<double> acc((size_t)r, 0.0);
    for (int64_t m = 0; m < M; ++m) {
      const double x = bf16_to_f64(X[m * h + k]) * (D ? D[m * h + k] : 1.0);
      for (int64_t j = 0; j < r; ++j) acc[(size_t)j] += x * U[(size_t)(m * r + j)];
    }
    for (int64_t j = 0; j < r; ++j) dL1[k * r + j] = s * acc[(size_t)j];
  }
#pragma omp parallel for schedule(static)
  for (int64_t n = 0; n < o; ++n) {                         /* dL2 = s T^T dY */
    std::vector<double> acc((size_t)r, 0.0);
    for (int64_t m = 0; m < M; ++m) {
      const double g = bf16_to_f64(dY[m * o + n]);
      for (int64_t j = 0; j < r; ++j) acc[(size_t)j] += T[(size_t)(m * r + j)] * g;
    }
    for (int64_t j = 0; j < r; ++j) dL2[j * o + n] = s * acc[(size_t)j];
  }
  return 0;
}

}  // extern "C"
