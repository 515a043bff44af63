// Device-side building blocks shared by the gfx950 kernels of the QLoRA linear path:
// the NF4 table (Appendix E of arXiv 2305.14314), nearest-value thresholds, the
// 8-bit-float (OCP E4M3) encode/decode used by Double Quantization (Section 3),
// bf16 helpers and wave-level reductions.  gfx950 only: wave64, MFMA, 160 KB LDS.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace qlora {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;   // plain 16-byte vector (usable in LDS)

constexpr int kBlock = 64;      // first-level blocksize (Section 3, after Eq. 6)
constexpr int kDqBlock = 256;   // second-level blocksize
constexpr float kF8Max = 448.0f;  // largest finite E4M3 magnitude

// The 16 values of the NF4 data type, index 0..15 (Appendix E).
#define QLORA_NF4_VALUES                                                                         \
  -1.0f, -0.6961928009986877f, -0.5250730514526367f, -0.39491748809814453f,                      \
  -0.28444138169288635f, -0.18477343022823334f, -0.09105003625154495f, 0.0f,                     \
  0.07958029955625534f, 0.16093020141124725f, 0.24611230194568634f, 0.33791524171829224f,        \
  0.44070982933044434f, 0.5626170039176941f, 0.7229568362236023f, 1.0f

__host__ __device__ constexpr float nf4_value(int i) {
  constexpr float t[16] = {QLORA_NF4_VALUES};
  return t[i];
}

// Decision threshold between index j and j+1: the midpoint of the two values
// rounded toward -infinity to fp32, so that for fp32 x  (x > threshold) holds
// exactly when x lies strictly above the real midpoint (ties go to the lower index).
__host__ __device__ constexpr float nf4_threshold(int j) {
  const double mid = ((double)nf4_value(j) + (double)nf4_value(j + 1)) * 0.5;   // exact
  float t = (float)mid;
  if ((double)t > mid) {
    uint32_t u = __builtin_bit_cast(uint32_t, t);
    u = (t > 0.0f) ? u - 1 : u + 1;          // next fp32 toward -infinity (t is never 0 here)
    t = __builtin_bit_cast(float, u);
  }
  return t;
}

// Nearest NF4 index of a normalised value: 4-level binary search over the 15 thresholds.
__host__ __device__ __forceinline__ uint32_t nf4_index_search(float x) {
  constexpr float t0 = nf4_threshold(0), t1 = nf4_threshold(1), t2 = nf4_threshold(2), t3 = nf4_threshold(3),
                  t4 = nf4_threshold(4), t5 = nf4_threshold(5), t6 = nf4_threshold(6), t7 = nf4_threshold(7),
                  t8 = nf4_threshold(8), t9 = nf4_threshold(9), t10 = nf4_threshold(10),
                  t11 = nf4_threshold(11), t12 = nf4_threshold(12), t13 = nf4_threshold(13),
                  t14 = nf4_threshold(14);
  const bool b3 = x > t7;
  const float ta = b3 ? t11 : t3;
  const bool b2 = x > ta;
  const float tb = b3 ? (b2 ? t13 : t9) : (b2 ? t5 : t1);
  const bool b1 = x > tb;
  const float tc = b3 ? (b2 ? (b1 ? t14 : t12) : (b1 ? t10 : t8)) : (b2 ? (b1 ? t6 : t4) : (b1 ? t2 : t0));
  const bool b0 = x > tc;
  return ((uint32_t)b3 << 3) | ((uint32_t)b2 << 2) | ((uint32_t)b1 << 1) | (uint32_t)b0;
}

// The same index in ~7 operations: the range is cut into 32 buckets of width 1/16,
// bucket(x) = clamp(floor(16 x) + 16, 0, 31) (16 x is exact, so the bucket edges are exact).  Neighbouring
// thresholds are at least 0.0805 > 1/16 apart, so a bucket holds at most one threshold: the index is the
// number of thresholds below the bucket plus one comparison against the bucket's own threshold.
struct Nf4Bucket { float thr; uint32_t base; };
__host__ __device__ constexpr Nf4Bucket nf4_bucket(int b) {
  const float lo = (float)(b - 16) / 16.0f, hi = (float)(b - 15) / 16.0f;     // exact
  uint32_t base = 0;
  float thr = __builtin_huge_valf();                        // no threshold inside: the comparison is always false
  int inside = 0;
  for (int j = 0; j < 15; ++j) {
    const float t = nf4_threshold(j);
    if (b > 0 && t < lo) ++base;                              // below the whole bucket (bucket 0 extends to -inf)
    else if (b == 31 || t < hi) { thr = t; ++inside; }        // bucket 31 extends to +inf
  }
  // more than one threshold in a bucket would break the scheme; base = 99 makes any test fail loudly
  return inside > 1 ? Nf4Bucket{thr, 99u} : Nf4Bucket{thr, base};
}
__host__ __device__ constexpr bool nf4_buckets_ok() {
  for (int b = 0; b < 32; ++b) if (nf4_bucket(b).base > 15u) return false;
  return true;
}
static_assert(nf4_buckets_ok(), "an NF4 bucket holds more than one decision threshold");

// Bucket number of a normalised value (shared by the device lookup and the host-side check).
__host__ __device__ __forceinline__ int nf4_bucket_of(float x) {
  int k = (int)__builtin_floorf(x * 16.0f) + 16;
  k = k < 0 ? 0 : k;
  return k > 31 ? 31 : k;
}
// Host/device reference of the bucket scheme with the table recomputed on the fly (slow; for checks).
__host__ __device__ inline uint32_t nf4_index_bucket_ref(float x) {
  const Nf4Bucket e = nf4_bucket(nf4_bucket_of(x));
  return e.base + (x > e.thr ? 1u : 0u);
}
// Device lookup: `table` is the 32-entry (threshold, base) table in LDS, 256 bytes = one pass over the
// 64 LDS banks, so lanes reading different entries never collide and equal entries broadcast.
__device__ __forceinline__ void nf4_bucket_table_init(Nf4Bucket* table /* LDS, 256-byte aligned */, int tid) {
  if (tid < 32) table[tid] = nf4_bucket(tid);
}
__device__ __forceinline__ uint32_t nf4_index(float x, const Nf4Bucket* table) {
  const Nf4Bucket e = table[nf4_bucket_of(x)];
  return e.base + (x > e.thr ? 1u : 0u);
}

// ---- the other 4-bit data types of the paper's comparison (Section 4) --------------------------
// Int4 (Eq. 1 with the range [-7, 7]), Float4 E2M1 and Float4 E3M0 go through the same blockwise scheme as NF4:
// only the 16-value table differs.  The paper prints no tables for the float types; they are the values of the bit
// fields (sign, exponent, mantissa; exponent field 0 = subnormal, no infinities or NaNs) divided by the largest
// magnitude, which removes the exponent bias.  Tables are ascending; the float types hold zero twice (entries 7, 8),
// Int4 has 15 levels and repeats the top one.  Thresholds are built as for NF4: midpoint rounded toward -infinity.
// data type ids: 0 NF4, 1 Float4 E2M1, 2 Float4 E3M0, 3 Int4
// 8-bit integers (Eq. 1 and Eq. 2 as printed: q = round(127 / absmax * x), x^ = q * absmax / 127): one signed byte
// per weight, no table; the constants absmax are stored like those of the 4-bit types.
constexpr int kTypeInt8 = 4;
// k-bit NormalFloat for k = 3 and 2 (Section 3 states the construction for general k): 2^k values in a 16-entry table
// whose tail repeats +1, stored in the 4-bit containers of the other types (codes >= 2^k never occur).
constexpr int kTypeNF3 = 5, kTypeNF2 = 6;
constexpr int kNumTypes = 7;
inline bool is_table_type(int dtype) { return dtype >= 0 && dtype < kNumTypes && dtype != kTypeInt8; }
struct Table4 { float v[16]; };
struct Thresholds4 { float t[15]; };

// Standard normal quantile for 1/2 <= p < 1 (host): Newton's iteration on Phi(x) = p from x = 0.  Phi is increasing
// and concave on x >= 0, so the iterates rise monotonically to the root and converge quadratically.
inline double normal_quantile_upper_host(double p) {
  double x = 0.0;
  for (int it = 0; it < 60; ++it) {
    const double cdf = 0.5 * __builtin_erfc(-x * 0.70710678118654752440);
    const double pdf = 0.39894228040143267794 * __builtin_exp(-0.5 * x * x);
    const double dx = (p - cdf) / pdf;
    x += dx;
    if (__builtin_fabs(dx) < 1e-16 * (1.0 + x)) break;
  }
  return x;
}

// NFk: 2^(k-1) evenly spaced probabilities from 1/2 to p_max on the negative side (the zero is dropped), 2^(k-1) + 1
// on the positive side, quantiles divided by the top one.  The paper gives no p_max; the tail mass
// (1 / 2^(k+1) + 1 / (2^(k+1) - 2)) / 2 is the one that reproduces its printed 4-bit table.
inline Table4 nfk_table_host(int k) {
  Table4 tab{};
  const int n_neg = 1 << (k - 1), n_pos = n_neg + 1, n = 1 << k;
  const double two = (double)(2 * n);
  const double p_max = 1.0 - 0.5 * (1.0 / two + 1.0 / (two - 2.0));
  const double top = normal_quantile_upper_host(p_max);
  for (int i = 1; i < n_neg - 1; ++i)
    tab.v[n_neg - 1 - i] = (float)(-normal_quantile_upper_host(0.5 + (p_max - 0.5) * (double)i / (double)(n_neg - 1)) / top);
  for (int i = 1; i < n_pos - 1; ++i)
    tab.v[n_neg - 1 + i] = (float)(normal_quantile_upper_host(0.5 + (p_max - 0.5) * (double)i / (double)(n_pos - 1)) / top);
  tab.v[0] = -1.0f;
  tab.v[n_neg - 1] = 0.0f;
  for (int i = n - 1; i < 16; ++i) tab.v[i] = 1.0f;
  return tab;
}

inline Table4 table4_host(int dtype) {
  Table4 tab{};
  if (dtype == kTypeNF3 || dtype == kTypeNF2) {              // derived once per process, not per launch
    static const Table4 nf3 = nfk_table_host(3), nf2 = nfk_table_host(2);
    return dtype == kTypeNF3 ? nf3 : nf2;
  }
  if (dtype == 0 || dtype == kTypeInt8) {        // Int8 reads no table
    for (int i = 0; i < 16; ++i) tab.v[i] = nf4_value(i);
  } else if (dtype == 3) {
    for (int i = 0; i < 15; ++i) tab.v[i] = (float)((double)(i - 7) / 7.0);
    tab.v[15] = 1.0f;
  } else {
    const double e2m1[8] = {0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0};
    const double e3m0[8] = {0.0, 1.0, 2.0, 4.0, 8.0, 16.0, 32.0, 64.0};
    const double* mag = dtype == 1 ? e2m1 : e3m0;
    for (int c = 0; c < 8; ++c) {
      const float v = (float)(mag[c] / mag[7]);
      tab.v[8 + c] = v;
      tab.v[7 - c] = c == 0 ? 0.0f : -v;
    }
  }
  return tab;
}

inline Thresholds4 thresholds4_host(const Table4& tab) {
  Thresholds4 th{};
  for (int j = 0; j < 15; ++j) {
    const double mid = ((double)tab.v[j] + (double)tab.v[j + 1]) * 0.5;       // exact
    float t = (float)mid;
    if ((double)t > mid) t = __builtin_nextafterf(t, -__builtin_huge_valf());
    th.t[j] = t;
  }
  return th;
}

// Nearest-value index for thresholds known only at run time: binary search over the 15 non-decreasing thresholds
// kept in LDS (`t`, 16 floats; selects between elements of a by-value argument would become a lane-indexed read
// of it, i.e. scratch memory).  Returns the number of thresholds strictly below x.
__device__ __forceinline__ uint32_t index_search4(float x, const float* t) {
  uint32_t lo = 0;
#pragma unroll
  for (uint32_t step = 8; step >= 1; step >>= 1)
    if (x > t[lo + step - 1]) lo += step;
  return lo;
}

// ---- bf16 ------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {   // RNE, lo in bits 15:0
  bf16x2 v;
  v[0] = (__bf16)lo;
  v[1] = (__bf16)hi;
  return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ uint16_t bf16_bits(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }
__device__ __forceinline__ float bf16_lo_to_f32(uint32_t pair) { return __builtin_bit_cast(float, pair << 16); }
__device__ __forceinline__ float bf16_hi_to_f32(uint32_t pair) { return __builtin_bit_cast(float, pair & 0xffff0000u); }

// ---- 8-bit float (OCP E4M3: 1-4-3, bias 7, no infinities, max 448) ---------------------------
// Exact value of a code (codes 0x7f / 0xff are NaN and never produced by the encoder).
__device__ __forceinline__ float e4m3_value(uint32_t code) {
  const uint32_t e = (code >> 3) & 15u, m = code & 7u;
  float mag = e ? __builtin_bit_cast(float, ((e + 120u) << 23) | (m << 20)) : (float)m * 0x1p-9f;
  return (code & 0x80u) ? -mag : mag;
}
// Decode-table entry used by doubleDequant: value / 448 as one correctly rounded fp32 division.
__device__ __forceinline__ float e4m3_unit(uint32_t code) { return __fdiv_rn(e4m3_value(code), kF8Max); }

// Storage position of the 8-bit constant of block `blk` (0 .. bpr-1) of row `row`: column-group-major, groups of
// 4 blocks (256 columns), the last group possibly narrower.  The double-quantisation runs are NOT permuted:
// block row * bpr + blk still belongs to c1[(row * bpr + blk) / 256].
__device__ __forceinline__ int64_t code_pos(int64_t rows, int bpr, int64_t row, int blk) {
  const int G = blk >> 2;
  const int w = (4 * G + 4 <= bpr) ? 4 : bpr - 4 * G;
  return (int64_t)4 * rows * G + row * w + (blk & 3);
}

// Round-to-nearest-even onto the E4M3 grid, saturating at +-448; a zero result is always 0x00.
__device__ __forceinline__ uint32_t e4m3_encode(float z) {
  const float a = __builtin_fabsf(z);
  uint32_t code;
  if (a >= kF8Max) {
    code = 0x7eu;
  } else if (a < 0x1p-6f) {
    code = (uint32_t)__builtin_rintf(a * 512.0f);          // subnormal grid 2^-9; 8 -> 0x08 = 2^-6
  } else {
    const uint32_t u = __builtin_bit_cast(uint32_t, a);
    const uint32_t r = u + 0x7ffffu + ((u >> 20) & 1u);      // RNE at mantissa bit 20, carry into exponent
    code = (r >> 20) - (120u << 3);
  }
  return (code != 0u && z < 0.0f) ? (code | 0x80u) : code;
}

// ---- wave-level helpers ----------------------------------------------------------------------
// max over aligned groups of 16 lanes (a DPP row); every lane of the row gets the result.
__device__ __forceinline__ float row16_max(float v) {
  int x = __builtin_bit_cast(int, v);
  // quad_perm [1,0,3,2], quad_perm [2,3,0,1], row_half_mirror, row_mirror
  v = __builtin_fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(x, 0xB1, 0xF, 0xF, true)));
  x = __builtin_bit_cast(int, v);
  v = __builtin_fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(x, 0x4E, 0xF, 0xF, true)));
  x = __builtin_bit_cast(int, v);
  v = __builtin_fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(x, 0x141, 0xF, 0xF, true)));
  x = __builtin_bit_cast(int, v);
  v = __builtin_fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(x, 0x140, 0xF, 0xF, true)));
  return v;
}
// max over the whole wave64; every lane gets the result.
__device__ __forceinline__ float wave_max(float v) {
  v = row16_max(v);
  v = __builtin_fmaxf(v, __shfl_xor(v, 16));
  v = __builtin_fmaxf(v, __shfl_xor(v, 32));
  return v;
}

}  // namespace qlora
