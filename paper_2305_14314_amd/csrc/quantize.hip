// Blockwise NF4 quantisation with Double Quantization (arXiv 2305.14314, Eq. 1 and Section 3).
//
// Four launches on the caller's stream, no host synchronisation:
//   zero_bins      clears the 256 exponent bins used for the exact mean
//   quantize_nf4   per 64-block: absmax (DPP row reduce), reciprocal, nearest NF4 index (32-bucket table
//                  in LDS plus one comparison), nibble pack;
//                  writes the fp32 constant c2 to scratch and adds it to the exponent bins
//   dq_mean        exact sum of all c2 from the bins, divided by n, rounded once to fp32
//   dq_encode      per run of 256 constants: c2 - mean, absmax -> c1, E4M3 codes
//
// The mean is exact and independent of summation order: every fp32 constant is
// mantissa * 2^(exponent), the mantissas are summed per exponent in 64-bit integers
// (integer atomics commute), and the bins are combined in multi-word integer arithmetic.
#include <mutex>

#include "common.hpp"
#include "launch.hpp"

namespace qlora {

// Loads in flight: kQUnroll float4 per lane, kQWgsPerCu workgroups per CU (grid-stride beyond that).  Measured on
// 8192 x 22016 tensors read cold (GB/s of algorithmic bytes): unroll x workgroups 2 x 6 and 3 x 4: 4.42 - 4.45;
// 1 x 6: 4.40; 2 x 8: 4.28; 4 x 16 (the first choice): 4.06; 2 x 32: 3.83 -- past ~48 KB in flight per CU more requests
// only queue up in front of the memory channels.
#ifndef QL_Q_UNROLL
#define QL_Q_UNROLL 2
#endif
#ifndef QL_Q_WGS_PER_CU
#define QL_Q_WGS_PER_CU 6
#endif
constexpr int kQThreads = 256;
constexpr int kQUnroll = QL_Q_UNROLL;

__global__ void zero_bins_kernel(unsigned long long* bins) { bins[threadIdx.x] = 0ull; }

// One float4 per lane per step; 16 consecutive lanes hold one 64-block.
// MODE 0: NF4.  1: one of the other 4-bit data types (Section 4); its decision thresholds arrive as an argument.
// 2: 8-bit integers, Eq. 1 as printed: q = round_to_nearest_even(fl32(127 / absmax) * x), one signed byte per weight.
template <int MODE>
__global__ __launch_bounds__(kQThreads) void quantize_nf4_kernel(
    const float4* __restrict__ W, int64_t n_vec4,          // n_vec4 = elements / 4
    void* __restrict__ packed,                             // one store per lane: 4 nibbles (16 bit) or 4 bytes
    float* __restrict__ c2_out, unsigned long long* __restrict__ bins, const Thresholds4 thr) {
  constexpr bool OTHER = MODE == 1;
  __shared__ unsigned long long lbins[256];
  __shared__ __attribute__((aligned(256))) Nf4Bucket buckets[32];
  __shared__ float th[16];
  lbins[threadIdx.x] = 0ull;
  nf4_bucket_table_init(buckets, threadIdx.x);
  if (OTHER && threadIdx.x == 0) {
#pragma unroll
    for (int j = 0; j < 15; ++j) th[j] = thr.t[j];
  }
  __syncthreads();

  // kQUnroll independent float4 loads are issued before any is used.
  const int64_t stride = (int64_t)gridDim.x * kQThreads;
  for (int64_t v0 = (int64_t)blockIdx.x * kQThreads + threadIdx.x; v0 < n_vec4; v0 += kQUnroll * stride) {
    float4 wv[kQUnroll];
#pragma unroll
    for (int u = 0; u < kQUnroll; ++u) {
      const int64_t v = v0 + u * stride;
      wv[u] = W[v < n_vec4 ? v : v0];                        // clamped: no branch around the load
    }
#pragma unroll
    for (int u = 0; u < kQUnroll; ++u) {
      const int64_t v = v0 + u * stride;
      if (v >= n_vec4) break;                                 // whole 16-lane rows drop out together
      const float4 w = wv[u];
      float amax = __builtin_fmaxf(__builtin_fmaxf(__builtin_fabsf(w.x), __builtin_fabsf(w.y)),
                                   __builtin_fmaxf(__builtin_fabsf(w.z), __builtin_fabsf(w.w)));
      amax = row16_max(amax);                                 // c2 of this lane's block
      // Eq. 1: the constant is range/absmax (range 1); elements are multiplied by it.
      float rc = (amax < __FLT_MIN__) ? 0.0f : __fdiv_rn(MODE == 2 ? 127.0f : 1.0f, amax);
      if constexpr (MODE == 2) {
        if (__builtin_isinf(rc)) rc = 0.0f;                   // 127 / absmax beyond fp32: the block quantises to zeros
        auto q8 = [&](float x) -> uint32_t {                  // the product lies in [-127, 127] up to rounding: clamp anyway
          const float t = __builtin_fminf(__builtin_fmaxf(__builtin_rintf(__fmul_rn(x, rc)), -127.0f), 127.0f);
          return (uint32_t)(int)t & 0xffu;
        };
        ((uint32_t*)packed)[v] = q8(w.x) | (q8(w.y) << 8) | (q8(w.z) << 16) | (q8(w.w) << 24);
      }
      uint32_t i0 = 0, i1 = 0, i2 = 0, i3 = 0;
      if constexpr (MODE == 2) {
      } else if constexpr (OTHER) {
        i0 = index_search4(__fmul_rn(w.x, rc), th);
        i1 = index_search4(__fmul_rn(w.y, rc), th);
        i2 = index_search4(__fmul_rn(w.z, rc), th);
        i3 = index_search4(__fmul_rn(w.w, rc), th);
      } else {
        i0 = nf4_index(__fmul_rn(w.x, rc), buckets);
        i1 = nf4_index(__fmul_rn(w.y, rc), buckets);
        i2 = nf4_index(__fmul_rn(w.z, rc), buckets);
        i3 = nf4_index(__fmul_rn(w.w, rc), buckets);
      }
      if constexpr (MODE != 2) ((uint16_t*)packed)[v] = (uint16_t)(i0 | (i1 << 4) | (i2 << 8) | (i3 << 12));
      if ((threadIdx.x & 15) == 0) {
        c2_out[v >> 4] = amax;
        const uint32_t u32 = __builtin_bit_cast(uint32_t, amax);
        uint32_t e = u32 >> 23, m = u32 & 0x7fffffu;
        if (e == 0) e = 1; else m |= 0x800000u;               // value = m * 2^(e - 150)
        atomicAdd(&lbins[e], (unsigned long long)m);
      }
    }
  }
  __syncthreads();
  const unsigned long long mine = lbins[threadIdx.x];
  if (mine) atomicAdd(&bins[threadIdx.x], mine);
}

// Single wave.  sum = SUM_e bins[e] * 2^(e-1) in units of 2^-149, as 12 x 32-bit limbs;
// mean = round_to_nearest_even_fp32(sum / n).  Only the non-empty bins (found with wave ballots)
// and the non-zero limbs are visited, so the serial part is a few dozen operations.
__global__ __launch_bounds__(64) void dq_mean_kernel(const unsigned long long* __restrict__ bins,
                                                     uint32_t n, float* __restrict__ mean_out) {
  __shared__ unsigned long long lb[256];
  unsigned long long present[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const unsigned long long v = bins[q * 64 + threadIdx.x];
    lb[q * 64 + threadIdx.x] = v;
    present[q] = __ballot(v != 0ull);
  }
  __syncthreads();
  if (threadIdx.x != 0) return;

  constexpr int L = 12;
  uint32_t acc[L];
  for (int k = 0; k < L; ++k) acc[k] = 0;
  int top_limb = -1;
  for (int q = 0; q < 4; ++q) {
    unsigned long long mask = present[q];
    while (mask) {
      const int e = q * 64 + __builtin_ctzll(mask);
      mask &= mask - 1;
      if (e < 1 || e > 254) continue;                       // exponent 255 (inf/nan) never occurs: inputs are finite
      const unsigned long long b = lb[e];
      const int sh = e - 1, limb = sh >> 5, off = sh & 31;
      // b < 2^56; b << off spans at most three limbs
      const uint32_t p0 = (uint32_t)(b << off);
      const unsigned long long hi = off ? (b >> (32 - off)) : (b >> 32);
      const uint32_t parts[3] = {p0, (uint32_t)hi, (uint32_t)(hi >> 32)};
      unsigned long long carry = 0;
      for (int k = 0; k < L - limb; ++k) {
        const unsigned long long t = (unsigned long long)acc[limb + k] + (k < 3 ? parts[k] : 0u) + carry;
        acc[limb + k] = (uint32_t)t;
        carry = t >> 32;
        if (t && limb + k > top_limb) top_limb = limb + k;
        if (k >= 2 && carry == 0) break;
      }
    }
  }
  uint32_t q[L];
  for (int k = 0; k < L; ++k) q[k] = 0;
  unsigned long long rem = 0;
  for (int k = top_limb; k >= 0; --k) {                      // long division by n < 2^32
    const unsigned long long cur = (rem << 32) | acc[k];
    q[k] = (uint32_t)(cur / n);
    rem = cur % n;
  }
  int top = -1;
  for (int k = top_limb; k >= 0; --k)
    if (q[k]) { top = k * 32 + 31 - __builtin_clz(q[k]); break; }
  // keep the 24 leading bits of q (all of q if it is shorter), round on the rest and on rem/n
  const int drop = top >= 24 ? top - 23 : 0;
  auto bit = [&](int i) -> uint32_t { return (q[i >> 5] >> (i & 31)) & 1u; };
  uint32_t kept = 0;
  for (int i = top; i >= drop; --i) kept = (kept << 1) | bit(i);
  bool half, sticky;
  if (drop == 0) {
    half = 2 * rem >= n;
    sticky = 2 * rem > n;
  } else {
    half = bit(drop - 1) != 0;
    sticky = rem != 0;
    for (int i = drop - 2; i >= 0 && !sticky; --i) sticky = bit(i) != 0;
  }
  if (half && (sticky || (kept & 1u))) ++kept;              // kept <= 2^24
  // result = kept * 2^(drop - 149) with kept <= 2^24: with drop = 0 the integer is the bit pattern itself
  // (subnormals and the first binades); each further dropped bit raises the exponent field by one.
  *mean_out = __builtin_bit_cast(float, kept + ((uint32_t)drop << 23));
}

// One workgroup per run of 256 first-level constants.
__global__ __launch_bounds__(kDqBlock) void dq_encode_kernel(const float* __restrict__ c2, int64_t n,
                                                             const float* __restrict__ mean_ptr,
                                                             uint8_t* __restrict__ code,
                                                             float* __restrict__ c1, uint32_t rows, uint32_t bpr) {
  __shared__ float wmax[kDqBlock / 64];
  const int64_t b = (int64_t)blockIdx.x * kDqBlock + threadIdx.x;
  const float mean = *mean_ptr;
  const float d = (b < n) ? __fsub_rn(c2[b], mean) : 0.0f;  // centred constant
  const float m = wave_max(__builtin_fabsf(d));
  if ((threadIdx.x & 63) == 0) wmax[threadIdx.x >> 6] = m;
  __syncthreads();
  const float amax = __builtin_fmaxf(__builtin_fmaxf(wmax[0], wmax[1]), __builtin_fmaxf(wmax[2], wmax[3]));
  float rc1 = (amax < __FLT_MIN__) ? 0.0f : __fdiv_rn(kF8Max, amax);
  if (__builtin_isinf(rc1)) rc1 = 0.0f;
  if (b < n) {                                               // runs follow the flattened order, storage is column-group-major
    const uint32_t row = (uint32_t)b / bpr, blk = (uint32_t)b - row * bpr;
    code[code_pos(rows, (int)bpr, row, (int)blk)] = (uint8_t)e4m3_encode(__fmul_rn(d, rc1));
  }
  if (threadIdx.x == 0) c1[blockIdx.x] = amax;
}

hipError_t launch_quantize(const float* W, int64_t rows, int64_t cols, uint8_t* packed, uint8_t* code, float* c1,
                           float* mean, void* scratch, hipStream_t st, int dtype, bool dq) {
  if (dtype < 0 || dtype >= kNumTypes) return hipErrorInvalidValue;
  const Thresholds4 thr = thresholds4_host(table4_host(dtype));
  const int64_t elems = rows * cols;
  const int64_t n = elems / kBlock;
  unsigned long long* bins = (unsigned long long*)scratch;           // 256 x u64
  // without Double Quantization the first-level constants are the result and go straight to the caller's buffer
  float* c2 = dq ? (float*)((char*)scratch + 256 * sizeof(unsigned long long)) : c1;
  const int64_t n_vec4 = elems / 4;
  int64_t blocks = (n_vec4 + kQThreads - 1) / kQThreads;
  const int64_t cap = 256 * QL_Q_WGS_PER_CU;                         // workgroups per CU
  if (blocks > cap) blocks = cap;
  hipLaunchKernelGGL(zero_bins_kernel, dim3(1), dim3(256), 0, st, bins);
  if (dtype == 0)
    hipLaunchKernelGGL(quantize_nf4_kernel<0>, dim3((unsigned)blocks), dim3(kQThreads), 0, st, (const float4*)W,
                       n_vec4, (void*)packed, c2, bins, thr);
  else if (dtype == kTypeInt8)
    hipLaunchKernelGGL(quantize_nf4_kernel<2>, dim3((unsigned)blocks), dim3(kQThreads), 0, st, (const float4*)W,
                       n_vec4, (void*)packed, c2, bins, thr);
  else
    hipLaunchKernelGGL(quantize_nf4_kernel<1>, dim3((unsigned)blocks), dim3(kQThreads), 0, st, (const float4*)W,
                       n_vec4, (void*)packed, c2, bins, thr);
  if (!dq) return hipGetLastError();
  hipLaunchKernelGGL(dq_mean_kernel, dim3(1), dim3(64), 0, st, bins, (uint32_t)n, mean);
  const int64_t n1 = (n + kDqBlock - 1) / kDqBlock;
  hipLaunchKernelGGL(dq_encode_kernel, dim3((unsigned)n1), dim3(kDqBlock), 0, st, c2, n, mean, code, c1,
                     (uint32_t)rows, (uint32_t)(cols / kBlock));
  return hipGetLastError();
}

// ---- the variant for callers that cannot allocate ---------------------------------------------------------------
// Its scratch (the exponent bins and the fp32 constants c2 of up to kStaticQuantBlocks blocks) is this array; every
// device the library runs on holds its own copy at its own address, found once per device.
static __device__ __align__(256) unsigned char scratch[kQuantBinsBytes + kStaticQuantBlocks * sizeof(float)];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};
}  // namespace

hipError_t quantize_static_scratch(void** ptr) {
  int dev = -1;
  if (hipError_t e = hipGetDevice(&dev)) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch))) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  return hipSuccess;
}

hipError_t launch_quantize_static(const float* W, int64_t rows, int64_t cols, uint8_t* packed, uint8_t* code,
                                  float* c1, float* mean, hipStream_t st, int dtype, bool dq) {
  if (rows * cols / kBlock > (int64_t)kStaticQuantBlocks) return hipErrorInvalidValue;
  void* ptr = nullptr;
  if (hipError_t e = quantize_static_scratch(&ptr)) return e;
  return launch_quantize(W, rows, cols, packed, code, c1, mean, ptr, st, dtype, dq);
}

}  // namespace qlora
