// Standalone doubleDequant (arXiv 2305.14314, Eq. 6 and Eq. 2): packed NF4 indices and
// double-quantised constants -> bf16 weights.  HBM-bound: 0.516 B read + 2 B written per element.
// One lane decodes one packed dword (8 weights of one 64-block) and stores 16 bytes.
#include "common.hpp"
#include "launch.hpp"

namespace qlora {

constexpr int kDeqThreads = 256;

// The 16 values of the data type into LDS: NF4 from constants; another type (Section 4) from the argument, copied
// by one thread with constant indices (a lane-indexed read of a by-value argument would go through scratch).
__device__ __forceinline__ void init_lut16(float* lut, int dtype, const Table4& tab) {
  if (dtype == 0) {
    if (threadIdx.x < 16) {
      constexpr float t[16] = {QLORA_NF4_VALUES};
      lut[threadIdx.x] = t[threadIdx.x];
    }
  } else if (threadIdx.x == 0) {
#pragma unroll
    for (int i = 0; i < 16; ++i) lut[i] = tab.v[i];
  }
}

// signed byte j of a dword as fp32
__device__ __forceinline__ float s8_to_f32(uint32_t p, int j) { return (float)((int)(p << (24 - 8 * j)) >> 24); }

// I8: 8-bit integers, Eq. 2 as printed: w = q * absmax / 127, as bf16(fl32(q * fl32(c2 / 127))).  A lane then reads
// 8 bytes instead of 4; `packed` and `n_dwords` count in lane-sized units (8 weights) either way.
template <bool DQ, bool I8, bool GAP>
__global__ __launch_bounds__(kDeqThreads) void dequant_nf4_kernel(
    const void* __restrict__ packed_v, const uint8_t* __restrict__ code, const float* __restrict__ c1,
    const float* __restrict__ mean_ptr, uint4* __restrict__ out, int64_t n_dwords, uint32_t rows, uint32_t bpr,
    const int dtype, const Table4 tab, const int64_t row_gap) {
  // GAP: the output rows are row_gap 16-byte groups apart (a wider buffer: several weights side by side); else back to back
  constexpr bool dq = DQ;                                    // Double Quantization, or the fp32 constants as they are
  const uint32_t* __restrict__ packed = (const uint32_t*)packed_v;
  __shared__ float lut[16];
  __shared__ float unit[256];
  init_lut16(lut, dtype, tab);
  unit[threadIdx.x] = e4m3_unit(threadIdx.x);               // 256 threads, 256 codes
  __syncthreads();
  const float mean = dq ? *mean_ptr : 0.0f;

  const int64_t stride = (int64_t)gridDim.x * kDeqThreads;
  for (int64_t d = (int64_t)blockIdx.x * kDeqThreads + threadIdx.x; d < n_dwords; d += stride) {
    uint32_t p, ph = 0;
    if constexpr (I8) {
      const uint2 pp = ((const uint2*)packed_v)[d];
      p = pp.x; ph = pp.y;
    } else {
      p = packed[d];
    }
    const uint32_t blk = (uint32_t)(d >> 3);                // 8 lanes per 64-block
    float c2;
    if (dq) {
      const uint32_t row = blk / bpr;
      const uint8_t cd = code[code_pos(rows, (int)bpr, row, (int)(blk - row * bpr))];
      // dequant(c1, c2): two separately rounded fp32 steps
      c2 = __fadd_rn(__fmul_rn(unit[cd], c1[blk >> 8]), mean);
    } else {
      c2 = c1[blk];                                           // no Double Quantization: the fp32 constant itself
    }
    uint4 o;
    if constexpr (I8) {
      const float step = __fdiv_rn(c2, 127.0f);
      o.x = pack_bf16x2(__fmul_rn(s8_to_f32(p, 0), step), __fmul_rn(s8_to_f32(p, 1), step));
      o.y = pack_bf16x2(__fmul_rn(s8_to_f32(p, 2), step), __fmul_rn(s8_to_f32(p, 3), step));
      o.z = pack_bf16x2(__fmul_rn(s8_to_f32(ph, 0), step), __fmul_rn(s8_to_f32(ph, 1), step));
      o.w = pack_bf16x2(__fmul_rn(s8_to_f32(ph, 2), step), __fmul_rn(s8_to_f32(ph, 3), step));
    } else {
      o.x = pack_bf16x2(__fmul_rn(lut[p & 15u], c2), __fmul_rn(lut[(p >> 4) & 15u], c2));
      o.y = pack_bf16x2(__fmul_rn(lut[(p >> 8) & 15u], c2), __fmul_rn(lut[(p >> 12) & 15u], c2));
      o.z = pack_bf16x2(__fmul_rn(lut[(p >> 16) & 15u], c2), __fmul_rn(lut[(p >> 20) & 15u], c2));
      o.w = pack_bf16x2(__fmul_rn(lut[(p >> 24) & 15u], c2), __fmul_rn(lut[p >> 28], c2));
    }
    if constexpr (GAP) out[d + (int64_t)(blk / bpr) * row_gap] = o;
    else out[d] = o;
  }
}

// Transposed variant for the forward GEMM: out[n][k] = dequant(W)[k][n], row stride ld_out >= h.
// A workgroup owns 64 input rows (k) x 256 columns (n); each wave a 64 x 64 sub-tile, i.e. one
// 64-block per row.  A lane loads one packed dword (8 n) from each of 8 consecutive rows and
// writes, for each of its 8 columns, the 8 k-consecutive bf16 as one 16-byte store, so stores
// form 128-byte runs along k.  No LDS staging of data.
//
// Workgroup rows beyond the weight's (blockIdx.y >= ceil(h / 64)) transpose the adapter's L2 (r x o, bf16) the same
// way into columns h + col0 .. h + col0 + r - 1 of `out` and write zeros to the rest of columns h .. h + rp - 1, so
// that one buffer of row stride ld_out >= h + rp holds both K segments of the forward product's weight-side operand
// and no launch of its own is spent on a 1 MB transpose.  (col0 > 0: several layers stacked along n share the adapter
// segment block-diagonally: a layer's rows hold its own L2^T in its own columns and zeros in the others'.)
template <bool DQ, bool I8>
__global__ __launch_bounds__(kDeqThreads) void dequant_nf4_t_kernel(
    const void* __restrict__ packed_v, const uint8_t* __restrict__ code, const float* __restrict__ c1,
    const float* __restrict__ mean_ptr, uint16_t* __restrict__ out, int h, int o, int64_t ld_out, const int dtype,
    const Table4 tab, const uint16_t* __restrict__ L2, int r, int col0) {
  constexpr bool dq = DQ;
  const uint32_t* __restrict__ packed = (const uint32_t*)packed_v;
  const int w_rows = (h + 63) >> 6;                          // workgroup rows of the weight
  if ((int)blockIdx.y >= w_rows) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int kg = lane >> 3, ng = lane & 7;
    const int n_blk = blockIdx.x * 4 + wave;
    if (n_blk * 64 >= o) return;
    const int t_base = ((int)blockIdx.y - w_rows) * 64 + kg * 8;
    const int n_first = n_blk * 64 + ng * 8;
    uint4 row[8];                                            // row[j] = L2[t_base + j][n_first .. n_first + 7]
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int t = t_base + j - col0;                        // row of L2 that belongs into column h + t_base + j
      row[j] = (t >= 0 && t < r) ? *(const uint4*)(L2 + (int64_t)t * o + n_first) : uint4{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      auto el = [&](int j) -> uint32_t {                     // element e of row j
        const uint32_t d = (e >> 1) == 0 ? row[j].x : (e >> 1) == 1 ? row[j].y : (e >> 1) == 2 ? row[j].z : row[j].w;
        return (e & 1) ? d >> 16 : d & 0xffffu;
      };
      uint4 q;
      q.x = el(0) | (el(1) << 16);
      q.y = el(2) | (el(3) << 16);
      q.z = el(4) | (el(5) << 16);
      q.w = el(6) | (el(7) << 16);
      *(uint4*)(out + (int64_t)(n_first + e) * ld_out + h + t_base) = q;
    }
    return;
  }
  __shared__ float lut[16];
  __shared__ float unit[256];
  init_lut16(lut, dtype, tab);
  unit[threadIdx.x] = e4m3_unit(threadIdx.x);
  __syncthreads();
  const float mean = dq ? *mean_ptr : 0.0f;

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int kg = lane >> 3, ng = lane & 7;
  const int n_blk = blockIdx.x * 4 + wave;                  // 64-column block index within a row
  if (n_blk * 64 >= o) return;
  const int k_base = blockIdx.y * 64 + kg * 8;
  const int blocks_per_row = o >> 6;

  uint32_t p[8], ph[8];
  float c2[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int k = k_base + j;
    const bool ok = k < h;
    const int64_t blk = (int64_t)(ok ? k : 0) * blocks_per_row + n_blk;
    if constexpr (I8) {                                       // 8 bytes = this lane's 8 columns of row k
      const uint2 pp = ((const uint2*)packed_v)[blk * 8 + ng];
      p[j] = ok ? pp.x : 0u;
      ph[j] = ok ? pp.y : 0u;
    } else {
      p[j] = ok ? packed[blk * 8 + ng] : 0x77777777u;         // index 7 is the exact zero
      ph[j] = 0u;
    }
    if (dq) c2[j] = ok ? __fadd_rn(__fmul_rn(unit[code[code_pos(h, blocks_per_row, k, n_blk)]], c1[blk >> 8]), mean) : 0.0f;
    else c2[j] = ok ? c1[blk] : 0.0f;
    if constexpr (I8) c2[j] = __fdiv_rn(c2[j], 127.0f);       // Eq. 2: the step absmax / 127
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    float v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      if constexpr (I8) v[j] = __fmul_rn(s8_to_f32(e < 4 ? p[j] : ph[j], e & 3), c2[j]);
      else v[j] = __fmul_rn(lut[(p[j] >> (4 * e)) & 15u], c2[j]);
    }
    uint4 q;
    q.x = pack_bf16x2(v[0], v[1]);
    q.y = pack_bf16x2(v[2], v[3]);
    q.z = pack_bf16x2(v[4], v[5]);
    q.w = pack_bf16x2(v[6], v[7]);
    const int n = n_blk * 64 + ng * 8 + e;
    if (k_base < h) *(uint4*)(out + (int64_t)n * ld_out + k_base) = q;   // h % 8 == 0: all 8 or none
  }
}

hipError_t launch_dequant_t(const NF4Dev& w, uint16_t* out, int64_t ld_out, hipStream_t st, const uint16_t* L2, int r,
                            int rp, int col0) {
  const int h = (int)w.rows, o = (int)w.cols;
  if (L2 == nullptr) { r = 0; col0 = 0; }                    // rp > 0 without an adapter: the segment is all zeros
  if (rp % 64 != 0 || col0 < 0 || col0 + r > rp || ld_out < h + rp || ld_out % 8 != 0) return hipErrorInvalidValue;
  dim3 grid((unsigned)((o + 255) / 256), (unsigned)((h + 63) / 64 + rp / 64));
  const bool i8 = w.dtype == kTypeInt8;
#define QL_DEQ_T(DQ, I8)                                                                                        \
  hipLaunchKernelGGL((dequant_nf4_t_kernel<DQ, I8>), grid, dim3(kDeqThreads), 0, st, (const void*)w.packed, w.code, \
                     w.c1, w.mean, out, h, o, ld_out, w.dtype, table4_host(w.dtype), L2, r, col0)
  if (w.dq) { if (i8) QL_DEQ_T(true, true); else QL_DEQ_T(true, false); }
  else      { if (i8) QL_DEQ_T(false, true); else QL_DEQ_T(false, false); }
#undef QL_DEQ_T
  return hipGetLastError();
}

// What the fused backward GEMM reads beside the packed codes: the data type's 16 values, and (with Double
// Quantization) the fp32 constant of every 64-block in flat order, dequant(c1, c2) of Eq. 6 with the two roundings of
// the kernels above.  0.0625 bytes written per weight.
__global__ __launch_bounds__(kDeqThreads) void block_consts_kernel(const uint8_t* __restrict__ code,
                                                                   const float* __restrict__ c1,
                                                                   const float* __restrict__ mean_ptr,
                                                                   float* __restrict__ out, int64_t n_blocks,
                                                                   uint32_t rows, uint32_t bpr, const int dtype,
                                                                   const Table4 tab, float* __restrict__ tab_out,
                                                                   const bool dq) {
  __shared__ float lut[16];
  __shared__ float unit[256];
  init_lut16(lut, dtype, tab);
  unit[threadIdx.x] = e4m3_unit(threadIdx.x);
  __syncthreads();
  if (blockIdx.x == 0 && threadIdx.x < 16) tab_out[threadIdx.x] = lut[threadIdx.x];
  if (!dq) return;
  const float mean = *mean_ptr;
  const int64_t stride = (int64_t)gridDim.x * kDeqThreads;
  for (int64_t b = (int64_t)blockIdx.x * kDeqThreads + threadIdx.x; b < n_blocks; b += stride) {
    const uint32_t row = (uint32_t)(b / bpr);
    const uint8_t cd = code[code_pos(rows, (int)bpr, row, (int)(b - (int64_t)row * bpr))];
    out[b] = __fadd_rn(__fmul_rn(unit[cd], c1[b >> 8]), mean);
  }
}

hipError_t launch_block_consts(const NF4Dev& w, float* consts, float* tab16, hipStream_t st) {
  if (w.dtype == kTypeInt8 || w.cols % 64 != 0) return hipErrorInvalidValue;
  const int64_t n_blocks = w.rows * (w.cols / 64);
  int64_t blocks = w.dq ? (n_blocks + kDeqThreads - 1) / kDeqThreads : 1;
  if (blocks > 256 * 8) blocks = 256 * 8;
  hipLaunchKernelGGL(block_consts_kernel, dim3((unsigned)blocks), dim3(kDeqThreads), 0, st, w.code, w.c1, w.mean, consts,
                     n_blocks, (uint32_t)w.rows, (uint32_t)(w.cols / 64), w.dtype, table4_host(w.dtype), tab16, w.dq);
  return hipGetLastError();
}

hipError_t launch_dequant(const NF4Dev& w, uint16_t* out, hipStream_t st, int64_t ld_out) {
  if (ld_out == 0) ld_out = w.cols;
  if (ld_out < w.cols || ld_out % 8 != 0) return hipErrorInvalidValue;
  const int64_t n_dwords = w.rows * w.cols / 8;
  int64_t blocks = (n_dwords + kDeqThreads - 1) / kDeqThreads;
  const int64_t cap = 256 * 32;
  if (blocks > cap) blocks = cap;
  const bool i8 = w.dtype == kTypeInt8;
#define QL_DEQ(DQ, I8, GAP)                                                                                 \
  hipLaunchKernelGGL((dequant_nf4_kernel<DQ, I8, GAP>), dim3((unsigned)blocks), dim3(kDeqThreads), 0, st,   \
                     (const void*)w.packed, w.code, w.c1, w.mean, (uint4*)out, n_dwords, (uint32_t)w.rows,  \
                     (uint32_t)(w.cols / 64), w.dtype, table4_host(w.dtype), (ld_out - w.cols) / 8)
  if (ld_out != w.cols) {
    if (w.dq) { if (i8) QL_DEQ(true, true, true); else QL_DEQ(true, false, true); }
    else      { if (i8) QL_DEQ(false, true, true); else QL_DEQ(false, false, true); }
  } else {
    if (w.dq) { if (i8) QL_DEQ(true, true, false); else QL_DEQ(true, false, false); }
    else      { if (i8) QL_DEQ(false, true, false); else QL_DEQ(false, false, false); }
  }
#undef QL_DEQ
  return hipGetLastError();
}

}  // namespace qlora
