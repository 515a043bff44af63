// Few-token (M <= 16) forward and input-gradient of the QLoRA linear layer (arXiv 2305.14314,
// Eq. 5 / Eq. 6 at generation-time batch sizes): bandwidth-bound streaming kernels that read the
// packed NF4 weight and its double-quantised constants exactly once (0.516 B per weight),
// dequantise in registers to the same bf16 values as the standalone doubleDequant, and feed
// MFMA 16x16x32 with the tokens as the 16-wide dimension.
//
//   forward : part[split][m][n] = sum over the split's k rows of X[m][k] * What[k][n]
//   backward: part[split][m][k] = sum over the split's n cols of dY[m][n] * What[k][n]
//   finalize: out = bf16( sum of splits + (s * T) * L2 )   resp.   (s * U) * L1^T   -- one rounding
//
// NF4 decode uses a 256-entry byte -> (value[lo nibble], value[hi nibble]) table in LDS, one
// 64-bit LDS read per two weights.
#include "common.hpp"
#include "launch.hpp"

namespace qlora {

constexpr int kFewThreads = 256;
typedef __attribute__((address_space(3))) char lds_c;

__device__ __forceinline__ void init_pair_lut(f32x2* lut2, float* unit) {
  constexpr float t[16] = {QLORA_NF4_VALUES};
  const int b = threadIdx.x;                                 // 256 threads, 256 byte values
  f32x2 v;
  v[0] = t[b & 15];
  v[1] = t[b >> 4];
  lut2[b] = v;
  unit[b] = e4m3_unit(b);
}

// ------------------------------------------------------------------------------------------------
// Forward.  W is [h][o], o contiguous.  A workgroup owns 128 output columns and a range of k rows;
// its 4 waves take interleaved 32-row steps and are summed through LDS at the end.
// Lane (i = lane % 16, g = lane / 16) loads, for rows kb + 8g + j (j = 0..7), the packed dword of
// columns n0 + 8i .. 8i+7.  MFMA e (0..7) multiplies the 16 tokens with columns {n0 + 8i + e}.
struct FewFwdArgs {
  const uint16_t* X; int M;
  const uint32_t* packed; const uint8_t* code; const float* c1; const float* mean;
  int h, o;
  float* part;           // [splits][M][o]
  int k_per_split;       // multiple of 32
};

__global__ __launch_bounds__(kFewThreads) void fewtok_fwd_kernel(const FewFwdArgs p) {
  __shared__ f32x2 lut2[256];
  __shared__ float unit[256];
  __shared__ float red[4][16][128];                          // per-wave output tiles for the final sum
  init_pair_lut(lut2, unit);
  __syncthreads();

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int i = lane & 15, g = lane >> 4;
  const int n0 = blockIdx.x * 128;
  const int k_begin = blockIdx.y * p.k_per_split;
  const int k_end = (k_begin + p.k_per_split < p.h) ? k_begin + p.k_per_split : p.h;
  const float mean = *p.mean;
  const int bpr = p.o >> 6;                                  // 64-blocks per row
  const int o_dw = p.o >> 3;                                 // packed dwords per row
  const bool col_ok = n0 + 8 * i < p.o;                      // o % 64 == 0: a dword is in or out as a whole
  const int nblk = (n0 + 8 * i) >> 6;

  f32x4 acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = f32x4{0.f, 0.f, 0.f, 0.f};

  for (int kb = k_begin + wave * 32; kb < k_end; kb += 4 * 32) {
    // token fragment: lane (token = i, k group g) holds X[token][kb + 8g .. +7]
    bf16x8 xa;
    {
      u32x4 raw = {0u, 0u, 0u, 0u};
      if (i < p.M && kb + 8 * g < k_end) raw = *(const u32x4*)(p.X + (int64_t)i * p.h + kb + 8 * g);
      xa = __builtin_bit_cast(bf16x8, raw);
    }
    uint32_t pk[8];
    float c2[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int k = kb + 8 * g + j;
      const bool ok = col_ok && k < k_end;
      const int64_t row = ok ? k : 0;
      pk[j] = ok ? p.packed[row * o_dw + (n0 >> 3) + i] : 0x77777777u;
      const int64_t blk = row * bpr + (ok ? nblk : 0);
      c2[j] = ok ? __fadd_rn(__fmul_rn(unit[p.code[blk]], p.c1[blk >> 8]), mean) : 0.0f;
    }
    float v[8][8];                                           // [row j][column e]
#pragma unroll
    for (int j = 0; j < 8; ++j) {
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const f32x2 q = lut2[(pk[j] >> (8 * b)) & 0xffu];
        v[j][2 * b] = __fmul_rn(q[0], c2[j]);
        v[j][2 * b + 1] = __fmul_rn(q[1], c2[j]);
      }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      u32x4 w;
      w[0] = pack_bf16x2(v[0][e], v[1][e]);
      w[1] = pack_bf16x2(v[2][e], v[3][e]);
      w[2] = pack_bf16x2(v[4][e], v[5][e]);
      w[3] = pack_bf16x2(v[6][e], v[7][e]);
      acc[e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa, __builtin_bit_cast(bf16x8, w), acc[e], 0, 0, 0);
    }
  }

  // D layout: column slot = lane % 16 (= i), token rows 4 * (lane / 16) + v
#pragma unroll
  for (int e = 0; e < 8; ++e)
#pragma unroll
    for (int vv = 0; vv < 4; ++vv) red[wave][4 * g + vv][8 * i + e] = acc[e][vv];
  __syncthreads();
  float* out = p.part + (int64_t)blockIdx.y * p.M * p.o;
  for (int idx = threadIdx.x; idx < p.M * 128; idx += kFewThreads) {
    const int m = idx >> 7, c = idx & 127;
    if (n0 + c < p.o) out[(int64_t)m * p.o + n0 + c] = red[0][m][c] + red[1][m][c] + red[2][m][c] + red[3][m][c];
  }
}

// ------------------------------------------------------------------------------------------------
// Backward (input gradient).  Contraction runs along o, the contiguous dimension of W, so a lane's
// 16-byte load is 32 consecutive k of one weight row and one quantisation constant.
// A workgroup owns 128 weight rows (4 waves x 32) and a range of o; per step of 128 columns a lane
// (i = lane % 16, g = lane / 16) loads rows r0 + i and r0 + 16 + i at columns kb + 32g .. +31.
// MFMA t (0..3) uses dword t of each load: columns kb + 32g + 8t .. +7.
struct FewBwdArgs {
  const uint16_t* dY; int M;
  const u32x4* packed; const uint8_t* code; const float* c1; const float* mean;
  int h, o;
  float* part;           // [splits][M][h]
  int c_per_split;       // multiple of 128
};

__global__ __launch_bounds__(kFewThreads) void fewtok_bwd_kernel(const FewBwdArgs p) {
  __shared__ f32x2 lut2[256];
  __shared__ float unit[256];
  init_pair_lut(lut2, unit);
  __syncthreads();

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int i = lane & 15, g = lane >> 4;
  const int r0 = blockIdx.x * 128 + wave * 32;
  const int c_begin = blockIdx.y * p.c_per_split;
  const int c_end = (c_begin + p.c_per_split < p.o) ? c_begin + p.c_per_split : p.o;
  const float mean = *p.mean;
  const int bpr = p.o >> 6;
  const int o_q = p.o >> 5;                                  // 16-byte groups (32 weights) per row

  f32x4 acc[2];
  acc[0] = f32x4{0.f, 0.f, 0.f, 0.f};
  acc[1] = f32x4{0.f, 0.f, 0.f, 0.f};

  for (int kb = c_begin; kb < c_end; kb += 128) {
    const int col = kb + 32 * g;
    const bool c_ok = col < c_end;                           // c_end % 64 == 0
    u32x4 wq[2];
    float c2[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int row = r0 + 16 * u + i;
      const bool ok = c_ok && row < p.h;
      const int64_t rr = ok ? row : 0;
      const int cc = ok ? col : 0;
      wq[u] = ok ? p.packed[rr * o_q + (cc >> 5)] : u32x4{0x77777777u, 0x77777777u, 0x77777777u, 0x77777777u};
      const int64_t blk = rr * bpr + (cc >> 6);
      c2[u] = ok ? __fadd_rn(__fmul_rn(unit[p.code[blk]], p.c1[blk >> 8]), mean) : 0.0f;
    }
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      bf16x8 ya;                                             // lane (token = i, g): dY[token][col + 8t .. +7]
      {
        u32x4 raw = {0u, 0u, 0u, 0u};
        if (i < p.M && c_ok) raw = *(const u32x4*)(p.dY + (int64_t)i * p.o + col + 8 * t);
        ya = __builtin_bit_cast(bf16x8, raw);
      }
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const uint32_t d = wq[u][t];
        u32x4 w;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          const f32x2 q = lut2[(d >> (8 * b)) & 0xffu];
          w[b] = pack_bf16x2(__fmul_rn(q[0], c2[u]), __fmul_rn(q[1], c2[u]));
        }
        acc[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ya, __builtin_bit_cast(bf16x8, w), acc[u], 0, 0, 0);
      }
    }
  }

  float* out = p.part + (int64_t)blockIdx.y * p.M * p.h;
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int row = r0 + 16 * u + i;                         // D column slot = lane % 16 = weight row
    if (row < p.h) {
#pragma unroll
      for (int vv = 0; vv < 4; ++vv) {
        const int m = 4 * g + vv;
        if (m < p.M) out[(int64_t)m * p.h + row] = acc[u][vv];
      }
    }
  }
}

// out[m][n] = bf16( sum_s part[s][m][n] + sum_j A[m][j] * B(j, n) ),  A = bf16(s * T) or bf16(s * U)
// (M x rp, zero-padded), B(j, n) = Bmat[j * ldb_j + n * ldb_n].
__global__ void fewtok_finalize_kernel(const float* __restrict__ part, int splits, int M, int N,
                                       const uint16_t* __restrict__ A, int rp, int r,
                                       const uint16_t* __restrict__ Bmat, int64_t ldb_j, int64_t ldb_n,
                                       uint16_t* __restrict__ out) {
  const int64_t total = (int64_t)M * N;
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
    const int m = (int)(e / N), n = (int)(e % N);
    float s = 0.0f;
    for (int sp = 0; sp < splits; ++sp) s += part[((int64_t)sp * M + m) * N + n];
    float l = 0.0f;
    for (int j = 0; j < r; ++j)
      l = __builtin_fmaf(bf16_lo_to_f32(A[(int64_t)m * rp + j]), bf16_lo_to_f32(Bmat[j * ldb_j + n * ldb_n]), l);
    out[e] = bf16_bits(s + l);
  }
}

static int pick_splits(int slabs, int steps_total, int min_steps) {
  int splits = (512 + slabs - 1) / slabs;                    // about two workgroups per CU
  int cap = steps_total / min_steps;
  if (cap < 1) cap = 1;
  if (splits > cap) splits = cap;
  if (splits > 64) splits = 64;
  if (splits < 1) splits = 1;
  return splits;
}

int fewtok_fwd_splits(int h, int o) { return pick_splits((o + 127) / 128, (h + 31) / 32, 16); }
int fewtok_bwd_splits(int h, int o) { return pick_splits((h + 127) / 128, (o + 127) / 128, 4); }

hipError_t launch_fewtok_fwd(const uint16_t* X, int M, const NF4Dev& w, float* part, int splits, hipStream_t st) {
  FewFwdArgs a;
  a.X = X; a.M = M; a.packed = (const uint32_t*)w.packed; a.code = w.code; a.c1 = w.c1; a.mean = w.mean;
  a.h = (int)w.rows; a.o = (int)w.cols; a.part = part;
  const int steps = (a.h + 31) / 32;
  a.k_per_split = ((steps + splits - 1) / splits) * 32;
  dim3 grid((unsigned)((a.o + 127) / 128), (unsigned)splits);
  hipLaunchKernelGGL(fewtok_fwd_kernel, grid, dim3(kFewThreads), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_fewtok_bwd(const uint16_t* dY, int M, const NF4Dev& w, float* part, int splits, hipStream_t st) {
  FewBwdArgs a;
  a.dY = dY; a.M = M; a.packed = (const u32x4*)w.packed; a.code = w.code; a.c1 = w.c1; a.mean = w.mean;
  a.h = (int)w.rows; a.o = (int)w.cols; a.part = part;
  const int steps = (a.o + 127) / 128;
  a.c_per_split = ((steps + splits - 1) / splits) * 128;
  dim3 grid((unsigned)((a.h + 127) / 128), (unsigned)splits);
  hipLaunchKernelGGL(fewtok_bwd_kernel, grid, dim3(kFewThreads), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_fewtok_finalize(const float* part, int splits, int M, int N, const uint16_t* A, int rp, int r,
                                  const uint16_t* Bmat, int64_t ldb_j, int64_t ldb_n, uint16_t* out, hipStream_t st) {
  int64_t blocks = ((int64_t)M * N + 255) / 256;
  if (blocks > 2048) blocks = 2048;
  hipLaunchKernelGGL(fewtok_finalize_kernel, dim3((unsigned)blocks), dim3(256), 0, st, part, splits, M, N, A, rp, r,
                     Bmat, ldb_j, ldb_n, out);
  return hipGetLastError();
}

}  // namespace qlora
