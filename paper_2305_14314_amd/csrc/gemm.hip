// bf16 MFMA GEMM for the large-token forward and backward products of the QLoRA linear layer
// (arXiv 2305.14314, Eq. 5 and the backward through the dequantised weight).
//
//   C[M x N] (bf16) = A0[M x K0] * B0[N x K0]^T  +  A1[M x K1] * B1[N x K1]^T      fp32 accumulate
//
// Both operands are K-contiguous ("NT").  Segment 0 is the frozen weight (B0 = dequantised W in
// the layout the direction needs), segment 1 the LoRA term (A1 = s * X L1 or s * dY L2^T, B1 = L2^T
// or L1): the adapter rides as extra K-steps of the same accumulators, so the output is rounded
// to bf16 exactly once.
//
// Tiling for gfx950: 256 x 256 output tile per workgroup of 4 waves (2 x 2), each wave 128 x 128
// as 4 x 4 MFMA 32x32x16 tiles (256 fp32 accumulators per lane), K-step 64.  Tiles are fetched
// with global_load_lds_dwordx4 (no VGPR staging) into two LDS stages of 2 x 32 KB; the 16-byte
// chunks of each 128-byte row are XOR-swizzled with the row index so ds_read_b128 of MFMA
// fragments is bank-conflict free.  Workgroup ids are remapped so that the 32 tiles resident on
// one XCD form a compact patch and share operand tiles in that XCD's L2.
#include "common.hpp"
#include "launch.hpp"

namespace qlora {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int kGemmThreads = 256;
constexpr int kTileBytes = BM * BK * 2;                     // 32 KB per operand per stage

typedef __attribute__((address_space(3))) void* lds_ptr_t;

struct GemmArgs {
  const uint16_t* A0; const uint16_t* B0; int64_t lda0, ldb0; int K0;
  const uint16_t* A1; const uint16_t* B1; int64_t lda1, ldb1; int K1;
  uint16_t* C; int64_t ldc;
  int M, N;
  int tiles_m, tiles_n;
};

// One operand tile (256 rows x 64 k) -> LDS.  Wave w, instruction j fills LDS rows (4j + w) * 8 .. + 7;
// lane l lands at row l / 8, physical chunk l % 8, and therefore fetches logical chunk (l % 8) ^ (l / 8).
__device__ __forceinline__ void load_tile(const uint16_t* __restrict__ base, const int64_t* row_off, int k0,
                                          char __attribute__((address_space(3)))* lds, int wave, int lane) {
  const int chunk = (lane & 7) ^ (lane >> 3);
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const uint16_t* g = base + row_off[j] + k0 + chunk * 8;
    __builtin_amdgcn_global_load_lds(g, (lds_ptr_t)(lds + (4 * j + wave) * 1024), 16, 0, 0);
  }
}

__device__ __forceinline__ bf16x8 read_frag(const char __attribute__((address_space(3)))* lds, int row, int chunk) {
  const int phys = chunk ^ (row & 7);
  return *(const bf16x8 __attribute__((address_space(3)))*)(lds + row * 128 + phys * 16);
}

__device__ __forceinline__ void compute_stage(const char __attribute__((address_space(3)))* sA,
                                              const char __attribute__((address_space(3)))* sB,
                                              int a_row, int b_row, int half, f32x16 (&acc)[4][4]) {
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    bf16x8 a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) a[i] = read_frag(sA, a_row + 32 * i, 2 * kk + half);
#pragma unroll
    for (int i = 0; i < 4; ++i) b[i] = read_frag(sB, b_row + 32 * i, 2 * kk + half);
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
      for (int ni = 0; ni < 4; ++ni)
        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mi], b[ni], acc[mi][ni], 0, 0, 0);
  }
}

__global__ __launch_bounds__(kGemmThreads) void gemm_nt_kernel(const GemmArgs p) {
  // separate objects per stage so the compiler can tell a DMA into one stage from reads of the other
  __shared__ __attribute__((aligned(1024))) char sA0[kTileBytes];
  __shared__ __attribute__((aligned(1024))) char sA1[kTileBytes];
  __shared__ __attribute__((aligned(1024))) char sB0[kTileBytes];
  __shared__ __attribute__((aligned(1024))) char sB1[kTileBytes];

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;

  // ---- workgroup id -> output tile, XCD-aware -------------------------------------------------
  // Hardware deals consecutive workgroup ids round-robin to the 8 XCDs.  Give each XCD a
  // contiguous range of the tile order, and order tiles in groups of 4 tile-rows so that the
  // tiles resident together share A and B tiles.
  const int n_tiles = p.tiles_m * p.tiles_n;
  int pid = blockIdx.x;
  {
    const int xcd = pid & 7, local = pid >> 3;
    const int q = n_tiles >> 3, rem = n_tiles & 7;
    pid = (xcd < rem) ? xcd * (q + 1) + local : rem * (q + 1) + (xcd - rem) * q + local;
  }
  constexpr int GM = 4;
  const int per_group = GM * p.tiles_n;
  const int group = pid / per_group;
  const int first_m = group * GM;
  const int gsz = (p.tiles_m - first_m < GM) ? p.tiles_m - first_m : GM;
  const int in_group = pid - group * per_group;
  const int tile_m = first_m + in_group % gsz;
  const int tile_n = in_group / gsz;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  // ---- per-lane global row offsets for the 8 load instructions per operand ---------------------
  int a_rows[8], b_rows[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int r = (4 * j + wave) * 8 + (lane >> 3);
    int ra = m0 + r; if (ra > p.M - 1) ra = p.M - 1;        // clamp: padded rows are never stored
    int rb = n0 + r; if (rb > p.N - 1) rb = p.N - 1;
    a_rows[j] = ra; b_rows[j] = rb;
  }
  int64_t a_off[8], b_off[8];

  const int wm = wave >> 1, wn = wave & 1;
  const int a_row = wm * 128 + (lane & 31), b_row = wn * 128 + (lane & 31), half = lane >> 5;

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

  auto sA0p = (char __attribute__((address_space(3)))*)sA0;
  auto sA1p = (char __attribute__((address_space(3)))*)sA1;
  auto sB0p = (char __attribute__((address_space(3)))*)sB0;
  auto sB1p = (char __attribute__((address_space(3)))*)sB1;

#pragma unroll 1
  for (int seg = 0; seg < 2; ++seg) {
    const uint16_t* A = seg ? p.A1 : p.A0;
    const uint16_t* B = seg ? p.B1 : p.B0;
    const int64_t lda = seg ? p.lda1 : p.lda0, ldb = seg ? p.ldb1 : p.ldb0;
    const int KT = (seg ? p.K1 : p.K0) / BK;
    if (KT == 0) continue;
#pragma unroll
    for (int j = 0; j < 8; ++j) { a_off[j] = a_rows[j] * lda; b_off[j] = b_rows[j] * ldb; }

    __syncthreads();                                        // previous segment's reads are done
    load_tile(A, a_off, 0, sA0p, wave, lane);
    load_tile(B, b_off, 0, sB0p, wave, lane);
#pragma unroll 1
    for (int kt = 0; kt < KT; kt += 2) {
      __syncthreads();                                      // stage 0 has landed; stage 1 is free
      if (kt + 1 < KT) {
        load_tile(A, a_off, (kt + 1) * BK, sA1p, wave, lane);
        load_tile(B, b_off, (kt + 1) * BK, sB1p, wave, lane);
      }
      compute_stage(sA0p, sB0p, a_row, b_row, half, acc);
      if (kt + 1 < KT) {
        __syncthreads();                                    // stage 1 has landed; stage 0 is free
        if (kt + 2 < KT) {
          load_tile(A, a_off, (kt + 2) * BK, sA0p, wave, lane);
          load_tile(B, b_off, (kt + 2) * BK, sB0p, wave, lane);
        }
        compute_stage(sA1p, sB1p, a_row, b_row, half, acc);
      }
    }
  }

  // ---- epilogue: one rounding to bf16; lane owns column n, rows 8*(v/4) + 4*half + v%4 ---------
#pragma unroll
  for (int ni = 0; ni < 4; ++ni) {
    const int n = n0 + wn * 128 + ni * 32 + (lane & 31);
    if (n >= p.N) continue;
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int m = m0 + wm * 128 + mi * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
        if (m < p.M) p.C[(int64_t)m * p.ldc + n] = bf16_bits(acc[mi][ni][v]);
      }
    }
  }
}

hipError_t launch_gemm_nt(const uint16_t* A0, const uint16_t* B0, int64_t lda0, int64_t ldb0, int K0,
                          const uint16_t* A1, const uint16_t* B1, int64_t lda1, int64_t ldb1, int K1,
                          uint16_t* C, int64_t ldc, int M, int N, hipStream_t st) {
  GemmArgs a;
  a.A0 = A0; a.B0 = B0; a.lda0 = lda0; a.ldb0 = ldb0; a.K0 = K0;
  a.A1 = A1; a.B1 = B1; a.lda1 = lda1; a.ldb1 = ldb1; a.K1 = K1;
  a.C = C; a.ldc = ldc; a.M = M; a.N = N;
  a.tiles_m = (M + BM - 1) / BM;
  a.tiles_n = (N + BN - 1) / BN;
  hipLaunchKernelGGL(gemm_nt_kernel, dim3((unsigned)(a.tiles_m * a.tiles_n)), dim3(kGemmThreads), 0, st, a);
  return hipGetLastError();
}

}  // namespace qlora
