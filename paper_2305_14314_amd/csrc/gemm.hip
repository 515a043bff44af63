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
// Design for gfx950 (256 CUs in 8 XCDs, 160 KB LDS, MFMA 32x32x16 bf16 = 32 cycles per SIMD):
//  * 256 x 256 output tile per workgroup of 4 waves (2 x 2), each wave 128 x 128 as 4 x 4 MFMA
//    tiles: 256 fp32 accumulators per lane (AGPRs), half an LDS fragment read per MFMA.
//  * K-step 32, five LDS stages of (A tile 16 KB, B tile 16 KB): all 160 KB of the CU.  Tiles arrive
//    by global_load_lds_dwordx4 (no VGPR staging).  One barrier per K-step, placed in the MIDDLE of
//    the step: it publishes stage k+1 (requested about three steps earlier) and frees the stage of
//    step k-1 for the DMA of step k+4, so fragment reads of the next step never wait at a barrier
//    and the MFMA stream continues across step boundaries.
//  * The 8 DMA instructions of a step are spread one per row of 4 MFMAs (waves issue in order: a
//    burst of DMAs would stall the MFMA stream behind the texture-address FIFO).
//  * Fragment reads are software-pipelined one 16-wide sub-step ahead (the compiler is left free
//    to place them among the MFMAs of the sub-step: pinning two reads per row of 4 MFMAs with
//    scheduling barriers measured 15 % slower).  They are issued through inline asm with hand-placed s_waitcnt: the compiler's
//    automatic wait insertion cannot tell a DMA into one stage from a read of another across the
//    loop back-edge and would drain all DMAs every iteration.
//  * LDS rows are 64 bytes (32 k); the four 16-byte chunks of row r sit at chunk ^ ((r >> 2) & 3).
//    LDS has 64 banks: a ds_read_b128 is served 16 lanes (256 bytes) per cycle, and 16 consecutive
//    rows then cover all 16 sixteen-byte bank groups (measured 225 B/clk/CU against 114 for the
//    8-lane pattern that would suit a 32-bank LDS).
//  * Workgroup ids are remapped so each XCD (which receives every 8th id) works on a contiguous
//    range of the tile order, and tiles are ordered in groups of GM tile-rows, so the 32 tiles
//    resident on an XCD share A and B tiles in that XCD's L2.
//  * Rows beyond M / N are clamped for loads and masked at the store; steps beyond the last
//    re-fetch the last tile into a free stage, which keeps the loop body free of branches.
#include "common.hpp"
#include "launch.hpp"

namespace qlora {

namespace {

constexpr int BM = 256, BK = 32, NST = 5;                    // BN is 256, or 128 for the tail launch (template parameter)
constexpr int kOpBytes = BM * BK * 2;                       // 16 KB per 256-row operand tile per stage
constexpr int GM = 4;                                       // tile-rows per raster group
#ifndef QL_GEMM_WAVES
#define QL_GEMM_WAVES 8
#endif
constexpr int kMainWaves = QL_GEMM_WAVES;                    // waves per workgroup of the main (BN = 256) kernel

typedef __attribute__((address_space(3))) char lchar;

struct GemmArgs {
  const uint16_t* A0; const uint16_t* B0; int64_t lda0, ldb0; int KT0;   // KT = K / BK
  const uint16_t* A1; const uint16_t* B1; int64_t lda1, ldb1; int KT1;
  uint16_t* C; int64_t ldc;
  int M, N, tiles_m, tiles_n;
  int n_begin;                                               // first output column of this launch
};

template <int NI> struct Frags { bf16x8 a[4], b[NI]; };

// DMA instruction j of an operand tile: wave w of NW fills LDS rows (NW j + w) * 16 .. + 15 of the stage;
// lane l lands at row l / 4, physical chunk l % 4 (the caller's pointer already selects the
// logical chunk (l % 4) ^ ((l >> 4) & 3) of that row).
template <int NW>
__device__ __forceinline__ void dma16(const uint16_t* g, lchar* stage_tile, int j, int wave) {
  __builtin_amdgcn_global_load_lds(g, (__attribute__((address_space(3))) void*)(stage_tile + (NW * j + wave) * 1024),
                                   16, 0, 0);
}
template <int N> __device__ __forceinline__ void wait_vmcnt() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }

#define QL_LDS_READ(dst, addr) asm volatile("ds_read_b128 %0, %1" : "=v"(dst) : "v"(addr))
__device__ __forceinline__ void wait_frags(Frags<4>& f) {
  asm volatile("s_waitcnt lgkmcnt(0)"
               : "+v"(f.a[0]), "+v"(f.a[1]), "+v"(f.a[2]), "+v"(f.a[3]), "+v"(f.b[0]), "+v"(f.b[1]),
                 "+v"(f.b[2]), "+v"(f.b[3]));
}
__device__ __forceinline__ void wait_frags(Frags<1>& f) {
  asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f.a[0]), "+v"(f.a[1]), "+v"(f.a[2]), "+v"(f.a[3]), "+v"(f.b[0]));
}
__device__ __forceinline__ void wait_frags(Frags<2>& f) {
  asm volatile("s_waitcnt lgkmcnt(0)"
               : "+v"(f.a[0]), "+v"(f.a[1]), "+v"(f.a[2]), "+v"(f.a[3]), "+v"(f.b[0]), "+v"(f.b[1]));
}
#define QL_WAIT_FRAGS(f) wait_frags(f)
// The MFMAs are volatile asm like the LDS reads and waits, so the instruction order below IS the program order:
// left to the scheduler, the reads of the next sub-step sank behind the rows that free their registers, the last
// ones three MFMAs before the wait that needs them, and every sub-step began with an exposed LDS latency (the
// MFMA pipes measured 62 % busy).
#define QL_MFMA(c, a, b) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b))
#define QL_MMA_ROW(f, i)                                                                                    \
  _Pragma("unroll") for (int ni_ = 0; ni_ < NI; ++ni_) QL_MFMA(acc[i][ni_], f.a[i], f.b[ni_]);

// BN = 256 is the main configuration.  BN = 128 serves the columns left over when the 256-wide tiles do not fill
// a whole number of rounds of the 256 CUs: half-width tiles finish that last, partly filled round in half the time.
// NW = waves per workgroup, laid out 2 x NW/2: wave tiles are 128 x (BN / (NW / 2)).  With NW = 8 every SIMD
// holds two waves, so one can issue MFMAs while the other sits at the barrier or waits for its fragments.
template <int BN, int NW>
__global__ __launch_bounds__(NW * 64) void gemm_nt_kernel(const GemmArgs p) {
  constexpr int WN = BN / (NW / 2);                          // wave tile width
  constexpr int NI = WN / 32;                                // MFMA columns per wave
  constexpr int NA = 16 / NW, NB = (BN / 16) / NW;           // DMA instructions per wave, step and operand
  static_assert(NI >= 2 && NA >= 1 && NB >= 1, "tile / wave split (the read schedule needs 4 NI >= 4 + NI)");
  constexpr int kStage = kOpBytes + BN * BK * 2;             // A tile + B tile
  __shared__ __attribute__((aligned(1024))) char smem[NST * kStage];             // 160 KB (120 KB for BN = 128)
  lchar* const lds = (lchar*)smem;

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;

  // ---- workgroup id -> output tile -------------------------------------------------------------
  const int n_tiles = p.tiles_m * p.tiles_n;
  int pid = blockIdx.x;
  {
    const int xcd = pid & 7, local = pid >> 3;
    const int q = n_tiles >> 3, rem = n_tiles & 7;
    pid = (xcd < rem) ? xcd * (q + 1) + local : rem * (q + 1) + (xcd - rem) * q + local;
  }
  const int per_group = GM * p.tiles_n;
  const int group = pid / per_group;
  const int first_m = group * GM;
  const int gsz = (p.tiles_m - first_m < GM) ? p.tiles_m - first_m : GM;
  const int in_group = pid - group * per_group;
  const int m0 = (first_m + in_group % gsz) * BM, n0 = p.n_begin + (in_group / gsz) * BN;

  // ---- per-lane global pointers of the 4 + 4 DMA instructions of a step ------------------------
  const int KT = p.KT0 + p.KT1;
  const int dma_chunk = ((lane & 3) ^ ((lane >> 4) & 3)) * 8;
  int a_rows[NA], b_rows[NB];
#pragma unroll
  for (int j = 0; j < NA; ++j) {
    const int r = (NW * j + wave) * 16 + (lane >> 2);
    a_rows[j] = (m0 + r < p.M) ? m0 + r : p.M - 1;          // clamp: padded rows are never stored
  }
#pragma unroll
  for (int j = 0; j < NB; ++j) {
    const int r = (NW * j + wave) * 16 + (lane >> 2);
    b_rows[j] = (n0 + r < p.N) ? n0 + r : p.N - 1;
  }
  const uint16_t* pa[NA];
  const uint16_t* pb[NB];
  auto seek = [&](auto& ptr, const auto& rows, int cnt, int k, bool is_a) {
    // pointers of step k (clamped to the last step); K segment 0 first, then segment 1
    const int kc = k < KT ? k : KT - 1;
    const bool s0 = kc < p.KT0;
    const uint16_t* base = is_a ? (s0 ? p.A0 : p.A1) : (s0 ? p.B0 : p.B1);
    const int64_t ld = is_a ? (s0 ? p.lda0 : p.lda1) : (s0 ? p.ldb0 : p.ldb1);
    const int kofs = (s0 ? kc : kc - p.KT0) * BK + dma_chunk;
#pragma unroll
    for (int j = 0; j < cnt; ++j) ptr[j] = base + (int64_t)rows[j] * ld + kofs;
  };
  // after issuing step k: move to step k + 1 (one add per pointer except at the segment switch)
  auto advance = [&](auto& ptr, const auto& rows, int cnt, int k, bool is_a) {
    if (k + 1 >= KT) return;                                // stay: the tail re-fetches the last tile
    if (k + 1 == p.KT0) { seek(ptr, rows, cnt, k + 1, is_a); return; }
#pragma unroll
    for (int j = 0; j < cnt; ++j) ptr[j] += BK;
  };

  // ---- per-lane LDS addresses of the fragments of the two 16-wide sub-steps ---------------------
  const int wm = wave / (NW / 2), wn = wave % (NW / 2);
  const int a_row = wm * 128 + (lane & 31), b_row = wn * WN + (lane & 31), half = lane >> 5;
  const uint32_t lds0 = (uint32_t)(uintptr_t)lds;
  uint32_t offA[2][4], offB[2][NI];
#pragma unroll
  for (int kk = 0; kk < 2; ++kk)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int ra = a_row + 32 * i, rb = b_row + 32 * i;
      offA[kk][i] = lds0 + ra * 64 + (((2 * kk + half) ^ ((ra >> 2) & 3)) * 16);
      if (i < NI) offB[kk][i] = lds0 + kOpBytes + rb * 64 + (((2 * kk + half) ^ ((rb >> 2) & 3)) * 16);
    }

  f32x16 acc[4][NI];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

  // ---- prologue: stages 0, 1 and 2 complete, the A half of stage 3 ----------------------------------
  // Steady state: the B tile of step k+3 goes out during the first half of step k, the A tile of
  // step k+4 during the second half, each DMA instruction behind one row of MFMAs.  A tile is thus
  // requested 2.5 - 3 steps (about 1.5 us) before the barrier that publishes it: with one step less
  // (four stages) every step waited ~0.3 us for tiles that miss the XCD's L2, and the MFMA pipes were
  // busy 62 % of the time.
  seek(pa, a_rows, NA, 0, true);
  seek(pb, b_rows, NB, 0, false);
#pragma unroll
  for (int s = 0; s < 3; ++s) {
#pragma unroll
    for (int j = 0; j < NA; ++j) dma16<NW>(pa[j], lds + s * kStage, j, wave);
#pragma unroll
    for (int j = 0; j < NB; ++j) dma16<NW>(pb[j], lds + s * kStage + kOpBytes, j, wave);
    advance(pa, a_rows, NA, s, true);
    advance(pb, b_rows, NB, s, false);
  }
#pragma unroll
  for (int j = 0; j < NA; ++j) dma16<NW>(pa[j], lds + 3 * kStage, j, wave);
  advance(pa, a_rows, NA, 3, true);
  // stage 0 landed; stages 1, 2 and the A half of stage 3 (2 (NA + NB) + NA instructions) in flight
  wait_vmcnt<2 * (NA + NB) + NA>();
  asm volatile("s_barrier" ::: "memory");

  Frags<NI> f0, f1;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    QL_LDS_READ(f0.a[i], offA[0][i]);
    if (i < NI) QL_LDS_READ(f0.b[i], offB[0][i]);
  }

  // One 16-wide sub-step: multiply fragments `cur` while fetching fragments `nxt` (stage `st`,
  // sub-step kk) and issuing the 4 DMA instructions `ptr` into tile `dst`.
#define QL_SUBSTEP(cur, nxt, st, kk, ptr, dst, ndma)                                                        \
  {                                                                                                         \
    const uint32_t sb_ = (st) * kStage;                                                                     \
    QL_WAIT_FRAGS(cur);                                                                                     \
    /* One fragment read of the next sub-step behind each of the first 4 + NI MFMAs (issued in the MFMA's */ \
    /* shadow, and landed long before the next wait); one DMA instruction behind each row.               */ \
    _Pragma("unroll") for (int i_ = 0; i_ < 4; ++i_) {                                                      \
      _Pragma("unroll") for (int ni_ = 0; ni_ < NI; ++ni_) {                                                \
        QL_MFMA(acc[i_][ni_], cur.a[i_], cur.b[ni_]);                                                       \
        const int r_ = i_ * NI + ni_;                        /* MFMA number; reads 0 .. 3 + NI: a[], then b[] */ \
        if (r_ < 4) QL_LDS_READ(nxt.a[r_ & 3], offA[kk][r_ & 3] + sb_);                                     \
        else if (r_ < 4 + NI) QL_LDS_READ(nxt.b[(r_ - 4) % NI], offB[kk][(r_ - 4) % NI] + sb_);             \
      }                                                                                                     \
      if (i_ < (ndma)) dma16<NW>(ptr[i_], dst, i_, wave);                                                       \
    }                                                                                                       \
  }
  // One K-step; ST is the (static) stage of step k.
#define QL_STEP(ST)                                                                                         \
  {                                                                                                         \
    QL_SUBSTEP(f0, f1, ST, 1, pb, lds + ((ST + 3) % NST) * kStage + kOpBytes, NB)   /* B of step k+3 */     \
    advance(pb, b_rows, NB, k + 3, false);                                                                  \
    /* stage k+1 has landed (this wave's part): only A, B of k+2 and k+3 may still be in flight */          \
    wait_vmcnt<2 * (NA + NB)>();                                                                            \
    asm volatile("s_barrier" ::: "memory");                   /* ... and everyone's; stage k-1 is free */   \
    QL_SUBSTEP(f1, f0, (ST + 1) % NST, 0, pa, lds + ((ST + 4) % NST) * kStage, NA)  /* A of step k+4 */     \
    advance(pa, a_rows, NA, k + 4, true);                                                                   \
    ++k;                                                                                                    \
  }

  int k = 0;
#pragma unroll 1
  while (k + 5 <= KT) {
    QL_STEP(0) QL_STEP(1) QL_STEP(2) QL_STEP(3) QL_STEP(4)
  }
  if (k < KT) QL_STEP(0)
  if (k < KT) QL_STEP(1)
  if (k < KT) QL_STEP(2)
  if (k < KT) QL_STEP(3)
#undef QL_STEP
#undef QL_SUBSTEP
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");  // drain the tail's redundant loads and reads

  // ---- epilogue: one rounding to bf16; lane owns column n, rows 8*(v/4) + 4*half + v%4 ----------
#pragma unroll
  for (int ni = 0; ni < NI; ++ni) {
    const int n = n0 + wn * WN + ni * 32 + (lane & 31);
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

}  // namespace

hipError_t launch_gemm_nt(const uint16_t* A0, const uint16_t* B0, int64_t lda0, int64_t ldb0, int K0,
                          const uint16_t* A1, const uint16_t* B1, int64_t lda1, int64_t ldb1, int K1,
                          uint16_t* C, int64_t ldc, int M, int N, hipStream_t st) {
  GemmArgs a;
  a.A0 = A0; a.B0 = B0; a.lda0 = lda0; a.ldb0 = ldb0; a.KT0 = K0 / BK;
  a.A1 = A1; a.B1 = B1; a.lda1 = lda1; a.ldb1 = ldb1; a.KT1 = K1 / BK;
  a.C = C; a.ldc = ldc; a.M = M; a.N = N;
  a.tiles_m = (M + BM - 1) / BM;
  const int tiles_n = (N + 255) / 256;
  // One workgroup per CU: tiles run in rounds of 256.  When the last round would be at most half full and is made
  // of whole tile columns, those columns go to a second launch with half-width tiles (twice as many workgroups,
  // half the time each) instead of occupying a full round.
  constexpr int kCUs = 256;
  const int total = a.tiles_m * tiles_n;
  const int rem = total % kCUs;
  int tail_cols = 0;
  if (total > kCUs && rem > 0 && 2 * rem <= kCUs && rem % a.tiles_m == 0) tail_cols = rem / a.tiles_m;
  a.n_begin = 0;
  a.tiles_n = tiles_n - tail_cols;
  hipLaunchKernelGGL((gemm_nt_kernel<256, kMainWaves>), dim3((unsigned)(a.tiles_m * a.tiles_n)), dim3(kMainWaves * 64), 0, st,
                     a);
  if (tail_cols > 0) {
    a.n_begin = a.tiles_n * 256;
    a.tiles_n = (N - a.n_begin + 127) / 128;
    hipLaunchKernelGGL((gemm_nt_kernel<128, 4>), dim3((unsigned)(a.tiles_m * a.tiles_n)), dim3(256), 0, st, a);
  }
  return hipGetLastError();
}

}  // namespace qlora
