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
// Design for gfx950 (256 CUs in 8 XCDs, 160 KB LDS):
//  * 256 x 256 output tile per workgroup of 4 waves (2 x 2), each wave 128 x 128 as 8 x 8 tiles of MFMA 16x16x32
//    bf16: 256 fp32 accumulators per lane (all AGPRs), one wave per SIMD.  The kernel is bound by the board's power
//    limit, not by issue slots: on the same Gaussian operands a register-only loop of 16x16x32 MFMAs sustains 6 %
//    more FLOP/s than one of 32x32x16 MFMAs (an accumulator is read and written once per 32 k instead of once
//    per 16), and the square wave tile reads a third less LDS per MFMA than 128 x 64.  Against 8 waves of 128 x 64
//    with 32x32x16 the same kernel measures 7 - 11 % faster per product, bit-identical results.
//  * K-step 64: a tile row is one whole 128-byte line.  With 32-wide steps every DMA instruction fetched 16 half
//    lines, each line was pulled from L2 twice (the L1 does not keep it for a step) and the MFMA pipes measured
//    67 % busy; the same kernel fetching whole lines (and nothing else changed) ran 5 - 17 % faster.
//  * Operand tiles (256 rows x 128 B = 32 KB) arrive by buffer_load_dwordx4 ... lds (no VGPR staging) into a ring
//    of five 32 KB slots -- all 160 KB of the CU -- in the order A(0) B(0) A(1) B(1) A(2) ...: tile n sits in slot
//    n % 5.  While step k is computed, A(k+1), B(k+1) and A(k+2) are resident or landing.
//  * A K-step is two 32-wide sub-steps (one MFMA 16x16x32 per accumulator tile each).  One barrier per K-step,
//    before its LAST sub-step (by then a wave holds the step's last fragments in registers): it publishes the
//    tiles of step k+1 -- so the first fragments of step k+1 are read during that last sub-step and the MFMA
//    stream continues across the step boundary -- and frees the two slots of step k, into which B(k+2) and A(k+3)
//    are requested over the following two sub-steps, one DMA instruction behind a row of MFMAs (waves issue in
//    order: a burst of DMAs would stall the MFMA stream).  B thus has one step (about 1 us) and A two steps to
//    arrive.
//  * Addresses cost no vector ALU instruction in the loop (VALU instructions share the MFMA's issue port): a DMA
//    instruction takes a buffer resource based at the tile's first row, a per-lane byte offset that never
//    changes and a scalar offset that advances by 128 per step; a fragment read takes one of a few base
//    registers plus a 16-bit immediate (slot, MFMA tile).
//  * Fragment reads are software-pipelined one sub-step ahead, one read behind each of the first MFMAs of a
//    sub-step; reads, MFMAs and waits are volatile asm so that this order is the program order, with
//    hand-placed s_waitcnt (the compiler's automatic waits cannot tell a DMA into one slot from a read of another
//    across the loop back-edge and would drain all DMAs every iteration).
//  * LDS rows are 128 bytes (64 k); the eight 16-byte chunks of row r sit at chunk ^ ((r >> 1) & 7).  LDS has 64
//    banks: a ds_read_b128 is served 16 lanes (256 bytes) per cycle -- the 16 rows of one operand tile at one
//    logical chunk -- which alternate between the two halves of the bank space while the swizzle spreads the 8
//    rows of each half over its 8 sixteen-byte groups: no bank conflicts (counter-checked).
//  * Workgroup ids are remapped so each XCD (which receives every 8th id) works on a contiguous
//    range of the tile order, and tiles are ordered in groups of GM tile-rows, so the 32 tiles
//    resident on an XCD share A and B tiles in that XCD's L2.
//  * Rows beyond M / N are clamped for loads and masked at the store; steps beyond the last
//    re-fetch the last tile into a free slot, which keeps the loop body free of branches.
#include <algorithm>

#include "common.hpp"
#include "launch.hpp"

namespace qlora {

namespace {

constexpr int BM = 256, BK = 64, NSLOT = 5;                  // BN is 256, or 128 for the tail launch (template parameter)
constexpr int kSlot = BM * BK * 2;                           // 32 KB: one 256-row operand tile
constexpr int GM = 4;                                       // tile-rows per raster group
constexpr int kMainWaves = 4;                                // waves per workgroup of the main (BN = 256) kernel

typedef __attribute__((address_space(3))) char lchar;

struct GemmArgs {
  const uint16_t* A0; const uint16_t* B0; int64_t lda0, ldb0; int KT0;   // KT = K / BK
  const uint16_t* A1; const uint16_t* B1; int64_t lda1, ldb1; int KT1;
  uint16_t* C; int64_t ldc;
  int M, N, tiles_m, tiles_n;
  int n_begin;                                               // first output column of this launch
  // FUSED kernels: the weight-side operand of K segment 0 comes as 4-bit codes, N rows of K0 / 2 bytes (low nibble
  // first), with one fp32 constant per 64 codes (N x K0 / 64) and the data type's 16 values; B0 / ldb0 are unused.
  const uint8_t* Bq; const float* Bc; const float* tab;
};

template <int NI> struct Frags { bf16x8 a[8], b[NI]; };      // 16-row / 16-column MFMA operand tiles of one 32-wide sub-step

// One operand's DMA state.  The tile's rows are addressed through a buffer resource based at the tile's first
// row: a per-lane byte offset that never changes (row * ld + chunk) plus a scalar byte offset that advances by one
// K-step.
template <int CNT> struct Dma {
  __amdgpu_buffer_rsrc_t rsrc;
  int soff;                                                  // scalar byte offset of the current step
  int voff[CNT];                                             // per-lane byte offset of DMA instruction j
};
constexpr int kRsrcFlags = 0x00020000;                       // raw buffer, 32-bit data format
__device__ __forceinline__ __amdgpu_buffer_rsrc_t tile_rsrc(const uint16_t* base) {
  return __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, 0x7FFFFFFF, kRsrcFlags);
}
// one DMA instruction: 64 lanes x 16 bytes from rsrc + voff (per lane) + soff (scalar) to 1 KB of LDS at dst
__device__ __forceinline__ void dma16(__amdgpu_buffer_rsrc_t rsrc, lchar* dst, int voff, int soff) {
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (__attribute__((address_space(3))) void*)dst, 16, voff, soff, 0, 0);
}
template <int N> __device__ __forceinline__ void wait_vmcnt() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }

// A raw buffer resource over `bytes` bytes at `base`, in scalar registers.
__device__ __forceinline__ u32x4 raw_rsrc(const void* base, uint32_t bytes) {
  const uint64_t a = (uint64_t)base;
  u32x4 r;
  r[0] = __builtin_amdgcn_readfirstlane((uint32_t)a);
  r[1] = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32) & 0xffffu);
  r[2] = __builtin_amdgcn_readfirstlane(bytes);
  r[3] = kRsrcFlags;
  return r;
}
// One row of a fused weight tile as it arrives: 64 codes (32 bytes) and their block constant.
struct Codes { uint64_t q[4]; float c; };
// Five loads (4 x 8 + 4 bytes).  Like the fragment reads they are volatile asm with hand-placed waits, and the
// registers they land in are read by volatile asm only (QL_TAKE_CODES, after an s_waitcnt that covers the loads):
// the compiler takes an asm's outputs as written when the statement ends, so ordinary code that read `dst` could be
// scheduled (or a register copy inserted) in front of the wait.
#define QL_LOAD_CODES(dst, kstep)                                                                            \
  asm volatile("buffer_load_dwordx2 %0, %4, %5, %6 offen\n\tbuffer_load_dwordx2 %1, %4, %5, %6 offen offset:8\n\t" \
               "buffer_load_dwordx2 %2, %4, %5, %6 offen offset:16\n\tbuffer_load_dwordx2 %3, %4, %5, %6 offen offset:24" \
               : "=&v"((dst).q[0]), "=&v"((dst).q[1]), "=&v"((dst).q[2]), "=&v"((dst).q[3])                  \
               : "v"(q_voff), "s"(q_rsrc), "s"((kstep) * 32));                                               \
  asm volatile("buffer_load_dword %0, %1, %2, %3 offen" : "=&v"((dst).c) : "v"(c_voff), "s"(c_rsrc), "s"((kstep) * 4))
// to = from, for a `from` whose loads an earlier s_waitcnt has covered; `to` is then an ordinary value
#define QL_TAKE_CODES(to, from)                                                                              \
  asm volatile("v_mov_b64 %0, %5\n\tv_mov_b64 %1, %6\n\tv_mov_b64 %2, %7\n\tv_mov_b64 %3, %8\n\tv_mov_b32 %4, %9" \
               : "=&v"((to).q[0]), "=&v"((to).q[1]), "=&v"((to).q[2]), "=&v"((to).q[3]), "=&v"((to).c)       \
               : "v"((from).q[0]), "v"((from).q[1]), "v"((from).q[2]), "v"((from).q[3]), "v"((from).c))
// dword d (0 .. 3) of two 8-byte pieces
__device__ __forceinline__ uint32_t code_dword(uint64_t a, uint64_t b, int d) {
  const uint64_t v = d < 2 ? a : b;
  return (d & 1) ? (uint32_t)(v >> 32) : (uint32_t)v;
}
// dst = tab[nibble]: the 16 values sit in lanes 0 .. 15 (and again in 16 .. 31, ...); the permute takes bits 7:2 of
// the address as the lane, so the two bits above the nibble may hold anything.  Lands with the LDS counter.
#define QL_BPERM(dst, addr) asm volatile("ds_bpermute_b32 %0, %1, %2" : "=v"(dst) : "v"(addr), "v"(tabv))
// The first reader of a looked-up value, volatile for the same reason: it stays behind the wait that covers the lookup.
#define QL_MUL(dst, a, b) asm volatile("v_mul_f32 %0, %1, %2" : "=v"(dst) : "v"(a), "v"(b))
// 16 bytes to LDS; the idle cycles keep a vector-ALU write of the data registers away from the store that reads them
#define QL_LDS_WRITE(addr, data, imm) \
  asm volatile("ds_write_b128 %0, %1 offset:%2\n\ts_nop 1" ::"v"(addr), "v"(data), "n"(imm))

#define QL_LDS_READ(dst, addr, imm) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(imm))
__device__ __forceinline__ void wait_frags(Frags<4>& f) {
  asm volatile("s_waitcnt lgkmcnt(0)"
               : "+v"(f.a[0]), "+v"(f.a[1]), "+v"(f.a[2]), "+v"(f.a[3]), "+v"(f.a[4]), "+v"(f.a[5]), "+v"(f.a[6]),
                 "+v"(f.a[7]), "+v"(f.b[0]), "+v"(f.b[1]), "+v"(f.b[2]), "+v"(f.b[3]));
}
__device__ __forceinline__ void wait_frags(Frags<8>& f) {
  asm volatile("s_waitcnt lgkmcnt(0)"
               : "+v"(f.a[0]), "+v"(f.a[1]), "+v"(f.a[2]), "+v"(f.a[3]), "+v"(f.a[4]), "+v"(f.a[5]), "+v"(f.a[6]),
                 "+v"(f.a[7]), "+v"(f.b[0]), "+v"(f.b[1]), "+v"(f.b[2]), "+v"(f.b[3]), "+v"(f.b[4]), "+v"(f.b[5]),
                 "+v"(f.b[6]), "+v"(f.b[7]));
}
// The MFMAs are volatile asm like the LDS reads and waits, so the instruction order below IS the program order:
// left to the scheduler, the reads of the next sub-step sank behind the rows that free their registers, the last
// ones three MFMAs before the wait that needs them, and every sub-step began with an exposed LDS latency.
#define QL_MFMA(c, a, b) asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b))

// BN = 256 is the main configuration.  BN = 128 serves the columns left over when the 256-wide tiles do not fill
// a whole number of rounds of the 256 CUs: half-width tiles finish that last, partly filled round in half the time.
// NW = waves per workgroup, laid out 2 x NW/2: wave tiles are 128 x 128 (main configuration, 4 waves) or 128 x 64
// (the half-width tail).
//
// FUSED: the weight-side tiles of K segment 0 are never in HBM as bf16.  Lane l of wave w owns row 64 w + l of every
// such tile: it loads the row's 32 bytes of codes and its block constant two steps ahead, looks the 64 values up
// with ds_bpermute (a 16-entry table in the lanes of one register: no LDS space, which the ring takes whole),
// multiplies, rounds to bf16 -- the same two roundings as the standalone dequantisation, so the tile is bit-identical
// to it -- and writes the row into the slot a DMA would have filled, all of it between the MFMAs of the step
// before the tile is read.  The adapter segment (at most one step) then comes FIRST, so that every tile the loop
// produces is a decoded one; its weight-side tile is the only one a DMA still brings.
template <int BN, int NW, bool FUSED>
__global__ __launch_bounds__(NW * 64) void gemm_nt_kernel(const GemmArgs p) {
  constexpr int WN = BN / (NW / 2);                          // wave tile width: 64, or 128 for 4 waves on a 256-wide tile
  constexpr int NI = WN / 16;                                // MFMA columns per wave
  static_assert(NI == 4 || NI == 8, "wave tiles are 128 x 64 or 128 x 128");
  constexpr int NA = 32 / NW, NB = (BN / 8) / NW;            // DMA instructions per wave, step and operand
  constexpr int PER = (FUSED ? NA : NA + NB) / 2;            // DMA instructions per wave and sub-step
  static_assert((NA + NB) % 2 == 0 && PER <= 8, "DMA instructions are spread evenly over the two sub-steps");
  static_assert(!FUSED || (BN == 256 && NW == 4), "fused tiles: 256 rows, one per lane of the workgroup");
  __shared__ __attribute__((aligned(1024))) char smem[NSLOT * kSlot];             // 160 KB
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

  // ---- DMA state of the two operands ------------------------------------------------------------
  const int KT = p.KT0 + p.KT1;
  int a_rows[NA], b_rows[NB], a_chunk[NA], b_chunk[NB];      // row within the tile (clamped to the matrix), logical chunk
#pragma unroll
  for (int j = 0; j < NA; ++j) {
    const int r = (NW * j + wave) * 8 + (lane >> 3);
    a_rows[j] = (m0 + r < p.M) ? r : p.M - 1 - m0;          // clamp: padded rows are never stored
    a_chunk[j] = ((lane & 7) ^ ((r >> 1) & 7)) * 8;
  }
#pragma unroll
  for (int j = 0; j < NB; ++j) {
    const int r = (NW * j + wave) * 8 + (lane >> 3);
    b_rows[j] = (n0 + r < p.N) ? r : p.N - 1 - n0;
    b_chunk[j] = ((lane & 7) ^ ((r >> 1) & 7)) * 8;
  }
  Dma<NA> da;
  Dma<NB> db;
  // DMA instruction j of an operand tile: wave w of NW fills LDS rows (NW j + w) * 8 .. + 7 of the slot (1 KB);
  // lane l lands at row l / 8, physical chunk l % 8 (its offset selects the logical chunk
  // (l % 8) ^ ((row >> 1) & 7) of that row).
#define QL_DMA16(d, slot, j) dma16((d).rsrc, (slot) + (NW * (j) + wave) * 1024, (d).voff[j], (d).soff)
  // state for step k (clamped to the last step); K segment 0 first, then segment 1
  auto seek = [&](auto& d, const auto& rows, const auto& chunk, int cnt, int row0, int k, bool is_a) {
    const int kc = k < KT ? k : KT - 1;
    const bool s0 = FUSED ? kc >= p.KT1 : kc < p.KT0;        // FUSED: segment 1 first
    const uint16_t* base = is_a ? (s0 ? p.A0 : p.A1) : (s0 ? p.B0 : p.B1);
    const int64_t ld = is_a ? (s0 ? p.lda0 : p.lda1) : (s0 ? p.ldb0 : p.ldb1);
    d.rsrc = tile_rsrc(base + (int64_t)row0 * ld);
    d.soff = (FUSED ? (s0 ? kc - p.KT1 : kc) : (s0 ? kc : kc - p.KT0)) * (BK * 2);
#pragma unroll
    for (int j = 0; j < cnt; ++j) d.voff[j] = (rows[j] * (int)ld + chunk[j]) * 2;
  };
  // after issuing step k: move to step k + 1 (one scalar add except at the segment switch)
  auto advance = [&](auto& d, const auto& rows, const auto& chunk, int cnt, int row0, int k, bool is_a) {
    if (k + 1 >= KT) return;                                // stay: the tail re-fetches the last tile
    if (k + 1 == (FUSED ? p.KT1 : p.KT0)) { seek(d, rows, chunk, cnt, row0, k + 1, is_a); return; }
    d.soff += BK * 2;
  };

  // ---- per-lane LDS addresses of the fragments --------------------------------------------------
  // Sub-step kk (32 k) of a tile: logical chunks 4 kk .. 4 kk + 3 of row r, at physical chunk (4 kk + g) ^ ((r >> 1) & 7).
  // ds_read takes a 16-bit immediate: one base register per sub-step, operand and 64 KB window of the ring; the
  // slot within the window and the 32-row MFMA tile (4 KB apart, same swizzle) are immediates.
  const int wm = wave / (NW / 2), wn = wave % (NW / 2);
  // MFMA 16x16x32: lane (i = lane % 16, g = lane / 16) holds row i of a 16-row operand tile at k = 8 g .. 8 g + 7 of
  // the 32-wide sub-step kk, i.e. logical chunk 4 kk + g.  16-row tiles are 2 KB apart and share the swizzle.
  const int a_row = wm * 128 + (lane & 15), b_row = wn * WN + (lane & 15), g4 = lane >> 4;
  const uint32_t lds0 = (uint32_t)(uintptr_t)lds;
  // FUSED: this lane's row of the weight tiles (clamped to the matrix like the DMA rows), its two buffers, the
  // table value of its lane, and where the row lies in a slot: chunk d at (wbase ^ 16 d), the XOR being the swizzle.
  u32x4 q_rsrc = {0u, 0u, 0u, 0u}, c_rsrc = {0u, 0u, 0u, 0u};
  int q_voff = 0, c_voff = 0;
  float tabv = 0.0f;
  uint32_t wbase[3] = {0u, 0u, 0u};
  if constexpr (FUSED) {
    const int rc = fused_row(n0, tid, p.N);
    q_rsrc = raw_rsrc(p.Bq, (uint32_t)p.N * (uint32_t)p.KT0 * 32u);
    c_rsrc = raw_rsrc(p.Bc, (uint32_t)p.N * (uint32_t)p.KT0 * 4u);
    q_voff = (int)fused_code_offset(rc, 0, p.KT0);           // a step adds 32 (codes) / 4 (constant) bytes: the scalar offset
    c_voff = (int)fused_const_offset(rc, 0, p.KT0);
    tabv = p.tab[lane & 15];
#pragma unroll
    for (int w = 0; w < 3; ++w) wbase[w] = lds0 + w * 65536 + tid * 128 + ((tid >> 1) & 7) * 16;
  }
  // step of segment 0 behind tile t of the fused order (t >= KT1), clamped to the last
  auto seg0_step = [&](int t) { return fused_seg0_step(t, KT, p.KT1); };
  uint32_t baseA[2][3], baseB[2][3];
#pragma unroll
  for (int kk = 0; kk < 2; ++kk)
#pragma unroll
    for (int w = 0; w < 3; ++w) {
      baseA[kk][w] = lds0 + w * 65536 + a_row * 128 + (((4 * kk + g4) ^ ((a_row >> 1) & 7)) * 16);
      baseB[kk][w] = lds0 + w * 65536 + b_row * 128 + (((4 * kk + g4) ^ ((b_row >> 1) & 7)) * 16);
    }
#define QL_READ_A(dst, slot, kk, i) QL_LDS_READ(dst, baseA[kk][(slot) >> 1], ((slot) & 1) * kSlot + (i) * 2048)
#define QL_READ_B(dst, slot, kk, i) QL_LDS_READ(dst, baseB[kk][(slot) >> 1], ((slot) & 1) * kSlot + (i) * 2048)

  f32x4 acc[8][NI];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.0f;
  // The MFMAs below are inline asm, invisible to the compiler's hazard recogniser: a vector-ALU write of an
  // accumulator register needs 2 wait states before an MFMA reads it as its addend.  Pin every initialisation
  // in front of a few idle cycles (without this the compiler sank the zeroing of one accumulator right in front
  // of its first MFMA, which then read the register's old contents).
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j) asm volatile("s_nop 3" : "+a"(acc[i][j]));

  // ---- prologue: A(0) B(0) A(1) B(1) A(2) into slots 0 .. 4 ---------------------------------------
  Codes U = {}, L = {};                                      // FUSED: rows of tiles in use / landing (see QL_ITER)
  uint64_t Vhi0 = 0, Vhi1 = 0;                               // second half and constant of the row being written
  float Vc = 0.0f;
  float lk[32];                                              // 32 looked-up values: half a row
#pragma unroll
  for (int i = 0; i < 32; ++i) lk[i] = 0.0f;
  int kq = 0;                                                // step of segment 0 the next row load asks for
  if constexpr (FUSED) {
    // tile 0 is the adapter's when there is one (a DMA), every other weight-side tile is decoded: tiles 0 / 1 right
    // here, tile 2 from the first iteration on (its first half is looked up here), tile 3 is landing.
    seek(da, a_rows, a_chunk, NA, m0, 0, true);
#pragma unroll
    for (int j = 0; j < NA; ++j) QL_DMA16(da, lds + 0 * kSlot, j);
    advance(da, a_rows, a_chunk, NA, m0, 0, true);
    if (p.KT1 > 0) {
      seek(db, b_rows, b_chunk, NB, n0, 0, false);
#pragma unroll
      for (int j = 0; j < NB; ++j) QL_DMA16(db, lds + 1 * kSlot, j);
    }
#pragma unroll
    for (int j = 0; j < NA; ++j) QL_DMA16(da, lds + 2 * kSlot, j);
    advance(da, a_rows, a_chunk, NA, m0, 1, true);
#pragma unroll
    for (int j = 0; j < NA; ++j) QL_DMA16(da, lds + 4 * kSlot, j);
    advance(da, a_rows, a_chunk, NA, m0, 2, true);
    Codes l0 = {}, l1 = {}, l2 = {}, c0 = {}, c1 = {};
    QL_LOAD_CODES(l0, seg0_step(p.KT1));                     // tile 0 if there is no adapter (else unused)
    QL_LOAD_CODES(l1, seg0_step(1));
    QL_LOAD_CODES(l2, seg0_step(2));
    QL_LOAD_CODES(L, seg0_step(3));
    kq = 4 - p.KT1;                                          // the fast loop counts on from here without clamping
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    QL_TAKE_CODES(c0, l0);
    QL_TAKE_CODES(c1, l1);
    QL_TAKE_CODES(U, l2);
    auto decode_now = [&](const Codes& cd, int slot) {
#pragma unroll
      for (int d = 0; d < 8; ++d) {
        const uint32_t x = d < 4 ? code_dword(cd.q[0], cd.q[1], d & 3) : code_dword(cd.q[2], cd.q[3], d & 3);
        float t[8];
#pragma unroll
        for (int j = 0; j < 8; ++j)
          t[j] = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute((int)(j == 0 ? x << 2 : x >> (4 * j - 2)),
                                                                        __builtin_bit_cast(int, tabv)));
        u32x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = pack_bf16x2(__fmul_rn(t[2 * e], cd.c), __fmul_rn(t[2 * e + 1], cd.c));
        QL_LDS_WRITE((wbase[0] ^ (16u * d)) + slot * kSlot, o, 0);
      }
    };
    if (p.KT1 == 0) decode_now(c0, 1);
    decode_now(c1, 3);
#pragma unroll
    for (int w = 0; w < 32; ++w) {
      const uint32_t x = code_dword(U.q[0], U.q[1], w >> 3);
      QL_BPERM(lk[w], (w & 7) == 0 ? x << 2 : x >> (4 * (w & 7) - 2));
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    asm volatile("s_barrier" ::: "memory");
  } else {
    seek(da, a_rows, a_chunk, NA, m0, 0, true);
    seek(db, b_rows, b_chunk, NB, n0, 0, false);
#pragma unroll
    for (int s = 0; s < 2; ++s) {
#pragma unroll
      for (int j = 0; j < NA; ++j) QL_DMA16(da, lds + (2 * s) * kSlot, j);
#pragma unroll
      for (int j = 0; j < NB; ++j) QL_DMA16(db, lds + (2 * s + 1) * kSlot, j);
      advance(da, a_rows, a_chunk, NA, m0, s, true);
      advance(db, b_rows, b_chunk, NB, n0, s, false);
    }
#pragma unroll
    for (int j = 0; j < NA; ++j) QL_DMA16(da, lds + 4 * kSlot, j);
    advance(da, a_rows, a_chunk, NA, m0, 2, true);
    // A(0), B(0) landed; A(1), B(1), A(2) (2 NA + NB instructions) in flight
    wait_vmcnt<2 * NA + NB>();
    asm volatile("s_barrier" ::: "memory");
  }

  Frags<NI> f0, f1;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    QL_READ_A(f0.a[i], 0, 0, i);
    if (i < NI) QL_READ_B(f0.b[i], 1, 0, i);
  }

  // One 32-wide sub-step: multiply fragments `cur` while fetching fragments `nxt` (sub-step kk of the tiles in
  // slots sa, sb) and issuing this sub-step's share q0 .. q0 + PER - 1 of the step's DMA instructions: first the
  // NB of B(k+2) into slot db_, then the NA of A(k+3) into slot da_.  One fragment read behind each of the first
  // 8 + NI MFMAs (issued in the MFMA's shadow, and landed long before the next wait); one DMA behind each row.
#define QL_DMA_Q(q, da_, db_)                                                                               \
  if constexpr (FUSED) { QL_DMA16(da, lds + (da_) * kSlot, (q) < NA ? (q) : 0); }                           \
  else if ((q) < NB) QL_DMA16(db, lds + (db_) * kSlot, (q) < NB ? (q) : 0);                               \
  else QL_DMA16(da, lds + (da_) * kSlot, (q) >= NB ? (q) - NB : 0);
  // FUSED, behind MFMA number r_ of a sub-step: for r_ < 32 value r_ of the half row looked up during the previous
  // sub-step is multiplied by the block constant `cc_`, pairs are rounded to bf16, and every eighth value completes
  // a 16-byte chunk (number cb_ + r_ / 8 of the row) that goes to slot ws_; for r_ >= 32 value r_ - 32 of the next
  // half row (codes in src_) is looked up.  The waits at the sub-step boundaries cover the lookups.
#define QL_DEC(r_, ws_, cb_, cc_, s0_, s1_)                                                                 \
  if ((r_) < 32) {                                                                                          \
    QL_MUL(pr[(r_) & 1], lk[(r_)], cc_);                                                                    \
    if ((r_) & 1) ob[((r_) >> 1) & 3] = pack_bf16x2(pr[0], pr[1]);                                          \
    if (((r_) & 7) == 7) {                                                                                  \
      QL_LDS_WRITE(wbase[(ws_) >> 1] ^ (16u * ((cb_) + ((r_) >> 3))), ob, ((ws_) & 1) * kSlot);             \
    }                                                                                                       \
  } else {                                                                                                  \
    const uint32_t x_ = code_dword(s0_, s1_, ((r_) - 32) >> 3);                                             \
    QL_BPERM(lk[(r_) - 32], (((r_) & 7) == 0) ? x_ << 2 : x_ >> (((r_) & 7) ? 4 * ((r_) & 7) - 2 : 0));     \
  }                                                                                                         \
  __builtin_amdgcn_sched_barrier(0);
#define QL_SUBSTEP(cur, nxt, sa, sb, kk, q0, da_, db_, with_dma, dec_, cb_, cc_, s0_, s1_)                  \
  {                                                                                                         \
    wait_frags(cur);                                                                                        \
    u32x4 ob = {0u, 0u, 0u, 0u};                                                                            \
    float pr[2] = {0.0f, 0.0f};                                                                             \
    _Pragma("unroll") for (int i_ = 0; i_ < 8; ++i_) {                                                      \
      _Pragma("unroll") for (int nj_ = 0; nj_ < NI; ++nj_) {                                                \
        const int ni_ = (i_ & 1) ? NI - 1 - nj_ : nj_;       /* serpentine: consecutive MFMAs share an operand */ \
        QL_MFMA(acc[i_][ni_], cur.b[ni_], cur.a[i_]);        /* D = (B tile) (A tile)^T: see the epilogue */      \
        const int r_ = i_ * NI + nj_;                        /* MFMA number; reads 0 .. 7 + NI: a[], then b[] */ \
        if (r_ < 8) QL_READ_A(nxt.a[r_ & 7], sa, kk, r_ & 7);                                               \
        else if (r_ < 8 + NI) QL_READ_B(nxt.b[(r_ - 8) % NI], sb, kk, (r_ - 8) % NI);                       \
        if constexpr (FUSED) {                                                                              \
          if (dec_) { QL_DEC(r_, db_, cb_, cc_, s0_, s1_) }                                                 \
        }                                                                                                   \
      }                                                                                                     \
      if ((with_dma) && i_ < PER) { QL_DMA_Q((q0) + i_, da_, db_) }                                         \
    }                                                                                                       \
  }
  // Sub-step 0 of a step whose tiles sit in slots SA, SB (its fragments are in f0).
#define QL_HEAD(SA, SB) QL_SUBSTEP(f0, f1, SA, SB, 1, 0, 0, 0, false, false, 0, Vc, Vhi0, Vhi1)
  // One iteration: the second sub-step of step k (tiles in slots S0 = 2k % 5 and S0 + 1) and the first of step k+1
  // (slots S0 + 2, S0 + 3), requesting B(k+2) into slot S0 and A(k+3) into slot S0 + 1.
#define QL_ITER(S0, FAST)                                                                                   \
  {                                                                                                         \
    constexpr int sa_ = ((S0) + 2) % NSLOT, sb_ = ((S0) + 3) % NSLOT, fa_ = (S0) % NSLOT, fb_ = ((S0) + 1) % NSLOT; \
    wait_frags(f1);                                           /* this wave has read all it needs of step k */ \
    wait_vmcnt<NA>();                                         /* its part of A(k+1), B(k+1) has landed      */ \
    if constexpr (FUSED) {                                                                                  \
      /* tile k+2: its first half was looked up during the previous sub-step; U moves on to tile k+3, */    \
      /* whose row, asked for a step ago, that wait has covered                                       */    \
      Vhi0 = U.q[2]; Vhi1 = U.q[3]; Vc = U.c;                                                               \
      QL_TAKE_CODES(U, L);                                                                                  \
    }                                                                                                       \
    asm volatile("s_barrier" ::: "memory");                   /* ... and everyone's; slots of step k are free */ \
    if constexpr (FUSED) {                                                                                  \
      if (!(FAST)) kq = seg0_step(k + 4);                                                                   \
      QL_LOAD_CODES(L, kq);                                                                                 \
      if (FAST) ++kq;                                                                                       \
    }                                                                                                       \
    QL_SUBSTEP(f1, f0, sa_, sb_, 0, 0 * PER, fb_, fa_, true, true, 0, Vc, Vhi0, Vhi1)                       \
    QL_SUBSTEP(f0, f1, sa_, sb_, 1, 1 * PER, fb_, fa_, true, true, 4, Vc, U.q[0], U.q[1])                   \
    if (FAST) {                                                                                             \
      if constexpr (!FUSED) db.soff += BK * 2;                                                              \
      da.soff += BK * 2;                                                                                    \
    } else {                                                                                                \
      if constexpr (!FUSED) advance(db, b_rows, b_chunk, NB, n0, k + 2, false);                             \
      advance(da, a_rows, a_chunk, NA, m0, k + 3, true);                                                    \
    }                                                                                                       \
    ++k;                                                                                                    \
  }

  QL_HEAD(0, 1)                                               // step 0, sub-step 0 (no DMA: the ring is full)
  int k = 0;                                                 // f1 holds the fragments of the last sub-step of step k
  // Steady state: every tile requested and every state advanced in these five iterations stays inside K segment 0
  // (the last advance moves A to step k + 8 < KT0), so the DMA state advances by one scalar add and no iteration
  // carries the branches and register copies of the segment switch.
#pragma unroll 1
  while (k + 8 < (FUSED ? KT : p.KT0)) {
    QL_ITER(0, true) QL_ITER(2, true) QL_ITER(4, true) QL_ITER(1, true) QL_ITER(3, true)
  }
#pragma unroll 1
  while (k + 5 < KT) {
    QL_ITER(0, false) QL_ITER(2, false) QL_ITER(4, false) QL_ITER(1, false) QL_ITER(3, false)
  }
  if (k + 1 < KT) QL_ITER(0, false)
  if (k + 1 < KT) QL_ITER(2, false)
  if (k + 1 < KT) QL_ITER(4, false)
  if (k + 1 < KT) QL_ITER(1, false)
  // the last sub-step of the last step; its fragments are in f1
  wait_frags(f1);
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) QL_MFMA(acc[i][ni], f1.b[ni], f1.a[i]);
#undef QL_ITER
#undef QL_HEAD
#undef QL_SUBSTEP
#undef QL_DEC
#undef QL_DMA_Q
#undef QL_DMA16
#undef QL_READ_A
#undef QL_READ_B
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");  // drain the tail's redundant loads
  if constexpr (FUSED) {
    // The last row load and the last lookups are never used, but they were in flight until that wait: naming their
    // registers here keeps the compiler from handing them to other values while the data could still land.
    asm volatile("" ::"v"(L.q[0]), "v"(L.q[1]), "v"(L.q[2]), "v"(L.q[3]), "v"(L.c));
    asm volatile("" ::"v"(lk[0]), "v"(lk[1]), "v"(lk[2]), "v"(lk[3]), "v"(lk[4]), "v"(lk[5]), "v"(lk[6]), "v"(lk[7]),
                 "v"(lk[8]), "v"(lk[9]), "v"(lk[10]), "v"(lk[11]), "v"(lk[12]), "v"(lk[13]), "v"(lk[14]), "v"(lk[15]));
    asm volatile("" ::"v"(lk[16]), "v"(lk[17]), "v"(lk[18]), "v"(lk[19]), "v"(lk[20]), "v"(lk[21]), "v"(lk[22]),
                 "v"(lk[23]), "v"(lk[24]), "v"(lk[25]), "v"(lk[26]), "v"(lk[27]), "v"(lk[28]), "v"(lk[29]), "v"(lk[30]),
                 "v"(lk[31]));
  }
  // likewise the other way: an MFMA's result may be read by the vector ALU only 18 wait states after its issue
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j) asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 3" : "+a"(acc[i][j]));

  // ---- epilogue: one rounding to bf16 ------------------------------------------------------------
  // The MFMAs take the weight-side fragment as their first operand, so an accumulator tile is the TRANSPOSE of
  // the output tile: lane (j = lane % 16, g = lane / 16) holds output row 16 mi + j and the four consecutive
  // columns 16 ni + 4 g .. + 3, which go out as one 8-byte store (a quarter of the store instructions of the
  // untransposed tile, whose lanes hold four rows of one column).  One 64-bit base per lane; tiles that lie wholly
  // inside M (all but the last tile-row) skip the per-row bound checks.  N % 4 == 0: a group of four columns is
  // inside or outside as a whole.
  const bool rows_inside = m0 + BM <= p.M;
  const int m_lane = m0 + wm * 128 + (lane & 15);            // first row this lane stores
  const int n_lane = n0 + wn * WN + 4 * g4;                  // its first column
  uint16_t* const cb = p.C + (int64_t)m_lane * p.ldc + n_lane;
#pragma unroll
  for (int mi = 0; mi < 8; ++mi) {
    if (!rows_inside && m_lane + mi * 16 >= p.M) continue;
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
      if (n_lane + ni * 16 >= p.N) continue;
      uint2 q;
      q.x = pack_bf16x2(acc[mi][ni][0], acc[mi][ni][1]);
      q.y = pack_bf16x2(acc[mi][ni][2], acc[mi][ni][3]);
      *(uint2*)(cb + (int64_t)(mi * 16) * p.ldc + ni * 16) = q;
    }
  }
}

}  // namespace

hipError_t launch_gemm_nt(const uint16_t* A0, const uint16_t* B0, int64_t lda0, int64_t ldb0, int K0,
                          const uint16_t* A1, const uint16_t* B1, int64_t lda1, int64_t ldb1, int K1,
                          uint16_t* C, int64_t ldc, int M, int N, hipStream_t st) {
  if (K0 <= 0 || K0 % BK != 0 || K1 < 0 || K1 % BK != 0) return hipErrorInvalidValue;
  if (N % 4 != 0 || ldc % 4 != 0 || ((uintptr_t)C & 7u)) return hipErrorInvalidValue;    // 8-byte output stores
  // a tile's rows are addressed with 32-bit byte offsets from its first row
  const int64_t ld_max = std::max(std::max(lda0, ldb0), std::max(K1 ? lda1 : 0, K1 ? ldb1 : 0));
  if (256 * ld_max * 2 + (int64_t)(K0 > K1 ? K0 : K1) * 2 >= (1ll << 31)) return hipErrorInvalidValue;
  GemmArgs a;
  a.Bq = nullptr; a.Bc = nullptr; a.tab = nullptr;
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
  hipLaunchKernelGGL((gemm_nt_kernel<256, kMainWaves, false>), dim3((unsigned)(a.tiles_m * a.tiles_n)),
                     dim3(kMainWaves * 64), 0, st, a);
  if (tail_cols > 0) {
    a.n_begin = a.tiles_n * 256;
    a.tiles_n = (N - a.n_begin + 127) / 128;
    hipLaunchKernelGGL((gemm_nt_kernel<128, 4, false>), dim3((unsigned)(a.tiles_m * a.tiles_n)), dim3(256), 0, st, a);
  }
  return hipGetLastError();
}

// ---- measurement aid: what the matrix pipes sustain on this board --------------------------------------------------
// One wave per SIMD on every CU runs independent 16x16x32 bf16 MFMAs on Gaussian operands held in registers, with no
// memory traffic at all (MODE 0), with the LDS fragment-read traffic of the main kernel's 128 x 128 wave tile (MODE 1:
// one ds_read_b128 per four MFMAs), or with that and the LDS write traffic of the operand tiles landing (MODE 2: one
// 16-byte write per lane and eight MFMAs, what the DMA of a 256 x 256 x 64 step puts into LDS per wave).  The board's
// power limit, not the issue rate, sets the result, and it depends on the operands' values: this is the ceiling the
// main GEMM's rate is to be read against.
namespace {
__device__ __forceinline__ float probe_gauss(uint32_t s) {
  auto pcg = [](uint32_t x) { x = x * 747796405u + 2891336453u; uint32_t w = ((x >> ((x >> 28) + 4)) ^ x) * 277803737u; return (w >> 22) ^ w; };
  const uint32_t a = pcg(s), b = pcg(a);
  return __builtin_sqrtf(-2.0f * __builtin_logf(((float)a + 1.0f) * 0x1p-32f)) * __builtin_cosf(6.2831853f * ((float)b * 0x1p-32f));
}
template <int MODE>
__global__ __launch_bounds__(256) void mfma_probe_kernel(float* out, int iters) {
  constexpr bool READS = MODE >= 1, WRITES = MODE >= 2;
  __shared__ float lds[8192];
  for (int i = threadIdx.x; i < 4096; i += 256) lds[i] = probe_gauss(i * 7u + blockIdx.x);
  __syncthreads();
  bf16x8 a[4], b[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      a[j][i] = (__bf16)probe_gauss(threadIdx.x * 64u + j * 8u + i);
      b[j][i] = (__bf16)probe_gauss(threadIdx.x * 64u + j * 8u + i + 99991u);
    }
  const uint32_t raddr = (uint32_t)(uintptr_t)lds + (threadIdx.x & 63) * 16u;
  f32x4 acc[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int i = 0; i < 16; ++i) asm volatile("s_nop 3" : "+a"(acc[i]));
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      QL_MFMA(acc[i], a[i & 3], b[i >> 2]);
      if (READS && (i & 3) == 3) QL_LDS_READ(a[(i >> 2) & 3], raddr, 0);
      if (WRITES && (i & 7) == 5) asm volatile("ds_write_b128 %0, %1 offset:16384" ::"v"(raddr), "v"(b[3]));
    }
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]));
  }
#pragma unroll
  for (int i = 0; i < 16; ++i) asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 3" : "+a"(acc[i]));
  float s = 0.0f;
#pragma unroll
  for (int i = 0; i < 16; ++i) s += acc[i][0];
  out[blockIdx.x * 256 + threadIdx.x] = s;
}
}  // namespace

// 256 workgroups x 4 waves x iters x 16 MFMAs of 2 * 16 * 16 * 32 flops; `out`: 256 * 256 floats of device memory.
hipError_t launch_mfma_probe(int mode, int iters, float* out, hipStream_t st) {
  if (iters <= 0 || iters > (1 << 20) || !out || mode < 0 || mode > 2) return hipErrorInvalidValue;
  if (mode == 2) hipLaunchKernelGGL(mfma_probe_kernel<2>, dim3(256), dim3(256), 0, st, out, iters);
  else if (mode == 1) hipLaunchKernelGGL(mfma_probe_kernel<1>, dim3(256), dim3(256), 0, st, out, iters);
  else hipLaunchKernelGGL(mfma_probe_kernel<0>, dim3(256), dim3(256), 0, st, out, iters);
  return hipGetLastError();
}

bool gemm_nt_fused_fits(int K0, int K1, int N) {
  return K0 > 0 && K0 % BK == 0 && (K1 == 0 || K1 == BK) && N > 0 && (int64_t)N * (K0 / 2) < (1ll << 31);
}

hipError_t launch_gemm_nt_fused(const uint16_t* A0, const uint8_t* Bq, const float* Bc, const float* tab16, int64_t lda0,
                                int K0, const uint16_t* A1, const uint16_t* B1, int64_t lda1, int64_t ldb1, int K1,
                                uint16_t* C, int64_t ldc, int M, int N, hipStream_t st) {
  if (!gemm_nt_fused_fits(K0, K1, N) || !Bq || !Bc || !tab16) return hipErrorInvalidValue;
  if (N % 4 != 0 || ldc % 4 != 0 || ((uintptr_t)C & 7u) || ((uintptr_t)Bq & 15u) || ((uintptr_t)Bc & 3u))
    return hipErrorInvalidValue;
  const int64_t ld_max = std::max(lda0, std::max(K1 ? lda1 : 0, K1 ? ldb1 : 0));
  if (256 * ld_max * 2 + (int64_t)(K0 > K1 ? K0 : K1) * 2 >= (1ll << 31)) return hipErrorInvalidValue;
  GemmArgs a;
  a.A0 = A0; a.B0 = nullptr; a.lda0 = lda0; a.ldb0 = 0; a.KT0 = K0 / BK;
  a.A1 = A1; a.B1 = B1; a.lda1 = lda1; a.ldb1 = ldb1; a.KT1 = K1 / BK;
  a.C = C; a.ldc = ldc; a.M = M; a.N = N;
  a.tiles_m = (M + BM - 1) / BM;
  a.tiles_n = (N + 255) / 256;
  a.n_begin = 0;
  a.Bq = Bq; a.Bc = Bc; a.tab = tab16;
  hipLaunchKernelGGL((gemm_nt_kernel<256, kMainWaves, true>), dim3((unsigned)(a.tiles_m * a.tiles_n)),
                     dim3(kMainWaves * 64), 0, st, a);
  return hipGetLastError();
}

}  // namespace qlora
