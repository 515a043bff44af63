// Few-token (M <= 16) forward and input-gradient of the QLoRA linear layer (arXiv 2305.14314,
// Eq. 5 / Eq. 6 at generation-time batch sizes): bandwidth-bound streaming kernels that read the
// packed NF4 weight and its double-quantised constants exactly once (0.516 B per weight),
// dequantise in registers to the same bf16 values as the standalone doubleDequant, and feed
// MFMA 16x16x32 with the tokens as the 16-wide dimension.  Two launches per call:
//
//   main    : part[split][m][n]  = partial sums of X * What   (forward)  or  dY * What^T (backward)
//             lpart[p][m][j]     = partial sums of the adapter's inner product T = X L1 or U = dY L2^T,
//                                  computed by a few extra workgroups of the same launch
//   finalize: out = bf16( sum of splits + s * (sum of lpart) * L2 )   resp.  ... * L1^T   -- one rounding
//
// The main loop keeps kDepth steps of global loads in flight per wave (a wave only runs 4-16 steps,
// so without explicit prefetch every step would expose the full HBM latency).
// NF4 decode uses a byte -> (value[lo nibble], value[hi nibble]) table in LDS, one 64-bit LDS read per
// two weights.  The table is replicated 32 times with the copies interleaved at 8-byte granularity
// (entry e of copy c at byte 256 e + 8 c), so lane l always reads the two banks of copy l % 32 whatever
// the entry: data-dependent lookups are bank-conflict free (a single shared copy measured ~3.5-way
// conflicts and bounded the kernels at 1.4 TB/s).
#include "common.hpp"
#include "launch.hpp"

namespace qlora {

namespace {

constexpr int kFewThreads = 512;             // 8 waves share one replicated decode table
constexpr int kLutCopies = 32;
constexpr int kDepth = 4;                    // steps of loads in flight per wave
constexpr int kLoraK = 2048;                 // forward: rows of L1 per adapter workgroup
constexpr int kLoraN = 4096;                 // backward: columns of L2 per adapter workgroup

__device__ __forceinline__ void init_pair_lut(f32x2* lut2 /* [256][32] */, float* unit /* [256] */) {
  constexpr float t[16] = {QLORA_NF4_VALUES};
  for (int e = threadIdx.x; e < 256 * kLutCopies; e += kFewThreads) {
    const int b = e / kLutCopies;
    f32x2 v;
    v[0] = t[b & 15];
    v[1] = t[b >> 4];
    lut2[e] = v;
  }
  if (threadIdx.x < 256) unit[threadIdx.x] = e4m3_unit(threadIdx.x);
}
// (value[lo nibble], value[hi nibble]) of byte `b` from this lane's copy of the table
__device__ __forceinline__ f32x2 pair_lookup(const f32x2* lut2, uint32_t b, int lane) {
  return lut2[b * kLutCopies + (lane & (kLutCopies - 1))];
}

struct FewArgs {
  const uint16_t* X; int M;                  // tokens x contraction dim (X for forward, dY for backward)
  const uint8_t* packed; const uint8_t* code; const float* c1; const float* mean;
  int h, o;
  float* part;                               // [splits][M][N]
  int per_split;                             // contraction elements per split
  int n_slabs, splits;
  // adapter inner product, handled by workgroups with blockIdx.x >= n_slabs * splits
  const uint16_t* L; int r;                  // forward: L1 (h x r); backward: L2 (r x o)
  float* lpart;                              // [n_lora_wgs][M][r]
};

// ---- adapter partials -----------------------------------------------------------------------------
// Both run on MFMA 16x16x32 with the tokens as one 16-wide dimension and 16 rank columns as the other,
// kDepth steps of loads in flight, and a cross-wave sum through LDS; one partial slot per workgroup.
//
// forward: lpart[wg][m][j] = sum over k in [kLoraK * wg, +kLoraK) of X[m][k] * L1[k][j]
// L1 is [h][r] (rank contiguous), so a fragment of 8 consecutive k for one rank column is gathered from
// 8 rows: lane (i, g) loads columns 4i .. 4i+3 of rows kb + 8g + j and splits them with byte permutes.
struct LFwdStep { uint32_t l[8][2]; u32x4 x; };

__device__ void lora_fwd_partial(const FewArgs& p, int wg, float* red /* [8][16][64] */) {
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;   // wave index is uniform
  const int i = lane & 15, g = lane >> 4;
  const int k_begin = wg * kLoraK;
  const int k_end = (k_begin + kLoraK < p.h) ? k_begin + kLoraK : p.h;
  const int stride = 8 * 32, kb0 = k_begin + wave * 32;      // 8 waves interleave 32-row steps
  float* out = p.lpart + (int64_t)wg * p.M * p.r;
  for (int j0 = 0; j0 < p.r; j0 += 64) {
    const bool col_ok = j0 + 4 * i < p.r;                    // r % 16 == 0: the 4 columns are in or out together
    auto load_step = [&](LFwdStep& s, int kb) {
      // loads are unconditional (addresses clamped into the tensor), values are masked afterwards:
      // a guarded load would become a branch and force a full wait at every join
      const bool x_ok = i < p.M && kb + 8 * g < k_end;
      const u32x4 xv = *(const u32x4*)(p.X + (x_ok ? (int64_t)i * p.h + kb + 8 * g : 0));
      s.x = x_ok ? xv : u32x4{0u, 0u, 0u, 0u};
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int k = kb + 8 * g + j;
        const bool ok = col_ok && k < k_end;
        const uint32_t* src = (const uint32_t*)(p.L + (ok ? (int64_t)k * p.r + j0 + 4 * i : 0));
        const uint32_t v0 = src[0], v1 = src[1];
        s.l[j][0] = ok ? v0 : 0u;
        s.l[j][1] = ok ? v1 : 0u;
      }
    };
    f32x4 acc[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) acc[e] = f32x4{0.f, 0.f, 0.f, 0.f};
    LFwdStep buf[kDepth];
#pragma unroll
    for (int d = 0; d < kDepth; ++d) load_step(buf[d], kb0 + d * stride);
    for (int kb = kb0; kb < k_end; kb += kDepth * stride) {
#pragma unroll
      for (int d = 0; d < kDepth; ++d) {
        if (kb + d * stride < k_end) {
          const bf16x8 xa = __builtin_bit_cast(bf16x8, buf[d].x);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
            u32x4 w;
#pragma unroll
            for (int jp = 0; jp < 4; ++jp)
              w[jp] = __builtin_amdgcn_perm(buf[d].l[2 * jp + 1][e >> 1], buf[d].l[2 * jp][e >> 1], sel);
            acc[e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa, __builtin_bit_cast(bf16x8, w), acc[e], 0, 0, 0);
          }
          load_step(buf[d], kb + (d + kDepth) * stride);
        }
      }
    }
    __syncthreads();                                         // previous chunk's sums have been read
    float* my = red + wave * (16 * 64);
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
      for (int vv = 0; vv < 4; ++vv) my[(4 * g + vv) * 64 + 4 * i + e] = acc[e][vv];
    __syncthreads();
    for (int idx = threadIdx.x; idx < p.M * 64; idx += kFewThreads) {
      const int m = idx >> 6, c = idx & 63;
      if (j0 + c < p.r) {
        float t = 0.0f;
#pragma unroll
        for (int w = 0; w < 8; ++w) t += red[w * 16 * 64 + idx];
        out[(int64_t)m * p.r + j0 + c] = t;
      }
    }
  }
}

// backward: lpart[wg][m][j] = sum over n in [kLoraN * wg, +kLoraN) of dY[m][n] * L2[j][n]
// Both operands are contiguous along n: fragments are plain 16-byte loads.
struct LBwdStep { u32x4 l[4]; u32x4 y; };

__device__ void lora_bwd_partial(const FewArgs& p, int wg, float* red /* [8][16][64] */) {
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;   // wave index is uniform
  const int i = lane & 15, g = lane >> 4;
  const int n_begin = wg * kLoraN;
  const int n_end = (n_begin + kLoraN < p.o) ? n_begin + kLoraN : p.o;
  const int stride = 8 * 32, nb0 = n_begin + wave * 32;      // 8 waves interleave 32-column steps
  float* out = p.lpart + (int64_t)wg * p.M * p.r;
  for (int j0 = 0; j0 < p.r; j0 += 64) {
    auto load_step = [&](LBwdStep& s, int nb) {
      const bool ok = nb + 8 * g < n_end;                    // o % 64 == 0
      const bool y_ok = i < p.M && ok;
      const u32x4 yv = *(const u32x4*)(p.X + (y_ok ? (int64_t)i * p.o + nb + 8 * g : 0));
      s.y = y_ok ? yv : u32x4{0u, 0u, 0u, 0u};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int j = j0 + 16 * e + i;
        const bool l_ok = j < p.r && ok;
        const u32x4 lv = *(const u32x4*)(p.L + (l_ok ? (int64_t)j * p.o + nb + 8 * g : 0));
        s.l[e] = l_ok ? lv : u32x4{0u, 0u, 0u, 0u};
      }
    };
    f32x4 acc[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) acc[e] = f32x4{0.f, 0.f, 0.f, 0.f};
    LBwdStep buf[kDepth];
#pragma unroll
    for (int d = 0; d < kDepth; ++d) load_step(buf[d], nb0 + d * stride);
    for (int nb = nb0; nb < n_end; nb += kDepth * stride) {
#pragma unroll
      for (int d = 0; d < kDepth; ++d) {
        if (nb + d * stride < n_end) {
          const bf16x8 ya = __builtin_bit_cast(bf16x8, buf[d].y);
#pragma unroll
          for (int e = 0; e < 4; ++e)
            acc[e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ya, __builtin_bit_cast(bf16x8, buf[d].l[e]), acc[e], 0, 0, 0);
          load_step(buf[d], nb + (d + kDepth) * stride);
        }
      }
    }
    __syncthreads();
    float* my = red + wave * (16 * 64);
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
      for (int vv = 0; vv < 4; ++vv) my[(4 * g + vv) * 64 + 16 * e + i] = acc[e][vv];
    __syncthreads();
    for (int idx = threadIdx.x; idx < p.M * 64; idx += kFewThreads) {
      const int m = idx >> 6, c = idx & 63;
      if (j0 + c < p.r) {
        float t = 0.0f;
#pragma unroll
        for (int w = 0; w < 8; ++w) t += red[w * 16 * 64 + idx];
        out[(int64_t)m * p.r + j0 + c] = t;
      }
    }
  }
}

// ---- forward main ---------------------------------------------------------------------------------
// W is [h][o], o contiguous.  A workgroup owns 128 output columns and a range of k rows; its 4 waves
// take interleaved 32-row steps and are summed through LDS at the end.  Lane (i = lane % 16,
// g = lane / 16) loads, for rows kb + 8g + j (j = 0..7), the packed dword of columns n0 + 8i .. +7;
// MFMA e (0..7) multiplies the 16 tokens with columns {n0 + 8i + e}.  The 64 constants of a step
// (32 rows x 2 blocks) are decoded one per lane and exchanged through a wave-private LDS strip.
struct FwdStep { uint32_t pk[8]; u32x4 x; uint32_t code; float c1; };   // raw loads only: nothing here is consumed before compute()

__global__ __launch_bounds__(kFewThreads) void fewtok_fwd_kernel(const FewArgs p) {
  __shared__ f32x2 lut2[256 * kLutCopies];                           // 64 KB
  __shared__ float unit[256];
  __shared__ __attribute__((aligned(16))) float red[4 * 16 * 128];   // per-wave output tiles of one column half
  __shared__ __attribute__((aligned(16))) float strip[8][2][32];     // per-wave constants: [block half][row]
  const int n_main = p.n_slabs * p.splits;
  if ((int)blockIdx.x >= n_main) { lora_fwd_partial(p, blockIdx.x - n_main, red); return; }   // uses 16 KB of red
  init_pair_lut(lut2, unit);
  __syncthreads();

  const int wave8 = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;  // uniform
  const int wave = wave8 & 3, chalf = wave8 >> 2;            // k interleave index, 128-column half of the slab
  const int i = lane & 15, g = lane >> 4;
  const int slab = blockIdx.x % p.n_slabs, split = blockIdx.x / p.n_slabs;
  const int n0 = slab * 256 + chalf * 128;
  const int k_begin = split * p.per_split;
  const int k_end = (k_begin + p.per_split < p.h) ? k_begin + p.per_split : p.h;
  const float mean = *p.mean;
  const int bpr = p.o >> 6, o_dw = p.o >> 3;
  const bool col_ok = n0 + 8 * i < p.o;                      // o % 64 == 0: a dword is in or out as a whole
  const uint32_t* packed = (const uint32_t*)p.packed;
  // the constant this lane decodes for a step: row kb + lane / 2, block half lane % 2
  const int c_blk = (n0 >> 6) + (lane & 1);
  const bool c_col_ok = c_blk < bpr;

  // Per-lane offsets are fixed for the whole kernel; a step only moves a wave-uniform base, so a load is
  // one instruction with no address arithmetic.  k ranges are multiples of 32 rows, so every row of a
  // step inside the range is valid; steps past the range (prefetch overrun) are redirected to the last
  // valid step and never consumed.  Lanes outside the tensor (columns >= o, tokens >= M) read a valid
  // dummy address and are masked once, at compute time.
  const int k_last = k_end - 32;
  uint32_t w_off[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) w_off[j] = (uint32_t)((8 * g + j) * o_dw + (col_ok ? (n0 >> 3) + i : 0));
  const bool x_row_ok = i < p.M;
  const uint32_t x_off = (uint32_t)((x_row_ok ? i : 0) * p.h + 8 * g);
  const uint32_t c_off = (uint32_t)((lane >> 1) * bpr + (c_col_ok ? c_blk : 0));
  auto load_step = [&](FwdStep& s, int kb) {
    const int kc = kb < k_end ? kb : k_last;                 // uniform
    const uint32_t* wbase = packed + (int64_t)kc * o_dw;
#pragma unroll
    for (int j = 0; j < 8; ++j) s.pk[j] = wbase[w_off[j]];
    s.x = *(const u32x4*)(p.X + kc + x_off);
    const int64_t cbase = (int64_t)kc * bpr;
    s.code = p.code[cbase + c_off];
    s.c1 = p.c1[(cbase + c_off) >> 8];
  };

  f32x4 acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = f32x4{0.f, 0.f, 0.f, 0.f};

  auto compute = [&](const FwdStep& s) {
    // dequant(c1, c2): two separately rounded fp32 steps; wave-private strip: no barrier needed
    strip[wave8][lane & 1][lane >> 1] = __fadd_rn(__fmul_rn(unit[s.code], s.c1), mean);
    const f32x4* sp = (const f32x4*)&strip[wave8][i >> 3][8 * g];
    const f32x4 ca = sp[0], cb = sp[1];
    const float c2[8] = {ca[0], ca[1], ca[2], ca[3], cb[0], cb[1], cb[2], cb[3]};
    float v[8][8];                                           // [row j][column e]
#pragma unroll
    for (int j = 0; j < 8; ++j) {
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const f32x2 q = pair_lookup(lut2, (s.pk[j] >> (8 * b)) & 0xffu, lane);
        v[j][2 * b] = __fmul_rn(q[0], c2[j]);
        v[j][2 * b + 1] = __fmul_rn(q[1], c2[j]);
      }
    }
    const bf16x8 xa = __builtin_bit_cast(bf16x8, x_row_ok ? s.x : u32x4{0u, 0u, 0u, 0u});
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      u32x4 w;
      w[0] = pack_bf16x2(v[0][e], v[1][e]);
      w[1] = pack_bf16x2(v[2][e], v[3][e]);
      w[2] = pack_bf16x2(v[4][e], v[5][e]);
      w[3] = pack_bf16x2(v[6][e], v[7][e]);
      acc[e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa, __builtin_bit_cast(bf16x8, w), acc[e], 0, 0, 0);
    }
  };

  // software pipeline over this wave's steps kb = k_begin + 32 * (wave + 4 t)
  const int stride = 4 * 32;
  const int kb0 = k_begin + wave * 32;
  FwdStep buf[kDepth];
#pragma unroll
  for (int d = 0; d < kDepth; ++d) load_step(buf[d], kb0 + d * stride);   // loads past k_end are masked off
  for (int kb = kb0; kb < k_end; kb += kDepth * stride) {
#pragma unroll
    for (int d = 0; d < kDepth; ++d) {
      if (kb + d * stride < k_end) {
        compute(buf[d]);
        load_step(buf[d], kb + (d + kDepth) * stride);
      }
    }
  }

  // D layout: column slot = lane % 16 (= i), token rows 4 * (lane / 16) + v.  The four waves of a column
  // half are summed through LDS, one half after the other.
  float* out = p.part + (int64_t)split * p.M * p.o;
  const int nbase = slab * 256;
  for (int hsel = 0; hsel < 2; ++hsel) {
    __syncthreads();
    if (chalf == hsel) {
      float* my = red + wave * (16 * 128);
#pragma unroll
      for (int e = 0; e < 8; ++e)
#pragma unroll
        for (int vv = 0; vv < 4; ++vv) my[(4 * g + vv) * 128 + 8 * i + e] = acc[e][vv];
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < p.M * 128; idx += kFewThreads) {
      const int m = idx >> 7, c = idx & 127;
      const int n = nbase + hsel * 128 + c;
      if (n < p.o)
        out[(int64_t)m * p.o + n] = red[idx] + red[16 * 128 + idx] + red[2 * 16 * 128 + idx] + red[3 * 16 * 128 + idx];
    }
  }
}

// ---- backward main --------------------------------------------------------------------------------
// Contraction runs along o, the contiguous dimension of W, so a lane's 16-byte load is 32 consecutive
// weights of one row and one quantisation constant.  A workgroup owns 128 weight rows (4 waves x 32)
// and a range of columns; per step of 128 columns a lane (i = lane % 16, g = lane / 16) loads rows
// r0 + i and r0 + 16 + i at columns kb + 32g .. +31; MFMA t (0..3) uses dword t of each load.
struct BwdStep { u32x4 w[2]; u32x4 y[4]; uint32_t code[2]; float c1[2]; };   // raw loads only

__global__ __launch_bounds__(kFewThreads) void fewtok_bwd_kernel(const FewArgs p) {
  __shared__ f32x2 lut2[256 * kLutCopies];                           // 64 KB
  __shared__ float unit[256];
  __shared__ __attribute__((aligned(16))) float red[8 * 16 * 64];    // cross-wave sum of the adapter workgroups
  const int n_main = p.n_slabs * p.splits;
  if ((int)blockIdx.x >= n_main) { lora_bwd_partial(p, blockIdx.x - n_main, red); return; }
  init_pair_lut(lut2, unit);
  __syncthreads();

  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;   // wave index is uniform
  const int i = lane & 15, g = lane >> 4;
  const int slab = blockIdx.x % p.n_slabs, split = blockIdx.x / p.n_slabs;
  const int r0 = slab * 256 + wave * 32;
  const int c_begin = split * p.per_split;
  const int c_end = (c_begin + p.per_split < p.o) ? c_begin + p.per_split : p.o;
  const float mean = *p.mean;
  const int bpr = p.o >> 6, o_q = p.o >> 5;                  // 16-byte groups (32 weights) per row
  const u32x4* packed = (const u32x4*)p.packed;

  // Fixed per-lane offsets, wave-uniform base per step (see the forward kernel).  The column range of a
  // split is a multiple of 64, a step is 128 wide: the last step may be half empty, which is masked on
  // the token operand (zeros) at compute time, with the weight loads redirected to valid addresses.
  const int c_last = c_end - 64;                             // start of the last valid 64-column block
  bool row_ok[2];
  uint32_t w_off[2], cd_off[2];
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int row = r0 + 16 * u + i;
    row_ok[u] = row < p.h;
    w_off[u] = (uint32_t)((row_ok[u] ? row : 0) * o_q);
    cd_off[u] = (uint32_t)((row_ok[u] ? row : 0) * bpr);
  }
  const bool y_row_ok = i < p.M;
  const uint32_t y_off = (uint32_t)((y_row_ok ? i : 0) * p.o);
  auto load_step = [&](BwdStep& s, int kb) {
    int col = kb + 32 * g;                                   // per lane
    if (col > c_last + 32) col = c_last + 32 * (g & 1);      // overrun: any valid column (masked at compute)
    const u32x4* wbase = packed + (col >> 5);
    const uint8_t* cbase = p.code + (col >> 6);
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      s.w[u] = wbase[w_off[u]];
      s.code[u] = cbase[cd_off[u]];
      s.c1[u] = p.c1[(cd_off[u] + (uint32_t)(col >> 6)) >> 8];
    }
    const uint16_t* ysrc = p.X + y_off + col;
#pragma unroll
    for (int t = 0; t < 4; ++t) s.y[t] = *(const u32x4*)(ysrc + 8 * t);
  };

  f32x4 acc[2];
  acc[0] = f32x4{0.f, 0.f, 0.f, 0.f};
  acc[1] = f32x4{0.f, 0.f, 0.f, 0.f};

  auto compute = [&](const BwdStep& s, int kb) {
    const bool y_ok = y_row_ok && kb + 32 * g < c_end;       // tokens >= M and columns past the split contribute zero
    float c2v[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) c2v[u] = __fadd_rn(__fmul_rn(unit[s.code[u]], s.c1[u]), mean);
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const bf16x8 ya = __builtin_bit_cast(bf16x8, y_ok ? s.y[t] : u32x4{0u, 0u, 0u, 0u});
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const uint32_t d = s.w[u][t];
        u32x4 w;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          const f32x2 q = pair_lookup(lut2, (d >> (8 * b)) & 0xffu, lane);
          w[b] = pack_bf16x2(__fmul_rn(q[0], c2v[u]), __fmul_rn(q[1], c2v[u]));
        }
        acc[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ya, __builtin_bit_cast(bf16x8, w), acc[u], 0, 0, 0);
      }
    }
  };

  BwdStep buf[kDepth];
#pragma unroll
  for (int d = 0; d < kDepth; ++d) load_step(buf[d], c_begin + d * 128);
  for (int kb = c_begin; kb < c_end; kb += kDepth * 128) {
#pragma unroll
    for (int d = 0; d < kDepth; ++d) {
      if (kb + d * 128 < c_end) {
        compute(buf[d], kb + d * 128);
        load_step(buf[d], kb + (d + kDepth) * 128);
      }
    }
  }

  float* out = p.part + (int64_t)split * p.M * p.h;
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

// ---- finalize -------------------------------------------------------------------------------------
// out[m][n] = bf16( sum_s part[s][m][n] + scale * sum_j T[m][j] * B(j, n) ),  T = sum_p lpart[p]
// forward: B(j, n) = L2[j][n] (Bmat is r x N); backward: B(j, n) = L1[n][j] (Bmat is N x r).
// Workgroup 0 also stores T as a [hi | lo] bf16 pair (M x 2r) when hl is given.
struct FinArgs {
  const float* part; int splits; int M, N;
  const float* lpart; int n_lparts; int r; float scale;
  const uint16_t* Bmat;
  uint16_t* out; uint16_t* hl;
};

constexpr int kFinThreads = 256;

template <bool BWD>
__global__ __launch_bounds__(kFinThreads) void fewtok_finalize_kernel(const FinArgs p) {
  constexpr int RC = 128;                                    // rank columns staged at a time
  __shared__ float Ts[16 * 256];                             // T[m][j], unscaled
  constexpr int kBsPitch = RC + 8;                           // backward tile row pitch: keeps 16-byte alignment
  __shared__ __attribute__((aligned(16))) uint16_t Bs[128 * kBsPitch];   // adapter tile: forward [RC][128], backward [128][pitch]
  const int n0 = blockIdx.x * 128;
  for (int e = threadIdx.x; e < p.M * p.r; e += kFinThreads) {
    float s = 0.0f;
#pragma unroll 4
    for (int q = 0; q < p.n_lparts; ++q) s += p.lpart[(int64_t)q * p.M * p.r + e];
    Ts[e] = s;
    if (p.hl && blockIdx.x == 0) {
      const int m = e / p.r, j = e - m * p.r;
      const uint16_t hi = bf16_bits(s);
      p.hl[(int64_t)m * 2 * p.r + j] = hi;
      p.hl[(int64_t)m * 2 * p.r + p.r + j] = bf16_bits(s - bf16_lo_to_f32(hi));
    }
  }
  const int c = threadIdx.x & 127, mh = threadIdx.x >> 7;    // column within the slab, token half
  const int n = n0 + c;
  float acc[8], lora[8];
#pragma unroll
  for (int u = 0; u < 8; ++u) { acc[u] = 0.0f; lora[u] = 0.0f; }
  if (n < p.N) {
#pragma unroll 4
    for (int sp = 0; sp < p.splits; ++sp) {
      const float* ps = p.part + (int64_t)sp * p.M * p.N + n;
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int m = mh * 8 + u;
        if (m < p.M) acc[u] += ps[(int64_t)m * p.N];
      }
    }
  }
  for (int j0 = 0; j0 < p.r; j0 += RC) {
    const int rc = (p.r - j0 < RC) ? p.r - j0 : RC;
    __syncthreads();                                         // Ts written / previous tile consumed
    // all loads of the tile are issued at once (coalesced); the products below run out of LDS
    u32x4 stage[RC / 16];
    if (!BWD) {                                              // rows j of L2, 128 columns = 16 chunks of 16 bytes
#pragma unroll
      for (int it = 0; it < RC / 16; ++it) {
        const int j = it * 16 + (threadIdx.x >> 4), cc = (threadIdx.x & 15) * 8;
        stage[it] = u32x4{0u, 0u, 0u, 0u};
        if (j < rc && n0 + cc < p.N) stage[it] = *(const u32x4*)(p.Bmat + (int64_t)(j0 + j) * p.N + n0 + cc);
      }
#pragma unroll
      for (int it = 0; it < RC / 16; ++it) {
        const int j = it * 16 + (threadIdx.x >> 4), cc = (threadIdx.x & 15) * 8;
        if (j < rc) *(u32x4*)(Bs + j * 128 + cc) = stage[it];
      }
    } else {                                                 // rows n0 + c of L1, rc rank columns = rc / 8 chunks
      const int cpr = rc >> 3;                               // chunks per row
#pragma unroll
      for (int it = 0; it < RC / 16; ++it) {
        const int e = it * kFinThreads + threadIdx.x;
        const int cc = e / cpr, ch = e - cc * cpr;
        stage[it] = u32x4{0u, 0u, 0u, 0u};
        if (cc < 128 && n0 + cc < p.N) stage[it] = *(const u32x4*)(p.Bmat + (int64_t)(n0 + cc) * p.r + j0 + ch * 8);
      }
#pragma unroll
      for (int it = 0; it < RC / 16; ++it) {
        const int e = it * kFinThreads + threadIdx.x;
        const int cc = e / cpr, ch = e - cc * cpr;
        if (cc < 128) *(u32x4*)(Bs + cc * kBsPitch + ch * 8) = stage[it];
      }
    }
    __syncthreads();
    for (int j = 0; j < rc; ++j) {
      const float b = bf16_lo_to_f32(BWD ? Bs[c * kBsPitch + j] : Bs[j * 128 + c]);
#pragma unroll
      for (int u = 0; u < 8; ++u) lora[u] = __builtin_fmaf(Ts[(mh * 8 + u) * p.r + j0 + j], b, lora[u]);
    }
  }
  if (n >= p.N) return;
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    const int m = mh * 8 + u;
    if (m < p.M) p.out[(int64_t)m * p.N + n] = bf16_bits(acc[u] + p.scale * lora[u]);
  }
}

// One 8-wave workgroup occupies a CU (its decode table alone is 64 KB of LDS), so the launch is sized to
// fit the 256 CUs in a single round: slabs * splits + adapter workgroups <= 256 whenever possible.
int pick_splits(int slabs, int steps_total, int min_steps, int reserved) {
  int splits = (256 - reserved) / slabs;
  int cap = steps_total / min_steps;
  if (cap < 1) cap = 1;
  if (splits > cap) splits = cap;
  if (splits > 64) splits = 64;
  if (splits < 1) splits = 1;
  return splits;
}

}  // namespace

int fewtok_fwd_lparts(int h, int r) { return r > 0 ? (h + kLoraK - 1) / kLoraK : 0; }
int fewtok_bwd_lparts(int o, int r) { return r > 0 ? (o + kLoraN - 1) / kLoraN : 0; }
// the split count leaves room for the adapter workgroups of the largest rank (same workspace for every r)
int fewtok_fwd_splits(int h, int o) { return pick_splits((o + 255) / 256, (h + 31) / 32, 16, fewtok_fwd_lparts(h, 16)); }
int fewtok_bwd_splits(int h, int o) { return pick_splits((h + 255) / 256, (o + 127) / 128, 4, fewtok_bwd_lparts(o, 16)); }

hipError_t launch_fewtok_fwd(const uint16_t* X, int M, const NF4Dev& w, float* part, int splits, const uint16_t* L1,
                             int r, float* lpart, hipStream_t st) {
  FewArgs a;
  a.X = X; a.M = M; a.packed = w.packed; a.code = w.code; a.c1 = w.c1; a.mean = w.mean;
  a.h = (int)w.rows; a.o = (int)w.cols; a.part = part;
  const int steps = (a.h + 31) / 32;
  a.per_split = ((steps + splits - 1) / splits) * 32;
  a.n_slabs = (a.o + 255) / 256; a.splits = splits;
  a.L = L1; a.r = r; a.lpart = lpart;
  const int lora_wgs = fewtok_fwd_lparts(a.h, r);
  hipLaunchKernelGGL(fewtok_fwd_kernel, dim3((unsigned)(a.n_slabs * splits + lora_wgs)), dim3(kFewThreads), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_fewtok_bwd(const uint16_t* dY, int M, const NF4Dev& w, float* part, int splits, const uint16_t* L2,
                             int r, float* lpart, hipStream_t st) {
  FewArgs a;
  a.X = dY; a.M = M; a.packed = w.packed; a.code = w.code; a.c1 = w.c1; a.mean = w.mean;
  a.h = (int)w.rows; a.o = (int)w.cols; a.part = part;
  const int steps = (a.o + 127) / 128;
  a.per_split = ((steps + splits - 1) / splits) * 128;
  a.n_slabs = (a.h + 255) / 256; a.splits = splits;
  a.L = L2; a.r = r; a.lpart = lpart;
  const int lora_wgs = fewtok_bwd_lparts(a.o, r);
  hipLaunchKernelGGL(fewtok_bwd_kernel, dim3((unsigned)(a.n_slabs * splits + lora_wgs)), dim3(kFewThreads), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_fewtok_finalize(bool bwd, const float* part, int splits, int M, int N, const float* lpart,
                                  int n_lparts, int r, float scale, const uint16_t* Bmat, uint16_t* out, uint16_t* hl,
                                  hipStream_t st) {
  FinArgs a;
  a.part = part; a.splits = splits; a.M = M; a.N = N; a.lpart = lpart; a.n_lparts = n_lparts; a.r = r;
  a.scale = scale; a.Bmat = Bmat; a.out = out; a.hl = hl;
  dim3 grid((unsigned)((N + 127) / 128));
  if (bwd) hipLaunchKernelGGL(fewtok_finalize_kernel<true>, grid, dim3(kFinThreads), 0, st, a);
  else hipLaunchKernelGGL(fewtok_finalize_kernel<false>, grid, dim3(kFinThreads), 0, st, a);
  return hipGetLastError();
}

}  // namespace qlora
