// Building blocks shared by the few-token (M <= 16) streaming kernels of the QLoRA linear layer
// (arXiv 2305.14314, Eq. 5 / Eq. 6 at generation-time batch sizes): the replicated byte -> (value, value)
// decode table in LDS, the per-layer argument block, the workgroup -> die map and the adapter's inner
// products T = X L1 and U = dY L2^T on MFMA 16x16x32.
#pragma once

#include "common.hpp"
#include "launch.hpp"

namespace qlora {
namespace few {

constexpr int kFewThreads = 1024;            // 16 waves share one replicated decode table (8 where 256 VGPRs are needed)
constexpr int kWaves = kFewThreads / 64;
constexpr int kLutCopies = 32;
constexpr int kBwdDepth = 2;
constexpr int kLoraDepth = 2;
constexpr int kLoraK = 1024;                 // forward: rows of L1 per adapter workgroup (short: they must not arrive last)
constexpr int kLoraN = 1024;                 // backward: columns of L2 per adapter workgroup

// LDS map of a main workgroup.  The decode table is dead once the main loop is over, so the cross-wave
// sums reuse the space from offset 0.
constexpr int kLutBytes = 256 * kLutCopies * 8;              // 64 KB
constexpr int kRedBytes = kWaves * 16 * 128 * 4;             // 128 KB: one 16 x 128 fp32 tile per wave
constexpr int kUnitOff = kRedBytes;                          // float[256]
constexpr int kStripOff = kUnitOff + 1024;                   // float[kWaves][2][32]
constexpr int kSmemBytes = kStripOff + kWaves * 256;
static_assert(kLutBytes <= kRedBytes && kSmemBytes <= 160 * 1024, "LDS map");

// The 16 values (NF4's from constants, another data type's from the arguments: Section 4) are staged in LDS by 16
// threads first (`stage`, 16 floats) -- a lane-indexed read of a constant array or of a by-value argument is a memory
// load per element.  Entry e = 32 b + copy of the table belongs to byte b = e / 32; thread t writes entries t, t + NT,
// ...: their low nibble (t / 32) % 16 is the same for all of them and their high nibble advances by NT / 512 per entry,
// so a thread reads the stage once for the low value and at compile-time positions for the high ones.
template <int NT>
__device__ __forceinline__ void init_pair_lut(f32x2* lut2 /* [256][32] */, float* unit /* [256] */, int dtype,
                                              const Table4& tab, float* stage) {
  static_assert(NT == 512 || NT == 1024, "entries per thread and their nibbles are worked out for these two");
  if (threadIdx.x < 16) {
    constexpr float t[16] = {QLORA_NF4_VALUES};
    float v = t[threadIdx.x];
    if (dtype != 0) {
#pragma unroll
      for (int i = 0; i < 16; ++i) v = (int)threadIdx.x == i ? tab.v[i] : v;
    }
    stage[threadIdx.x] = v;
  }
  __syncthreads();
  const int b0 = threadIdx.x / kLutCopies;                   // byte of this thread's first entry: < NT / 32
  const float lo = stage[b0 & 15];
#pragma unroll
  for (int k = 0; k < 256 * kLutCopies / NT; ++k) {
    const int hi_nibble = (NT == 512) ? k : 2 * k + (b0 >> 4);
    f32x2 v;
    v[0] = lo;
    v[1] = stage[hi_nibble];
    lut2[threadIdx.x + NT * k] = v;
  }
  if (threadIdx.x < 256) unit[threadIdx.x] = e4m3_unit(threadIdx.x);
}
// (value[lo nibble], value[hi nibble]) of byte B (0..3) of packed dword `pk`, from this lane's copy of the table.
// Entry e of copy c sits at byte offset 256 e + 8 c: the offset is assembled by one byte permute
// (byte 1 = the weight byte, byte 0 = 8 * copy), instead of shift, mask and add.
template <int B>
__device__ __forceinline__ f32x2 pair_lookup(const f32x2* lut2, uint32_t pk, uint32_t lane_off /* 8 * (lane % 32) */) {
  const uint32_t off = __builtin_amdgcn_perm(pk, lane_off, 0x0c0c0400u + ((uint32_t)B << 8));
  return *(const f32x2*)((const char*)lut2 + off);
}

// the same with the byte number as a (constant-folded) argument
__device__ __forceinline__ f32x2 pair_lookup_b(const f32x2* lut2, uint32_t pk, uint32_t lane_off, int b) {
  switch (b) {
    case 0: return pair_lookup<0>(lut2, pk, lane_off);
    case 1: return pair_lookup<1>(lut2, pk, lane_off);
    case 2: return pair_lookup<2>(lut2, pk, lane_off);
    default: return pair_lookup<3>(lut2, pk, lane_off);
  }
}

struct FewArgs {
  const uint16_t* X; int M;                  // tokens x contraction dim (X for forward, dY for backward)
  const uint8_t* packed; const uint8_t* code; const float* c1; const float* mean;
  int dtype; Table4 tab;                     // data type of the weight (0 = NF4) and, for the others, its 16 values
  int h, o;
  float* part;                               // [splits][M][N]
  int per_split;                             // contraction elements per split
  int n_slabs, splits;
  // adapter inner product, handled by the first n_lparts workgroups in work_index() order
  const uint16_t* L; int r;                  // forward: L1 (h x r); backward: L2 (r x o)
  float* lpart;                              // [n_lparts][M][r]
  int n_lparts;
  // output stage, run by the last workgroup to arrive at a slab
  unsigned* ctr;                             // arrival counters (split arrivals, adapter handshakes, adapter count); zero on entry and exit
  const uint16_t* Bmat;                      // forward: L2 (r x o); backward: L1 (h x r)
  float scale;
  uint16_t* out;                             // M x N bf16
  uint16_t* hl;                              // M x 2r: T (resp. U) as a [hi | lo] bf16 pair, or NULL
  int lora_chunk;                            // contraction elements per adapter workgroup (kLoraK / kLoraN in the one-layer kernels)
  // work-list kernels only
  unsigned* hdr;                             // start of the counter header (status word)
  unsigned nonce;                            // this call's tag, in bits 31:24 of every arrival word it touches
  int spin_limit;                            // polls of a slab's last contributor for the adapter's partials
};

// Workgroup b runs on die (XCD) b % 8, and each die has its own L2.  The work list -- adapter partials first,
// then (split, slab) pairs in split-major order -- is cut into 8 contiguous pieces, one per die, so that the
// workgroups of one split sit together: they read the same rows of the token operand and, in the forward, the
// same 128-byte lines of the 8-bit constants (a line holds one row's constants of 32 slabs).  With the plain
// b -> (b % n_slabs, b / n_slabs) map every die pulled every constant line: 1.5x the algorithmic HBM bytes.
__device__ __forceinline__ int work_index() {
  const int grid = gridDim.x, b = blockIdx.x;
  const int x = b & 7, q = b >> 3;
  return x * (grid >> 3) + (x < (grid & 7) ? x : (grid & 7)) + q;
}

// ---- adapter partials -----------------------------------------------------------------------------
// Both run on MFMA 16x16x32 with the tokens as one 16-wide dimension and 16 rank columns as the other,
// kLoraDepth steps of loads in flight, and a cross-wave sum through LDS; one partial slot per workgroup.
//
// forward: lpart[wg][m][j] = sum over k in [kLoraK * wg, +kLoraK) of X[m][k] * L1[k][j]
// L1 is [h][r] (rank contiguous), so a fragment of 8 consecutive k for one rank column is gathered from
// 8 rows: lane (i, g) loads columns 4i .. 4i+3 of rows kb + 8g + j and splits them with byte permutes.
struct LFwdStep { uint32_t l[8][2]; u32x4 x; };

template <int NT>
__device__ void lora_fwd_partial(const FewArgs& p, int wg, float* red /* [NT / 64][16][64] */) {
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;   // wave index is uniform
  const int i = lane & 15, g = lane >> 4;
  const int k_begin = wg * p.lora_chunk;
  const int k_end = (k_begin + p.lora_chunk < p.h) ? k_begin + p.lora_chunk : p.h;
  const int stride = (NT / 64) * 32, kb0 = k_begin + wave * 32; // the waves interleave 32-row steps
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
    LFwdStep buf[kLoraDepth];
#pragma unroll
    for (int d = 0; d < kLoraDepth; ++d) load_step(buf[d], kb0 + d * stride);
    for (int kb = kb0; kb < k_end; kb += kLoraDepth * stride) {
#pragma unroll
      for (int d = 0; d < kLoraDepth; ++d) {
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
          load_step(buf[d], kb + (d + kLoraDepth) * stride);
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
    for (int idx = threadIdx.x; idx < p.M * 64; idx += NT) {
      const int m = idx >> 6, c = idx & 63;
      if (j0 + c < p.r) {
        float t = 0.0f;
#pragma unroll
        for (int w = 0; w < NT / 64; ++w) t += red[w * 16 * 64 + idx];
        __hip_atomic_store(out + (int64_t)m * p.r + j0 + c, t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
  }
}

// backward: lpart[wg][m][j] = sum over n in [kLoraN * wg, +kLoraN) of dY[m][n] * L2[j][n]
// Both operands are contiguous along n: fragments are plain 16-byte loads.
struct LBwdStep { u32x4 l[4]; u32x4 y; };

template <int NT>
__device__ void lora_bwd_partial(const FewArgs& p, int wg, float* red /* [NT / 64][16][64] */) {
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;   // wave index is uniform
  const int i = lane & 15, g = lane >> 4;
  const int n_begin = wg * p.lora_chunk;
  const int n_end = (n_begin + p.lora_chunk < p.o) ? n_begin + p.lora_chunk : p.o;
  const int stride = (NT / 64) * 32, nb0 = n_begin + wave * 32; // the waves interleave 32-column steps
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
    LBwdStep buf[kLoraDepth];
#pragma unroll
    for (int d = 0; d < kLoraDepth; ++d) load_step(buf[d], nb0 + d * stride);
    for (int nb = nb0; nb < n_end; nb += kLoraDepth * stride) {
#pragma unroll
      for (int d = 0; d < kLoraDepth; ++d) {
        if (nb + d * stride < n_end) {
          const bf16x8 ya = __builtin_bit_cast(bf16x8, buf[d].y);
#pragma unroll
          for (int e = 0; e < 4; ++e)
            acc[e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ya, __builtin_bit_cast(bf16x8, buf[d].l[e]), acc[e], 0, 0, 0);
          load_step(buf[d], nb + (d + kLoraDepth) * stride);
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
    for (int idx = threadIdx.x; idx < p.M * 64; idx += NT) {
      const int m = idx >> 6, c = idx & 63;
      if (j0 + c < p.r) {
        float t = 0.0f;
#pragma unroll
        for (int w = 0; w < NT / 64; ++w) t += red[w * 16 * 64 + idx];
        __hip_atomic_store(out + (int64_t)m * p.r + j0 + c, t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
  }
}

}  // namespace few
}  // namespace qlora
