// Skinny bf16 MFMA GEMMs of the LoRA branch (arXiv 2305.14314, Eq. 3 / Eq. 5 and the adapter
// gradients): T = X L1, U = dY L2^T, dL1 = s X^T U, dL2 = s T^T dY.  One dimension is the adapter
// rank (<= 256), so these are bound by streaming X or dY from HBM, not by MFMA.
//
//   part[split][I x J] (fp32) = sum over this split's K range of A(i,k) * B(k,j)
//   finalize: out = bf16(scale * sum over splits) and/or the sum as a [hi | lo] pair of bf16 matrices
//
// Such a pair carries 16 significant bits of an intermediate (T or U) into the adapter gradients.  Where it is
// an operand (HL = 1: A, HL = 2: B) the kernel loads both halves' tiles and issues two MFMAs per fragment of
// the other operand into the same accumulators, so X (resp. dY) is streamed once.
//
// MASK: LoRA dropout on the adapter's input (hyperparameter appendix): operand A is X, and an element of X enters as
// zero where its bit in the caller's keep-mask (bit e % 8 of byte e / 8 for the flat element index e = token * h + k)
// is clear; the 1/(1-p) of the kept elements is folded into the scale of the finalize step.
//
// Operand layouts are template flags: TA = false means A is stored [i][k] (K-contiguous),
// TA = true means A is stored [k][i] (the contraction index is the row index, as for X^T);
// likewise TB for B ([j][k] or [k][j]).  K-contiguous tiles are kept in LDS XOR-swizzled in 16-byte
// chunks and read with ds_read_b128; row-index-contracted tiles are kept as loaded ([k][64 rows], pitch 72)
// and their MFMA fragments come from the transposing LDS read of gfx950 (ds_read_b64_tr_b16): within a group
// of 16 lanes, lane c supplies the address of an 8-byte chunk and lane i receives element i % 4 of the chunks
// i / 4, i / 4 + 4, i / 4 + 8, i / 4 + 12 -- so with lane c pointing at (k0 + c / 4, rows R0 + 4 (c % 4) .. +3),
// lane i ends up with row R0 + i at k0 .. k0 + 3, which is half an MFMA fragment (8 gathers of 16 bits before).
#include "common.hpp"
#include "launch.hpp"

namespace qlora {

constexpr int ST = 64;                       // tile edge in I, J and K
constexpr int kSmallThreads = 256;
constexpr int kTPitch = 72;                  // elements per k-row of a row-index-contracted tile: 4 consecutive k-rows hit distinct banks
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;

struct SmallArgs {
  const uint16_t* A; int64_t lda;
  const uint16_t* B; int64_t ldb;
  int64_t hl_off;            // HL != 0: element offset of the pair's lo half from its hi half (same row)
  const uint8_t* amask;      // MASK: keep-bits of A's elements in storage order, one bit each
  float* part;
  int I, J, K, k_per_split;
};

typedef __attribute__((address_space(3))) char lds_char;

// fetch one 16-byte chunk of an operand tile (zero outside the matrix)
template <bool T>
__device__ __forceinline__ u32x4 fetch_chunk(const uint16_t* __restrict__ src, int64_t ld, int r0, int R, int k0,
                                             int k_end, int c) {
  const u32x4 z = {0u, 0u, 0u, 0u};
  if constexpr (!T) {                         // src[row][k]: chunk = (row, 8 consecutive k)
    const int row = r0 + (c >> 3), k = k0 + (c & 7) * 8;
    if (row < R && k < k_end) return *(const u32x4*)(src + (int64_t)row * ld + k);
    return z;
  } else {                                    // src[k][row]: chunk = (k, 8 consecutive rows)
    const int k = k0 + (c >> 3), row = r0 + (c & 7) * 8;
    if (k < k_end && row < R) return *(const u32x4*)(src + (int64_t)k * ld + row);
    return z;
  }
}

// the same for operand A under a keep-mask: a chunk is 8 consecutive elements of storage, i.e. one mask byte
template <bool T>
__device__ __forceinline__ u32x4 fetch_chunk_masked(const uint16_t* __restrict__ src, const uint8_t* __restrict__ mask,
                                                    int64_t ld, int r0, int R, int k0, int k_end, int c) {
  u32x4 v = {0u, 0u, 0u, 0u};
  int64_t off;
  bool ok;
  if constexpr (!T) {
    const int row = r0 + (c >> 3), k = k0 + (c & 7) * 8;
    ok = row < R && k < k_end;
    off = (int64_t)row * ld + k;
  } else {
    const int k = k0 + (c >> 3), row = r0 + (c & 7) * 8;
    ok = k < k_end && row < R;
    off = (int64_t)k * ld + row;
  }
  if (ok) {
    v = *(const u32x4*)(src + off);
    const uint32_t b = mask[off >> 3];                       // ld and the chunk start are multiples of 8
#pragma unroll
    for (int d = 0; d < 4; ++d)
      v[d] &= (((b >> (2 * d)) & 1u) ? 0x0000ffffu : 0u) | (((b >> (2 * d + 1)) & 1u) ? 0xffff0000u : 0u);
  }
  return v;
}

template <bool T>
__device__ __forceinline__ void stash_chunk(lds_char* tile, int c, u32x4 v) {
  if constexpr (!T) {
    const int row = c >> 3, kc = c & 7;
    *(u32x4 __attribute__((address_space(3)))*)(tile + row * 128 + ((kc ^ (row & 7)) * 16)) = v;
  } else {
    *(u32x4 __attribute__((address_space(3)))*)(tile + (c >> 3) * (kTPitch * 2) + (c & 7) * 16) = v;   // [k][64 rows], as loaded
  }
}

// MFMA 32x32x16 fragment: lane holds row (lane % 32) of the 32-row sub-tile, 8 consecutive k
template <bool T>
__device__ __forceinline__ bf16x8 small_frag(const lds_char* tile, int row, int kk, int half) {
  if constexpr (!T) {
    const int chunk = (2 * kk + half) ^ (row & 7);
    return *(const bf16x8 __attribute__((address_space(3)))*)(tile + row * 128 + chunk * 16);
  } else {
    // lane l = 32 half + row32: 16-lane group g = l / 16 covers rows R0 = 16 (g % 2) .. +15 of the sub-tile
    const int lane = threadIdx.x & 63, c = lane & 15;
    const int r0 = (row & ~31) + (lane & 16);               // first row of this group's 16 rows
    const int k0 = kk * 16 + half * 8;
    const lds_char* src = tile + ((k0 + (c >> 2)) * kTPitch + r0 + 4 * (c & 3)) * 2;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)src);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (s16x4 __attribute__((address_space(3)))*)(src + 4 * kTPitch * 2));
    typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8;
    const s16x8 f = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, f);
  }
}

template <bool TA, bool TB, int HL, bool MASK>
__global__ __launch_bounds__(kSmallThreads) void small_gemm_kernel(const SmallArgs p) {
  static_assert(HL == 0 || (HL == 1 && TA) || (HL == 2 && TB), "a [hi | lo] operand is stored token-major");
  static_assert(!MASK || HL != 1, "the masked operand is X itself");
  __shared__ __attribute__((aligned(16))) char sA_[ST * kTPitch * 2];
  __shared__ __attribute__((aligned(16))) char sB_[ST * kTPitch * 2];
  __shared__ __attribute__((aligned(16))) char sC_[HL ? ST * kTPitch * 2 : 16];
  lds_char* sA = (lds_char*)sA_;
  lds_char* sB = (lds_char*)sB_;
  lds_char* sC = (lds_char*)sC_;

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int i0 = blockIdx.x * ST, j0 = blockIdx.y * ST;
  const int k_begin = blockIdx.z * p.k_per_split;
  const int k_end = (k_begin + p.k_per_split < p.K) ? k_begin + p.k_per_split : p.K;
  const int wi = wave >> 1, wj = wave & 1;
  const int a_row = wi * 32 + (lane & 31), b_row = wj * 32 + (lane & 31), half = lane >> 5;
  const uint16_t* lo_src = (HL == 1) ? p.A + p.hl_off : p.B + p.hl_off;
  const int64_t lo_ld = (HL == 1) ? p.lda : p.ldb;
  const int lo_r0 = (HL == 1) ? i0 : j0, lo_R = (HL == 1) ? p.I : p.J;

  f32x16 acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.0f;

  // Two steps of operand tiles are kept in flight in registers (sets 0 and 1 alternate): with two or three
  // workgroups per CU one step ahead is too little to cover the HBM latency.
  struct Regs { u32x4 a[2], b[2], c[2]; };
  auto fetch = [&](Regs& R, int k0) {                       // k0 >= k_end loads nothing and yields zeros
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      if constexpr (MASK) R.a[u] = fetch_chunk_masked<TA>(p.A, p.amask, p.lda, i0, p.I, k0, k_end, tid + 256 * u);
      else R.a[u] = fetch_chunk<TA>(p.A, p.lda, i0, p.I, k0, k_end, tid + 256 * u);
      R.b[u] = fetch_chunk<TB>(p.B, p.ldb, j0, p.J, k0, k_end, tid + 256 * u);
      if constexpr (HL != 0) R.c[u] = fetch_chunk<true>(lo_src, lo_ld, lo_r0, lo_R, k0, k_end, tid + 256 * u);
    }
  };
  auto step = [&](Regs& R, int k_next) {
    __syncthreads();                                        // previous step's fragment reads are done
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      stash_chunk<TA>(sA, tid + 256 * u, R.a[u]);
      stash_chunk<TB>(sB, tid + 256 * u, R.b[u]);
      if constexpr (HL != 0) stash_chunk<true>(sC, tid + 256 * u, R.c[u]);
    }
    __syncthreads();
    fetch(R, k_next);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const bf16x8 a = small_frag<TA>(sA, a_row, kk, half);
      const bf16x8 b = small_frag<TB>(sB, b_row, kk, half);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
      if constexpr (HL == 1) {
        const bf16x8 a2 = small_frag<true>(sC, a_row, kk, half);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a2, b, acc, 0, 0, 0);
      }
      if constexpr (HL == 2) {
        const bf16x8 b2 = small_frag<true>(sC, b_row, kk, half);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b2, acc, 0, 0, 0);
      }
    }
  };
  Regs R0, R1;
  fetch(R0, k_begin);
  fetch(R1, k_begin + ST);
  for (int k0 = k_begin; k0 < k_end; k0 += 2 * ST) {
    step(R0, k0 + 2 * ST);
    if (k0 + ST < k_end) step(R1, k0 + 3 * ST);
  }

  float* out = p.part + (int64_t)blockIdx.z * p.I * p.J;
  const int j = j0 + wj * 32 + (lane & 31);
  if (j < p.J) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int i = i0 + wi * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
      if (i < p.I) out[(int64_t)i * p.J + j] = acc[v];
    }
  }
}

// Reduces the split partials in a fixed order (deterministic) and writes up to two bf16 outputs.
//   sum(i, j)  = sum over splits of part[s][i][j]
//   out0[i][j] = bf16(scale0 * sum) for j < J, zero for J <= j < w0                    (row stride ld0)
//   hl[i][j]   = bf16(sum),  hl[i][J + j] = bf16(sum - hl[i][j])                       (row stride 2 J)
//   acc[i][j] += scale0 * sum                                      (fp32, row stride J: gradient accumulation)
__global__ void small_finalize_kernel(const float* __restrict__ part, int splits, int I, int J,
                                      uint16_t* __restrict__ out0, int64_t ld0, int w0, float scale0,
                                      uint16_t* __restrict__ hl, float* __restrict__ acc) {
  const int wmax = (out0 && w0 > J) ? w0 : J;
  const int64_t total = (int64_t)I * wmax;
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
    const int i = (int)(e / wmax), j = (int)(e % wmax);
    float s = 0.0f;
    if (j < J) {
#pragma unroll 8
      for (int sp = 0; sp < splits; ++sp) s += part[(int64_t)sp * I * J + (int64_t)i * J + j];
    }
    if (out0 && j < w0) out0[(int64_t)i * ld0 + j] = bf16_bits(s * scale0);
    if (acc && j < J) acc[(int64_t)i * J + j] += s * scale0;
    if (hl && j < J) {
      const uint16_t hi = bf16_bits(s);
      hl[(int64_t)i * 2 * J + j] = hi;
      hl[(int64_t)i * 2 * J + J + j] = bf16_bits(s - bf16_lo_to_f32(hi));
    }
  }
}

// dst[row][0..Cp) = src[row][0..C) followed by zeros
__global__ void copy_pad_kernel(const uint16_t* __restrict__ src, int R, int C, uint16_t* __restrict__ dst, int Cp,
                                int64_t ld_dst) {
  const int64_t total = (int64_t)R * Cp;
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
    const int row = (int)(e / Cp), c = (int)(e % Cp);
    dst[(int64_t)row * ld_dst + c] = (c < C) ? src[(int64_t)row * C + c] : (uint16_t)0;
  }
}

int small_gemm_splits(int I, int J, int K) {
  const int tiles = ((I + ST - 1) / ST) * ((J + ST - 1) / ST);
  const int ksteps = (K + ST - 1) / ST;
  // ~2 workgroups per CU: every further split adds an fp32 partial tile to write and read back, and past this
  // point that traffic costs more than the extra loads in flight gain (measured: 256 -> +30 %, 1024 -> +8 % time)
  int splits = (512 + tiles - 1) / tiles;
  if (splits > ksteps) splits = ksteps;
  if (splits > 64) splits = 64;
  if (splits < 1) splits = 1;
  return splits;
}

hipError_t launch_small_gemm(const uint16_t* A, int64_t lda, bool ta, const uint16_t* B, int64_t ldb, bool tb, int hl,
                             int64_t hl_off, int I, int J, int K, float* part, int splits, hipStream_t st,
                             const uint8_t* amask) {
  SmallArgs a;
  a.A = A; a.lda = lda; a.B = B; a.ldb = ldb; a.hl_off = hl_off; a.part = part; a.I = I; a.J = J; a.K = K;
  a.amask = amask;
  if (amask && lda % 8 != 0) return hipErrorInvalidValue;
  const int ksteps = (K + ST - 1) / ST;
  a.k_per_split = ((ksteps + splits - 1) / splits) * ST;
  dim3 grid((unsigned)((I + ST - 1) / ST), (unsigned)((J + ST - 1) / ST), (unsigned)splits);
  dim3 block(kSmallThreads);
  if (amask) {
    if (!ta && tb && hl == 0) hipLaunchKernelGGL((small_gemm_kernel<false, true, 0, true>), grid, block, 0, st, a);
    else if (ta && tb && hl == 2) hipLaunchKernelGGL((small_gemm_kernel<true, true, 2, true>), grid, block, 0, st, a);
    else return hipErrorInvalidValue;
  }
  else if (!ta && tb && hl == 0) hipLaunchKernelGGL((small_gemm_kernel<false, true, 0, false>), grid, block, 0, st, a);
  else if (!ta && !tb && hl == 0) hipLaunchKernelGGL((small_gemm_kernel<false, false, 0, false>), grid, block, 0, st, a);
  else if (ta && tb && hl == 1) hipLaunchKernelGGL((small_gemm_kernel<true, true, 1, false>), grid, block, 0, st, a);
  else if (ta && tb && hl == 2) hipLaunchKernelGGL((small_gemm_kernel<true, true, 2, false>), grid, block, 0, st, a);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_small_finalize(const float* part, int splits, int I, int J, uint16_t* out0, int64_t ld0, int w0,
                                 float scale0, uint16_t* hl, float* acc, hipStream_t st) {
  const int wmax = (out0 && w0 > J) ? w0 : J;
  int64_t blocks = ((int64_t)I * wmax + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(small_finalize_kernel, dim3((unsigned)blocks), dim3(256), 0, st, part, splits, I, J, out0, ld0, w0,
                     scale0, hl, acc);
  return hipGetLastError();
}

// LoRA dropout, input gradient: the main GEMM has written dX = dY What^T + Us L1^T with Us = bf16(s/(1-p) dY L2^T),
// which is right wherever the adapter saw the input element; a dropped element gets no gradient through the
// adapter, so its adapter term -- recomputed here from the same bf16 operands -- is taken off again (one more
// rounding for those elements).  A workgroup takes 256 mask bytes (2048 consecutive elements), lists the dropped
// ones in LDS (a few per cent) and spreads them over its threads, eight lanes to a dot product of length r: with
// one thread per mask byte nearly every wave would walk all eight bit positions for two or three useful lanes.
__global__ __launch_bounds__(256) void dropout_dx_fix_kernel(uint16_t* __restrict__ dX, int64_t n_bytes, int h,
                                                             const uint8_t* __restrict__ mask,
                                                             const uint16_t* __restrict__ Us, int ld_us,
                                                             const uint16_t* __restrict__ L1, int r) {
  __shared__ uint16_t list[2048];
  __shared__ int wave_cnt[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t q = (int64_t)blockIdx.x * 256 + tid;
  const uint32_t drop = q < n_bytes ? (~(uint32_t)mask[q]) & 0xffu : 0u;
  const int cnt = __builtin_popcount(drop);
  // exclusive prefix sum of cnt over the workgroup: within the wave by shuffles, across the 4 waves through LDS
  int incl = cnt;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int up = __shfl_up(incl, d, 64);
    if (lane >= d) incl += up;
  }
  if (lane == 63) wave_cnt[wave] = incl;
  __syncthreads();
  int base = 0, total = 0;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const int c = wave_cnt[w];
    if (w < wave) base += c;
    total += c;
  }
  int pos = base + incl - cnt;
  for (uint32_t d = drop; d != 0; d &= d - 1) list[pos++] = (uint16_t)(tid * 8 + (__builtin_ctz(d)));
  __syncthreads();
  // eight lanes per dropped element, 16 bytes of both rows per lane and step, summed by shuffles; two elements per
  // lane group and iteration, so that the loads of the second are in flight while the first is summed
  const int64_t e_base = (int64_t)blockIdx.x * 2048;
  const int sub = tid & 7;
  for (int idx0 = 0; idx0 < total; idx0 += 64) {             // uniform trip count: the shuffles below need every lane
    int64_t e[2];
    bool live[2];
    float dot[2], old[2];
    u32x4 a[2], w[2];
    const uint16_t* us[2];
    const uint16_t* l1[2];
#pragma unroll
    for (int z = 0; z < 2; ++z) {
      const int idx = idx0 + 32 * z + (tid >> 3);
      live[z] = idx < total;
      e[z] = e_base + list[live[z] ? idx : 0];               // flat element index token * h + k
      const int m = (int)(e[z] / h), k = (int)(e[z] - (int64_t)m * h);
      us[z] = Us + (int64_t)m * ld_us;
      l1[z] = L1 + (int64_t)k * r;
      const bool in = 8 * sub < r;                           // r % 16 == 0: a lane's chunk is inside the row or not at all
      a[z] = *(const u32x4*)(us[z] + (in ? 8 * sub : 0));
      w[z] = *(const u32x4*)(l1[z] + (in ? 8 * sub : 0));
      old[z] = bf16_lo_to_f32(dX[e[z]]);
      dot[z] = 0.0f;
      if (!in) { a[z] = u32x4{0u, 0u, 0u, 0u}; }
    }
#pragma unroll
    for (int z = 0; z < 2; ++z) {
      for (int t = 8 * sub;;) {
#pragma unroll
        for (int d = 0; d < 4; ++d) {
          dot[z] = __builtin_fmaf(bf16_lo_to_f32(a[z][d]), bf16_lo_to_f32(w[z][d]), dot[z]);
          dot[z] = __builtin_fmaf(bf16_lo_to_f32(a[z][d] >> 16), bf16_lo_to_f32(w[z][d] >> 16), dot[z]);
        }
        t += 64;
        if (t >= r) break;
        a[z] = *(const u32x4*)(us[z] + t);
        w[z] = *(const u32x4*)(l1[z] + t);
      }
      dot[z] += __shfl_xor(dot[z], 1, 64);
      dot[z] += __shfl_xor(dot[z], 2, 64);
      dot[z] += __shfl_xor(dot[z], 4, 64);
      if (live[z] && sub == 0) dX[e[z]] = bf16_bits(old[z] - dot[z]);
    }
  }
}

hipError_t launch_dropout_dx_fix(uint16_t* dX, int M, int h, const uint8_t* mask, const uint16_t* Us, int ld_us,
                                 const uint16_t* L1, int r, hipStream_t st) {
  const int64_t n = (int64_t)M * h / 8;
  hipLaunchKernelGGL(dropout_dx_fix_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, dX, n, h, mask, Us,
                     ld_us, L1, r);
  return hipGetLastError();
}

hipError_t launch_copy_pad(const uint16_t* src, int R, int C, uint16_t* dst, int Cp, hipStream_t st, int64_t ld_dst) {
  if (ld_dst == 0) ld_dst = Cp;
  if (ld_dst < Cp) return hipErrorInvalidValue;
  int64_t blocks = ((int64_t)R * Cp + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(copy_pad_kernel, dim3((unsigned)blocks), dim3(256), 0, st, src, R, C, dst, Cp, ld_dst);
  return hipGetLastError();
}

}  // namespace qlora
