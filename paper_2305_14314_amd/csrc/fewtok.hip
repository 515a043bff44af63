// Few-token (M <= 16) forward and input-gradient of the QLoRA linear layer (arXiv 2305.14314,
// Eq. 5 / Eq. 6 at generation-time batch sizes): bandwidth-bound streaming kernels that read the
// packed NF4 weight and its double-quantised constants exactly once (0.516 B per weight),
// dequantise in registers to the same bf16 values as the standalone doubleDequant, and feed
// MFMA 16x16x32 with the tokens as the 16-wide dimension.  One launch per call:
//
//   main workgroups    : part[split][m][n] = partial sums of X * What (forward) or dY * What^T (backward)
//                        over the split's share of the contraction, for a slab of 256 outputs
//   adapter workgroups : lpart[p][m][j] = partial sums of the adapter's inner product T = X L1 or U = dY L2^T
//   last arriver       : every workgroup counts itself in at its slab's arrival counter (device-scope atomic
//                        after a fence); the workgroup that brings in a slab's last split then meets the adapter
//                        workgroups, each of which counts itself in at every slab's handshake word.  Whoever
//                        completes that count computes
//                        out = bf16( sum of splits + s * (sum of lpart) * L2 )  resp.  ... * L1^T  -- one rounding.
//                        The only wait is a bounded poll of the last split for the adapter, so every wave exits
//                        whatever the scheduling; the sums are taken in a fixed order, so results do not depend
//                        on who arrives last.
// The counters live in the zeroed header of the caller's workspace and are reset by the last arriver.  A kernel
// boundary costs ~3 us of idle GPU plus ~4 us of fixed launch cost here, which a separate reduction kernel
// would pay on top of a 20-40 us stream.
//
// A step of a wave costs address-unit, LDS-lookup, VALU and MFMA time one after the other (a wave issues
// in order), so workgroups are 16 waves (4 per SIMD, 128 VGPRs each) and every wave keeps 2-3 steps of
// global loads in flight.
// NF4 decode uses a byte -> (value[lo nibble], value[hi nibble]) table in LDS, one 64-bit LDS read per
// two weights.  The table is replicated 32 times with the copies interleaved at 8-byte granularity
// (entry e of copy c at byte 256 e + 8 c), so lane l always reads the two banks of copy l % 32 whatever
// the entry: data-dependent lookups are bank-conflict free (a single shared copy measured ~3.5-way
// conflicts and bounded the kernels at 1.4 TB/s).
#include "fewtok_common.hpp"

namespace qlora {

namespace {

using namespace few;


// Counter map of the workspace header (4096 words): [slab] counts the splits of a slab; [kCtrShake + slab] is the
// handshake of the slab's last split with the adapter workgroups.
constexpr int kCtrShake = 2048;
constexpr int kSpinLimit = 64;               // bounded wait (polls) of a slab's last split for the adapter


// Counts this workgroup in at *c; true for the workgroup that completes `total` arrivals.  Everything the
// workgroup stored before the call is visible to the last arriver.  Only thread 0 pays for the device-scope
// fences (a release is an L2 write-back, an acquire an L2 invalidate on this multi-die part): the barriers
// order the other threads' stores before its release and their later loads after its acquire.  The partials
// themselves are stored write-through (relaxed device-scope atomic stores), which leaves the write-back
// nothing to do: plain stores followed by full fences in every wave measured 8x slower kernels.
__device__ __forceinline__ bool arrive_last(unsigned* c, unsigned total, volatile int* flag) {
  __syncthreads();
  if (threadIdx.x == 0) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    const unsigned old = atomicAdd(c, 1u);
    const int last = old + 1 == total;
    if (last) {
      atomicExch(c, 0u);                                     // nobody else touches this counter any more
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    }
    *flag = last;
  }
  __syncthreads();
  return *flag != 0;
}

// The workgroup that brought in a slab's last split meets the adapter here: the slab's handshake word counts the
// adapter workgroups (each counts itself in at every slab) plus this one.  The adapter's workgroups read a few
// hundred KB and are normally long done; when they are a little late (the smallest layers, cold adapter matrices)
// the split waits for them -- a BOUNDED number of polls, so every wave exits whatever happens -- and only then
// counts itself in.  Whoever completes the count owns the output stage: true = this workgroup.
__device__ __forceinline__ bool meet_adapter(unsigned* shake, unsigned n_adapter, volatile int* flag, unsigned early) {
  __syncthreads();                                           // everybody has read the previous flag
  if (threadIdx.x == 0) {
    int mine = early == n_adapter;                           // seen complete already (the count cannot change any more)
    for (int it = 0; !mine && it < kSpinLimit; ++it) {
      if (__hip_atomic_load(shake, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == n_adapter) { mine = 1; break; }
      __builtin_amdgcn_s_sleep(16);
    }
    if (mine) {
      // every adapter workgroup is in, so this arrival is the last: the word only has to go back to zero
      // (nobody reads it any more), and there is no round trip to wait for
      __hip_atomic_store(shake, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");     // the adapter's partials
    } else {
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");     // hands the splits' partials on to the adapter workgroup that will be last
      const unsigned old = atomicAdd(shake, 1u);
      mine = old == n_adapter;                               // it came in after the last poll after all
      if (mine) {
        atomicExch(shake, 0u);
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
      }
    }
    *flag = mine;
  }
  __syncthreads();
  return *flag != 0;
}

// ---- output stage ---------------------------------------------------------------------------------
// out[m][n] = bf16( sum_s part[s][m][n] + scale * sum_j T[m][j] * B(j, n) ),  T = sum_p lpart[p], for the 256
// outputs n of one slab; forward: B(j, n) = L2[j][n]; backward: B(j, n) = L1[n][j].  Run by all NT threads of one
// workgroup: a thread owns one column and four tokens per pass.  Slab 0 also stores T as a [hi | lo] bf16 pair.
template <bool BWD, int NT>
__device__ void finalize_slab(const FewArgs& p, int slab, char* smem, unsigned* shake, volatile int* flag) {
  constexpr int RC = 64;                                     // rank columns staged at a time
  constexpr int kPitch = RC + 8;                             // backward tile row pitch keeps 16-byte alignment
  constexpr int P = 1024 / NT;                               // passes over the tokens (4 per 256 threads and pass)
  constexpr int IT = 2048 / NT;                              // an adapter tile is at most 2048 chunks of 16 bytes
  float* Ts = (float*)smem;                                  // T[j][m], unscaled: 16 KB
  uint16_t* Bs = (uint16_t*)(smem + 16384);                  // forward [RC][256], backward [256][kPitch]
  const int N = BWD ? p.h : p.o;
  const int n0 = slab * 256;
  const int c = threadIdx.x & 255, tq = threadIdx.x >> 8;    // column within the slab, token quad of a pass
  const int n = n0 + c;
  const bool n_ok = n < N;

  // Everything that does not depend on the adapter's partials is loaded first: the split partials of this
  // thread's outputs and the first tile of the adapter's outer matrix.
  u32x4 stage[IT];
  int dst[IT];
  auto stage_load = [&](int j0, int rc) {
    const int cpr = rc >> 3;                                 // backward: 16-byte chunks per row
#pragma unroll
    for (int it = 0; it < IT; ++it) {
      const int e = it * NT + threadIdx.x;
      bool ok, inside;
      int64_t off;
      if (!BWD) {                                            // row j0 + e / 32 of L2, columns n0 + 8 (e % 32) .. +7
        const int j = e >> 5, ch = e & 31;
        inside = j < rc;
        ok = inside && n0 + 8 * ch < N;
        off = (int64_t)(j0 + j) * N + n0 + 8 * ch;
        dst[it] = j * 256 + 8 * ch;
      } else {                                               // row n0 + cc of L1, rank columns j0 + 8 ch .. +7
        const int cc = e / cpr, ch = e - cc * cpr;
        inside = cc < 256;
        ok = inside && n0 + cc < N;
        off = (int64_t)(n0 + cc) * p.r + j0 + 8 * ch;
        dst[it] = cc * kPitch + 8 * ch;
      }
      const u32x4 v = *(const u32x4*)(p.Bmat + (ok ? off : 0));
      stage[it] = ok ? v : u32x4{0u, 0u, 0u, 0u};
      if (!inside) dst[it] = -1;                             // outside the tile: nothing to store
    }
  };
  if (p.r > 0) stage_load(0, p.r < RC ? p.r : RC);           // without an adapter Bmat may be NULL: no load at all
  // a first look at the adapter's count, in flight together with the loads of the split partials below
  unsigned early = 0u;
  if (p.r > 0 && shake && threadIdx.x == 0) early = __hip_atomic_load(shake, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);

  float acc[P][4], lora[P][4];
#pragma unroll
  for (int q = 0; q < P; ++q) {
    const int m0 = 4 * tq + q * (NT / 64);
#pragma unroll
    for (int u = 0; u < 4; ++u) { acc[q][u] = 0.0f; lora[q][u] = 0.0f; }
    if (m0 < p.M) {                                          // uniform per wave
      const int64_t nn = n_ok ? n : 0;
#pragma unroll 4
      for (int sp = 0; sp < p.splits; ++sp) {
        const float* ps = p.part + (int64_t)sp * p.M * N + nn;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int m = m0 + u;
          const float v = ps[(int64_t)(m < p.M ? m : 0) * N];
          acc[q][u] += m < p.M ? v : 0.0f;
        }
      }
    }
  }
  if (p.r > 0) {
    if (shake && !meet_adapter(shake, (unsigned)p.n_lparts, flag, early)) return;         // the adapter came after the bounded wait: the slab is its
    for (int e = threadIdx.x; e < p.M * p.r; e += NT) {
      float t = 0.0f;
      for (int q0 = 0; q0 < p.n_lparts; q0 += 8) {           // 8 loads in flight, then a fixed-order sum
        float v[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          const bool ok = q0 + q < p.n_lparts;
          const float x = p.lpart[(int64_t)(ok ? q0 + q : 0) * p.M * p.r + e];
          v[q] = ok ? x : 0.0f;
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) t += v[q];
      }
      const int m = e / p.r, j = e - m * p.r;
      Ts[j * 16 + m] = t;
      if (p.hl && slab == 0) {
        const uint16_t hi = bf16_bits(t);
        p.hl[(int64_t)m * 2 * p.r + j] = hi;
        p.hl[(int64_t)m * 2 * p.r + p.r + j] = bf16_bits(t - bf16_lo_to_f32(hi));
      }
    }
    for (int j0 = 0; j0 < p.r; j0 += RC) {
      const int rc = (p.r - j0 < RC) ? p.r - j0 : RC;
      if (j0 > 0) {
        __syncthreads();                                     // previous tile consumed
        stage_load(j0, rc);
      }
#pragma unroll
      for (int it = 0; it < IT; ++it)
        if (dst[it] >= 0) *(u32x4*)(Bs + dst[it]) = stage[it];
      __syncthreads();                                       // tile and Ts visible
#pragma unroll
      for (int q = 0; q < P; ++q) {
        const int m0 = 4 * tq + q * (NT / 64);
        if (m0 < p.M) {
#pragma unroll 8
          for (int j = 0; j < rc; ++j) {
            const float b = bf16_lo_to_f32(BWD ? Bs[c * kPitch + j] : Bs[j * 256 + c]);
            const f32x4 t = *(const f32x4*)&Ts[(j0 + j) * 16 + m0];
#pragma unroll
            for (int u = 0; u < 4; ++u) lora[q][u] = __builtin_fmaf(t[u], b, lora[q][u]);
          }
        }
      }
    }
  }
  if (!n_ok) return;
#pragma unroll
  for (int q = 0; q < P; ++q) {
    const int m0 = 4 * tq + q * (NT / 64);
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (m0 + u < p.M) p.out[(int64_t)(m0 + u) * N + n] = bf16_bits(acc[q][u] + p.scale * lora[q][u]);
  }
}

// Called by every adapter workgroup after its partial is stored: it counts itself in at every slab's handshake.
// A slab whose count it completes (the slab's splits gave up waiting: rare) is finished right here.
template <bool BWD, int NT>
__device__ void adapter_arrive(const FewArgs& p, char* smem, volatile int* flag) {
  int* npend = (int*)(smem + 65536);                         // beyond what finalize_slab uses
  int* pend = npend + 1;
  if (threadIdx.x == 0) *npend = 0;
  __syncthreads();                                           // the partial of this workgroup is stored
  for (int t = threadIdx.x; t < p.n_slabs; t += NT) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    const unsigned old = atomicAdd(p.ctr + kCtrShake + t, 1u);
    if (old == (unsigned)p.n_lparts) {                       // every other adapter workgroup and the slab's splits are in
      atomicExch(p.ctr + kCtrShake + t, 0u);
      pend[atomicAdd(npend, 1)] = t;
    }
  }
  __syncthreads();
  const int n = *npend;
  if (n > 0) {
    if (threadIdx.x == 0) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");   // everybody counted before us
    __syncthreads();
  }
  for (int q = 0; q < n; ++q) {
    finalize_slab<BWD, NT>(p, pend[q], smem, nullptr, flag);
    __syncthreads();
  }
}



// ---- forward main ---------------------------------------------------------------------------------
// W is [h][o], o contiguous.  A workgroup owns a slab of 256 output columns (128 packed bytes per row: one
// full L2 line) and a range of k rows; its 16 waves take interleaved 16-row steps and are summed through
// LDS at the end.  Lane (c = lane % 32, rh = lane / 32) loads, for rows kb + 8 rh + j (j = 0..7), packed
// dword c of the slab, so every load instruction reads two whole 128-byte lines (a wave that reads half
// lines, the other half going to a sibling wave, measured 25% less HBM bandwidth, and reading the constants
// as one byte per row-major line halved it again: they are stored column-group-major for this reason).
//
// MFMA 16x16x32 wants lane (s = lane % 16, g = lane / 16) to hold 8 k-values of B column slot s.  Here
// g = 2 rh + c / 16: the groups g in {0, 2} hold columns 8 (c % 16) + e of the first 128 columns (rows
// kb .. +7 and kb + 8 .. +15), the groups {1, 3} the same rows of the second 128 columns.  The token operand
// selects: its k-slots of the groups that do not belong are zero.
//   MT = 8  (M <= 8): A rows 0-7 = tokens with the first-half groups, rows 8-15 = the same tokens with the
//           second-half groups; one MFMA per column phase e, D rows 0-7 / 8-15 = first / second 128 columns.
//   MT = 16 (M <= 16): two MFMAs per phase, A1 (groups 0, 2) and A2 (groups 1, 3), two accumulator sets.
// Each MFMA thus contracts 16 rows; the matrix pipe has the room (it is ~15% busy).
// The 64 constants of a step (16 rows x 4 blocks, 64 contiguous bytes) are decoded one per lane and exchanged
// through a wave-private LDS strip.
struct FwdStep { uint32_t pk[8]; u32x4 x; uint32_t code; float c1; };   // raw loads only: nothing here is consumed before compute()

// `work` is this workgroup's position in the call's work list: the adapter partials first, then (split, slab) pairs.
template <int MT, int NT>
__device__ __forceinline__ void fewtok_fwd_body(const FewArgs& p, const int work) {
  constexpr int NA = MT / 8;                                 // accumulator sets (and MFMAs per column phase)
  constexpr int kDepth = 3;
  constexpr int NW = NT / 64;                                // waves: 16 with 128 VGPRs each, or 8 with 256 (MT = 16)
  static_assert(NW * MT * 1024 <= kRedBytes, "one [MT][256] fp32 tile per wave");
  __shared__ __attribute__((aligned(256))) char smem[kSmemBytes];
  f32x2* lut2 = (f32x2*)smem;
  float* red = (float*)smem;
  float* unit = (float*)(smem + kUnitOff);
  __shared__ int flag;
  if (work < p.n_lparts) {
    lora_fwd_partial<NT>(p, work, red);
    adapter_arrive<false, NT>(p, smem, &flag);
    return;
  }

  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;   // uniform
  const int c = lane & 31, rh = lane >> 5;
  const int sl = lane & 15, g = lane >> 4;                   // MFMA slot and k group
  const uint32_t lane_off = 8u * (uint32_t)(lane & (kLutCopies - 1));
  float* strip = (float*)(smem + kStripOff) + wave * 64;     // [block 4][row 16]
  const int slab = (work - p.n_lparts) % p.n_slabs, split = (work - p.n_lparts) / p.n_slabs;
  const int k_begin = split * p.per_split;
  const int k_end = (k_begin + p.per_split < p.h) ? k_begin + p.per_split : p.h;
  const float mean = *p.mean;
  const int bpr = p.o >> 6, o_dw = p.o >> 3;
  const bool col_ok = slab * 256 + 8 * c < p.o;              // o % 64 == 0: a dword is in or out as a whole
  const uint32_t* packed = (const uint32_t*)p.packed;

  // Per-lane offsets are fixed for the whole kernel; a step only moves a wave-uniform base.  k ranges are
  // multiples of 16 rows, so every row of a step inside the range is valid; steps past the range (prefetch
  // overrun, empty splits) are redirected to the last valid step and never consumed.  Lanes outside the
  // tensor (columns >= o, tokens >= M) read a valid dummy address and are masked at compute time, or
  // produce output columns that are never stored.
  const int k_last = k_end - 16;
  uint32_t w_off[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) w_off[j] = (uint32_t)((8 * rh + j) * o_dw + (col_ok ? slab * 32 + c : 0));
  // token operand: lane (sl, g) feeds k-slots of rows kb + 8 (g / 2) .. +7
  const int tok = MT == 8 ? (sl & 7) : sl;
  const bool x_ok = tok < p.M && (MT == 16 || (g & 1) == (sl >> 3));
  const uint32_t x_off = (uint32_t)((tok < p.M ? tok : 0) * p.h + 8 * (g >> 1));
  // the constant this lane decodes for a step: row kb + lane / 4, block 4 slab + lane % 4 (64 contiguous bytes)
  const int c_blk = 4 * slab + (lane & 3);
  const int cw = (4 * slab + 4 <= bpr) ? 4 : bpr - 4 * slab; // blocks in this column group
  const bool c_ok = (lane & 3) < cw;
  const uint8_t* code_g = p.code + (int64_t)4 * p.h * slab + (c_ok ? (lane & 3) : 0);
  const uint32_t c_row = (uint32_t)(lane >> 2);
  auto load_step = [&](FwdStep& s, int kb) {
    const int kc = kb < k_end ? kb : k_last;                 // uniform
    const uint32_t* wbase = packed + (int64_t)kc * o_dw;
#pragma unroll
    for (int j = 0; j < 8; ++j) s.pk[j] = wbase[w_off[j]];
    s.x = *(const u32x4*)(p.X + kc + x_off);
    const uint32_t crow = (uint32_t)kc + c_row;
    s.code = code_g[(int64_t)crow * cw];
    s.c1 = p.c1[(crow * (uint32_t)bpr + (uint32_t)(c_ok ? c_blk : 4 * slab)) >> 8];
  };

  // the first loads are in flight while the decode table is built
  const int stride = NW * 16;
  const int kb0 = k_begin + wave * 16;
  FwdStep buf[kDepth];
#pragma unroll
  for (int d = 0; d < kDepth; ++d) load_step(buf[d], kb0 + d * stride);
  init_pair_lut<NT>(lut2, unit, p.dtype, p.tab, (float*)(smem + kStripOff));
  __syncthreads();

  f32x4 acc[NA][8];
#pragma unroll
  for (int a = 0; a < NA; ++a)
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[a][e] = f32x4{0.f, 0.f, 0.f, 0.f};

  auto compute = [&](const FwdStep& s) {
    // dequant(c1, c2): two separately rounded fp32 steps; wave-private strip: no barrier needed
    strip[(lane & 3) * 16 + (lane >> 2)] = __fadd_rn(__fmul_rn(unit[s.code], s.c1), mean);
    const f32x4* sp = (const f32x4*)&strip[(c >> 3) * 16 + 8 * rh];
    const f32x4 ca = sp[0], cb = sp[1];
    const float c2[8] = {ca[0], ca[1], ca[2], ca[3], cb[0], cb[1], cb[2], cb[3]};
    const u32x4 zero = u32x4{0u, 0u, 0u, 0u};
    bf16x8 xa[NA];
    if (MT == 8) {
      xa[0] = __builtin_bit_cast(bf16x8, x_ok ? s.x : zero);
    } else {
      xa[0] = __builtin_bit_cast(bf16x8, (x_ok && !(g & 1)) ? s.x : zero);
      xa[NA - 1] = __builtin_bit_cast(bf16x8, (x_ok && (g & 1)) ? s.x : zero);
    }
    // The table lookups of byte b + 1 are issued before the arithmetic of byte b and the scheduler is told not to move
    // anything across that point: left alone it puts every lookup right in front of its first use, and each then costs
    // the wave a full LDS round trip (32 of them per step).
    // (With 1024 threads there are no registers for the batch ahead: the 8 lookups of a byte are issued together and
    // waited for, 4 round trips per step.)
    constexpr bool kAhead = NT <= 512;
    f32x2 qn[8];
    if (kAhead) {
#pragma unroll
      for (int j = 0; j < 8; ++j) qn[j] = pair_lookup_b(lut2, s.pk[j], lane_off, 0);
    }
#pragma unroll
    for (int b = 0; b < 4; ++b) {                            // byte b of every row: columns 2b, 2b + 1 of the dword
      f32x2 q[8];
      if (kAhead) {
#pragma unroll
        for (int j = 0; j < 8; ++j) q[j] = qn[j];
        if (b < 3) {
#pragma unroll
          for (int j = 0; j < 8; ++j) qn[j] = pair_lookup_b(lut2, s.pk[j], lane_off, b + 1);
        }
      } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) q[j] = pair_lookup_b(lut2, s.pk[j], lane_off, b);
      }
      __builtin_amdgcn_sched_barrier(0);
      float lo[8], hi[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        lo[j] = __fmul_rn(q[j][0], c2[j]);
        hi[j] = __fmul_rn(q[j][1], c2[j]);
      }
      u32x4 w;
#pragma unroll
      for (int jp = 0; jp < 4; ++jp) w[jp] = pack_bf16x2(lo[2 * jp], lo[2 * jp + 1]);
#pragma unroll
      for (int a = 0; a < NA; ++a)
        acc[a][2 * b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa[a], __builtin_bit_cast(bf16x8, w), acc[a][2 * b], 0, 0, 0);
#pragma unroll
      for (int jp = 0; jp < 4; ++jp) w[jp] = pack_bf16x2(hi[2 * jp], hi[2 * jp + 1]);
#pragma unroll
      for (int a = 0; a < NA; ++a)
        acc[a][2 * b + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa[a], __builtin_bit_cast(bf16x8, w), acc[a][2 * b + 1], 0, 0, 0);
    }
  };

  // software pipeline over this wave's steps kb = k_begin + 16 * (wave + 16 t)
  for (int kb = kb0; kb < k_end; kb += kDepth * stride) {
#pragma unroll
    for (int d = 0; d < kDepth; ++d) {
      if (kb + d * stride < k_end) {
        compute(buf[d]);
        load_step(buf[d], kb + (d + kDepth) * stride);
      }
    }
  }

  // D layout: column slot = lane % 16, rows 4 * (lane / 16) + v.  Row R of accumulator set a is token R % MT of
  // column half (MT == 8 ? R / 8 : a); column within the half = 8 slot + e.  The waves store [MT][256] tiles over
  // the decode table (dead now) and the tiles are summed.
  float* out = p.part + (int64_t)split * p.M * p.o;
  auto store_tile = [&](float* my) {
#pragma unroll
    for (int a = 0; a < NA; ++a)
#pragma unroll
      for (int e = 0; e < 8; ++e)
#pragma unroll
        for (int vv = 0; vv < 4; ++vv) {
          const int R = 4 * g + vv;
          const int m = MT == 8 ? (R & 7) : R, half = MT == 8 ? (R >> 3) : a;
          my[m * 256 + half * 128 + 8 * sl + e] = acc[a][e][vv];
        }
  };
  constexpr int kTile = MT * 256;
  __syncthreads();                                           // every wave is done with the decode table
  store_tile(red + wave * kTile);
  __syncthreads();
  for (int idx = threadIdx.x; idx < p.M * 256; idx += NT) {
    const int n = slab * 256 + (idx & 255);
    float t = 0.0f;
#pragma unroll
    for (int w = 0; w < NW; ++w) t += red[w * kTile + idx];
    if (n < p.o) __hip_atomic_store(out + (int64_t)(idx >> 8) * p.o + n, t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  if (!arrive_last(p.ctr + slab, (unsigned)p.splits, &flag)) return;
  finalize_slab<false, NT>(p, slab, smem, p.ctr + kCtrShake + slab, &flag);
}

template <int MT, int NT>
__global__ __launch_bounds__(NT) void fewtok_fwd_kernel(const FewArgs p) {
  fewtok_fwd_body<MT, NT>(p, work_index());
}

// Several layers that read the same token rows (the q / k / v or the gate / up projections of a decoder block) in
// one launch: the fixed cost of a call -- launch, arrival chain, output stage -- is paid once for all of them.
// The work list holds every layer's adapter partials first, then every layer's (split, slab) pairs.
struct FewMulti {
  int n;
  int a_first[kFewMaxLayers + 1];            // first adapter workgroup of layer l; [n] = their total
  int w_first[kFewMaxLayers + 1];            // first (split, slab) workgroup of layer l; [n] = the grid size
  FewArgs a[kFewMaxLayers];
};

template <int MT, int NT>
__global__ __launch_bounds__(NT) void fewtok_fwd_multi_kernel(const FewMulti m) {
  const int work = work_index();
  const bool adapter = work < m.a_first[m.n];
  const int* first = adapter ? m.a_first : m.w_first;
  int l = 0;
  while (l + 1 < m.n && work >= first[l + 1]) ++l;
  const FewArgs p = m.a[l];
  fewtok_fwd_body<MT, NT>(p, (adapter ? 0 : p.n_lparts) + work - first[l]);
}

// ---- backward main --------------------------------------------------------------------------------
// Contraction runs along o, the contiguous dimension of W, so a lane's 16-byte load is 32 consecutive
// weights of one row and one quantisation constant.  A workgroup owns 256 weight rows and a range of
// columns: wave (rg = wave % 4, cw = wave / 4) owns rows 64 rg .. +63 and takes the 128-column steps
// cw, cw + 4, ...; the 4 waves of a row group are summed through LDS at the end.  Per step a lane
// (i = lane % 16, g = lane / 16) loads rows r0 + 16u + i (u = 0..3) at columns kb + 32g .. +31; MFMA t
// (0..3) uses dword t of each load, so one token fragment serves four weight rows.
struct BwdStep { u32x4 w[4]; u32x4 y[4]; uint32_t code[4]; float c1[4]; };   // raw loads only

__global__ __launch_bounds__(kFewThreads) void fewtok_bwd_kernel(const FewArgs p) {
  constexpr int NT = kFewThreads;
  __shared__ __attribute__((aligned(256))) char smem[kSmemBytes];
  f32x2* lut2 = (f32x2*)smem;
  float* red = (float*)smem;
  float* unit = (float*)(smem + kUnitOff);
  __shared__ int flag;
  const int work = work_index();
  if (work < p.n_lparts) {
    lora_bwd_partial<NT>(p, work, red);
    adapter_arrive<true, NT>(p, smem, &flag);
    return;
  }

  const int wave16 = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;   // uniform
  const int rg = wave16 & 3, cw = wave16 >> 2;
  const int i = lane & 15, g = lane >> 4;
  const uint32_t lane_off = 8u * (uint32_t)(lane & (kLutCopies - 1));
  const int slab = (work - p.n_lparts) % p.n_slabs, split = (work - p.n_lparts) / p.n_slabs;
  const int r0 = slab * 256 + rg * 64;
  const int c_begin = split * p.per_split;
  const int c_end = (c_begin + p.per_split < p.o) ? c_begin + p.per_split : p.o;
  const float mean = *p.mean;
  const int bpr = p.o >> 6, o_q = p.o >> 5;                  // 16-byte groups (32 weights) per row
  const u32x4* packed = (const u32x4*)p.packed;

  // Fixed per-lane offsets, wave-uniform base per step (see the forward kernel).  The column range of a
  // split is a multiple of 64, a step is 128 wide: the last step may be half empty, which is masked on
  // the token operand (zeros) at compute time, with the weight loads redirected to valid addresses.
  const int c_last = c_end - 64;                             // start of the last valid 64-column block
  uint32_t w_off[4], cd_off[4], row_c[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int row = r0 + 16 * u + i;
    const bool row_ok = row < p.h;
    row_c[u] = (uint32_t)(row_ok ? row : 0);
    w_off[u] = row_c[u] * (uint32_t)o_q;
    cd_off[u] = row_c[u] * (uint32_t)bpr;
  }
  const bool y_row_ok = i < p.M;
  const uint32_t y_off = (uint32_t)((y_row_ok ? i : 0) * p.o);
  auto load_step = [&](BwdStep& s, int kb) {
    int col = kb + 32 * g;                                   // per lane
    if (col >= c_end) col = c_last + 32 * (g & 1);           // overrun: any valid column (masked at compute)
    const u32x4* wbase = packed + (col >> 5);
    // constants are stored column-group-major: the 16 rows x 2 blocks of one load sit within 64 bytes
    const int blk = col >> 6, G = blk >> 2;
    const uint32_t cw = (4 * G + 4 <= bpr) ? 4u : (uint32_t)(bpr - 4 * G);
    const uint8_t* cbase = p.code + (int64_t)4 * p.h * G + (blk & 3);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      s.w[u] = wbase[w_off[u]];
      s.code[u] = cbase[row_c[u] * cw];
      s.c1[u] = p.c1[(cd_off[u] + (uint32_t)blk) >> 8];
    }
    const uint16_t* ysrc = p.X + y_off + col;
#pragma unroll
    for (int t = 0; t < 4; ++t) s.y[t] = *(const u32x4*)(ysrc + 8 * t);
  };

  const int stride = 4 * 128;
  const int kb0 = c_begin + cw * 128;
  BwdStep buf[kBwdDepth];
#pragma unroll
  for (int d = 0; d < kBwdDepth; ++d) load_step(buf[d], kb0 + d * stride);   // in flight while the table is built
  init_pair_lut<NT>(lut2, unit, p.dtype, p.tab, (float*)(smem + kStripOff));
  __syncthreads();

  f32x4 acc[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) acc[u] = f32x4{0.f, 0.f, 0.f, 0.f};

  auto compute = [&](const BwdStep& s, int kb) {
    const bool y_ok = y_row_ok && kb + 32 * g < c_end;       // tokens >= M and columns past the split contribute zero
    float c2v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) c2v[u] = __fadd_rn(__fmul_rn(unit[s.code[u]], s.c1[u]), mean);
    // the 4 lookups of a dword are issued together, then waited for (left alone the scheduler puts every lookup right
    // in front of its first use: 64 LDS round trips per step instead of 16; 1024 threads leave no registers for more)
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const bf16x8 ya = __builtin_bit_cast(bf16x8, y_ok ? s.y[t] : u32x4{0u, 0u, 0u, 0u});
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const uint32_t d = s.w[u][t];
        f32x2 q[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) q[b] = pair_lookup_b(lut2, d, lane_off, b);
        __builtin_amdgcn_sched_barrier(0);
        u32x4 w;
#pragma unroll
        for (int b = 0; b < 4; ++b) w[b] = pack_bf16x2(__fmul_rn(q[b][0], c2v[u]), __fmul_rn(q[b][1], c2v[u]));
        acc[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ya, __builtin_bit_cast(bf16x8, w), acc[u], 0, 0, 0);
      }
    }
  };

  for (int kb = kb0; kb < c_end; kb += kBwdDepth * stride) {
#pragma unroll
    for (int d = 0; d < kBwdDepth; ++d) {
      if (kb + d * stride < c_end) {
        compute(buf[d], kb + d * stride);
        load_step(buf[d], kb + (d + kBwdDepth) * stride);
      }
    }
  }

  // D layout: column slot = lane % 16 = weight row within the 16-row group, token rows 4 * (lane / 16) + v.
  // Every wave stores its 16 x 64 tile over the dead decode table; the 4 tiles of a row group are summed.
  __syncthreads();
  float* my = red + wave16 * (16 * 64);
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int vv = 0; vv < 4; ++vv) my[(4 * g + vv) * 64 + 16 * u + i] = acc[u][vv];
  __syncthreads();
  float* out = p.part + (int64_t)split * p.M * p.h;
  for (int idx = threadIdx.x; idx < p.M * 256; idx += kFewThreads) {
    const int m = idx >> 8, rr = idx & 255;
    const int row = slab * 256 + rr;
    const float* src = red + (rr >> 6) * (16 * 64) + m * 64 + (rr & 63);
    float t = 0.0f;
#pragma unroll
    for (int c = 0; c < 4; ++c) t += src[c * 4 * 16 * 64];
    if (row < p.h) __hip_atomic_store(out + (int64_t)m * p.h + row, t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  if (!arrive_last(p.ctr + slab, (unsigned)p.splits, &flag)) return;
  finalize_slab<true, NT>(p, slab, smem, p.ctr + kCtrShake + slab, &flag);
}

// One 16-wave workgroup occupies a CU (its LDS map is 133 KB), so the launch is sized to fit the 256 CUs
// in a single round: slabs * splits + adapter workgroups <= 256 whenever possible.
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
int fewtok_fwd_splits(int h, int o) { return pick_splits((o + 255) / 256, (h + 15) / 16, 32, fewtok_fwd_lparts(h, 16)); }
int fewtok_bwd_splits(int h, int o) { return pick_splits((h + 255) / 256, (o + 127) / 128, 8, fewtok_bwd_lparts(o, 16)); }

int fewtok_fwd_slabs(int o) { return (o + 255) / 256; }
int fewtok_bwd_slabs(int h) { return (h + 255) / 256; }

hipError_t launch_fewtok_fwd(const uint16_t* X, int M, const NF4Dev& w, float* part, int splits, const uint16_t* L1,
                             const uint16_t* L2, int r, float scale, float* lpart, unsigned* ctr, uint16_t* Y,
                             uint16_t* T_hl, hipStream_t st) {
  FewArgs a;
  a.X = X; a.M = M; a.packed = w.packed; a.code = w.code; a.c1 = w.c1; a.mean = w.mean;
  a.dtype = w.dtype; a.tab = table4_host(w.dtype);
  a.h = (int)w.rows; a.o = (int)w.cols; a.part = part;
  const int steps = (a.h + 15) / 16;
  a.per_split = ((steps + splits - 1) / splits) * 16;
  a.n_slabs = fewtok_fwd_slabs(a.o); a.splits = splits;
  a.L = L1; a.r = r; a.lpart = lpart; a.n_lparts = fewtok_fwd_lparts(a.h, r);
  a.ctr = ctr; a.Bmat = L2; a.scale = scale; a.out = Y; a.hl = r > 0 ? T_hl : nullptr;
  a.lora_chunk = kLoraK; a.hdr = ctr; a.nonce = 0u; a.spin_limit = kSpinLimit;
  if (a.n_slabs > kFewMaxSlabs) return hipErrorInvalidValue;
  const dim3 grid((unsigned)(a.n_slabs * splits + a.n_lparts));
  if (M <= 8) hipLaunchKernelGGL((fewtok_fwd_kernel<8, 1024>), grid, dim3(1024), 0, st, a);
  else hipLaunchKernelGGL((fewtok_fwd_kernel<16, 512>), grid, dim3(512), 0, st, a);
  return hipGetLastError();
}

int fewtok_multi_splits(int n, int h, const int* o, int r_max) {
  int slabs = 0, reserved = 0;
  for (int l = 0; l < n; ++l) { slabs += fewtok_fwd_slabs(o[l]); reserved += fewtok_fwd_lparts(h, r_max > 0 ? 16 : 0); }
  return pick_splits(slabs, (h + 15) / 16, 32, reserved);
}

hipError_t launch_fewtok_fwd_multi(const uint16_t* X, int M, int n, const FewLayer* layers, int splits, unsigned* ctr,
                                   hipStream_t st) {
  if (n < 1 || n > kFewMaxLayers) return hipErrorInvalidValue;
  FewMulti m;
  m.n = n;
  int adapters = 0, slab0 = 0;
  for (int l = 0; l < n; ++l) {
    const FewLayer& y = layers[l];
    FewArgs& a = m.a[l];
    a.X = X; a.M = M; a.packed = y.w.packed; a.code = y.w.code; a.c1 = y.w.c1; a.mean = y.w.mean;
    a.dtype = y.w.dtype; a.tab = table4_host(y.w.dtype);
    a.h = (int)y.w.rows; a.o = (int)y.w.cols; a.part = y.part;
    const int steps = (a.h + 15) / 16;
    a.per_split = ((steps + splits - 1) / splits) * 16;
    a.n_slabs = fewtok_fwd_slabs(a.o); a.splits = splits;
    a.L = y.L1; a.r = y.r; a.lpart = y.lpart; a.n_lparts = fewtok_fwd_lparts(a.h, y.r);
    a.ctr = ctr + slab0;                                     // every layer its own range of slab counters
    a.Bmat = y.L2; a.scale = y.scale; a.out = y.Y; a.hl = nullptr;
    a.lora_chunk = kLoraK; a.hdr = ctr; a.nonce = 0u; a.spin_limit = kSpinLimit;
    m.a_first[l] = adapters;
    adapters += a.n_lparts;
    slab0 += a.n_slabs;
  }
  if (slab0 > kFewMaxSlabs) return hipErrorInvalidValue;
  m.a_first[n] = adapters;
  int work = adapters;
  for (int l = 0; l < n; ++l) { m.w_first[l] = work; work += m.a[l].n_slabs * splits; }
  m.w_first[n] = work;
  for (int l = n + 1; l <= kFewMaxLayers; ++l) { m.a_first[l] = adapters; m.w_first[l] = work; }
  for (int l = n; l < kFewMaxLayers; ++l) m.a[l] = m.a[0];
  const dim3 grid((unsigned)work);
  if (M <= 8) hipLaunchKernelGGL((fewtok_fwd_multi_kernel<8, 1024>), grid, dim3(1024), 0, st, m);
  else hipLaunchKernelGGL((fewtok_fwd_multi_kernel<16, 512>), grid, dim3(512), 0, st, m);
  return hipGetLastError();
}

hipError_t launch_fewtok_bwd(const uint16_t* dY, int M, const NF4Dev& w, float* part, int splits, const uint16_t* L1,
                             const uint16_t* L2, int r, float scale, float* lpart, unsigned* ctr, uint16_t* dX,
                             uint16_t* U_hl, hipStream_t st) {
  FewArgs a;
  a.X = dY; a.M = M; a.packed = w.packed; a.code = w.code; a.c1 = w.c1; a.mean = w.mean;
  a.dtype = w.dtype; a.tab = table4_host(w.dtype);
  a.h = (int)w.rows; a.o = (int)w.cols; a.part = part;
  const int steps = (a.o + 127) / 128;
  // a split's column range is a whole number of 128-byte lines (256 columns): a line straddling two splits is
  // fetched by both workgroups, from different XCDs (measured +19 % HBM traffic on the 8192 x 8192 layers)
  a.per_split = ((steps + 2 * splits - 1) / (2 * splits)) * 256;
  a.n_slabs = fewtok_bwd_slabs(a.h); a.splits = splits;
  a.L = L2; a.r = r; a.lpart = lpart; a.n_lparts = fewtok_bwd_lparts(a.o, r);
  a.ctr = ctr; a.Bmat = L1; a.scale = scale; a.out = dX; a.hl = r > 0 ? U_hl : nullptr;
  a.lora_chunk = kLoraN; a.hdr = ctr; a.nonce = 0u; a.spin_limit = kSpinLimit;
  if (a.n_slabs > kFewMaxSlabs) return hipErrorInvalidValue;
  hipLaunchKernelGGL(fewtok_bwd_kernel, dim3((unsigned)(a.n_slabs * splits + a.n_lparts)), dim3(kFewThreads), 0, st, a);
  return hipGetLastError();
}

// Zeroes the counter header of a workspace (a fill kernel, not a memset node, so it can be captured in a graph).
namespace {
__global__ void zero_header_kernel(unsigned* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0u;
}
}  // namespace
hipError_t launch_workspace_init(void* workspace, hipStream_t st) {
  const int n = (int)(kWorkspaceHeaderBytes / sizeof(unsigned));
  hipLaunchKernelGGL(zero_header_kernel, dim3((n + 255) / 256), dim3(256), 0, st, (unsigned*)workspace, n);
  return hipGetLastError();
}

}  // namespace qlora
