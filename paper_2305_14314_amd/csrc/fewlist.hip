// Few-token (M <= 16) forward and input gradient of a LIST of QLoRA linear layers in one persistent launch
// (arXiv 2305.14314, Eq. 5 / Eq. 6 at generation-time batch sizes; adapters on every linear layer of a block,
// Section 5).  Each layer brings its own token rows; the layers do not depend on each other.
//
// Why a list: at a few tokens a layer is 35 - 93 MB of packed weights, i.e. 4 - 12 us of HBM time, while a launch
// of its own costs 16 - 19 us of fixed time on this machine (dispatch, decode table, pipeline fill, the chain
// partial -> fence -> count -> last arriver's loads -> output).  Here that is paid once per list:
//
//   * one workgroup per compute unit, alive for the whole list; the byte -> (value, value) decode table is
//     built once and stays in LDS;
//   * the work of all layers is one line of UNITS (forward: 16 weight rows x 256 columns = 2 KB of nibbles;
//     backward: 256 rows x 128 columns = 16 KB), layer after layer, slab after slab; workgroup rho takes the
//     contiguous range [start(rho), start(rho + 1)) of that line, so every compute unit streams the same
//     number of bytes whatever the shapes (the per-layer launches left 10 - 30 % of the chip idle);
//   * a range crosses slab (and layer) boundaries: the software pipeline of global loads runs on across them
//     -- the next slab's nibbles are in flight while this slab's partial sums are reduced, stored and counted in;
//   * a slab of 256 outputs is covered by 1 - 3 workgroups; each stores its fp32 partial, and the last one to
//     arrive sums them in a fixed order, adds the adapter's term and rounds once (same output stage as the
//     one-layer kernels, so the result does not depend on who arrives last);
//   * the adapter's inner products (T = X L1, U = dY L2^T) are the first items of the first workgroups, which
//     get correspondingly fewer units.
//
// Arrival words (in the caller's counter header) are bit masks tagged with the call's nonce in bits 31:24:
// contributor j sets bit j.  A word that is neither zero nor tagged with this call's nonce, or that already
// holds the arriving bit, was left behind by something else (an abandoned call, an uninitialised header): the
// kernel raises the header's sticky status word, which qlora_workspace_check reports.  Every wait is a bounded
// poll, so all waves exit whatever the header held.
#include <algorithm>
#include <vector>

#include "fewtok_common.hpp"

// Launch shapes (threads per workgroup, ring depth of the load pipeline) of the three kernels.  The load cursor of the
// next segment costs registers: with 1024 threads (128 registers a lane) the forward kernel for up to 8 tokens spilled
// 61 and the backward kernel 103 registers to scratch, which showed as 40 and 97 MiB of HBM writes per launch.  With
// 512 threads nothing spills.  Measured on the seven linears of a 65B-shaped block, 1 / 4 / 16 tokens, microseconds
// per launch: backward 1024 threads, depth 2: 207 / 217 / 245; 512 threads, depth 3: 177 / 182 / 209 (depth 4 spills
// again).  Forward, up to 8 tokens: 1024 threads, depth 3: 174 / 177; 512 threads, depth 4: 175 / 178, depth 6:
// 179 / 183.  Forward, 16 tokens (512 threads): depth 3, 4, 5: 204, 203, 205.
#ifndef QL_LIST_FWD8_NT
#define QL_LIST_FWD8_NT 512
#endif
#ifndef QL_LIST_FWD8_DEPTH
#define QL_LIST_FWD8_DEPTH 4
#endif
#ifndef QL_LIST_FWD16_DEPTH
#define QL_LIST_FWD16_DEPTH 3
#endif
#ifndef QL_LIST_BWD_NCW
#define QL_LIST_BWD_NCW 2
#endif
#ifndef QL_LIST_BWD_DEPTH
#define QL_LIST_BWD_DEPTH 3
#endif
// Cost model of the partition, in units of streaming one unit (forward 2 KB, backward 16 KB): what the end of a
// segment costs, what a slab's output stage costs, what an adapter item costs.  From the timing probe of a debug build
// (forward, one token, 65B block: a unit 0.12 us; reduction + partial store + arrival about 6 us; an output stage about
// 12 us; an adapter item about 20 us, part of it overlapped; backward units are 8 times larger), then chosen by
// measurement on the same block (1 / 4 / 16 tokens, us per launch; forward as tail, stage, item): 50, 100, 100: 136 /
// 146 / 164; 40, 130, 150: 137 / 140 / 166; 60, 160, 100: 136 / 139 / 163; 70, 200, 120: 137 / 138 / 159; 60, 240, 100:
// 138 / 140 / 161; 30, 100, 60: 141 / 144 / 166 (equal units with a credit of 64 per item, the previous rule: 148 / 154 /
// 178).  Backward: 6, 12, 12: 170 / 178 / 214; 0, 0, 8: 167 / 174 / 208; 3, 6, 8: 161 / 169 / 204; 2, 4, 6: 161 / 167 / 199;
// 4, 8, 8: 164 / 170 / 203; 10, 20, 16: 173 / 178 / 210.
#ifndef QL_LIST_TAIL_FWD
#define QL_LIST_TAIL_FWD 70
#endif
#ifndef QL_LIST_FIN_FWD
#define QL_LIST_FIN_FWD 200
#endif
#ifndef QL_LIST_ITEM_FWD
#define QL_LIST_ITEM_FWD 120
#endif
#ifndef QL_LIST_TAIL_BWD
#define QL_LIST_TAIL_BWD 2
#endif
#ifndef QL_LIST_FIN_BWD
#define QL_LIST_FIN_BWD 4
#endif
#ifndef QL_LIST_ITEM_BWD
#define QL_LIST_ITEM_BWD 6
#endif

namespace qlora {

namespace {

using namespace few;

// LDS map of a persistent workgroup.  The decode table is never overwritten.
constexpr int kLRed = 64 * 1024;                             // 64 KB: cross-wave sums, output-stage staging, adapter sums
constexpr int kLUnit = 128 * 1024;                           // float[256]
constexpr int kLStrip = kLUnit + 1024;                       // float[16 waves][64]
constexpr int kLPend = kLStrip + 16 * 256;                   // int[1 + kFewMaxSlabs]
constexpr int kListSmem = kLPend + 4 * (1 + 2048);
static_assert(kLutBytes <= kLRed && kListSmem <= 160 * 1024, "LDS map");

constexpr int kCtrShake = 2048;                              // [kCtrShake + slab]: handshake of a slab's last contributor with the adapter
constexpr int kCtrStatus = 2047;                             // sticky: an arrival word was found in a state no call leaves behind
constexpr unsigned kMask24 = 0x00ffffffu;
constexpr unsigned kSplitBit = 1u << 23;                     // handshake word: the slab's contributors (bits 0 .. 22: adapter items)

struct ListLayer {
  const uint16_t* X;                                         // M x h (forward) or dY, M x o (backward)
  const uint8_t* packed; const uint8_t* code; const float* c1; const float* mean;
  const uint16_t* L;                                         // adapter's inner matrix: L1 (forward), L2 (backward)
  const uint16_t* Bmat;                                      // adapter's outer matrix: L2 (forward), L1 (backward)
  float* part;                                               // [n_slabs][max_contrib][M][256]
  float* lpart;                                              // [n_lparts][M][r]
  uint16_t* out;                                             // M x o (forward) or M x h (backward)
  uint16_t* hl;                                              // M x 2r [hi | lo] pair of the adapter's inner product, or NULL
  int h, o, r; float scale;
  int n_slabs, ups;                                          // slabs of 256 outputs; units per slab
  int unit0, a0;                                             // first unit / first adapter item of this layer in the list
  int n_lparts, lora_chunk, ctr0, max_contrib;
};

struct ListArgs {
  int n, M, dtype;
  unsigned nonce;
  int spin_limit;
  unsigned* hdr;
  ListPart part;
  Table4 tab;
  ListLayer L[kListMax];
};
static_assert(sizeof(ListArgs) <= 4096, "kernel arguments are limited to 4 KB");

__device__ __forceinline__ FewArgs layer_args(const ListArgs& A, const ListLayer& y) {
  FewArgs p;
  p.X = y.X; p.M = A.M; p.packed = y.packed; p.code = y.code; p.c1 = y.c1; p.mean = y.mean; p.dtype = A.dtype;
  p.h = y.h; p.o = y.o; p.part = y.part; p.per_split = 0; p.n_slabs = y.n_slabs; p.splits = 0;
  p.L = y.L; p.r = y.r; p.lpart = y.lpart; p.n_lparts = y.n_lparts; p.ctr = A.hdr + y.ctr0; p.Bmat = y.Bmat;
  p.scale = y.scale; p.out = y.out; p.hl = y.hl; p.lora_chunk = y.lora_chunk; p.hdr = A.hdr; p.nonce = A.nonce;
  p.spin_limit = A.spin_limit;
  return p;
}

// A word this call may find: zero, or its own tag with bits inside `allowed`.
__device__ __forceinline__ bool word_dirty(unsigned w, unsigned nonce, unsigned allowed) {
  return w != 0u && ((w >> 24) != nonce || (w & kMask24 & ~allowed) != 0u);
}
__device__ __forceinline__ void raise_status(unsigned* hdr) { atomicOr(hdr + kCtrStatus, 1u); }

// Contributor j of `total` arrives at *c; true for the one that completes the mask.  Everything the workgroup
// stored before the call is visible to the last arriver: thread 0 alone pays for the device-scope fences, the
// barriers extend them to the workgroup (the partials are stored write-through, so the release has nothing to
// write back).
__device__ __forceinline__ bool arrive_mask(const FewArgs& p, unsigned* c, int j, int total, volatile int* flag) {
  __syncthreads();
  if (threadIdx.x == 0) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    const unsigned bit = 1u << j, full = (1u << total) - 1u;
    const unsigned old = atomicOr(c, (p.nonce << 24) | bit);
    if (word_dirty(old, p.nonce, full) || (old & bit)) raise_status(p.hdr);
    const int last = ((old | bit) & kMask24) == full;
    if (last) {
      atomicExch(c, 0u);                                     // nobody else touches this word any more
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    }
    *flag = last;
  }
  __syncthreads();
  return *flag != 0;
}

// The workgroup that completed a slab's partials meets the adapter at the slab's handshake word: adapter item q
// sets bit q there (at every slab of its layer), the slab's side sets kSplitBit.  The adapter's items are the
// first things the first workgroups do and are normally long done; otherwise the slab's side polls a BOUNDED
// number of times and then sets its bit and leaves: whoever completes the mask owns the output stage.
__device__ __forceinline__ bool meet_adapter_mask(const FewArgs& p, unsigned* shake, volatile int* flag, unsigned early) {
  const unsigned adapters = (1u << p.n_lparts) - 1u;
  __syncthreads();                                           // everybody has read the previous flag
  if (threadIdx.x == 0) {
    if (word_dirty(early, p.nonce, adapters)) raise_status(p.hdr);
    int mine = (early & kMask24) == adapters;                // seen complete already (the mask cannot change any more)
    for (int it = 0; !mine && it < p.spin_limit; ++it) {
      if ((__hip_atomic_load(shake, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & kMask24) == adapters) { mine = 1; break; }
      __builtin_amdgcn_s_sleep(16);
    }
    if (mine) {
      __hip_atomic_store(shake, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // nobody reads it any more
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");     // the adapter's partials
    } else {
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");     // hands the slab's partials on to the adapter item that will be last
      const unsigned old = atomicOr(shake, (p.nonce << 24) | kSplitBit);
      if (word_dirty(old, p.nonce, adapters)) raise_status(p.hdr);
      mine = (old & kMask24) == adapters;                    // it came in after the last poll after all
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
// out[m][n] = bf16( sum_j part[j][m][c] + scale * sum_t T[m][t] * B(t, n) ),  T = sum_q lpart[q], for the 256 outputs
// n = 256 slab + c of one slab; forward: B(t, n) = L2[t][n]; backward: B(t, n) = L1[n][t].  `part` points at the slab's
// [contrib][M][256] tiles.  Run by all NT threads of one workgroup: a thread owns one column and four tokens per pass.
// Slab 0 also stores T as a [hi | lo] bf16 pair.  `scratch`: 52 KB of LDS.
template <bool BWD, int NT>
__device__ void list_finalize(const FewArgs& p, int slab, const float* part, int contrib, char* scratch, unsigned* shake,
                              volatile int* flag) {
  constexpr int RC = 64;                                     // rank columns staged at a time
  constexpr int kPitch = RC + 8;                             // backward tile row pitch keeps 16-byte alignment
  constexpr int P = 1024 / NT;                               // passes over the tokens (4 per 256 threads and pass)
#ifndef QL_LIST_FIN_JB
#define QL_LIST_FIN_JB 8
#endif
#ifndef QL_LIST_FIN_JB_BWD
#define QL_LIST_FIN_JB_BWD 2
#endif
  constexpr int JB = BWD ? QL_LIST_FIN_JB_BWD : QL_LIST_FIN_JB;   // ranks per batch of LDS reads in the adapter product
  constexpr int IT = 2048 / NT;                              // an adapter tile is at most 2048 chunks of 16 bytes
  float* Ts = (float*)scratch;                               // T[t][m], unscaled: 16 KB
  uint16_t* Bs = (uint16_t*)(scratch + 16384);               // forward [RC][256], backward [256][kPitch]
  const int N = BWD ? p.h : p.o;
  const int n0 = slab * 256;
  const int c = threadIdx.x & 255, tq = threadIdx.x >> 8;    // column within the slab, token quad of a pass
  const int n = n0 + c;
  const bool n_ok = n < N;

  // everything that does not depend on the adapter's partials is loaded first
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
  unsigned early = 0u;
  if (p.r > 0 && shake && threadIdx.x == 0) early = __hip_atomic_load(shake, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);

  // The loads of a stage are all issued before any is used (clamped addresses, values masked afterwards: no branch
  // between them), and the sums run in a fixed order: a stage costs one memory round trip, not one per contributor and
  // pass -- with the loads interleaved with their sums the output stage took 10 us at one token and 26 us at 16.
  float acc[P][4], lora[P][4];
#pragma unroll
  for (int q = 0; q < P; ++q)
#pragma unroll
    for (int u = 0; u < 4; ++u) { acc[q][u] = 0.0f; lora[q][u] = 0.0f; }
#ifndef QL_LIST_FIN_BATCH
#define QL_LIST_FIN_BATCH 4
#endif
  constexpr int CB = QL_LIST_FIN_BATCH;                      // contributors per batch: P * CB * 4 loads in flight
  for (int sp0 = 0; sp0 < contrib; sp0 += CB) {
    float v[P][CB][4];
#pragma unroll
    for (int q = 0; q < P; ++q) {
      const int m0 = 4 * tq + q * (NT / 64);
#pragma unroll
      for (int b = 0; b < CB; ++b) {
        const bool ok = m0 < p.M && sp0 + b < contrib;
        const float* ps = part + (int64_t)(ok ? sp0 + b : 0) * p.M * 256 + c;
#pragma unroll
        for (int u = 0; u < 4; ++u) v[q][b][u] = ps[(ok && m0 + u < p.M ? m0 + u : 0) * 256];
      }
    }
    // Nothing above uses a loaded value; the barrier keeps the scheduler from moving the masks and sums up between
    // the loads, where each would wait for its own load.
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int q = 0; q < P; ++q) {
      const int m0 = 4 * tq + q * (NT / 64);
#pragma unroll
      for (int b = 0; b < CB; ++b)
#pragma unroll
        for (int u = 0; u < 4; ++u) acc[q][u] += (m0 + u < p.M && sp0 + b < contrib) ? v[q][b][u] : 0.0f;
    }
  }
  if (p.r > 0) {
    if (shake && !meet_adapter_mask(p, shake, flag, early)) return;   // the adapter comes later: the slab is its
    const int n_e = p.M * p.r;
    for (int e0 = threadIdx.x; e0 < n_e; e0 += 2 * NT) {     // two elements of T per thread and turn
      float t[2] = {0.0f, 0.0f};
      for (int q0 = 0; q0 < p.n_lparts; q0 += 8) {           // 16 loads in flight, then a fixed-order sum
        float v[2][8];
#pragma unroll
        for (int w = 0; w < 2; ++w) {
          const int e = e0 + w * NT;
#pragma unroll
          for (int q = 0; q < 8; ++q) {
            const bool ok = e < n_e && q0 + q < p.n_lparts;
            v[w][q] = p.lpart[(int64_t)(ok ? q0 + q : 0) * n_e + (ok ? e : 0)];
          }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int w = 0; w < 2; ++w)
#pragma unroll
          for (int q = 0; q < 8; ++q) t[w] += (e0 + w * NT < n_e && q0 + q < p.n_lparts) ? v[w][q] : 0.0f;
      }
#pragma unroll
      for (int w = 0; w < 2; ++w) {
        const int e = e0 + w * NT;
        if (e < n_e) {
          const int m = e / p.r, j = e - m * p.r;
          Ts[j * 16 + m] = t[w];
          if (p.hl && slab == 0) {
            const uint16_t hi = bf16_bits(t[w]);
            p.hl[(int64_t)m * 2 * p.r + j] = hi;
            p.hl[(int64_t)m * 2 * p.r + p.r + j] = bf16_bits(t[w] - bf16_lo_to_f32(hi));
          }
        }
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
      // The LDS reads of JB ranks are issued together and the products follow in rank order (the order of the sums
      // is that of a plain loop over the ranks): read by read, each rank cost one LDS round trip.
      for (int jb = 0; jb < rc; jb += JB) {
        float bb[JB];
        f32x4 tt[P][JB];
#pragma unroll
        for (int i = 0; i < JB; ++i) {
          const int j = jb + i < rc ? jb + i : rc - 1;       // past the tile: a valid row, its product is skipped
          bb[i] = bf16_lo_to_f32(BWD ? Bs[c * kPitch + j] : Bs[j * 256 + c]);
#pragma unroll
          for (int q = 0; q < P; ++q) tt[q][i] = *(const f32x4*)&Ts[(j0 + j) * 16 + 4 * tq + q * (NT / 64)];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int q = 0; q < P; ++q)
#pragma unroll
          for (int i = 0; i < JB; ++i)
            if (jb + i < rc) {
#pragma unroll
              for (int u = 0; u < 4; ++u) lora[q][u] = __builtin_fmaf(tt[q][i][u], bb[i], lora[q][u]);
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

// How many workgroups contribute to a slab, and which of them this one is (both from the partition formula).
struct Contrib { int j, total; };
__device__ __forceinline__ Contrib slab_contrib(const ListPart& part, const ListLayer& y, int slab, int rho) {
  const int U0 = y.unit0 + slab * y.ups;
  const int first = list_rho_of(part, U0), last = list_rho_of(part, U0 + y.ups - 1);
  return Contrib{rho - first, last - first + 1};
}
__device__ __forceinline__ const float* slab_part(const FewArgs& p, const ListLayer& y, int slab) {
  return y.part + (int64_t)slab * y.max_contrib * p.M * 256;
}

// Called by a workgroup after it has stored adapter partial `item` of a layer: it sets its bit at every slab's
// handshake word.  A slab whose mask it completes (the slab's side gave up waiting: rare) is finished right here.
template <bool BWD, int NT>
__device__ void list_adapter_arrive(const ListArgs& A, const ListLayer& y, const FewArgs& p, int item, char* scratch,
                                    int* npend, volatile int* flag) {
  int* pend = npend + 1;
  const unsigned adapters = (1u << p.n_lparts) - 1u, bit = 1u << item;
  if (threadIdx.x == 0) *npend = 0;
  __syncthreads();                                           // the partial of this workgroup is stored
  for (int t = threadIdx.x; t < p.n_slabs; t += NT) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    const unsigned old = atomicOr(p.ctr + kCtrShake + t, (p.nonce << 24) | bit);
    if (word_dirty(old, p.nonce, adapters | kSplitBit) || (old & bit)) raise_status(p.hdr);
    if (((old | bit) & kMask24) == (adapters | kSplitBit)) {  // every other adapter item and the slab's side are in
      atomicExch(p.ctr + kCtrShake + t, 0u);
      pend[atomicAdd(npend, 1)] = t;
    }
  }
  __syncthreads();
  const int n = *npend;
  if (n > 0) {
    if (threadIdx.x == 0) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");   // everybody arrived before us
    __syncthreads();
  }
  for (int q = 0; q < n; ++q) {
    const int slab = pend[q];
    const int U0 = y.unit0 + slab * y.ups;
    const int contrib = list_rho_of(A.part, U0 + y.ups - 1) - list_rho_of(A.part, U0) + 1;
    list_finalize<BWD, NT>(p, slab, slab_part(p, y, slab), contrib, scratch, nullptr, flag);
    __syncthreads();
  }
}

// One segment of a workgroup's range: steps [s0, s1) of one slab of one layer.
struct Seg { int l, slab, s0, s1, u_end; };
__device__ __forceinline__ Seg seg_at(const ListArgs& A, int u, int u1) {
  Seg s;
  s.l = 0;
  while (s.l + 1 < A.n && u >= A.L[s.l + 1].unit0) ++s.l;
  const int rel = u - A.L[s.l].unit0, ups = A.L[s.l].ups;
  s.slab = rel / ups;
  s.s0 = rel - s.slab * ups;
  s.s1 = (s.s0 + (u1 - u) < ups) ? s.s0 + (u1 - u) : ups;
  s.u_end = u + (s.s1 - s.s0);
  return s;
}
// steps of a segment that fall to lane-group `w` of `nw` (they interleave), and that count rounded up to the ring depth
// QL_LIST_ROTATE: in round i lane-group w takes step nw i + (w + i) % nw instead of nw i + w, so that a wave does not
// keep to one residue class of rows (nw is a power of two).
#ifndef QL_LIST_ROTATE
#define QL_LIST_ROTATE 0
#endif
// QL_LIST_BWD_GROUP (backward only): a wave takes its 128-column steps in runs of this many adjacent ones -- steps
// G (nw j + w) .. + G - 1 -- so that the 64-byte pieces of a weight row that share a 128-byte line (and, with 4, the
// neighbouring line) are asked for by the same wave, one ring position apart.  Measured on the 65B block (1 / 4 / 16
// tokens, us per launch): 1: 161 / 167 / 199; 2: 155 / 162 / 194; 4: 157 / 164 / 195; 8: 158 / 165 / 194.
#ifndef QL_LIST_BWD_GROUP
#define QL_LIST_BWD_GROUP 2
#endif
__device__ __forceinline__ int group_step_of(int w, int i, int nw) {
  constexpr int G = QL_LIST_BWD_GROUP;
  return G * (nw * (i / G) + w) + (i % G);
}
__device__ __forceinline__ int group_seg_steps(int len, int w, int nw) {
  constexpr int G = QL_LIST_BWD_GROUP;
  const int groups = (len + G - 1) / G;                      // the last group may be short
  if (groups <= w) return 0;
  const int mine = (groups - w + nw - 1) / nw;               // groups w, w + nw, ...
  const int last = w + nw * (mine - 1);
  return G * mine - (last == groups - 1 ? groups * G - len : 0);
}
__device__ __forceinline__ int step_of(int w, int i, int nw) {
  return QL_LIST_ROTATE ? nw * i + ((w + i) & (nw - 1)) : nw * i + w;
}
__device__ __forceinline__ int seg_steps(const Seg& s, int w, int nw) {
  const int len = s.s1 - s.s0;
  if (QL_LIST_ROTATE) {
    const int full = len / nw, rem = len - full * nw;
    return full + ((((w + full) & (nw - 1)) < rem) ? 1 : 0);
  }
  return len > w ? (len - w + nw - 1) / nw : 0;
}

// ---- forward --------------------------------------------------------------------------------------
// See the one-layer forward kernel for the lane layout of a step (16 weight rows x 256 columns per wave and step).
struct LFwd { uint32_t pk[8]; u32x4 x; uint32_t code; float c1; float mean; };   // raw loads only

template <int MT, int NT, int kDepth>
__global__ __launch_bounds__(NT) void fewlist_fwd_kernel(const ListArgs A) {
  constexpr int NA = MT / 8;                                 // accumulator sets (and MFMAs per column phase)
  constexpr int NW = NT / 64, HW = NW / 2;
  constexpr int kTile = MT * 256;                            // floats of one wave's [MT][256] tile
  static_assert(HW * kTile * 4 <= 64 * 1024, "half of the waves' tiles fit the sum area");
  __shared__ __attribute__((aligned(256))) char smem[kListSmem];
  __shared__ int flag;
  f32x2* lut2 = (f32x2*)smem;
  float* red = (float*)(smem + kLRed);
  float* unit = (float*)(smem + kLUnit);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;   // uniform
  const int rho = work_index();
  const int G = (int)gridDim.x;

  // the adapter's inner products first
  for (int it = rho; it < A.part.n_adapter; it += G) {
    int l = 0;
    while (l + 1 < A.n && it >= A.L[l + 1].a0) ++l;
    const FewArgs p = layer_args(A, A.L[l]);
    lora_fwd_partial<NT>(p, it - A.L[l].a0, red);
    list_adapter_arrive<false, NT>(A, A.L[l], p, it - A.L[l].a0, smem + kLRed, (int*)(smem + kLPend), &flag);
    __syncthreads();
  }
  const int u0 = list_start(A.part, rho), u1 = list_start(A.part, rho + 1);
  if (u0 >= u1) return;

  const int c = lane & 31, rh = lane >> 5;
  const int sl = lane & 15, g = lane >> 4;                   // MFMA slot and k group
  const uint32_t lane_off = 8u * (uint32_t)(lane & (kLutCopies - 1));
  float* strip = (float*)(smem + kLStrip) + wave * 64;       // [block 4][row 16]
  const int tok = MT == 8 ? (sl & 7) : sl;
  const bool x_ok = tok < A.M && (MT == 16 || (g & 1) == (sl >> 3));
  const uint32_t c_row = (uint32_t)(lane >> 2);

  // ---- load cursor: runs kDepth positions ahead of the compute cursor, across segment boundaries ----
  // A load address is a wave-uniform 64-bit base (layer, slab, row of the step) plus a per-lane 32-bit byte offset
  // that changes only with the segment: the loads take the scalar-base form and cost no vector address arithmetic.
  Seg ls = seg_at(A, u0, u1);
  const char* l_packed; const char* l_X; const uint8_t* l_code; const float* l_c1; const float* l_mean;
  int l_rowb, l_bpr, l_cw;                                   // bytes per packed row, blocks per row, blocks in the column group
  uint32_t w_lane, x_lane, code_lane, c1_lane;
  auto setup_load = [&]() {
    const ListLayer& y = A.L[ls.l];
    l_packed = (const char*)y.packed; l_X = (const char*)y.X; l_c1 = y.c1; l_mean = y.mean;
    l_rowb = y.o >> 1; l_bpr = y.o >> 6;
    const bool col_ok = ls.slab * 256 + 8 * c < y.o;         // o % 64 == 0: a dword is in or out as a whole
    w_lane = (uint32_t)(8 * rh * l_rowb + 4 * (col_ok ? ls.slab * 32 + c : 0));
    x_lane = (uint32_t)(2 * ((tok < A.M ? tok : 0) * y.h + 8 * (g >> 1)));
    l_cw = (4 * ls.slab + 4 <= l_bpr) ? 4 : l_bpr - 4 * ls.slab;   // blocks in this column group
    const bool c_ok = (lane & 3) < l_cw;
    code_lane = c_row * (uint32_t)l_cw + (c_ok ? (uint32_t)(lane & 3) : 0u);
    c1_lane = c_row * (uint32_t)l_bpr + (uint32_t)(4 * ls.slab + (c_ok ? (lane & 3) : 0));
    l_code = y.code + (int64_t)4 * y.h * ls.slab;
  };
  setup_load();
  int ln = seg_steps(ls, wave, NW), lit = (ln + kDepth - 1) / kDepth * kDepth, li = 0;
  bool l_done = false;
  int kc_last = ls.s0 * 16;                                  // where a position without a step loads from (never consumed)
  auto skip_empty = [&]() {                                  // move the load cursor to the next segment that gives this wave steps
    while (!l_done && li >= lit) {
      if (ls.u_end >= u1) { l_done = true; break; }
      ls = seg_at(A, ls.u_end, u1);
      setup_load();
      ln = seg_steps(ls, wave, NW); lit = (ln + kDepth - 1) / kDepth * kDepth; li = 0;
      kc_last = ls.s0 * 16;
    }
  };
  skip_empty();
  // one position of the load cursor; the move to another segment (skip_empty) is left to the caller, outside the
  // innermost loop: a rarely taken path that rejoins there makes the compiler wait for every load in flight
  auto next_load = [&](LFwd& s) {
    const bool valid = !l_done && li < ln;
    const int kc = valid ? (ls.s0 + step_of(wave, li, NW)) * 16 : kc_last;
    kc_last = kc;
    const char* wbase = l_packed + (int64_t)kc * l_rowb;
#pragma unroll
    for (int j = 0; j < 8; ++j) s.pk[j] = *(const uint32_t*)(wbase + (int64_t)j * l_rowb + w_lane);
    s.x = *(const u32x4*)(l_X + 2 * kc + x_lane);
    s.code = (l_code + (int64_t)kc * l_cw)[code_lane];
    s.c1 = l_c1[((uint32_t)(kc * l_bpr) + c1_lane) >> 8];
    s.mean = *l_mean;
    ++li;
  };

  LFwd buf[kDepth];
#pragma unroll
  for (int d = 0; d < kDepth; ++d) next_load(buf[d]);        // in flight while the decode table is built
  skip_empty();
  init_pair_lut<NT>(lut2, unit, A.dtype, A.tab, (float*)(smem + kLStrip));
  __syncthreads();

  f32x4 acc[NA][8];
  auto zero_acc = [&]() {
#pragma unroll
    for (int a = 0; a < NA; ++a)
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[a][e] = f32x4{0.f, 0.f, 0.f, 0.f};
  };
  zero_acc();

  auto compute = [&](const LFwd& s) {
    // dequant(c1, c2): two separately rounded fp32 steps; wave-private strip: no barrier needed
    strip[(lane & 3) * 16 + (lane >> 2)] = __fadd_rn(__fmul_rn(unit[s.code], s.c1), s.mean);
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
    f32x2 qn[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) qn[j] = pair_lookup_b(lut2, s.pk[j], lane_off, 0);
#pragma unroll
    for (int b = 0; b < 4; ++b) {                            // byte b of every row: columns 2b, 2b + 1 of the dword
      f32x2 q[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) q[j] = qn[j];
      if (b < 3) {
#pragma unroll
        for (int j = 0; j < 8; ++j) qn[j] = pair_lookup_b(lut2, s.pk[j], lane_off, b + 1);
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

  // D layout: column slot = lane % 16, rows 4 * (lane / 16) + v.  Row R of accumulator set a is token R % MT of
  // column half (MT == 8 ? R / 8 : a); column within the half = 8 slot + e.
  auto tile_index = [&](int a, int e, int vv) {
    const int R = 4 * g + vv;
    const int m = MT == 8 ? (R & 7) : R, half = MT == 8 ? (R >> 3) : a;
    return m * 256 + half * 128 + 8 * sl + e;
  };

  for (Seg cs = seg_at(A, u0, u1);; cs = seg_at(A, cs.u_end, u1)) {
    const int cn = seg_steps(cs, wave, NW), cit = (cn + kDepth - 1) / kDepth * kDepth;
    for (int i = 0; i < cit;) {
      // as many positions as the load cursor can take without changing its segment (both counts are multiples of
      // the ring depth, so the ring stays aligned)
      const int room = l_done ? cit - i : lit - li;
      const int i_end = (cit - i < room) ? cit : i + room;
      for (; i < i_end; i += kDepth) {
#pragma unroll
        for (int d = 0; d < kDepth; ++d) {
          if (i + d < cn) compute(buf[d]);
          next_load(buf[d]);
        }
      }
      skip_empty();
    }
    // ---- the segment's partial: sum over the waves (half of them at a time: the decode table stays) ----
    if (wave >= HW) {
      float* my = red + (wave - HW) * kTile;
#pragma unroll
      for (int a = 0; a < NA; ++a)
#pragma unroll
        for (int e = 0; e < 8; ++e)
#pragma unroll
          for (int vv = 0; vv < 4; ++vv) my[tile_index(a, e, vv)] = acc[a][e][vv];
    }
    __syncthreads();
    if (wave < HW) {
      float* my = red + wave * kTile;
#pragma unroll
      for (int a = 0; a < NA; ++a)
#pragma unroll
        for (int e = 0; e < 8; ++e)
#pragma unroll
          for (int vv = 0; vv < 4; ++vv) {
            const int ix = tile_index(a, e, vv);
            my[ix] += acc[a][e][vv];
          }
    }
    __syncthreads();
    const ListLayer& y = A.L[cs.l];
    const FewArgs p = layer_args(A, y);
    const Contrib cb = slab_contrib(A.part, y, cs.slab, rho);
    const float* pslab = slab_part(p, y, cs.slab);
    float* out = (float*)pslab + (int64_t)cb.j * p.M * 256;
    for (int idx = threadIdx.x; idx < p.M * 256; idx += NT) {
      float t = 0.0f;
#pragma unroll
      for (int w = 0; w < HW; ++w) t += red[w * kTile + idx];
      __hip_atomic_store(out + idx, t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (arrive_mask(p, p.ctr + cs.slab, cb.j, cb.total, &flag))
      list_finalize<false, NT>(p, cs.slab, pslab, cb.total, smem + kLRed, p.ctr + kCtrShake + cs.slab, &flag);
    if (cs.u_end >= u1) break;
    zero_acc();
    __syncthreads();                                         // the sum area is free again
  }
}

// ---- backward -------------------------------------------------------------------------------------
// See the one-layer backward kernel for the lane layout: wave (rg = wave % 4, cw = wave / 4) owns weight rows
// 64 rg .. +63 of the slab and takes the 128-column steps cw, cw + NCW, ... of a segment (NCW waves per row group).
struct LBwd { u32x4 w[4]; u32x4 y[4]; uint32_t code[4]; float c1[4]; float mean; };   // raw loads only

template <int NCW, int kDepth>
__global__ __launch_bounds__(256 * NCW) void fewlist_bwd_kernel(const ListArgs A) {
  constexpr int NT = 256 * NCW;
  static_assert(NCW == 2 || NCW == 4, "two or four waves per row group");
  __shared__ __attribute__((aligned(256))) char smem[kListSmem];
  __shared__ int flag;
  f32x2* lut2 = (f32x2*)smem;
  float* red = (float*)(smem + kLRed);
  float* unit = (float*)(smem + kLUnit);
  const int wave16 = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;   // uniform
  const int rho = work_index();
  const int G = (int)gridDim.x;

  for (int it = rho; it < A.part.n_adapter; it += G) {
    int l = 0;
    while (l + 1 < A.n && it >= A.L[l + 1].a0) ++l;
    const FewArgs p = layer_args(A, A.L[l]);
    lora_bwd_partial<NT>(p, it - A.L[l].a0, red);
    list_adapter_arrive<true, NT>(A, A.L[l], p, it - A.L[l].a0, smem + kLRed, (int*)(smem + kLPend), &flag);
    __syncthreads();
  }
  const int u0 = list_start(A.part, rho), u1 = list_start(A.part, rho + 1);
  if (u0 >= u1) return;

  const int rg = wave16 & 3, cw = wave16 >> 2;
  auto bwd_steps = [&](const Seg& sg, int w) { return group_seg_steps(sg.s1 - sg.s0, w, NCW); };
  auto bwd_step = [&](int w, int i) { return group_step_of(w, i, NCW); };
  const int i = lane & 15, g = lane >> 4;
  const uint32_t lane_off = 8u * (uint32_t)(lane & (kLutCopies - 1));
  const bool y_row_ok = i < A.M;

  Seg ls = seg_at(A, u0, u1);
  const u32x4* l_packed; const uint16_t* l_X; const uint8_t* l_code; const float* l_c1; const float* l_mean;
  int l_o, l_h, l_bpr;
  uint32_t w_off[4], cd_off[4], row_c[4], y_off;
  auto setup_load = [&]() {
    const ListLayer& y = A.L[ls.l];
    l_packed = (const u32x4*)y.packed; l_X = y.X; l_code = y.code; l_c1 = y.c1; l_mean = y.mean;
    l_o = y.o; l_h = y.h; l_bpr = y.o >> 6;
    const int r0 = ls.slab * 256 + rg * 64;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int row = r0 + 16 * u + i;
      row_c[u] = (uint32_t)(row < y.h ? row : 0);
      w_off[u] = row_c[u] * (uint32_t)(y.o >> 5);            // 16-byte groups (32 weights) per row
      cd_off[u] = row_c[u] * (uint32_t)l_bpr;
    }
    y_off = (uint32_t)((y_row_ok ? i : 0) * y.o);
  };
  setup_load();
  int ln = bwd_steps(ls, cw), lit = (ln + kDepth - 1) / kDepth * kDepth, li = 0;
  bool l_done = false;
  int kb_last = ls.s0 * 128;
  auto skip_empty = [&]() {
    while (!l_done && li >= lit) {
      if (ls.u_end >= u1) { l_done = true; break; }
      ls = seg_at(A, ls.u_end, u1);
      setup_load();
      ln = bwd_steps(ls, cw); lit = (ln + kDepth - 1) / kDepth * kDepth; li = 0;
      kb_last = ls.s0 * 128;
    }
  };
  skip_empty();
  auto next_load = [&](LBwd& s) {                            // see the forward kernel
    const bool valid = !l_done && li < ln;
    const int kb = valid ? (ls.s0 + bwd_step(cw, li)) * 128 : kb_last;
    kb_last = kb;
    int col = kb + 32 * g;                                   // per lane
    if (col >= l_o) col = l_o - 64 + 32 * (g & 1);           // the half-empty last step: any valid column (masked at compute)
    const u32x4* wbase = l_packed + (col >> 5);
    // constants are stored column-group-major: the 16 rows x 2 blocks of one load sit within 64 bytes
    const int blk = col >> 6, Gc = blk >> 2;
    const uint32_t cwid = (4 * Gc + 4 <= l_bpr) ? 4u : (uint32_t)(l_bpr - 4 * Gc);
    const uint8_t* cbase = l_code + (int64_t)4 * l_h * Gc + (blk & 3);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      s.w[u] = wbase[w_off[u]];
      s.code[u] = cbase[row_c[u] * cwid];
      s.c1[u] = l_c1[(cd_off[u] + (uint32_t)blk) >> 8];
    }
    const uint16_t* ysrc = l_X + y_off + col;
#pragma unroll
    for (int t = 0; t < 4; ++t) s.y[t] = *(const u32x4*)(ysrc + 8 * t);
    s.mean = *l_mean;
    ++li;
  };

  LBwd buf[kDepth];
#pragma unroll
  for (int d = 0; d < kDepth; ++d) next_load(buf[d]);        // in flight while the table is built
  skip_empty();
  init_pair_lut<NT>(lut2, unit, A.dtype, A.tab, (float*)(smem + kLStrip));
  __syncthreads();

  f32x4 acc[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) acc[u] = f32x4{0.f, 0.f, 0.f, 0.f};

  auto compute = [&](const LBwd& s, bool y_ok) {             // y_ok: this lane's 32 columns exist and its token row too
    float c2v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) c2v[u] = __fadd_rn(__fmul_rn(unit[s.code[u]], s.c1[u]), s.mean);
    // 8 groups of 8 lookups: dword t of weight-row groups 2 uh, 2 uh + 1; the lookups of the next group are issued
    // before the arithmetic of this one (see the forward kernel)
    auto lookups = [&](f32x2 (&q)[2][4], int grp) {
      const int t = grp >> 1, uh = grp & 1;
#pragma unroll
      for (int v = 0; v < 2; ++v)
#pragma unroll
        for (int b = 0; b < 4; ++b) q[v][b] = pair_lookup_b(lut2, s.w[2 * uh + v][t], lane_off, b);
    };
    f32x2 qn[2][4];
    lookups(qn, 0);
#pragma unroll
    for (int grp = 0; grp < 8; ++grp) {
      const int t = grp >> 1, uh = grp & 1;
      f32x2 q[2][4];
#pragma unroll
      for (int v = 0; v < 2; ++v)
#pragma unroll
        for (int b = 0; b < 4; ++b) q[v][b] = qn[v][b];
      if (grp < 7) lookups(qn, grp + 1);
      __builtin_amdgcn_sched_barrier(0);
      const bf16x8 ya = __builtin_bit_cast(bf16x8, y_ok ? s.y[t] : u32x4{0u, 0u, 0u, 0u});
#pragma unroll
      for (int v = 0; v < 2; ++v) {
        const int u = 2 * uh + v;
        u32x4 w;
#pragma unroll
        for (int b = 0; b < 4; ++b) w[b] = pack_bf16x2(__fmul_rn(q[v][b][0], c2v[u]), __fmul_rn(q[v][b][1], c2v[u]));
        acc[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ya, __builtin_bit_cast(bf16x8, w), acc[u], 0, 0, 0);
      }
    }
  };

  for (Seg cs = seg_at(A, u0, u1);; cs = seg_at(A, cs.u_end, u1)) {
    const int cn = bwd_steps(cs, cw), cit = (cn + kDepth - 1) / kDepth * kDepth;
    const int o_cs = A.L[cs.l].o;
    for (int it = 0; it < cit;) {
      const int room = l_done ? cit - it : lit - li;
      const int it_end = (cit - it < room) ? cit : it + room;
      for (; it < it_end; it += kDepth) {
#pragma unroll
        for (int d = 0; d < kDepth; ++d) {
          if (it + d < cn) compute(buf[d], y_row_ok && (cs.s0 + bwd_step(cw, it + d)) * 128 + 32 * g < o_cs);
          next_load(buf[d]);
        }
      }
      skip_empty();
    }
    // D layout: column slot = lane % 16 = weight row within the 16-row group, token rows 4 * (lane / 16) + v.
    // Every wave stores its 16 x 64 tile; the NCW tiles of a row group are summed.
    float* my = red + wave16 * (16 * 64);
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int vv = 0; vv < 4; ++vv) my[(4 * g + vv) * 64 + 16 * u + i] = acc[u][vv];
    __syncthreads();
    const ListLayer& y = A.L[cs.l];
    const FewArgs p = layer_args(A, y);
    const Contrib cb = slab_contrib(A.part, y, cs.slab, rho);
    const float* pslab = slab_part(p, y, cs.slab);
    float* out = (float*)pslab + (int64_t)cb.j * p.M * 256;
    for (int idx = threadIdx.x; idx < p.M * 256; idx += NT) {
      const int m = idx >> 8, rr = idx & 255;
      const float* src = red + (rr >> 6) * (16 * 64) + m * 64 + (rr & 63);
      float t = 0.0f;
#pragma unroll
      for (int q = 0; q < NCW; ++q) t += src[q * 4 * 16 * 64];
      __hip_atomic_store(out + idx, t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (arrive_mask(p, p.ctr + cs.slab, cb.j, cb.total, &flag))
      list_finalize<true, NT>(p, cs.slab, pslab, cb.total, smem + kLRed, p.ctr + kCtrShake + cs.slab, &flag);
    if (cs.u_end >= u1) break;
#pragma unroll
    for (int u = 0; u < 4; ++u) acc[u] = f32x4{0.f, 0.f, 0.f, 0.f};
    __syncthreads();                                         // the sum area is free again
  }
}

}  // namespace

// ---- host side ------------------------------------------------------------------------------------
// The partition is a pure function of the shapes: the size queries, the launcher and the kernel evaluate the same
// formulas (list_start / list_rho_of in launch.hpp).
ListPlan fewlist_plan(bool bwd, int M, int n, const int* h, const int* o, const int* r) {
  ListPlan P{};
  if (n < 1 || n > kListMax || M < 1 || M > kFewTokens) return P;
  int64_t units = 0;
  int adapters = 0, slabs = 0, ups_max = 1;
  for (int l = 0; l < n; ++l) {
    const int outs = bwd ? h[l] : o[l], contr = bwd ? o[l] : h[l];
    P.n_slabs[l] = (outs + 255) / 256;
    P.ups[l] = bwd ? (contr + 127) / 128 : (contr + 15) / 16;
    P.unit0[l] = (int)units;
    units += (int64_t)P.n_slabs[l] * P.ups[l];
    if (units >= (1ll << 30)) return P;
    ups_max = std::max(ups_max, P.ups[l]);
    // adapter items: at most 23 per layer (bits 0 .. 22 of a handshake word), at least kLoraK contraction elements each
    int chunk = kListLoraChunk;
    if (r[l] > 0 && (contr + chunk - 1) / chunk > 23) chunk = ((contr + 22) / 23 + 63) / 64 * 64;
    P.lora_chunk[l] = chunk;
    P.n_lparts[l] = r[l] > 0 ? (contr + chunk - 1) / chunk : 0;
    P.a0[l] = adapters;
    adapters += P.n_lparts[l];
    P.ctr0[l] = slabs;
    slabs += P.n_slabs[l];
  }
  if (slabs > kFewMaxSlabs - 1) return P;                    // the last word of the slab range is the status word
  P.total_units = (int)units;
  P.total_slabs = slabs;
  // Estimated time of a workgroup in units of streaming one unit: its units, plus kTail for every segment (a run of
  // units within one slab: reduction, partial store, arrival), plus kFin for every slab that begins inside its range
  // (of the workgroups that share a slab the one with the slab's first units gets there last, at the end of its own
  // range, and runs the slab's output stage), plus kItem for every adapter item it computes first.  Boundaries: the
  // smallest bound T for which a greedy walk (every workgroup takes what fits under T) covers the line with `grid`
  // workgroups.
  const int kTail = bwd ? QL_LIST_TAIL_BWD : QL_LIST_TAIL_FWD, kFin = bwd ? QL_LIST_FIN_BWD : QL_LIST_FIN_FWD;
  const int kItem = bwd ? QL_LIST_ITEM_BWD : QL_LIST_ITEM_FWD;
  std::vector<int> slab_end;                                 // ascending unit index where each slab ends
  for (int l = 0; l < n; ++l)
    for (int sidx = 0; sidx < P.n_slabs[l]; ++sidx) slab_end.push_back(P.unit0[l] + (sidx + 1) * P.ups[l]);
  auto walk = [&](int grid, int64_t T, int* start) -> bool { // fills start[0 .. grid] when it returns true
    int u = 0, next_end = 0;                                 // next_end: index of the first slab that ends after u
    for (int rho = 0; rho < grid; ++rho) {
      if (start) start[rho] = u;
      const int items = rho < adapters ? (adapters - rho + grid - 1) / grid : 0;
      int64_t budget = T - (int64_t)kItem * items;
      bool took = false;
      while (u < (int)units && budget > 0) {
        while (slab_end[next_end] <= u) ++next_end;
        const int s_begin = next_end == 0 ? 0 : slab_end[next_end - 1];
        const int64_t overhead = kTail + (u == s_begin ? kFin : 0);
        if (budget <= overhead) {                            // not worth another segment; but nobody with a budget leaves empty-handed
          if (!took) { ++u; took = true; }
          break;
        }
        const int64_t room = budget - overhead;
        const int to_end = slab_end[next_end] - u;
        const int take = room >= to_end ? to_end : (int)room;
        u += take; budget -= overhead + take; took = true;
      }
    }
    if (start) start[grid] = (int)units;
    return u >= (int)units;
  };
  // fewer workgroups than compute units when there is less than one unit each, or when a slab would otherwise be
  // shared by more workgroups than an arrival word has bits for
  for (int grid = (int)std::min<int64_t>(kListGridMax, units); grid >= 1; grid = grid > 32 ? grid - 32 : grid - 1) {
    ListPart q{};
    q.grid = grid;
    q.n_adapter = adapters;
    int64_t lo = 0, hi = units + (int64_t)(kTail + kFin) * slabs + (int64_t)kItem * adapters + 1;   // walk(hi) succeeds with one workgroup
    while (hi - lo > 1) {
      const int64_t mid = (lo + hi) / 2;
      if (walk(grid, mid, nullptr)) hi = mid; else lo = mid;
    }
    walk(grid, hi, q.start);
    int worst = 1;
    for (int l = 0; l < n; ++l) {
      int mc = 1;
      for (int s = 0; s < P.n_slabs[l]; ++s) {
        const int U0 = P.unit0[l] + s * P.ups[l];
        mc = std::max(mc, list_rho_of(q, U0 + P.ups[l] - 1) - list_rho_of(q, U0) + 1);
      }
      P.max_contrib[l] = mc;
      worst = std::max(worst, mc);
    }
    if (worst <= 23) { P.part = q; P.ok = true; break; }
  }
  if (!P.ok) return P;
  for (int l = 0; l < n; ++l) {
    P.part_floats[l] = (size_t)P.n_slabs[l] * P.max_contrib[l] * M * 256;
    P.lpart_floats[l] = (size_t)P.n_lparts[l] * M * r[l] + 4;
  }
  return P;
}

hipError_t launch_fewlist(bool bwd, int M, int n, const ListLayerDesc* layers, const ListPlan& P, unsigned* hdr,
                          unsigned nonce, int spin_limit, hipStream_t st) {
  if (!P.ok || n < 1 || n > kListMax) return hipErrorInvalidValue;
  ListArgs A{};
  A.n = n; A.M = M; A.dtype = layers[0].w.dtype; A.nonce = nonce; A.spin_limit = spin_limit; A.hdr = hdr;
  A.part = P.part;
  A.tab = table4_host(A.dtype);
  for (int l = 0; l < n; ++l) {
    const ListLayerDesc& d = layers[l];
    if (d.w.dtype != A.dtype) return hipErrorInvalidValue;    // one decode table per launch
    ListLayer& y = A.L[l];
    y.X = d.X; y.packed = d.w.packed; y.code = d.w.code; y.c1 = d.w.c1; y.mean = d.w.mean;
    y.L = bwd ? d.L2 : d.L1; y.Bmat = bwd ? d.L1 : d.L2;
    y.part = d.part; y.lpart = d.lpart; y.out = d.out; y.hl = d.r > 0 ? d.hl : nullptr;
    y.h = (int)d.w.rows; y.o = (int)d.w.cols; y.r = d.r; y.scale = d.scale;
    y.n_slabs = P.n_slabs[l]; y.ups = P.ups[l]; y.unit0 = P.unit0[l]; y.a0 = P.a0[l];
    y.n_lparts = d.r > 0 ? P.n_lparts[l] : 0; y.lora_chunk = P.lora_chunk[l]; y.ctr0 = P.ctr0[l];
    y.max_contrib = P.max_contrib[l];
  }
  for (int l = n; l < kListMax; ++l) { A.L[l] = A.L[n - 1]; A.L[l].unit0 = 0x7fffffff; A.L[l].a0 = 0x7fffffff; }
  const dim3 grid((unsigned)P.part.grid);
  if (bwd) hipLaunchKernelGGL((fewlist_bwd_kernel<QL_LIST_BWD_NCW, QL_LIST_BWD_DEPTH>), grid, dim3(256 * QL_LIST_BWD_NCW), 0, st, A);
  else if (M <= 8)
    hipLaunchKernelGGL((fewlist_fwd_kernel<8, QL_LIST_FWD8_NT, QL_LIST_FWD8_DEPTH>), grid, dim3(QL_LIST_FWD8_NT), 0, st, A);
  else hipLaunchKernelGGL((fewlist_fwd_kernel<16, 512, QL_LIST_FWD16_DEPTH>), grid, dim3(512), 0, st, A);
  return hipGetLastError();
}

}  // namespace qlora
