// Internal launchers behind the C ABI.  Each enqueues kernels on `st` and returns hipGetLastError().
// Shapes have been validated by the caller (api.cpp); nothing here synchronises or allocates.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace qlora {

struct NF4Dev {            // device views of one quantised h x o weight
  const uint8_t* packed;
  const uint8_t* code;
  const float* c1;
  const float* mean;
  int64_t rows, cols;      // h, o
  int dtype;               // 0 NF4; 1 Float4 E2M1, 2 Float4 E3M0, 3 Int4 (the data types of the paper's comparison)
  bool dq;                 // Double Quantization; false: `c1` holds the rows * cols / 64 fp32 constants c2, code and mean unused
};

// quantize.hip
constexpr size_t kQuantBinsBytes = 256 * sizeof(unsigned long long);
//   dq = false: no Double Quantization; the fp32 constants c2 go to `c1` (rows * cols / 64 floats), code and mean untouched.
hipError_t launch_quantize(const float* W, int64_t rows, int64_t cols, uint8_t* packed, uint8_t* code, float* c1,
                           float* mean, void* scratch, hipStream_t st, int dtype = 0, bool dq = true);
// The same with the scratch in a device array of the library itself (no allocation anywhere on the way): tensors of
// up to kStaticQuantBlocks blocks.  Calls on one device share the array: calls that overlap there race.
constexpr size_t kStaticQuantBlocks = (size_t)4 << 20;
hipError_t launch_quantize_static(const float* W, int64_t rows, int64_t cols, uint8_t* packed, uint8_t* code,
                                  float* c1, float* mean, hipStream_t st, int dtype = 0, bool dq = true);

// dequant.hip
//   out[k][n] = dequant(W)[k][n] with row stride ld_out elements (0: cols; else >= cols and a multiple of 8)
hipError_t launch_dequant(const NF4Dev& w, uint16_t* out, hipStream_t st, int64_t ld_out = 0);
// out[n][k] = dequant(W)[k][n] with row stride ld_out (elements); requires h % 8 == 0.
// rp > 0 (a multiple of 64, ld_out >= h + rp): the same launch also writes the adapter segment, columns h .. h + rp - 1:
// out[n][h + col0 + t] = L2[t][n] for t < r (L2: r x o bf16, col0 + r <= rp; NULL: none) and zeros elsewhere.
hipError_t launch_dequant_t(const NF4Dev& w, uint16_t* out, int64_t ld_out, hipStream_t st,
                            const uint16_t* L2 = nullptr, int r = 0, int rp = 0, int col0 = 0);

// gemm.hip: C[M x N] = A0 B0^T + A1 B1^T, all operands K-contiguous bf16, K0 and K1 multiples of 64.
hipError_t launch_gemm_nt(const uint16_t* A0, const uint16_t* B0, int64_t lda0, int64_t ldb0, int K0,
                          const uint16_t* A1, const uint16_t* B1, int64_t lda1, int64_t ldb1, int K1,
                          uint16_t* C, int64_t ldc, int M, int N, hipStream_t st);

// The same product with the weight-side operand of segment 0 decoded inside the kernel: Bq = N rows of K0 / 2 bytes of
// 4-bit codes, Bc = N x K0 / 64 fp32 block constants, tab16 = the data type's 16 values (all device memory).  The
// weight tiles are bit-identical to launch_dequant's; the adapter segment (K1 = 0 or 64) is accumulated first.
bool gemm_nt_fused_fits(int K0, int K1, int N);
// Index arithmetic of the fused kernel's row loads, shared with the host-side check.  Tiles are numbered in the order
// the kernel consumes them: KT1 adapter tiles (0 or 1) first, then the KT0 steps of segment 0; KT = KT0 + KT1.
//   step of segment 0 behind tile t (t >= KT1); tiles past the end repeat the last step (their rows are never used)
__host__ __device__ inline int fused_seg0_step(int t, int KT, int KT1) { return (t < KT ? t : KT - 1) - KT1; }
//   weight row that thread `tid` (0 .. 255) of the workgroup at output column n0 decodes, clamped to the matrix
__host__ __device__ inline int fused_row(int n0, int tid, int N) { return n0 + tid < N ? n0 + tid : N - 1; }
//   byte offsets of that row's 32 bytes of codes and of its fp32 constant for one step (K0 = 64 KT0)
__host__ __device__ inline int64_t fused_code_offset(int row, int step, int KT0) { return ((int64_t)row * KT0 + step) * 32; }
__host__ __device__ inline int64_t fused_const_offset(int row, int step, int KT0) { return ((int64_t)row * KT0 + step) * 4; }
hipError_t launch_gemm_nt_fused(const uint16_t* A0, const uint8_t* Bq, const float* Bc, const float* tab16, int64_t lda0,
                                int K0, const uint16_t* A1, const uint16_t* B1, int64_t lda1, int64_t ldb1, int K1,
                                uint16_t* C, int64_t ldc, int M, int N, hipStream_t st);
// dequant.hip: the block constants (Double Quantization only; else w.c1 holds them already) and the value table the
// fused product reads.  4-bit types with cols % 64 == 0.
hipError_t launch_block_consts(const NF4Dev& w, float* consts, float* tab16, hipStream_t st);

// Measurement aid: register-only MFMA loop on Gaussian operands; mode 1 adds the main kernel's LDS fragment-read
// traffic, mode 2 also the LDS writes of its operand tiles; 256 * 4 * iters * 16 MFMAs of 16384 flops.  out: 256 * 256 floats.
hipError_t launch_mfma_probe(int mode, int iters, float* out, hipStream_t st);

// Measurement aid (adam.hip): a plain stream over `bytes` bytes (a multiple of 16): mode 0 reads src, 1 writes dst, 2 copies
// src to dst; sink: one device word (written only in the practically impossible case that the XOR of the data equals a
// constant, which keeps the loads alive).
hipError_t launch_hbm_probe(int mode, const void* src, void* dst, int64_t bytes, uint32_t* sink, int wgs_per_cu,
                            hipStream_t st);

// small.hip: skinny GEMMs of the LoRA branch with split-K fp32 partials, and layout helpers.
//   part[split][I x J] = A(i,k) B(k,j);  ta: A stored [k][i] instead of [i][k];  tb: B stored [k][j] instead of [j][k].
//   hl = 1 / 2: A / B is a [hi | lo] pair (the lo half hl_off elements behind the hi half) and enters as hi + lo;
//   supported: (ta, tb, hl) = (0,1,0), (0,0,0), (1,1,1), (1,1,2).
int small_gemm_splits(int I, int J, int K);
//   amask (LoRA dropout; only with (0,1,0) and (1,1,2), lda % 8 == 0): elements of A whose keep-bit -- bit e % 8 of byte
//   e / 8, e the element's offset from A -- is clear enter as zero.
hipError_t launch_small_gemm(const uint16_t* A, int64_t lda, bool ta, const uint16_t* B, int64_t ldb, bool tb, int hl,
                             int64_t hl_off, int I, int J, int K, float* part, int splits, hipStream_t st,
                             const uint8_t* amask = nullptr);
//   LoRA dropout: dX[m][k] -= sum_t Us[m][t] L1[k][t] (bf16 operands, fp32 sum, one more rounding to bf16) wherever the
//   keep-bit of element (m, k) is clear.  dX is M x h, Us M x ld_us (first r columns used), L1 h x r.
hipError_t launch_dropout_dx_fix(uint16_t* dX, int M, int h, const uint8_t* mask, const uint16_t* Us, int ld_us,
                                 const uint16_t* L1, int r, hipStream_t st);
//   Sums the splits, then writes out0 = bf16(scale0 * sum) (w0 columns, zeros beyond J) and/or
//   hl = [bf16(sum) | bf16(sum - bf16(sum))] (row stride 2 J) and/or adds scale0 * sum to the fp32 matrix acc (I x J).
hipError_t launch_small_finalize(const float* part, int splits, int I, int J, uint16_t* out0, int64_t ld0, int w0,
                                 float scale0, uint16_t* hl, float* acc, hipStream_t st);
//   dst[row][0 .. Cp) = src[row][0 .. C) then zeros; dst rows ld_dst elements apart (0: Cp)
hipError_t launch_copy_pad(const uint16_t* src, int R, int C, uint16_t* dst, int Cp, hipStream_t st, int64_t ld_dst = 0);

// fewtok.hip: few-token (M <= 16) streaming path, one launch per call: fp32 split partials of the frozen product,
// partials of the adapter's inner product, and the output written by the last workgroup to arrive at each slab
// of 256 outputs.  `ctr` points at the workspace header (kWorkspaceHeaderBytes, zero on entry, zero again on exit).
constexpr int kFewTokens = 16;
constexpr size_t kWorkspaceHeaderBytes = 16384;
constexpr int kFewMaxSlabs = 2047;
constexpr int kHeaderStatusWord = 2047;     // sticky status word of the counter header (work-list kernels)
int fewtok_fwd_splits(int h, int o);
int fewtok_bwd_splits(int h, int o);
int fewtok_fwd_slabs(int o);
int fewtok_bwd_slabs(int h);
int fewtok_fwd_lparts(int h, int r);          // number of [M][r] partial slots of T = X L1
int fewtok_bwd_lparts(int o, int r);          // ... of U = dY L2^T
//   Y = bf16(X dequant(W) + scale (X L1) L2); part: [splits][M][o] floats, lpart: [lparts][M][r] floats;
//   T_hl (M x 2r, may be NULL) receives X L1 as [hi | lo].
hipError_t launch_fewtok_fwd(const uint16_t* X, int M, const NF4Dev& w, float* part, int splits, const uint16_t* L1,
                             const uint16_t* L2, int r, float scale, float* lpart, unsigned* ctr, uint16_t* Y,
                             uint16_t* T_hl, hipStream_t st);
//   dX = bf16(dY dequant(W)^T + scale (dY L2^T) L1^T); part: [splits][M][h], lpart: [lparts][M][r];
//   U_hl (M x 2r, may be NULL) receives dY L2^T as [hi | lo].
hipError_t launch_fewtok_bwd(const uint16_t* dY, int M, const NF4Dev& w, float* part, int splits, const uint16_t* L1,
                             const uint16_t* L2, int r, float scale, float* lpart, unsigned* ctr, uint16_t* dX,
                             uint16_t* U_hl, hipStream_t st);
// Forward of up to kFewMaxLayers layers that read the same X (M x h) in one launch; every layer brings its own
// partial buffers; `ctr` as above (the layers' slabs together must not exceed kFewMaxSlabs).
constexpr int kFewMaxLayers = 4;
struct FewLayer {
  NF4Dev w; const uint16_t* L1; const uint16_t* L2; int r; float scale;
  float* part;                               // [splits][M][o]
  float* lpart;                              // [fewtok_fwd_lparts][M][r]
  uint16_t* Y;                               // M x o
};
int fewtok_multi_splits(int n, int h, const int* o, int r_max);
hipError_t launch_fewtok_fwd_multi(const uint16_t* X, int M, int n, const FewLayer* layers, int splits, unsigned* ctr,
                                   hipStream_t st);
hipError_t launch_workspace_init(void* workspace, hipStream_t st);

// fewlist.hip: the same two products for a LIST of independent layers (each with its own token rows) in one
// persistent launch.  The work of all layers is one line of units (forward: 16 weight rows x 256 columns; backward:
// 256 rows x 128 columns) and workgroup rho of `grid` takes units [start[rho], start[rho + 1]); the first n_adapter
// workgroups also compute one partial of an adapter's inner product each.  The host chooses the boundaries so that
// the workgroups' estimated times are equal (a range that crosses slab boundaries pays for the ends of its segments);
// the table travels in the kernel arguments, and host and device read it through the same two functions.
constexpr int kListMax = 8;
constexpr int kListGridMax = 256;
constexpr int kListLoraChunk = 1024;         // contraction elements per adapter item (more when a layer would need over 23 items)
struct ListPart {
  int grid, n_adapter;
  int start[kListGridMax + 1];               // ascending, start[0] = 0, start[grid] = total units; equal neighbours: an empty range
};
__host__ __device__ inline int list_start(const ListPart& p, int rho) { return p.start[rho]; }
// the workgroup whose range holds unit u (0 <= u < total units): the last rho with start[rho] <= u
__host__ __device__ inline int list_rho_of(const ListPart& p, int u) {
  int lo = 0, hi = p.grid;                   // invariant: start[lo] <= u < start[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (p.start[mid] <= u) lo = mid; else hi = mid;
  }
  return lo;
}
struct ListPlan {
  bool ok;                                   // false: not a few-token list (too many tokens, layers or slabs)
  ListPart part;
  int total_units, total_slabs;
  int n_slabs[kListMax], ups[kListMax], unit0[kListMax], a0[kListMax], ctr0[kListMax];
  int n_lparts[kListMax], lora_chunk[kListMax], max_contrib[kListMax];
  size_t part_floats[kListMax], lpart_floats[kListMax];      // sizes of the two partial buffers of every layer
};
ListPlan fewlist_plan(bool bwd, int M, int n, const int* h, const int* o, const int* r);
struct ListLayerDesc {
  NF4Dev w;
  const uint16_t* X;                         // forward: X (M x h); backward: dY (M x o)
  const uint16_t* L1; const uint16_t* L2; int r; float scale;
  float* part; float* lpart;                 // part_floats / lpart_floats of the plan
  uint16_t* out;                             // forward: Y (M x o); backward: dX (M x h)
  uint16_t* hl;                              // M x 2r [hi | lo] pair of X L1 (forward) or dY L2^T (backward), or NULL
};
//   hdr: the workspace's counter header; nonce: 1 .. 255, different for consecutive calls on one header;
//   spin_limit: polls of a slab's last contributor for the adapter's partials (0: never wait)
hipError_t launch_fewlist(bool bwd, int M, int n, const ListLayerDesc* layers, const ListPlan& plan, unsigned* hdr,
                          unsigned nonce, int spin_limit, hipStream_t st);

// kbit.hip: between the 4-bit container (elems / 2 bytes) and the k-bit stream (elems * k / 8 bytes), k = 2 or 3,
// elems a multiple of 32; codes above 2^k - 1 lose their upper bits when packed.
hipError_t launch_kbit_pack(const uint8_t* packed4, int64_t elems, int k, uint8_t* stream, hipStream_t st);
hipError_t launch_kbit_unpack(const uint8_t* stream, int64_t elems, int k, uint8_t* packed4, hipStream_t st);

// adam.hip: optimizer step of the LoRA parameters.  Scalars derived from the hyperparameters are computed by the
// caller in double precision and rounded once to fp32.
struct AdamConsts {
  float b1, b2, omb1, omb2;                  // beta, 1 - beta
  float bc1, bc2;                            // 1 - beta^t
  float eps, lr, lrwd;                       // lrwd = lr * weight_decay (0: no decay)
  int zero_grad;                             // clear the gradient after it has been used
  double grad_scale, max_norm;               // gradient coefficient = grad_scale * min(1, max_norm / (|grad_scale| sqrt(*sqnorm)))
  const double* sqnorm;                      // device; NULL or max_norm <= 0: no clipping
};
hipError_t launch_grad_sqnorm(const float* g, int64_t n, double* accum, hipStream_t st);
hipError_t launch_adam(float* p, float* m, float* v, float* g, uint16_t* p_bf16, int64_t n, const AdamConsts& c,
                       hipStream_t st);

}  // namespace qlora
