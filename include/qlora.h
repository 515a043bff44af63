/*
 * qlora.h -- C ABI of the MI355X (gfx950) library for the QLoRA frozen linear
 * layer (arXiv 2305.14314): blockwise NF4 quantisation with Double
 * Quantization, doubleDequant, and the forward / backward products of one
 * linear layer with a LoRA adapter.
 *
 * Notation follows the paper (Eq. 3, Eq. 5): X is M x h (tokens x in-features),
 * W is h x o row-major (in x out), L1 is h x r, L2 is r x o, s is a scalar.
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers (HIP global memory) owned by the
 *     caller; the library allocates and frees nothing and keeps no state
 *     between calls.  Buffers must be 16-byte aligned, must not overlap between
 *     inputs and outputs, and must stay alive until the stream has executed the
 *     call.  `const qlora_nf4_view*` itself is a HOST pointer to a small struct
 *     of device pointers; it is read before the call returns.
 *   - 16-bit tensors are bf16 bit patterns (uint16_t), row-major, dense.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default
 *     stream).  Calls only enqueue work; they never synchronise.
 *   - Return value: QLORA_OK or a negative qlora_status.  Arguments are checked
 *     on the host before any HIP call is made; on an argument error nothing is
 *     launched and no output is touched.  No exception or abort crosses the ABI.
 *   - Outputs are overwritten, never accumulated into -- except the fp32
 *     gradient accumulators of qlora_linear_bwd_acc / qlora_linear_bwd_dropout,
 *     which exist to be added to.  Inputs must be finite.
 *   - Workspace / scratch contents are undefined on entry and on exit, with one
 *     exception: the first QLORA_WORKSPACE_HEADER_BYTES of a qlora_linear_*
 *     workspace hold arrival counters of the few-token kernels.  They must be
 *     zero before the first call that uses the buffer (qlora_workspace_init, or
 *     any zero fill), every call leaves them zero again, and the caller must not
 *     write them in between.  Two calls that share a workspace must be ordered
 *     on one stream.
 */
#ifndef QLORA_H
#define QLORA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t qlora_status;
enum {
  QLORA_OK = 0,
  QLORA_ERR_NULL = -1,        /* a required pointer is NULL                                  */
  QLORA_ERR_SHAPE = -2,       /* non-positive size, cols not a multiple of blocksize, ...    */
  QLORA_ERR_UNSUPPORTED = -3, /* blocksize != 64, dq_blocksize not 256 or 0, r not supported, ... */
  QLORA_ERR_WORKSPACE = -4,   /* workspace / scratch smaller than the *_sizes call reports   */
  QLORA_ERR_ALIGN = -5,       /* a pointer is not 16-byte aligned                            */
  QLORA_ERR_HIP = -6,         /* a kernel launch failed; see qlora_last_hip_error()          */
  QLORA_ERR_STATE = -7        /* qlora_workspace_check: a kernel found the counter header dirty */
};

/* Human-readable name of a status code (static storage, never NULL). */
const char* qlora_status_string(qlora_status st);

/* hipError_t (as int) of the most recent failed launch on the calling thread, 0 if none. */
int qlora_last_hip_error(void);

/* A quantised weight: views onto caller-owned device buffers.
 *
 * Storage layout (Section 3; the paper fixes the types, the byte layout is this
 * library's):  the h x o matrix is flattened row-major and cut into contiguous
 * blocks of `blocksize` = 64 elements (Eq. 1 and the paragraph after Eq. 2).
 *   packed  : rows*cols/2 bytes; byte i holds element 2i in bits 3:0 and element
 *             2i+1 in bits 7:4, each a 4-bit index into the NF4 table (Appendix E).
 *   c2_code : n = rows*cols/blocksize bytes, the 8-bit-float codes of the
 *             mean-subtracted first-level constants (OCP E4M3 bit patterns),
 *             quantised in runs of `dq_blocksize` = 256 consecutive blocks of the
 *             flattened matrix (Double Quantization).  The codes are STORED
 *             column-group-major: the bpr = cols/blocksize blocks of a row are taken
 *             in groups of 4 (256 columns), and group G holds, row after row, the
 *             codes of its w blocks (w = 4, or bpr - 4G for the last group):
 *               position(row, blk) = 4*rows*(blk/4) + row*w + blk%4.
 *             Both products of the linear layer then find the constants of the
 *             weights they stream in contiguous runs, whichever dimension they
 *             contract over.  Which constants share a c1 is not affected.
 *   c1      : ceil(n / dq_blocksize) fp32 second-level constants; block
 *             b = row*bpr + blk uses c1[b / dq_blocksize].
 *   c2_mean : one fp32, the mean that was subtracted from c2 (per tensor).
 * cols must be a multiple of blocksize, so a block never straddles two rows.
 *
 * Without Double Quantization (dq_blocksize = 0; Section 3 prices the fp32 constants at 32/64 = 0.5 bit per
 * parameter, 4.5 bit in all): `c1` holds the n fp32 first-level constants c2 themselves, in flattened block order,
 * and c2_code / c2_mean are not read (may be NULL).  Such a weight is accepted by quantise, dequantise and the
 * linear-layer calls, which then take the large-GEMM path at any M -- the few-token streaming kernels read
 * double-quantised constants; the sizes qlora_linear_fwd_sizes / _bwd_sizes report cover that plan -- and refused with
 * QLORA_ERR_UNSUPPORTED by qlora_linear_fwd_multi at M <= 16.
 *
 * 8-bit integers (dtype = QLORA_INT8; Eq. 1 and Eq. 2 as printed): `packed` holds one signed byte per weight,
 * rows*cols bytes in flattened order, the constants are stored as above (with or without Double Quantization).
 * Accepted and refused exactly like a weight without Double Quantization: large-GEMM path at any M.
 */
typedef struct {
  const uint8_t* packed;
  const uint8_t* c2_code;
  const float* c1;
  const float* c2_mean;
  int64_t rows;          /* h, in-features  */
  int64_t cols;          /* o, out-features */
  int32_t blocksize;     /* 64  */
  int32_t dq_blocksize;  /* 256 */
  int32_t dtype;         /* QLORA_NF4 (0) or one of the other data types below */
  int32_t reserved;      /* 0 */
} qlora_nf4_view;

/* The 4-bit data types of the paper's comparison (Section 4: Int4, Float4 E2M1, Float4 E3M0 beside NFloat4).  All go
 * through the same blockwise scheme, storage layout and kernels; only the 16-value table differs, so a view of any
 * of them can be passed wherever a qlora_nf4_view is taken.  The paper prints a table for NF4 only (Appendix E).
 * The float types are the values of their bit fields (sign, exponent, mantissa; exponent field 0 is subnormal, no
 * infinities or NaNs) divided by the largest magnitude -- E2M1: +-{0, 1/12, 1/6, 1/4, 1/3, 1/2, 2/3, 1}, E3M0:
 * +-{0, 1/64, 1/32, ..., 1/2, 1}, each with two zeros -- and Int4 is Eq. 1 with the range [-7, 7]: j/7, 15 levels
 * (code 15 repeats the top value and is never produced).  Quantisation picks the nearest value, the lower code on an
 * exact tie, as for NF4. */
enum { QLORA_NF4 = 0, QLORA_FP4_E2M1 = 1, QLORA_FP4_E3M0 = 2, QLORA_INT4 = 3, QLORA_INT8 = 4, QLORA_NF3 = 5, QLORA_NF2 = 6 };

/* k-bit NormalFloat for k = 3 and 2 (Section 3 gives the construction for general k and prints the k = 4 table only):
 * 2^(k-1) evenly spaced probabilities from 1/2 to p_max on the negative side (the zero among them dropped), 2^(k-1) + 1
 * on the positive side, the normal quantiles divided by the top one, rounded to fp32.  p_max is not in the paper: the
 * tail mass 1 - p_max = (1 / 2^(k+1) + 1 / (2^(k+1) - 2)) / 2 is the one that reproduces the printed k = 4 table.
 * QLORA_NF3 and QLORA_NF2 are table types like the 4-bit ones: 16-entry tables whose entries from 2^k on repeat +1, the
 * codes sit in the same 4-bit containers (codes >= 2^k are never produced), so they show the error of fewer levels,
 * not a smaller footprint. */

/* A real k-bit footprint for QLORA_NF3 and QLORA_NF2 (k = 3, 2): at rest the codes of such a weight are one dense bit
 * stream over the flattened weight -- code i in bits [k*i, k*i + k), bit b of the stream = bit b % 8 of byte b / 8 --
 * of rows*cols*k/8 bytes (3.127 and 2.127 bits per parameter with the constants, which do not change).  The paper gives
 * the k-bit construction (Section 3) and no memory format; this one is the library's.  qlora_kbit_pack writes the stream
 * from the 4-bit container qlora_quantize_4bit fills (codes above 2^k - 1, which those data types never produce, would
 * lose their upper bits); qlora_kbit_unpack restores the container, which every other call reads -- a transient buffer
 * of rows*cols/2 bytes, like the dequantised weight of the GEMM path.  Device pointers, 16-byte aligned; shapes as for
 * quantisation; k other than 2 or 3: QLORA_ERR_UNSUPPORTED. */
qlora_status qlora_kbit_sizes(int64_t rows, int64_t cols, int32_t k, size_t* stream_bytes);
qlora_status qlora_kbit_pack(const uint8_t* packed4, int64_t rows, int64_t cols, int32_t k, uint8_t* stream,
                             void* hip_stream);
qlora_status qlora_kbit_unpack(const uint8_t* stream, int64_t rows, int64_t cols, int32_t k, uint8_t* packed4,
                               void* hip_stream);

/* The 16 values of a table data type (the 4-bit ones, QLORA_NF3, QLORA_NF2), ascending, as fp32 (host array).
 * QLORA_ERR_UNSUPPORTED for an unknown type and for QLORA_INT8, which has no table. */
qlora_status qlora_codebook_4bit(int32_t dtype, float* values16);

/* Byte sizes of the buffers of a quantised rows x cols tensor and of the scratch
 * qlora_nf4_quantize needs.  Any out-pointer may be NULL.
 * 4 + 8/64 + 32/(64*256) = 4.127 bits per parameter (Section 3); with dq_blocksize = 0
 * (no Double Quantization) code_bytes is 0 and c1_bytes = 4 * rows*cols/blocksize: 4.5 bits. */
qlora_status qlora_nf4_sizes(int64_t rows, int64_t cols, int32_t blocksize, int32_t dq_blocksize,
                             size_t* packed_bytes, size_t* code_bytes, size_t* c1_bytes,
                             size_t* scratch_bytes);

/* The same for any data type of the enum: QLORA_INT8 stores rows*cols bytes in `packed`, everything else is as
 * for NF4 (the constants do not depend on the data type). */
qlora_status qlora_quant_sizes(int64_t rows, int64_t cols, int32_t blocksize, int32_t dq_blocksize, int32_t dtype,
                               size_t* packed_bytes, size_t* code_bytes, size_t* c1_bytes,
                               size_t* scratch_bytes);

/* Blockwise NF4 quantisation with Double Quantization (Eq. 1; Section 3,
 * "4-bit NormalFloat Quantization" step (3) and "Double Quantization").
 *   W (in, fp32, rows x cols) -> packed, c2_code, c1, c2_mean as laid out above.
 * Per block: c2 = absmax; x = w * fl32(1/c2) (0 when c2 < FLT_MIN); index = the
 * nearest NF4 value (the lower index on an exact tie).  Then, per tensor:
 * mean = correctly rounded fp32 mean of all c2; per run of 256 constants
 * c1 = absmax(c2 - mean) and code = E4M3(round-to-nearest-even, saturating)
 * of (c2 - mean) * fl32(448 / c1).
 * W must be finite: an Inf or NaN is not detected and gives unspecified codes and
 * constants for the tensor (all accesses stay in bounds).
 * dq_blocksize = 0 stops after the first step: c1 receives the n constants c2, and
 * c2_code / c2_mean (may be NULL) are not written.
 * scratch: device buffer of at least the size qlora_nf4_sizes reports. */
qlora_status qlora_nf4_quantize(const float* W, int64_t rows, int64_t cols,
                                int32_t blocksize, int32_t dq_blocksize,
                                uint8_t* packed, uint8_t* c2_code, float* c1, float* c2_mean,
                                void* scratch, size_t scratch_bytes, void* hip_stream);

/* For callers that cannot allocate device memory and have no scratch buffer to pass (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): qlora_nf4_quantize with its scratch in a device array that
 * the library itself holds (16 MiB + 2 KiB on every device it runs on, until the process ends).  Same arguments,
 * same results bit for bit, no allocation on the way; tensors of at most QLORA_STATIC_QUANT_MAX_WEIGHTS weights,
 * QLORA_ERR_WORKSPACE beyond that.  All calls on one device share the array: two calls that overlap there (on
 * different streams or threads) race; calls on one stream are ordered and fine. */
#define QLORA_STATIC_QUANT_MAX_WEIGHTS ((int64_t)1 << 28)
qlora_status qlora_nf4_quantize_static(const float* W, int64_t rows, int64_t cols,
                                       int32_t blocksize, int32_t dq_blocksize,
                                       uint8_t* packed, uint8_t* c2_code, float* c1, float* c2_mean,
                                       void* hip_stream);

/* The same with one of the other table data types (Section 4's 4-bit ones, QLORA_NF3, QLORA_NF2); dtype = QLORA_NF4
 * is qlora_nf4_quantize.  The
 * buffers, their sizes and the Double Quantization of the constants do not depend on the data type. */
qlora_status qlora_quantize_4bit(const float* W, int64_t rows, int64_t cols,
                                 int32_t blocksize, int32_t dq_blocksize, int32_t dtype,
                                 uint8_t* packed, uint8_t* c2_code, float* c1, float* c2_mean,
                                 void* scratch, size_t scratch_bytes, void* hip_stream);

/* Blockwise 8-bit integers, Eq. 1 as printed: per block c2 = absmax, c = fl32(127 / c2) (0 when c2 < FLT_MIN or the
 * quotient overflows), q8 = round-to-nearest-even(fl32(c * w)) clamped to [-127, 127]; the constants c2 then go through
 * Double Quantization as in qlora_nf4_quantize (dq_blocksize = 0: kept as fp32 in c1).  q8: rows*cols signed bytes.
 * Dequantisation (qlora_nf4_dequant and the linear-layer calls on a view with dtype = QLORA_INT8) is Eq. 2:
 * w = bf16_rne(fl32(q8 * fl32(c2hat / 127))).  scratch: the size qlora_quant_sizes reports.  Not a 4-bit type:
 * qlora_quantize_4bit refuses QLORA_INT8. */
qlora_status qlora_quantize_int8(const float* W, int64_t rows, int64_t cols,
                                 int32_t blocksize, int32_t dq_blocksize,
                                 int8_t* q8, uint8_t* c2_code, float* c1, float* c2_mean,
                                 void* scratch, size_t scratch_bytes, void* hip_stream);

/* doubleDequant (Eq. 6, Eq. 2): W_bf16[rows x cols] =
 *   bf16_rne( NF4[index] * fl32( fl32(E4M3(code)/448 * c1) + mean ) ). */
qlora_status qlora_nf4_dequant(const qlora_nf4_view* Wq, uint16_t* W_bf16, void* hip_stream);

/* Size of the counter header at the start of every qlora_linear_* workspace. */
#define QLORA_WORKSPACE_HEADER_BYTES 16384

/* Zeroes the counter header of a freshly allocated workspace (one small fill
 * kernel on the stream; safe to capture in a HIP graph).  Needed once per
 * buffer, before its first use by qlora_linear_fwd / qlora_linear_bwd; a buffer
 * that was allocated zero-filled needs no call.  Call it again only after a
 * call on that buffer was abandoned half-way (device reset, failed launch). */
qlora_status qlora_workspace_init(void* workspace, size_t workspace_bytes, void* hip_stream);

/* Workspace (bytes) qlora_linear_fwd / qlora_linear_bwd need for this shape
 * (header included), whatever the weight's data type: at M <= 16 a 4-bit
 * double-quantised weight takes the streaming kernels and any other weight
 * (QLORA_INT8, dq_blocksize = 0) the dequantise + GEMM plan; the larger of
 * the two sizes is reported. */
qlora_status qlora_linear_fwd_sizes(int64_t M, int64_t h, int64_t o, int32_t r, size_t* workspace_bytes);
qlora_status qlora_linear_bwd_sizes(int64_t M, int64_t h, int64_t o, int32_t r, size_t* workspace_bytes);

/* Forward of one QLoRA linear layer (Eq. 5 with the scalar s of Eq. 3):
 *   Y = X * doubleDequant(Wq) + s * (X * L1) * L2          (bf16 in, fp32 accumulate, bf16 out)
 * X: M x h, L1: h x r, L2: r x o, Y: M x o, with h = Wq->rows and o = Wq->cols.
 * r may be 0 (then L1, L2 may be NULL and the adapter term is skipped); otherwise
 * r must be a multiple of 16 and at most 256.  T_save (M x 2r bf16, may be NULL)
 * receives T = X * L1 for the backward pass as a pair of bf16 matrices side by
 * side: columns [0, r) hold bf16(T), columns [r, 2r) hold bf16(T - bf16(T)).  Any M >= 1 is accepted: a few
 * tokens (M <= 16) take a bandwidth-bound streaming path, larger M the MFMA
 * GEMM path. */
qlora_status qlora_linear_fwd(const uint16_t* X, const qlora_nf4_view* Wq,
                              const uint16_t* L1, const uint16_t* L2, float s,
                              int64_t M, int32_t r,
                              uint16_t* Y, uint16_t* T_save,
                              void* workspace, size_t workspace_bytes, void* hip_stream);

/* Backward of the same layer (Section 3, after Eq. 6): gradients flow through
 * the dequantised bf16 weight to the input and to the adapter only; dE/dW is
 * never formed.
 *   dX  = dY * doubleDequant(Wq)^T + s * (dY * L2^T) * L1^T     (M x h)
 *   dL1 = s * X^T * (dY * L2^T)                                  (h x r)
 *   dL2 = s * (X * L1)^T * dY                                    (r x o)
 * Each of dX, dL1, dL2 may be NULL and is then not computed.  X is needed only
 * for dL1 / dL2 (may be NULL when both are NULL).  T_saved is the T_save of the
 * forward call or NULL, in which case X * L1 is recomputed (gradient
 * checkpointing).  With r = 0 only dX is produced. */
qlora_status qlora_linear_bwd(const uint16_t* dY, const uint16_t* X, const qlora_nf4_view* Wq,
                              const uint16_t* L1, const uint16_t* L2, float s,
                              int64_t M, int32_t r, const uint16_t* T_saved,
                              uint16_t* dX, uint16_t* dL1, uint16_t* dL2,
                              void* workspace, size_t workspace_bytes, void* hip_stream);

/* The same backward pass with gradient accumulation: the adapter gradients are ADDED, in fp32, to the caller's
 * accumulators instead of being written as bf16 (Section 3 after Eq. 6 gives the gradients; an optimizer step over
 * several micro-batches, as the batch sizes of the hyperparameter appendix imply, sums them before the update):
 *   dL1_acc (h x r, fp32) += s * X^T * (dY * L2^T),     dL2_acc (r x o, fp32) += s * (X * L1)^T * dY.
 * The caller zeroes the accumulators before the first micro-batch.  Either may be NULL; dX, T_saved, the workspace
 * and every other rule are those of qlora_linear_bwd.  The sums are not rounded to bf16 on the way. */
qlora_status qlora_linear_bwd_acc(const uint16_t* dY, const uint16_t* X, const qlora_nf4_view* Wq,
                                  const uint16_t* L1, const uint16_t* L2, float s,
                                  int64_t M, int32_t r, const uint16_t* T_saved,
                                  uint16_t* dX, float* dL1_acc, float* dL2_acc,
                                  void* workspace, size_t workspace_bytes, void* hip_stream);

/* LoRA dropout (hyperparameter appendix: rate 0.1 for models up to 13B, 0.05 for 33B and 65B).  The paper gives the
 * rate only; the placement is the one of the LoRA method it builds on -- inverted dropout on the INPUT of the adapter
 * branch, the frozen product never sees it:
 *   Y   = X * doubleDequant(Wq) + s * ((D o X) * L1) * L2,      D[m][k] = keep(m, k) / (1 - p)
 *   dX  = dY * doubleDequant(Wq)^T + s * D o ((dY * L2^T) * L1^T)
 *   dL1 = s * (D o X)^T * (dY * L2^T),      dL2 = s * ((D o X) * L1)^T * dY.
 * The random draw is the caller's: keep_mask (device, M*h/8 bytes) holds one bit per element of X, bit e % 8 of byte
 * e / 8 for e = m*h + k, 1 = kept; the same mask must be passed to the forward and the backward call of a step.
 * 0 <= p < 1 (else QLORA_ERR_SHAPE); keep_mask may be NULL only when r = 0, where the calls are the plain ones.
 * T_save / T_saved hold (B o X) * L1 for the 0/1 mask B, as a [hi | lo] pair (the 1/(1-p) is applied with s).
 * These calls always take the large-GEMM path (no few-token streaming kernel); workspaces are sized by
 * qlora_linear_dropout_sizes (either out-pointer may be NULL).  The backward call takes both kinds of adapter
 * gradient outputs of qlora_linear_bwd and qlora_linear_bwd_acc; any of them may be NULL.  Everything else --
 * layouts, alignment, ownership, errors, tolerance -- as for qlora_linear_fwd / qlora_linear_bwd. */
qlora_status qlora_linear_dropout_sizes(int64_t M, int64_t h, int64_t o, int32_t r, size_t* fwd_bytes,
                                        size_t* bwd_bytes);
qlora_status qlora_linear_fwd_dropout(const uint16_t* X, const qlora_nf4_view* Wq,
                                      const uint16_t* L1, const uint16_t* L2, float s,
                                      int64_t M, int32_t r, const uint8_t* keep_mask, float p,
                                      uint16_t* Y, uint16_t* T_save,
                                      void* workspace, size_t workspace_bytes, void* hip_stream);
qlora_status qlora_linear_bwd_dropout(const uint16_t* dY, const uint16_t* X, const qlora_nf4_view* Wq,
                                      const uint16_t* L1, const uint16_t* L2, float s,
                                      int64_t M, int32_t r, const uint8_t* keep_mask, float p,
                                      const uint16_t* T_saved,
                                      uint16_t* dX, uint16_t* dL1, uint16_t* dL2,
                                      float* dL1_acc, float* dL2_acc,
                                      void* workspace, size_t workspace_bytes, void* hip_stream);

/* Forward of several QLoRA linear layers that read the SAME input (Eq. 5 applied per layer: the q / k / v or the
 * gate / up projections of a decoder block, where the adapter sits on every linear layer -- Section 5 and the
 * hyperparameter appendix):
 *   Y[l] = X * doubleDequant(Wq[l]) + s[l] * (X * L1[l]) * L2[l],   l = 0 .. n-1,  1 <= n <= QLORA_MULTI_MAX.
 * X: M x h with h = Wq[l].rows for every l (else QLORA_ERR_SHAPE); Wq is an array of n views; L1, L2, Y are host
 * arrays of n device pointers, s and r host arrays of n values (r[l] = 0 skips layer l's adapter, and then L1[l],
 * L2[l] are not read; L1 and L2 themselves may be NULL when every r[l] is 0).  At M <= 16 all layers run in ONE
 * launch of the streaming kernel, so the fixed cost of a call is paid once; at larger M the layers run one after
 * the other exactly as n calls of qlora_linear_fwd would.  Results meet the same tolerance as qlora_linear_fwd but
 * need not be bit-identical to it (the contraction may be split differently).  Same rules for the workspace
 * (counter header first, qlora_workspace_init once per buffer), alignment, ownership and errors. */
#define QLORA_MULTI_MAX 4
qlora_status qlora_linear_fwd_multi_sizes(int64_t M, int32_t n, int64_t h, const int64_t* o, const int32_t* r,
                                          size_t* workspace_bytes);
qlora_status qlora_linear_fwd_multi(const uint16_t* X, int32_t n, const qlora_nf4_view* Wq,
                                    const uint16_t* const* L1, const uint16_t* const* L2, const float* s,
                                    int64_t M, const int32_t* r, uint16_t* const* Y,
                                    void* workspace, size_t workspace_bytes, void* hip_stream);

/* The same layers at training token counts with ONE matrix product for all of them (Eq. 5 per layer): the
 * dequantised weights are stacked along the output dimension, the adapters share the second contraction segment
 * block-diagonally (layer l's s[l] * X * L1[l] meets only layer l's L2[l]), and the outputs come out side by side:
 *   Y is M x (o[0] + ... + o[n-1]), row-major; layer l's output is the column range starting at o[0] + ... + o[l-1].
 * T_save: NULL, or a host array of n device pointers (entries may be NULL): T_save[l] receives X * L1[l] as the
 * M x 2 r[l] [hi | lo] pair qlora_linear_bwd takes.  Any M >= 1 (few tokens take the same path).  Workspace: the size
 * qlora_linear_fwd_stacked_sizes reports, (sum o) * (h + sum of the ranks rounded up to 64) bf16 values and a few
 * small buffers; same rules otherwise.  Each layer's output meets the tolerance of qlora_linear_fwd. */
qlora_status qlora_linear_fwd_stacked_sizes(int64_t M, int32_t n, int64_t h, const int64_t* o, const int32_t* r,
                                            size_t* workspace_bytes);
qlora_status qlora_linear_fwd_stacked(const uint16_t* X, int32_t n, const qlora_nf4_view* Wq,
                                      const uint16_t* const* L1, const uint16_t* const* L2, const float* s,
                                      int64_t M, const int32_t* r, uint16_t* Y, uint16_t* const* T_save,
                                      void* workspace, size_t workspace_bytes, void* hip_stream);

/* The backward of the same group of layers.  Layers that read one input have ONE input gradient, the sum of theirs
 * (Section 3 after Eq. 6, per layer; the sum is the chain rule at the shared input):
 *   dX = sum over l of  dY_l * doubleDequant(Wq[l])^T + s[l] * (dY_l * L2[l]^T) * L1[l]^T,
 * computed as one matrix product whose contraction runs over all layers' outputs and then over all layers' ranks, so
 * no per-layer gradients are written and added afterwards.  dY is M x (o[0] + ... + o[n-1]) in the layout
 * qlora_linear_fwd_stacked writes; dX is M x h.  dL1 / dL2: NULL, or host arrays of n device pointers (entries may be
 * NULL): dL1[l] (h x r[l]) and dL2[l] (r[l] x o[l]) receive layer l's adapter gradients as bf16, exactly as
 * qlora_linear_bwd computes them; X (M x h) is needed only for those.  T_saved: NULL, or n pointers to the pairs
 * qlora_linear_fwd_stacked saved (a NULL entry: X * L1[l] is recomputed).  Any M >= 1.  Workspace:
 * qlora_linear_bwd_stacked_sizes, h * (sum o) bf16 values and a few small buffers; same rules otherwise. */
qlora_status qlora_linear_bwd_stacked_sizes(int64_t M, int32_t n, int64_t h, const int64_t* o, const int32_t* r,
                                            size_t* workspace_bytes);
qlora_status qlora_linear_bwd_stacked(const uint16_t* dY, const uint16_t* X, int32_t n, const qlora_nf4_view* Wq,
                                      const uint16_t* const* L1, const uint16_t* const* L2, const float* s,
                                      int64_t M, const int32_t* r, const uint16_t* const* T_saved, uint16_t* dX,
                                      uint16_t* const* dL1, uint16_t* const* dL2,
                                      void* workspace, size_t workspace_bytes, void* hip_stream);

/* Forward of a LIST of independent QLoRA linear layers at a few tokens in ONE launch (Eq. 5 applied per layer; the
 * adapter sits on every linear layer of a decoder block -- Section 5 and the hyperparameter appendix):
 *   Y[l] = X[l] * doubleDequant(Wq[l]) + s[l] * (X[l] * L1[l]) * L2[l],   l = 0 .. n-1,  1 <= n <= QLORA_LIST_MAX.
 * Unlike qlora_linear_fwd_multi every layer has its own input X[l] (M x Wq[l].rows) and any shape; the layers must not
 * depend on each other (a layer's input is never another layer's output of the same call).  X, L1, L2, Y are host
 * arrays of n device pointers, Wq an array of n views, s and r host arrays of n values (r[l] = 0: no adapter, L1[l]
 * and L2[l] are not read).  At M <= 16 one persistent kernel streams all layers' packed weights back to back -- the
 * fixed cost of a launch is paid once and every compute unit gets the same number of bytes -- and all views must be
 * double-quantised 4-bit weights of one data type (else QLORA_ERR_UNSUPPORTED); at larger M the layers run one
 * after the other exactly as n calls of qlora_linear_fwd.  Results meet the tolerance of qlora_linear_fwd but need
 * not be bit-identical to it.  Workspace rules as for qlora_linear_fwd (counter header first).
 * qlora_linear_bwd_list is the input gradient of the same list (no adapter gradients):
 *   dX[l] = dY[l] * doubleDequant(Wq[l])^T + s[l] * (dY[l] * L2[l]^T) * L1[l]^T,   dY[l]: M x Wq[l].cols. */
#define QLORA_LIST_MAX 8
qlora_status qlora_linear_fwd_list_sizes(int64_t M, int32_t n, const int64_t* h, const int64_t* o, const int32_t* r,
                                         size_t* workspace_bytes);
qlora_status qlora_linear_bwd_list_sizes(int64_t M, int32_t n, const int64_t* h, const int64_t* o, const int32_t* r,
                                         size_t* workspace_bytes);
qlora_status qlora_linear_fwd_list(int32_t n, const uint16_t* const* X, const qlora_nf4_view* Wq,
                                   const uint16_t* const* L1, const uint16_t* const* L2, const float* s,
                                   int64_t M, const int32_t* r, uint16_t* const* Y,
                                   void* workspace, size_t workspace_bytes, void* hip_stream);
qlora_status qlora_linear_bwd_list(int32_t n, const uint16_t* const* dY, const qlora_nf4_view* Wq,
                                   const uint16_t* const* L1, const uint16_t* const* L2, const float* s,
                                   int64_t M, const int32_t* r, uint16_t* const* dX,
                                   void* workspace, size_t workspace_bytes, void* hip_stream);

/* Has a few-token kernel found the counter header of this workspace in a state no call leaves behind (not zeroed
 * before first use, written by the caller, left half-way by an abandoned call)?  The arrival words of the list
 * kernels carry a per-call tag, so stale contents are noticed by the kernel that meets them: it raises a sticky
 * status word in the header, every wave still exits, and the outputs of that call are unspecified.  This call
 * SYNCHRONISES hip_stream (the one entry point that does), reads the word and returns QLORA_ERR_STATE if it is set,
 * QLORA_OK otherwise.  qlora_workspace_init clears it. */
qlora_status qlora_workspace_check(const void* workspace, size_t workspace_bytes, void* hip_stream);

/* Measurement aid for the benchmark (not part of the method): the rate the matrix cores sustain on this board, to
 * read the main GEMM's rate against.  One wave per SIMD on all 256 CUs runs `iters` x 16 independent 16x16x32 bf16
 * MFMAs on Gaussian operands held in registers -- with no memory traffic (lds_traffic = 0), with the LDS
 * fragment-read traffic of the main kernel's wave tile, one 16-byte read per lane and four MFMAs (1), or with that and
 * the LDS writes of the operand tiles that land per K-step, one 16-byte write per lane and eight MFMAs (2).
 * Flops of one call: 256 * 4 * iters * 16 * 16384.  out: at least 256 * 256 floats of device memory (written so that
 * the loop is not optimised away).  iters in 1 .. 2^20. */
qlora_status qlora_mfma_probe(int32_t lds_traffic, int32_t iters, float* out, size_t out_bytes, void* hip_stream);

/* Measurement aid for the benchmark (not part of the method): what a plain stream reaches on this board, to read the
 * bandwidth-bound kernels' rates against.  mode 0 reads `bytes` bytes at src (16-byte loads; sink: one device word that
 * keeps the loads alive and is practically never written), mode 1 writes them at dst, mode 2 copies src to dst.
 * bytes: a positive multiple of 16; src / dst 16-byte aligned device memory; wgs_per_cu in 1 .. 64 workgroups of 256
 * threads per compute unit, each lane with four 16-byte accesses in flight. */
qlora_status qlora_hbm_probe(int32_t mode, const void* src, void* dst, int64_t bytes, uint32_t* sink, int32_t wgs_per_cu,
                             void* hip_stream);

/* Which of two forms of the large-token backward product runs (arXiv 2305.14314, Eq. 5-6 and the backward through the
 * dequantised weight): mode 0 dequantises the weight into the workspace and multiplies; mode 1 decodes the weight's
 * tiles inside the product (codes and block constants go from HBM to the matrix cores' LDS tiles, the bf16 weight is
 * never in HBM).  The decoded tiles are the same bits either way; the adapter term is added first instead of last in
 * mode 1, so outputs may differ in the last bf16 bit.  Mode 1 applies to 4-bit types with cols % 64 == 0 and r <= 64
 * and falls back to mode 0 otherwise.  mode < 0 only queries.  Returns the previous mode.  Process-wide. */
int32_t qlora_bwd_fused_dequant(int32_t mode);

/* Testing aid: how many times a slab's last contributor polls for the adapter's partial sums before it hands the
 * slab's output stage to the adapter's workgroups (default 64; 0 = never wait, so that hand-over path can be
 * exercised).  Process-wide; affects the few-token list kernels only; results are the same bits either way. */
void qlora_fewtok_poll_limit(int32_t polls);

/* ---- optimizer step of the LoRA parameters ---------------------------------------------------------------------
 * The paper trains the adapters with Adam, beta2 = 0.999, a maximum gradient norm of 0.3 and a constant learning rate
 * of 2e-4 (7B, 13B) or 1e-4 (33B, 65B) (hyperparameter appendix), and keeps the optimizer state in memory that can be
 * paged (Section 3, "Paged Optimizers").  The paging is not built; the state lives in device buffers of the caller.
 * The paper does not print the update rule: this is the published algorithm (Kingma & Ba 2015, Algorithm 1) with bias
 * correction.  All buffers are device memory; the fp32 ones 16-byte aligned, param_bf16 8-byte aligned. */
typedef struct {
  double lr;            /* learning rate                                                             */
  double beta1;         /* 0.9 unless the caller says otherwise                                      */
  double beta2;         /* 0.999 (hyperparameter appendix)                                           */
  double eps;           /* 1e-8                                                                      */
  double weight_decay;  /* decoupled: p <- p - lr * weight_decay * p before the step; 0 = none       */
  double grad_scale;    /* the accumulators hold a sum over micro-batches: 1 / their number          */
  double max_grad_norm; /* 0.3 in the paper; <= 0 or sqnorm = NULL: no clipping                      */
  int64_t step;         /* 1 for the first step (bias correction 1 - beta^step)                      */
  int32_t zero_grad;    /* != 0: the gradient buffer is cleared after use                            */
  int32_t reserved;     /* 0 */
} qlora_adam_config;

/* *sqnorm_accum += sum of grad[i]^2 in double precision (order of the additions unspecified).  The caller clears the
 * device double once, calls this for every gradient buffer of the model (the fp32 accumulators that
 * qlora_linear_bwd_acc adds to), and passes the same pointer to every qlora_adam_step of the step. */
qlora_status qlora_grad_sqnorm(const float* grad, int64_t n, double* sqnorm_accum, void* hip_stream);

/* One Adam step on n parameters, per element in fp32, each operation rounded separately, in this order:
 *   g' = coef * g      coef = fl32(grad_scale * min(1, max_grad_norm / (|grad_scale| * sqrt(*sqnorm))))
 *   m  = beta1 * m + (1 - beta1) * g'
 *   v  = beta2 * v + (1 - beta2) * (g' * g')
 *   p  = p - (lr * weight_decay) * p                      (only when weight_decay != 0)
 *   p  = p - lr * ((m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps))
 * (the scalars 1 - beta, 1 - beta^step, lr * weight_decay are computed in double precision on the host and rounded
 * once).  param, m, v are read and written; grad is read (and cleared when zero_grad is set); param_bf16 (may be NULL)
 * receives the round-to-nearest-even bf16 copy of the new parameters, which is what qlora_linear_fwd / _bwd read as
 * L1 / L2.  All LoRA parameters of a model can sit in one flat buffer and take one call.  sqnorm: NULL, or the device
 * double that qlora_grad_sqnorm filled for ALL gradients of this step.  n = 0 is accepted and does nothing. */
qlora_status qlora_adam_step(float* param, float* m, float* v, float* grad, uint16_t* param_bf16, int64_t n,
                             const qlora_adam_config* cfg, const double* sqnorm, void* hip_stream);

/* Measurement aid for the benchmark (not part of the method): while enabled, every launch of the
 * main MFMA GEMM kernel made by qlora_linear_fwd / qlora_linear_bwd is bracketed by a pair of HIP
 * events recorded on the call's stream.  qlora_profile_gemm_read waits for those events, returns
 * the summed kernel time in milliseconds, the number of launches and the summed algorithmic FLOPs
 * (2*M*N*K per launch, adapter segment included), and clears the record.  The event pairs (at most
 * 4096 between two reads; launches beyond that run unbracketed) are created on first use and kept for
 * reuse: they are the only objects the library ever creates, and only while this aid is enabled.
 * Safe to call from several host threads. */
void qlora_profile_gemm(int enable);
qlora_status qlora_profile_gemm_read(double* total_ms, int64_t* launches, double* total_flops);

#ifdef __cplusplus
}
#endif
#endif
