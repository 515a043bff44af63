/*
 * CPU oracle for the QLoRA frozen-linear hot path (arXiv 2305.14314).
 *
 * TEST INFRASTRUCTURE ONLY.  This library is the slow, plain, obviously-correct
 * statement of what the path computes, written from the paper.  It shares no
 * source, table, constant generator or helper with the HIP library, is never
 * linked into it, and must only be used by tests, the smoke check and the
 * benchmark's cpu_baseline leg.
 *
 * All arithmetic is fp64 unless the paper (or the stated reading of it) fixes a
 * narrower type; every fp32 / bf16 / 8-bit-float rounding below is a single
 * IEEE round-to-nearest-even step emulated exactly through fp64.
 *
 * Shapes follow the paper's notation (Eq. 3): X is b x h (here M x h), W is
 * h x o row-major, L1 is h x r, L2 is r x o.  16-bit tensors are passed as raw
 * bf16 bit patterns (uint16_t).  All pointers are host pointers owned by the
 * caller.  Functions returning int return 0 on success and a negative value on
 * a bad argument (nothing is written in that case).
 *
 * Parity pins (tests marked "not gpu"):
 *   - NF4 table: the values printed in Appendix E; re-derived from N(0,1)
 *     quantiles (asymmetric construction of Section 3) to <= 2e-7.
 *   - index assignment: brute-force nearest value on small inputs.
 *   - 8-bit float encode/decode: an OCP E4M3 library conversion.
 *   - bf16 rounding: a library bf16 cast.
 *   - forward/backward: library fp64 matmul and central finite differences.
 *   - the 8-bit code VALUES are "parity unpinned" against the paper, which
 *     does not state the 8-bit float format; they are pinned only against the
 *     reading stated at oracle_nf4_quantize.
 */
#ifndef QLORA_ORACLE_H
#define QLORA_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Number of OpenMP threads the matmul routines will use. */
int oracle_num_threads(void);

/* Appendix E: the 16 NF4 values, index 0..15, as fp32. */
void oracle_nf4_table(float out[16]);

/* Section 3 (4-bit NormalFloat): asymmetric quantile construction.  Positive
 * half: Q(p) at 2^(k-1)+1 = 9 evenly spaced p in [1/2, p_max]; negative half:
 * -Q(p) at 2^(k-1) = 8 evenly spaced p in [1/2, p_max]; union with one of the
 * two zeros removed, divided by Q(p_max).  Q is the N(0,1) quantile function.
 * The paper does not state p_max; tests fit it (1 - (1/32 + 1/30)/2). */
void oracle_nf4_derive(double p_max, double out[16]);

/* N(0,1) quantile function Q_X of Eq. 4, by bisection on erfc (|err| < 1e-14). */
double oracle_normal_quantile(double p);

/* Nearest NF4 index of a normalised value (Section 3 step (3), "quantize as
 * usual"): the number of midpoints (q_j + q_{j+1})/2, taken as exact reals,
 * that lie strictly below xhat; an exact tie goes to the lower index. */
int oracle_nf4_index(float xhat);

/* fp32 -> bf16 bits, round to nearest even. */
uint16_t oracle_bf16_rne(float v);

/* 8-bit float of Double Quantization, read as OCP E4M3 (1-4-3, bias 7, no
 * infinities, max finite 448, subnormals).  encode: nearest representable
 * value, ties to the even code, saturating at +-448, zero always 0x00.
 * value: exact real value of a code (NaN for 0x7f / 0xff).
 * unit: fl32(value / 448), the decode table entry used by doubleDequant. */
uint8_t oracle_e4m3_encode(float z);
float oracle_e4m3_value(uint8_t code);
float oracle_e4m3_unit(uint8_t code);

/* Eq. 1 blockwise + Double Quantization (Section 3).  W: rows x cols fp32,
 * flattened row-major and cut into contiguous blocks of `blocksize`;
 * rows*cols must be a multiple of 2 and of blocksize.
 *   c2[b]   = max |w| over block b                          (n = rows*cols/blocksize)
 *   rc      = fl32(1 / c2[b])  (0 when c2[b] < FLT_MIN)
 *   xhat    = fl32(w * rc);  idx = oracle_nf4_index(xhat)
 *   packed[i] = idx[2i] | idx[2i+1] << 4
 *   mean    = fl32(exact sum of c2 / n), one mean per tensor
 *   c2'     = fl32(c2 - mean)
 *   c1[B]   = max |c2'| over the B-th run of dq_blocksize constants (last run may be short)
 *   rc1     = fl32(448 / c1[B])  (0 when c1[B] < FLT_MIN)
 *   code[b] = e4m3_encode(fl32(c2'[b] * rc1))
 * Outputs: packed (rows*cols/2), code (n), c1 (ceil(n/dq_blocksize)), mean (1);
 * c2_out (n fp32) may be NULL. */
int oracle_nf4_quantize(const float* W, int64_t rows, int64_t cols,
                        int32_t blocksize, int32_t dq_blocksize,
                        uint8_t* packed, uint8_t* code, float* c1, float* mean,
                        float* c2_out);

/* Eq. 6 doubleDequant, Eq. 2.
 *   c2hat[b] = fl32(fl32(unit(code[b]) * c1[b / dq_blocksize]) + mean)
 *   w_i      = bf16_rne(fl32(nf4[idx_i] * c2hat[i / blocksize]))
 * Outputs: W_bf16 (rows*cols), c2hat_out (n fp32, may be NULL). */
int oracle_nf4_dequant(const uint8_t* packed, const uint8_t* code, const float* c1,
                       float mean, int64_t rows, int64_t cols,
                       int32_t blocksize, int32_t dq_blocksize,
                       uint16_t* W_bf16, float* c2hat_out);

/* The other 4-bit data types of the paper's comparison (Section 4: Int4, Float4 E2M1, Float4 E3M0 beside
 * NFloat4) through the same blockwise scheme: only the 16-value table changes.  kind: 0 NF4 (Appendix E),
 * 1 Float4 E2M1, 2 Float4 E3M0, 3 Int4 (Eq. 1 with range [-7, 7]).  The paper prints no value tables for the
 * float types: they are enumerated from the bit fields (exponent field 0 = subnormal, no infinities / NaNs) and
 * normalised by the largest magnitude -- PARITY UNPINNED against the paper, pinned against that definition.
 * Returns 0, -1 (NULL) or -2 (unknown kind). */
int oracle_codebook4(int kind, float out[16]);
/* Nearest entry of a non-decreasing 16-value table, the lower index on an exact tie. */
int oracle_index4(const float* table, float xhat);
/* oracle_nf4_quantize / oracle_nf4_dequant with the table as an argument. */
int oracle_quantize4(const float* table, const float* W, int64_t rows, int64_t cols,
                     int32_t blocksize, int32_t dq_blocksize,
                     uint8_t* packed, uint8_t* code, float* c1, float* mean,
                     float* c2_out);
int oracle_dequant4(const float* table, const uint8_t* packed, const uint8_t* code, const float* c1,
                    float mean, int64_t rows, int64_t cols,
                    int32_t blocksize, int32_t dq_blocksize,
                    uint16_t* W_bf16, float* c2hat_out);

/* 8-bit integers, Eq. 1 and Eq. 2 as printed (the paper's example of blockwise quantisation and its Int8 baseline):
 *   q = clamp(round_to_nearest_even(fl32(c * x)), -127, 127),  c = fl32(127 / absmax(block))  (0 if that is not a
 *   finite positive number);  the constants absmax are double-quantised like those of the 4-bit types
 *   (dq_blocksize = 0: kept, code / c1 / mean may be NULL);  c2_out (n fp32) receives them in any case.
 *   w = bf16_rne(fl32(q * fl32(c2hat / 127))).
 * oracle_dq_constants reconstructs c2hat from the double-quantised constants. */
/* k-bit NormalFloat values for k = 2, 3, 4 from N(0,1) quantiles (Section 3; p_max for k != 4 is a reading, see the
 * source): 2^k values ascending, then +1 repeated up to 16 entries.  oracle_codebook4 kinds 5 (NF3) and 6 (NF2) are
 * these rounded to fp32. */
int oracle_nfk_derive(int k, double out[16]);

int oracle_quantize_int8(const float* W, int64_t rows, int64_t cols, int32_t blocksize, int32_t dq_blocksize,
                         int8_t* q8, uint8_t* code, float* c1, float* mean, float* c2_out);
int oracle_dequant_int8(const int8_t* q8, const float* c2hat, int64_t rows, int64_t cols, int32_t blocksize,
                        uint16_t* W_bf16);
int oracle_dq_constants(const uint8_t* code, const float* c1, float mean, int64_t n, int32_t dq_blocksize,
                        float* c2hat);

/* doubleDequant's second step alone, for weights stored WITHOUT Double Quantization (Section 3 prices the fp32
 * constants at 0.5 bit per parameter; Double Quantization is what brings them to 0.127):
 *   w_i = bf16_rne(fl32(table[idx_i] * c2[i / blocksize])),  c2 the fp32 absmax constants of oracle_quantize4
 * (its c2_out).  table: the 16 values of the data type (oracle_codebook4). */
int oracle_dequant4_nodq(const float* table, const uint8_t* packed, const float* c2,
                         int64_t rows, int64_t cols, int32_t blocksize, uint16_t* W_bf16);

/* Eq. 5 with the scalar s of Eq. 3:  Y = X What + s (X L1) L2, all sums fp64,
 * no intermediate rounding.  What is the h x o bf16 matrix from
 * oracle_nf4_dequant.  Only the token rows listed in row_sel (n_sel of them,
 * NULL = all M rows in order) are computed; Y is n_sel x o fp64.  r may be 0.
 *
 * LoRA dropout (hyperparameter appendix: rate 0.1 up to 13B, 0.05 above; the
 * paper gives the rate only, the placement is the one of the LoRA method it
 * builds on: on the input of the adapter branch): D, if not NULL, is an M x h
 * fp64 matrix of multipliers (0 for a dropped element, 1/(1-p) for a kept one)
 * and the branch reads D o X:   Y = X What + s ((D o X) L1) L2.
 * Placement: PARITY UNPINNED against the paper. */
int oracle_linear_fwd(const uint16_t* X, const uint16_t* What,
                      const uint16_t* L1, const uint16_t* L2, double s,
                      int64_t M, int64_t h, int64_t o, int64_t r,
                      const int64_t* row_sel, int64_t n_sel, const double* D, double* Y);

/* Same product, only for the output columns in col_sel; Y is M x n_sel. */
int oracle_linear_fwd_cols(const uint16_t* X, const uint16_t* What,
                           const uint16_t* L1, const uint16_t* L2, double s,
                           int64_t M, int64_t h, int64_t o, int64_t r,
                           const int64_t* col_sel, int64_t n_sel, double* Y);

/* Backward through the frozen weight (Section 3, after Eq. 6):
 *   dX = dY What^T + s D o ((dY L2^T) L1^T)          (D = all ones when NULL)
 * for the token rows in row_sel (NULL = all); dX is n_sel x h fp64. */
int oracle_linear_bwd_dx(const uint16_t* dY, const uint16_t* What,
                         const uint16_t* L1, const uint16_t* L2, double s,
                         int64_t M, int64_t h, int64_t o, int64_t r,
                         const int64_t* row_sel, int64_t n_sel, const double* D, double* dX);

/* Same, only for the input-feature columns in col_sel; dX is M x n_sel. */
int oracle_linear_bwd_dx_cols(const uint16_t* dY, const uint16_t* What,
                              const uint16_t* L1, const uint16_t* L2, double s,
                              int64_t M, int64_t h, int64_t o, int64_t r,
                              const int64_t* col_sel, int64_t n_sel, double* dX);

/* Adapter gradients (only dE/dL_i are formed, never dE/dW), fp64, with
 * Xd = D o X (= X when D is NULL):
 *   dL1 = s Xd^T (dY L2^T)   (h x r),   dL2 = s (Xd L1)^T dY   (r x o). */
int oracle_linear_bwd_dl(const uint16_t* dY, const uint16_t* X,
                         const uint16_t* L1, const uint16_t* L2, double s,
                         int64_t M, int64_t h, int64_t o, int64_t r,
                         const double* D, double* dL1, double* dL2);

#ifdef __cplusplus
}
#endif
#endif
