/*
 * slicer_ref.h -- CPU oracle of the SLICER intermediate-feature codec.
 *
 * TEST INFRASTRUCTURE ONLY.  This is the slow, plain, obviously-correct
 * statement of what the codec computes, written from the paper
 * (arXiv 2511.11608, Sec. 3: ATKF, MS, ABQ, Eq. "dequnt").  It shares no code,
 * header, table or constant generator with the HIP library; only tests, the
 * smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * All pointers are HOST pointers.  Layout of `stream` and `meta` is the wire
 * format (version 1) described at the top of slicer_ref.c.
 */
#ifndef SLICER_REF_H
#define SLICER_REF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { SLICER_REF_F32 = 0, SLICER_REF_BF16 = 1 };

/* Worst-case buffer sizes (every block at max(bit_set)).  Returns 0 or <0. */
int slicer_ref_sizes(int dtype, int64_t rows, int64_t row_len, double keep_ratio,
                     int n_blocks, uint32_t bit_set,
                     size_t* stream_capacity_bytes, size_t* meta_bytes);

/* Encode rows*row_len elements (row-major) into stream + meta.
 * n_threads <= 1: serial; > 1: OpenMP over rows (rows are independent).
 * Returns 0 or <0 (invalid argument). */
int slicer_ref_encode(const void* x, int dtype, int64_t rows, int64_t row_len,
                      double keep_ratio, int n_blocks, uint32_t bit_set,
                      double distortion_budget, void* stream, void* meta,
                      int n_threads);

/* Fixed multi-level mode (Sec. 4.1: Q = [q_1 > ... > q_M], assigned in descending order of
 * magnitude): block m of each sign class is quantised with ladder[m] bits, 1..16, no search.
 * Buffers sized by slicer_ref_sizes with bit_set = the set of ladder values. */
int slicer_ref_encode_ladder(const void* x, int dtype, int64_t rows, int64_t row_len,
                             double keep_ratio, int n_blocks, const uint8_t* ladder,
                             void* stream, void* meta, int n_threads);

/* Paper-literal guard (Sec. 3.2.1, Eq. "DS"): bitwidths are lowered greedily from
 * q_bit = max(bit_set) through bit_set in descending order while
 *   DS(q) = (1/n) sum | floor(c(q_bit) / 2^(q_bit - q)) - c(q) |  <=  delta,
 * stopping at the first violation.  delta >= 0.  The infeasible flag is never set. */
int slicer_ref_encode_ds(const void* x, int dtype, int64_t rows, int64_t row_len,
                         double keep_ratio, int n_blocks, uint32_t bit_set, double delta,
                         void* stream, void* meta, int n_threads);

/* Two-dimensional instances (Sec. 3.2: X of shape N x K; step 3: CSR(X_m) = (v_m, c_m, r_m)): x holds
 * `rows` tensors of n_rows x n_cols, each one codec instance over its flattened view; every block is
 * stored as values, columns and n_rows + 1 row pointers (see slicer_ref.c).  slicer_ref_decode reads the
 * index format from the header. */
int slicer_ref_sizes_csr(int dtype, int64_t rows, int64_t n_rows, int64_t n_cols, double keep_ratio,
                         int n_blocks, uint32_t bit_set, size_t* stream_capacity_bytes, size_t* meta_bytes);
int slicer_ref_encode_csr(const void* x, int dtype, int64_t rows, int64_t n_rows, int64_t n_cols,
                          double keep_ratio, int n_blocks, uint32_t bit_set, double distortion_budget,
                          void* stream, void* meta, int n_threads);

/* Upper bound of the payload before any data is seen (Sec. 3.3): value bits at
 * q_bit = max(bit_set), index bits, header bits (meta + word padding of the rows). */
int slicer_ref_bound(int dtype, int64_t rows, int64_t row_len, double keep_ratio, int n_blocks,
                     uint32_t bit_set, uint64_t* value_bits, uint64_t* index_bits,
                     uint64_t* header_bits);

/* Separate block counts per sign class (Sec. 3.3 lists M(+) and M(-) as two knobs):
 * n_blocks blocks for the positive class, n_blocks_neg for the negative one.  Block order in
 * meta and stream: +0..+M-1, -0..-M(-)-1.  slicer_ref_encode is the case n_blocks_neg = n_blocks. */
int slicer_ref_sizes_pn(int dtype, int64_t rows, int64_t row_len, double keep_ratio,
                        int n_blocks, int n_blocks_neg, uint32_t bit_set,
                        size_t* stream_capacity_bytes, size_t* meta_bytes);
int slicer_ref_encode_pn(const void* x, int dtype, int64_t rows, int64_t row_len,
                         double keep_ratio, int n_blocks, int n_blocks_neg, uint32_t bit_set,
                         double distortion_budget, void* stream, void* meta, int n_threads);

/* Asymmetric thresholds of Sec. 3.1: tau = k-th largest |x|, tau+ = (1 + lambda) tau,
 * tau- = -(1 - lambda) tau; retained are x > tau+ and x < tau-, filled up to k from |x| <= tau
 * downwards, or cut to the k largest when there are more (see the top of slicer_ref.c).
 * lambda in [0, 1), used as an fp32 value; lambda = 0 equals slicer_ref_encode_pn. */
int slicer_ref_encode_atkf(const void* x, int dtype, int64_t rows, int64_t row_len,
                           double keep_ratio, double lambda, int n_blocks, int n_blocks_neg,
                           uint32_t bit_set, double distortion_budget, void* stream, void* meta,
                           int n_threads);
/* per-element view of one row under the same rule (n_blocks for both classes) */
int slicer_ref_analyze_row_atkf(const void* x_row, int dtype, int64_t row_len, double keep_ratio,
                                double lambda, int n_blocks, uint32_t bit_set, double distortion_budget,
                                int32_t* block_of, uint32_t* code_of, float* vmin, float* vmax, uint8_t* qb);

/* Decode into dense y (same dtype and shape as the encoded tensor). */
int slicer_ref_decode(const void* stream, const void* meta, void* y, int n_threads);

/* Per-element view of ONE row, before packing (for stage-by-stage checks):
 *   block_of[i] = -1 if element i is not transmitted, else its block number in
 *                 [0, 2*n_blocks): positive class first, block 0 = largest
 *                 magnitudes;
 *   code_of[i]  = integer code of element i at its block's chosen bitwidth;
 *   vmin/vmax/qb = per-block range and chosen bitwidth (bit 7 of qb = no
 *                 bitwidth met the budget), arrays of 2*n_blocks;
 *   s_int[b*17+q] = integer residual energy S_b(q) for q in 1..16 (0 if q not in
 *                 bit_set), e_int[b] = integer block energy, e_exp[b] = exponent e.
 * Any output pointer may be NULL. */
int slicer_ref_analyze_row(const void* x_row, int dtype, int64_t row_len,
                           double keep_ratio, int n_blocks, uint32_t bit_set,
                           double distortion_budget,
                           int32_t* block_of, uint32_t* code_of,
                           float* vmin, float* vmax, uint8_t* qb,
                           uint64_t* s_int, uint64_t* e_int, int32_t* e_exp);

#ifdef __cplusplus
}
#endif
#endif
