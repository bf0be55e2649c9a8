/*
 * slicer.h -- C ABI of the MI355X (gfx950) implementation of the SLICER
 * intermediate-feature (IF) codec (arXiv 2511.11608, Sec. 3).
 *
 * The codec treats every row of a [rows, row_len] tensor as one instance of the
 * paper's pipeline (the paper flattens an IF to one vector, Sec. 3.2 footnote):
 *
 *   ATKF  (Sec. 3.1, Eq. "split_filter", lambda = 0): keep the
 *         k = floor(keep_ratio * row_len) entries of largest magnitude; ties at
 *         the threshold go to the lower index; exact zeros are never sent;
 *   MS    (Sec. 3.2): split by sign, order each sign class by magnitude, cut it
 *         into n_blocks equal-cardinality blocks (K = floor(n / n_blocks), the
 *         last block takes the remainder), store each block CSR-style as an
 *         index list and a value list;
 *   ABQ   (Sec. 3.2.1): per block, asymmetric min/max integer quantisation at the
 *         smallest bitwidth of bit_set whose squared error stays within
 *         distortion_budget times the block's energy;
 *   decode (Eq. "dequnt"): scatter vmin + code * step, with the class sign, into
 *         a zero tensor.
 *
 * Every pointer named x, y, stream, meta or workspace is a DEVICE pointer owned by
 * the caller; the library neither allocates nor frees device memory, and keeps no
 * state between calls.  Kernels are enqueued on `hip_stream` (a hipStream_t cast
 * to void*, NULL = the default stream); unless stated otherwise a call returns
 * without waiting for them.  Calls return SLICER_OK (0) or a negative code.
 *
 * Wire format, version 1, little-endian:
 *   stream  32-bit words; row r starts at word row_word_off[r].  A row holds, for
 *           its blocks in the order (+0..+M-1, -0..-M-1; block 0 = largest
 *           magnitudes) and ascending index inside a block, first every index
 *           (w = max(1, ceil(log2 row_len)) bits each), then every code (q_b bits
 *           each), least-significant bit first, padded with zeros to a word.
 *   meta    0 u32 magic 0x52434C53   4 u32 version   8 u32 dtype   12 u32 M
 *           16 u64 rows   24 u64 row_len   32 u64 k   40 u32 bit_set   44 u32 w
 *           48 u64 total_words   56 u32 M(-) if the negative class has its own block count
 *           (0: it has M blocks too)   60 u32 n_cols of a two-dimensional instance (0: flat indices)
 *           then  u64 row_word_off[R], u32 n_pos[R], u32 n_neg[R],
 *                 f32 vmin[R][B], f32 vmax[R][B], u8 q[R][B] with B = M + M(-) blocks per row
 *                 (bit 7 of q: no bitwidth met the budget, the largest was used), padded to 8 bytes.
 */
#ifndef SLICER_H
#define SLICER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { SLICER_F32 = 0, SLICER_BF16 = 1 } slicer_dtype;

enum {
    SLICER_OK = 0,
    SLICER_EINVAL = -1,       /* null pointer or argument out of range */
    SLICER_EUNSUPPORTED = -2, /* unknown dtype */
    SLICER_EHIP = -3,         /* a HIP call failed; see slicer_last_hip_error() */
    SLICER_EFORMAT = -4,      /* meta header is not a version-1 header */
    SLICER_ETOOBIG = -5       /* slicer_encode_static: the shape needs more scratch than the library holds */
};

#define SLICER_MAX_BLOCKS 64  /* n_blocks (per sign class) accepted by the library */

/*
 * Buffer sizes for one encode call (Sec. 3.3 upper bound: every block at
 * q_bit = max(bit_set)).  Host-only, no GPU work.
 *   stream_capacity_bytes  rows * ceil(k * (w + q_bit) / 32) * 4
 *   meta_bytes             64 + 16 rows + 18 rows n_blocks, rounded up to 8
 *   workspace_bytes        scratch the encoder needs (contents are undefined
 *                          before and after a call)
 * Any output pointer may be NULL.  Errors: SLICER_EINVAL for rows <= 0,
 * row_len <= 0 or >= 2^31, keep_ratio outside [0,1] or NaN, n_blocks outside
 * [1, SLICER_MAX_BLOCKS], bit_set empty or with bits outside 1..16;
 * SLICER_EUNSUPPORTED for an unknown dtype.
 */
int slicer_sizes(slicer_dtype dt, int64_t rows, int64_t row_len, double keep_ratio,
                 int n_blocks, uint32_t bit_set,
                 size_t* stream_capacity_bytes, size_t* meta_bytes, size_t* workspace_bytes);

/*
 * Encode (Sec. 3.1-3.2.1: ATKF -> MS -> ABQ -> packing).
 *   x          [rows][row_len], row-major contiguous, fp32 or bf16 (dt); finite values
 *   keep_ratio 1 - s of Sec. 3.1, in [0, 1]
 *   n_blocks   M, applied to each sign class (M(+) = M(-))
 *   bit_set    bit q set <=> bitwidth q allowed, 1 <= q <= 16
 *   distortion_budget  beta >= 0: per block, sum (a - a~)^2 <= beta * sum a^2
 *   stream, meta, workspace  at least the sizes slicer_sizes reports; 256-byte aligned
 * Asynchronous.  The number of stream words actually used is meta.total_words
 * (slicer_stream_words).  Errors as slicer_sizes, plus SLICER_EINVAL for a null
 * pointer or a negative / NaN budget, SLICER_EHIP if a launch fails.
 */
int slicer_encode(const void* x, slicer_dtype dt, int64_t rows, int64_t row_len,
                  double keep_ratio, int n_blocks, uint32_t bit_set,
                  double distortion_budget,
                  void* stream, void* meta, void* workspace, void* hip_stream);

/*
 * slicer_encode for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The call
 * allocates nothing (no hipMalloc, hipFree or allocating library routine); its workspace is a
 * static device array of SLICER_STATIC_SCRATCH_BYTES inside the library, of which every GPU the
 * library runs on holds a copy until the process ends.  Arguments, output and errors as
 * slicer_encode (same kernels, byte-identical stream and meta), plus SLICER_ETOOBIG when the
 * shape's workspace_bytes (slicer_sizes) exceed SLICER_STATIC_SCRATCH_BYTES.  All calls on one
 * GPU share that GPU's array: calls that overlap in time on one GPU (two streams, two host
 * threads) race and give undefined output; calls on one stream are ordered and safe.  The
 * array keeps the last call's contents; the kernels write every word before they read it.
 */
#define SLICER_STATIC_SCRATCH_BYTES (64u << 20)
int slicer_encode_static(const void* x, slicer_dtype dt, int64_t rows, int64_t row_len,
                         double keep_ratio, int n_blocks, uint32_t bit_set,
                         double distortion_budget, void* stream, void* meta, void* hip_stream);

/*
 * Decode (Eq. "dequnt": de-quantise every block and scatter it into a zero
 * tensor).  y receives [rows][row_len] in the dtype recorded in meta; every
 * element is written.  This call first copies the 64-byte header to the host and
 * waits for `hip_stream`, validates it (SLICER_EFORMAT), then enqueues the decode
 * kernel.
 */
int slicer_decode(const void* stream, const void* meta, void* y, void* hip_stream);

/*
 * Same decode for callers that already hold the shape on the host: no header
 * read, no wait.  dt, rows, row_len and n_blocks must be the values passed to
 * slicer_encode; the header in meta is not consulted.
 */
int slicer_decode_as(const void* stream, const void* meta, void* y, slicer_dtype dt,
                     int64_t rows, int64_t row_len, int n_blocks, void* hip_stream);

/*
 * Separate block counts for the two sign classes (Sec. 3.3 lists M(+) and M(-) as two knobs of
 * the configuration): n_blocks blocks for the positive class, n_blocks_neg for the negative
 * one, each in [1, SLICER_MAX_BLOCKS].  Block order in meta and stream: +0..+M-1, then
 * -0..-M(-)-1; meta holds n_blocks + n_blocks_neg entries per row (meta_bytes = 64 + 16 rows +
 * 9 rows (n_blocks + n_blocks_neg), rounded up to 8), and header offset 56 holds n_blocks_neg
 * when it differs from n_blocks (0 otherwise, so equal counts give the bytes of slicer_encode).
 * slicer_decode reads both counts from the header.  Everything else as the calls without _pn.
 */
int slicer_sizes_pn(slicer_dtype dt, int64_t rows, int64_t row_len, double keep_ratio,
                    int n_blocks, int n_blocks_neg, uint32_t bit_set,
                    size_t* stream_capacity_bytes, size_t* meta_bytes, size_t* workspace_bytes);
int slicer_encode_pn(const void* x, slicer_dtype dt, int64_t rows, int64_t row_len,
                     double keep_ratio, int n_blocks, int n_blocks_neg, uint32_t bit_set,
                     double distortion_budget,
                     void* stream, void* meta, void* workspace, void* hip_stream);
/*
 * The asymmetric thresholds of Sec. 3.1 (Eq. "split_filter" with an asymmetry factor lambda in
 * [0, 1), used as an fp32 value): tau = the k-th largest |x| of the row, tau+ = (1 + lambda) tau,
 * tau- = -(1 - lambda) tau (one fp32 multiplication each); strictly retained are x > tau+ and
 * x < tau-.  Fewer than k of them: the set is filled up to k from the elements with |x| <= tau
 * that are not in it, largest magnitude first (equal magnitudes: lower index first), so positive
 * values in (tau, tau+] are never sent.  k or more (the section is silent; its exact count
 * decides): the k largest magnitudes of the set stay.  lambda = 0 is slicer_encode_pn and takes
 * its kernels; lambda > 0 needs a second selection over a subset of the row, which is built in the
 * row-resident kernel (bf16 rows up to 8192 elements, fp32 rows up to 4096) and in the generic
 * one-workgroup-per-row kernel for everything else.  Buffers, format and decode as slicer_encode_pn;
 * SLICER_EINVAL for lambda outside [0, 1).
 */
int slicer_encode_atkf(const void* x, slicer_dtype dt, int64_t rows, int64_t row_len,
                       double keep_ratio, double lambda, int n_blocks, int n_blocks_neg,
                       uint32_t bit_set, double distortion_budget,
                       void* stream, void* meta, void* workspace, void* hip_stream);
int slicer_decode_as_pn(const void* stream, const void* meta, void* y, slicer_dtype dt,
                        int64_t rows, int64_t row_len, int n_blocks, int n_blocks_neg,
                        void* hip_stream);
int slicer_check_pn(const void* meta, uint64_t stream_words, slicer_dtype dt, int64_t rows,
                    int64_t row_len, int n_blocks, int n_blocks_neg, void* scratch,
                    void* hip_stream);

/*
 * Two-dimensional instances (Sec. 3.2: an IF X of shape N x K; step 3: every block stored as
 * CSR(X_m) = (v_m, c_m, r_m)).  x holds `instances` tensors of n_rows x n_cols (row-major), each one
 * codec instance: ATKF and MS work on its flattened view of length n_rows * n_cols (the footnote of
 * Sec. 3.2 step 1), so kept set, blocks, ranges, bitwidths and codes are those of slicer_encode on rows
 * of that length.  The index encoding differs: per instance the stream holds, for its blocks in order,
 * first every block's n_rows + 1 row pointers (r: pointer j = number of the block's entries in tensor
 * rows before j, the exclusive scan of its per-row counts; wp = max(1, ceil(log2(k + 1))) bits each),
 * then the column of every entry (c: wc = max(1, ceil(log2 n_cols)) bits, row-major inside a block),
 * then the codes (v), LSB-first, padded to a word.  Header: offset 44 holds wc, offset 60 n_cols (0
 * there marks the flat index format of slicer_encode); meta arrays as slicer_encode.
 *   stream_capacity_bytes  instances * ceil((2 n_blocks (n_rows + 1) wp + k (wc + q_bit)) / 32) * 4
 * n_rows * n_cols < 2^31.  The flat encoder of the shape does the work (its stream goes to the
 * workspace) and two short kernels re-pack the index section into this form.  slicer_decode reads the
 * index format from the header; slicer_decode_as_csr takes the shape from the caller (it reads k from
 * the header in meta for the pointer width, nothing else).  slicer_check_csr is slicer_check for these
 * metas (slicer_check itself rejects them); the decoder clamps every row pointer to its block and every
 * column to its tensor row, so after SLICER_OK a forged stream cannot take it outside stream or y.
 * Errors as slicer_sizes / slicer_encode / slicer_decode_as / slicer_check.
 */
int slicer_sizes_csr(slicer_dtype dt, int64_t instances, int64_t n_rows, int64_t n_cols, double keep_ratio,
                     int n_blocks, uint32_t bit_set,
                     size_t* stream_capacity_bytes, size_t* meta_bytes, size_t* workspace_bytes);
int slicer_encode_csr(const void* x, slicer_dtype dt, int64_t instances, int64_t n_rows, int64_t n_cols,
                      double keep_ratio, int n_blocks, uint32_t bit_set, double distortion_budget,
                      void* stream, void* meta, void* workspace, void* hip_stream);
int slicer_decode_as_csr(const void* stream, const void* meta, void* y, slicer_dtype dt, int64_t instances,
                         int64_t n_rows, int64_t n_cols, int n_blocks, void* hip_stream);
int slicer_check_csr(const void* meta, uint64_t stream_words, slicer_dtype dt, int64_t instances,
                     int64_t n_rows, int64_t n_cols, int n_blocks, void* scratch, void* hip_stream);

/*
 * Encode with the paper's own guard (Sec. 3.2.1, Eq. "DS" and the greedy search stated under it:
 * start at the largest bitwidth q_bit and step down while the mismatch stays within delta):
 * with q_bit = max(bit_set) and c(q) the block's AIQ codes at q bits,
 *     DS(q) = (1/n) * sum | floor(c(q_bit) / 2^(q_bit - q)) - c(q) |,
 * a block's bitwidth goes down through bit_set in descending order while DS(q) <= delta and
 * stops at the first violation.  The integer sum is compared as (double)sum <= delta * n.
 * delta >= 0; the infeasible flag of slicer_encode is never set.  Everything else (arguments,
 * buffers, errors, asynchrony) as slicer_encode.
 */
int slicer_encode_ds(const void* x, slicer_dtype dt, int64_t rows, int64_t row_len,
                     double keep_ratio, int n_blocks, uint32_t bit_set, double delta,
                     void* stream, void* meta, void* workspace, void* hip_stream);

/*
 * Fixed multi-level mode (Sec. 4.1, the list Q = [q_1, ..., q_M] of the experiments: one
 * bitwidth per block, the widest for the largest magnitudes): block m of
 * either sign class (block 0 = largest magnitudes) is quantised with ladder[m] bits; there
 * is no bitwidth search and no distortion guard, everything else is slicer_encode.
 *   ladder   HOST pointer, n_blocks entries, each 1..16 (any order is accepted; it is read
 *            during the call, not afterwards).
 * Buffers are sized by slicer_sizes with bit_set = slicer_ladder_bit_set(ladder, n_blocks),
 * which is also the bit_set written to the header.  Errors as slicer_encode; SLICER_EINVAL for
 * a null ladder or an entry outside 1..16.
 */
int slicer_encode_ladder(const void* x, slicer_dtype dt, int64_t rows, int64_t row_len,
                         double keep_ratio, int n_blocks, const uint8_t* ladder,
                         void* stream, void* meta, void* workspace, void* hip_stream);

/* The set of bitwidths of a ladder (bit q set <=> some ladder[m] == q); 0 for an invalid ladder. */
uint32_t slicer_ladder_bit_set(const uint8_t* ladder, int n_blocks);

/*
 * Upper bound of the payload, known before any data is seen (Sec. 3.3, "Predictive Bit/Time
 * Model": every block at q_bit = max(bit_set), plus index and header bits), for a control
 * plane that must check a bit budget before execution.  Host computation only.
 *   value_bits   rows * k * q_bit
 *   index_bits   rows * k * w
 *   header_bits  8 * meta_bytes + the zero bits that pad every row's segment to a 32-bit word
 * The three add up to 8 * (stream_capacity_bytes + meta_bytes) of slicer_sizes; no encode
 * call with these arguments produces more.  Any output pointer may be null.
 */
int slicer_bound(slicer_dtype dt, int64_t rows, int64_t row_len, double keep_ratio, int n_blocks,
                 uint32_t bit_set, uint64_t* value_bits, uint64_t* index_bits, uint64_t* header_bits);

/*
 * Which kernel family slicer_encode uses for a shape (for benchmarks and profiles, which
 * name the dominant kernel): 0 = generic (one workgroup per row, any shape), 1 = row-resident
 * (one wavefront per row, rows up to 4096 elements), 2 = long-row stages
 * (rows of more than 4096 elements that the other two do not take), 3 = one workgroup per row
 * (rows of 4097..32768 bf16 / 4097..16384 fp32 elements).
 * Assumes a 16-byte aligned x and the budget guard.  Negative: error code.
 */
int slicer_encode_path(slicer_dtype dt, int64_t rows, int64_t row_len, double keep_ratio,
                       int n_blocks, uint32_t bit_set);

/*
 * The decode calls TRUST stream and meta: they must be the bytes an encode call produced
 * (the kernels guard only the scatter index, so a forged meta can make them read outside the
 * stream).  A receiver of bytes from elsewhere calls slicer_check first: it verifies, on the
 * GPU and without touching the stream, that the header matches (dt, rows, row_len, n_blocks),
 * that every row's counts are possible (n_pos + n_neg <= k <= row_len), every bitwidth is in
 * 1..16 and in the header's bit_set, every row's offset is the exclusive scan of the exact word
 * counts implied by counts and bitwidths, and that total_words <= stream_words, the number of
 * 32-bit words the caller actually holds.  After SLICER_OK, slicer_decode / slicer_decode_as
 * with the same arguments stay inside stream[0, stream_words) and y.
 *   scratch   device memory, at least 4 bytes, 4-byte aligned (overwritten)
 * Waits for `hip_stream`.  SLICER_EFORMAT for any inconsistency, SLICER_EINVAL for bad
 * arguments.
 */
int slicer_check(const void* meta, uint64_t stream_words, slicer_dtype dt, int64_t rows,
                 int64_t row_len, int n_blocks, void* scratch, void* hip_stream);

/* Reads meta.total_words (the packed size of Sec. 3.3's payload, in 32-bit words)
 * to the host.  Waits for `hip_stream`. */
int slicer_stream_words(const void* meta, uint64_t* words, void* hip_stream);

/*
 * Timing hook for benchmarks.  While both events are non-NULL (hipEvent_t cast to
 * void*), every slicer_encode / slicer_decode / slicer_decode_as issued by the
 * calling thread records `start` immediately before and `stop` immediately after
 * its dominant kernel (the per-row encode kernel, or the decode kernel) on the
 * call's stream, so that the kernel's own duration can be read with
 * hipEventElapsedTime.  Pass NULL, NULL to switch it off (the default).
 */
int slicer_profile_events(void* start_event, void* stop_event);

/*
 * Diagnostic: runs ONE elementary operation of the codec's arithmetic (Sec. 3.2.1, Eq. "dequnt": the
 * divisions, products, sums, roundings and scalings behind AIQ, the guard and the decoder), written as
 * the kernels write it, on n pairs of 32-bit operands; for tests that compare the results bit for bit
 * with the host's IEEE arithmetic.  a, b, out: device arrays of n 32-bit words (fp32 bit patterns).
 *   op 0  a / b            1  __fdiv_rn(a, b)     2  a * b        3  a + b        4  a - b
 *      5  rintf(a)         6  ldexpf(a, b mod 301 - 150)          7  a * b + 2^23 (two operations)
 *      8  fp32 -> bf16, round to nearest even (result in the low 16 bits)
 *      9  a + b * b (two operations)
 *     10  energy grid: rint(|a| * 2^(20 - e)), e = ilogb(|a|) + 1 + (b mod 3), on the significand
 *     11  hi ^ lo words of the double (a * a) * (double)b * 2^-30, all products in double
 * Asynchronous on hip_stream.  SLICER_EINVAL for a null pointer, n <= 0 or an unknown op.
 */
int slicer_arith_probe(int op, const void* a, const void* b, void* out, int64_t n, void* hip_stream);

/* hipError_t of the most recent failed HIP call made by this library on the
 * calling thread (0 if none). */
int slicer_last_hip_error(void);

/* Static, human-readable text for a return code. */
const char* slicer_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* SLICER_H */
