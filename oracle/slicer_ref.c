/*
 * slicer_ref.c -- CPU oracle of the SLICER intermediate-feature codec.
 *
 * TEST INFRASTRUCTURE ONLY (see slicer_ref.h).  Plain C, one row at a time, a
 * full sort per row, scalar loops, no blocking or fusion: every function is
 * meant to be checked against the paper by eye.  Build with
 *   gcc -O2 -std=c11 -ffp-contract=off -fno-fast-math -fopenmp
 * so that every fp32 operation below is one IEEE round-to-nearest-even
 * operation and no multiply-add is contracted.
 *
 * What is computed, per row of N elements (a row is one codec instance; the
 * paper flattens an IF to one vector, Sec. 3.2 footnote):
 *
 *  1. ATKF (Sec. 3.1, Eq. "split_filter", lambda = 0): k = floor(keep_ratio*N);
 *     keep the k largest |x|; ties at the threshold go to the LOWER index
 *     (the paper picks ties at random; a fixed rule makes the result unique).
 *  2. Exact zeros are not transmitted (Sec. 3.2 step 1: Omega = non-zeros).
 *  3. Sign separation (Sec. 3.2 pre-step): class + (x > 0), class - (x < 0),
 *     value a = |x|.
 *  4. MS (Sec. 3.2 steps 1-2): per class sort by magnitude descending (equal
 *     magnitudes: lower index first), K = floor(n/M); rank r goes to block
 *     min(r / K, M-1) (all to block M-1 when K = 0), so blocks 0..M-2 hold
 *     exactly K and the last block takes the remainder.
 *  5. AIQ (Sec. 3.2.1): per block affine min/max quantiser at q bits,
 *     L = 2^q - 1, taken on the block's own scale so that it behaves the same for
 *     tensors of any magnitude: with er = ilogb(rng), rng1 = rng * 2^-er in [1, 2),
 *     inv = L / rng1, y = ((a - vmin) * 2^-er) * inv, c = clamp(rint(y), 0, L),
 *     reconstruction vmin + c * (rng / L).  (Zero-point folded into vmin; the
 *     printed ceil is read as round-to-nearest-even; the two power-of-two scalings
 *     are exact, so y is (a - vmin) * (L / rng) whenever that quotient is an
 *     ordinary fp32 number.)  Only a block of range exactly 0 is degenerate: it is
 *     sent as its minimum (all codes 0).
 *  6. ABQ (Sec. 3.2.1 "rate-distortion solver"): smallest q in bit_set whose
 *     distortion is within the budget: sum (a - a~)^2 <= beta * sum a^2 per
 *     block, both sums taken on integer grids so they do not depend on the
 *     order of summation (the paper's guard is an integer metric as well):
 *       residual  rho_i = rint((y_i - c_i) * 2^15)            S = sum rho_i^2
 *       energy    A_i   = rint(a_i * 2^(20-e)), e = ilogb(vmax)+1   E = sum A_i^2
 *       feasible  <=>  o*o * S * 2^-30  <=  beta * E * 2^(2e-40)   (in double)
 *     If no q is feasible the largest is used and bit 7 of the stored q is set.
 *  7. CSR-style packing (Sec. 3.2 step 3): per row, for blocks in order
 *     (+0..+M-1, -0..-M-1) and ascending index inside a block: first all
 *     indices (w = max(1, ceil(log2 N)) bits each), then all codes (q_b bits
 *     each), LSB-first in little-endian 32-bit words, row padded to a word.
 *  8. Decode (Eq. "dequnt"): y = 0; y[idx] = +-(vmin + c * o).
 *
 * Fixed multi-level mode (Sec. 4.1 "multi-level quantization", Q = [q_1 > ... > q_M]):
 * block m of either sign class is quantised with the given q_m (block 0 = largest
 * magnitudes gets q_1); there is no search and no distortion guard, everything else
 * (ATKF, MS, AIQ, packing) is as above.  The header's bit_set is the set of ladder values.
 *
 * Paper-literal guard (Sec. 3.2.1, Eq. "DS" and the greedy search under it): with
 * q_bit = max(bit_set) and c_i(q) the AIQ code of element i at q bits,
 *       DS(q) = (1/n) * sum_i | floor(c_i(q_bit) / 2^(q_bit - q)) - c_i(q) |,
 * the bitwidth is lowered from q_bit through the allowed bitwidths in descending order for
 * as long as DS(q) <= delta, and stops at the first violation (greedy: a lower bitwidth that
 * would pass again is not looked at).  The sum is an integer; the test is
 * (double)sum <= delta * (double)n.  See slicer_ref_encode_ds.
 *
 * Asymmetric thresholds (Sec. 3.1 with lambda in [0,1); slicer_ref_encode_atkf): with tau the
 * k-th largest |x| of the row, tau+ = (1+lambda)*tau and tau- = (1-lambda)*tau (each one fp32
 * operation on lambda rounded to fp32), the strictly retained set is
 *       S = { x > tau+ }  union  { x < -tau- }.
 * |S| < k: S is filled up to k elements from { i not in S : |x_i| <= tau }, largest magnitude
 * first (the ties at tau, then the next lower magnitudes; equal magnitudes: lower index first).
 * Positive values in (tau, tau+] are therefore never sent: that is what the shifted cut-off does.
 * |S| >= k (the paper is silent; its claim of an exact count decides): the k largest magnitudes
 * of S are kept (equal magnitudes: lower index first).  lambda = 0 gives item 1 above.
 *
 * Two-dimensional instance (Sec. 3.2: an IF X of shape N x K, and step 3, CSR(X_m) = (v_m, c_m, r_m);
 * slicer_ref_encode_csr): one codec instance is a whole n_rows x n_cols tensor.  ATKF and MS work on
 * its flattened view of length T = n_rows * n_cols (the footnote of Sec. 3.2 step 1), so kept set,
 * blocks, ranges, bitwidths and codes are those of a flat row of length T.  Only the index encoding
 * differs: every block is stored as a CSR triple - its values in row-major order (v), the column of
 * every value (c), and n_rows + 1 row pointers (r): r[j] = number of the block's entries in tensor
 * rows before j, i.e. the exclusive scan of the block's per-row counts, r[n_rows] = block size.
 * Segment of an instance: all row pointers (blocks in order, wp = max(1, ceil(log2(k + 1))) bits
 * each: any block size fits), then all columns (wc = max(1, ceil(log2 n_cols)) bits each, blocks
 * in order, row-major inside a block), then all codes.  Header: offset 44 holds wc, offset 60 holds
 * n_cols (0 there marks flat indices).
 *
 * Payload bound (Sec. 3.3, "Predictive Bit/Time Model"): every kept slot at the largest
 * bitwidth, plus index and header bits; see slicer_ref_bound.
 *
 * Wire format, version 1 (little-endian):
 *   meta:  0 u32 magic 0x52434C53   4 u32 version   8 u32 dtype   12 u32 M
 *         16 u64 rows  24 u64 row_len  32 u64 k  40 u32 bit_set  44 u32 w
 *         48 u64 total_words  56 u32 M(-) if it differs from M (else 0)
 *         60 u32 n_cols of a two-dimensional instance (0: flat indices)
 *         64            u64 row_word_off[R]   (exclusive scan of row words)
 *         64+8R         u32 n_pos[R]
 *         64+12R        u32 n_neg[R]
 *         64+16R        f32 vmin[R][B]     B = M + M(-) blocks per row (2M when equal)
 *         64+16R+4RB    f32 vmax[R][B]
 *         64+16R+8RB    u8  q[R][B]
 *         size = 64 + 16R + 9RB rounded up to a multiple of 8
 *   stream: total_words 32-bit words, rows concatenated.
 */
#include "slicer_ref.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define REF_MAGIC 0x52434C53u
#define REF_VERSION 1u
#define REF_HDR 64

typedef struct { uint32_t key, idx; } kv_t;

/* ---- element access --------------------------------------------------- */

static uint32_t load_bits(const void* x, int dt, int64_t i) /* fp32 pattern of element i */
{
    if (dt == SLICER_REF_F32) {
        uint32_t u;
        memcpy(&u, (const char*)x + 4 * i, 4);
        return u;
    } else {
        uint16_t h;
        memcpy(&h, (const char*)x + 2 * i, 2);
        return (uint32_t)h << 16; /* bf16 -> fp32 is exact */
    }
}

static float bits_to_float(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
static uint32_t float_to_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }

static uint16_t float_to_bf16_rne(float f)
{
    uint32_t u = float_to_bits(f);
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7FFFu + lsb;
    return (uint16_t)(u >> 16);
}

/* ---- argument checks ---------------------------------------------------- */

static int check_args(int dt, int64_t rows, int64_t N, double keep, int M, uint32_t bit_set)
{
    if (dt != SLICER_REF_F32 && dt != SLICER_REF_BF16) return -2;
    if (rows <= 0 || N <= 0 || N >= ((int64_t)1 << 31)) return -1;
    if (!(keep >= 0.0 && keep <= 1.0)) return -1;
    if (M < 1 || M > 128) return -1;
    if (bit_set == 0 || (bit_set & ~0x1FFFEu)) return -1; /* bits 1..16 only */
    return 0;
}

static int64_t keep_count(double keep, int64_t N) /* ATKF: k = floor((1-s) N) */
{
    return (int64_t)floor(keep * (double)N);
}

static int index_bits(int64_t N)
{
    int w = 1;
    while (((int64_t)1 << w) < N) ++w;
    return w;
}

static int max_bit(uint32_t bit_set) { int q = 16; while (!((bit_set >> q) & 1u)) --q; return q; }
static int min_bit(uint32_t bit_set) { int q = 1;  while (!((bit_set >> q) & 1u)) ++q; return q; }

/* B2 = number of blocks per row = M(+) + M(-) */
static size_t meta_size(int64_t R, int B2)
{
    size_t s = REF_HDR + 16 * (size_t)R + 9 * (size_t)R * (size_t)B2;
    return (s + 7) & ~(size_t)7;
}

int slicer_ref_sizes_pn(int dt, int64_t rows, int64_t N, double keep, int M, int Mn, uint32_t bit_set,
                        size_t* stream_cap, size_t* meta_bytes)
{
    int rc = check_args(dt, rows, N, keep, M, bit_set);
    if (rc) return rc;
    if (Mn < 1 || Mn > 128) return -1;
    int64_t k = keep_count(keep, N);
    uint64_t bits = (uint64_t)k * (uint64_t)(index_bits(N) + max_bit(bit_set));
    uint64_t words = (bits + 31) / 32;
    if (stream_cap) *stream_cap = (size_t)(words * 4 * (uint64_t)rows);
    if (meta_bytes) *meta_bytes = meta_size(rows, M + Mn);
    return 0;
}

int slicer_ref_sizes(int dt, int64_t rows, int64_t N, double keep, int M, uint32_t bit_set,
                     size_t* stream_cap, size_t* meta_bytes)
{
    return slicer_ref_sizes_pn(dt, rows, N, keep, M, M, bit_set, stream_cap, meta_bytes);
}

static int bits_for_count(int64_t k) /* bits that hold any value in 0..k */
{
    int w = 1;
    while (((int64_t)1 << w) <= k) ++w;
    return w;
}

/* Two-dimensional instances: `rows` tensors of n_rows x n_cols each. */
int slicer_ref_sizes_csr(int dt, int64_t rows, int64_t n_rows, int64_t n_cols, double keep, int M,
                         uint32_t bit_set, size_t* stream_cap, size_t* meta_bytes)
{
    if (n_rows <= 0 || n_cols <= 0 || n_rows > ((int64_t)1 << 31) / n_cols) return -1;
    const int64_t T = n_rows * n_cols;
    int rc = check_args(dt, rows, T, keep, M, bit_set);
    if (rc) return rc;
    const int64_t k = keep_count(keep, T);
    const uint64_t bits = (uint64_t)(2 * M) * (uint64_t)(n_rows + 1) * (uint64_t)bits_for_count(k)
                        + (uint64_t)k * (uint64_t)(index_bits(n_cols) + max_bit(bit_set));
    if (stream_cap) *stream_cap = (size_t)(((bits + 31) / 32) * 4 * (uint64_t)rows);
    if (meta_bytes) *meta_bytes = meta_size(rows, 2 * M);
    return 0;
}

/* ---- one row: everything up to (but not including) packing ------------- */

static int cmp_mag_desc_idx_asc(const void* pa, const void* pb)
{
    const kv_t* a = (const kv_t*)pa;
    const kv_t* b = (const kv_t*)pb;
    if (a->key != b->key) return a->key > b->key ? -1 : 1;
    if (a->idx != b->idx) return a->idx < b->idx ? -1 : 1;
    return 0;
}

typedef struct {
    /* per element */
    int32_t* block_of;  /* [N] */
    uint32_t* code_of;  /* [N] */
    /* per block, 2M entries */
    float* vmin;
    float* vmax;
    uint8_t* qb;
    uint32_t* count;    /* elements in block */
    uint64_t* s_int;    /* [2M][17], may be NULL */
    uint64_t* e_int;    /* [2M], may be NULL */
    int32_t* e_exp;     /* [2M], may be NULL */
    uint32_t n_pos, n_neg;
} row_result;

/* The quantiser works on the block's own scale (Sec. 3.2.1 defines the step o = range / (2^q - 1)
 * for any non-zero range): er = ilogb(range), and both the range and every offset a - vmin are
 * multiplied by 2^-er, which is exact. */
static int range_exp(float rng) { return ilogbf(rng); }
static float unit_range(float rng, int er) { return ldexpf(rng, -er); }   /* in [1, 2) */

/* AIQ code of value a in a block [vmin, vmin+rng] at L = 2^q - 1 levels, inv = L / unit_range;
 * also returns the scaled position y. */
static uint32_t aiq_code(float a, float vmin, int er, float inv, float L, float* y_out)
{
    float y = ldexpf(a - vmin, -er) * inv;
    float r = rintf(y);
    if (r < 0.0f) r = 0.0f;
    if (r > L) r = L;
    *y_out = y;
    return (uint32_t)r;
}

/* DS guard (Eq. "DS"): greedy descent from q_bit; returns the chosen bitwidth.
 * ds_sum (17 entries, may be NULL) receives the integer sums of the bitwidths that were looked at. */
static int ds_greedy(const kv_t* el, uint32_t cnt, uint32_t bit_set, double delta,
                     float vmin, float rng, int degenerate, uint64_t* ds_sum)
{
    const int er = degenerate ? 0 : range_exp(rng);
    const float rng1 = degenerate ? 1.0f : unit_range(rng, er);
    const int qbit = max_bit(bit_set);
    uint32_t* c0 = (uint32_t*)malloc(sizeof(uint32_t) * (size_t)cnt);
    const float L0 = (float)((1u << qbit) - 1u);
    const float inv0 = degenerate ? 0.0f : L0 / rng1;
    for (uint32_t j = 0; j < cnt; ++j) {
        float y;
        c0[j] = degenerate ? 0u : aiq_code(bits_to_float(el[j].key), vmin, er, inv0, L0, &y);
    }
    int chosen = qbit;
    for (int q = qbit - 1; q >= 1; --q) {
        if (!((bit_set >> q) & 1u)) continue;
        const float L = (float)((1u << q) - 1u);
        const float inv = degenerate ? 0.0f : L / rng1;
        uint64_t D = 0;
        for (uint32_t j = 0; j < cnt; ++j) {
            float y;
            uint32_t c = degenerate ? 0u : aiq_code(bits_to_float(el[j].key), vmin, er, inv, L, &y);
            uint32_t ref = c0[j] >> (qbit - q);
            D += ref > c ? ref - c : c - ref;
        }
        if (ds_sum) ds_sum[q] = D;
        if ((double)D <= delta * (double)cnt) chosen = q; else break;
    }
    free(c0);
    return chosen;
}

/* fixed_q > 0: the block's bitwidth is given (multi-level mode), no search;
 * fixed_q < 0: the DS guard with delta = beta (greedy descent) */
static void quantise_block(const kv_t* el, uint32_t cnt, uint32_t bit_set, double beta,
                           int fixed_q, int b, row_result* out)
{
    /* block range (Sec. 3.2.1: v^min, v^max) */
    float vmin = bits_to_float(el[0].key), vmax = vmin;
    for (uint32_t j = 1; j < cnt; ++j) {
        float a = bits_to_float(el[j].key);
        if (a < vmin) vmin = a;
        if (a > vmax) vmax = a;
    }
    float rng = vmax - vmin;
    out->vmin[b] = vmin;
    out->vmax[b] = vmax;

    /* integer block energy on a 20-bit grid scaled to vmax */
    int e = ilogbf(vmax) + 1;
    uint64_t E = 0;
    for (uint32_t j = 0; j < cnt; ++j) {
        float a = bits_to_float(el[j].key);
        uint64_t A = (uint64_t)rintf(ldexpf(a, 20 - e));
        E += A * A;
    }
    if (out->e_int) out->e_int[b] = E;
    if (out->e_exp) out->e_exp[b] = e;

    int degenerate = !(rng > 0.0f);
    const int er = degenerate ? 0 : range_exp(rng);
    const float rng1 = degenerate ? 1.0f : unit_range(rng, er);
    int chosen = fixed_q > 0 ? fixed_q : -1;
    if (fixed_q < 0)
        chosen = ds_greedy(el, cnt, bit_set, beta, vmin, rng, degenerate,
                           out->s_int ? out->s_int + (size_t)b * 17 : NULL);
    for (int q = 1; q <= 16 && fixed_q == 0; ++q) {
        if (!((bit_set >> q) & 1u)) continue;
        if (chosen >= 0 && !out->s_int) break; /* later sums only wanted for inspection */
        uint64_t S = 0;
        float L = (float)((1u << q) - 1u);
        float o = 0.0f;
        if (!degenerate) {
            o = rng / L;
            float inv = L / rng1;
            for (uint32_t j = 0; j < cnt; ++j) {
                float a = bits_to_float(el[j].key);
                float y;
                uint32_t c = aiq_code(a, vmin, er, inv, L, &y);
                int64_t rho = (int64_t)rintf((y - (float)c) * 32768.0f);
                S += (uint64_t)(rho * rho);
            }
        }
        if (out->s_int) out->s_int[(size_t)b * 17 + q] = S;
        if (chosen < 0) {
            int feasible;
            if (degenerate) {
                feasible = 1;
            } else {
                double lhs = ((double)o * (double)o) * (double)S * 0x1p-30;
                double rhs = beta * ldexp((double)E, 2 * e - 40);
                feasible = lhs <= rhs;
            }
            if (feasible) chosen = q;
        }
    }
    uint8_t qstore;
    int q;
    if (chosen < 0) { q = max_bit(bit_set); qstore = (uint8_t)(q | 0x80); }
    else            { q = chosen;           qstore = (uint8_t)q; }
    out->qb[b] = qstore;

    /* codes at the chosen bitwidth */
    float L = (float)((1u << q) - 1u);
    float inv = degenerate ? 0.0f : L / rng1;
    for (uint32_t j = 0; j < cnt; ++j) {
        uint32_t c = 0;
        if (!degenerate) {
            float y;
            c = aiq_code(bits_to_float(el[j].key), vmin, er, inv, L, &y);
        }
        out->code_of[el[j].idx] = c;
    }
}

/* ladder != NULL: multi-level mode, ladder[m] = bitwidth of block m of each class;
 * ds != 0: the DS guard with delta = beta instead of the relative-error budget */
/* M, Mn: blocks of the positive and of the negative class (Sec. 3.3: M(+), M(-)); block
 * numbers are +0..+M-1 then -0..-Mn-1 */
/* ATKF with asymmetric thresholds (Sec. 3.1): `all` holds the row in (magnitude desc, index asc)
 * order; writes the retained elements to `sel` in the same order and returns their number (<= k). */
static int64_t atkf_asymmetric(const void* x, int dt, const kv_t* all, int64_t N, int64_t k, float lambda, kv_t* sel)
{
    if (k <= 0) return 0;
    const float tau = bits_to_float(all[k - 1].key);           /* k-th largest |x| */
    const float one_plus = 1.0f + lambda, one_minus = 1.0f - lambda;
    const float tau_pos = one_plus * tau;                        /* tau+ = (1 + lambda) tau */
    const float tau_neg = one_minus * tau;                       /* |tau-| = (1 - lambda) tau */
    uint8_t* strict = (uint8_t*)malloc((size_t)N);
    if (!strict) return -1;
    int64_t c = 0;
    for (int64_t r = 0; r < N; ++r) {                           /* S_strict = { x > tau+ or x < tau- } */
        const float a = bits_to_float(all[r].key);
        const int neg = (int)(load_bits(x, dt, all[r].idx) >> 31);
        strict[r] = neg ? (a > tau_neg) : (a > tau_pos);
        c += strict[r];
    }
    int64_t n = 0;
    if (c >= k) {                                               /* more than asked for: the k largest of S_strict */
        for (int64_t r = 0; r < N && n < k; ++r)
            if (strict[r]) sel[n++] = all[r];
    } else {                                                    /* S_strict, filled from |x| <= tau downwards */
        int64_t fill = k - c;
        for (int64_t r = 0; r < N; ++r) {
            if (strict[r]) sel[n++] = all[r];
            else if (fill > 0 && all[r].key <= all[k - 1].key) { sel[n++] = all[r]; --fill; }
        }
    }
    free(strict);
    return n;
}

/* lambda < 0: plain top-K (the k largest magnitudes); lambda >= 0: asymmetric thresholds */
static int analyze_row(const void* x, int dt, int64_t N, int64_t k, int M, int Mn, uint32_t bit_set,
                       double beta, const uint8_t* ladder, int ds, float lambda, row_result* out)
{
    kv_t* all = (kv_t*)malloc(sizeof(kv_t) * (size_t)N);
    kv_t* cls = (kv_t*)malloc(sizeof(kv_t) * (size_t)(k > 0 ? k : 1));
    kv_t* sel = (kv_t*)malloc(sizeof(kv_t) * (size_t)(k > 0 ? k : 1));
    if (!all || !cls || !sel) { free(all); free(cls); free(sel); return -3; }

    /* ATKF: order all elements by magnitude (bit pattern with the sign cleared
     * orders finite values by |x|), ties by lower index; keep the first k. */
    for (int64_t i = 0; i < N; ++i) {
        all[i].key = load_bits(x, dt, i) & 0x7FFFFFFFu;
        all[i].idx = (uint32_t)i;
        out->block_of[i] = -1;
        out->code_of[i] = 0;
    }
    qsort(all, (size_t)N, sizeof(kv_t), cmp_mag_desc_idx_asc);
    int64_t n_sel = k;
    if (lambda >= 0.0f) {
        n_sel = atkf_asymmetric(x, dt, all, N, k, lambda, sel);
        if (n_sel < 0) { free(all); free(cls); free(sel); return -3; }
    } else {
        for (int64_t r = 0; r < k; ++r) sel[r] = all[r];
    }

    for (int b = 0; b < M + Mn; ++b) {
        out->vmin[b] = 0.0f; out->vmax[b] = 0.0f;
        out->qb[b] = ladder ? ladder[b < M ? b : b - M] : (uint8_t)min_bit(bit_set);   /* empty blocks keep this */
        out->count[b] = 0;
        if (out->e_int) out->e_int[b] = 0;
        if (out->e_exp) out->e_exp[b] = 0;
        if (out->s_int) for (int q = 0; q < 17; ++q) out->s_int[(size_t)b * 17 + q] = 0;
    }

    for (int s = 0; s < 2; ++s) { /* s = 0: positive class, s = 1: negative class */
        /* kept non-zeros of this sign, still in (magnitude desc, index asc) order */
        uint32_t n = 0;
        for (int64_t r = 0; r < n_sel; ++r) {
            if (sel[r].key == 0) continue;                       /* exact zero: not sent */
            int neg = (int)(load_bits(x, dt, sel[r].idx) >> 31);
            if (neg == s) cls[n++] = sel[r];
        }
        if (s == 0) out->n_pos = n; else out->n_neg = n;

        /* MS: equal-cardinality blocks in rank order, remainder to the last */
        const int Ms = s ? Mn : M;
        uint32_t K = n / (uint32_t)Ms;
        uint32_t start = 0;
        for (int m = 0; m < Ms; ++m) {
            uint32_t cnt = (m < Ms - 1) ? K : n - start;
            int b = s * M + m;
            out->count[b] = cnt;
            if (cnt > 0) {
                for (uint32_t j = 0; j < cnt; ++j) out->block_of[cls[start + j].idx] = b;
                quantise_block(cls + start, cnt, bit_set, beta, ladder ? (int)ladder[m] : (ds ? -1 : 0), b, out);
            }
            start += cnt;
        }
    }
    free(all);
    free(cls);
    free(sel);
    return 0;
}

/* ---- packing ---------------------------------------------------------- */

typedef struct { uint32_t* words; uint64_t bitpos; } bitw_t;

static void put_bits(bitw_t* bw, uint32_t v, int nbits) /* LSB first */
{
    for (int i = 0; i < nbits; ++i) {
        if ((v >> i) & 1u) bw->words[bw->bitpos >> 5] |= 1u << (bw->bitpos & 31);
        ++bw->bitpos;
    }
}

static uint32_t get_bits(const uint32_t* words, uint64_t bitpos, int nbits)
{
    uint32_t v = 0;
    for (int i = 0; i < nbits; ++i, ++bitpos)
        v |= ((words[bitpos >> 5] >> (bitpos & 31)) & 1u) << i;
    return v;
}

/* Pack one analysed row into `words` (zero-filled by the caller); returns the
 * number of 32-bit words used. */
static uint64_t pack_row(const row_result* rr, int64_t N, int B2, int w, uint32_t* words,
                         uint32_t* scratch_idx /* [n_pos+n_neg] */)
{
    /* element indices in stream order: block by block, ascending inside
     * (one ascending sweep appends each kept index to its block's list) */
    uint32_t n = 0;
    uint32_t* fill = (uint32_t*)malloc(sizeof(uint32_t) * (size_t)B2);
    for (int b = 0; b < B2; ++b) { fill[b] = n; n += rr->count[b]; }
    for (int64_t i = 0; i < N; ++i)
        if (rr->block_of[i] >= 0) scratch_idx[fill[rr->block_of[i]]++] = (uint32_t)i;
    free(fill);
    bitw_t bw = { words, 0 };
    for (uint32_t j = 0; j < n; ++j) put_bits(&bw, scratch_idx[j], w);
    for (uint32_t j = 0; j < n; ++j) {
        uint32_t i = scratch_idx[j];
        put_bits(&bw, rr->code_of[i], rr->qb[rr->block_of[i]] & 0x7F);
    }
    return (bw.bitpos + 31) / 32;
}

/* Sec. 3.2 step 3 for a two-dimensional instance: every block as CSR(values, columns, row pointers).
 * The row pointers of a block are the exclusive scan of its per-row entry counts. */
static uint64_t pack_row_csr(const row_result* rr, int64_t n_rows, int64_t n_cols, int B2, int wp, int wc,
                             uint32_t* words, uint32_t* scratch_idx /* [n_pos+n_neg] */)
{
    const int64_t T = n_rows * n_cols;
    uint32_t n = 0;
    uint32_t* fill = (uint32_t*)malloc(sizeof(uint32_t) * (size_t)B2);
    uint32_t* start = (uint32_t*)malloc(sizeof(uint32_t) * (size_t)(B2 + 1));
    for (int b = 0; b < B2; ++b) { fill[b] = n; start[b] = n; n += rr->count[b]; }
    start[B2] = n;
    for (int64_t i = 0; i < T; ++i)                      /* row-major sweep: CSR order inside every block */
        if (rr->block_of[i] >= 0) scratch_idx[fill[rr->block_of[i]]++] = (uint32_t)i;
    free(fill);
    bitw_t bw = { words, 0 };
    uint32_t* per_row = (uint32_t*)malloc(sizeof(uint32_t) * (size_t)n_rows);
    for (int b = 0; b < B2; ++b) {                       /* r: row pointers */
        memset(per_row, 0, sizeof(uint32_t) * (size_t)n_rows);
        for (uint32_t j = start[b]; j < start[b + 1]; ++j) per_row[scratch_idx[j] / (uint32_t)n_cols]++;
        uint32_t acc = 0;
        for (int64_t row = 0; row < n_rows; ++row) { put_bits(&bw, acc, wp); acc += per_row[row]; }
        put_bits(&bw, acc, wp);
    }
    free(per_row);
    free(start);
    for (uint32_t j = 0; j < n; ++j) put_bits(&bw, scratch_idx[j] % (uint32_t)n_cols, wc);     /* c: columns */
    for (uint32_t j = 0; j < n; ++j) {                                                       /* v: codes */
        uint32_t i = scratch_idx[j];
        put_bits(&bw, rr->code_of[i], rr->qb[rr->block_of[i]] & 0x7F);
    }
    return (bw.bitpos + 31) / 32;
}

/* ---- meta accessors ---------------------------------------------------- */

static void put_u32(uint8_t* p, uint32_t v) { memcpy(p, &v, 4); }
static void put_u64(uint8_t* p, uint64_t v) { memcpy(p, &v, 8); }
static uint32_t get_u32(const uint8_t* p) { uint32_t v; memcpy(&v, p, 4); return v; }
static uint64_t get_u64(const uint8_t* p) { uint64_t v; memcpy(&v, p, 8); return v; }

static size_t off_rowoff(int64_t R, int B2) { (void)R; (void)B2; return REF_HDR; }
static size_t off_npos(int64_t R, int B2)   { (void)B2; return REF_HDR + 8 * (size_t)R; }
static size_t off_nneg(int64_t R, int B2)   { (void)B2; return REF_HDR + 12 * (size_t)R; }
static size_t off_vmin(int64_t R, int B2)   { (void)B2; return REF_HDR + 16 * (size_t)R; }
static size_t off_vmax(int64_t R, int B2)   { return REF_HDR + 16 * (size_t)R + 4 * (size_t)R * B2; }
static size_t off_q(int64_t R, int B2)      { return REF_HDR + 16 * (size_t)R + 8 * (size_t)R * B2; }

static void row_result_alloc(row_result* rr, int64_t N, int B2, int with_sums)
{
    memset(rr, 0, sizeof(*rr));
    rr->block_of = (int32_t*)malloc(sizeof(int32_t) * (size_t)N);
    rr->code_of = (uint32_t*)malloc(sizeof(uint32_t) * (size_t)N);
    rr->vmin = (float*)malloc(sizeof(float) * (size_t)B2);
    rr->vmax = (float*)malloc(sizeof(float) * (size_t)B2);
    rr->qb = (uint8_t*)malloc((size_t)B2);
    rr->count = (uint32_t*)malloc(sizeof(uint32_t) * (size_t)B2);
    if (with_sums) {
        rr->s_int = (uint64_t*)malloc(sizeof(uint64_t) * 17 * (size_t)B2);
        rr->e_int = (uint64_t*)malloc(sizeof(uint64_t) * (size_t)B2);
        rr->e_exp = (int32_t*)malloc(sizeof(int32_t) * (size_t)B2);
    }
}

static void row_result_free(row_result* rr)
{
    free(rr->block_of); free(rr->code_of); free(rr->vmin); free(rr->vmax);
    free(rr->qb); free(rr->count); free(rr->s_int); free(rr->e_int); free(rr->e_exp);
}

/* ---- public: encode ---------------------------------------------------- */

/* csr_cols > 0: two-dimensional instances of (N / csr_cols) x csr_cols, blocks stored as CSR triples */
static int encode_common(const void* x, int dt, int64_t R, int64_t N, double keep, int M, int Mn,
                         uint32_t bit_set, double beta, const uint8_t* ladder, int ds, float lambda,
                         void* stream, void* meta, int n_threads, int64_t csr_cols)
{
    int rc = check_args(dt, R, N, keep, M, bit_set);
    if (rc) return rc;
    if (Mn < 1 || Mn > 128) return -1;
    const int B2 = M + Mn;
    if (!x || !stream || !meta) return -1;
    if (!(beta >= 0.0)) return -1;

    const int64_t k = keep_count(keep, N);
    const int64_t csr_rows = csr_cols > 0 ? N / csr_cols : 0;
    const int w = csr_cols > 0 ? index_bits(csr_cols) : index_bits(N);
    const int wp = bits_for_count(k);
    const size_t esz = dt == SLICER_REF_F32 ? 4 : 2;
    const uint64_t cap_words = (((csr_cols > 0 ? (uint64_t)B2 * (uint64_t)(csr_rows + 1) * (uint64_t)wp : 0)
                                 + (uint64_t)k * (uint64_t)(w + max_bit(bit_set))) + 31) / 32;
    uint8_t* mt = (uint8_t*)meta;
    memset(mt, 0, meta_size(R, B2));

    /* per-row segments go to private buffers first; offsets need all rows */
    uint32_t** seg = (uint32_t**)calloc((size_t)R, sizeof(uint32_t*));
    uint64_t* seg_words = (uint64_t*)calloc((size_t)R, sizeof(uint64_t));
    int fail = 0;
    if (n_threads < 1) n_threads = 1;

#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1) num_threads(n_threads)
#endif
    for (int64_t r = 0; r < R; ++r) {
        row_result rr;
        row_result_alloc(&rr, N, B2, 0);
        uint32_t* idxbuf = (uint32_t*)malloc(sizeof(uint32_t) * (size_t)(k > 0 ? k : 1));
        seg[r] = (uint32_t*)calloc((size_t)(cap_words > 0 ? cap_words : 1), 4);
        const void* xr = (const char*)x + (size_t)r * (size_t)N * esz;
        if (analyze_row(xr, dt, N, k, M, Mn, bit_set, beta, ladder, ds, lambda, &rr) != 0) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            fail = 1;
        } else {
            seg_words[r] = csr_cols > 0 ? pack_row_csr(&rr, csr_rows, csr_cols, B2, wp, w, seg[r], idxbuf)
                                        : pack_row(&rr, N, B2, w, seg[r], idxbuf);
            put_u32(mt + off_npos(R, B2) + 4 * (size_t)r, rr.n_pos);
            put_u32(mt + off_nneg(R, B2) + 4 * (size_t)r, rr.n_neg);
            for (int b = 0; b < B2; ++b) {
                size_t e = (size_t)r * B2 + b;
                memcpy(mt + off_vmin(R, B2) + 4 * e, &rr.vmin[b], 4);
                memcpy(mt + off_vmax(R, B2) + 4 * e, &rr.vmax[b], 4);
                mt[off_q(R, B2) + e] = rr.qb[b];
            }
        }
        free(idxbuf);
        row_result_free(&rr);
    }

    uint64_t total = 0;
    uint32_t* out = (uint32_t*)stream;
    for (int64_t r = 0; r < R; ++r) {
        put_u64(mt + off_rowoff(R, B2) + 8 * (size_t)r, total);
        if (seg[r]) memcpy(out + total, seg[r], (size_t)seg_words[r] * 4);
        total += seg_words[r];
        free(seg[r]);
    }
    free(seg);
    free(seg_words);

    put_u32(mt + 0, REF_MAGIC);
    put_u32(mt + 4, REF_VERSION);
    put_u32(mt + 8, (uint32_t)dt);
    put_u32(mt + 12, (uint32_t)M);
    put_u64(mt + 16, (uint64_t)R);
    put_u64(mt + 24, (uint64_t)N);
    put_u64(mt + 32, (uint64_t)k);
    put_u32(mt + 40, bit_set);
    put_u32(mt + 44, (uint32_t)w);
    put_u64(mt + 48, total);
    put_u32(mt + 56, Mn != M ? (uint32_t)Mn : 0u);   /* 0: M(-) = M(+) */
    put_u32(mt + 60, (uint32_t)csr_cols);            /* 0: flat indices */
    return fail ? -3 : 0;
}

int slicer_ref_encode(const void* x, int dt, int64_t R, int64_t N, double keep, int M,
                      uint32_t bit_set, double beta, void* stream, void* meta, int n_threads)
{
    return encode_common(x, dt, R, N, keep, M, M, bit_set, beta, NULL, 0, -1.0f, stream, meta, n_threads, 0);
}

int slicer_ref_encode_pn(const void* x, int dt, int64_t R, int64_t N, double keep, int M, int Mn,
                         uint32_t bit_set, double beta, void* stream, void* meta, int n_threads)
{
    return encode_common(x, dt, R, N, keep, M, Mn, bit_set, beta, NULL, 0, -1.0f, stream, meta, n_threads, 0);
}

/* Sec. 3.2 with X of shape n_rows x n_cols per instance: CSR triples per block */
int slicer_ref_encode_csr(const void* x, int dt, int64_t R, int64_t n_rows, int64_t n_cols, double keep, int M,
                          uint32_t bit_set, double beta, void* stream, void* meta, int n_threads)
{
    if (n_rows <= 0 || n_cols <= 0 || n_rows > ((int64_t)1 << 31) / n_cols) return -1;
    return encode_common(x, dt, R, n_rows * n_cols, keep, M, M, bit_set, beta, NULL, 0, -1.0f, stream, meta, n_threads, n_cols);
}

/* Sec. 3.1 with an asymmetry factor: lambda in [0, 1), rounded to fp32 once */
int slicer_ref_encode_atkf(const void* x, int dt, int64_t R, int64_t N, double keep, double lambda, int M, int Mn,
                           uint32_t bit_set, double beta, void* stream, void* meta, int n_threads)
{
    if (!(lambda >= 0.0 && lambda < 1.0)) return -1;
    return encode_common(x, dt, R, N, keep, M, Mn, bit_set, beta, NULL, 0, (float)lambda, stream, meta, n_threads, 0);
}

/* set of the ladder's bitwidths; 0 if an entry is outside 1..16 */
static uint32_t ladder_bit_set(const uint8_t* ladder, int M)
{
    uint32_t bs = 0;
    for (int m = 0; m < M; ++m) {
        if (ladder[m] < 1 || ladder[m] > 16) return 0;
        bs |= 1u << ladder[m];
    }
    return bs;
}

int slicer_ref_encode_ladder(const void* x, int dt, int64_t R, int64_t N, double keep, int M,
                             const uint8_t* ladder, void* stream, void* meta, int n_threads)
{
    if (!ladder || M < 1 || M > 64) return -1;
    uint32_t bs = ladder_bit_set(ladder, M);
    if (!bs) return -1;
    return encode_common(x, dt, R, N, keep, M, M, bs, 0.0, ladder, 0, -1.0f, stream, meta, n_threads, 0);
}

int slicer_ref_encode_ds(const void* x, int dt, int64_t R, int64_t N, double keep, int M,
                         uint32_t bit_set, double delta, void* stream, void* meta, int n_threads)
{
    return encode_common(x, dt, R, N, keep, M, M, bit_set, delta, NULL, 1, -1.0f, stream, meta, n_threads, 0);
}

/* Sec. 3.3: value bits with every block at q_bit = max(bit_set), index bits, header bits.
 * Every row is taken to send its full k entries; the zero bits that pad a row's segment to
 * a whole word are counted with the header, so the three parts add up to the worst-case
 * size of stream + meta in bits. */
int slicer_ref_bound(int dt, int64_t R, int64_t N, double keep, int M, uint32_t bit_set,
                     uint64_t* value_bits, uint64_t* idx_bits, uint64_t* header_bits)
{
    int rc = check_args(dt, R, N, keep, M, bit_set);
    if (rc) return rc;
    const uint64_t k = (uint64_t)keep_count(keep, N);
    const uint64_t w = (uint64_t)index_bits(N), qb = (uint64_t)max_bit(bit_set);
    const uint64_t row_bits = k * (w + qb);
    const uint64_t pad = (32 - row_bits % 32) % 32;
    if (value_bits) *value_bits = (uint64_t)R * k * qb;
    if (idx_bits) *idx_bits = (uint64_t)R * k * w;
    if (header_bits) *header_bits = 8 * (uint64_t)meta_size(R, 2 * M) + (uint64_t)R * pad;
    return 0;
}

/* ---- public: decode (Eq. "dequnt") -------------------------------------- */

int slicer_ref_decode(const void* stream, const void* meta, void* y, int n_threads)
{
    if (!stream || !meta || !y) return -1;
    const uint8_t* mt = (const uint8_t*)meta;
    if (get_u32(mt) != REF_MAGIC || get_u32(mt + 4) != REF_VERSION) return -1;
    const int dt = (int)get_u32(mt + 8);
    const int M = (int)get_u32(mt + 12);
    const int Mn = get_u32(mt + 56) ? (int)get_u32(mt + 56) : M;      /* 0: M(-) = M(+) */
    const int B2 = M + Mn;
    const int64_t R = (int64_t)get_u64(mt + 16);
    const int64_t N = (int64_t)get_u64(mt + 24);
    const int w = (int)get_u32(mt + 44);
    const int64_t csr_cols = (int64_t)get_u32(mt + 60);                /* 0: flat indices */
    const int64_t csr_rows = csr_cols > 0 ? N / csr_cols : 0;
    const int wp = bits_for_count((int64_t)get_u64(mt + 32));
    const uint32_t* words = (const uint32_t*)stream;
    const size_t esz = dt == SLICER_REF_F32 ? 4 : 2;
    if (n_threads < 1) n_threads = 1;

    memset(y, 0, (size_t)R * (size_t)N * esz); /* zero-initialised tensor */

#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1) num_threads(n_threads)
#endif
    for (int64_t r = 0; r < R; ++r) {
        const uint32_t* rw = words + get_u64(mt + off_rowoff(R, B2) + 8 * (size_t)r);
        const uint32_t n_cls[2] = { get_u32(mt + off_npos(R, B2) + 4 * (size_t)r),
                                    get_u32(mt + off_nneg(R, B2) + 4 * (size_t)r) };
        const uint64_t n = (uint64_t)n_cls[0] + n_cls[1];
        const uint64_t ptr_bits = csr_cols > 0 ? (uint64_t)B2 * (uint64_t)(csr_rows + 1) * (uint64_t)wp : 0;
        uint64_t ppos = 0;               /* bit cursor in the row pointers of the current block */
        uint64_t ipos = ptr_bits;        /* bit cursor in the index (column) section */
        uint64_t cpos = ptr_bits + n * (uint64_t)w; /* bit cursor in the code section */
        for (int s = 0; s < 2; ++s) {
            const int Ms = s ? Mn : M;
            uint32_t K = n_cls[s] / (uint32_t)Ms, start = 0;
            for (int m = 0; m < Ms; ++m) {
                uint32_t cnt = (m < Ms - 1) ? K : n_cls[s] - start;
                start += cnt;
                size_t e = (size_t)r * B2 + (size_t)(s * M + m);
                float vmin, vmax;
                memcpy(&vmin, mt + off_vmin(R, B2) + 4 * e, 4);
                memcpy(&vmax, mt + off_vmax(R, B2) + 4 * e, 4);
                int q = mt[off_q(R, B2) + e] & 0x7F;
                float L = (float)((1u << q) - 1u);
                float o = (vmax - vmin) / L;
                int64_t trow = 0;        /* CSR: tensor row of the current entry */
                for (uint32_t j = 0; j < cnt; ++j) {
                    uint32_t idx = get_bits(rw, ipos, w); ipos += (uint64_t)w;
                    if (csr_cols > 0) {  /* entry j lies in the row whose pointer range holds j: r[trow] <= j < r[trow+1] */
                        while (trow + 1 < csr_rows && get_bits(rw, ppos + (uint64_t)(trow + 1) * wp, wp) <= j) ++trow;
                        idx = (uint32_t)(trow * csr_cols) + idx;
                    }
                    uint32_t c = get_bits(rw, cpos, q);   cpos += (uint64_t)q;
                    float prod = (float)c * o;   /* two roundings: no fused multiply-add */
                    float a = vmin + prod;
                    if (s) a = -a;
                    size_t at = (size_t)r * (size_t)N + idx;
                    if (dt == SLICER_REF_F32) memcpy((char*)y + 4 * at, &a, 4);
                    else { uint16_t h = float_to_bf16_rne(a); memcpy((char*)y + 2 * at, &h, 2); }
                }
                ppos += (uint64_t)(csr_rows + 1) * wp;
            }
        }
    }
    return 0;
}

/* ---- public: per-element view of one row -------------------------------- */

static int analyze_row_public(const void* x_row, int dt, int64_t N, double keep, float lambda, int M,
                              uint32_t bit_set, double beta, int32_t* block_of, uint32_t* code_of,
                              float* vmin, float* vmax, uint8_t* qb, uint64_t* s_int,
                              uint64_t* e_int, int32_t* e_exp)
{
    int rc = check_args(dt, 1, N, keep, M, bit_set);
    if (rc) return rc;
    if (!x_row || !(beta >= 0.0)) return -1;
    row_result rr;
    row_result_alloc(&rr, N, 2 * M, 1);
    rc = analyze_row(x_row, dt, N, keep_count(keep, N), M, M, bit_set, beta, NULL, 0, lambda, &rr);
    if (rc == 0) {
        if (block_of) memcpy(block_of, rr.block_of, sizeof(int32_t) * (size_t)N);
        if (code_of) memcpy(code_of, rr.code_of, sizeof(uint32_t) * (size_t)N);
        if (vmin) memcpy(vmin, rr.vmin, sizeof(float) * 2 * (size_t)M);
        if (vmax) memcpy(vmax, rr.vmax, sizeof(float) * 2 * (size_t)M);
        if (qb) memcpy(qb, rr.qb, 2 * (size_t)M);
        if (s_int) memcpy(s_int, rr.s_int, sizeof(uint64_t) * 17 * 2 * (size_t)M);
        if (e_int) memcpy(e_int, rr.e_int, sizeof(uint64_t) * 2 * (size_t)M);
        if (e_exp) memcpy(e_exp, rr.e_exp, sizeof(int32_t) * 2 * (size_t)M);
    }
    row_result_free(&rr);
    return rc;
}

int slicer_ref_analyze_row(const void* x_row, int dt, int64_t N, double keep, int M,
                           uint32_t bit_set, double beta, int32_t* block_of, uint32_t* code_of,
                           float* vmin, float* vmax, uint8_t* qb, uint64_t* s_int,
                           uint64_t* e_int, int32_t* e_exp)
{
    return analyze_row_public(x_row, dt, N, keep, -1.0f, M, bit_set, beta, block_of, code_of, vmin, vmax, qb, s_int, e_int, e_exp);
}

int slicer_ref_analyze_row_atkf(const void* x_row, int dt, int64_t N, double keep, double lambda, int M,
                                uint32_t bit_set, double beta, int32_t* block_of, uint32_t* code_of,
                                float* vmin, float* vmax, uint8_t* qb)
{
    if (!(lambda >= 0.0 && lambda < 1.0)) return -1;
    return analyze_row_public(x_row, dt, N, keep, (float)lambda, M, bit_set, beta, block_of, code_of, vmin, vmax, qb, NULL, NULL, NULL);
}
