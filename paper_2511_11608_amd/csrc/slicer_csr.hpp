// Two-dimensional instances (Sec. 3.2: an IF X of shape N x K; step 3: CSR(X_m) = (v_m, c_m, r_m)).
//
// ATKF and MS work on the flattened tensor, so the encoder proper is the flat one (whichever kernel
// family serves the shape); only the index encoding of the stream differs.  The flat encode writes its
// stream into the workspace, and two short kernels turn it into the CSR form:
//
//   csr_sizes   per instance: words of the CSR segment (closed form from the counts and bitwidths in
//               meta), and a copy of the flat segment's offset; the row-offset scan then runs on them;
//   csr_repack  one workgroup per window of 256 output words: the row pointers that fall into the window
//               (pointer j of block b = number of the block's entries in tensor rows before j: a
//               lower-bound search for j * n_cols in the block's ascending flat indices), the columns
//               (flat index mod n_cols) and the code bits (copied with the new bit offset), assembled
//               in LDS and written once.
//
// Segment of an instance: all row pointers (wp bits each), all columns (wc bits), all codes.
#pragma once

#include "slicer_encode_generic.hpp"

namespace slicer {

constexpr int kCsrWin = 256;          // output words per repack workgroup

struct CsrArgs {
    int64_t R, n_rows, n_cols, k;     // R instances of n_rows x n_cols
    int M, Mn, w, wc, wp, dt;         // w: bits of a flat index; wc: of a column; wp: of a row pointer
    u32 bit_set;
    int nwin;                         // windows per instance (worst-case segment length)
    const u32* flat;                  // the flat stream
    u64* flat_off;                    // [R] offsets of the flat segments
    u64* row_words;                   // [R] words of the CSR segments
    const u64* row_off_local;         // [R] from the row-offset scan
    const u64* chunk_tot;
    u32* stream;
    void* meta;
    MetaView mv;
};

__device__ inline u32 csr_block_count(u32 n_cls, int Ms, int m)
{
    const u32 K = n_cls / (u32)Ms;
    return m < Ms - 1 ? K : n_cls - K * (u32)(Ms - 1);
}

__global__ __launch_bounds__(256) void csr_sizes_kernel(CsrArgs a)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= a.R) return;
    const int B2 = a.M + a.Mn;
    const u32 n_cls[2] = { a.mv.n_pos[i], a.mv.n_neg[i] };
    u64 bits = (u64)B2 * (u64)(a.n_rows + 1) * (u64)a.wp + (u64)(n_cls[0] + n_cls[1]) * (u64)a.wc;
    for (int b = 0; b < B2; ++b) {
        const int s = b >= a.M ? 1 : 0;
        bits += (u64)csr_block_count(n_cls[s], s ? a.Mn : a.M, b - s * a.M) * (u64)(a.mv.q[(size_t)i * B2 + b] & 0x7Fu);
    }
    a.row_words[i] = (bits + 31) >> 5;
    a.flat_off[i] = a.mv.row_off[i];
}

__global__ __launch_bounds__(256) void csr_repack_kernel(CsrArgs a)
{
    __shared__ u32 stage[kCsrWin];
    __shared__ u32 bstart[kMaxB2 + 1];
    __shared__ u64 cstart[kMaxB2 + 1];        // first code bit of the block in the flat segment's code section
    __shared__ u32 qv[kMaxB2];
    __shared__ u64 s_off[2];
    const int tid = threadIdx.x;
    const u32 lane = lane_id();
    const int64_t inst = (int64_t)blockIdx.x / a.nwin;
    const int win = (int)((int64_t)blockIdx.x % a.nwin);
    const int B2 = a.M + a.Mn;
    // offset of the instance's segment: totals of the preceding scan chunks + offset inside its chunk
    if (tid < kWave) {
        const int64_t my_chunk = inst / kScanRows, n_chunks = (a.R + kScanRows - 1) / kScanRows;
        const bool want_total = blockIdx.x == 0;
        u64 before = 0, total = 0;
        for (int64_t j = lane; j < (want_total ? n_chunks : my_chunk); j += kWave) {
            const u64 t = a.chunk_tot[j];
            total += t;
            if (j < my_chunk) before += t;
        }
#pragma unroll
        for (int d = kWave / 2; d > 0; d >>= 1) { before += __shfl_xor(before, d); total += __shfl_xor(total, d); }
        if (lane == 0) { s_off[0] = before + a.row_off_local[inst]; s_off[1] = total; }
        if (want_total) {                     // header: the flat encode wrote it; index width, n_cols and the total change
            __builtin_amdgcn_wave_barrier();
            if (lane == 0) {
                u32* h32 = (u32*)a.meta;
                u64* h64 = (u64*)a.meta;
                h32[11] = (u32)a.wc; h32[15] = (u32)a.n_cols; h64[6] = total;
            }
        }
    }
    const u32 n_cls[2] = { a.mv.n_pos[inst], a.mv.n_neg[inst] };
    const u32 n = n_cls[0] + n_cls[1];
    if (tid < B2) {
        const int s = tid >= a.M ? 1 : 0, m = tid - s * a.M;
        bstart[tid] = (s ? n_cls[0] : 0u) + (u32)m * (n_cls[s] / (u32)(s ? a.Mn : a.M));
        qv[tid] = a.mv.q[(size_t)inst * B2 + tid] & 0x7Fu;
    }
    if (tid == 0) bstart[B2] = n;
    for (int i = tid; i < kCsrWin; i += 256) stage[i] = 0;
    __syncthreads();
    if (tid == 0) {
        u64 acc = 0;
        for (int b = 0; b < B2; ++b) { cstart[b] = acc; acc += (u64)(bstart[b + 1] - bstart[b]) * (u64)qv[b]; }
        cstart[B2] = acc;
    }
    __syncthreads();
    const u64 off = s_off[0];
    if (win == 0 && tid == 0) a.mv.row_off[inst] = off;
    const u64 words = a.row_words[inst];
    const u64 w0 = (u64)win * kCsrWin;
    if (w0 >= words) return;                              // (the whole workgroup: no barrier below is skipped by some)
    const u64 w1 = w0 + kCsrWin < words ? w0 + kCsrWin : words;
    const u64 lo = w0 << 5, hi = w1 << 5;
    const u32* __restrict__ fseg = a.flat + a.flat_off[inst];
    const int w = a.w, wc = a.wc, wp = a.wp;
    const u64 n_ptr = (u64)B2 * (u64)(a.n_rows + 1);
    const u64 ptr_bits = n_ptr * (u64)wp;
    const u64 col_end = ptr_bits + (u64)n * (u64)wc;
    const u64 code_end = col_end + cstart[B2];
    // (1) row pointers
    if (lo < ptr_bits) {
        const u64 f0 = lo / (u64)wp;
        u64 f1 = (hi + (u64)wp - 1) / (u64)wp;
        if (f1 > n_ptr) f1 = n_ptr;
        for (u64 f = f0 + tid; f < f1; f += 256) {
            const u32 b = (u32)(f / (u64)(a.n_rows + 1));
            const u64 target = (f % (u64)(a.n_rows + 1)) * (u64)a.n_cols;
            u32 l = bstart[b], h = bstart[b + 1];
            while (l < h) {
                const u32 mid = (l + h) >> 1;
                if ((u64)read_bits(fseg, (u64)mid * (u64)w, w) < target) l = mid + 1; else h = mid;
            }
            stage_or_bits(stage, lo, hi, f * (u64)wp, l - bstart[b], wp);
        }
    }
    // (2) columns
    if (lo < col_end && hi > ptr_bits) {
        const u64 e0 = lo > ptr_bits ? (lo - ptr_bits) / (u64)wc : 0;
        u64 e1 = (hi - ptr_bits + (u64)wc - 1) / (u64)wc;
        if (e1 > n) e1 = n;
        for (u64 e = e0 + tid; e < e1; e += 256) {
            const u32 idx = read_bits(fseg, e * (u64)w, w);
            stage_or_bits(stage, lo, hi, ptr_bits + e * (u64)wc, (u32)((u64)idx % (u64)a.n_cols), wc);
        }
    }
    // (3) code bits: the flat segment's code section, moved to its new bit offset, 32 bits at most per step
    if (hi > col_end && lo < code_end) {
        for (u64 wi = w0 + tid; wi < w1; wi += 256) {
            const u64 b0 = wi << 5;
            const u64 o_lo = b0 > col_end ? b0 : col_end;
            u64 o_hi = b0 + 32 < code_end ? b0 + 32 : code_end;
            if (o_hi > o_lo) {
                const int nb = (int)(o_hi - o_lo);
                const u32 v = read_bits(fseg, (u64)n * (u64)w + (o_lo - col_end), nb);
                stage_or_bits(stage, lo, hi, o_lo, v, nb);
            }
        }
    }
    __syncthreads();
    u32* __restrict__ dst = a.stream + off + w0;
    for (int i = tid; i < (int)(w1 - w0); i += 256) dst[i] = stage[i];
}

}  // namespace slicer
