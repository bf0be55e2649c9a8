// Decoder (Eq. "dequnt"): de-quantise every block and scatter it into a zero tensor.
// A workgroup owns a contiguous chunk of one output row: it builds the chunk in
// LDS (zeros, then the decoded entries whose index falls in the chunk) and writes
// it out once, coalesced, so every output byte goes to HBM exactly once.
#pragma once

#include "slicer_common.hpp"

namespace slicer {

constexpr int kDecChunkBytes = 16384;   // output bytes per workgroup of the long-row decoder (its LDS image)

struct DecArgs {
    const u32* stream;
    void* y;
    int64_t R, N;
    int M, Mn, w;             // blocks of the positive / negative class
    int chunks_per_row;
    MetaView mv;
    const u64* total_words;   // header field
    int stage_words;          // short rows: words of LDS per wave for the row's stream segment
    int xcd_map;              // long rows: all chunks of a row run on one XCD (grid = kXcds * ceil(R / kXcds) * chunks_per_row)
};

template <int DT, int BLOCK>
__global__ __launch_bounds__(BLOCK) void dec_kernel(DecArgs a)
{
    typedef typename Elem<DT>::raw_t raw_t;
    constexpr int kDecChunk = kDecChunkBytes / (int)sizeof(raw_t);
    __shared__ raw_t tile[kDecChunk];
    __shared__ float vminf[kMaxB2], stepf[kMaxB2];
    __shared__ int qv[kMaxB2];
    __shared__ u32 istart[kMaxB2 + 1];     // first element of the block in stream order
    __shared__ u64 cstart[kMaxB2 + 1];     // first code bit of the block
    __shared__ u64 cbits[kMaxB2];          // code bits of the block
    __shared__ u32 act_lo[kMaxB2];         // first element of the block that lands in this chunk
    __shared__ u32 s_hi[kMaxB2];           // first element of the block beyond this chunk
    __shared__ u32 pre[kMaxB2 + 1];        // prefix of per-block counts landing in this chunk

    const int tid = threadIdx.x;
    // Workgroups are dealt to the XCDs round-robin and every XCD has its own L2.  The chunks of a
    // row all search the row's index lists, so with enough rows to go round, row r is decoded on
    // XCD r % 8 only and its stream segment is fetched into one L2 instead of eight.
    int64_t r, ch;
    if (a.xcd_map) {
        const int64_t j = (int64_t)blockIdx.x / kXcds;
        r = (j / a.chunks_per_row) * kXcds + (int64_t)blockIdx.x % kXcds;
        ch = j % a.chunks_per_row;
        if (r >= a.R) return;                       // the whole workgroup: no barrier is skipped
    } else {
        r = blockIdx.x / a.chunks_per_row;
        ch = blockIdx.x % a.chunks_per_row;
    }
    const int64_t c0 = ch * kDecChunk;
    const int64_t c1 = c0 + kDecChunk < a.N ? c0 + kDecChunk : a.N;
    const int len = (int)(c1 - c0);
    const int M = a.M, B2 = a.M + a.Mn, w = a.w;
    const u32* __restrict__ rw = a.stream + a.mv.row_off[r];
    u32 n_cls[2] = { a.mv.n_pos[r], a.mv.n_neg[r] };
    if ((u64)n_cls[0] + n_cls[1] > (u64)a.N) n_cls[0] = n_cls[1] = 0;   // not a valid row: write zeros
    const u64 n = (u64)n_cls[0] + n_cls[1];

    // block sizes in closed form (K, ..., K, K + remainder per class); every block's thread
    // then sums the code bits of the blocks before it
    for (int b = tid; b < B2; b += BLOCK) {
        size_t mi = (size_t)r * (size_t)B2 + (size_t)b;
        int q = a.mv.q[mi] & 0x7F;
        float vmin = a.mv.vmin[mi], vmax = a.mv.vmax[mi];
        float L = (float)((1u << q) - 1u);
        qv[b] = q;
        vminf[b] = vmin;
        stepf[b] = (vmax - vmin) / L;
        const int s = b >= M ? 1 : 0, m = b - s * M, Ms = s ? a.Mn : M;
        const u32 K = n_cls[s] / (u32)Ms;
        const u32 cnt = (m < Ms - 1) ? K : n_cls[s] - K * (u32)(Ms - 1);
        istart[b] = (s ? n_cls[0] : 0u) + (u32)m * K;
        cbits[b] = (u64)cnt * (u64)q;
    }
    if (tid == 0) istart[B2] = (u32)n;
    for (int i = tid; i < len; i += BLOCK) tile[i] = 0;
    __syncthreads();
    for (int b = tid; b <= B2; b += BLOCK) {
        u64 ca = n * (u64)w;
        for (int i = 0; i < b; ++i) ca += cbits[i];
        cstart[b] = ca;
    }
    __syncthreads();

    // Entries of each block that land in [c0, c1): indices ascend inside a block, so both ends
    // are lower bounds.  Every probe is a dependent global load: G lanes share one search and
    // probe G points of the interval at once (G + 1 parts per step instead of two).
    if (a.chunks_per_row > 1) {
        int G = BLOCK / (2 * B2);                  // lanes per (block, end); a power of two that divides the wavefront
        G = G >= 16 ? 16 : G >= 8 ? 8 : G >= 4 ? 4 : G >= 2 ? 2 : 1;
        const u32 lane = lane_id();
        const u32 gl = lane & (u32)(G - 1), gbase = lane - gl;
        const u64 gmask = (G == 64 ? ~0ull : ((1ull << G) - 1ull)) << gbase;
        for (int unit0 = 0; unit0 < 2 * B2; unit0 += BLOCK / G) {
            const int unit = unit0 + tid / G;
            const bool on = unit < 2 * B2;
            const int b = on ? unit >> 1 : 0;
            const int64_t target = (unit & 1) ? c1 : c0;
            const u32 first = istart[b], cnt = istart[b + 1] - first;
            u32 l = 0, h = on ? cnt : 0;           // first j with idx >= target
            while (__any(l < h)) {
                // probe i < G sits at l + floor(span * (i + 1) / (G + 1)): ascending, all below h
                const u32 span = h - l, Gp = (u32)G + 1u;
                const u32 qd = span / Gp, rm = span - qd * Gp;
                auto point = [&](u32 m) -> u32 { return l + qd * m + udiv16(rm * m, Gp); };   // l + floor(span * m / Gp)
                bool below = false;
                if (l < h) below = (int64_t)read_bits(rw, (u64)(first + point(gl + 1u)) * w, w) < target;
                const u64 bal = __ballot(below) & gmask;
                if (l < h) {
                    const u32 t = (u32)__popcll(bal);          // probes below the target (a prefix of them)
                    const u32 nl = t ? point(t) + 1u : l;      // one past probe t - 1
                    const u32 nh = t < (u32)G ? point(t + 1u) : h;   // probe t
                    l = nl; h = nh;
                }
            }
            if (on && gl == 0) { if (unit & 1) s_hi[b] = l; else act_lo[b] = l; }
        }
        __syncthreads();
        for (int b = tid; b < B2; b += BLOCK) pre[b + 1] = s_hi[b] - act_lo[b];
    } else {
        for (int b = tid; b < B2; b += BLOCK) { act_lo[b] = 0; pre[b + 1] = istart[b + 1] - istart[b]; }
    }
    __syncthreads();
    if (tid == 0) {
        u32 acc = 0;
        pre[0] = 0;
        for (int b = 0; b < B2; ++b) { acc += pre[b + 1]; pre[b + 1] = acc; }
    }
    __syncthreads();

    const u32 total = pre[B2];
    for (u32 t0 = tid; t0 < total; t0 += 4 * BLOCK) {      // four entries per thread with all their loads in flight
        int bb[4];
        u32 idx4[4], c4[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const u32 t = t0 + (u32)u * BLOCK;
            bb[u] = -1; idx4[u] = 0; c4[u] = 0;
            if (t < total) {
                int lo = 0, hi = B2 - 1;               // block b with pre[b] <= t < pre[b+1]
                while (lo < hi) { int mid = (lo + hi) >> 1; if (pre[mid + 1] <= t) lo = mid + 1; else hi = mid; }
                const int b = lo;
                const u32 j = act_lo[b] + (t - pre[b]);
                bb[u] = b;
                idx4[u] = read_bits(rw, (u64)(istart[b] + j) * w, w);
                c4[u] = read_bits(rw, cstart[b] + (u64)j * (u64)qv[b], qv[b]);
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (bb[u] < 0) continue;
            const int b = bb[u];
            float val = __fadd_rn(vminf[b], __fmul_rn((float)c4[u], stepf[b]));   // two roundings, never fused
            if (b >= M) val = -val;
            const int64_t rel = (int64_t)idx4[u] - c0;
            if (rel >= 0 && rel < len) {
                if (DT == 0) tile[rel] = (raw_t)__float_as_uint(val);
                else tile[rel] = (raw_t)f32_to_bf16_rne(val);
            }
        }
    }
    __syncthreads();

    const size_t g0 = (size_t)r * (size_t)a.N + (size_t)c0;
    if (DT == 0) {
        u32* __restrict__ out = (u32*)a.y + g0;
        for (int i = tid; i < len; i += BLOCK) __builtin_nontemporal_store((u32)tile[i], out + i);
    } else {
        uint16_t* __restrict__ out = (uint16_t*)a.y + g0;
        const int head = (int)(g0 & 1);
        if (head && tid == 0) out[0] = (uint16_t)tile[0];
        const int npair = (len - head) >> 1;
        u32* __restrict__ out2 = (u32*)(out + head);
        for (int t = tid; t < npair; t += BLOCK)
            __builtin_nontemporal_store((u32)tile[head + 2 * t] | ((u32)tile[head + 2 * t + 1] << 16), out2 + t);
        if (((len - head) & 1) && tid == 0) out[len - 1] = (uint16_t)tile[len - 1];
    }
}

// ---- consistency of a (stream, meta) pair that did not come from this process --------------
// One thread per row: the row's counts, bitwidths and segment must be what an encoder
// produces (offsets are the exclusive scan of the exact word counts), and the whole stream
// must fit the words the caller holds.  Any violation sets a bit of *flag; nothing is decoded.
struct CheckArgs {
    const void* meta;
    int64_t R, N;
    int M, Mn, w, dt;
    u64 avail_words;
    u32* flag;          // device word, zeroed by the same launch sequence
    int64_t csr_cols;   // > 0: two-dimensional instances of (N / csr_cols) x csr_cols, w = bits of a column
};

__global__ __launch_bounds__(64) void meta_flag_clear_kernel(u32* flag) { if (threadIdx.x == 0) *flag = 0u; }

__global__ __launch_bounds__(256) void meta_check_kernel(CheckArgs a)
{
    const int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const u32* h32 = (const u32*)a.meta;
    const u64* h64 = (const u64*)a.meta;
    const MetaView mv = meta_view(const_cast<void*>(a.meta), a.R, a.M + a.Mn);
    u32 bad = 0;
    const u64 total = h64[6];
    if (r == 0) {
        if (h32[0] != kMagic || h32[1] != kVersion) bad |= 1u;
        if (h32[14] != (a.Mn != a.M ? (u32)a.Mn : 0u) || h32[15] != (u32)a.csr_cols) bad |= 2u;
        if (h32[2] != (u32)a.dt || h32[3] != (u32)a.M || h64[2] != (u64)a.R || h64[3] != (u64)a.N || h32[11] != (u32)a.w) bad |= 2u;
        if (h64[4] > (u64)a.N || (h32[10] & ~0x1FFFEu) || h32[10] == 0u) bad |= 2u;
        if (total > a.avail_words || mv.row_off[0] != 0ull) bad |= 4u;
    }
    if (r < a.R) {
        const u64 n_pos = mv.n_pos[r], n_neg = mv.n_neg[r];
        if (n_pos + n_neg > h64[4] || n_pos + n_neg > (u64)a.N) {
            bad |= 8u;
        } else {
            u64 bits = (n_pos + n_neg) * (u64)a.w;
            if (a.csr_cols > 0) {                      // row pointers of every block: n_rows + 1 fields that hold 0..k
                int wp = 1;
                while (wp < 32 && (1ull << wp) <= h64[4]) ++wp;
                bits += (u64)(a.M + a.Mn) * (u64)(a.N / a.csr_cols + 1) * (u64)wp;
            }
            for (int b = 0; b < a.M + a.Mn; ++b) {
                const u32 q = mv.q[(size_t)r * (a.M + a.Mn) + b] & 0x7Fu;
                if (q < 1u || q > 16u || !((h32[10] >> q) & 1u)) bad |= 16u;
                const int Ms = b < a.M ? a.M : a.Mn, m = b < a.M ? b : b - a.M;
                const u64 nc = b < a.M ? n_pos : n_neg, K = nc / (u64)Ms;
                const u64 cnt = m < Ms - 1 ? K : nc - K * (u64)(Ms - 1);
                bits += cnt * q;
            }
            const u64 off0 = mv.row_off[r];
            const u64 off1 = r + 1 < a.R ? mv.row_off[r + 1] : total;
            if (off1 < off0 || off1 - off0 != (bits + 31) >> 5 || off1 > total) bad |= 32u;
        }
    }
    if (bad) atomicOr(a.flag, bad);
}

// ---- two-dimensional instances: blocks stored as CSR triples (Sec. 3.2 step 3) ------------------
// One workgroup per tensor row of an instance.  The row pointers of every block give the block's
// entries that lie in this tensor row directly (no search); their columns and codes are read, the
// values de-quantised (Eq. "dequnt") and placed into an LDS image of the row (a piece of it when the
// row is longer than the image), which leaves with coalesced stores: every output element is
// written exactly once.
struct DecCsrArgs {
    const u32* stream;
    void* y;
    int64_t R, n_rows, n_cols;     // R instances of n_rows x n_cols
    int M, Mn, wc;
    int rows_per_wg;               // consecutive tensor rows a workgroup decodes (their elements fit the LDS image)
    int64_t groups;                // workgroups per instance = ceil(n_rows / rows_per_wg)
    MetaView mv;
    const u64* k_keep;             // header field k: fixes the width of a row pointer
};

constexpr int kCsrImage = 8192;    // elements of the LDS image
constexpr int kCsrRows = 16;       // tensor rows per workgroup at most

template <int DT>
__global__ __launch_bounds__(256) void dec_csr_kernel(DecCsrArgs a)
{
    typedef typename Elem<DT>::raw_t raw_t;
    __shared__ raw_t tile[kCsrImage];
    __shared__ float vminf[kMaxB2], stepf[kMaxB2];
    __shared__ int qv[kMaxB2];
    __shared__ u32 istart[kMaxB2 + 1], pre[kMaxB2 + 1];
    __shared__ u32 ptrs[kMaxB2][kCsrRows + 1];       // row pointers trow0 .. trow0 + nr of every block
    __shared__ u64 cstart[kMaxB2 + 1];
    const int tid = threadIdx.x;
    const int64_t inst = (int64_t)blockIdx.x / a.groups;
    const int64_t trow0 = ((int64_t)blockIdx.x % a.groups) * a.rows_per_wg;
    const int nr = (int)(a.n_rows - trow0 < a.rows_per_wg ? a.n_rows - trow0 : a.rows_per_wg);
    const int M = a.M, B2 = a.M + a.Mn, wc = a.wc;
    const int64_t T = a.n_rows * a.n_cols;
    const u32* __restrict__ rw = a.stream + a.mv.row_off[inst];
    u32 n_cls[2] = { a.mv.n_pos[inst], a.mv.n_neg[inst] };
    if ((u64)n_cls[0] + n_cls[1] > (u64)T) n_cls[0] = n_cls[1] = 0;     // not a valid instance: write zeros
    const u32 n = n_cls[0] + n_cls[1];
    int wp = 1;
    {
        const u64 k = *a.k_keep;
        while (wp < 32 && (1ull << wp) <= k) ++wp;
    }
    const u64 ptr_bits = (u64)B2 * (u64)(a.n_rows + 1) * (u64)wp;
    if (tid < B2) {
        const int s = tid >= M ? 1 : 0, m = tid - s * M, Ms = s ? a.Mn : M;
        const size_t mi = (size_t)inst * (size_t)B2 + tid;
        const int q = a.mv.q[mi] & 0x7F;
        qv[tid] = q;
        const float vmin = a.mv.vmin[mi], vmax = a.mv.vmax[mi];
        vminf[tid] = vmin;
        stepf[tid] = __fdiv_rn(__fsub_rn(vmax, vmin), (float)((1u << q) - 1u));
        istart[tid] = (s ? n_cls[0] : 0u) + (u32)m * (n_cls[s] / (u32)Ms);
    }
    if (tid == 0) istart[B2] = n;
    // the blocks' shares of these tensor rows: entries [r[trow0], r[trow0 + nr]) of every block, row by row;
    // pointers are clamped to the block and made non-decreasing, so a forged stream cannot leave it
    for (int i = tid; i < B2 * (nr + 1); i += 256) {
        const int b = i / (nr + 1), j = i - b * (nr + 1);
        const int s = b >= M ? 1 : 0, m = b - s * M, Ms = s ? a.Mn : M;
        const u32 K = n_cls[s] / (u32)Ms;
        const u32 cnt = (m < Ms - 1) ? K : n_cls[s] - (u32)m * K;
        const u32 v = read_bits(rw, ((u64)b * (u64)(a.n_rows + 1) + (u64)(trow0 + j)) * (u64)wp, wp);
        ptrs[b][j] = v < cnt ? v : cnt;
    }
    __syncthreads();
    if (tid < B2) {
        u32 run = ptrs[tid][0];
        for (int j = 1; j <= nr; ++j) { run = ptrs[tid][j] > run ? ptrs[tid][j] : run; ptrs[tid][j] = run; }
    }
    __syncthreads();
    if (tid == 0) {
        u64 acc = ptr_bits + (u64)n * (u64)wc;
        u32 cnt = 0;
        for (int b = 0; b < B2; ++b) {
            cstart[b] = acc; acc += (u64)(istart[b + 1] - istart[b]) * (u64)qv[b];
            pre[b] = cnt; cnt += ptrs[b][nr] - ptrs[b][0];
        }
        pre[B2] = cnt;
    }
    __syncthreads();
    const u32 total = pre[B2];
    raw_t* __restrict__ yrow = (raw_t*)a.y + (size_t)inst * (size_t)T + (size_t)trow0 * (size_t)a.n_cols;
    // one piece of columns at a time (a single piece unless one tensor row is longer than the image)
    for (int64_t c0 = 0; c0 < a.n_cols; c0 += kCsrImage) {
        const int len = (int)(a.n_cols - c0 < kCsrImage ? a.n_cols - c0 : kCsrImage);
        const int img = nr * len;                                  // nr > 1 only when a whole row fits: len = n_cols then
        for (int i = tid; i < img; i += 256) tile[i] = (raw_t)0;
        __syncthreads();
        // all entries of these tensor rows at once: entry t belongs to the block whose range of the prefix
        // holds t, and to the tensor row whose pointer range holds its position in the block
        for (u32 t = (u32)tid; t < total; t += 256) {
            int bl = 0, bh = B2 - 1;                     // last block whose prefix is <= t
            while (bl < bh) {
                const int mid = (bl + bh + 1) >> 1;
                if (pre[mid] <= t) bl = mid; else bh = mid - 1;
            }
            const int b = bl;
            const u32 p = ptrs[b][0] + (t - pre[b]);
            int row = 0;
            while (row + 1 < nr && ptrs[b][row + 1] <= p) ++row;
            const int q = qv[b];
            const int64_t col = (int64_t)read_bits(rw, ptr_bits + (u64)(istart[b] + p) * (u64)wc, wc) - c0;
            if (col < 0 || col >= len) continue;
            const u32 c = read_bits(rw, cstart[b] + (u64)p * (u64)q, q);
            float v = __fadd_rn(vminf[b], __fmul_rn((float)c, stepf[b]));
            if (b >= M) v = -v;
            if (DT == 0) tile[row * len + (int)col] = (raw_t)__float_as_uint(v);
            else tile[row * len + (int)col] = (raw_t)f32_to_bf16_rne(v);
        }
        __syncthreads();
        if (nr > 1) {
            for (int i = tid; i < img; i += 256) yrow[i] = tile[i];           // whole rows, contiguous in y
        } else {
            for (int i = tid; i < len; i += 256) yrow[c0 + i] = tile[i];
        }
        __syncthreads();
    }
}

// ---- short rows: one wavefront per row, no workgroup barrier ---------------------------
// Lane b * lpb + sub (lpb = 64 / 2M lanes per block) decodes entries sub, sub + lpb, ... of
// block b, so neighbouring lanes read neighbouring bit fields; block offsets come from one
// scan across the lanes.  The row's stream segment is staged in LDS with one coalesced load
// (when it fits), the row is assembled in LDS and written with 16-byte stores.

// bit field from a word array in LDS; the array is padded by one readable word
__device__ inline u32 read_bits_lds(const u32* words, u32 bitpos, u32 nbits)
{
    const u32 wi = bitpos >> 5, sh = bitpos & 31u;
    const u64 two = (u64)words[wi] | ((u64)words[wi + 1] << 32);
    return (u32)(two >> sh) & ((1u << nbits) - 1u);       // nbits <= 16
}

template <int DT>
__global__ __launch_bounds__(kWave) void dec_small_kernel(DecArgs a)
{
    typedef typename Elem<DT>::raw_t raw_t;
    constexpr int ESZ = DT == 0 ? 4 : 2;
    extern __shared__ uint4 dec_smem[];
    const u32 lane = lane_id();
    const int wid = threadIdx.x / kWave;
    const int64_t r = xcd_row((int64_t)blockIdx.x, a.R);       // one wave per workgroup
    if (r >= a.R) return;
    const int N = (int)a.N, M = a.M, B2 = a.M + a.Mn, w = a.w;
    const int row_bytes = N * ESZ;                       // multiple of 16
    const int per_wave16 = row_bytes / 16 + (a.stage_words + 4) / 4;
    uint4* tile4 = dec_smem + (size_t)wid * per_wave16;
    raw_t* tile = (raw_t*)tile4;
    u32* sw = (u32*)(tile4 + row_bytes / 16);            // [stage_words + 1..4]

    const u64 off0 = a.mv.row_off[r];
    const u64 off1 = r + 1 < a.R ? a.mv.row_off[r + 1] : *a.total_words;
    const u32 n_pos = a.mv.n_pos[r], n_neg = a.mv.n_neg[r];
    const u32* __restrict__ rw = a.stream + off0;
    const u32 nw = (u32)(off1 - off0);
    const bool staged = off1 >= off0 && nw <= (u32)a.stage_words;
    if (staged) {
        for (u32 i = lane; i <= nw; i += kWave) sw[i] = i < nw ? rw[i] : 0u;
    }
    for (int i = lane; i < row_bytes / 16; i += kWave) tile4[i] = make_uint4(0, 0, 0, 0);

    const u32 lpb = (u32)kWave / (u32)B2;
    const u32 myb = lane / lpb, sub = lane - myb * lpb;
    u32 cnt = 0, q = 0;
    float vmin = 0.f, step = 0.f;
    if (myb < (u32)B2 && (u64)n_pos + n_neg <= (u64)N) {
        const u32 cls = myb >= (u32)M ? 1u : 0u, m = myb - cls * (u32)M;
        const u32 Ms = cls ? (u32)a.Mn : (u32)M;
        const u32 nc = cls ? n_neg : n_pos, K = nc / Ms;
        cnt = (m < Ms - 1u) ? K : nc - K * (Ms - 1u);
        const size_t mi = (size_t)r * (size_t)B2 + myb;
        q = a.mv.q[mi] & 0x7Fu;
        vmin = a.mv.vmin[mi];
        step = (a.mv.vmax[mi] - vmin) / (float)((1u << q) - 1u);
    }
    // first entry and first code bit of my block: scans over one lane per block
    const bool head = sub == 0;
    const u32 ie = wave_scan_dpp(head ? cnt : 0u) - (head ? cnt : 0u);
    const u32 ce = wave_scan_dpp(head ? cnt * q : 0u) - (head ? cnt * q : 0u);
    const u32 n = n_pos + n_neg;
    const u32 istart = (u32)__shfl((int)ie, (int)(myb * lpb));
    const u32 cstart = n * (u32)w + (u32)__shfl((int)ce, (int)(myb * lpb));
    wave_sync();

    if (staged && (u64)cstart + (u64)cnt * q <= (u64)nw * 32u) {
        for (u32 j = sub; j < cnt; j += lpb) {
            const u32 idx = read_bits_lds(sw, (istart + j) * (u32)w, (u32)w);
            const u32 c = read_bits_lds(sw, cstart + j * q, q);
            float val = __fadd_rn(vmin, __fmul_rn((float)c, step));      // two roundings, never fused
            if (myb >= (u32)M) val = -val;
            if (idx < (u32)N) tile[idx] = DT == 0 ? (raw_t)__float_as_uint(val) : (raw_t)f32_to_bf16_rne(val);
        }
    } else {
        for (u32 j = sub; j < cnt; j += lpb) {
            const u32 idx = read_bits(rw, (u64)(istart + j) * (u32)w, w);
            const u32 c = read_bits(rw, (u64)cstart + (u64)j * q, (int)q);
            float val = __fadd_rn(vmin, __fmul_rn((float)c, step));      // two roundings, never fused
            if (myb >= (u32)M) val = -val;
            if (idx < (u32)N) tile[idx] = DT == 0 ? (raw_t)__float_as_uint(val) : (raw_t)f32_to_bf16_rne(val);
        }
    }
    wave_sync();

    uint4* __restrict__ out = (uint4*)((char*)a.y + (size_t)r * (size_t)row_bytes);
    // the output is written once and not read back by this library: streaming (non-temporal) stores
    typedef u32 u32x4 __attribute__((ext_vector_type(4)));
    for (int i = lane; i < row_bytes / 16; i += kWave) {
        const uint4 t = tile4[i];
        u32x4 v4;
        v4.x = t.x; v4.y = t.y; v4.z = t.z; v4.w = t.w;
        __builtin_nontemporal_store(v4, (u32x4*)(out + i));       // one 16-byte store
    }
}

}  // namespace slicer
