// Encoder for long rows (tens of thousands of elements and more): every pass over a
// row is spread over many workgroups, the per-row state lives in the workspace, and
// the stages are separate launches on the caller's stream:
//
//   hist      per 8192-element chunk: 2048-bin histogram of the key's top 11 bits, stored
//             as "elements at or above the bin" (so sums over chunks are cumulative too)
//   select    per row: the bin B1 that holds overall rank k-1, the list offsets of the chunks
//   compact   per chunk: ordered compaction of everything at or above B1 into the row's
//             list L (ascending index), plus a 2-byte list of the entries' fine bins
//   bounds    per row: 8192-bin fine histogram of the list in LDS (three scans of the 2-byte
//             list; members of the few bins that matter are fetched from L), ranks of the bins; the comp
//             of overall rank k-1 (ATKF cut, Sec. 3.1) and of class ranks j*K-1 (block boundaries, Sec. 3.2), each resolved
//             inside its bin by pairwise comparison of the bin's members
//   blockcount / scatter   per 2048 list entries: block id, per-block counts, block min/max;
//             then a stable split by block id (ascending index inside a block)
//   abq / choose / pack    integer ABQ sums (Sec. 3.2.1) with 64-bit atomics, per-block
//             bitwidth, bit offsets, and the row's stream image, one window of words per workgroup
//
// Every stage is bound by the latency of its loads, not by their volume: a thread issues all
// its loads before it uses the first, and nothing is a chain of dependent global loads.
//
// comp = key << w | (2^w - 1 - index): larger comp = larger magnitude, then lower index.
// Rows that do not fit the lists (heavy ties, more zeros than dropped elements) are
// flagged and redone by the generic encoder inside the row-scan kernel.
#pragma once

#include "slicer_common.hpp"
#include "slicer_encode_generic.hpp"

namespace slicer {

constexpr int kLCH = 8192;          // elements per hist / compact workgroup
constexpr int kLBins = 2048;        // coarse bins: top 11 bits of the key
constexpr int kFB = 8192;           // fine bins of the list (kept in LDS by the bounds stage)
constexpr int kLCE = 2048;          // list entries per blockcount / scatter workgroup
constexpr int kPCH = 2048;          // block-ordered positions per abq workgroup
constexpr int kCutCap = 2048;       // members of the top-K cut bin
constexpr int kPackWords = 1024;    // stream words per pack workgroup
constexpr u64 kTop = 1ull << 63;

struct LargeArgs {
    const void* x;
    int64_t R, N, k;
    int M, Mn, w, nq;       // blocks of the positive / negative class
    int qlist[kMaxQ];
    double beta;
    u64 cap_words;
    int C, LC;              // chunks per row, list chunks per row
    int pack_words;         // stream words per pack workgroup in the index section (<= kPackWords)
    int pack_words_code;    // ... from the first word with code bits on (fields there are short: fewer words per workgroup)
    int nwin_idx;           // windows that lie in the index section for sure (worst case of its length)
    int nwin;               // pack workgroups (windows) per row
    u32* win_range;         // [R][nwin][2] block-ordered entries whose code field meets the window
    u32 capL;               // list capacity per row
    u32* ch_cum;            // [R][C][kLBins]  elements of the chunk at or above the bin
    u32* ch_off;            // [R][C]
    u64* L;                 // [R][capL]       class << 63 | key << 32 | index
    uint16_t* Lfine;        // [R][capL]       fine bin of the entry | class << 15 (capL is a multiple of 8)
    uint8_t* Lblk;          // [R][capL]       block of the entry, 255 = not kept
    u32* rowst;             // [R][16]  0 t_lo 1 sh 2 nL 3 n_pos 4 n_neg 5 K0 6 K1 7 ntg 8 nt0
    u64* thr;               // [R][1 + kMaxB2] thr[0] = cut comp, then boundaries (class on top)
    u32* blk_start;         // [R][B2 + 1]
    u32* blkcnt;            // [R][LC][B2]
    u32* vminb;             // [R][B2]  keys
    u32* vmaxb;
    u64* sums;              // [R][B2][nq + 1]
    u32* qsel;              // [R][B2]
    float* inv_sel;         // [R][B2]
    u64* code_off;          // [R][B2 + 1]
    u32* bo_idx;            // [R][k]
    u32* bo_val;            // [R][k]
    u64* row_words;
    u32* slots;
    u32* fallback;
    MetaView mv;
    Ladder lad;             // fixed multi-level mode
    int guard;              // 0: relative squared-error budget; 1: DS mismatch, greedy descent (beta = delta)
};

template <int DT>
__global__ __launch_bounds__(256) void lr_hist_kernel(LargeArgs a)
{
    typedef Elem<DT> E;
    typedef typename E::raw_t raw_t;
    constexpr int KS = E::kKeyBits - 11;
    __shared__ u32 h[kLBins];
    __shared__ u32 scr[256 / kWave + 1];
    const int tid = threadIdx.x, c = blockIdx.x;
    const int64_t r = blockIdx.y;
    const int B2 = a.M + a.Mn;
    for (int i = tid; i < kLBins; i += 256) h[i] = 0;
    // this launch also clears what later stages accumulate into
    if (c == 0) {
        for (int b = tid; b < B2; b += 256) { a.vminb[r * B2 + b] = 0xFFFFFFFFu; a.vmaxb[r * B2 + b] = 0; }
        for (int i = tid; i < B2 * (a.nq + 1); i += 256) a.sums[(size_t)r * B2 * (a.nq + 1) + i] = 0;
    }
    __syncthreads();
    // 16-byte loads (the row length is a multiple of a 16-byte chunk); exact zeros are not
    // counted: they are never sent, and skipping them keeps the hot bin of post-ReLU
    // features out of the LDS atomics (a row whose cut falls among them is redone generically)
    constexpr int EPC = DT == 0 ? 4 : 8;
    const int64_t i0 = (int64_t)c * kLCH;
    const uint4* __restrict__ x4 = (const uint4*)((const char*)a.x + ((size_t)r * (size_t)a.N + (size_t)i0) * sizeof(raw_t));
#pragma unroll
    for (int j = 0; j < kLCH / (256 * EPC); ++j) {
        const int q = j * 256 + tid;
        if (i0 + (int64_t)q * EPC < a.N) {
            const uint4 v = x4[q];
            const u32 wd[4] = { v.x, v.y, v.z, v.w };
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                if (DT == 0) {
                    const u32 key = wd[d] & 0x7FFFFFFFu;
                    if (key) atomicAdd(&h[key >> KS], 1u);
                } else {
                    const u32 k0 = wd[d] & 0x7FFFu, k1 = (wd[d] >> 16) & 0x7FFFu;
                    if (k0) atomicAdd(&h[k0 >> KS], 1u);
                    if (k1) atomicAdd(&h[k1 >> KS], 1u);
                }
            }
        }
    }
    __syncthreads();
    // "at or above": running sum from the top bin down; thread t owns the 8 bins below 2048 - 8t
    const int hi = kLBins - tid * 8;
    u32 local = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) local += h[hi - 1 - j];
    u32 tot;
    u32 acc = block_excl_scan<256>(local, scr, &tot);
    u32* __restrict__ out = a.ch_cum + ((size_t)r * a.C + c) * kLBins;
#pragma unroll
    for (int j = 0; j < 8; ++j) { acc += h[hi - 1 - j]; out[hi - 1 - j] = acc; }
}

template <int DT>
__global__ __launch_bounds__(1024) void lr_select_kernel(LargeArgs a)
{
    constexpr int KS = Elem<DT>::kKeyBits - 11;
    __shared__ u32 rc[kLBins + 1];
    __shared__ u32 scr[1024 / kWave + 1];
    __shared__ u32 res[2];
    const int tid = threadIdx.x;
    const int64_t r = blockIdx.x;
    // sum of the chunks' cumulative histograms: a thread takes four bins (one 16-byte load per
    // chunk) of every second chunk, eight independent loads in flight
    for (int bin = tid; bin <= kLBins; bin += 1024) rc[bin] = 0;
    if (tid == 0) { res[0] = 0; res[1] = 0; }
    __syncthreads();
    {
        const int q = tid & (kLBins / 4 - 1), g = tid / (kLBins / 4);          // 512 quads x 2 chunk groups
        const uint4* __restrict__ src = (const uint4*)(a.ch_cum + (size_t)r * a.C * kLBins) + q;
        u32 s0 = 0, s1 = 0, s2 = 0, s3 = 0;
        for (int c0 = g; c0 < a.C; c0 += 16) {
            uint4 t[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int c = c0 + 2 * u;
                t[u] = c < a.C ? src[(size_t)c * (kLBins / 4)] : make_uint4(0, 0, 0, 0);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) { s0 += t[u].x; s1 += t[u].y; s2 += t[u].z; s3 += t[u].w; }
        }
        atomicAdd(&rc[4 * q + 0], s0); atomicAdd(&rc[4 * q + 1], s1);
        atomicAdd(&rc[4 * q + 2], s2); atomicAdd(&rc[4 * q + 3], s3);
    }
    __syncthreads();
    const u32 km1 = a.k > 0 ? (u32)(a.k - 1) : 0u;
    for (int bin = tid; bin < kLBins; bin += 1024) {
        if (rc[bin] > km1 && rc[bin + 1] <= km1) res[0] = (u32)bin;       // holds rank k-1
        if (rc[bin] > 0 && rc[bin + 1] == 0) res[1] = (u32)bin;           // highest occupied
    }
    __syncthreads();
    const u32 B1 = res[0], top = res[1];
    const u32 nL = rc[B1];
    const u32 t_lo = B1 << KS;
    const u32 range = (((top + 1u) << KS) - 1u) - t_lo;
    const int sh = range < (u32)kFB ? 0 : (32 - __clz((int)range)) - 13;   // 13 = log2(kFB)
    // bin 0 holds the exact zeros, which are never sent: such rows go to the generic kernel
    const bool bad = a.k > 0 && (B1 == 0 || nL > a.capL);
    const bool live = a.k > 0 && !bad;
    u32 v = 0;
    if (live && tid < a.C) v = a.ch_cum[((size_t)r * a.C + tid) * kLBins + B1];
    u32 tot;
    const u32 ex = block_excl_scan<1024>(v, scr, &tot);
    if (tid < a.C) a.ch_off[(size_t)r * a.C + tid] = ex;
    if (tid == 0) {
        u32* st = a.rowst + (size_t)r * 16;
        st[0] = t_lo; st[1] = (u32)sh; st[2] = live ? nL : 0u;
        a.fallback[r] = bad ? 1u : 0u;
    }
}

template <int DT>
__global__ __launch_bounds__(256) void lr_compact_kernel(LargeArgs a)
{
    typedef Elem<DT> E;
    constexpr int EPC = DT == 0 ? 4 : 8;
    constexpr int NJ = kLCH / 4 / (kWave * EPC);          // 16-byte loads per lane
    __shared__ u32 wtot[4];
    const int tid = threadIdx.x, c = blockIdx.x, wid = tid / kWave;
    const u32 lane = lane_id();
    const int64_t r = blockIdx.y;
    if (a.fallback[r]) return;
    const u32* st = a.rowst + (size_t)r * 16;
    const u32 t_lo = st[0], nL = st[2];
    const int sh = (int)st[1];
    if (nL == 0) return;
    const int64_t seg0 = (int64_t)c * kLCH + (int64_t)wid * (kLCH / 4);
    const uint4* __restrict__ xr4 = (const uint4*)((const char*)a.x + ((size_t)r * (size_t)a.N + (size_t)seg0) * (DT == 0 ? 4 : 2));
    uint4 v[NJ];
    u32 cntj[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        const int64_t e0 = seg0 + (int64_t)(j * kWave + (int)lane) * EPC;
        v[j] = e0 < a.N ? xr4[j * kWave + lane] : make_uint4(0, 0, 0, 0);
    }
    auto raw_of = [&](int j, int e) -> u32 {
        const u32 wd = (DT == 0) ? (e == 0 ? v[j].x : e == 1 ? v[j].y : e == 2 ? v[j].z : v[j].w)
                                 : ((e >> 1) == 0 ? v[j].x : (e >> 1) == 1 ? v[j].y : (e >> 1) == 2 ? v[j].z : v[j].w);
        return (DT == 0) ? wd : ((e & 1) ? wd >> 16 : wd & 0xFFFFu);
    };
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        u32 n1 = 0;
#pragma unroll
        for (int e = 0; e < EPC; ++e) n1 += E::key((typename E::raw_t)raw_of(j, e)) >= t_lo ? 1u : 0u;   // t_lo > 0: zeros drop out
        cntj[j] = n1;
    }
    u32 basej[NJ];
    u32 wsum = 0;
#pragma unroll
    for (int g = 0; g < (NJ + 2) / 3; ++g) {              // three counts per scan, 10-bit fields
        u32 pk = cntj[3 * g];
        if (3 * g + 1 < NJ) pk |= cntj[3 * g + 1] << 10;
        if (3 * g + 2 < NJ) pk |= cntj[3 * g + 2] << 20;
        const u32 incl = wave_scan_dpp(pk);
        const u32 tot = bcast(incl, kWave - 1);
        const u32 ex = incl - pk;
#pragma unroll
        for (int jj = 0; jj < 3; ++jj) {
            if (3 * g + jj < NJ) {
                basej[3 * g + jj] = wsum + ((ex >> (10 * jj)) & 0x3FFu);
                wsum += (tot >> (10 * jj)) & 0x3FFu;
            }
        }
    }
    if (lane == 0) wtot[wid] = wsum;
    __syncthreads();
    u32 wbase = a.ch_off[(size_t)r * a.C + c];
    for (int v2 = 0; v2 < wid; ++v2) wbase += wtot[v2];
    u64* __restrict__ L = a.L + (size_t)r * a.capL;
    uint16_t* __restrict__ Lfine = a.Lfine + (size_t)r * a.capL;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        u32 pos = wbase + basej[j];
        const u32 idx0 = (u32)(seg0 + (int64_t)(j * kWave + (int)lane) * EPC);
#pragma unroll
        for (int e = 0; e < EPC; ++e) {
            const u32 raw = raw_of(j, e);
            const u32 key = E::key((typename E::raw_t)raw);
            if (key >= t_lo) {
                const u32 neg = E::neg((typename E::raw_t)raw);
                if (pos < a.capL) {
                    L[pos] = ((u64)neg << 63) | ((u64)key << 32) | (u64)(idx0 + e);
                    Lfine[pos] = (uint16_t)(((key - t_lo) >> sh) | (neg << 15));     // what the bounds stage scans
                }
                ++pos;
            }
        }
    }
}

__device__ inline u64 lr_comp(u64 e, int w)       // key << w | inverted index
{
    return (((e >> 32) & 0x7FFFFFFFull) << w) | (((1ull << w) - 1ull) - (e & 0xFFFFFFFFull));
}

// Visit the row's 2-byte list in groups of eight entries (one 16-byte load), four independent
// loads in flight per thread: f(first position, the eight entries, number of valid ones).
template <typename F>
__device__ inline void lr_for_each_fine(const uint16_t* __restrict__ Lfine, u32 nL, F f)
{
    const uint4* __restrict__ q4 = (const uint4*)Lfine;
    const u32 ng = (nL + 7u) / 8u;
    for (u32 g0 = 0; g0 < ng; g0 += 4 * 1024) {
        uint4 t[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) { const u32 g = g0 + (u32)u * 1024 + threadIdx.x; t[u] = g < ng ? q4[g] : make_uint4(0, 0, 0, 0); }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const u32 g = g0 + (u32)u * 1024 + threadIdx.x;
            if (g < ng) {
                const u32 v[8] = { t[u].x & 0xFFFFu, t[u].x >> 16, t[u].y & 0xFFFFu, t[u].y >> 16,
                                   t[u].z & 0xFFFFu, t[u].z >> 16, t[u].w & 0xFFFFu, t[u].w >> 16 };
                const u32 left = nL - g * 8u;
                f(g * 8u, v, left < 8u ? left : 8u);
            }
        }
    }
}

__global__ __launch_bounds__(1024) void lr_bounds_kernel(LargeArgs a)
{
    // fine histogram of the list in LDS: kFB bins, positive count | negative count << 16
    __shared__ u32 fh[kFB];                      // later: members of the boundary bins
    __shared__ u64 cutmem[kCutCap];              // members of the cut bin
    __shared__ u32 tpre_p[1024], tpre_n[1024];   // first class rank of each thread's group of bins
    __shared__ u32 bitmap[kFB / 32];
    __shared__ u32 scr[1024 / kWave + 1];
    __shared__ u32 tgbin[kMaxB2], tgrem[kMaxB2], tcnt[kMaxB2];
    __shared__ u32 s_cut[3], s_n[4];
    __shared__ u64 s_thrK;
    constexpr int BPT = kFB / 1024;              // bins per thread
    const int tid = threadIdx.x;
    const int64_t r = blockIdx.x;
    if (a.fallback[r]) return;
    const int M = a.M, Mn = a.Mn, B2 = a.M + a.Mn, w = a.w;
    u32* st = a.rowst + (size_t)r * 16;
    const u32 nL = st[2];
    const u64* __restrict__ L = a.L + (size_t)r * a.capL;
    const uint16_t* __restrict__ Lfine = a.Lfine + (size_t)r * a.capL;
    const u32 k = (u32)a.k;

    for (int i = tid; i < kFB; i += 1024) fh[i] = 0;
    for (int i = tid; i < kFB / 32; i += 1024) bitmap[i] = 0;
    if (tid < kMaxB2) tcnt[tid] = 0;
    if (tid == 0) { s_cut[0] = 0xFFFFFFFFu; s_n[0] = 0; s_n[1] = 0; s_n[2] = 0; s_n[3] = 0; s_thrK = 0; }
    __syncthreads();
    lr_for_each_fine(Lfine, nL, [&](u32, const u32 (&v)[8], u32 nv) {
#pragma unroll
        for (int d = 0; d < 8; ++d)
            if ((u32)d < nv) atomicAdd(&fh[v[d] & 0x7FFFu], (v[d] >> 15) ? 0x10000u : 1u);
    });
    __syncthreads();

    // (a) class ranks from the top: thread t owns the BPT bins below kFB - BPT * t
    const int hi = kFB - tid * BPT;
    u32 cp[BPT], cn[BPT];
    u32 lp = 0, ln = 0;
#pragma unroll
    for (int j = 0; j < BPT; ++j) { const u32 c = fh[hi - 1 - j]; cp[j] = c & 0xFFFFu; cn[j] = c >> 16; lp += cp[j]; ln += cn[j]; }
    u32 tp, tn;
    const u32 ep = block_excl_scan<1024>(lp, scr, &tp);
    const u32 en = block_excl_scan<1024>(ln, scr, &tn);
    tpre_p[tid] = ep; tpre_n[tid] = en;
    // a 16-bit count that wrapped shows up as a wrong total: such rows are redone generically
    if (tp + tn != nL) { if (tid == 0) a.fallback[r] = 1u; return; }
    {
        u32 ap = ep, an = en;
#pragma unroll
        for (int j = 0; j < BPT; ++j) {
            const u32 cnt = cp[j] + cn[j];
            if (nL > k && cnt && ap + an <= k - 1 && k - 1 < ap + an + cnt) { s_cut[0] = (u32)(hi - 1 - j); s_cut[1] = ap; s_cut[2] = an; }
            ap += cp[j]; an += cn[j];
        }
    }
    __syncthreads();

    // (b) ATKF cut: the comp of overall rank k-1 inside the cut bin
    u32 n_pos = tp, n_neg = tn;
    u64 thrK = 0;
    if (nL > k) {
        const u32 cut = s_cut[0];
        // positions first, then the members themselves with all loads in flight together
        lr_for_each_fine(Lfine, nL, [&](u32 p, const u32 (&v)[8], u32 nv) {
            u32 hits = 0;
#pragma unroll
            for (int d = 0; d < 8; ++d) hits |= ((u32)d < nv && (v[d] & 0x7FFFu) == cut) ? 1u << d : 0u;
            while (hits) {
                const u32 d = (u32)__builtin_ctz(hits);
                hits &= hits - 1u;
                const u32 slot = atomicAdd(&s_n[0], 1u);
                if (slot < (u32)kCutCap) cutmem[slot] = (u64)(p + d);
            }
        });
        __syncthreads();
        const u32 nm = s_n[0];
        if (nm > (u32)kCutCap) { if (tid == 0) a.fallback[r] = 1u; return; }
        for (u32 i = tid; i < nm; i += 1024) {
            const u64 e = L[(u32)cutmem[i]];
            cutmem[i] = (e & kTop) | lr_comp(e, w);
        }
        __syncthreads();
        const u32 rem = (k - 1) - (s_cut[1] + s_cut[2]);
        for (u32 i = tid; i < nm; i += 1024) {
            const u64 me = cutmem[i] & ~kTop;
            u32 gt = 0;
            for (u32 j = 0; j < nm; ++j) gt += (cutmem[j] & ~kTop) > me ? 1u : 0u;
            if (gt == rem) s_thrK = me;
            if (gt <= rem) atomicAdd((cutmem[i] & kTop) ? &s_n[2] : &s_n[1], 1u);
        }
        __syncthreads();
        thrK = s_thrK;
        n_pos = s_cut[1] + s_n[1];
        n_neg = s_cut[2] + s_n[2];
    }

    // (c) block boundaries: class ranks j*K-1, one thread per boundary: first the group of
    //     bins (binary search over the threads' first ranks), then the bin inside the group
    const u32 Kc0 = n_pos / (u32)M, Kc1 = n_neg / (u32)Mn;
    const int nt0 = Kc0 ? M - 1 : 0, nt1 = Kc1 ? Mn - 1 : 0, ntg = nt0 + nt1;
    if (tid < ntg) {
        const int cls = tid >= nt0 ? 1 : 0;
        const int j = (cls ? tid - nt0 : tid) + 1;
        const u32 Rk = (u32)j * (cls ? Kc1 : Kc0) - 1u;
        const u32* tpre = cls ? tpre_n : tpre_p;
        int lo = 0, hi2 = 1023;                      // last group whose first rank is <= Rk
        while (lo < hi2) {
            const int mid = (lo + hi2 + 1) >> 1;
            if (tpre[mid] <= Rk) lo = mid; else hi2 = mid - 1;
        }
        u32 acc = tpre[lo];
        const int top = kFB - lo * BPT;
        u32 bin = (u32)(top - 1);
        for (int jj = 0; jj < BPT; ++jj) {           // the bin of the group that holds rank Rk
            const u32 c = fh[top - 1 - jj];
            const u32 cc = cls ? c >> 16 : c & 0xFFFFu;
            if (Rk < acc + cc) { bin = (u32)(top - 1 - jj); break; }
            acc += cc;
        }
        tgbin[tid] = bin;
        tgrem[tid] = Rk - acc;
        atomicOr(&bitmap[bin >> 5], 1u << (bin & 31));
    }
    __syncthreads();                                 // the histogram is dead from here on
    u64* tmem = (u64*)fh;                            // [ntg][tcap]
    const u32 tcap = ntg ? (u32)(kFB / 2) / (u32)ntg : 1u;
    // members of the boundary bins: their positions go to a flat list first (the cut's storage is
    // free now), then one thread per hit finds its boundaries and fetches the member
    u32* hitpos = (u32*)cutmem;
    constexpr u32 kHitCap = 2 * kCutCap;
    if (tid == 0) s_n[3] = 0;
    __syncthreads();
    lr_for_each_fine(Lfine, nL, [&](u32 p, const u32 (&v)[8], u32 nv) {
        u32 hits = 0;
#pragma unroll
        for (int d = 0; d < 8; ++d) {
            const u32 b = v[d] & 0x7FFFu;
            hits |= ((u32)d < nv && ((bitmap[b >> 5] >> (b & 31u)) & 1u)) ? 1u << d : 0u;
        }
        while (hits) {
            const u32 d = (u32)__builtin_ctz(hits);
            hits &= hits - 1u;
            const u32 slot = atomicAdd(&s_n[3], 1u);
            if (slot < kHitCap) hitpos[slot] = p + d;
        }
    });
    __syncthreads();
    const u32 nhits = s_n[3];
    if (nhits > kHitCap) { if (tid == 0) a.fallback[r] = 1u; return; }
    for (u32 i = tid; i < nhits; i += 1024) {
        const u32 p = hitpos[i];
        const u64 e = L[p];
        const u32 v = Lfine[p], d = v & 0x7FFFu;
        const int cls = (int)(v >> 15);
        const int t0 = cls ? nt0 : 0, t1 = cls ? ntg : nt0;
        for (int t = t0; t < t1; ++t) {
            if (tgbin[t] == d) {
                const u32 slot = atomicAdd(&tcnt[t], 1u);
                if (slot < tcap) tmem[(u32)t * tcap + slot] = lr_comp(e, w);
            }
        }
    }
    __syncthreads();
    int over = 0;
    if (tid < ntg && tcnt[tid] > tcap) over = 1;
    if (__syncthreads_or(over)) { if (tid == 0) a.fallback[r] = 1u; return; }
    const u32 nslots = (u32)ntg * tcap;              // <= kFB / 2
    u64* __restrict__ thr = a.thr + (size_t)r * (1 + kMaxB2);
    for (u32 i = tid; i < nslots; i += 1024) {       // the member with exactly `rem` class-mates above it
        const u32 t = i / tcap, sl = i - t * tcap, cnt = tcnt[t];
        if (sl < cnt) {
            const u64 me = tmem[i];
            u32 gt = 0;
            for (u32 j = 0; j < cnt; ++j) gt += tmem[t * tcap + j] > me ? 1u : 0u;
            if (gt == tgrem[t]) thr[1 + t] = me | ((int)t >= nt0 ? 0ull : kTop);
        }
    }
    if (tid == 0) {
        thr[0] = thrK;
        st[3] = n_pos; st[4] = n_neg; st[5] = Kc0; st[6] = Kc1; st[7] = (u32)ntg; st[8] = (u32)nt0;
    }
    for (int b = tid; b <= B2; b += 1024) {          // K, ..., K, K + remainder per class
        u32 v;
        if (b == B2) v = n_pos + n_neg;
        else { const int s2 = b >= M ? 1 : 0, m = b - s2 * M; v = (s2 ? n_pos : 0u) + (u32)m * (s2 ? Kc1 : Kc0); }
        a.blk_start[(size_t)r * (B2 + 1) + b] = v;
    }
}

__global__ __launch_bounds__(256) void lr_blockcount_kernel(LargeArgs a)
{
    __shared__ u64 thr_s[1 + kMaxB2];
    __shared__ u32 cnt[kMaxB2], kmin[kMaxB2], kmax[kMaxB2];
    const int tid = threadIdx.x, lc = blockIdx.x;
    const int64_t r = blockIdx.y;
    if (a.fallback[r]) return;
    const int M = a.M, Mn = a.Mn, B2 = a.M + a.Mn, w = a.w;
    const u32* st = a.rowst + (size_t)r * 16;
    const u32 nL = st[2];
    const u32 Kc[2] = { st[5], st[6] };
    const int ntg = (int)st[7], nt0 = (int)st[8];
    const u64* __restrict__ L = a.L + (size_t)r * a.capL;
    uint8_t* __restrict__ Lblk = a.Lblk + (size_t)r * a.capL;
    const u32 p0 = (u32)lc * kLCE, p1 = p0 + kLCE < nL ? p0 + kLCE : nL;
    constexpr int NJ = kLCE / 256;
    u64 ev[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) { const u32 p = p0 + (u32)j * 256 + (u32)tid; ev[j] = p < p1 ? L[p] : 0ull; }   // all loads in flight at once
    for (int i = tid; i <= ntg; i += 256) thr_s[i] = a.thr[(size_t)r * (1 + kMaxB2) + i];
    for (int b = tid; b < B2; b += 256) { cnt[b] = 0; kmin[b] = 0xFFFFFFFFu; kmax[b] = 0; }
    __syncthreads();
    const u64 thrK = thr_s[0];
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        const u32 p = p0 + (u32)j * 256 + (u32)tid;
        if (p >= p1) break;
        const u64 e = ev[j];
        const u64 comp = lr_comp(e, w);
        u32 b = 255u;
        if (comp >= thrK) {
            const u32 cls = (u32)(e >> 63);
            const u64 cx = comp | (cls ? 0ull : kTop);
            int lo = 0, hi = ntg;                   // boundaries above cx (they are sorted, largest first)
            while (lo < hi) { const int mid = (lo + hi) >> 1; if (thr_s[1 + mid] > cx) lo = mid + 1; else hi = mid; }
            const u32 m = Kc[cls] ? (u32)lo - (cls ? (u32)nt0 : 0u) : (u32)((cls ? Mn : M) - 1);
            b = cls * (u32)M + m;
            const u32 key = (u32)(e >> 32) & 0x7FFFFFFFu;
            atomicAdd(&cnt[b], 1u);
            atomicMin(&kmin[b], key);
            atomicMax(&kmax[b], key);
        }
        Lblk[p] = (uint8_t)b;
    }
    __syncthreads();
    for (int b = tid; b < B2; b += 256) {
        a.blkcnt[((size_t)r * a.LC + lc) * B2 + b] = cnt[b];
        if (cnt[b]) { atomicMin(&a.vminb[r * B2 + b], kmin[b]); atomicMax(&a.vmaxb[r * B2 + b], kmax[b]); }
    }
}

template <int DT>
__global__ __launch_bounds__(256) void lr_scatter_kernel(LargeArgs a)
{
    __shared__ u32 base[kMaxB2];
    __shared__ u32 cw[4][kMaxB2];
    const int tid = threadIdx.x, lc = blockIdx.x, wid = tid / kWave;
    const int64_t r = blockIdx.y;
    if (a.fallback[r]) return;
    const int B2 = a.M + a.Mn;
    const u32 nL = a.rowst[(size_t)r * 16 + 2];
    if ((u32)lc * kLCE >= nL) return;
    const u64* __restrict__ L = a.L + (size_t)r * a.capL;
    const uint8_t* __restrict__ Lblk = a.Lblk + (size_t)r * a.capL;
    // this thread's entries, all loads in flight at once
    constexpr int NJ = kLCE / 256;
    u32 bl[NJ];
    u64 ev[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        const u32 p = (u32)lc * kLCE + (u32)j * 256 + (u32)tid;
        bl[j] = p < nL ? (u32)Lblk[p] : 255u;
        ev[j] = p < nL ? L[p] : 0ull;
    }
    for (int b = tid; b < B2; b += 256) {
        base[b] = a.blk_start[(size_t)r * (B2 + 1) + b];
        for (int v2 = 0; v2 < 4; ++v2) cw[v2][b] = 0;
    }
    __syncthreads();
    {   // plus the block counts of the list chunks before this one (contiguous: [chunk][block])
        const u32* __restrict__ bc = a.blkcnt + (size_t)r * a.LC * B2;
        const u32 tot = (u32)lc * (u32)B2;
        for (u32 i0 = (u32)tid; i0 < tot; i0 += 256 * 8) {
            u32 t[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) { const u32 i = i0 + (u32)u * 256; t[u] = i < tot ? bc[i] : 0u; }
#pragma unroll
            for (int u = 0; u < 8; ++u) { const u32 i = i0 + (u32)u * 256; if (t[u]) atomicAdd(&base[i % (u32)B2], t[u]); }
        }
    }
    __syncthreads();
    int nbits = 0;
    while ((1 << nbits) < B2) ++nbits;
    u32* __restrict__ bo_idx = a.bo_idx + (size_t)r * (size_t)a.k;
    u32* __restrict__ bo_val = a.bo_val + (size_t)r * (size_t)a.k;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        const bool kept = bl[j] != 255u;
        const u32 b = kept ? bl[j] : 0u;
        const u64 e = ev[j];
        const u64 km = __ballot(kept);
        u32 plo = (u32)km, phi = (u32)(km >> 32);
        for (int bit = 0; bit < nbits; ++bit) {
            const u32 onm = (u32)__builtin_amdgcn_sbfe((int)b, (u32)bit, 1u);
            const u64 bal = __ballot(onm != 0u);
            plo &= ~((u32)bal ^ onm);
            phi &= ~((u32)(bal >> 32) ^ onm);
        }
        const u32 before = __builtin_amdgcn_mbcnt_hi(phi, __builtin_amdgcn_mbcnt_lo(plo, 0u));
        if (kept && before == 0) cw[wid][b] = (u32)__popc(plo) + (u32)__popc(phi);
        __syncthreads();
        if (kept) {
            u32 pos = base[b] + before;
            for (int v2 = 0; v2 < wid; ++v2) pos += cw[v2][b];
            if ((int64_t)pos < a.k) {
                bo_idx[pos] = (u32)e;
                bo_val[pos] = DT == 0 ? ((u32)(e >> 32) & 0x7FFFFFFFu) : (((u32)(e >> 32) & 0x7FFFu) << 16);
            }
        }
        __syncthreads();
        for (int bb = tid; bb < B2; bb += 256) {
            u32 s = 0;
            for (int v2 = 0; v2 < 4; ++v2) { s += cw[v2][bb]; cw[v2][bb] = 0; }
            base[bb] += s;
        }
        __syncthreads();
    }
}

// NQ > 0: the number of allowed bitwidths is known at compile time; NQ == 0: any number up to 16.
template <int DT, int NQ>
__global__ __launch_bounds__(256) void lr_abq_kernel(LargeArgs a)
{
    typedef Elem<DT> E;
    constexpr int QN = NQ ? NQ : kMaxQ;
    constexpr int NJ = kPCH / 256;               // entries per thread: u32 partial sums hold 8 residuals of 2^28
    static_assert(NJ <= 8, "u32 partial sums");
    __shared__ u32 bs[kMaxB2 + 1];
    __shared__ float vminf[kMaxB2];
    __shared__ int e_tab[kMaxB2], er_tab[kMaxB2], degen[kMaxB2];
    __shared__ float inv_tab[kMaxB2][kMaxQ];
    __shared__ u64 sums[kMaxB2][kMaxQ + 1];
    const int tid = threadIdx.x, pc = blockIdx.x;
    const int64_t r = blockIdx.y;
    // the values first: their loads need nothing but the launch geometry (positions beyond the
    // row's count hold leftovers and are never used) and are the longest wait of the kernel
    const u32 p0 = (u32)pc * kPCH;
    const u32* __restrict__ bo_val = a.bo_val + (size_t)r * (size_t)a.k;
    u32 vb[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) { const u32 p = p0 + (u32)j * 256 + (u32)tid; vb[j] = (int64_t)p < a.k ? bo_val[p] : 0u; }
    if (a.fallback[r]) return;
    const int B2 = a.M + a.Mn, nq = NQ ? NQ : a.nq;
    const u32* st = a.rowst + (size_t)r * 16;
    const u32 n = st[3] + st[4];
    const u32 p1 = p0 + kPCH < n ? p0 + kPCH : n;
    if (p0 >= n) return;
    for (int b = tid; b <= B2; b += 256) bs[b] = a.blk_start[(size_t)r * (B2 + 1) + b];
    __syncthreads();
    for (int b = tid; b < B2; b += 256) {
        const u32 cnt = bs[b + 1] - bs[b];
        int dg = 1, e = 0, er = 0;
        float rng1 = 1.f, vmin = 0.f;
        if (cnt) {
            const u32 lo = E::value_bits(a.vminb[r * B2 + b]), hi = E::value_bits(a.vmaxb[r * B2 + b]);
            vmin = __uint_as_float(lo);
            const float rng = __uint_as_float(hi) - vmin;
            dg = !(rng > 0.f);                       // only a range of exactly 0 is degenerate
            if (!dg) { er = range_exp(rng); rng1 = unit_range(rng, er); }
            e = ilogb_bits(hi) + 1;
        }
        vminf[b] = vmin; degen[b] = dg; e_tab[b] = e; er_tab[b] = er;
        for (int t = 0; t < nq; ++t) {
            inv_tab[b][t] = dg ? 0.f : (float)((1u << a.qlist[t]) - 1u) / rng1;
            sums[b][t] = 0;
        }
        sums[b][kMaxQ] = 0;
    }
    bool small_q = true;
#pragma unroll
    for (int t = 0; t < QN; ++t)
        if ((NQ || t < nq) && a.qlist[t] > 8) small_q = false;
    __syncthreads();
    {
        int cur = -1;
        u32 acc[QN];
        u64 accE = 0;
        float inv[QN], inv15[QN];
#pragma unroll
        for (int t = 0; t < QN; ++t) { acc[t] = 0; inv[t] = 0.f; inv15[t] = 0.f; }
        float vmin = 0.f;
        int e = 0, dg = 1, er = 0;
        auto flush = [&]() {
            if (cur < 0) return;
#pragma unroll
            for (int t = 0; t < QN; ++t)
                if ((NQ || t < nq) && acc[t]) { atomicAdd(&sums[cur][t], (u64)acc[t]); acc[t] = 0; }
            if (accE) { atomicAdd(&sums[cur][kMaxQ], accE); accE = 0; }
        };
        const int top = nq - 1, qtop = a.qlist[top];
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const u32 p = p0 + (u32)j * 256 + (u32)tid;
            if (p >= p1) break;
            int b = cur < 0 ? 0 : cur;
            while (b < B2 - 1 && p >= bs[b + 1]) ++b;
            if (b != cur) {
                flush();
                cur = b; vmin = vminf[b]; e = e_tab[b]; dg = degen[b]; er = er_tab[b];
#pragma unroll
                for (int t = 0; t < QN; ++t) {
                    inv[t] = (NQ || t < nq) ? inv_tab[b][t] : 0.f;
                    inv15[t] = inv[t] * 32768.0f;        // the scale is at most 2^16 - 1
                }
            }
            const float av = __uint_as_float(vb[j]);
            const u64 A = (u64)(u32)rintf(ldexpf(av, 20 - e));     // 20-bit energy grid scaled to vmax
            accE += A * A;
            if (dg) continue;
            const float d = to_unit(av - vmin, er);
            if (a.guard == 1) {
                // Eq. "DS": | (code at q_bit >> (q_bit - q)) - code at q | for every lower bitwidth
                float inv_top = 0.f;
#pragma unroll
                for (int t = 0; t < QN; ++t) inv_top = t == top ? inv[t] : inv_top;
                const u32 c0 = (u32)rintf(d * inv_top);               // within [0, 2^q - 1]: no clamp needed
#pragma unroll
                for (int t = 0; t < QN; ++t) {
                    if ((NQ || t < nq) && t < top) {
                        const u32 c = (u32)rintf(d * inv[t]);
                        const u32 ref = c0 >> (u32)(qtop - a.qlist[t]);
                        acc[t] += ref > c ? ref - c : c - ref;
                    }
                }
            } else {
                // residual on the 2^-15 grid: rint(y * 2^15) reduced to 15 signed bits (Sec. 3.2.1 metric
                // in the code domain); bitwidths up to 8 keep y * 2^15 below 2^23, where adding 2^23
                // rounds to the integer grid with the same round-half-even
#pragma unroll
                for (int t = 0; t < QN; ++t) {
                    if (NQ || t < nq) {
                        const u32 zi = small_q ? __float_as_uint(d * inv15[t] + 8388608.0f)
                                               : (u32)rintf((d * inv[t]) * 32768.0f);
                        const int rho = __builtin_amdgcn_sbfe((int)zi, 0u, 15u);
                        acc[t] += (u32)(rho * rho);
                    }
                }
            }
        }
        // The positions of a wavefront are consecutive, so its lanes are nearly always in one
        // block: the sums are then added up across the wavefront first (16-bit and 22-bit
        // pieces, so that the lane sums fit 32 bits) and one lane adds them to the table.
        const int cur0 = __builtin_amdgcn_readfirstlane(cur);
        if (__all(cur == cur0)) {
            if (cur0 >= 0) {
#pragma unroll
                for (int t = 0; t < QN; ++t) {
                    if (NQ || t < nq) {
                        const u32 lo16 = wave_sum(acc[t] & 0xFFFFu), hi16 = wave_sum(acc[t] >> 16);
                        if ((tid & (kWave - 1)) == 0 && (lo16 | hi16)) atomicAdd(&sums[cur0][t], (u64)lo16 + ((u64)hi16 << 16));
                    }
                }
                const u32 e0 = wave_sum((u32)accE & 0x3FFFFFu), e1 = wave_sum((u32)(accE >> 22) & 0x3FFFFFu), e2 = wave_sum((u32)(accE >> 44));
                if ((tid & (kWave - 1)) == 0 && (e0 | e1 | e2)) atomicAdd(&sums[cur0][kMaxQ], (u64)e0 + ((u64)e1 << 22) + ((u64)e2 << 44));
            }
        } else {
            flush();
        }
    }
    __syncthreads();
    for (int i = tid; i < B2 * (nq + 1); i += 256) {
        const int b = i / (nq + 1), t = i - b * (nq + 1);
        const u64 v = sums[b][t == nq ? kMaxQ : t];
        if (v) atomicAdd(&a.sums[((size_t)r * B2 + b) * (nq + 1) + t], v);
    }
}

// Window x of a row's slot for the pack stage: windows of pack_words words up to the first word
// that holds code bits (word wb), windows of pack_words_code words from there on.  Returns the
// first word and the number of words (0: nothing to do).
__device__ inline void lr_pack_window(const LargeArgs& a, int x, u64 wb, u64 row_words, u64* c0, u64* cw)
{
    u64 lo, hi;
    if (x < a.nwin_idx) {
        lo = (u64)x * (u64)a.pack_words;
        hi = lo + (u64)a.pack_words;
        hi = hi < wb ? hi : wb;
    } else {
        lo = wb + (u64)(x - a.nwin_idx) * (u64)a.pack_words_code;
        hi = lo + (u64)a.pack_words_code;
    }
    hi = hi < row_words ? hi : row_words;
    *c0 = lo;
    *cw = hi > lo ? hi - lo : 0;
}

template <int DT>
__global__ __launch_bounds__(128) void lr_choose_kernel(LargeArgs a)
{
    typedef Elem<DT> E;
    __shared__ u32 bits_s[kMaxB2], q_s[kMaxB2], bs_s[kMaxB2 + 1];
    __shared__ u64 co_s[kMaxB2 + 1];
    __shared__ u64 s_words;
    const int b = threadIdx.x;
    const int64_t r = blockIdx.x;
    if (a.fallback[r]) return;
    const int B2 = a.M + a.Mn, nq = a.nq;
    const u32* st = a.rowst + (size_t)r * 16;
    const u32 n = st[3] + st[4];
    if (b < B2) {
        const u32 cnt = a.blk_start[(size_t)r * (B2 + 1) + b + 1] - a.blk_start[(size_t)r * (B2 + 1) + b];
        float vmin = 0.f, vmax = 0.f, inv = 0.f;
        int q = a.qlist[0];
        u32 flag = 0;
        if (cnt) {
            const u32 hi = E::value_bits(a.vmaxb[r * B2 + b]);
            vmin = __uint_as_float(E::value_bits(a.vminb[r * B2 + b]));
            vmax = __uint_as_float(hi);
            const float rng = vmax - vmin;
            if (rng > 0.f) {
                const float rng1 = unit_range(rng, range_exp(rng));
                const int e = ilogb_bits(hi) + 1;
                const u64* sm = a.sums + ((size_t)r * B2 + b) * (nq + 1);
                const double rhs = a.beta * ldexp((double)sm[nq], 2 * e - 40);
                flag = 0x80u;
                for (int t = 0; t < nq && flag; ++t) {
                    const float Lq = (float)((1u << a.qlist[t]) - 1u);
                    const float o = rng / Lq;
                    const double lhs = ((double)o * (double)o) * (double)sm[t] * 0x1p-30;
                    q = a.qlist[t]; inv = Lq / rng1;
                    if (lhs <= rhs) flag = 0;
                }
            }
        }
        if (a.guard == 1) {         // greedy descent from q_bit while the mismatch stays within delta
            int chosen = cnt ? nq - 1 : 0;
            const u64* sm = a.sums + ((size_t)r * B2 + b) * (nq + 1);
            for (int t = nq - 2; t >= 0 && cnt; --t) {
                if ((double)sm[t] <= a.beta * (double)cnt) chosen = t; else break;
            }
            q = a.qlist[chosen]; flag = 0; inv = 0.f;
            if (cnt && vmax - vmin > 0.f) inv = (float)((1u << q) - 1u) / unit_range(vmax - vmin, range_exp(vmax - vmin));
        }
        if (a.lad.on) {             // the bitwidth is given, also for empty and degenerate blocks
            q = a.qlist[ladder_index(a.lad, b < a.M ? b : b - a.M)];
            flag = 0; inv = 0.f;
            if (cnt && vmax - vmin > 0.f) inv = (float)((1u << q) - 1u) / unit_range(vmax - vmin, range_exp(vmax - vmin));
        }
        a.qsel[r * B2 + b] = (u32)q;
        a.inv_sel[r * B2 + b] = inv;
        q_s[b] = (u32)q;
        bs_s[b] = a.blk_start[(size_t)r * (B2 + 1) + b];
        if (b == B2 - 1) bs_s[B2] = bs_s[b] + cnt;
        bits_s[b] = cnt * (u32)q;             // < 2^31 * 16 would overflow: the list capacity keeps cnt small
        const size_t mi = (size_t)r * (size_t)B2 + b;
        a.mv.vmin[mi] = vmin; a.mv.vmax[mi] = vmax; a.mv.q[mi] = (uint8_t)((u32)q | flag);
    }
    __syncthreads();
    if (b == 0) {
        u64 acc = 0;
        u64* co = a.code_off + (size_t)r * (B2 + 1);
        for (int i = 0; i < B2; ++i) { co[i] = acc; co_s[i] = acc; acc += bits_s[i]; }
        co[B2] = acc; co_s[B2] = acc;
        const u64 bits = (u64)n * (u64)a.w + acc;
        u64 words = (bits + 31) >> 5;
        if (words > a.cap_words) words = a.cap_words;
        a.row_words[r] = words;
        s_words = words;
        a.mv.n_pos[r] = st[3];
        a.mv.n_neg[r] = st[4];
    }
    __syncthreads();
    // for every window of the pack stage: the block-ordered entries whose code field meets it.
    // Code fields lie at or after word wb, i.e. in the short windows only: every block's thread
    // walks the few windows its code section meets.
    {
        const u64 idx_bits = (u64)n * (u64)a.w, wb = idx_bits >> 5;
        u32* __restrict__ wr = a.win_range + (size_t)r * a.nwin * 2;
        for (int wi = b; wi < a.nwin; wi += 128) { wr[2 * wi] = n; wr[2 * wi + 1] = 0; }
        __syncthreads();
        const int csh = 31 - __clz(a.pack_words_code);          // pack_words_code is a power of two
        const int tpb = 128 / B2 > 0 ? 128 / B2 : 1;           // threads per block (B2 <= 128)
        const int bb = b / tpb, sub = b - bb * tpb;
        if (bb < B2) {
            const u32 cnt = bs_s[bb + 1] - bs_s[bb];
            const u64 cs = idx_bits + co_s[bb], ce = idx_bits + co_s[bb + 1];
            if (cnt && ce > cs) {
                const u32 q = q_s[bb];
                const int w0 = a.nwin_idx + (int)(((cs >> 5) - wb) >> csh), w1 = a.nwin_idx + (int)((((ce - 1) >> 5) - wb) >> csh);
                for (int wi = w0 + sub; wi <= w1 && wi < a.nwin; wi += tpb) {
                    u64 c0, cw;
                    lr_pack_window(a, wi, wb, s_words, &c0, &cw);
                    const u64 lo = c0 << 5, hi = (c0 + cw) << 5;
                    if (cw == 0 || ce <= lo || cs >= hi) continue;
                    const u32 dlo = (u32)((lo > cs ? lo : cs) - cs), dhi = (u32)((hi < ce ? hi : ce) - cs);   // < 2^31: one block's bits
                    atomicMin(&wr[2 * wi], bs_s[bb] + dlo / q);
                    atomicMax(&wr[2 * wi + 1], bs_s[bb] + (dhi + q - 1) / q);
                }
            }
        }
    }
}

// A thread packs a run of consecutive fields into whole words in registers and writes each
// word of the window image once: the first and the last word of a run may be shared with the
// neighbouring runs (atomic OR), the words between belong to this run alone (plain store).
struct RunPacker {
    u32* stage;
    int nwords;          // words of the window
    u64 acc;
    int fill, wi;
    bool first;
    __device__ inline void begin(u32* st, int nw, int rel)      // rel: first bit, relative to the window (may be negative)
    {
        stage = st; nwords = nw;
        wi = rel >> 5; fill = rel & 31; acc = 0; first = true;
    }
    __device__ inline void put(u32 wd, bool shared)
    {
        if (wi >= 0 && wi < nwords) {
            if (shared) atomicOr(&stage[wi], wd); else stage[wi] = wd;
        }
    }
    __device__ inline void append(u32 v, int nb)                 // nb <= 32, v < 2^nb
    {
        acc |= (u64)v << fill;
        fill += nb;
        if (fill >= 32) {
            put((u32)acc, first);
            first = false;
            acc >>= 32; fill -= 32; ++wi;
        }
    }
    __device__ inline void finish() { if (fill > 0) put((u32)acc, true); }
};

template <int DT>
__global__ __launch_bounds__(256) void lr_pack_kernel(LargeArgs a)
{
    typedef Elem<DT> E;
    constexpr int RUN = 8;                        // consecutive entries per thread and run
    __shared__ u32 sA[kPackWords];
    __shared__ u32 bs[kMaxB2 + 1], qsel[kMaxB2];
    __shared__ u32 crel[kMaxB2];                  // first code bit of the block relative to the window, modulo 2^32
    __shared__ float vminf[kMaxB2], invs[kMaxB2];
    __shared__ int ers[kMaxB2];
    const int tid = threadIdx.x;
    const int64_t r = blockIdx.y;
    const int B2 = a.M + a.Mn, w = a.w;
    // everything the workgroup needs to know its work, in one round of loads
    const u32 fb = a.fallback[r];
    const u64 row_words = a.row_words[r];
    const u32 n = a.rowst[(size_t)r * 16 + 3] + a.rowst[(size_t)r * 16 + 4];
    // the windows with code fields hold the most entries: they are started first
    const int nwc = a.nwin - a.nwin_idx;
    const int win = (int)blockIdx.x < nwc ? a.nwin_idx + (int)blockIdx.x : (int)blockIdx.x - nwc;
    const u32 cq0 = a.win_range[((size_t)r * a.nwin + win) * 2 + 0];
    const u32 cq1 = a.win_range[((size_t)r * a.nwin + win) * 2 + 1];
    if (fb) return;
    const u64 idx_bits = (u64)n * (u64)w;
    u64 c0, cw;
    lr_pack_window(a, win, idx_bits >> 5, row_words, &c0, &cw);
    if (cw == 0) return;
    const u64 lo = c0 << 5, hi = (c0 + cw) << 5;
    const u32* __restrict__ bo_idx = a.bo_idx + (size_t)r * (size_t)a.k;
    const u32* __restrict__ bo_val = a.bo_val + (size_t)r * (size_t)a.k;
    // index fields that meet the window
    u32 iq0 = 0, iq1 = 0;
    if (lo < idx_bits) {
        iq0 = (u32)(lo / (u64)w);
        const u64 t1 = (hi + (u64)w - 1) / (u64)w;
        iq1 = t1 > (u64)n ? n : (u32)t1;
    }
    // first run of both sections: the loads are in flight while the block tables arrive
    u32 vi[RUN], vc[RUN];
#pragma unroll
    for (int u = 0; u < RUN; ++u) { const u32 p = iq0 + (u32)tid * RUN + (u32)u; vi[u] = p < iq1 ? bo_idx[p] : 0u; }
#pragma unroll
    for (int u = 0; u < RUN; ++u) { const u32 p = cq0 + (u32)tid * RUN + (u32)u; vc[u] = p < cq1 ? bo_val[p] : 0u; }
    for (int b = tid; b < B2; b += 256) {
        const u32 b0 = a.blk_start[(size_t)r * (B2 + 1) + b];
        bs[b] = b0;
        if (b == B2 - 1) bs[B2] = a.blk_start[(size_t)r * (B2 + 1) + B2];
        qsel[b] = a.qsel[r * B2 + b];
        invs[b] = a.inv_sel[r * B2 + b];
        vminf[b] = __uint_as_float(E::value_bits(a.vminb[r * B2 + b]));
        {
            const float rng = __uint_as_float(E::value_bits(a.vmaxb[r * B2 + b])) - vminf[b];
            ers[b] = rng > 0.f ? range_exp(rng) : 0;      // blocks of range 0 have inv = 0 and are not scaled
        }
        crel[b] = (u32)(idx_bits + a.code_off[(size_t)r * (B2 + 1) + b] - lo);
    }
    for (int i = tid; i < (int)cw; i += 256) sA[i] = 0;
    __syncthreads();
    // Bit positions are taken relative to the window in 32-bit arithmetic: the true value of
    // every position handled here lies within a few bits of the window, so the wrapped
    // difference is exact.
    RunPacker rp;
    {
        const u32 lo32 = (u32)lo;
        for (u32 p0 = iq0 + (u32)tid * RUN; p0 < iq1; p0 += 256 * RUN) {
            if (p0 != iq0 + (u32)tid * RUN) {
#pragma unroll
                for (int u = 0; u < RUN; ++u) { const u32 p = p0 + (u32)u; vi[u] = p < iq1 ? bo_idx[p] : 0u; }
            }
            rp.begin(sA, (int)cw, (int)(p0 * (u32)w - lo32));
#pragma unroll
            for (int u = 0; u < RUN; ++u)
                if (p0 + (u32)u < iq1) rp.append(vi[u], w);
            rp.finish();
        }
    }
    {
        // the block's constants stay in registers until the position leaves the block; the code
        // sections of consecutive blocks are contiguous in the stream, so a run may cross blocks
        int b = 0;
        for (u32 p0 = cq0 + (u32)tid * RUN; p0 < cq1; p0 += 256 * RUN) {
            if (p0 != cq0 + (u32)tid * RUN) {
#pragma unroll
                for (int u = 0; u < RUN; ++u) { const u32 p = p0 + (u32)u; vc[u] = p < cq1 ? bo_val[p] : 0u; }
            }
            while (b < B2 - 1 && p0 >= bs[b + 1]) ++b;
            u32 b_end = b < B2 - 1 ? bs[b + 1] : 0xFFFFFFFFu;
            int q = (int)qsel[b];
            float inv = invs[b], vmin = vminf[b], qmaxf = (float)((1u << q) - 1u);
            int er = ers[b];
            rp.begin(sA, (int)cw, (int)(crel[b] + (p0 - bs[b]) * (u32)q));
#pragma unroll
            for (int u = 0; u < RUN; ++u) {
                const u32 p = p0 + (u32)u;
                if (p >= cq1) break;
                if (p >= b_end) {
                    while (b < B2 - 1 && p >= bs[b + 1]) ++b;
                    b_end = b < B2 - 1 ? bs[b + 1] : 0xFFFFFFFFu;
                    q = (int)qsel[b]; inv = invs[b]; vmin = vminf[b]; qmaxf = (float)((1u << q) - 1u); er = ers[b];
                }
                u32 c = 0;
                if (inv != 0.f) {
                    const float y = to_unit(__uint_as_float(vc[u]) - vmin, er) * inv;
                    c = (u32)fminf(fmaxf(rintf(y), 0.f), qmaxf);
                }
                rp.append(c, q);
            }
            rp.finish();
        }
    }
    __syncthreads();
    u32* __restrict__ slot = a.slots + (size_t)r * (size_t)a.cap_words;
    for (int i = tid; i < (int)cw; i += 256) slot[c0 + i] = sA[i];
}

}  // namespace slicer
