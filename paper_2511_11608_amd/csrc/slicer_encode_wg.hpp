// Row-resident encoder for rows of 4 K to 32 K bf16 (16 K fp32) elements: ONE WORKGROUP (4 or 16
// wavefronts) PER ROW.  A single wavefront needs about 30 us for an 8192-element row,
// nearly all of it dependent-instruction and LDS latency, and holds so much of the row per lane that
// only two or three wavefronts fit a SIMD; a batch of a few hundred rows
// (one auto-regressive decode step of Sec. 2.1, one hidden state per client) also leaves three
// quarters of the SIMDs idle.  Here the wavefronts of a workgroup share the row (four when the batch
// fills the chip anyway, sixteen for the smallest batches: more wavefronts per SIMD hide each other's
// latencies).
//
// Same method and same data structures as the one-wavefront kernel (slicer_encode_small.hpp):
// comps "key, inverted index, class bit" order everything; a 2048-bin LDS histogram over a window
// that hangs from the row's largest key gives the bin of rank k-1 (ATKF, Sec. 3.1); everything at
// or above it is compacted, in index order, into a list; the list is bucketed into 1024 fine bins,
// the top-K cut and the block boundaries (MS, Sec. 3.2) are order statistics located over the bins
// and resolved inside their bin; an entry's block is the number of boundaries above it; a stable
// split by block, integer ABQ sums (Sec. 3.2.1), bitwidth choice, packing through an LDS image.
// What changes is who does what: per-element passes and per-entry passes are dealt to the NW
// wavefronts (thread t owns 16-byte chunks t, t + 64 NW, ...; wavefront v owns list slots v, v + NW,
// ...), scans run over the workgroup, the two short serial steps (cut, boundaries) run on
// wavefront 0, and workgroup barriers separate the stages.
//
// Either guard or a fixed ladder, lambda = 0; rows it cannot hold are flagged for the generic kernel.  bf16 entries
// are one word (sign, key, inverted index); fp32 entries keep the raw word in the list and the index
// beside it, and the members of a fine bin compare on "in-bin key bits, inverted index, class".
#pragma once

#include "slicer_encode_small.hpp"

namespace slicer {

constexpr int kWgMaxSlots = 32;        // list slots (64 entries): lists of up to 2048 entries
constexpr int kWgMisc = 64;            // broadcast words (0..15), per-wavefront maxima (16..31), scan scratch (32..)

// words of LDS: the one-wavefront layout (list in LDS) followed by the workgroup's own tables
__host__ __device__ inline int wg_main_words(int dt, int cap, int region0, int B2)
{
    return small_lds_words(dt, cap, region0, B2, 0, kCoarseBins);
}
__host__ __device__ inline int wg_lds_words(int dt, int cap, int region0, int B2)
{
    // misc, chunk totals and their prefix (2 x 64), per-slot per-block counts as 16-bit (cap / 64 slots)
    return wg_main_words(dt, cap, region0, B2) + kWgMisc + 128 + ((cap / kWave) * B2 + 1) / 2 + 2;
}

// wavefronts per SIMD the register allocator must leave room for (same rule as the one-wavefront kernel)
constexpr int wg_min_waves(int dt, int nw, int ept)
{
    const int row_regs = dt == 0 ? ept : ept / 2;
    const int per_wg = (nw + 3) / 4;                  // wavefronts of one workgroup on a SIMD
    const int want = row_regs <= 32 ? 5 : row_regs == 64 ? 3 : 1;
    return want > per_wg ? want : per_wg;
}

template <int DT, int NW, int EPT, int NQ>
__global__ __launch_bounds__(NW * kWave) __attribute__((amdgpu_waves_per_eu(wg_min_waves(DT, NW, EPT)))) void enc_wg_kernel(SmallArgs a)
{
    typedef Elem<DT> E;
    constexpr int kWgThreads = NW * kWave, kWgWaves = NW;
    constexpr int kWgSlots = (kWgMaxSlots + NW - 1) / NW;     // list slots per wavefront
    typedef typename std::conditional<DT == 0, u64, u32>::type comp_t;   // bf16: key + index fit 31 bits
    constexpr comp_t kClsBit = (comp_t)1 << (8 * sizeof(comp_t) - 1);       // set for the positive class
    constexpr int kHiShift = DT == 0 ? 32 : 0;       // position of the key word in a comp
    constexpr u32 kKeyMask = DT == 0 ? 0x7FFFFFFFu : 0x7FFFu;
    constexpr int kRegThr = 14;
    constexpr int QN = NQ ? NQ : kMaxQ;
    constexpr int EPC = DT == 0 ? 4 : 8, NCH = EPT / EPC;   // elements per 16-byte chunk, chunks per thread
    static_assert(NCH * kWgWaves <= kWave, "chunk totals are scanned by one wavefront");
    extern __shared__ u32 smem[];

    const u32 tid = threadIdx.x, lane = lane_id(), wv = tid / kWave;
    const int64_t r = (int64_t)blockIdx.x;
    if (r >= a.R) return;
    const int N = (int)a.N, M = a.M, Mn = a.Mn, w = a.w, B2 = a.M + a.Mn, nq = NQ ? NQ : a.nq, cap = a.cap;
    const int k = (int)a.k;
    SmallLds L = small_carve(smem, DT, cap, a.region0_words, B2, 0);
    u32* misc = smem + wg_main_words(DT, cap, a.region0_words, B2);      // broadcast words and scan scratch
    u32* ctab = misc + kWgMisc;                                           // [NCH][4] chunk totals per wavefront, then their prefixes
    uint16_t* stab = (uint16_t*)(ctab + 128);                        // [slot][B2] entries of block b in slot s
    auto give_up = [&]() { if (tid == 0) a.fallback[r] = 1u; };      // callers return right after, all threads alike
    if (__builtin_amdgcn_groupstaticsize() != 0u) {                  // integer LDS addresses assume offset 0
        give_up();
        return;
    }
    const u32 lent_off = (u32)(L.Lent - smem) * 4u;

    // ---- 1. load the row ---------------------------------------------------------------------
    const uint4* __restrict__ xr = (const uint4*)((const char*)a.x + (size_t)r * (size_t)N * (DT == 0 ? 4 : 2));
    uint4 v[NCH];
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int base = (c * kWgThreads + (int)tid) * EPC;
        v[c] = base < N ? xr[c * kWgThreads + tid] : make_uint4(0, 0, 0, 0);
    }
    auto word_of = [&](int c, int d) -> u32 { return d == 0 ? v[c].x : d == 1 ? v[c].y : d == 2 ? v[c].z : v[c].w; };

    // List length and positions for a lower key bound t_lo: counts per chunk, positions inside the
    // wavefront (three chunk counts share a scan: 10-bit fields, at most 512 keys per wavefront and
    // chunk), then the wavefronts' chunk totals are scanned in chunk order by wavefront 0.
    u32 t_lo = 1u, nL = 0;
    u32 cntc[NCH], basec[NCH];
    auto count_pass = [&]() {
        const u32 C16 = (0x8000u - t_lo) * 0x10001u;             // bit 15 / 31 of (key + C16) <=> key >= t_lo
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            u32 n1 = 0;
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                if (DT == 0) n1 += (word_of(c, d) & 0x7FFFFFFFu) >= t_lo ? 1u : 0u;
                else n1 += (u32)__popc(((word_of(c, d) & 0x7FFF7FFFu) + C16) & 0x80008000u);
            }
            cntc[c] = n1;
        }
#pragma unroll
        for (int g = 0; g < (NCH + 2) / 3; ++g) {
            u32 pk = cntc[3 * g];
            if (3 * g + 1 < NCH) pk |= cntc[3 * g + 1] << 10;
            if (3 * g + 2 < NCH) pk |= cntc[3 * g + 2] << 20;
            const u32 incl = wave_scan_dpp(pk);
            const u32 tot = bcast(incl, kWave - 1);
            const u32 ex = incl - pk;
#pragma unroll
            for (int j = 0; j < 3; ++j) {
                if (3 * g + j < NCH) {
                    basec[3 * g + j] = (ex >> (10 * j)) & 0x3FFu;
                    if (lane == 0) ctab[(3 * g + j) * kWgWaves + (int)wv] = (tot >> (10 * j)) & 0x3FFu;
                }
            }
        }
        __syncthreads();
        if (wv == 0) {
            const u32 t = (int)lane < NCH * kWgWaves ? ctab[lane] : 0u;
            const u32 incl = wave_scan_dpp(t);
            ctab[64 + lane] = incl - t;
            if (lane == kWave - 1) misc[4] = incl;
        }
        __syncthreads();
        nL = misc[4];
#pragma unroll
        for (int c = 0; c < NCH; ++c) basec[c] += ctab[64 + c * kWgWaves + (int)wv];
        __syncthreads();                             // the tables are free for the next use
    };

    // Threshold hint (see slicer_encode_small.hpp): the cut key an earlier row left in the workspace,
    // lowered a few steps; accepted when it keeps at least k keys and not many more.  The count decides.
    const u32 hslot = (u32)blockIdx.x & (u32)(kHintSlots - 1);
    bool hinted = false;
    if (k > 0) {
        const u32 hint_key = a.hint[hslot] & kKeyMask;
        const u32 dlt = kHintDelta << (DT == 0 ? 16 : 0);
        t_lo = hint_key > dlt ? hint_key - dlt : 1u;
        count_pass();
        hinted = nL >= (u32)k && nL <= (u32)k + 2u * kHintSlack && (int)nL <= cap;
    }

    u32 kmax = 0;
    if (!hinted) {
    // largest magnitude key of the row
    {
        u32 mx = 0;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                if (DT == 0) mx = max(mx, word_of(c, d) & 0x7FFFFFFFu);
                else mx = pk_max_u16(mx, word_of(c, d) & 0x7FFF7FFFu);
            }
        }
        if (DT == 1) mx = max(mx & 0xFFFFu, mx >> 16);
        mx = wave_max_dpp(mx);
        if (lane == 0) misc[16 + wv] = mx;
        __syncthreads();
        kmax = 0;
#pragma unroll
        for (int i = 0; i < NW; ++i) kmax = max(kmax, misc[16 + i]);
        __syncthreads();
    }

    // ---- coarse histogram: 2048 bins hanging from wtop, bin = (wtop - key) >> S ---------------
    constexpr int S1 = DT == 0 ? 16 : 0;             // fp32: 65536 keys per bin (the same 128 bins per octave as bf16)
    u32 wtop = kmax, above = 0;
    int S = S1;
    u32 B1 = 0, c_gt = 0, cnt1 = 0;
    bool found = false;
    const u32 rank_t = k > 0 ? (u32)(k - 1) : 0u;
    auto hist_pass = [&](auto shift) {
        constexpr int SH = decltype(shift)::value;
        constexpr int SHB = SH >= 2 ? SH - 2 : 0;      // fp32: shift that leaves the bin number times 4
        {
            uint4* h4 = (uint4*)smem;
            for (int i = (int)tid; i < kCoarseBins / 4; i += kWgThreads) h4[i] = make_uint4(0, 0, 0, 0);
            if (tid < 4) misc[tid] = 0;
        }
        __syncthreads();
        const u32 wt2 = wtop * 0x10001u;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            if ((c * kWgThreads + (int)tid) * EPC < N) {
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    if (DT == 0) {
                        const u32 key = word_of(c, d) & 0x7FFFFFFFu;
                        const u32 df = wtop > key ? wtop - key : 0u;
                        lds_inc(min((df >> SHB) & ~3u, (u32)(4 * kCoarseBins - 4)), 1u);
                    } else {
                        const u32 kp = word_of(c, d) & 0x7FFF7FFFu;
                        u32 b = pk_sub_sat_u16(wt2, kp);
                        if (SH) b = pk_shr_u16(b, SH);
                        b = pk_shl_u16(pk_min_u16(b, (u32)(kCoarseBins - 1) * 0x10001u), 2);
                        lds_inc(b & 0xFFFFu, 1u);
                        lds_inc(b >> 16, 1u);
                    }
                }
            }
        }
        __syncthreads();
        if (above && tid == 0) smem[0] -= above;     // keys above the window were counted in bin 0
        __syncthreads();
        // scan from the top: every thread sums its BPT bins; the thread that holds the rank opens them
        constexpr int BPT = kCoarseBins / kWgThreads;
        u32 cs[BPT];
#pragma unroll
        for (int j = 0; j < BPT; ++j) cs[j] = smem[(int)tid * BPT + j];
        u32 local = 0;
#pragma unroll
        for (int j = 0; j < BPT; ++j) local += cs[j];
        u32 total;
        const u32 excl = block_excl_scan<kWgThreads>(local, misc + 32, &total);
        const u32 rem = rank_t - above;
        if (local > 0 && excl <= rem && rem < excl + local) {
            u32 acc = excl;
#pragma unroll
            for (int j = 0; j < BPT; ++j) {
                if (acc <= rem && rem < acc + cs[j]) { misc[0] = tid * BPT + j; misc[1] = acc; misc[2] = cs[j]; misc[3] = 1u; }
                acc += cs[j];
            }
        }
        __syncthreads();
        found = misc[3] != 0u;
        if (found) { B1 = misc[0]; c_gt = misc[1]; cnt1 = misc[2]; }
        __syncthreads();
    };
    hist_pass(std::integral_constant<int, S1>());
    if (found && B1 == (u32)(kCoarseBins - 1) && (wtop >> S1) > (u32)(kCoarseBins - 1)) {
        above = c_gt;
        wtop -= (u32)(kCoarseBins - 1) << S1;
        S = S1 + 4;
        hist_pass(std::integral_constant<int, S1 + 4>());
    }
    c_gt += above;
    const long long lowk = (long long)wtop - ((long long)(B1 + 1u) << S) + 1;
    t_lo = lowk > 1 ? (u32)lowk : 1u;                            // smallest non-zero key of bin B1
    if (k > 0 && lowk >= 1 && (int)(c_gt + cnt1) > cap) {
        give_up();
        return;
    }
    if (k > 0) count_pass();
    }   // !hinted


    // ---- 2. ordered compaction into the list (ascending index) -----------------------------------
    if (k == 0) nL = 0;
    if (k > 0) {
        const u32 C16 = (0x8000u - t_lo) * 0x10001u;
        if ((int)nL > cap) {                                      // uniform
            give_up();
            return;
        }
        const u32 lidx_off = (u32)((u32*)L.Lidx - smem) * 4u;
        u32 linv = 0xFFFFu - tid * (u32)EPC;
        asm volatile("" : "+v"(linv));
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            u32 wa = lent_off + basec[c] * 4u;
            const u32 idx0 = (u32)((c * kWgThreads + (int)tid) * EPC);
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const u32 wd = word_of(c, d);
                if (DT == 0) {
                    const u32 fl = (wd & 0x7FFFFFFFu) >= t_lo ? 1u : 0u;
                    if (fl) {
                        *lds_at(wa) = wd;
                        *(__attribute__((address_space(3))) uint16_t*)(uintptr_t)(lidx_off + ((wa - lent_off) >> 1)) = (uint16_t)(idx0 + d);
                    }
                    wa += fl << 2;
                    continue;
                }
                const u32 f = (wd & 0x7FFF7FFFu) + C16;
                u32 f0 = (f >> 15) & 1u, f1 = f >> 31;
                asm volatile("" : "+v"(f0));
                asm volatile("" : "+v"(f1));
                const u32 i0 = linv - (u32)(c * kWgThreads * EPC + 2 * d), i1 = linv - (u32)(c * kWgThreads * EPC + 2 * d + 1);
                if (f0) *lds_at(wa) = (wd << 16) | i0;
                wa += f0 << 2;
                asm volatile("" : "+v"(wa));
                if (f1) *lds_at(wa) = __builtin_amdgcn_perm(wd, i1, 0x07060100u);   // wd's high half : i1's low half
                wa += f1 << 2;
                asm volatile("" : "+v"(wa));
            }
        }
    }
    __syncthreads();
    // wavefront v takes list slots v, v + 4, ...: entries into registers (sign, key, inverted index in one word)
    const int nslots = (int)((nL + kWave - 1) / kWave);
    u32 ent[kWgSlots], eix[DT == 0 ? kWgSlots : 1];           // fp32: the entry's index beside its raw word
#pragma unroll
    for (int j = 0; j < kWgSlots; ++j) {
        const u32 p = (u32)(j * kWgWaves + (int)wv) * kWave + lane;
        ent[j] = p < nL ? L.Lent[p] : 0u;
        if (DT == 0) eix[DT == 0 ? j : 0] = p < nL ? (u32)L.Lidx[p] : 0u;
    }
    auto ent_key = [&](int j) -> u32 { return DT == 0 ? ent[j] & 0x7FFFFFFFu : (ent[j] >> 16) & 0x7FFFu; };
    auto ent_idx = [&](int j) -> u32 { return DT == 0 ? eix[DT == 0 ? j : 0] : 0xFFFFu - (ent[j] & 0xFFFFu); };
    if (hinted) {                                                 // the row's largest key is the list's largest
        u32 mx = 0;
#pragma unroll
        for (int j = 0; j < kWgSlots; ++j) mx = max(mx, ent[j] & 0x7FFFFFFFu);
        mx = wave_max_dpp(mx) >> (DT == 0 ? 0 : 16);
        if (lane == 0) misc[16 + wv] = mx;
    }
    __syncthreads();                                              // (the histogram region overlays the list's neighbours)
    if (hinted) {
        kmax = 0;
#pragma unroll
        for (int i = 0; i < NW; ++i) kmax = max(kmax, misc[16 + i]);
    }
    {
        uint4* h4 = (uint4*)L.hist;
        for (int i = (int)tid; i < kFineBins / 4; i += kWgThreads) h4[i] = make_uint4(0, 0, 0, 0);
        if (tid < 16) misc[tid] = 0;
        if ((int)tid < QN && (NQ || (int)tid < nq)) L.qtab[tid] = (u32)a.qlist[tid];
        for (int i = (int)tid; i < (nslots * B2 + 1) / 2; i += kWgThreads) ((u32*)stab)[i] = 0;
    }
    __syncthreads();

    // ---- 3. fine bins: 1024 bins linear in (key - t_lo) >> sh, both classes packed 11 + 11 bits --------
    const u32 range = kmax > t_lo ? kmax - t_lo : 0u;
    const int sh = range < (u32)kFineBins ? 0 : (32 - __clz((int)range)) - 10;
    if (DT == 0 && sh + w + 1 > 32) {                             // in-bin key bits, index and class must share a word
        give_up();
        return;
    }
    const u32 inmask = (1u << sh) - 1u, idxmask = (1u << w) - 1u;
#pragma unroll
    for (int j = 0; j < kWgSlots; ++j) {
        const u32 p = (u32)(j * kWgWaves + (int)wv) * kWave + lane;
        if (p < nL) lds_inc(((ent_key(j) - t_lo) >> sh) << 2, (ent[j] >> 31) ? 0x800u : 1u);
    }
    __syncthreads();
    u32 n_pos, n_neg;
    {   // exclusive prefix from the top in the counting format pos | neg << 11 (fill << 22 is added later)
        constexpr int FPT = kFineBins / kWgThreads;     // 4, 2 or 1
        const int hi = kFineBins - (int)tid * FPT;
        u32 cs[FPT];
#pragma unroll
        for (int j = 0; j < FPT; ++j) cs[j] = L.hist[hi - 1 - j];
        u32 local = 0, big = 0;
#pragma unroll
        for (int j = 0; j < FPT; ++j) { local += cs[j]; big |= ((cs[j] & 0x7FFu) + (cs[j] >> 11)) >> 10; }
        if (nL >= 1024u && big != 0u) misc[10] = 1u;        // a fine bin with 1024+ members overflows its 10-bit fill field
        __syncthreads();                                    // (no library reduction here: it would bring static LDS)
        if (misc[10]) {
            give_up();
            return;
        }
        u32 tot;
        const u32 excl = block_excl_scan<kWgThreads>(local, misc + 32, &tot);
        n_pos = tot & 0x7FFu; n_neg = tot >> 11;
        const u32 incl = excl + local;
        const u32 ov_ex = (excl & 0x7FFu) + (excl >> 11), ov_in = (incl & 0x7FFu) + (incl >> 11);
        if (k > 0 && ov_ex <= (u32)(k - 1) && (u32)(k - 1) < ov_in) misc[5] = tid;     // the thread whose bins hold overall rank k-1
        u32 acc = excl, o[FPT];
#pragma unroll
        for (int j = 0; j < FPT; ++j) { o[j] = acc; acc += cs[j]; }
#pragma unroll
        for (int j = 0; j < FPT; ++j) L.hist[hi - 1 - j] = o[j];
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kWgSlots; ++j) {
        const u32 p = (u32)(j * kWgWaves + (int)wv) * kWave + lane;
        if (p < nL) {
            const u32 e = ent[j];
            const u32 rel = ent_key(j) - t_lo;
            const u32 old = atomicAdd(&L.hist[rel >> sh], 1u << 22);
            const u32 at = (old & 0x7FFu) + ((old >> 11) & 0x7FFu) + (old >> 22);
            if (DT == 0) L.S[at] = ((((rel & inmask) << w) | (idxmask - ent_idx(j))) << 1) | (e >> 31);
            else L.S[at] = e;
        }
    }
    __syncthreads();
    // members of a fine bin compare on the plain comp; their class; their class-extended comp
    auto s_plain = [&](u32 s) -> u32 { return DT == 0 ? s >> 1 : s & 0x7FFFFFFFu; };
    auto s_neg = [&](u32 s) -> u32 { return DT == 0 ? s & 1u : s >> 31; };
    auto s_cx = [&](u32 s, u32 bin) -> comp_t {
        if (DT == 0) {
            const u32 key = ((bin << sh) | ((s >> 1) >> w)) + t_lo;
            const u32 idx = idxmask - ((s >> 1) & idxmask);
            return ((comp_t)(key | ((s & 1u) ? 0u : 0x80000000u)) << kHiShift) | (comp_t)(u32)(~idx);
        }
        return (comp_t)(s ^ 0x80000000u);
    };

    // ---- top-K cut and block boundaries: wavefront 0 ------------------------------------------------
    const int ntg = B2 - 2;
    comp_t* thr = (comp_t*)L.thr;
    if (wv == 0) {
        comp_t thrK = 0;                                // plain comp; every entry of the list is kept when nL <= k
        if (nL > (u32)k) {
            constexpr int FPT = kFineBins / kWgThreads;
            const int hi = kFineBins - (int)misc[5] * FPT;
            const u32 wj = lane < (u32)FPT ? L.hist[hi - 1 - (int)lane] : 0xFFFFFFFFu;
            const u64 mj = __ballot(lane < (u32)FPT && (wj & 0x7FFu) + ((wj >> 11) & 0x7FFu) <= (u32)(k - 1));
            const int lo = hi - (int)__popcll(mj);
            const u32 wd = L.hist[lo];
            const u32 pe = wd & 0x7FFu, ne = (wd >> 11) & 0x7FFu, cnt = wd >> 22, base = pe + ne;
            const u32 rem = (u32)(k - 1) - base;
            u32 kp = 0, kn = 0;
            for (u32 g = 0; g < cnt; g += kWave) {
                const u32 i = g + lane;
                u32 me = 0, gt = 0;
                if (i < cnt) {
                    me = L.S[base + i];
                    for (u32 j = 0; j < cnt; ++j) gt += s_plain(L.S[base + j]) > s_plain(me) ? 1u : 0u;
                }
                const bool in = i < cnt && gt <= rem;
                kp += (u32)__popcll(__ballot(in && !s_neg(me)));
                kn += (u32)__popcll(__ballot(in && s_neg(me)));
                const u64 hit = __ballot(i < cnt && gt == rem);
                if (hit) {
                    const int hl = (int)__builtin_ctzll(hit);
                    const comp_t cx = s_cx(me, (u32)lo) & ~kClsBit;
                    if (DT == 0) thrK = ((comp_t)bcast((u32)((u64)cx >> kHiShift), hl) << kHiShift) | (comp_t)bcast((u32)cx, hl);
                    else thrK = (comp_t)bcast((u32)cx, hl);
                }
            }
            n_pos = pe + kp; n_neg = ne + kn;
        }
        const u32 Kc[2] = { n_pos / (u32)M, n_neg / (u32)Mn };
        if (lane == 0) { misc[6] = (u32)thrK; misc[11] = (u32)((u64)thrK >> kHiShift); misc[7] = n_pos; misc[8] = n_neg; }
        // boundaries: comps of class ranks j*K-1, one lane per boundary
        const int ntp = ntg > 0 ? ntg : 1;
        u32* tg_bin = L.tg; u32* tg_base = L.tg + ntp; u32* tg_cnt = L.tg + 2 * ntp; u32* tg_rem = L.tg + 3 * ntp; u32* tg_pre = L.tg + 4 * ntp;
        const bool mine = (int)lane < ntg;
        const int cls = (int)lane >= M - 1 ? 1 : 0;
        const int jb = (cls ? (int)lane - (M - 1) : (int)lane) + 1;
        const bool act = mine && Kc[cls] > 0;
        const u32 Rk = act ? (u32)jb * Kc[cls] - 1u : 0u;
        int lo = 0, hi = kFineBins - 1;                 // smallest bin whose first class rank is <= Rk
        for (int it = 0; it < 10; ++it) {
            const int mid = (lo + hi) >> 1;
            const u32 wd = L.hist[mid];
            const u32 pc = cls ? (wd >> 11) & 0x7FFu : wd & 0x7FFu;
            if (pc <= Rk) hi = mid; else lo = mid + 1;
        }
        const u32 wd = L.hist[lo];
        const u32 pe = wd & 0x7FFu, ne = (wd >> 11) & 0x7FFu;
        const u32 cnt = act ? wd >> 22 : 0u;
        const u32 incl = wave_scan_dpp(cnt);
        if (mine) {
            tg_bin[lane] = (u32)lo; tg_base[lane] = pe + ne; tg_cnt[lane] = cnt;
            tg_rem[lane] = Rk - (cls ? ne : pe);
            tg_pre[lane] = incl - cnt;
            if (!act) thr[lane] = cls ? (comp_t)(kClsBit - 1) : ~(comp_t)0;
        }
        const u32 npairs = bcast(incl, kWave - 1);
        wave_sync();
        for (u32 g = 0; g < npairs; g += kWave) {
            const u32 pr = g + lane;
            if (pr < npairs) {
                int tl = 0, th = ntg - 1;
                while (tl < th) {
                    const int mid = (tl + th + 1) >> 1;
                    if (tg_pre[mid] <= pr) tl = mid; else th = mid - 1;
                }
                const int t = tl;
                const u32 tc = (u32)(t >= M - 1 ? 1 : 0);
                const u32 bs = tg_base[t], cn = tg_cnt[t];
                const u32 me = L.S[bs + (pr - tg_pre[t])];
                if (s_neg(me) == tc) {
                    // one compare per member: with the class bit moved to the top and set for the boundary's
                    // class, "same class and larger comp" is a plain unsigned "larger"
                    const u32 fm = DT == 0 ? (tc ^ 1u) : (tc ? 0u : 0x80000000u);
                    auto key_of = [&](u32 sv) -> u32 {
                        const u32 xv = sv ^ fm;
                        return DT == 0 ? __builtin_amdgcn_alignbit(xv, xv, 1) : xv;     // fp32: rotate the class bit up
                    };
                    const u32 mk = key_of(me);
                    u32 gt = 0;
                    for (u32 jj = 0; jj < cn; ++jj) gt += key_of(L.S[bs + jj]) > mk ? 1u : 0u;
                    if (gt == tg_rem[t]) thr[t] = s_cx(me, tg_bin[t]);
                }
            }
        }
    }
    __syncthreads();
    const comp_t thrK = DT == 0 ? (comp_t)(((u64)misc[11] << kHiShift) | (u64)misc[6]) : (comp_t)misc[6];
    n_pos = misc[7]; n_neg = misc[8];
    const u32 n = n_pos + n_neg;
    const u32 Kc[2] = { n_pos / (u32)M, n_neg / (u32)Mn };
    if ((int)tid < B2) {
        const int s = (int)tid >= M ? 1 : 0, m = (int)tid - s * M;
        L.blk_start[tid] = (s ? n_pos : 0u) + (u32)m * Kc[s];
        L.vminb[tid] = 0xFFFFFFFFu; L.vmaxb[tid] = 0;
    }
    if (tid == 0) L.blk_start[B2] = n;

    // ---- 4. blocks and stable split -----------------------------------------------------------------
    u32* bo_val = L.S;
    uint16_t* bo_idx = (uint16_t*)(L.hist);
    u32* stage = L.hist + (k + 1) / 2;
    int nbits = 0;
    while ((1 << nbits) < B2) ++nbits;
    comp_t tx[kRegThr];
#pragma unroll
    for (int j = 0; j < kRegThr; ++j) tx[j] = j < ntg ? thr[j] : (comp_t)0;
    const bool tree8 = DT == 1 && M == 8 && Mn == 8;      // (one-word comps: a select is one instruction)
    __syncthreads();                                 // S, the fine bins and the boundaries have been read: their storage is reused
    u32 info[kWgSlots];                              // kept << 31 | block << 16 | entries of the same block before this one in the slot
#pragma unroll
    for (int j = 0; j < kWgSlots; ++j) {
        const int slot = j * kWgWaves + (int)wv;
        const u32 p = (u32)slot * kWave + lane;
        bool kept = false;
        u32 b = 0;
        if (slot < nslots && p < nL) {
            const comp_t cx = DT == 0 ? ((comp_t)(ent[j] ^ 0x80000000u) << kHiShift) | (comp_t)(u32)(~ent_idx(j))
                                      : (comp_t)(ent[j] ^ 0x80000000u);
            if ((cx & ~kClsBit) >= thrK) {
                kept = true;
                u32 abv;
                if (tree8) {
                    const bool c1 = !(cx & kClsBit);
                    comp_t m = c1 ? tx[10] : tx[3];
                    const bool c2 = m > cx;
                    m = c1 ? (c2 ? tx[12] : tx[8]) : (c2 ? tx[5] : tx[1]);
                    const bool c3 = m > cx;
                    const comp_t lo4 = c3 ? (c2 ? tx[6] : tx[2]) : (c2 ? tx[4] : tx[0]);
                    const comp_t hi4 = c3 ? (c2 ? tx[13] : tx[9]) : (c2 ? tx[11] : tx[7]);
                    m = c1 ? hi4 : lo4;
                    const bool c4 = m > cx;
                    abv = (c1 ? 8u : 0u) + (c2 ? 4u : 0u) + (c3 ? 2u : 0u) + (c4 ? 1u : 0u);
                } else {
                    abv = (cx & kClsBit) ? 0u : 1u;
#pragma unroll
                    for (int t = 0; t < kRegThr; ++t) abv += tx[t] > cx ? 1u : 0u;
                    for (int t = kRegThr; t < ntg; ++t) abv += thr[t] > cx ? 1u : 0u;
                }
                b = abv;
                const u32 key = ent_key(j);
                atomicMin(&L.vminb[b], key);
                atomicMax(&L.vmaxb[b], key);
            }
        }
        if (slot < nslots) {                         // uniform in the wavefront
            const u64 km = __ballot(kept);
            u32 plo = (u32)km, phi = (u32)(km >> 32);
            for (int bit = 0; bit < nbits; ++bit) {
                const u32 onm = (u32)__builtin_amdgcn_sbfe((int)b, (u32)bit, 1u);
                const u64 bal = __ballot(onm != 0u);
                plo &= ~((u32)bal ^ onm);
                phi &= ~((u32)(bal >> 32) ^ onm);
            }
            const u32 before = __builtin_amdgcn_mbcnt_hi(phi, __builtin_amdgcn_mbcnt_lo(plo, 0u));
            if (kept && before == 0) stab[slot * B2 + (int)b] = (uint16_t)(__popc(plo) + __popc(phi));
            info[j] = (kept ? 0x80000000u : 0u) | (b << 16) | before;
        } else {
            info[j] = 0;
        }
    }
    __syncthreads();
    if ((int)tid < B2) {                             // per block: entries in earlier slots
        u32 acc = 0;
        for (int s = 0; s < nslots; ++s) {
            const u32 c = stab[s * B2 + (int)tid];
            stab[s * B2 + (int)tid] = (uint16_t)acc;
            acc += c;
        }
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kWgSlots; ++j) {
        const int slot = j * kWgWaves + (int)wv;
        if (info[j] >> 31) {
            const u32 b = (info[j] >> 16) & 0x7FFFu, before = info[j] & 0xFFFFu;
            const u32 pos = L.blk_start[b] + (u32)stab[slot * B2 + (int)b] + before;
            bo_val[pos] = E::value_bits(ent_key(j));             // |x| as fp32 bits (bf16: exact widening)
            bo_idx[pos] = (uint16_t)ent_idx(j);
        }
    }
    __syncthreads();

    // ---- 5. ABQ: each block is walked by (64 NW) / B2 threads ---------------------------------------
    u64* sums = (u64*)(L.hist + ((((k + 1) / 2 + (int)a.cap_words) + 1) & ~1));
    float* invt = (float*)(sums + B2 * (nq + 1));
    const u32 lpb = (u32)kWgThreads / (u32)B2;
    // every row of 16 lanes then lies inside one block's threads: the lanes' sums are added up across the row
    // first (16 lanes meeting on one LDS address cost more than the whole loop), and lane 15 adds to the table
    const bool row_one_block = lpb % 16u == 0u;
    const bool row_last = (lane & 15u) == 15u;
    const u32 myb = udiv16(tid, lpb), sub = tid - myb * lpb;
    const bool on = myb < (u32)B2;
    u32 r0 = 0, r1 = 0, bs0 = 0, mycnt = 0;
    float vmin = 0.f, rng = 0.f, rng1 = 1.f;
    int e = 0, dg = 1, er = 0;
    u32 vmaxbits = 0;
    if (on) {
        bs0 = L.blk_start[myb];
        const u32 be = L.blk_start[myb + 1];
        mycnt = be - bs0;
        const u32 perb = udiv16(mycnt + lpb - 1, lpb);
        r0 = bs0 + sub * perb; r0 = r0 < be ? r0 : be;
        r1 = r0 + perb < be ? r0 + perb : be;
        if (mycnt) {
            vmaxbits = E::value_bits(L.vmaxb[myb]);
            vmin = __uint_as_float(E::value_bits(L.vminb[myb]));
            rng = __uint_as_float(vmaxbits) - vmin;
            dg = !(rng > 0.f);                       // only a range of exactly 0 is degenerate
            if (!dg) { er = range_exp(rng); rng1 = unit_range(rng, er); }
            e = ilogb_bits(vmaxbits) + 1;
        }
    }
    const u32 mc0 = n_pos - Kc[0] * (u32)(M - 1), mc1 = n_neg - Kc[1] * (u32)(Mn - 1);
    const u32 T = udiv16((mc0 > mc1 ? mc0 : mc1) + lpb - 1, lpb);
    __syncthreads();                                 // vminb / vmaxb / run have been read before `run` is reused below
    if (on) {
        for (u32 t = sub; t < (u32)nq; t += lpb) {
            const float Lq = (float)((1u << L.qtab[t]) - 1u);
            invt[myb * (u32)nq + t] = dg ? 0.f : Lq / rng1;
        }
        if (sub == 0) {
            for (int t = 0; t <= nq; ++t) sums[myb * (nq + 1) + t] = 0;
            // budget guard: index of the chosen bitwidth, nq = none feasible yet; DS guard: mask of violations
            L.run[myb] = (mycnt && !dg && a.guard == 0) ? (u32)nq : 0u;
        }
    }
    __syncthreads();
    float inv[QN];
    bool small_q = true;
#pragma unroll
    for (int t = 0; t < QN; ++t) {
        inv[t] = (on && (NQ || t < nq)) ? invt[myb * (u32)nq + t] : 0.f;
        if ((NQ || t < nq) && a.qlist[t] > 8) small_q = false;
    }
    if (!a.lad.on && a.guard == 1) {
        // Eq. "DS": sum over the block of | (code at q_bit >> (q_bit - q)) - code at q | for every lower bitwidth
        const int top = nq - 1, qtop = (int)L.qtab[top];
        const float inv_top = on ? invt[myb * (u32)nq + (u32)top] : 0.f;
        for (u32 i0 = 0; i0 < T; i0 += 8) {             // 8 differences below 2^16 each
            u32 acc[QN];
#pragma unroll
            for (int t = 0; t < QN; ++t) acc[t] = 0;
            const u32 i1 = i0 + 8 < T ? i0 + 8 : T;
            for (u32 i = i0; i < i1; ++i) {
                const u32 p = r0 + i;
                if (p < r1) {
                    const float d = to_unit(__uint_as_float(bo_val[p]) - vmin, er);
                    const u32 c0 = (u32)rintf(d * inv_top);           // within [0, 2^q - 1]: no clamp needed
#pragma unroll
                    for (int t = 0; t < QN; ++t) {
                        if ((NQ || t < nq) && t < top) {
                            const u32 c = (u32)rintf(d * inv[t]);
                            const u32 ref = c0 >> (u32)(qtop - a.qlist[t]);
                            acc[t] += ref > c ? ref - c : c - ref;
                        }
                    }
                }
            }
#pragma unroll
            for (int t = 0; t < QN; ++t) {
                if ((NQ || t < nq) && t < top) {
                    if (row_one_block) {                             // 16 lane sums below 2^19 fit 32 bits
                        const u32 tot = row_scan_dpp(acc[t]);
                        if (row_last && tot) atomicAdd(&sums[myb * (nq + 1) + t], (u64)tot);
                    } else if (acc[t]) {
                        atomicAdd(&sums[myb * (nq + 1) + t], (u64)acc[t]);
                    }
                }
            }
        }
    } else if (!a.lad.on) {
        // residual on the 2^-15 grid: rint(y * 2^15) reduced to 15 signed bits; bitwidths up to 8 keep
        // y * 2^15 below 2^23, where adding 2^23 rounds to the integer grid with the same round-half-even
        float inv15[QN];
#pragma unroll
        for (int t = 0; t < QN; ++t) inv15[t] = inv[t] * 32768.0f;
        u64 accE = 0;
        for (u32 i0 = 0; i0 < T; i0 += 8) {             // u32 partial sums hold 8 residuals of 2^28
            u32 acc[QN];
#pragma unroll
            for (int t = 0; t < QN; ++t) acc[t] = 0;
            const u32 i1 = i0 + 8 < T ? i0 + 8 : T;
            for (u32 i = i0; i < i1; ++i) {
                const u32 p = r0 + i;
                if (p < r1) {
                    const float av = __uint_as_float(bo_val[p]);
                    const u64 A = (u64)(u32)rintf(ldexpf(av, 20 - e));   // 20-bit energy grid scaled to vmax
                    accE += A * A;
                    const float d = to_unit(av - vmin, er);
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
            if (row_one_block) {
                // 16-bit pieces, so that the sums over a row fit 32 bits
#pragma unroll
                for (int t = 0; t < QN; ++t) {
                    if (NQ || t < nq) {
                        const u32 lo16 = row_scan_dpp(acc[t] & 0xFFFFu);
                        const u32 hi16 = row_scan_dpp(acc[t] >> 16);
                        if (row_last && (lo16 | hi16)) atomicAdd(&sums[myb * (nq + 1) + t], (u64)lo16 + ((u64)hi16 << 16));
                    }
                }
            } else {
#pragma unroll
                for (int t = 0; t < QN; ++t)
                    if ((NQ || t < nq) && acc[t]) atomicAdd(&sums[myb * (nq + 1) + t], (u64)acc[t]);
            }
        }
        if (row_one_block) {
            const u32 e0 = row_scan_dpp((u32)accE & 0x3FFFFFu);
            const u32 e1 = row_scan_dpp((u32)(accE >> 22) & 0x3FFFFFu);
            const u32 e2 = row_scan_dpp((u32)(accE >> 44));
            if (row_last && (e0 | e1 | e2)) atomicAdd(&sums[myb * (nq + 1) + nq], (u64)e0 + ((u64)e1 << 22) + ((u64)e2 << 44));
        } else if (accE) {
            atomicAdd(&sums[myb * (nq + 1) + nq], accE);
        }
    }
    __syncthreads();
    if (a.lad.on) {
        if (on && sub == 0) L.run[myb] = ladder_index(a.lad, (int)(myb >= (u32)M ? myb - (u32)M : myb));
    } else if (a.guard == 1) {
        // greedy descent: the chosen index is one above the highest violating candidate below q_bit
        if (on && mycnt && !dg) {
            for (u32 t = sub; t + 1 < (u32)nq; t += lpb)
                if (!((double)sums[myb * (nq + 1) + t] <= a.beta * (double)mycnt)) atomicOr(&L.run[myb], 1u << t);
        }
        __syncthreads();
        if (on && sub == 0) {
            const u32 viol = L.run[myb];
            L.run[myb] = viol ? 32u - (u32)__clz((int)viol) : 0u;
        }
    } else if (on && mycnt && !dg) {
        const double rhs = a.beta * ldexp((double)sums[myb * (nq + 1) + nq], 2 * e - 40);
        for (u32 t = sub; t < (u32)nq; t += lpb) {
            const float Lq = (float)((1u << L.qtab[t]) - 1u);
            const float o = rng / Lq;
            const double lhs = ((double)o * (double)o) * (double)sums[myb * (nq + 1) + t] * 0x1p-30;
            if (lhs <= rhs) { atomicMin(&L.run[myb], t); break; }
        }
    }
    __syncthreads();
    u32 myq = 0, flag = 0;
    float my_inv = 0.f;
    if (on) {
        u32 tb = L.run[myb];
        if (tb == (u32)nq) { flag = 0x80u; tb = (u32)nq - 1u; }   // none feasible: the largest bitwidth, flagged
        myq = L.qtab[tb];
        my_inv = invt[myb * (u32)nq + tb];
    }
    if (on && sub == 0) {
        const size_t mi = (size_t)r * (size_t)B2 + myb;
        a.mv.vmin[mi] = mycnt ? vmin : 0.f;
        a.mv.vmax[mi] = mycnt ? __uint_as_float(vmaxbits) : 0.f;
        a.mv.q[mi] = (uint8_t)(myq | flag);
        L.thr[myb] = mycnt * myq;                    // code bits of the block (the boundaries are dead)
    }
    __syncthreads();
    if (wv == 0) {                                   // bit offsets of the blocks' code sections
        const u32 bits = (int)lane < B2 ? L.thr[lane] : 0u;
        const u32 incl = wave_scan_dpp(bits);
        if ((int)lane < B2) L.tg[lane] = incl - bits;
        if (lane == kWave - 1) misc[9] = incl;
    }
    __syncthreads();
    const u32 code_bits = misc[9];
    const u32 coff = on ? L.tg[myb] : 0u;
    const u32 idx_bits = n * (u32)w;
    const u32 row_bits = idx_bits + code_bits;
    u32 row_words = (row_bits + 31u) >> 5;
    if ((u64)row_words > a.cap_words) row_words = (u32)a.cap_words;   // cannot happen (worst-case capacity)
    __syncthreads();                                 // sums and scales have been read: the stage image overlays nothing live
    for (u32 i = tid; i < row_words; i += kWgThreads) stage[i] = 0;
    __syncthreads();

    // ---- packing ---------------------------------------------------------------------------------
    for (u32 i = 0; i < T; ++i) {
        const u32 p = r0 + i;
        if (p < r1) {
            u32 c = 0;
            if (!dg) c = (u32)rintf(to_unit(__uint_as_float(bo_val[p]) - vmin, er) * my_inv);   // already within [0, 2^q - 1]
            {
                const u32 P = __umul24(p, (u32)w), wi = P >> 5, sft = P & 31u, val = bo_idx[p];
                atomicOr(&stage[wi], val << sft);
                if (sft + (u32)w > 32u) atomicOr(&stage[wi + 1], val >> (32u - sft));
            }
            {
                const u32 P = idx_bits + coff + __umul24(p - bs0, myq), wi = P >> 5, sft = P & 31u;
                atomicOr(&stage[wi], c << sft);
                if (sft + myq > 32u) atomicOr(&stage[wi + 1], c >> (32u - sft));
            }
        }
    }
    __syncthreads();
    u32* __restrict__ slot = a.slots + (size_t)r * (size_t)a.cap_words;
    for (u32 i = tid; i < row_words; i += kWgThreads) slot[i] = stage[i];
    if (tid == 0) {
        a.row_words[r] = row_words;
        a.mv.n_pos[r] = n_pos;
        a.mv.n_neg[r] = n_neg;
        a.fallback[r] = 0u;
        if (k > 0) a.hint[hslot] = nL > (u32)k ? (DT == 0 ? (u32)((u64)thrK >> kHiShift) & 0x7FFFFFFFu : ((u32)thrK >> 16) & 0x7FFFu)
                                               : t_lo;           // this row's cut key, for a later row
    }
}

}  // namespace slicer
