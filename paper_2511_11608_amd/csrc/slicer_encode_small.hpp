// Row-resident encoder for short rows: ONE WAVEFRONT PER ROW, the row held in
// registers, every list in LDS, no workgroup barrier anywhere.
//
// All ordering is done on one integer per element, the "comp": magnitude key in the high
// bits, inverted index in the low bits (larger comp = larger magnitude, then lower index:
// the tie rule of the top-K filter and of the block ranks), and the sign class as the top
// bit, positive class on top.  Comps are distinct, so a comp is a complete rank threshold.
//
//   1. load the row (16-byte coalesced loads); its largest magnitude key; a 2048-bin
//      histogram in LDS over a window that hangs from that key (bf16: one key per bin);
//      two-level scan from the top -> the bin B1 that holds rank k-1;
//   2. ordered compaction of everything at or above B1 into a short list L
//      (ascending index: the kept set plus the undecided bin);
//   3. L is bucketed into 1024 fine bins, linear in the key from the list's lower
//      bound, both sign classes counted in one packed table; an exclusive scan from
//      the top gives every bin's first rank, overall and per class.  Order
//      statistics (rank k-1 overall for the top-K cut of Sec. 3.1; ranks j*K-1 per
//      class for the block boundaries of Sec. 3.2) are located over the bins, one lane
//      per boundary, and resolved inside their bin by comparing the bin's few members
//      pairwise;
//   4. an entry's block is the number of boundaries above it (plus one for the negative
//      class); a stable split by block id (wave ballots) restores ascending index inside
//      each block;
//   5. ABQ sums on integer grids, bitwidth choice, bit offsets, packing through an
//      LDS image of the row's stream segment.
//
// Rows the list cannot hold (heavy ties around the threshold, more zeros than
// dropped elements, ...) are flagged and redone by the generic kernel.
#pragma once

#include <type_traits>

#include "slicer_common.hpp"

namespace slicer {

struct SmallArgs {
    const void* x;
    int64_t R, N, k;
    int M, Mn, w, nq;   // blocks of the positive / negative class
    int qlist[kMaxQ];
    double beta;
    u64 cap_words;
    u64* row_words;     // [R]
    u32* slots;         // [R][cap_words]
    u32* fallback;      // [R] 1 = redo this row with the generic kernel
    MetaView mv;
    int cap;            // list capacity, multiple of 64, < 2048
    int region0_words;  // fine histogram, later block-ordered indices + stream image
    Ladder lad;         // fixed multi-level mode: no sums, no search
    int guard;          // 0: relative squared-error budget; 1: DS mismatch of Eq. "DS", greedy descent (beta = delta)
    float one_plus, one_minus;   // asymmetric thresholds of Sec. 3.1 (ASYM kernels): 1 + lambda, 1 - lambda in fp32
    u32* hint;          // [kHintSlots] cut keys of rows encoded earlier with this workspace (any contents are safe)
};

// Threshold hints.  Rows of one tensor (tokens of one sequence, successive decode steps) have their
// top-K cut at nearly the same magnitude, so a wave first tries the cut key some earlier row left in
// the workspace, lowered by kHintDelta steps of the key's top 15 bits: if the number of keys at or
// above it lies in [k, k + kHintSlack] the list is built from it directly, and the row's largest key,
// the 2048-bin histogram and its scan are skipped.  The count decides, not the hint: a stale,
// foreign or garbage value only sends the row down the histogram path, and the output never depends on it.
constexpr int kHintSlots = 512;
constexpr u32 kHintDelta = 8;
constexpr u32 kHintSlack = 120;

constexpr int kCoarseBits = 11;
constexpr int kCoarseBins = 1 << kCoarseBits;
constexpr int kFineBins = 1024;

// LDS carve-up of one wave (word offsets); small_lds_words() on the host must match.
// The coarse histogram (2048 16-bit counters) overlays everything: nothing else is live before the
// compaction.  Region 0 is the fine histogram first; once the boundaries are known it holds
// the block-ordered indices, the stream image, the ABQ sums and the quantiser scales.
// MAXS > 0: the list is copied into registers after the compaction, so the bin-ordered
// list S reuses the storage of L.
struct SmallLds {
    u32* hist;      // [region0]   fine histogram; later bo_idx, stream image, sums, invt
    u32* Lent;      // [cap]       list entries, ascending index: bf16 raw << 16 | ~idx; fp32 raw
    u32* S;         // [cap]       entries arranged by fine bin; later bo_val
    uint16_t* Lidx; // [cap]       fp32 only: index of the entry (inside region 0 when MAXS > 0)
    u32* thr;       // [2 * B2]    block boundaries (class-extended comps), positive class first
    u32* tg;        // [5][ntg]    boundary work table: bin, base, count, rank in bin, pair prefix
    u32* qtab;      // [16]        allowed bitwidths
    u32* blk_start; // [B2 + 1]
    u32* vminb;     // [B2] key of the block's smallest / largest element
    u32* vmaxb;     // [B2]
    u32* run;       // [B2]        next free position of the block; later the chosen bitwidth index
};

__host__ __device__ inline int small_tg_words(int B2)
{
    const int ntg = B2 > 2 ? B2 - 2 : 1;
    return (5 * ntg + 1) & ~1;
}

// words of region 0: fine histogram, or indices + stream image + sums + scales
__host__ __device__ inline int small_region0_words(int64_t k, u64 cap_words, int B2, int nq)
{
    const int64_t late = (((k + 1) / 2 + (int64_t)cap_words + 1) & ~(int64_t)1) + 2 * B2 * (nq + 1) + B2 * nq;
    const int64_t r0 = late > kFineBins ? late : kFineBins;
    return (int)((r0 + 1) & ~(int64_t)1);
}

// floor: words of the coarse histogram, which overlays the carve-up (16-bit counters in the one-wavefront
// kernel: kCoarseBins / 2; 32-bit counters in the workgroup-per-row kernel: kCoarseBins)
__host__ __device__ inline int small_lds_words(int dt, int cap, int region0, int B2, int maxs, int floor = kCoarseBins / 2)
{
    int wds = region0 + cap + (maxs ? 0 : cap) + ((dt == 0 && !maxs) ? cap / 2 : 0);
    wds += 2 * B2 + small_tg_words(B2) + 16;
    wds += (B2 + 1) + B2 * 3;
    if (wds < floor) wds = floor;
    return wds;
}

__device__ inline SmallLds small_carve(u32* base, int dt, int cap, int region0, int B2, int maxs)
{
    SmallLds L;
    u32* p = base;
    L.hist = p;            p += region0;           // region0 is even
    L.Lent = p;            p += cap;
    L.S = maxs ? L.Lent : p;
    p += maxs ? 0 : cap;
    L.Lidx = maxs ? (uint16_t*)base : (uint16_t*)p;
    p += (dt == 0 && !maxs) ? cap / 2 : 0;
    L.thr = p;             p += 2 * B2;            // cap is a multiple of 64: still 8-byte aligned
    L.tg = p;              p += small_tg_words(B2);
    L.qtab = p;            p += 16;
    L.blk_start = p;       p += B2 + 1;
    L.vminb = p;           p += B2;
    L.vmaxb = p;           p += B2;
    L.run = p;             p += B2;
    return L;
}

// LDS by byte offset: dynamic shared memory starts at offset 0 when the kernel has no static
// LDS (checked at run time), so an address computed as an integer needs no base register.
typedef __attribute__((address_space(3))) u32 lds_u32;
__device__ inline lds_u32* lds_at(u32 byte_off) { return (lds_u32*)(uintptr_t)byte_off; }
__device__ inline void lds_inc(u32 byte_off, u32 v)
{
    __hip_atomic_fetch_add(lds_at(byte_off), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

// NQ > 0: the number of allowed bitwidths is known at compile time (loops over the
// candidate bitwidths unroll without predicates); NQ == 0: any number up to 16.
// MAXS > 0: the list has at most 64 * MAXS entries and lives in registers.
// ASYM: the asymmetric thresholds of Sec. 3.1 with lambda > 0.  The kept set is not a
// plain top-K then: after the first selection has given tau, the strict set is counted, a second
// selection over a subset of the row (the fill candidates, or the strict set when it is too large)
// gives the last key taken, and the list is built from that rule; the equal keys at the end are cut
// in index order.  Both selections need the exact key of their rank, i.e. one key per histogram bin:
// rows whose ranks lie below the 2048-key window are flagged for the generic kernel.
// Wavefronts per SIMD the register allocator must leave room for.  The variants that hold the row in at most
// 32 registers come out at 84 to 101 VGPRs, a few of them just above the limit of five wavefronts (96 VGPRs):
// asking for five costs those a handful of spill moves outside every loop.  fp32 rows of 4096 elements (64
// registers for the row, 166 to 181 in all) are asked for three wavefronts (168) instead of two.
constexpr int small_min_waves(int dt, int epl, int nq, int maxs, bool asym)
{
    const int row_regs = dt == 0 ? epl : epl / 2;
    return row_regs <= 32 ? 5 : (dt == 0 && row_regs == 64) ? 3 : 1;
}

template <int DT, int EPL, int NQ, int MAXS, bool ASYM = false>
__global__ __launch_bounds__(kWave) __attribute__((amdgpu_waves_per_eu(small_min_waves(DT, EPL, NQ, MAXS, ASYM)))) void enc_small_kernel(SmallArgs a)
{
    typedef Elem<DT> E;
    typedef typename std::conditional<DT == 0, u64, u32>::type comp_t;   // bf16: key + index fit 31 bits
    constexpr comp_t kClsBit = (comp_t)1 << (8 * sizeof(comp_t) - 1);       // set for the positive class
    constexpr int kHiShift = DT == 0 ? 32 : 0;                               // position of the key word in a comp
    constexpr int kRegThr = 14;                                              // boundaries held in registers
    constexpr int QN = NQ ? NQ : kMaxQ;
    constexpr int EPC = DT == 0 ? 4 : 8;            // elements per 16-byte chunk
    constexpr int NCH = EPL / EPC;                  // chunks per lane
    extern __shared__ u32 smem[];

    const u32 lane = lane_id();
    const int64_t r = xcd_row((int64_t)blockIdx.x, a.R);        // neighbouring rows stay on one XCD
    if (r >= a.R) return;
    const int N = (int)a.N, M = a.M, Mn = a.Mn, w = a.w, B2 = a.M + a.Mn, nq = NQ ? NQ : a.nq, cap = a.cap;
    const int k = (int)a.k;
    const u32 idxmask = (1u << w) - 1u;
    SmallLds L = small_carve(smem, DT, cap, a.region0_words, B2, MAXS);
    if (__builtin_amdgcn_groupstaticsize() != 0u) {             // integer LDS addresses assume offset 0
        if (lane == 0) a.fallback[r] = 1u;
        return;
    }
    const u32 lent_off = (u32)(L.Lent - smem) * 4u;

    // ---- list entry accessors ---------------------------------------------------------------
    // bf16: one word holds sign, key and inverted index, i.e. the comp with the class bit flipped
    constexpr int SLN = MAXS ? MAXS : 32;          // slots of 64 entries (cap < 2048)
    u32 ent[MAXS ? MAXS : 1], eix[(MAXS && DT == 0) ? MAXS : 1];
    auto ent_word = [&](int s) -> u32 { return MAXS ? ent[MAXS ? s : 0] : L.Lent[s * kWave + (int)lane]; };
    auto ent_index = [&](int s) -> u32 {          // fp32 only
        return MAXS ? eix[(MAXS && DT == 0) ? s : 0] : (u32)L.Lidx[s * kWave + (int)lane];
    };
    auto ent_cx = [&](int s) -> comp_t {          // class-extended comp of this lane's entry of slot s
        if (DT == 0) return ((comp_t)(ent_word(s) ^ 0x80000000u) << kHiShift) | (comp_t)(u32)(~ent_index(s));
        return (comp_t)(ent_word(s) ^ 0x80000000u);
    };
    auto cx_key = [&](comp_t cx) -> u32 {         // magnitude key
        if (DT == 0) return (u32)((u64)cx >> kHiShift) & 0x7FFFFFFFu;
        return ((u32)cx >> 16) & 0x7FFFu;
    };
    auto cx_idx = [&](comp_t cx) -> u32 {
        if (DT == 0) return ~(u32)cx;
        return 0xFFFFu - ((u32)cx & 0xFFFFu);
    };

    // ---- 1. load the row, coarse histogram ------------------------------------------
    const uint4* __restrict__ xr = (const uint4*)((const char*)a.x + (size_t)r * (size_t)N * (DT == 0 ? 4 : 2));
    uint4 v[NCH];
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int base = (c * kWave + (int)lane) * EPC;
        v[c] = base < N ? xr[c * kWave + lane] : make_uint4(0, 0, 0, 0);
    }
    auto word_of = [&](int c, int d) -> u32 { return d == 0 ? v[c].x : d == 1 ? v[c].y : d == 2 ? v[c].z : v[c].w; };
    constexpr bool kHint = !ASYM && MAXS > 0;       // (the list must be in registers: its largest key is taken from there)
    const u32 hslot = (u32)blockIdx.x & (u32)(kHintSlots - 1);
    u32 hint_key = 0;
    if (kHint) hint_key = a.hint[hslot] & (DT == 0 ? 0x7FFFFFFFu : 0x7FFFu);

    // Largest magnitude key of the row: the histogram window hangs from it.
    u32 kmax = 0;
    auto row_kmax = [&]() {
        u32 mx = 0;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const u32 wd = word_of(c, d);
                if (DT == 0) mx = max(mx, wd & 0x7FFFFFFFu);
                else mx = pk_max_u16(mx, wd & 0x7FFF7FFFu);
            }
        }
        if (DT == 1) mx = max(mx & 0xFFFFu, mx >> 16);
        kmax = wave_max_dpp(mx);
    };

    // Coarse histogram over a window of 2048 bins that hangs from `wtop`: bin = (wtop - key) >> S,
    // bin 0 on top.  First pass: S = 0 (bf16: one key per bin) or 16 (fp32: the same 128 bins per
    // octave), i.e. 16 octaves below the largest key, everything further down in the last bin.
    // Values of one row crowd into a few octaves, so bins this fine keep the lanes of an LDS
    // atomic on different addresses, and the bin of rank k-1 holds little beyond the kept set.
    // If rank k-1 lies below the window, a second pass with 16 times wider bins hangs from the
    // window's lower end and reaches key 0.
    constexpr int S1 = DT == 0 ? 16 : 0;
    u32 wtop = 0, above = 0;                        // above = number of keys > wtop
    int S = S1;
    u32 B1 = 0, c_gt = 0, cnt1 = 0;
    bool found = false;
    u32 rank_t = k > 0 ? (u32)(k - 1) : 0u;         // the rank the pass looks for (among the keys the functor lets through)
    auto all_keys = [](u32 wd) -> u32 { return wd & (DT == 0 ? 0x7FFFFFFFu : 0x7FFF7FFFu); };   // fp32: one key; bf16: a pair
    // skip0: keys that the functor turned into 0 are not counted at all (they would all meet on one
    // LDS address); the pass then reports found = false when the rank lies beyond the counted keys
    // windowed (fp32 narrowing passes): keys above the window or below its 2048 bins are not counted at all
    // (they would all meet on the first or the last bin's LDS address); `above` then only enters the rank
    auto hist_pass = [&](auto shift, auto key_pair, auto skip0, auto windowed) {
        constexpr int SH = decltype(shift)::value;
        constexpr bool kSkip0 = decltype(skip0)::value;
        constexpr bool kWindowed = decltype(windowed)::value;
        constexpr int SHB = SH >= 2 ? SH - 2 : 0;      // fp32: shift that leaves the bin number times 4
        // two 16-bit counters per word (a row has fewer than 2^16 elements): bin b is half b & 1 of word b >> 1
        auto bin_inc = [](u32 b4) { lds_inc((b4 >> 1) & ~3u, 1u << ((b4 & 4u) << 2)); };
        {
            uint4* h4 = (uint4*)smem;
#pragma unroll
            for (int i = 0; i < kCoarseBins / 8 / kWave; ++i) h4[i * kWave + lane] = make_uint4(0, 0, 0, 0);
        }
        wave_sync();
        const u32 wt2 = wtop * 0x10001u;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            if ((c * kWave + (int)lane) * EPC < N) {
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    const u32 wd = word_of(c, d);
                    if (DT == 0) {
                        const u32 key = key_pair(wd);
                        const u32 df = wtop > key ? wtop - key : 0u;
                        const u32 b4 = SH >= 2 ? min((df >> SHB) & ~3u, (u32)(4 * kCoarseBins - 4))
                                               : (min(df >> SH, (u32)(kCoarseBins - 1)) << 2);
                        if (kWindowed) {
                            if ((!kSkip0 || key) && key <= wtop && (df >> SH) < (u32)kCoarseBins) bin_inc(b4);
                        } else if (!kSkip0 || key) {
                            bin_inc(b4);
                        }
                    } else {
                        const u32 kp = key_pair(wd);
                        u32 b = pk_sub_sat_u16(wt2, kp);
                        if (SH) b = pk_shr_u16(b, SH);
                        b = pk_shl_u16(pk_min_u16(b, (u32)(kCoarseBins - 1) * 0x10001u), 2);
                        if (!kSkip0 || (kp & 0xFFFFu)) bin_inc(b & 0xFFFFu);
                        if (!kSkip0 || (kp >> 16)) bin_inc(b >> 16);
                    }
                }
            }
        }
        wave_sync();
        if (!kWindowed && above && lane == 0) smem[0] -= above;   // keys above the window were counted in bin 0
        wave_sync();
        // Scan from the top in two levels: every lane sums 32 bins, the lane that holds the rank
        // is then opened bin by bin.
        constexpr int BPL = kCoarseBins / kWave;       // 32 bins = 16 words
        const uint4* h4 = (const uint4*)(smem + (int)lane * (BPL / 2));
        u32 both = 0;                                  // the halves add up separately: no sum reaches 2^16
#pragma unroll
        for (int j = 0; j < BPL / 8; ++j) {
            const uint4 t = h4[j];
            both += (t.x + t.y) + (t.z + t.w);
        }
        const u32 local = (both & 0xFFFFu) + (both >> 16);
        const u32 incl = wave_scan_dpp(local), excl = incl - local;
        const u32 rem = rank_t - above;
        const u64 m_src = __ballot(local > 0 && excl <= rem && rem < incl);
        const int src = m_src ? (int)__builtin_ctzll(m_src) : 0;
        const u32 ex_src = bcast(excl, src);
        const u32 w2 = lane < (u32)BPL ? smem[src * (BPL / 2) + (int)(lane >> 1)] : 0u;
        const u32 c2 = (lane & 1u) ? w2 >> 16 : w2 & 0xFFFFu;
        const u32 inc2 = wave_scan_dpp(c2);            // lanes 0..31: running count inside lane `src`
        const u64 m_b1 = __ballot(lane < (u32)BPL && ex_src + inc2 > rem);
        found = m_src && m_b1;
        if (found) {
            const int j1 = (int)__builtin_ctzll(m_b1);
            B1 = (u32)(src * BPL + j1);
            cnt1 = bcast(c2, j1);
            c_gt = ex_src + bcast(inc2, j1) - cnt1;
        }
        wave_sync();
    };
    // List length and positions for a lower key bound t_lo: per 16-byte chunk the number of keys at or
    // above it, then exclusive positions (three chunk counts share one scan: 10-bit fields, a chunk
    // holds at most 512 keys).
    u32 t_lo = 1u, nL = 0;
    u32 cntc[NCH], basec[NCH];
    auto scan_counts = [&]() {
        nL = 0;
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
                    basec[3 * g + j] = nL + ((ex >> (10 * j)) & 0x3FFu);
                    nL += (tot >> (10 * j)) & 0x3FFu;
                }
            }
        }
    };
    auto count_plain = [&]() {
        const u32 C16 = (0x8000u - t_lo) * 0x10001u;            // bf16: bit 15 / 31 of (key + C16) <=> key >= t_lo
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            u32 n1 = 0;
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const u32 wd = word_of(c, d);
                if (DT == 0) n1 += ((wd & 0x7FFFFFFFu) >= t_lo) ? 1u : 0u;
                else n1 += (u32)__popc(((wd & 0x7FFF7FFFu) + C16) & 0x80008000u);
            }
            cntc[c] = n1;
        }
        scan_counts();
    };
    // the hinted bound: accepted when it keeps at least k keys and not many more
    bool hinted = false;
    if (kHint && k > 0) {
        const u32 dlt = kHintDelta << (DT == 0 ? 16 : 0);
        t_lo = hint_key > dlt ? hint_key - dlt : 1u;
        count_plain();
        hinted = nL >= (u32)k && nL <= (u32)k + kHintSlack && (int)nL <= cap;
    }
    if (!hinted && ASYM && DT == 0) row_kmax();      // (its selections run further down)
    if (!hinted && !(ASYM && DT == 0)) {
        row_kmax();
        wtop = kmax;
        hist_pass(std::integral_constant<int, S1>(), all_keys, std::false_type(), std::false_type());
        if (found && B1 == (u32)(kCoarseBins - 1) && (wtop >> S1) > (u32)(kCoarseBins - 1)) {
            above = c_gt;
            wtop -= (u32)(kCoarseBins - 1) << S1;
            S = S1 + 4;
            hist_pass(std::integral_constant<int, S1 + 4>(), all_keys, std::false_type(), std::false_type());
        }
        c_gt += above;
    }

    // ---- asymmetric thresholds: strict set, second selection ------------------------------------
    // Everything per pair of keys (packed 16-bit lanes): st = 1 where the element is strictly
    // retained, inF = 1 where it is a fill candidate (not strict, at or below tau).
    constexpr u32 kOne2 = 0x00010001u;
    u32 tau2 = 0, tp2 = 0, dthr2 = 0, t2_2 = 0;     // tau, tau+ and (tau- minus tau+), last key taken: duplicated in both halves
    u32 t2_key = 0, need_ties = 0, cnt_ties = 0, tn_key = 0;
    bool trim = false;
    auto gt01 = [&](u32 a2, u32 b2) -> u32 { return pk_min_u16(pk_sub_sat_u16(a2, b2), kOne2); };   // a > b, per half
    // (each use starts from an opaque copy of the word: the flags are recomputed where they are needed
    //  instead of being held in registers for the whole row from one phase to the next)
    auto strict01 = [&](u32 wd) -> u32 {
        asm volatile("" : "+v"(wd));
        const u32 neg01 = (wd >> 15) & kOne2;
        return gt01(wd & 0x7FFF7FFFu, pk_add_u16(tp2, pk_mul_lo_u16(neg01, dthr2)));
    };
    auto fill01 = [&](u32 wd, u32 st) -> u32 {
        asm volatile("" : "+v"(wd));
        return (st ^ kOne2) & (gt01(wd & 0x7FFF7FFFu, tau2) ^ kOne2);
    };
    // fp32: the exact key of rank rank_t among the keys a functor lets through, by histogram passes over
    // narrowing windows: bins of 2^16 keys, then 2^5 inside the bin found, then single keys (2^20, 2^9, 1
    // when the values spread over more than 16 octaves).  Starts from wtop with above = 0; on success
    // wtop - B1 is the key, above + c_gt the number of counted keys above it, cnt1 its multiplicity.
    auto narrow = [&](int sh_done) { above += c_gt; wtop -= B1 << sh_done; };
    auto exact_select32 = [&](auto key_fn, auto skip0) {
        hist_pass(std::integral_constant<int, 16>(), key_fn, skip0, std::false_type());
        if (!found) return;
        if (B1 == (u32)(kCoarseBins - 1) && (wtop >> 16) > (u32)(kCoarseBins - 1)) {
            narrow(16);
            hist_pass(std::integral_constant<int, 20>(), key_fn, skip0, std::true_type());
            if (!found) return;
            narrow(20);
            hist_pass(std::integral_constant<int, 9>(), key_fn, skip0, std::true_type());
            if (!found) return;
            narrow(9);
        } else {
            narrow(16);
            hist_pass(std::integral_constant<int, 5>(), key_fn, skip0, std::true_type());
            if (!found) return;
            narrow(5);
        }
        hist_pass(std::integral_constant<int, 0>(), key_fn, skip0, std::true_type());
    };
    u32 tp_key32 = 0, tau_key32 = 0;
    auto strict32 = [&](u32 wd) -> bool { return (wd & 0x7FFFFFFFu) > ((wd >> 31) ? tn_key : tp_key32); };
    auto fill32 = [&](u32 wd) -> bool { return !strict32(wd) && (wd & 0x7FFFFFFFu) <= tau_key32; };
    if (ASYM && DT == 0 && k > 0) {
        // tau = the k-th largest magnitude, exactly (the first pass above has run on the same window: redo it
        // as the first level of the exact selection)
        wtop = kmax; above = 0; S = 0;
        exact_select32(all_keys, std::false_type());
        if (!found) {                                // cannot happen: every key is counted
            if (lane == 0) a.fallback[r] = 1u;
            return;
        }
        tau_key32 = wtop - B1;
        const float tau = __uint_as_float(tau_key32);
        tp_key32 = __float_as_uint(__fmul_rn(a.one_plus, tau));
        tn_key = __float_as_uint(__fmul_rn(a.one_minus, tau));
        u32 accS = 0, accF = 0;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            if ((c * kWave + (int)lane) * EPC < N) {
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    const u32 wd = word_of(c, d);
                    accS += strict32(wd) ? 1u : 0u;
                    accF += fill32(wd) ? 1u : 0u;
                }
            }
        }
        const u32 tot = bcast(wave_scan_dpp(accS | (accF << 16)), kWave - 1);
        const u32 c_strict = tot & 0xFFFFu, f_fill = tot >> 16;
        trim = c_strict >= (u32)k;
        const u32 D = trim ? 0u : (u32)k - c_strict;
        if (trim || f_fill > D) {
            rank_t = trim ? (u32)(k - 1) : D - 1u;
            wtop = trim ? kmax : tau_key32;
            above = 0;
            if (trim) exact_select32([&](u32 wd) -> u32 { return strict32(wd) ? wd & 0x7FFFFFFFu : 0u; }, std::true_type());
            else exact_select32([&](u32 wd) -> u32 { return fill32(wd) ? wd & 0x7FFFFFFFu : 0u; }, std::true_type());
            if (found) {
                t2_key = wtop - B1;
                need_ties = rank_t + 1u - (above + c_gt);
                cnt_ties = cnt1;
            }                                            // else: the rank lies among zeros, every non-zero candidate is taken
        }
        if (t2_key == 0) { t2_key = 1; need_ties = 0; cnt_ties = 0; }
        S = 0; B1 = 0;
    }
    if (ASYM && DT == 1 && k > 0) {
        if (!found || S != 0) {                      // tau is not the key of one bin
            if (lane == 0) a.fallback[r] = 1u;
            return;
        }
        const u32 tau_key = wtop - B1;
        const float tau = __uint_as_float(tau_key << 16);
        const u32 tp_key = __float_as_uint(__fmul_rn(a.one_plus, tau)) >> 16;    // (key << 16) > T  <=>  key > (T >> 16)
        tn_key = __float_as_uint(__fmul_rn(a.one_minus, tau)) >> 16;
        tau2 = tau_key * 0x10001u; tp2 = tp_key * 0x10001u; dthr2 = ((tn_key - tp_key) & 0xFFFFu) * 0x10001u;
        u32 accS = 0, accF = 0;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            if ((c * kWave + (int)lane) * EPC < N) {
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    const u32 wd = word_of(c, d);
                    const u32 st = strict01(wd);
                    accS = pk_add_u16(accS, st);
                    accF = pk_add_u16(accF, fill01(wd, st));
                }
            }
        }
        const u32 both = ((accS & 0xFFFFu) + (accS >> 16)) | (((accF & 0xFFFFu) + (accF >> 16)) << 16);
        const u32 tot = bcast(wave_scan_dpp(both), kWave - 1);
        const u32 c_strict = tot & 0xFFFFu, f_fill = tot >> 16;
        trim = c_strict >= (u32)k;
        const u32 D = trim ? 0u : (u32)k - c_strict;
        if (trim || f_fill > D) {
            // rank k-1 of the strict set, or rank D-1 of the fill candidates: the other keys count as 0
            rank_t = trim ? (u32)(k - 1) : D - 1u;
            wtop = trim ? kmax : tau_key;
            above = 0;
            if (trim) hist_pass(std::integral_constant<int, 0>(), [&](u32 wd) -> u32 { return pk_mul_lo_u16(wd & 0x7FFF7FFFu, strict01(wd)); }, std::true_type(), std::false_type());
            else hist_pass(std::integral_constant<int, 0>(), [&](u32 wd) -> u32 { return pk_mul_lo_u16(wd & 0x7FFF7FFFu, fill01(wd, strict01(wd))); }, std::true_type(), std::false_type());
            if (found) {
                if (B1 == (u32)(kCoarseBins - 1) && wtop > (u32)(kCoarseBins - 1)) {     // below the window of single keys
                    if (lane == 0) a.fallback[r] = 1u;
                    return;
                }
                t2_key = wtop - B1;
                need_ties = rank_t + 1u - c_gt;
                cnt_ties = cnt1;
            }                                            // else: the rank lies among zeros, every non-zero candidate is taken
        }
        if (t2_key == 0) { t2_key = 1; need_ties = 0; cnt_ties = 0; }     // the rank falls on zeros (never sent) or every candidate is taken
        t2_2 = t2_key * 0x10001u;
    }

    // the list takes every non-zero key from bin B1 up (a bin that reaches key 0 also counts the
    // zeros, which never enter the list: its length is known after the counting pass below)
    if (!hinted) {
        const long long lowk = (long long)wtop - ((long long)(B1 + 1u) << S) + 1;
        t_lo = lowk > 1 ? (u32)lowk : 1u;                        // smallest non-zero key of bin B1
        if (ASYM && k > 0) t_lo = trim ? t2_key : min(t2_key, tn_key + 1u);   // smallest key the list can hold
        if (!ASYM && k > 0 && lowk >= 1 && (int)(c_gt + cnt1) > cap) {
            if (lane == 0) a.fallback[r] = 1u;
            return;
        }
    }

    // ---- 2. ordered compaction into L -------------------------------------------------
    if (k == 0) nL = 0;
    if (k > 0) {
        const u32 C16 = (0x8000u - t_lo) * 0x10001u;            // bf16: bit 15 / 31 of (key + C16) <=> key >= t_lo
        // bits 15 and 31: the element goes to the list
        auto list_flags = [&](u32 wd) -> u32 {
            if (!ASYM) return (wd & 0x7FFF7FFFu) + C16;
            const u32 st = strict01(wd);
            u32 wk = wd;
            asm volatile("" : "+v"(wk));
            const u32 ge = gt01(t2_2, wk & 0x7FFF7FFFu) ^ kOne2;              // key >= last key taken
            return (trim ? (st & ge) : (st | (fill01(wd, st) & ge))) << 15;
        };
        // fp32: the element goes to the list
        auto flag32 = [&](u32 wd) -> u32 {
            const u32 key = wd & 0x7FFFFFFFu;
            if (!ASYM) return key >= t_lo ? 1u : 0u;
            const bool st = strict32(wd), ge = key >= t2_key;
            return (trim ? (st && ge) : (st || (fill32(wd) && ge))) ? 1u : 0u;
        };
        if (ASYM) {
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                u32 n1 = 0;
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    if (DT == 0) n1 += flag32(word_of(c, d));
                    else n1 += (u32)__popc(list_flags(word_of(c, d)) & 0x80008000u);
                }
                cntc[c] = n1;
            }
            scan_counts();
        } else if (!hinted) {
            count_plain();
        }
        // every flagged element is stored at a running byte address that advances by its flag
        const u32 lidx_off = (u32)((u32*)L.Lidx - smem) * 4u;
        if ((int)nL > cap) {                                      // uniform
            if (lane == 0) a.fallback[r] = 1u;
            return;
        }
        // (the empty asm statements pin values in registers: the optimiser would otherwise
        //  re-derive each flag and each inverted index with longer instruction sequences)
        u32 linv = 0xFFFFu - lane * (u32)EPC;
        asm volatile("" : "+v"(linv));
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            u32 wa = lent_off + basec[c] * 4u;
            const u32 idx0 = (u32)((c * kWave + (int)lane) * EPC);
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const u32 wd = word_of(c, d);
                if (DT == 0) {
                    const u32 fl = flag32(wd);
                    if (fl) {
                        *lds_at(wa) = wd;
                        *(__attribute__((address_space(3))) uint16_t*)(uintptr_t)(lidx_off + ((wa - lent_off) >> 1)) = (uint16_t)(idx0 + d);
                    }
                    wa += fl << 2;
                } else {
                    const u32 f = list_flags(wd);
                    u32 f0 = (f >> 15) & 1u, f1 = f >> 31;
                    asm volatile("" : "+v"(f0));
                    asm volatile("" : "+v"(f1));
                    const u32 i0 = linv - (u32)(c * kWave * EPC + 2 * d), i1 = linv - (u32)(c * kWave * EPC + 2 * d + 1);
                    if (f0) *lds_at(wa) = (wd << 16) | i0;
                    wa += f0 << 2;
                    asm volatile("" : "+v"(wa));
                    if (f1) *lds_at(wa) = __builtin_amdgcn_perm(wd, i1, 0x07060100u);   // wd's high half : i1's low half
                    wa += f1 << 2;
                    asm volatile("" : "+v"(wa));
                }
            }
        }
    }
    if (ASYM && k > 0 && need_ties < cnt_ties) {
        // The list holds every candidate with the last key taken; only the first need_ties of them
        // in index order stay.  The list is in index order: the others are squeezed out in place.
        wave_sync();
        u32 seen = 0, dead = 0;
        for (u32 p0 = 0; p0 < nL; p0 += kWave) {
            const u32 p = p0 + lane;
            u32 e = 0, ei = 0;
            bool tie = false;
            if (p < nL) {
                e = L.Lent[p];
                if (DT == 0) {
                    ei = L.Lidx[p];
                    const bool cand = trim ? strict32(e) : fill32(e);
                    tie = cand && (e & 0x7FFFFFFFu) == t2_key;
                } else {
                    const u32 wd = e >> 16;                              // sign and key in the low half, as in the row
                    const u32 st = strict01(wd) & 1u;
                    const u32 cand = trim ? st : (fill01(wd, st) & 1u);
                    tie = cand && (wd & 0x7FFFu) == t2_key;
                }
            }
            const u64 mt = __ballot(tie);
            const bool drop = tie && seen + mask_rank(mt) >= need_ties;
            const u64 md = __ballot(drop);
            wave_sync();
            if (p < nL && !drop) {
                L.Lent[p - dead - mask_rank(md)] = e;
                if (DT == 0) L.Lidx[p - dead - mask_rank(md)] = (uint16_t)ei;
            }
            wave_sync();
            seen += (u32)__popcll(mt);
            dead += (u32)__popcll(md);
        }
        nL -= dead;
    }
    if (MAXS) {
        // the list moves into registers: its LDS storage is free for the bin-ordered list
        wave_sync();
#pragma unroll
        for (int s = 0; s < SLN; ++s) {
            const u32 p = s * kWave + lane;
            if (MAXS) ent[MAXS ? s : 0] = p < nL ? L.Lent[p] : 0u;
            if (MAXS && DT == 0) eix[(MAXS && DT == 0) ? s : 0] = p < nL ? (u32)L.Lidx[p] : 0u;
        }
        wave_sync();
        if (kHint && hinted) {                        // the row's largest key is the list's largest
            u32 mx = 0;
#pragma unroll
            for (int s = 0; s < SLN; ++s) mx = max(mx, ent[MAXS ? s : 0] & 0x7FFFFFFFu);
            kmax = wave_max_dpp(mx);
            if (DT == 1) kmax >>= 16;
        }
    }
    {
        uint4* h4 = (uint4*)L.hist;
#pragma unroll
        for (int i = 0; i < kFineBins / 4 / kWave; ++i) h4[i * kWave + lane] = make_uint4(0, 0, 0, 0);
    }
    if (lane == 0) {
#pragma unroll
        for (int t = 0; t < QN; ++t)
            if (NQ || t < nq) L.qtab[t] = (u32)a.qlist[t];
    }
    wave_sync();

    // ---- 3. fine bins ---------------------------------------------------------------------
    // 1024 bins, linear in (key - t_lo) >> sh; sh from the top of the highest occupied coarse
    // bin.  fp32 keeps the in-bin key bits, the inverted index and the class in one word of S.
    const int nslots = (int)((nL + kWave - 1) / kWave);
    const u32 range = kmax > t_lo ? kmax - t_lo : 0u;
    const int sh = range < (u32)kFineBins ? 0 : (32 - __clz((int)range)) - 10;
    if (DT == 0 && sh + w + 1 > 32) {
        if (lane == 0) a.fallback[r] = 1u;
        return;
    }
    const u32 inmask = (1u << sh) - 1u;
#pragma unroll(MAXS ? MAXS : 1)
    for (int s = 0; s < SLN; ++s) {
        if (s >= nslots) break;
        const u32 p = s * kWave + lane;
        if (p < nL) {
            const u32 e = ent_word(s);
            const u32 key = DT == 0 ? (e & 0x7FFFFFFFu) : ((e >> 16) & 0x7FFFu);
            lds_inc(((key - t_lo) >> sh) << 2, (e >> 31) ? 0x800u : 1u);    // 11-bit fields: the list has fewer than 2048 entries
        }
    }
    wave_sync();
    u32 n_pos, n_neg;
    int cut_lane = 0;
    {   // exclusive prefix from the top, per class, in the counting format pos | neg << 11 (fill << 22 is added later)
        const int hi = kFineBins - (int)lane * 16;
        u32 cs[16];
        uint4* h4 = (uint4*)(L.hist + hi - 16);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint4 t = h4[3 - j];
            cs[4 * j + 0] = t.w; cs[4 * j + 1] = t.z; cs[4 * j + 2] = t.y; cs[4 * j + 3] = t.x;
        }
        u32 local = 0;
#pragma unroll
        for (int j = 0; j < 16; ++j) local += cs[j];
        if (nL >= 1024u) {                              // a fine bin with 1024+ members overflows its 10-bit fill field
            u32 big = 0;
#pragma unroll
            for (int j = 0; j < 16; ++j) big |= ((cs[j] & 0x7FFu) + (cs[j] >> 11)) >> 10;
            if (__ballot(big != 0u)) {
                if (lane == 0) a.fallback[r] = 1u;
                return;
            }
        }
        const u32 incl = wave_scan_dpp(local);
        const u32 tot = bcast(incl, kWave - 1);
        n_pos = tot & 0x7FFu; n_neg = tot >> 11;        // class sizes of L (of the kept set once cut)
        const u32 excl = incl - local;
        // the lane whose bins hold overall rank k-1 (meaningful when nL > k)
        const u32 ov_ex = (excl & 0x7FFu) + (excl >> 11), ov_in = (incl & 0x7FFu) + (incl >> 11);
        const u64 mc = __ballot(k > 0 && ov_ex <= (u32)(k - 1) && (u32)(k - 1) < ov_in);
        cut_lane = mc ? (int)__builtin_ctzll(mc) : 0;
        u32 acc = excl;
        u32 o[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            o[j] = acc;
            acc += cs[j];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) h4[3 - j] = make_uint4(o[4 * j + 3], o[4 * j + 2], o[4 * j + 1], o[4 * j + 0]);
    }
    wave_sync();
#pragma unroll(MAXS ? MAXS : 1)
    for (int s = 0; s < SLN; ++s) {
        if (s >= nslots) break;
        const u32 p = s * kWave + lane;
        if (p < nL) {
            const u32 e = ent_word(s);
            const u32 key = DT == 0 ? (e & 0x7FFFFFFFu) : ((e >> 16) & 0x7FFFu);
            const u32 rel = key - t_lo;
            const u32 old = atomicAdd(&L.hist[rel >> sh], 1u << 22);
            const u32 at = (old & 0x7FFu) + ((old >> 11) & 0x7FFu) + (old >> 22);
            if (DT == 0) L.S[at] = ((((rel & inmask) << w) | (idxmask - ent_index(s))) << 1) | (e >> 31);
            else L.S[at] = e;
        }
    }
    wave_sync();
    // members of a fine bin compare on the plain comp; their class
    auto s_plain = [&](u32 s) -> u32 { return DT == 0 ? s >> 1 : s & 0x7FFFFFFFu; };
    auto s_neg = [&](u32 s) -> u32 { return DT == 0 ? s & 1u : s >> 31; };
    // class-extended comp of a member of fine bin `bin`
    auto s_cx = [&](u32 s, u32 bin) -> comp_t {
        if (DT == 0) {
            const u32 key = ((bin << sh) | ((s >> 1) >> w)) + t_lo;
            const u32 idx = idxmask - ((s >> 1) & idxmask);
            return ((comp_t)(key | ((s & 1u) ? 0u : 0x80000000u)) << kHiShift) | (comp_t)(u32)(~idx);
        }
        return (comp_t)(s ^ 0x80000000u);
    };

    // ---- top-K cut: the comp of overall rank k-1 (ATKF) -----------------------------------------
    comp_t thrK = 0;                                // plain comp; every entry of L is kept when nL <= k
    if (nL > (u32)k) {
        // open the 16 bins of the lane found by the scan: the last one whose first rank is <= k-1
        const int hi = kFineBins - cut_lane * 16;
        const u32 wj = lane < 16u ? L.hist[hi - 1 - (int)lane] : 0xFFFFFFFFu;
        const u64 mj = __ballot(lane < 16u && (wj & 0x7FFu) + ((wj >> 11) & 0x7FFu) <= (u32)(k - 1));
        const int lo = hi - (int)__popcll(mj);
        const u32 wd = L.hist[lo];
        const u32 pe = wd & 0x7FFu, ne = (wd >> 11) & 0x7FFu, cnt = wd >> 22, base = pe + ne;
        const u32 rem = (u32)(k - 1) - base;
        u32 kp = 0, kn = 0;
        for (u32 g = 0; g < cnt; g += kWave) {       // members in groups of 64, one per lane
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
    const u32 n = n_pos + n_neg;
    const u32 Kc[2] = { n_pos / (u32)M, n_neg / (u32)Mn };

    // ---- block boundaries: comps of class ranks j*K-1, one lane per boundary ------------------------
    // M-1 boundaries for the positive class, then Mn-1 for the negative one.  A class with fewer than M members has
    // K = 0 and every member in its last block: its boundaries sit above every comp of the class.
    const int ntg = B2 - 2;
    comp_t* thr = (comp_t*)L.thr;
    {
        const int ntp = ntg > 0 ? ntg : 1;
        u32* tg_bin = L.tg; u32* tg_base = L.tg + ntp; u32* tg_cnt = L.tg + 2 * ntp; u32* tg_rem = L.tg + 3 * ntp; u32* tg_pre = L.tg + 4 * ntp;
        const bool mine = (int)lane < ntg;
        const int cls = (int)lane >= M - 1 ? 1 : 0;
        const int j = (cls ? (int)lane - (M - 1) : (int)lane) + 1;
        const bool act = mine && Kc[cls] > 0;
        const u32 R = act ? (u32)j * Kc[cls] - 1u : 0u;
        int lo = 0, hi = kFineBins - 1;             // smallest bin whose first class rank is <= R
        for (int it = 0; it < 10; ++it) {
            const int mid = (lo + hi) >> 1;
            const u32 wd = L.hist[mid];
            const u32 pc = cls ? (wd >> 11) & 0x7FFu : wd & 0x7FFu;
            if (pc <= R) hi = mid; else lo = mid + 1;
        }
        const u32 wd = L.hist[lo];
        const u32 pe = wd & 0x7FFu, ne = (wd >> 11) & 0x7FFu;
        const u32 cnt = act ? wd >> 22 : 0u;
        const u32 incl = wave_scan_dpp(cnt);
        if (mine) {
            tg_bin[lane] = (u32)lo; tg_base[lane] = pe + ne; tg_cnt[lane] = cnt;
            tg_rem[lane] = R - (cls ? ne : pe);
            tg_pre[lane] = incl - cnt;
            if (!act) thr[lane] = cls ? (comp_t)(kClsBit - 1) : ~(comp_t)0;
        }
        const u32 npairs = bcast(incl, kWave - 1);
        wave_sync();
        // one lane per (boundary, member of its bin): the member of the boundary's class
        // with exactly `rem` class-mates above it is the boundary element
        for (u32 g = 0; g < npairs; g += kWave) {
            const u32 pr = g + lane;
            if (pr < npairs) {
                int tl = 0, th = ntg - 1;           // boundary t with tg_pre[t] <= pr < tg_pre[t] + tg_cnt[t]
                while (tl < th) {
                    const int mid = (tl + th + 1) >> 1;
                    if (tg_pre[mid] <= pr) tl = mid; else th = mid - 1;
                }
                const int t = tl;
                const u32 tc = (u32)(t >= M - 1 ? 1 : 0);
                const u32 bs = tg_base[t], cn = tg_cnt[t];
                const u32 me = L.S[bs + (pr - tg_pre[t])];
                if (s_neg(me) == tc) {
                    // one compare per member: with the class bit moved to the top and set for the
                    // boundary's class, "same class and larger comp" is a plain unsigned "larger"
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

    // block starts in closed form (K, ..., K, K + remainder per class)
    if ((int)lane < B2) {
        const int s = (int)lane >= M ? 1 : 0, m = (int)lane - s * M;
        const u32 st = (s ? n_pos : 0u) + (u32)m * Kc[s];
        L.blk_start[lane] = st;
        L.run[lane] = st;
        L.vminb[lane] = 0xFFFFFFFFu; L.vmaxb[lane] = 0;
    }
    if (lane == 0) L.blk_start[B2] = n;
    wave_sync();

    // ---- 4. blocks, stable split by block, block-ordered arrays -----------------------------------
    // S and the fine bins are dead (boundaries are resolved): S's storage takes the
    // block-ordered values, the histogram region the indices and the stream image
    u32* bo_val = L.S;
    uint16_t* bo_idx = (uint16_t*)(L.hist);
    u32* stage = L.hist + (k + 1) / 2;
    int nbits = 0;
    while ((1 << nbits) < B2) ++nbits;
    // An entry's block = number of boundaries above it, plus one for the negative class: a
    // positive entry is above every negative boundary, a negative entry below every positive
    // one.  Up to kRegThr boundaries are held in registers.
    comp_t tx[kRegThr];
#pragma unroll
    for (int j = 0; j < kRegThr; ++j) tx[j] = j < ntg ? thr[j] : (comp_t)0;
    const bool tree8 = DT == 1 && M == 8 && Mn == 8;      // (one-word comps: a select is one instruction)
#pragma unroll(MAXS ? MAXS : 1)
    for (int s = 0; s < SLN; ++s) {
        if (s >= nslots) break;
        const u32 p = s * kWave + lane;
        bool kept = false;
        u32 b = 0, key = 0, idx = 0;
        if (p < nL) {
            const comp_t cx = ent_cx(s);
            if ((cx & ~kClsBit) >= thrK) {
                kept = true;
                u32 above;
                if (tree8) {
                    // 8 + 8 blocks: the 14 boundaries and the class bit are 15 separators in descending
                    // order; four compares walk them as a binary tree (the first is the class bit itself)
                    const bool c1 = !(cx & kClsBit);
                    comp_t m = c1 ? tx[10] : tx[3];
                    const bool c2 = m > cx;
                    m = c1 ? (c2 ? tx[12] : tx[8]) : (c2 ? tx[5] : tx[1]);
                    const bool c3 = m > cx;
                    const comp_t lo4 = c3 ? (c2 ? tx[6] : tx[2]) : (c2 ? tx[4] : tx[0]);
                    const comp_t hi4 = c3 ? (c2 ? tx[13] : tx[9]) : (c2 ? tx[11] : tx[7]);
                    m = c1 ? hi4 : lo4;
                    const bool c4 = m > cx;
                    above = (c1 ? 8u : 0u) + (c2 ? 4u : 0u) + (c3 ? 2u : 0u) + (c4 ? 1u : 0u);
                } else {
                    above = (cx & kClsBit) ? 0u : 1u;
#pragma unroll
                    for (int j = 0; j < kRegThr; ++j) above += tx[j] > cx ? 1u : 0u;
                    for (int j = kRegThr; j < ntg; ++j) above += thr[j] > cx ? 1u : 0u;
                }
                b = above;
                key = cx_key(cx);
                idx = cx_idx(cx);
                atomicMin(&L.vminb[b], key);
                atomicMax(&L.vmaxb[b], key);
            }
        }
        // lanes of this slot in the same block: one ballot per bit of the block id
        // (lanes that are not kept drop out through the first mask)
        const u64 km = __ballot(kept);
        u32 plo = (u32)km, phi = (u32)(km >> 32);
        for (int bit = 0; bit < nbits; ++bit) {
            const u32 onm = (u32)__builtin_amdgcn_sbfe((int)b, (u32)bit, 1u);   // all ones if the bit is set
            const u64 bal = __ballot(onm != 0u);
            plo &= ~((u32)bal ^ onm);
            phi &= ~((u32)(bal >> 32) ^ onm);
        }
        const u32 before = __builtin_amdgcn_mbcnt_hi(phi, __builtin_amdgcn_mbcnt_lo(plo, 0u));
        u32 basep = 0;
        if (kept) basep = L.run[b];
        wave_sync();
        if (kept) {
            if (before == 0) L.run[b] = basep + (u32)__popc(plo) + (u32)__popc(phi);
            const u32 pos = basep + before;
            bo_val[pos] = E::value_bits(key);
            bo_idx[pos] = (uint16_t)idx;
        }
        wave_sync();
    }

    // ---- 5. ABQ -----------------------------------------------------------------------------------
    // Each block is walked by kWave / B2 lanes, each lane a contiguous run of the block-ordered
    // list, so a lane's quantiser constants and partial sums live in registers.
    u64* sums = (u64*)(L.hist + ((((k + 1) / 2 + (int)a.cap_words) + 1) & ~1));
    float* invt = (float*)(sums + B2 * (nq + 1));
    const u32 lpb = (u32)kWave / (u32)B2;
    const u32 myb = udiv16(lane, lpb), sub = lane - myb * lpb;
    const bool lane_on = myb < (u32)B2;
    u32 r0 = 0, r1 = 0, bs0 = 0, mycnt = 0;
    float vmin = 0.f, rng = 0.f, rng1 = 1.f;
    int e = 0, dg = 1, er = 0;
    u32 vmaxbits = 0;
    if (lane_on) {
        bs0 = L.blk_start[myb];
        const u32 be = L.blk_start[myb + 1];
        mycnt = be - bs0;
        const u32 perb = udiv16(mycnt + lpb - 1, lpb);
        r0 = bs0 + sub * perb; r0 = r0 < be ? r0 : be;
        r1 = r0 + perb < be ? r0 + perb : be;
        if (mycnt) {
            const u32 lo = E::value_bits(L.vminb[myb]);
            vmaxbits = E::value_bits(L.vmaxb[myb]);
            vmin = __uint_as_float(lo);
            rng = __uint_as_float(vmaxbits) - vmin;
            dg = !(rng > 0.f);                       // only a range of exactly 0 is degenerate
            if (!dg) { er = range_exp(rng); rng1 = unit_range(rng, er); }
            e = ilogb_bits(vmaxbits) + 1;
        }
    }
    // longest run of any lane: the largest block holds K + (n mod M) entries
    const u32 mc0 = n_pos - Kc[0] * (u32)(M - 1), mc1 = n_neg - Kc[1] * (u32)(Mn - 1);
    const u32 T = udiv16((mc0 > mc1 ? mc0 : mc1) + lpb - 1, lpb);
    // quantiser scales L / (range brought to [1, 2)): the lanes of a block share the divisions through LDS
    if (lane_on) {
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
    wave_sync();
    // Residual of a code on the 2^-15 grid, rho = rint((y - rint(y)) * 2^15) with y = d * inv:
    // z = d * (inv * 2^15) equals y * 2^15 exactly, rint(y) * 2^15 is a multiple of 2^15, and
    // |rho| <= 2^14, so rho is rint(z) reduced to 15 signed bits (for |rho| = 2^14 the sign is
    // lost, the square is not).  Bitwidths up to 8 keep z below 2^23, where adding 2^23 rounds
    // to the integer grid with the same round-half-even.
    float inv[QN];
    bool small_q = true;
#pragma unroll
    for (int t = 0; t < QN; ++t) {
        inv[t] = (lane_on && (NQ || t < nq)) ? invt[myb * (u32)nq + t] : 0.f;
        if ((NQ || t < nq) && a.qlist[t] > 8) small_q = false;
    }
    auto abq_sums = [&](auto fast) {
        constexpr bool kFast = decltype(fast)::value;
        // bitwidths up to 8: y * 2^15 stays below 2^23, one multiply per code
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
                            // (wider bitwidths: y first, then the exact scaling, so that nothing overflows)
                            const u32 zi = kFast ? __float_as_uint(d * inv15[t] + 8388608.0f)
                                                 : (u32)rintf((d * inv[t]) * 32768.0f);
                            const int rho = __builtin_amdgcn_sbfe((int)zi, 0u, 15u);
                            acc[t] += (u32)(rho * rho);
                        }
                    }
                }
            }
#pragma unroll
            for (int t = 0; t < QN; ++t)
                if ((NQ || t < nq) && acc[t]) atomicAdd(&sums[myb * (nq + 1) + t], (u64)acc[t]);
        }
        if (accE) atomicAdd(&sums[myb * (nq + 1) + nq], accE);
    };
    // Eq. "DS": sum over the block of | (code at q_bit >> (q_bit - q)) - code at q | for every lower bitwidth
    auto ds_sums = [&]() {
        const int top = nq - 1, qtop = (int)L.qtab[top];
        const float inv_top = lane_on ? invt[myb * (u32)nq + (u32)top] : 0.f;
        for (u32 i0 = 0; i0 < T; i0 += 8) {
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
            for (int t = 0; t < QN; ++t)
                if ((NQ || t < nq) && acc[t]) atomicAdd(&sums[myb * (nq + 1) + t], (u64)acc[t]);
        }
    };
    if (!a.lad.on) {
        if (a.guard == 1) ds_sums();
        else if (small_q) abq_sums(std::true_type());
        else abq_sums(std::false_type());
    }
    wave_sync();

    // smallest feasible bitwidth per block: the lanes of a block test different candidates in
    // ascending order and keep the minimum
    if (a.lad.on) {
        if (lane_on && sub == 0) L.run[myb] = ladder_index(a.lad, (int)(myb >= (u32)M ? myb - (u32)M : myb));
    } else if (a.guard == 1) {
        // greedy descent: the chosen index is one above the highest violating candidate below q_bit
        if (lane_on && mycnt && !dg) {
            for (u32 t = sub; t + 1 < (u32)nq; t += lpb)
                if (!((double)sums[myb * (nq + 1) + t] <= a.beta * (double)mycnt)) atomicOr(&L.run[myb], 1u << t);
        }
        wave_sync();
        if (lane_on && sub == 0) {
            const u32 viol = L.run[myb];
            L.run[myb] = viol ? 32u - (u32)__clz((int)viol) : 0u;
        }
    } else if (lane_on && mycnt && !dg) {
        const double rhs = a.beta * ldexp((double)sums[myb * (nq + 1) + nq], 2 * e - 40);
        for (u32 t = sub; t < (u32)nq; t += lpb) {
            const float Lq = (float)((1u << L.qtab[t]) - 1u);
            const float o = rng / Lq;
            const double lhs = ((double)o * (double)o) * (double)sums[myb * (nq + 1) + t] * 0x1p-30;
            if (lhs <= rhs) { atomicMin(&L.run[myb], t); break; }
        }
    }
    wave_sync();
    u32 myq = 0, flag = 0;
    float my_inv = 0.f;
    if (lane_on) {
        u32 tb = L.run[myb];
        if (tb == (u32)nq) { flag = 0x80u; tb = (u32)nq - 1u; }   // none feasible: the largest bitwidth, flagged
        myq = L.qtab[tb];
        my_inv = invt[myb * (u32)nq + tb];
    }
    if (lane_on && sub == 0) {
        const size_t mi = (size_t)r * (size_t)B2 + myb;
        a.mv.vmin[mi] = mycnt ? vmin : 0.f;
        a.mv.vmax[mi] = mycnt ? __uint_as_float(vmaxbits) : 0.f;
        a.mv.q[mi] = (uint8_t)(myq | flag);
    }
    // bit offsets of the blocks' code sections: scan over one lane per block
    const u32 mybits = (lane_on && sub == 0) ? mycnt * myq : 0u;
    const u32 incl_bits = wave_scan_dpp(mybits);
    const u32 code_bits = bcast(incl_bits, kWave - 1);
    const u32 my_off = incl_bits - mybits;              // valid in the block's first lane ...
    const u32 coff = (u32)__shfl((int)my_off, (int)(myb * lpb));   // ... fetched by its other lanes
    const u32 idx_bits = n * (u32)w;
    const u32 row_bits = idx_bits + code_bits;
    u32 row_words = (row_bits + 31u) >> 5;
    if ((u64)row_words > a.cap_words) row_words = (u32)a.cap_words;   // cannot happen (worst-case capacity)
    for (u32 i = lane; i < row_words; i += kWave) stage[i] = 0;
    wave_sync();

    // ---- packing ----------------------------------------------------------------------------------
    {
        for (u32 i = 0; i < T; ++i) {
            const u32 p = r0 + i;
            if (p < r1) {
                u32 c = 0;
                if (!dg) {
                    const float y = to_unit(__uint_as_float(bo_val[p]) - vmin, er) * my_inv;
                    c = (u32)rintf(y);                    // already within [0, 2^q - 1]
                }
                {   // index field
                    const u32 P = __umul24(p, (u32)w), wi = P >> 5, sft = P & 31u, val = bo_idx[p];
                    atomicOr(&stage[wi], val << sft);
                    if (sft + (u32)w > 32u) atomicOr(&stage[wi + 1], val >> (32u - sft));
                }
                {   // code field
                    const u32 P = idx_bits + coff + __umul24(p - bs0, myq), wi = P >> 5, sft = P & 31u;
                    atomicOr(&stage[wi], c << sft);
                    if (sft + myq > 32u) atomicOr(&stage[wi + 1], c >> (32u - sft));
                }
            }
        }
    }
    wave_sync();
    u32* __restrict__ slot = a.slots + (size_t)r * (size_t)a.cap_words;
    for (u32 i = lane; i < row_words; i += kWave) slot[i] = stage[i];
    if (lane == 0) {
        a.row_words[r] = row_words;
        a.mv.n_pos[r] = n_pos;
        a.mv.n_neg[r] = n_neg;
        a.fallback[r] = 0u;
        if (kHint && k > 0) a.hint[hslot] = nL > (u32)k ? cx_key(thrK) : t_lo;    // this row's cut key, for a later row
    }
}

}  // namespace slicer
