// Row-resident encoder for short rows: ONE WAVEFRONT PER ROW, the row held in
// registers, every list in LDS, no workgroup barrier anywhere.
//
//   1. load the row (16-byte coalesced loads), 10-bit histogram of the magnitude
//      key's top bits in LDS, scan from the top -> the bin that holds rank k-1;
//   2. ordered compaction of everything at or above that bin into a short list L
//      (ascending index; it contains the kept set plus the undecided bin);
//   3. L is bucket-sorted: 1024 fine bins, linear in the key from the list's lower
//      bound, both sign classes counted in one packed table; an exclusive scan from
//      the top gives every bin's first rank, and an all-pairs comparison among the
//      few members of a bin gives every entry its exact rank in the order
//      "magnitude descending, lower index first" -- overall (top-K, Sec. 3.1) and
//      within its sign class (MS, Sec. 3.2);
//   4. block = rank / K; a stable split by block id (wave ballots) restores
//      ascending index inside each block; the elements of rank m*K and (m+1)*K-1
//      are the block's max and min;
//   5. ABQ sums on integer grids, bitwidth choice, bit offsets, packing through an
//      LDS image of the row's stream segment.
//
// Rows the list cannot hold (heavy ties around the threshold, more zeros than
// dropped elements, ...) are flagged and redone by the generic kernel.
#pragma once

#include "slicer_common.hpp"

namespace slicer {

struct SmallArgs {
    const void* x;
    int64_t R, N, k;
    int M, w, nq;
    int qlist[kMaxQ];
    double beta;
    u64 cap_words;
    u64* row_words;     // [R]
    u32* slots;         // [R][cap_words]
    u32* fallback;      // [R] 1 = redo this row with the generic kernel
    MetaView mv;
    int cap;            // list capacity, multiple of 64, <= 1023
    int region0_words;  // histogram region, later block-ordered arrays + stream image
};

constexpr int kFineBins = 1024;

__device__ inline void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

__device__ inline u32 bcast(u32 v, int src) { return (u32)__builtin_amdgcn_readlane((int)v, src); }

// LDS carve-up of one wave (word offsets); must match small_lds_words() on the host
struct SmallLds {
    u32* hist;      // [region0]   coarse / fine histogram; later bo_val, bo_idx, stage
    u32* Lraw;      // [cap]       raw element bits of the list, ascending index
    u32* S;         // [cap]       list entries arranged by fine bin: inbin_comp << 1 | class
    uint16_t* Lidx; // [cap]
    uint16_t* Lr;   // [cap]       class rank of a kept entry, 0xFFFF otherwise
    u32* blk_start; // [B2 + 1]
    u32* vminb;     // [B2] key of the block's smallest / largest element
    u32* vmaxb;     // [B2]
    u32* run;       // [B2]
    u32* qsel;      // [B2]
    u32* code_off;  // [B2 + 1]
    int* e_tab;     // [B2]
    int* degen;     // [B2]
    float* inv_tab; // [B2][nq]
    u64* sums;      // [B2][nq + 1]
};

__host__ __device__ inline int small_lds_words(int cap, int region0, int B2, int nq)
{
    int wds = region0 + cap + cap + cap / 2 + cap / 2;
    wds += (B2 + 1) + B2 * 4 + (B2 + 1) + B2 * 2 + B2 * nq;
    wds = (wds + 1) & ~1;
    wds += 2 * B2 * (nq + 1);
    return wds;
}

__device__ inline SmallLds small_carve(u32* base, int cap, int region0, int B2, int nq)
{
    SmallLds L;
    u32* p = base;
    L.hist = p;            p += region0;
    L.Lraw = p;            p += cap;
    L.S = p;               p += cap;
    L.Lidx = (uint16_t*)p; p += cap / 2;
    L.Lr = (uint16_t*)p;   p += cap / 2;
    L.blk_start = p;       p += B2 + 1;
    L.vminb = p;           p += B2;
    L.vmaxb = p;           p += B2;
    L.run = p;             p += B2;
    L.qsel = p;            p += B2;
    L.code_off = p;        p += B2 + 1;
    L.e_tab = (int*)p;     p += B2;
    L.degen = (int*)p;     p += B2;
    L.inv_tab = (float*)p; p += B2 * nq;
    if ((p - base) & 1) ++p;
    L.sums = (u64*)p;
    return L;
}

template <int DT, int EPL>
__global__ __launch_bounds__(kWave) void enc_small_kernel(SmallArgs a)
{
    typedef Elem<DT> E;
    constexpr int EPC = DT == 0 ? 4 : 8;            // elements per 16-byte chunk
    constexpr int NCH = EPL / EPC;                  // chunks per lane
    constexpr int KS = E::kKeyBits - 10;            // coarse digit = key >> KS
    extern __shared__ u32 smem[];

    const u32 lane = lane_id();
    const int64_t r = blockIdx.x;
    const int N = (int)a.N, M = a.M, w = a.w, B2 = 2 * a.M, nq = a.nq, cap = a.cap;
    const int k = (int)a.k;
    const u32 idxmask = (1u << w) - 1u;
    SmallLds L = small_carve(smem, cap, a.region0_words, B2, nq);

    // ---- 1. load the row -------------------------------------------------------
    const uint4* __restrict__ xr = (const uint4*)((const char*)a.x + (size_t)r * (size_t)N * (DT == 0 ? 4 : 2));
    uint4 v[NCH];
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int base = (c * kWave + (int)lane) * EPC;
        v[c] = base < N ? xr[c * kWave + lane] : make_uint4(0, 0, 0, 0);
    }
    auto raw_of = [&](int c, int e) -> u32 {       // raw bits of element e of chunk c
        const u32 wd = (DT == 0) ? (&v[c].x)[e] : (&v[c].x)[e >> 1];
        return (DT == 0) ? wd : ((e & 1) ? wd >> 16 : wd & 0xFFFFu);
    };

    for (int i = lane; i < kFineBins; i += kWave) L.hist[i] = 0;
    wave_sync();

    // coarse histogram over the top 10 bits of the key
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        if ((c * kWave + (int)lane) * EPC < N) {
#pragma unroll
            for (int e = 0; e < EPC; ++e) atomicAdd(&L.hist[E::key((typename E::raw_t)raw_of(c, e)) >> KS], 1u);
        }
    }
    wave_sync();

    // scan from the top: bin of rank k-1, count above it, highest occupied bin
    u32 B1 = 0, c_gt = 0, cnt1 = 0, top_bin = 0;
    {
        const int hi = kFineBins - (int)lane * 16;
        u32 cs[16];
        u32 local = 0;
#pragma unroll
        for (int j = 0; j < 16; ++j) { cs[j] = L.hist[hi - 1 - j]; local += cs[j]; }
        const u32 incl = wave_incl_scan(local), excl = incl - local;
        const u32 rem = k > 0 ? (u32)(k - 1) : 0u;
        const bool mine = local > 0 && excl <= rem && rem < incl;
        u32 b = 0, ab = 0, cn = 0, tb = 0;
        {
            u32 acc = excl;
            bool found = false, seen = false;
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                if (!seen && cs[j]) { seen = true; tb = (u32)(hi - 1 - j); }
                if (!found && rem < acc + cs[j]) { found = true; b = (u32)(hi - 1 - j); ab = acc; cn = cs[j]; }
                acc += cs[j];
            }
        }
        const u64 mm = __ballot(mine);
        const u64 occ = __ballot(local > 0);
        if (mm) { const int src = (int)__builtin_ctzll(mm); B1 = bcast(b, src); c_gt = bcast(ab, src); cnt1 = bcast(cn, src); }
        if (occ) top_bin = bcast(tb, (int)__builtin_ctzll(occ));
    }
    wave_sync();

    // the list must hold everything from bin B1 up; fine bins must leave room for
    // the in-bin key bits, the index and the class bit in one 32-bit word
    const u32 t_lo = B1 << KS;                                   // smallest key of bin B1
    const u32 range = (((top_bin + 1u) << KS) - 1u) - t_lo;      // largest possible key - t_lo
    const int sh = range < (u32)kFineBins ? 0 : (32 - __clz((int)range)) - 10;
    const bool hard = (k > 0) && ((int)(c_gt + cnt1) > cap || sh + w > 31);
    if (hard) {
        if (lane == 0) a.fallback[r] = 1u;
        return;
    }

    // ---- 2. ordered compaction into L ----------------------------------------------
    u32 nL = 0;
    if (k > 0) {
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            u32 cntl = 0;
#pragma unroll
            for (int e = 0; e < EPC; ++e) {
                const u32 key = E::key((typename E::raw_t)raw_of(c, e));
                cntl += (key >= t_lo && key != 0u) ? 1u : 0u;
            }
            const u32 incl = wave_incl_scan(cntl);
            u32 pos = nL + incl - cntl;
            const int base = (c * kWave + (int)lane) * EPC;
#pragma unroll
            for (int e = 0; e < EPC; ++e) {
                const u32 raw = raw_of(c, e);
                const u32 key = E::key((typename E::raw_t)raw);
                if (key >= t_lo && key != 0u) {
                    if (pos < (u32)cap) { L.Lraw[pos] = raw; L.Lidx[pos] = (uint16_t)(base + e); }
                    ++pos;
                }
            }
            nL += bcast(incl, kWave - 1);
        }
        if (nL > (u32)cap) nL = (u32)cap;      // cannot happen: nL <= c_gt + cnt1 <= cap
    }
    for (int i = lane; i < kFineBins; i += kWave) L.hist[i] = 0;
    wave_sync();

    // ---- 3. fine bins, ranks ----------------------------------------------------------
    const int nslots = (int)((nL + kWave - 1) / kWave);
    for (int s = 0; s < nslots; ++s) {
        const u32 p = s * kWave + lane;
        if (p < nL) {
            const u32 raw = L.Lraw[p];
            const u32 d = (E::key((typename E::raw_t)raw) - t_lo) >> sh;
            atomicAdd(&L.hist[d], E::neg((typename E::raw_t)raw) ? 0x10000u : 1u);
        }
    }
    wave_sync();
    {   // exclusive prefix from the top, per class; repack as pos | neg << 11 | fill << 22
        const int hi = kFineBins - (int)lane * 16;
        u32 cs[16];
        u32 local = 0;
#pragma unroll
        for (int j = 0; j < 16; ++j) { cs[j] = L.hist[hi - 1 - j]; local += cs[j]; }
        u32 acc = wave_incl_scan(local) - local;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            L.hist[hi - 1 - j] = (acc & 0xFFFFu) | ((acc >> 16) << 11);
            acc += cs[j];
        }
    }
    wave_sync();
    const u32 inmask = (1u << sh) - 1u;
    for (int s = 0; s < nslots; ++s) {
        const u32 p = s * kWave + lane;
        if (p < nL) {
            const u32 raw = L.Lraw[p];
            const u32 rel = E::key((typename E::raw_t)raw) - t_lo;
            const u32 old = atomicAdd(&L.hist[rel >> sh], 1u << 22);
            const u32 at = (old & 0x7FFu) + ((old >> 11) & 0x7FFu) + (old >> 22);
            const u32 comp = ((rel & inmask) << w) | (idxmask - (u32)L.Lidx[p]);
            L.S[at] = (comp << 1) | E::neg((typename E::raw_t)raw);
        }
    }
    wave_sync();
    u32 n_pos = 0, n_neg = 0;
    for (int s = 0; s < nslots; ++s) {
        const u32 p = s * kWave + lane;
        bool kept = false;
        u32 neg = 0;
        if (p < nL) {
            const u32 raw = L.Lraw[p];
            neg = E::neg((typename E::raw_t)raw);
            const u32 rel = E::key((typename E::raw_t)raw) - t_lo;
            const u32 wd = L.hist[rel >> sh];
            const u32 pe = wd & 0x7FFu, ne = (wd >> 11) & 0x7FFu, cnt = wd >> 22;
            const u32 comp = ((rel & inmask) << w) | (idxmask - (u32)L.Lidx[p]);
            u32 gt_all = 0, gt_same = 0;
            if (cnt > 1) {
                const u32 base = pe + ne;
                for (u32 j = 0; j < cnt; ++j) {
                    const u32 o = L.S[base + j];
                    const u32 g = (o >> 1) > comp ? 1u : 0u;
                    gt_all += g;
                    gt_same += g & ((o & 1u) == neg ? 1u : 0u);
                }
            }
            kept = (pe + ne + gt_all) < (u32)k;               // overall rank < k (ATKF)
            L.Lr[p] = kept ? (uint16_t)((neg ? ne : pe) + gt_same) : (uint16_t)0xFFFFu;
        }
        n_pos += (u32)__popcll(__ballot(kept && !neg));
        n_neg += (u32)__popcll(__ballot(kept && neg));
    }
    const u32 n = n_pos + n_neg;
    const u32 n_cls[2] = { n_pos, n_neg };
    const u32 Kc[2] = { n_pos / (u32)M, n_neg / (u32)M };

    // block starts in closed form (K, ..., K, K + remainder per class)
    if ((int)lane < B2) {
        const int s = (int)lane >= M ? 1 : 0, m = (int)lane - s * M;
        L.blk_start[lane] = (s ? n_pos : 0u) + (u32)m * Kc[s];
        L.run[lane] = 0;
        L.vminb[lane] = 0; L.vmaxb[lane] = 0;
    }
    if (lane == 0) L.blk_start[B2] = n;
    wave_sync();

    // ---- 4. blocks, stable split by block, block-ordered arrays ---------------------------
    // (the histogram region is free now: it becomes bo_val | bo_idx | stream image)
    u32* bo_val = L.hist;
    uint16_t* bo_idx = (uint16_t*)(L.hist + k);
    u32* stage = L.hist + k + (k + 1) / 2;
    int nbits = 0;
    while ((1 << nbits) < B2) ++nbits;
    for (int s = 0; s < nslots; ++s) {
        const u32 p = s * kWave + lane;
        bool kept = false;
        u32 b = 0, raw = 0, idx = 0;
        if (p < nL) {
            const u32 rr = L.Lr[p];
            if (rr != 0xFFFFu) {
                kept = true;
                raw = L.Lraw[p];
                idx = L.Lidx[p];
                const int cls = (int)E::neg((typename E::raw_t)raw);
                const u32 K = Kc[cls];
                u32 m = (u32)(M - 1);
                if (K) {
                    u32 qd = (u32)((float)rr * (1.0f / (float)K));       // rr / K with a +-1 repair
                    if (qd * K > rr) --qd;
                    if ((qd + 1) * K <= rr) ++qd;
                    m = qd < (u32)(M - 1) ? qd : (u32)(M - 1);
                }
                b = (u32)cls * (u32)M + m;
                const u32 last = (m < (u32)(M - 1)) ? (m + 1) * K - 1 : n_cls[cls] - 1;
                if (rr == m * K) L.vmaxb[b] = E::key((typename E::raw_t)raw);
                if (rr == last) L.vminb[b] = E::key((typename E::raw_t)raw);
            }
        }
        u64 peers = __ballot(kept);
        for (int bit = 0; bit < nbits; ++bit) {
            const bool on = (b >> bit) & 1u;
            const u64 bal = __ballot(kept && on);
            peers &= on ? bal : ~bal;
        }
        const u32 before = mask_rank(peers);
        u32 basep = 0;
        if (kept) basep = L.run[b];
        wave_sync();
        if (kept) {
            if (before == 0) L.run[b] = basep + (u32)__popcll(peers);
            const u32 pos = L.blk_start[b] + basep + before;
            if (pos < (u32)k) { bo_val[pos] = E::value_bits(E::key((typename E::raw_t)raw)); bo_idx[pos] = (uint16_t)idx; }
        }
        wave_sync();
    }

    // ---- 5. ABQ tables --------------------------------------------------------------------------
    if ((int)lane < B2) {
        const u32 cnt = L.blk_start[lane + 1] - L.blk_start[lane];
        int dg = 1, e = 0;
        float rng = 0.f;
        if (cnt) {
            const u32 lo = E::value_bits(L.vminb[lane]), hi = E::value_bits(L.vmaxb[lane]);
            rng = __uint_as_float(hi) - __uint_as_float(lo);
            dg = !(rng >= 0x1p-100f);
            e = ilogb_bits(hi) + 1;
        }
        L.degen[lane] = dg; L.e_tab[lane] = e;
        for (int t = 0; t < nq; ++t) {
            const float Lq = (float)((1u << a.qlist[t]) - 1u);
            L.inv_tab[lane * nq + t] = dg ? 0.f : Lq / rng;
            L.sums[lane * (nq + 1) + t] = 0;
        }
        L.sums[lane * (nq + 1) + nq] = 0;
    }
    wave_sync();

    // integer residual / energy sums; each lane walks a contiguous run of the
    // block-ordered list, so its partial sums stay in registers across a block
    const u32 per = (n + kWave - 1) / kWave;
    {
        const u32 p0 = lane * per, p1 = (p0 + per < n) ? p0 + per : n;
        int cur = -1;
        u32 acc[kMaxQ];
        u64 accE = 0;
#pragma unroll
        for (int t = 0; t < kMaxQ; ++t) acc[t] = 0;
        float vmin = 0.f;
        int e = 0, dg = 1;
        u32 held = 0;
        auto flush = [&]() {
            if (cur < 0) return;
#pragma unroll
            for (int t = 0; t < kMaxQ; ++t)
                if (t < nq && acc[t]) { atomicAdd(&L.sums[cur * (nq + 1) + t], (u64)acc[t]); acc[t] = 0; }
            if (accE) { atomicAdd(&L.sums[cur * (nq + 1) + nq], accE); accE = 0; }
            held = 0;
        };
        for (u32 p = p0; p < p1; ++p) {
            int b = cur < 0 ? 0 : cur;
            while (b < B2 - 1 && p >= L.blk_start[b + 1]) ++b;
            if (b != cur || held >= 8) {
                flush();
                cur = b;
                vmin = __uint_as_float(E::value_bits(L.vminb[b]));
                e = L.e_tab[b]; dg = L.degen[b];
            }
            const u32 abits = bo_val[p];
            const u64 A = energy_grid(abits, e);
            accE += A * A;
            ++held;
            if (!dg) {
                const float d = __uint_as_float(abits) - vmin;
#pragma unroll
                for (int t = 0; t < kMaxQ; ++t) {
                    if (t < nq) {
                        const float Lq = (float)((1u << a.qlist[t]) - 1u);
                        const float y = d * L.inv_tab[b * nq + t];
                        const float c = fminf(fmaxf(rintf(y), 0.f), Lq);
                        const int rho = (int)rintf((y - c) * 32768.0f);
                        acc[t] += (u32)(rho * rho);
                    }
                }
            }
        }
        flush();
    }
    wave_sync();

    // smallest feasible bitwidth per block; meta; bit offsets
    u32 myq = 0, mybits = 0;
    float my_inv = 0.f;
    if ((int)lane < B2) {
        const u32 cnt = L.blk_start[lane + 1] - L.blk_start[lane];
        float vmin = 0.f, vmax = 0.f;
        int q = a.qlist[0], tsel = 0;
        u32 flag = 0;
        if (cnt) {
            vmin = __uint_as_float(E::value_bits(L.vminb[lane]));
            vmax = __uint_as_float(E::value_bits(L.vmaxb[lane]));
            if (!L.degen[lane]) {
                const float rng = vmax - vmin;
                const int e = L.e_tab[lane];
                const double rhs = a.beta * ldexp((double)L.sums[lane * (nq + 1) + nq], 2 * e - 40);
                int chosen = -1;
                for (int t = 0; t < nq && chosen < 0; ++t) {
                    const float Lq = (float)((1u << a.qlist[t]) - 1u);
                    const float o = rng / Lq;
                    const double lhs = ((double)o * (double)o) * (double)L.sums[lane * (nq + 1) + t] * 0x1p-30;
                    if (lhs <= rhs) chosen = t;
                }
                if (chosen < 0) { chosen = nq - 1; flag = 0x80u; }
                tsel = chosen; q = a.qlist[chosen];
            }
            my_inv = L.inv_tab[lane * nq + tsel];
        }
        myq = (u32)q; mybits = cnt * (u32)q;
        const size_t mi = (size_t)r * (size_t)B2 + lane;
        a.mv.vmin[mi] = vmin;
        a.mv.vmax[mi] = vmax;
        a.mv.q[mi] = (uint8_t)((u32)q | flag);
    }
    const u32 incl_bits = wave_incl_scan(mybits);
    const u32 code_bits = bcast(incl_bits, kWave - 1);
    wave_sync();                      // inv_tab reads above are done: reuse its first B2 words
    if ((int)lane < B2) {
        L.qsel[lane] = myq;
        L.code_off[lane] = incl_bits - mybits;
        L.inv_tab[lane] = my_inv;     // inverse step at the chosen bitwidth
    }
    const u32 idx_bits = n * (u32)w;
    const u32 row_bits = idx_bits + code_bits;
    u32 row_words = (row_bits + 31u) >> 5;
    if ((u64)row_words > a.cap_words) row_words = (u32)a.cap_words;   // cannot happen (worst-case capacity)
    for (u32 i = lane; i < row_words; i += kWave) stage[i] = 0;
    wave_sync();

    // ---- packing ----------------------------------------------------------------------------------
    {
        const u32 p0 = lane * per, p1 = (p0 + per < n) ? p0 + per : n;
        int b = 0;
        for (u32 p = p0; p < p1; ++p) {
            while (b < B2 - 1 && p >= L.blk_start[b + 1]) ++b;
            const u32 q = L.qsel[b];
            u32 c = 0;
            if (!L.degen[b]) {
                const float Lq = (float)((1u << q) - 1u);
                const float vmin = __uint_as_float(E::value_bits(L.vminb[b]));
                const float y = (__uint_as_float(bo_val[p]) - vmin) * L.inv_tab[b];
                c = (u32)fminf(fmaxf(rintf(y), 0.f), Lq);
            }
            {   // index field
                const u32 P = p * (u32)w, wi = P >> 5, sft = P & 31u, val = bo_idx[p];
                atomicOr(&stage[wi], val << sft);
                if (sft + (u32)w > 32u) atomicOr(&stage[wi + 1], val >> (32u - sft));
            }
            {   // code field
                const u32 P = idx_bits + L.code_off[b] + (p - L.blk_start[b]) * q, wi = P >> 5, sft = P & 31u;
                atomicOr(&stage[wi], c << sft);
                if (sft + q > 32u) atomicOr(&stage[wi + 1], c >> (32u - sft));
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
    }
}

}  // namespace slicer
