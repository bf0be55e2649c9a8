// Generic encoder: one workgroup per row, the row read from global memory as many
// times as the selection needs, per-row lists kept in the caller's workspace.
// Works for any row length, keep ratio and block count the library accepts; the
// row-resident kernels in slicer_encode_small.hpp are the fast path for short rows.
//
// Order statistics are taken on a composite integer that is distinct per element,
//     comp(i) = key(i) << w  |  (2^w - 1 - i),        key = |x| as an integer,
// so "larger comp" means "larger magnitude, then lower index": the tie rule of the
// top-K filter (Sec. 3.1) and of the magnitude sort (Sec. 3.2 step 1) at once.  A
// most-significant-digit radix select finds the comp of a given rank; it stops as
// soon as the target is the smallest member of its digit bin, because then the bin
// prefix alone is an exact threshold.
#pragma once

#include "slicer_common.hpp"

namespace slicer {

struct EncArgs {
    const void* x;
    int64_t R, N, k;
    int M, Mn, w, nq;       // blocks of the positive / negative class (block order +0..+M-1, -0..-Mn-1)
    int qlist[kMaxQ];       // allowed bitwidths, ascending
    double beta;
    u64 cap_words;          // per-row slot capacity in words
    // workspace
    u64* row_words;         // [R]
    u32* slots;             // [R][cap_words]
    u64* kept;              // [R][k]   class<<63 | key<<32 | idx, ascending idx
    u32* bo_idx;            // [R][k]   block-ordered indices
    u32* bo_val;            // [R][k]   block-ordered |x| (fp32 bits)
    const u32* only_flagged;// if set: rows with a zero flag are skipped (already encoded)
    int64_t rows_per_wg;    // consecutive rows a workgroup walks (1 unless only_flagged is set)
    Ladder lad;             // fixed multi-level mode: no search, block m uses qlist[index(m)]
    int guard;              // 0: relative squared-error budget (beta); 1: the DS mismatch of Eq. "DS" (beta = delta), greedy descent
    int asym;               // 1: asymmetric thresholds of Sec. 3.1 (lambda > 0)
    float one_plus, one_minus;   // 1 + lambda, 1 - lambda in fp32
    // meta
    MetaView mv;
};

constexpr int kStageWords = 4096;   // LDS staging / histogram region, 16 KB
constexpr int kSelBits = 11;        // digit width of the single-target select
constexpr int kMsBits = 8;          // digit width of the multi-target select
constexpr int kTgtBatch = kStageWords >> kMsBits;  // 16 targets per batch

// Locate, walking from the top bin down, the bin that holds descending rank `rem`
// (0-based) of a histogram: out[0] = bin, out[1] = elements in higher bins,
// out[2] = elements in the bin.  Needs rem < sum(hist).
template <int BLOCK>
__device__ inline void block_find_desc(const u32* hist, int NB, u32 rem, u32* scan_scratch, u32* out)
{
    const int seg = (NB + BLOCK - 1) / BLOCK;
    const int hi = NB - (int)threadIdx.x * seg;
    const int lo = hi - seg > 0 ? hi - seg : 0;
    u32 local = 0;
    for (int b = hi - 1; b >= lo; --b) local += hist[b];
    u32 total;
    u32 excl = block_excl_scan<BLOCK>(local, scan_scratch, &total);
    if (local > 0 && excl <= rem && rem < excl + local) {
        u32 acc = excl;
        for (int b = hi - 1; b >= lo; --b) {
            u32 c = hist[b];
            if (rem < acc + c) { out[0] = (u32)b; out[1] = acc; out[2] = c; break; }
            acc += c;
        }
    }
    __syncthreads();
}

// Same search by one wave over a 256-bin histogram; result valid in every lane.
__device__ inline void wave_find_desc256(const u32* hist, u32 rem, u32& bin, u32& above, u32& cnt)
{
    const u32 lane = lane_id();
    const int hi = 256 - (int)lane * 4;
    u32 c3 = hist[hi - 1], c2 = hist[hi - 2], c1 = hist[hi - 3], c0 = hist[hi - 4];
    u32 local = c0 + c1 + c2 + c3;
    u32 incl = wave_incl_scan(local);
    u32 excl = incl - local;
    bool mine = local > 0 && excl <= rem && rem < incl;
    u32 b = 0, a = 0, c = 0;
    if (mine) {
        u32 acc = excl;
        if (rem < acc + c3) { b = hi - 1; a = acc; c = c3; }
        else { acc += c3;
            if (rem < acc + c2) { b = hi - 2; a = acc; c = c2; }
            else { acc += c2;
                if (rem < acc + c1) { b = hi - 3; a = acc; c = c1; }
                else { acc += c1; b = hi - 4; a = acc; c = c0; } } }
    }
    u64 m = __ballot(mine);
    int src = m ? (int)__builtin_ctzll(m) : 0;
    bin = __shfl(b, src); above = __shfl(a, src); cnt = __shfl(c, src);
}

__device__ inline void stage_or_bits(u32* stage, u64 lo, u64 hi, u64 P, u32 v, int nb)
{
    if (P + (u64)nb <= lo || P >= hi) return;
    if (P < lo) { int drop = (int)(lo - P); v >>= drop; nb -= drop; P = lo; }
    if (P + (u64)nb > hi) { nb = (int)(hi - P); v &= (1u << nb) - 1u; }
    u32 rel = (u32)(P - lo);
    u32 wi = rel >> 5, sh = rel & 31u;
    atomicOr(&stage[wi], v << sh);
    if (sh + (u32)nb > 32u) atomicOr(&stage[wi + 1], v >> (32u - sh));
}

// Encodes rows [r_begin, r_end) one after the other with the whole workgroup; with
// a.only_flagged set, only the rows whose flag is non-zero.
template <int DT, int BLOCK>
__device__ inline void enc_generic_rows(const EncArgs& a, const int64_t r_begin, const int64_t r_end)
{
    typedef Elem<DT> E;
    typedef typename E::raw_t raw_t;
    constexpr int NW = BLOCK / kWave;

    __shared__ u32 sA[kStageWords];              // histograms / pack staging
    __shared__ u32 s_scan[NW + 1];
    __shared__ u32 s_out[4];
    __shared__ u64 s_thr[2][kMaxBlocks];         // MS thresholds per class
    __shared__ u64 tg_prefix[kTgtBatch];
    __shared__ u32 tg_rem[kTgtBatch];
    __shared__ int tg_cls[kTgtBatch], tg_j[kTgtBatch], tg_done[kTgtBatch], tg_owner[kTgtBatch];
    __shared__ u32 blk_start[kMaxB2 + 1];
    __shared__ u32 vminb[kMaxB2], vmaxb[kMaxB2];
    __shared__ int e_tab[kMaxB2], er_tab[kMaxB2], degen[kMaxB2], qsel[kMaxB2];
    __shared__ float inv_sel[kMaxB2];
    __shared__ u64 code_off[kMaxB2 + 1];
    __shared__ float inv_tab[kMaxB2][kMaxQ];
    __shared__ u64 sums[kMaxB2][kMaxQ + 1];
    __shared__ u32 cnt_wave[NW][kMaxB2];
    __shared__ u32 run_base[kMaxB2];
    __shared__ u32 s_range[2];
    __shared__ u32 s_asym[4];                    // asymmetric thresholds: smallest kept key, |S_strict|, fill candidates

    const int tid = threadIdx.x;
    const u32 lane = lane_id();
    const int wid = tid / kWave;
    if (a.only_flagged) {       // one coalesced look at this workgroup's flags: usually none is set
        int any = 0;
        for (int64_t r = r_begin + tid; r < r_end; r += BLOCK) any |= (int)a.only_flagged[r];
        if (!__syncthreads_or(any)) return;
    }
    for (int64_t r = r_begin; r < r_end; ++r) {
    if (a.only_flagged && !a.only_flagged[r]) continue;      // uniform: the whole workgroup skips
    const int64_t N = a.N;
    const int M = a.M, Mn = a.Mn, w = a.w, B2 = a.M + a.Mn;
    const int Mc[2] = { M, Mn };
    const raw_t* __restrict__ xr = (const raw_t*)a.x + (size_t)r * (size_t)N;
    u64* __restrict__ kept = a.kept + (size_t)r * (size_t)a.k;
    u32* __restrict__ bo_idx = a.bo_idx + (size_t)r * (size_t)a.k;
    u32* __restrict__ bo_val = a.bo_val + (size_t)r * (size_t)a.k;
    u32* __restrict__ slot = a.slots + (size_t)r * (size_t)a.cap_words;

    const u64 idxmask = (1ull << w) - 1ull;
    const int TB = E::kKeyBits + w;

    // ------------------------------------------------------------------
    // ATKF: comp of descending rank k-1 over the whole row -> kept <=> comp >= thrK
    // ------------------------------------------------------------------
    // select_rank(pred, rank): a comp threshold t such that exactly rank + 1 of the elements with
    // pred(key, neg) have comp >= t (MSD radix select; needs rank < number of such elements)
    auto select_rank = [&](auto pred, u32 rank) -> u64 {
        u64 prefix = 0;
        int hi = TB;
        u32 rem = rank;
        for (;;) {
            const int bits = hi < kSelBits ? hi : kSelBits;
            const int shift = hi - bits;
            const int NB = 1 << bits;
            for (int i = tid; i < NB; i += BLOCK) sA[i] = 0;
            __syncthreads();
            for (int64_t i = tid; i < N; i += BLOCK) {
                const raw_t rv = xr[i];
                u32 key = E::key(rv);
                u64 comp = ((u64)key << w) | (idxmask - (u64)i);
                if (pred(key, E::neg(rv)) && (comp >> hi) == prefix) atomicAdd(&sA[(u32)(comp >> shift) & (u32)(NB - 1)], 1u);
            }
            __syncthreads();
            block_find_desc<BLOCK>(sA, NB, rem, s_scan, s_out);
            const u32 bin = s_out[0], above = s_out[1], cnt = s_out[2];
            __syncthreads();
            rem -= above;
            prefix = (prefix << bits) | bin;
            hi = shift;
            if (rem == cnt - 1 || hi == 0) break;
        }
        return prefix << hi;
    };
    u64 thrK = ~0ull;      // k == 0: nothing kept
    if (a.k > 0) thrK = select_rank([](u32, u32) { return true; }, (u32)(a.k - 1));

    // Asymmetric thresholds (Sec. 3.1, lambda > 0).  tau = the k-th largest magnitude = the smallest
    // key at or above thrK; strictly retained are the positives above (1 + lambda) tau and the
    // negatives above (1 - lambda) tau.  Fewer than k of them: the set is filled from the elements
    // at or below tau that are not in it, largest first (thr2 is the last one taken); k or more:
    // only the k largest of the set stay (thr2 is the last one kept).
    u32 tp_bits = 0, tn_bits = 0, tau_key = 0;
    u64 thr2 = 0;
    bool asym_trim = false;
    auto is_strict = [&](u32 key, u32 neg) -> bool {       // |x| as an fp32 pattern orders like the value
        return E::value_bits(key) > (neg ? tn_bits : tp_bits);
    };
    if (a.asym && a.k > 0) {
        if (tid == 0) { s_asym[0] = 0xFFFFFFFFu; s_asym[1] = 0; s_asym[2] = 0; }
        __syncthreads();
        u32 kmin = 0xFFFFFFFFu;
        for (int64_t i = tid; i < N; i += BLOCK) {
            const u32 key = E::key(xr[i]);
            const u64 comp = ((u64)key << w) | (idxmask - (u64)i);
            if (comp >= thrK) kmin = key < kmin ? key : kmin;
        }
        atomicMin(&s_asym[0], kmin);
        __syncthreads();
        tau_key = s_asym[0];
        const float tau = __uint_as_float(E::value_bits(tau_key));
        tp_bits = __float_as_uint(__fmul_rn(a.one_plus, tau));
        tn_bits = __float_as_uint(__fmul_rn(a.one_minus, tau));
        u32 c_loc = 0, f_loc = 0;
        for (int64_t i = tid; i < N; i += BLOCK) {
            const raw_t rv = xr[i];
            const u32 key = E::key(rv);
            if (is_strict(key, E::neg(rv))) ++c_loc;
            else if (key <= tau_key) ++f_loc;
        }
        atomicAdd(&s_asym[1], c_loc);
        atomicAdd(&s_asym[2], f_loc);
        __syncthreads();
        const u32 c = s_asym[1], f = s_asym[2];
        __syncthreads();
        if ((int64_t)c >= a.k) {
            asym_trim = true;
            thr2 = select_rank(is_strict, (u32)(a.k - 1));
        } else {
            const u32 D = (u32)(a.k - (int64_t)c);
            if (f > D) thr2 = select_rank([&](u32 key, u32 neg) { return !is_strict(key, neg) && key <= tau_key; }, D - 1u);
            else thr2 = 0;                                  // every candidate is taken
        }
    }

    // ------------------------------------------------------------------
    // compaction of the kept non-zeros, ascending index; class counts
    // ------------------------------------------------------------------
    u32 n = 0, n_neg = 0;
    for (int64_t base = 0; base < N; base += BLOCK) {
        const int64_t i = base + tid;
        u32 flag = 0, neg = 0, key = 0;
        if (i < N) {
            raw_t rv = xr[i];
            key = E::key(rv);
            neg = E::neg(rv);
            u64 comp = ((u64)key << w) | (idxmask - (u64)i);
            if (a.asym && a.k > 0) {
                const bool st = is_strict(key, neg);
                const bool in = asym_trim ? (st && comp >= thr2) : (st || (key <= tau_key && comp >= thr2));
                flag = (in && key != 0) ? 1u : 0u;
            } else {
                flag = (comp >= thrK && key != 0) ? 1u : 0u;
            }
        }
        // one scan carries both counts: kept in the low half, kept negatives in the high half
        u32 tot;
        u32 pos = block_excl_scan<BLOCK>(flag | ((flag & neg) << 16), s_scan, &tot) & 0xFFFFu;
        if (flag && (int64_t)(n + pos) < a.k) kept[n + pos] = ((u64)neg << 63) | ((u64)key << 32) | (u64)(u32)i;
        n += tot & 0xFFFFu;
        n_neg += tot >> 16;
    }
    if ((int64_t)n > a.k) n = (u32)a.k;                     // cannot happen: exactly k comps reach thrK
    if (n_neg > n) n_neg = n;
    const u32 n_cls[2] = { n - n_neg, n_neg };
    __threadfence_block();
    __syncthreads();

    // block sizes in closed form (Sec. 3.2 step 2: K = floor(n / M), rest to the last)
    if (tid == 0) {
        u32 acc = 0;
        for (int s = 0; s < 2; ++s) {
            u32 K = n_cls[s] / (u32)Mc[s];
            for (int m = 0; m < Mc[s]; ++m) {
                blk_start[s * M + m] = acc;
                acc += (m < Mc[s] - 1) ? K : n_cls[s] - K * (u32)(Mc[s] - 1);
            }
        }
        blk_start[B2] = acc;
    }
    for (int b = tid; b < B2; b += BLOCK) {
        vminb[b] = 0xFFFFFFFFu; vmaxb[b] = 0u; run_base[b] = 0;
        for (int v = 0; v < NW; ++v) cnt_wave[v][b] = 0;
    }
    __syncthreads();

    // ------------------------------------------------------------------
    // MS: thresholds comp(rank j*K - 1), j = 1..M-1, per class, in batches
    // ------------------------------------------------------------------
    {
        const u32 Kc[2] = { n_cls[0] / (u32)M, n_cls[1] / (u32)Mn };
        const int nt[2] = { Kc[0] ? M - 1 : 0, Kc[1] ? Mn - 1 : 0 };
        const int ntot = nt[0] + nt[1];
        for (int t0 = 0; t0 < ntot; t0 += kTgtBatch) {
            const int nb = ntot - t0 < kTgtBatch ? ntot - t0 : kTgtBatch;
            if (tid < nb) {
                int t = t0 + tid;
                int s = t < nt[0] ? 0 : 1;
                int j = (s == 0 ? t : t - nt[0]) + 1;
                tg_cls[tid] = s; tg_j[tid] = j;
                tg_rem[tid] = (u32)j * Kc[s] - 1u;
                tg_prefix[tid] = 0; tg_done[tid] = 0;
            }
            int hi = TB;
            for (;;) {
                const int bits = hi < kMsBits ? hi : kMsBits;
                const int shift = hi - bits;
                __syncthreads();
                if (tid < nb) {
                    int own = -1;
                    if (!tg_done[tid]) {
                        own = tid;
                        for (int u = tid - 1; u >= 0; --u)
                            if (!tg_done[u] && tg_cls[u] == tg_cls[tid] && tg_prefix[u] == tg_prefix[tid]) own = u;
                    }
                    tg_owner[tid] = own;
                }
                for (int i = tid; i < kStageWords; i += BLOCK) sA[i] = 0;
                __syncthreads();
                for (u32 p = tid; p < n; p += BLOCK) {
                    u64 e = kept[p];
                    int s = (int)(e >> 63);
                    u64 comp = (((e >> 32) & 0x7FFFFFFFull) << w) | (idxmask - (e & 0xFFFFFFFFull));
                    u64 pfx = comp >> hi;
                    for (int u = 0; u < nb; ++u) {
                        if (tg_owner[u] == u && tg_cls[u] == s && tg_prefix[u] == pfx) {
                            atomicAdd(&sA[(u << kMsBits) + ((u32)(comp >> shift) & ((1u << bits) - 1u))], 1u);
                            break;
                        }
                    }
                }
                __syncthreads();
                int pending = 0;
                for (int u = wid; u < nb; u += NW) {
                    if (tg_done[u]) continue;            // wave-uniform
                    u32 bin, above, cnt;
                    wave_find_desc256(sA + (tg_owner[u] << kMsBits), tg_rem[u], bin, above, cnt);
                    u32 rem = tg_rem[u] - above;
                    u64 prefix = (tg_prefix[u] << bits) | bin;
                    bool done = (rem == cnt - 1) || shift == 0;
                    if (lane == 0) {
                        tg_rem[u] = rem; tg_prefix[u] = prefix;
                        if (done) { tg_done[u] = 1; s_thr[tg_cls[u]][tg_j[u] - 1] = prefix << shift; }
                    }
                    if (!done) pending = 1;
                }
                hi = shift;
                if (!__syncthreads_or(pending)) break;
            }
            __syncthreads();
        }
    }
    __syncthreads();

    // ------------------------------------------------------------------
    // block id per kept element, block min/max, stable scatter to block order
    // ------------------------------------------------------------------
    for (u32 base = 0; base < n; base += BLOCK) {
        const u32 p = base + tid;
        const bool valid = p < n;
        u32 b = 0, key = 0, idx = 0;
        if (valid) {
            u64 e = kept[p];
            int s = (int)(e >> 63);
            key = (u32)(e >> 32) & 0x7FFFFFFFu;
            idx = (u32)e;
            u64 comp = ((u64)key << w) | (idxmask - (u64)idx);
            const int Ms = s ? Mn : M;
            int m = Ms - 1;
            if (n_cls[s] >= (u32)Ms) {      // K >= 1: block = #{j : comp < thr_j}, thr decreasing in j
                int lo = 0, hi = Ms - 1;    // count of thresholds above comp lies in [lo, hi]
                while (lo < hi) {
                    int mid = (lo + hi) >> 1;           // is thr[mid] > comp ?
                    if (s_thr[s][mid] > comp) lo = mid + 1; else hi = mid;
                }
                m = lo;
            }
            b = (u32)(s * M + m);
            atomicMin(&vminb[b], key);
            atomicMax(&vmaxb[b], key);
        }
        u64 remaining = __ballot(valid);
        u32 myrank = 0;
        while (remaining) {
            int leader = (int)__builtin_ctzll(remaining);
            u32 b0 = __shfl(b, leader);
            u64 m = __ballot(valid && b == b0);
            if (valid && b == b0) myrank = mask_rank(m);
            if ((int)lane == leader) cnt_wave[wid][b0] = (u32)__popcll(m);
            remaining &= ~m;
        }
        __syncthreads();
        if (valid) {
            u32 off = run_base[b];
            for (int v = 0; v < wid; ++v) off += cnt_wave[v][b];
            u32 pos = blk_start[b] + off + myrank;
            if (pos < n) {
                bo_idx[pos] = idx;
                bo_val[pos] = E::value_bits(key);
            }
        }
        __syncthreads();
        for (int bb = tid; bb < B2; bb += BLOCK) {
            u32 s = 0;
            for (int v = 0; v < NW; ++v) { s += cnt_wave[v][bb]; cnt_wave[v][bb] = 0; }
            run_base[bb] += s;
        }
        __syncthreads();
    }
    __threadfence_block();
    __syncthreads();

    // ------------------------------------------------------------------
    // ABQ: per-block quantiser tables, integer residual / energy sums
    // ------------------------------------------------------------------
    for (int b = tid; b < B2; b += BLOCK) {
        u32 cnt = blk_start[b + 1] - blk_start[b];
        int dg = 1, e = 0, er = 0;
        float rng1 = 1.f;
        if (cnt) {
            u32 vminbits = E::value_bits(vminb[b]), vmaxbits = E::value_bits(vmaxb[b]);
            const float rng = __uint_as_float(vmaxbits) - __uint_as_float(vminbits);
            dg = !(rng > 0.f);                       // only a range of exactly 0 is degenerate
            if (!dg) { er = range_exp(rng); rng1 = unit_range(rng, er); }
            e = ilogb_bits(vmaxbits) + 1;
        }
        degen[b] = dg; e_tab[b] = e; er_tab[b] = er;
        for (int t = 0; t < a.nq; ++t) {
            float L = (float)((1u << a.qlist[t]) - 1u);
            inv_tab[b][t] = dg ? 0.f : L / rng1;
            sums[b][t] = 0;
        }
        sums[b][kMaxQ] = 0;
    }
    __syncthreads();
    {
        int cur = -1;
        u64 acc[kMaxQ];
        u64 accE = 0;
#pragma unroll
        for (int t = 0; t < kMaxQ; ++t) acc[t] = 0;
        float vmin = 0.f;
        int e = 0, dg = 1, er = 0;
        auto flush = [&]() {
            if (cur < 0) return;
#pragma unroll
            for (int t = 0; t < kMaxQ; ++t)
                if (t < a.nq && acc[t]) { atomicAdd(&sums[cur][t], acc[t]); acc[t] = 0; }
            if (accE) { atomicAdd(&sums[cur][kMaxQ], accE); accE = 0; }
        };
        for (u32 p = tid; p < n; p += BLOCK) {
            int b = cur < 0 ? 0 : cur;
            while (b < B2 - 1 && p >= blk_start[b + 1]) ++b;
            if (b != cur) {
                flush();
                cur = b;
                vmin = __uint_as_float(E::value_bits(vminb[b]));
                e = e_tab[b]; dg = degen[b]; er = er_tab[b];
            }
            u32 abits = bo_val[p];
            float av = __uint_as_float(abits);
            u64 A = energy_grid(abits, e);
            accE += A * A;
            if (!dg && a.guard == 1) {
                // Eq. "DS": codes at q_bit shifted down against the codes at q
                const float d = to_unit(av - vmin, er);
                const int top = a.nq - 1, qtop = a.qlist[top];
                const u32 c0 = (u32)fminf(fmaxf(rintf(d * inv_tab[b][top]), 0.f), (float)((1u << qtop) - 1u));
#pragma unroll
                for (int t = 0; t < kMaxQ; ++t) {
                    if (t < top) {
                        const float L = (float)((1u << a.qlist[t]) - 1u);
                        const u32 c = (u32)fminf(fmaxf(rintf(d * inv_tab[b][t]), 0.f), L);
                        const u32 ref = c0 >> (qtop - a.qlist[t]);
                        acc[t] += (u64)(ref > c ? ref - c : c - ref);
                    }
                }
            } else if (!dg) {
                float d = to_unit(av - vmin, er);
#pragma unroll
                for (int t = 0; t < kMaxQ; ++t) {
                    if (t < a.nq) {
                        float L = (float)((1u << a.qlist[t]) - 1u);
                        float y = d * inv_tab[b][t];
                        float c = fminf(fmaxf(rintf(y), 0.f), L);
                        int rho = (int)rintf((y - c) * 32768.0f);
                        acc[t] += (u64)(u32)(rho * rho);
                    }
                }
            }
        }
        flush();
    }
    __syncthreads();

    // ------------------------------------------------------------------
    // ABQ: smallest feasible bitwidth per block; meta
    // ------------------------------------------------------------------
    for (int b = tid; b < B2; b += BLOCK) {
        u32 cnt = blk_start[b + 1] - blk_start[b];
        float vmin = 0.f, vmax = 0.f;
        int q = a.qlist[0], tsel = 0;
        u32 flag = 0;
        if (cnt) {
            vmin = __uint_as_float(E::value_bits(vminb[b]));
            vmax = __uint_as_float(E::value_bits(vmaxb[b]));
            if (!degen[b]) {
                float rng = vmax - vmin;
                const int e = e_tab[b];
                const double rhs = a.beta * ldexp((double)sums[b][kMaxQ], 2 * e - 40);
                int chosen = -1;
                for (int t = 0; t < a.nq && chosen < 0; ++t) {
                    float L = (float)((1u << a.qlist[t]) - 1u);
                    float o = rng / L;
                    double lhs = ((double)o * (double)o) * (double)sums[b][t] * 0x1p-30;
                    if (lhs <= rhs) chosen = t;
                }
                if (chosen < 0) { chosen = a.nq - 1; flag = 0x80u; }
                tsel = chosen; q = a.qlist[chosen];
            }
        }
        if (a.guard == 1) {         // greedy descent from q_bit while the mismatch stays within delta
            int chosen = cnt ? a.nq - 1 : 0;
            for (int t = a.nq - 2; t >= 0 && cnt; --t) {
                if ((double)sums[b][t] <= a.beta * (double)cnt) chosen = t; else break;
            }
            tsel = chosen; q = a.qlist[chosen]; flag = 0;
        }
        if (a.lad.on) {             // the bitwidth is given, also for empty and degenerate blocks
            tsel = (int)ladder_index(a.lad, b < M ? b : b - M);
            q = a.qlist[tsel]; flag = 0;
        }
        qsel[b] = q;
        inv_sel[b] = cnt ? inv_tab[b][tsel] : 0.f;
        size_t mi = (size_t)r * (size_t)B2 + (size_t)b;
        a.mv.vmin[mi] = vmin;
        a.mv.vmax[mi] = vmax;
        a.mv.q[mi] = (uint8_t)((u32)q | flag);
    }
    __syncthreads();
    if (tid == 0) {
        u64 acc = 0;
        for (int b = 0; b < B2; ++b) {
            code_off[b] = acc;
            acc += (u64)(blk_start[b + 1] - blk_start[b]) * (u64)qsel[b];
        }
        code_off[B2] = acc;
        a.mv.n_pos[r] = n_cls[0];
        a.mv.n_neg[r] = n_cls[1];
    }
    __syncthreads();

    // ------------------------------------------------------------------
    // packing into the row's slot, staged through LDS one chunk at a time
    // ------------------------------------------------------------------
    const u64 idx_bits = (u64)n * (u64)w;
    const u64 row_bits = idx_bits + code_off[B2];
    u64 row_words = (row_bits + 31) >> 5;
    if (row_words > a.cap_words) row_words = a.cap_words;   // cannot happen: the capacity is the worst case
    if (tid == 0) a.row_words[r] = row_words;
    for (u64 c0 = 0; c0 < row_words; c0 += kStageWords) {
        const u64 cw = row_words - c0 < (u64)kStageWords ? row_words - c0 : (u64)kStageWords;
        const u64 lo = c0 << 5, hi = (c0 + cw) << 5;
        for (int i = tid; i < (int)cw; i += BLOCK) sA[i] = 0;
        if (tid == 0) {     // elements whose code field meets [lo, hi)
            u32 plo = n, phi = 0;
            for (int b = 0; b < B2; ++b) {
                u32 cnt = blk_start[b + 1] - blk_start[b];
                if (!cnt) continue;
                u64 cs = idx_bits + code_off[b], ce = idx_bits + code_off[b + 1];
                if (ce <= lo || cs >= hi) continue;
                u64 q = (u64)qsel[b];
                u64 jlo = ((lo > cs ? lo : cs) - cs) / q;
                u64 jhi = ((hi < ce ? hi : ce) - cs + q - 1) / q;
                u32 a0 = blk_start[b] + (u32)jlo, a1 = blk_start[b] + (u32)jhi;
                plo = a0 < plo ? a0 : plo;
                phi = a1 > phi ? a1 : phi;
            }
            s_range[0] = plo; s_range[1] = phi;
        }
        __syncthreads();
        if (lo < idx_bits) {
            u64 p0 = lo / (u64)w;
            u64 p1 = (hi + (u64)w - 1) / (u64)w;
            if (p1 > n) p1 = n;
            for (u64 p = p0 + tid; p < p1; p += BLOCK)
                stage_or_bits(sA, lo, hi, p * (u64)w, bo_idx[p], w);
        }
        {
            const u32 p0 = s_range[0], p1 = s_range[1];
            int b = 0;
            for (u32 p = p0 + tid; p < p1; p += BLOCK) {
                while (b < B2 - 1 && p >= blk_start[b + 1]) ++b;
                u32 c = 0;
                const int q = qsel[b];
                if (!degen[b]) {
                    float L = (float)((1u << q) - 1u);
                    float vmin = __uint_as_float(E::value_bits(vminb[b]));
                    float y = to_unit(__uint_as_float(bo_val[p]) - vmin, er_tab[b]) * inv_sel[b];
                    c = (u32)fminf(fmaxf(rintf(y), 0.f), L);
                }
                stage_or_bits(sA, lo, hi, idx_bits + code_off[b] + (u64)(p - blk_start[b]) * (u64)q, c, q);
            }
        }
        __syncthreads();
        for (int i = tid; i < (int)cw; i += BLOCK) slot[c0 + i] = sA[i];
        __syncthreads();
    }
    __syncthreads();
    }   // rows of this workgroup
}

template <int DT, int BLOCK>
__global__ __launch_bounds__(BLOCK) void enc_generic_kernel(EncArgs a)
{
    const int64_t r0 = (int64_t)blockIdx.x * a.rows_per_wg;
    enc_generic_rows<DT, BLOCK>(a, r0, r0 + a.rows_per_wg < a.R ? r0 + a.rows_per_wg : a.R);
}

// ---- row offsets (exclusive scan of the row word counts), header, gather ------------------
// Batches of more than kScanRows rows take two launches: (1) every workgroup scans the word counts of 256 consecutive rows and
// leaves the rows' offsets relative to its chunk plus the chunk total; (2) the gather
// kernel adds the totals of the preceding chunks, writes the final offsets and the header
// and copies each row's slot to its place in the contiguous stream.

constexpr int kScanRows = 256;
constexpr int kGatherWords = 1024;   // slot words one wavefront copies

struct FinishArgs {
    int64_t R, N, k;
    int M, Mn, w, dt;
    u32 bit_set;
    const u64* row_words;   // [R]
    u64* row_off_local;     // [R]  offset of the row inside its chunk of kScanRows rows
    u64* chunk_tot;         // [ceil(R / kScanRows)]
    const u32* slots;
    u64 cap_words;
    int chunks_per_row;     // gather wavefronts per row (kGatherWords words each)
    u32* stream;
    void* meta;
    MetaView mv;
};

__device__ inline void rowscan_chunk(const FinishArgs& a)
{
    __shared__ u64 s_part[kScanRows / kWave];
    const int tid = threadIdx.x;
    const u32 lane = lane_id();
    const int wid = tid / kWave;
    const int64_t i = (int64_t)blockIdx.x * kScanRows + tid;
    const u64 v = i < a.R ? a.row_words[i] : 0ull;
    u64 inc = v;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        u64 t = __shfl_up(inc, d);
        if (lane >= (u32)d) inc += t;
    }
    if (lane == kWave - 1) s_part[wid] = inc;
    __syncthreads();
    u64 wbase = 0, tot = 0;
    for (int v2 = 0; v2 < kScanRows / kWave; ++v2) {
        const u64 sp = s_part[v2];
        if (v2 < wid) wbase += sp;
        tot += sp;
    }
    if (i < a.R) a.row_off_local[i] = wbase + inc - v;
    if (tid == 0) a.chunk_tot[blockIdx.x] = tot;
}

__global__ __launch_bounds__(kScanRows) void enc_rowscan_kernel(FinishArgs a)
{
    rowscan_chunk(a);
}

// The same scan, preceded by the generic encoder for the rows of this chunk that a fast
// path flagged (normally none: one coalesced look at the flags, then straight to the scan).
template <int DT>
__global__ __launch_bounds__(kScanRows) void enc_fix_rowscan_kernel(EncArgs ea, FinishArgs a)
{
    const int64_t r0 = (int64_t)blockIdx.x * kScanRows;
    enc_generic_rows<DT, kScanRows>(ea, r0, r0 + kScanRows < ea.R ? r0 + kScanRows : ea.R);
    __syncthreads();
    rowscan_chunk(a);
}

// one lane writes the header of the meta block (format v1) and zeroes the padding after the last array
__device__ inline void write_header(const FinishArgs& a, u64 total)
{
    u32* h32 = (u32*)a.meta;
    u64* h64 = (u64*)a.meta;
    h32[0] = kMagic; h32[1] = kVersion; h32[2] = (u32)a.dt; h32[3] = (u32)a.M;
    h64[2] = (u64)a.R; h64[3] = (u64)a.N; h64[4] = (u64)a.k;
    h32[10] = a.bit_set; h32[11] = (u32)a.w;
    h64[6] = total;
    h32[14] = a.Mn != a.M ? (u32)a.Mn : 0u;        // 0: the negative class has M blocks too
    h32[15] = 0;
    uint8_t* m8 = (uint8_t*)a.meta;
    for (size_t o = kHeaderBytes + 16 * (size_t)a.R + 9 * (size_t)a.R * (a.M + a.Mn); o < meta_bytes(a.R, a.M + a.Mn); ++o) m8[o] = 0;
}

// one wavefront copies words [c * kGatherWords, (c + 1) * kGatherWords) of row r's slot to the stream
__device__ inline void gather_item(const FinishArgs& a, int64_t r, u64 c, u64 off)
{
    const u32 lane = lane_id();
    const u64 nw = a.row_words[r];
    const u64 j0 = c * (u64)kGatherWords;
    if (j0 >= nw) return;
    const u64 j1 = j0 + (u64)kGatherWords < nw ? j0 + (u64)kGatherWords : nw;
    const u32* __restrict__ src = a.slots + (size_t)r * a.cap_words;
    u32* __restrict__ dst = a.stream + off;
    for (u64 j = j0 + lane; j < j1; j += kWave) dst[j] = src[j];
}

__global__ __launch_bounds__(256) void enc_gather_kernel(FinishArgs a)
{
    // one wavefront per (row, kGatherWords-word chunk of its slot); no workgroup barrier
    const u32 lane = lane_id();
    const int64_t n_items = a.R * a.chunks_per_row;
    const int64_t wg = xcd_row((int64_t)blockIdx.x, (n_items + 3) / 4);   // neighbouring rows stay on one XCD
    const int64_t item = wg * (256 / kWave) + threadIdx.x / kWave;
    const int64_t r = item / a.chunks_per_row;
    const u64 c = (u64)(item % a.chunks_per_row);
    if (r >= a.R) return;
    const int64_t my_chunk = r / kScanRows;
    const int64_t n_chunks = (a.R + kScanRows - 1) / kScanRows;
    const bool want_total = item == 0;               // this wave also writes the header
    const int64_t upto = want_total ? n_chunks : my_chunk;
    u64 before = 0, total = 0;
    for (int64_t j = lane; j < upto; j += kWave) {
        const u64 t = a.chunk_tot[j];
        total += t;
        if (j < my_chunk) before += t;
    }
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) { before += __shfl_xor(before, d); total += __shfl_xor(total, d); }

    const u64 off = before + a.row_off_local[r];
    if (c == 0 && lane == 0) a.mv.row_off[r] = off;
    if (want_total && lane == 0) write_header(a, total);
    gather_item(a, r, c, off);
}

// Batches of up to kScanRows rows (one decode step, one feature map, a batch of long rows): repair, row
// offsets, header and gather in ONE launch.  Every workgroup scans the (at most 256) word counts itself and
// copies its share of the slots.  If a fast path flagged any row, which is rare, workgroup 0 alone redoes
// those rows with the generic encoder and then copies every row; the others leave at once.
template <int DT>
__global__ __launch_bounds__(kScanRows) void enc_finish_small_kernel(EncArgs ea, FinishArgs a)
{
    __shared__ u64 s_off[kScanRows + 1];
    __shared__ u64 s_wave[kScanRows / kWave];
    const int tid = threadIdx.x, wid = tid / kWave;
    const u32 lane = lane_id();
    bool alone = false;
    if (ea.only_flagged) {
        const int any = tid < a.R ? (int)ea.only_flagged[tid] : 0;
        if (__syncthreads_or(any)) {
            if (blockIdx.x != 0) return;             // the whole workgroup
            enc_generic_rows<DT, kScanRows>(ea, 0, a.R);
            __syncthreads();
            alone = true;
        }
    }
    {   // exclusive scan of the word counts
        const u64 v = tid < a.R ? a.row_words[tid] : 0ull;
        u64 inc = v;
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
            const u64 t = __shfl_up(inc, d);
            if (lane >= (u32)d) inc += t;
        }
        if (lane == kWave - 1) s_wave[wid] = inc;
        __syncthreads();
        u64 wbase = 0, tot = 0;
        for (int v2 = 0; v2 < kScanRows / kWave; ++v2) {
            const u64 sp = s_wave[v2];
            if (v2 < wid) wbase += sp;
            tot += sp;
        }
        s_off[tid] = wbase + inc - v;
        if (tid == 0) s_off[kScanRows] = tot;
        __syncthreads();
    }
    const int64_t n_items = a.R * a.chunks_per_row;
    const int64_t first = alone ? wid : xcd_row((int64_t)blockIdx.x, (n_items + 3) / 4) * (kScanRows / kWave) + wid;
    const int64_t step = alone ? kScanRows / kWave : n_items;      // (not alone: one item per wavefront)
    for (int64_t item = first; item < n_items; item += step) {
        const int64_t r = item / a.chunks_per_row;
        const u64 c = (u64)(item % a.chunks_per_row);
        const u64 off = s_off[r];
        if (c == 0 && lane == 0) a.mv.row_off[r] = off;
        if (item == 0 && lane == 0) write_header(a, s_off[kScanRows]);
        gather_item(a, r, c, off);
    }
}

}  // namespace slicer
