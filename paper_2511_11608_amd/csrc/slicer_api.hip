// C ABI of the SLICER IF codec for MI355X (see include/slicer.h): argument
// checks, workspace carving and kernel launches.  No device memory is allocated.
#include "../../include/slicer.h"

#include <hip/hip_runtime.h>
#include <algorithm>
#include <cmath>
#include <mutex>

#include "slicer_common.hpp"
#include "slicer_encode_generic.hpp"
#include "slicer_encode_small.hpp"
#include "slicer_encode_wg.hpp"
#include "slicer_encode_large.hpp"
#include "slicer_decode.hpp"
#include "slicer_csr.hpp"

using namespace slicer;

// Scratch of slicer_encode_static: the workspace of an encode call for callers that cannot
// allocate.  Every GPU the library runs on holds its own copy until the process ends.
static __device__ __align__(256) unsigned char scratch[SLICER_STATIC_SCRATCH_BYTES];

namespace {

thread_local int g_last_hip_error = 0;
thread_local hipEvent_t g_ev_start = nullptr, g_ev_stop = nullptr;

inline int hip_fail(hipError_t e)
{
    g_last_hip_error = (int)e;
    return SLICER_EHIP;
}

#define SLICER_HIP(call)                                   \
    do {                                                   \
        hipError_t e_ = (call);                            \
        if (e_ != hipSuccess) return hip_fail(e_);         \
    } while (0)

int check_shape(int dt, int64_t rows, int64_t row_len, int n_blocks)
{
    if (dt != SLICER_F32 && dt != SLICER_BF16) return SLICER_EUNSUPPORTED;
    if (rows <= 0 || row_len <= 0 || row_len >= ((int64_t)1 << 31)) return SLICER_EINVAL;
    if (n_blocks < 1 || n_blocks > SLICER_MAX_BLOCKS) return SLICER_EINVAL;
    return SLICER_OK;
}

int check_args(int dt, int64_t rows, int64_t row_len, double keep_ratio, int n_blocks, uint32_t bit_set)
{
    int rc = check_shape(dt, rows, row_len, n_blocks);
    if (rc) return rc;
    if (!(keep_ratio >= 0.0 && keep_ratio <= 1.0)) return SLICER_EINVAL;
    if (bit_set == 0 || (bit_set & ~0x1FFFEu)) return SLICER_EINVAL;
    return SLICER_OK;
}

int index_bits(int64_t N)
{
    int w = 1;
    while (((int64_t)1 << w) < N) ++w;
    return w;
}

struct Plan {
    int64_t k;
    int w, qmax;
    u64 cap_words;          // per row
    size_t off_row_words, off_slots, off_kept, off_bo_idx, off_bo_val, off_fallback, off_row_local, off_chunk_tot, off_hint, total;
    // row-resident fast path (0 = not eligible)
    int small_epl, small_cap, small_region0, small_lds_bytes, small_maxs;
    // workgroup-per-row path for bf16 rows of up to 32768 elements (0 = not eligible)
    int wg_ept, wg_nw, wg_cap, wg_region0, wg_lds_bytes;
    // long-row path (large_C == 0: not eligible)
    int large_C, large_LC;
    u32 large_capL;
    size_t lo_ch_cum, lo_ch_off, lo_L, lo_Lblk, lo_Lfine, lo_rowst, lo_thr, lo_blk_start,
           lo_blkcnt, lo_vminb, lo_vmaxb, lo_sums, lo_qsel, lo_inv_sel, lo_code_off, lo_win_range;
};

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

int count_bits(int64_t k)      // bits that hold any value in 0..k
{
    int w = 1;
    while (((int64_t)1 << w) <= k) ++w;
    return w;
}

Plan make_plan(int dt, int64_t rows, int64_t row_len, double keep_ratio, int n_blocks, int n_blocks_neg, uint32_t bit_set)
{
    const int B2_all = n_blocks + n_blocks_neg;          // blocks per row
    Plan p;
    p.k = (int64_t)std::floor(keep_ratio * (double)row_len);   // ATKF: k = floor((1-s) N)
    p.w = index_bits(row_len);
    p.qmax = 16;
    while (!((bit_set >> p.qmax) & 1u)) --p.qmax;
    p.cap_words = ((u64)p.k * (u64)(p.w + p.qmax) + 31) / 32;

    size_t o = 0;
    p.off_row_words = o; o = align256(o + 8 * (size_t)rows);
    p.off_slots = o;     o = align256(o + 4 * (size_t)rows * (size_t)p.cap_words);
    p.off_kept = o;      o = align256(o + 8 * (size_t)rows * (size_t)p.k);
    p.off_bo_idx = o;    o = align256(o + 4 * (size_t)rows * (size_t)p.k);
    p.off_bo_val = o;    o = align256(o + 4 * (size_t)rows * (size_t)p.k);
    p.off_fallback = o;  o = align256(o + 4 * (size_t)rows);
    p.off_row_local = o; o = align256(o + 8 * (size_t)rows);
    p.off_chunk_tot = o; o = align256(o + 8 * (size_t)((rows + kScanRows - 1) / kScanRows));
    p.off_hint = o;      o = align256(o + 4 * (size_t)kHintSlots);
    // Long rows: every pass is spread over many workgroups (slicer_encode_large.hpp).
    p.large_C = 0; p.large_LC = 0; p.large_capL = 0;
    {
        const int epc_l = dt == SLICER_F32 ? 4 : 8;
        const int64_t C = (row_len + kLCH - 1) / kLCH;
        const int64_t capL = (p.k + std::max<int64_t>(4096, row_len / 16) + 7) & ~(int64_t)7;   // whole 16-byte groups of 2-byte entries
        int nq_l = 0;
        for (int q = 1; q <= 16; ++q) nq_l += (bit_set >> q) & 1u;
        if (row_len > 4096 && row_len % epc_l == 0 && C <= 1024 && rows <= 65535 && capL < ((int64_t)1 << 27)) {
            const size_t R = (size_t)rows, B2 = (size_t)B2_all;
            p.large_C = (int)C; p.large_capL = (u32)capL; p.large_LC = (int)((capL + kLCE - 1) / kLCE);
            p.lo_ch_cum = o;    o = align256(o + 4 * R * (size_t)C * kLBins);
            p.lo_ch_off = o;    o = align256(o + 4 * R * (size_t)C);
            p.lo_L = o;         o = align256(o + 8 * R * (size_t)capL);
            p.lo_Lblk = o;      o = align256(o + R * (size_t)capL);
            p.lo_Lfine = o;     o = align256(o + 2 * R * (size_t)capL);
            p.lo_rowst = o;     o = align256(o + 4 * R * 16);
            p.lo_thr = o;       o = align256(o + 8 * R * (1 + kMaxB2));
            p.lo_blk_start = o; o = align256(o + 4 * R * (B2 + 1));
            p.lo_blkcnt = o;    o = align256(o + 4 * R * (size_t)p.large_LC * B2);
            p.lo_vminb = o;     o = align256(o + 4 * R * B2);
            p.lo_vmaxb = o;     o = align256(o + 4 * R * B2);
            p.lo_sums = o;      o = align256(o + 8 * R * B2 * (size_t)(nq_l + 1));
            p.lo_qsel = o;      o = align256(o + 4 * R * B2);
            p.lo_inv_sel = o;   o = align256(o + 4 * R * B2);
            p.lo_code_off = o;  o = align256(o + 8 * R * (B2 + 1));
            p.lo_win_range = o; o = align256(o + 8 * R * (size_t)(p.cap_words / 64 + 8));    // pack windows of >= 64 words
        }
    }
    p.total = o ? o : 256;

    // The one-wave-per-row kernel holds the row in registers (64 * EPL elements) and
    // its lists in LDS; it needs whole 16-byte chunks, 16-bit indices, one lane per
    // block and a list capacity below 2048 entries (11-bit rank fields).
    p.small_epl = 0; p.small_cap = 0; p.small_region0 = 0; p.small_lds_bytes = 0; p.small_maxs = 0;
    const int epc = dt == SLICER_F32 ? 4 : 8;
    const int64_t max_n = dt == SLICER_F32 ? 4096 : 8192;
    int nq = 0;
    for (int q = 1; q <= 16; ++q) nq += (bit_set >> q) & 1u;
    if (row_len % epc == 0 && row_len <= max_n && B2_all <= kWave) {
        const int64_t margin = std::max<int64_t>(64, row_len / (dt == SLICER_F32 ? 16 : 32));  // room for the undecided coarse bin
        int64_t cap = std::min<int64_t>(1984, (p.k + margin + 63) / 64 * 64);   // ranks are 11-bit fields
        int epl = epc;
        while ((int64_t)epl * kWave < row_len) epl *= 2;
        // fp32 rows of the common transformer widths 768 and 1280: three and five chunks per lane instead of four and eight
        if (dt == SLICER_F32 && row_len > 512 && row_len <= 768) epl = 12;
        if (dt == SLICER_F32 && row_len > 1024 && row_len <= 1280) epl = 20;
        const int maxs = cap <= 640 ? 10 : cap <= 1280 ? 20 : 0;             // list held in registers
        const int64_t region0 = small_region0_words(p.k, p.cap_words, B2_all, nq);
        const int64_t lds = 4 * (int64_t)small_lds_words(dt, (int)cap, (int)region0, B2_all, maxs);
        if (p.k + 64 <= cap && lds <= 64 * 1024) {
            p.small_epl = epl; p.small_cap = (int)cap; p.small_region0 = (int)region0; p.small_lds_bytes = (int)lds;
            p.small_maxs = maxs;
        }
    }
    // One workgroup per row (the wavefronts of a workgroup share the row): every row of more than 4096 and up to
    // 32768 bf16 / 16384 fp32 elements.  For bf16 rows of 4097..8192 elements, which one wavefront could hold,
    // it is the faster kernel at every batch size (16384 rows of 8192: 238 against 293 us; 4096 rows of 6144:
    // 68 against 74 us); at 4096 elements and below one wavefront per row wins (115 against 189 us).
    p.wg_ept = 0; p.wg_nw = 0; p.wg_cap = 0; p.wg_region0 = 0; p.wg_lds_bytes = 0;
    {
        const int64_t wg_max = dt == SLICER_F32 ? 16384 : 32768;
        if (row_len % epc == 0 && row_len > 4096 && row_len <= wg_max && B2_all <= kWave) {
            const int64_t margin = std::max<int64_t>(64, row_len / (dt == SLICER_F32 ? 16 : 32));
            const int64_t cap = std::min<int64_t>(1984, (p.k + margin + 63) / 64 * 64);
            const int64_t region0 = small_region0_words(p.k, p.cap_words, B2_all, nq);
            const int64_t lds = 4 * (int64_t)wg_lds_words(dt, (int)cap, (int)region0, B2_all);
            if (p.k + 64 <= cap && lds <= 64 * 1024) {
                // wavefronts per row: sixteen for the smallest batches (more wavefronts per SIMD hide each other's
                // latencies: 4 % less latency per call), four otherwise (a 256-row batch on sixteen leaves no room
                // for a neighbouring stream's kernels: 20 % less throughput when steps overlap)
                p.wg_nw = rows <= 128 ? 16 : 4;
                const int64_t chunks = (row_len / epc + 64 * p.wg_nw - 1) / (64 * p.wg_nw);     // 16-byte chunks per thread
                p.wg_ept = (int)(chunks <= 1 ? 1 : chunks <= 2 ? 2 : chunks <= 4 ? 4 : chunks <= 8 ? 8 : 16);    // (kept as a chunk count)
                p.wg_cap = (int)cap; p.wg_region0 = (int)region0; p.wg_lds_bytes = (int)lds;
            }
        }
    }
    return p;
}

// p.wg_ept: 16-byte chunks per thread (1..16; at most 64 chunk totals for the one-wavefront scan: 4 with 16 wavefronts)
template <int DT, int NW, int NQ>
void launch_wg_nw(const SmallArgs& sa, const Plan& p, hipStream_t st)
{
    constexpr int EPC = DT == 0 ? 4 : 8;
    const dim3 g((unsigned)sa.R), b(NW * kWave);
    const size_t lds = (size_t)p.wg_lds_bytes;
    if constexpr (NW == 16) {
        if (p.wg_ept <= 1) hipLaunchKernelGGL((enc_wg_kernel<DT, 16, 1 * EPC, NQ>), g, b, lds, st, sa);
        else if (p.wg_ept == 2) hipLaunchKernelGGL((enc_wg_kernel<DT, 16, 2 * EPC, NQ>), g, b, lds, st, sa);
        else hipLaunchKernelGGL((enc_wg_kernel<DT, 16, 4 * EPC, NQ>), g, b, lds, st, sa);
    } else {
        if (p.wg_ept <= 4) hipLaunchKernelGGL((enc_wg_kernel<DT, 4, 4 * EPC, NQ>), g, b, lds, st, sa);
        else if (p.wg_ept == 8) hipLaunchKernelGGL((enc_wg_kernel<DT, 4, 8 * EPC, NQ>), g, b, lds, st, sa);
        else hipLaunchKernelGGL((enc_wg_kernel<DT, 4, 16 * EPC, NQ>), g, b, lds, st, sa);
    }
}

template <int DT>
int launch_wg(const SmallArgs& sa, const Plan& p, hipStream_t st)
{
    if (p.wg_nw == 16) {
        if (sa.nq == 7) launch_wg_nw<DT, 16, 7>(sa, p, st); else launch_wg_nw<DT, 16, 0>(sa, p, st);
    } else {
        if (sa.nq == 7) launch_wg_nw<DT, 4, 7>(sa, p, st); else launch_wg_nw<DT, 4, 0>(sa, p, st);
    }
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? SLICER_OK : hip_fail(e);
}

template <int DT, int EPL, bool ASYM>
void launch_small_variant(const SmallArgs& sa, dim3 g, dim3 b, size_t lds, int maxs, hipStream_t st)
{
    // the paper's bitwidth ladders are short; 7 = {2..8} is the benchmarked one
    if (sa.nq == 7) {
        if (maxs == 10) hipLaunchKernelGGL((enc_small_kernel<DT, EPL, 7, 10, ASYM>), g, b, lds, st, sa);
        else if (maxs == 20) hipLaunchKernelGGL((enc_small_kernel<DT, EPL, 7, 20, ASYM>), g, b, lds, st, sa);
        else hipLaunchKernelGGL((enc_small_kernel<DT, EPL, 7, 0, ASYM>), g, b, lds, st, sa);
    } else {
        if (maxs == 10) hipLaunchKernelGGL((enc_small_kernel<DT, EPL, 0, 10, ASYM>), g, b, lds, st, sa);
        else if (maxs == 20) hipLaunchKernelGGL((enc_small_kernel<DT, EPL, 0, 20, ASYM>), g, b, lds, st, sa);
        else hipLaunchKernelGGL((enc_small_kernel<DT, EPL, 0, 0, ASYM>), g, b, lds, st, sa);
    }
}

// asym: the asymmetric thresholds of Sec. 3.1 with lambda > 0 (bf16 rows only)
template <int DT, int EPL>
void launch_small_epl(const SmallArgs& sa, int lds_bytes, int maxs, hipStream_t st, bool asym)
{
    const dim3 g((unsigned)xcd_grid(sa.R)), b(kWave);
    const size_t lds = (size_t)lds_bytes;
    if (asym) {
        launch_small_variant<DT, EPL, true>(sa, g, b, lds, maxs, st);
        return;
    }
    launch_small_variant<DT, EPL, false>(sa, g, b, lds, maxs, st);
}

template <int DT>
int launch_small(const SmallArgs& sa, const Plan& p, hipStream_t st, bool asym)
{
    constexpr int E0 = DT == 0 ? 4 : 16;      // smallest instantiated elements-per-lane
    const int lds = p.small_lds_bytes;
    if constexpr (DT == 0) {
        if (p.small_epl == 12 || p.small_epl == 20) {
            if (p.small_epl == 12) launch_small_epl<0, 12>(sa, lds, p.small_maxs, st, asym);
            else launch_small_epl<0, 20>(sa, lds, p.small_maxs, st, asym);
            hipError_t e = hipGetLastError();
            return e == hipSuccess ? SLICER_OK : hip_fail(e);
        }
    }
    if (p.small_epl <= E0) launch_small_epl<DT, E0>(sa, lds, p.small_maxs, st, asym);
    else if (p.small_epl == E0 * 2) launch_small_epl<DT, E0 * 2>(sa, lds, p.small_maxs, st, asym);
    else if (p.small_epl == E0 * 4) launch_small_epl<DT, E0 * 4>(sa, lds, p.small_maxs, st, asym);
    else if (p.small_epl == E0 * 8 || DT != 0) launch_small_epl<DT, E0 * 8>(sa, lds, p.small_maxs, st, asym);
    else launch_small_epl<DT, DT == 0 ? E0 * 16 : E0 * 8>(sa, lds, p.small_maxs, st, asym);   // fp32 rows of 4096
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? SLICER_OK : hip_fail(e);
}

template <int DT>
int launch_large(const LargeArgs& la, const Plan& p, hipStream_t st)
{
    const dim3 gC((unsigned)la.C, (unsigned)la.R), gL((unsigned)la.LC, (unsigned)la.R), gR((unsigned)la.R);
    const dim3 gP((unsigned)std::max<int64_t>(1, (la.k + kPCH - 1) / kPCH), (unsigned)la.R);
    const dim3 gW((unsigned)la.nwin, (unsigned)la.R);
    hipLaunchKernelGGL((lr_hist_kernel<DT>), gC, dim3(256), 0, st, la);
    hipLaunchKernelGGL((lr_select_kernel<DT>), gR, dim3(1024), 0, st, la);
    hipLaunchKernelGGL((lr_compact_kernel<DT>), gC, dim3(256), 0, st, la);
    hipLaunchKernelGGL(lr_bounds_kernel, gR, dim3(1024), 0, st, la);
    hipLaunchKernelGGL(lr_blockcount_kernel, gL, dim3(256), 0, st, la);
    hipLaunchKernelGGL((lr_scatter_kernel<DT>), gL, dim3(256), 0, st, la);
    if (la.nq == 7) hipLaunchKernelGGL((lr_abq_kernel<DT, 7>), gP, dim3(256), 0, st, la);   // {2..8}: the benchmarked set
    else hipLaunchKernelGGL((lr_abq_kernel<DT, 0>), gP, dim3(256), 0, st, la);
    hipLaunchKernelGGL((lr_choose_kernel<DT>), gR, dim3(128), 0, st, la);
    hipLaunchKernelGGL((lr_pack_kernel<DT>), gW, dim3(256), 0, st, la);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? SLICER_OK : hip_fail(e);
}

template <int DT>
int launch_encode(const EncArgs& ea, hipStream_t st)
{
    const bool timed = g_ev_start && g_ev_stop && !ea.only_flagged;
    if (timed) SLICER_HIP(hipEventRecord(g_ev_start, st));
    const unsigned grid = (unsigned)((ea.R + ea.rows_per_wg - 1) / ea.rows_per_wg);
    if (ea.N >= 32768)
        hipLaunchKernelGGL((enc_generic_kernel<DT, 1024>), dim3(grid), dim3(1024), 0, st, ea);
    else
        hipLaunchKernelGGL((enc_generic_kernel<DT, 256>), dim3(grid), dim3(256), 0, st, ea);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e);
    if (timed) SLICER_HIP(hipEventRecord(g_ev_stop, st));
    return SLICER_OK;
}

int launch_decode(const void* stream, const void* meta, void* y, int dt, int64_t rows, int64_t row_len,
                  int n_blocks, int n_blocks_neg, hipStream_t st)
{
    DecArgs da;
    da.stream = (const u32*)stream;
    da.y = y;
    da.R = rows; da.N = row_len; da.M = n_blocks; da.Mn = n_blocks_neg; da.w = index_bits(row_len);
    const int64_t dec_chunk = kDecChunkBytes / (dt == SLICER_F32 ? 4 : 2);
    da.chunks_per_row = (int)((row_len + dec_chunk - 1) / dec_chunk);
    da.mv = meta_view(const_cast<void*>(meta), rows, n_blocks + n_blocks_neg);
    da.total_words = (const u64*)meta + 6;
    // the stream segment of a row at keep ratios up to about 0.2 (longer segments are read from global memory)
    da.stage_words = (int)std::min<int64_t>(1020, (row_len / 16 + 3) / 4 * 4);
    da.xcd_map = (rows >= 32 && da.chunks_per_row > 1) ? 1 : 0;
    const u64 grid = (u64)(da.xcd_map ? xcd_grid(rows) : rows) * (u64)da.chunks_per_row;
    if (grid >= (1ull << 31)) return SLICER_EINVAL;
    const bool timed = g_ev_start && g_ev_stop;
    if (timed) SLICER_HIP(hipEventRecord(g_ev_start, st));
    // short rows: one wavefront per row, the row assembled in LDS (16 KB per wave at most)
    const int64_t row_bytes = row_len * (dt == SLICER_F32 ? 4 : 2);
    if (row_bytes % 16 == 0 && row_bytes <= 16 * 1024 && n_blocks + n_blocks_neg <= kWave && ((uintptr_t)y & 15) == 0) {
        // one wave per workgroup: the LDS of a row (image + stream segment) is the unit of occupancy
        const size_t lds = (size_t)row_bytes + 16 * (size_t)((da.stage_words + 4) / 4);
        if (dt == SLICER_F32)
            hipLaunchKernelGGL((dec_small_kernel<0>), dim3((unsigned)xcd_grid(rows)), dim3(kWave), lds, st, da);
        else
            hipLaunchKernelGGL((dec_small_kernel<1>), dim3((unsigned)xcd_grid(rows)), dim3(kWave), lds, st, da);
    } else if (dt == SLICER_F32)
        hipLaunchKernelGGL((dec_kernel<0, 256>), dim3((unsigned)grid), dim3(256), 0, st, da);
    else
        hipLaunchKernelGGL((dec_kernel<1, 256>), dim3((unsigned)grid), dim3(256), 0, st, da);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e);
    if (timed) SLICER_HIP(hipEventRecord(g_ev_stop, st));
    return SLICER_OK;
}

}  // namespace

extern "C" {

int slicer_sizes_pn(slicer_dtype dt, int64_t rows, int64_t row_len, double keep_ratio, int n_blocks,
                    int n_blocks_neg, uint32_t bit_set, size_t* stream_capacity_bytes, size_t* meta_bytes_out,
                    size_t* workspace_bytes)
{
    int rc = check_args((int)dt, rows, row_len, keep_ratio, n_blocks, bit_set);
    if (rc) return rc;
    if (n_blocks_neg < 1 || n_blocks_neg > SLICER_MAX_BLOCKS) return SLICER_EINVAL;
    Plan p = make_plan((int)dt, rows, row_len, keep_ratio, n_blocks, n_blocks_neg, bit_set);
    if (stream_capacity_bytes) *stream_capacity_bytes = (size_t)(p.cap_words * 4ull * (u64)rows);
    if (meta_bytes_out) *meta_bytes_out = meta_bytes(rows, n_blocks + n_blocks_neg);
    if (workspace_bytes) *workspace_bytes = p.total;
    return SLICER_OK;
}

int slicer_sizes(slicer_dtype dt, int64_t rows, int64_t row_len, double keep_ratio, int n_blocks,
                 uint32_t bit_set, size_t* stream_capacity_bytes, size_t* meta_bytes_out,
                 size_t* workspace_bytes)
{
    return slicer_sizes_pn(dt, rows, row_len, keep_ratio, n_blocks, n_blocks, bit_set, stream_capacity_bytes,
                           meta_bytes_out, workspace_bytes);
}

int slicer_encode_path(slicer_dtype dt, int64_t rows, int64_t row_len, double keep_ratio, int n_blocks,
                       uint32_t bit_set)
{
    int rc = check_args((int)dt, rows, row_len, keep_ratio, n_blocks, bit_set);
    if (rc) return rc;
    Plan p = make_plan((int)dt, rows, row_len, keep_ratio, n_blocks, n_blocks, bit_set);
    return p.wg_ept ? 3 : p.small_epl ? 1 : (p.large_C ? 2 : 0);
}

static int encode_impl(const void* x, slicer_dtype dt, int64_t rows, int64_t row_len, double keep_ratio,
                       int n_blocks, int n_blocks_neg, uint32_t bit_set, double distortion_budget, const Ladder& lad, int guard,
                       void* stream, void* meta, void* workspace, void* hip_stream, double lambda = 0.0)
{
    if (!(lambda >= 0.0 && lambda < 1.0)) return SLICER_EINVAL;
    const bool asym = (float)lambda > 0.0f;      // lambda = 0 is the plain top-K filter: every fast path applies
    int rc = check_args((int)dt, rows, row_len, keep_ratio, n_blocks, bit_set);
    if (rc) return rc;
    if (!x || !stream || !meta || !workspace) return SLICER_EINVAL;
    if (!(distortion_budget >= 0.0)) return SLICER_EINVAL;
    if (rows >= ((int64_t)1 << 31)) return SLICER_EINVAL;
    if (n_blocks_neg < 1 || n_blocks_neg > SLICER_MAX_BLOCKS) return SLICER_EINVAL;
    hipStream_t st = (hipStream_t)hip_stream;
    Plan p = make_plan((int)dt, rows, row_len, keep_ratio, n_blocks, n_blocks_neg, bit_set);
    char* ws = (char*)workspace;

    EncArgs ea;
    ea.x = x;
    ea.R = rows; ea.N = row_len; ea.k = p.k;
    ea.M = n_blocks; ea.Mn = n_blocks_neg; ea.w = p.w;
    ea.nq = 0;
    for (int q = 1; q <= 16; ++q)
        if ((bit_set >> q) & 1u) ea.qlist[ea.nq++] = q;
    for (int t = ea.nq; t < kMaxQ; ++t) ea.qlist[t] = 0;
    ea.beta = distortion_budget;
    ea.cap_words = p.cap_words;
    ea.row_words = (u64*)(ws + p.off_row_words);
    ea.slots = (u32*)(ws + p.off_slots);
    ea.kept = (u64*)(ws + p.off_kept);
    ea.bo_idx = (u32*)(ws + p.off_bo_idx);
    ea.bo_val = (u32*)(ws + p.off_bo_val);
    ea.mv = meta_view(meta, rows, n_blocks + n_blocks_neg);
    ea.only_flagged = nullptr;
    ea.rows_per_wg = 1;
    ea.lad = lad;
    ea.guard = guard;
    ea.asym = asym ? 1 : 0;
    ea.one_plus = 1.0f + (float)lambda;
    ea.one_minus = 1.0f - (float)lambda;

    // asymmetric thresholds need a second selection over a subset of the row: the generic kernel has it for
    // every shape, the row-resident kernel for bf16 rows (rows it flags are redone generically, same rule)
    const bool use_wg = p.wg_ept && !asym && ((uintptr_t)x & 15) == 0;
    if (use_wg) {
        // one workgroup per row; rows it cannot hold are flagged and redone by the generic kernel
        SmallArgs sa;
        sa.x = x; sa.R = rows; sa.N = row_len; sa.k = p.k;
        sa.M = n_blocks; sa.Mn = n_blocks_neg; sa.w = p.w; sa.nq = ea.nq;
        for (int t = 0; t < kMaxQ; ++t) sa.qlist[t] = ea.qlist[t];
        sa.beta = distortion_budget;
        sa.cap_words = p.cap_words;
        sa.row_words = ea.row_words; sa.slots = ea.slots;
        sa.fallback = (u32*)(ws + p.off_fallback);
        sa.mv = ea.mv;
        sa.cap = p.wg_cap; sa.region0_words = p.wg_region0;
        sa.lad = lad;
        sa.guard = guard;
        sa.one_plus = ea.one_plus; sa.one_minus = ea.one_minus;
        sa.hint = (u32*)(ws + p.off_hint);
        const bool timed = g_ev_start && g_ev_stop;
        if (timed) SLICER_HIP(hipEventRecord(g_ev_start, st));
        rc = dt == SLICER_F32 ? launch_wg<0>(sa, p, st) : launch_wg<1>(sa, p, st);
        if (rc) return rc;
        if (timed) SLICER_HIP(hipEventRecord(g_ev_stop, st));
        ea.only_flagged = sa.fallback;
    }
    if (!use_wg && p.small_epl && ((uintptr_t)x & 15) == 0) {
        // fast path; rows it cannot hold are flagged and redone by the generic kernel
        SmallArgs sa;
        sa.x = x; sa.R = rows; sa.N = row_len; sa.k = p.k;
        sa.M = n_blocks; sa.Mn = n_blocks_neg; sa.w = p.w; sa.nq = ea.nq;
        for (int t = 0; t < kMaxQ; ++t) sa.qlist[t] = ea.qlist[t];
        sa.beta = distortion_budget;
        sa.cap_words = p.cap_words;
        sa.row_words = ea.row_words; sa.slots = ea.slots;
        sa.fallback = (u32*)(ws + p.off_fallback);
        sa.mv = ea.mv;
        sa.cap = p.small_cap; sa.region0_words = p.small_region0;
        sa.lad = lad;
        sa.guard = guard;
        sa.one_plus = ea.one_plus; sa.one_minus = ea.one_minus;
        sa.hint = (u32*)(ws + p.off_hint);
        const bool timed = g_ev_start && g_ev_stop;
        if (timed) SLICER_HIP(hipEventRecord(g_ev_start, st));
        rc = dt == SLICER_F32 ? launch_small<0>(sa, p, st, asym) : launch_small<1>(sa, p, st, asym);
        if (rc) return rc;
        if (timed) SLICER_HIP(hipEventRecord(g_ev_stop, st));
        ea.only_flagged = sa.fallback;
    }
    if (!asym && !ea.only_flagged && p.large_C && ((uintptr_t)x & 15) == 0) {
        // long rows: multi-workgroup stages; rows they cannot hold are flagged for the generic kernel
        LargeArgs la;
        la.x = x; la.R = rows; la.N = row_len; la.k = p.k;
        la.M = n_blocks; la.Mn = n_blocks_neg; la.w = p.w; la.nq = ea.nq;
        for (int t = 0; t < kMaxQ; ++t) la.qlist[t] = ea.qlist[t];
        la.beta = distortion_budget; la.cap_words = p.cap_words;
        la.C = p.large_C; la.LC = p.large_LC; la.capL = p.large_capL;
        // pack windows: index fields are w bits, code fields as short as one bit, so the windows
        // from the first code bit on are a quarter of the others; all are smaller while the launch is small
        la.pack_words = kPackWords;
        while (la.pack_words > 128 && (u64)rows * ((p.cap_words + (u64)la.pack_words - 1) / (u64)la.pack_words) < 1024) la.pack_words /= 2;
        la.pack_words_code = std::max(64, la.pack_words / 4);
        {
            const u64 idx_words_max = ((u64)p.k * (u64)p.w) / 32;                              // largest first word with code bits
            la.nwin_idx = (int)((idx_words_max + (u64)la.pack_words - 1) / (u64)la.pack_words);
            const u64 code_words_max = ((u64)p.k * (u64)p.qmax + 31) / 32 + 2;                  // words from there to the end
            la.nwin = la.nwin_idx + (int)((code_words_max + (u64)la.pack_words_code - 1) / (u64)la.pack_words_code);
        }
        la.win_range = (u32*)(ws + p.lo_win_range);
        la.ch_cum = (u32*)(ws + p.lo_ch_cum);     la.ch_off = (u32*)(ws + p.lo_ch_off);
        la.L = (u64*)(ws + p.lo_L);               la.Lblk = (uint8_t*)(ws + p.lo_Lblk);
        la.Lfine = (uint16_t*)(ws + p.lo_Lfine);
        la.rowst = (u32*)(ws + p.lo_rowst);       la.thr = (u64*)(ws + p.lo_thr);
        la.blk_start = (u32*)(ws + p.lo_blk_start); la.blkcnt = (u32*)(ws + p.lo_blkcnt);
        la.vminb = (u32*)(ws + p.lo_vminb);       la.vmaxb = (u32*)(ws + p.lo_vmaxb);
        la.sums = (u64*)(ws + p.lo_sums);         la.qsel = (u32*)(ws + p.lo_qsel);
        la.inv_sel = (float*)(ws + p.lo_inv_sel); la.code_off = (u64*)(ws + p.lo_code_off);
        la.bo_idx = ea.bo_idx; la.bo_val = ea.bo_val;
        la.row_words = ea.row_words; la.slots = ea.slots;
        la.fallback = (u32*)(ws + p.off_fallback);
        la.mv = ea.mv;
        la.lad = lad;
        la.guard = guard;
        const bool timed = g_ev_start && g_ev_stop;
        if (timed) SLICER_HIP(hipEventRecord(g_ev_start, st));
        rc = dt == SLICER_F32 ? launch_large<0>(la, p, st) : launch_large<1>(la, p, st);
        if (rc) return rc;
        if (timed) SLICER_HIP(hipEventRecord(g_ev_stop, st));
        ea.only_flagged = la.fallback;
        ea.rows_per_wg = 1;
    }
    if (!ea.only_flagged) {
        rc = dt == SLICER_F32 ? launch_encode<0>(ea, st) : launch_encode<1>(ea, st);
        if (rc) return rc;
    }

    FinishArgs fa;
    fa.R = rows; fa.N = row_len; fa.k = p.k;
    fa.M = n_blocks; fa.Mn = n_blocks_neg; fa.w = p.w; fa.dt = (int)dt;
    fa.bit_set = bit_set;
    fa.row_words = ea.row_words;
    fa.row_off_local = (u64*)(ws + p.off_row_local);
    fa.chunk_tot = (u64*)(ws + p.off_chunk_tot);
    fa.slots = ea.slots;
    fa.cap_words = p.cap_words;
    fa.chunks_per_row = (int)std::max<u64>(1, (p.cap_words + kGatherWords - 1) / kGatherWords);
    fa.stream = (u32*)stream;
    fa.meta = meta;
    fa.mv = ea.mv;
    const u64 grid = (u64)xcd_grid((int64_t)(((u64)rows * (u64)fa.chunks_per_row + 3) / 4));     // four wavefronts per workgroup
    if (grid >= (1ull << 31)) return SLICER_EINVAL;
    if (rows <= kScanRows) {        // small batches: repair, offsets, header and gather in one launch
        if (dt == SLICER_F32) hipLaunchKernelGGL((enc_finish_small_kernel<0>), dim3((unsigned)grid), dim3(kScanRows), 0, st, ea, fa);
        else hipLaunchKernelGGL((enc_finish_small_kernel<1>), dim3((unsigned)grid), dim3(kScanRows), 0, st, ea, fa);
        hipError_t e1 = hipGetLastError();
        return e1 == hipSuccess ? SLICER_OK : hip_fail(e1);
    }
    const dim3 gscan((unsigned)((rows + kScanRows - 1) / kScanRows));
    if (!ea.only_flagged)
        hipLaunchKernelGGL(enc_rowscan_kernel, gscan, dim3(kScanRows), 0, st, fa);
    else if (dt == SLICER_F32)      // rows a fast path flagged are redone here, just before the scan of their chunk
        hipLaunchKernelGGL((enc_fix_rowscan_kernel<0>), gscan, dim3(kScanRows), 0, st, ea, fa);
    else
        hipLaunchKernelGGL((enc_fix_rowscan_kernel<1>), gscan, dim3(kScanRows), 0, st, ea, fa);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e);
    hipLaunchKernelGGL(enc_gather_kernel, dim3((unsigned)grid), dim3(256), 0, st, fa);
    e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e);
    return SLICER_OK;
}

int slicer_encode(const void* x, slicer_dtype dt, int64_t rows, int64_t row_len, double keep_ratio,
                  int n_blocks, uint32_t bit_set, double distortion_budget, void* stream, void* meta,
                  void* workspace, void* hip_stream)
{
    Ladder none;
    none.on = 0;
    for (int j = 0; j < kMaxBlocks / 8; ++j) none.nib[j] = 0;
    return encode_impl(x, dt, rows, row_len, keep_ratio, n_blocks, n_blocks, bit_set, distortion_budget, none, 0,
                       stream, meta, workspace, hip_stream);
}

// Address of this device's copy of `scratch`, looked up once per device.  The array's name is a
// host-side stand-in: only the pointer hipGetSymbolAddress returns is usable as a kernel argument.
static int static_scratch(void** out)
{
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void* ptr[kMaxDevices] = {};
    int dev = 0;
    SLICER_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return SLICER_EINVAL;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void* p = nullptr;
        SLICER_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return SLICER_EHIP;
        ptr[dev] = p;
    }
    *out = ptr[dev];
    return SLICER_OK;
}

int slicer_encode_static(const void* x, slicer_dtype dt, int64_t rows, int64_t row_len, double keep_ratio,
                         int n_blocks, uint32_t bit_set, double distortion_budget, void* stream, void* meta,
                         void* hip_stream)
{
    int rc = check_args((int)dt, rows, row_len, keep_ratio, n_blocks, bit_set);
    if (rc) return rc;
    const Plan p = make_plan((int)dt, rows, row_len, keep_ratio, n_blocks, n_blocks, bit_set);
    if (p.total > (size_t)SLICER_STATIC_SCRATCH_BYTES) return SLICER_ETOOBIG;
    if (!x || !stream || !meta) return SLICER_EINVAL;
    void* ws = nullptr;
    rc = static_scratch(&ws);
    if (rc) return rc;
    Ladder none;
    none.on = 0;
    for (int j = 0; j < kMaxBlocks / 8; ++j) none.nib[j] = 0;
    return encode_impl(x, dt, rows, row_len, keep_ratio, n_blocks, n_blocks, bit_set, distortion_budget, none, 0,
                       stream, meta, ws, hip_stream);
}

int slicer_encode_pn(const void* x, slicer_dtype dt, int64_t rows, int64_t row_len, double keep_ratio,
                     int n_blocks, int n_blocks_neg, uint32_t bit_set, double distortion_budget, void* stream,
                     void* meta, void* workspace, void* hip_stream)
{
    Ladder none;
    none.on = 0;
    for (int j = 0; j < kMaxBlocks / 8; ++j) none.nib[j] = 0;
    return encode_impl(x, dt, rows, row_len, keep_ratio, n_blocks, n_blocks_neg, bit_set, distortion_budget, none, 0,
                       stream, meta, workspace, hip_stream);
}

static int check_csr_shape(int64_t n_rows, int64_t n_cols)
{
    if (n_rows <= 0 || n_cols <= 0 || n_cols >= ((int64_t)1 << 31) || n_rows > (((int64_t)1 << 31) - 1) / n_cols) return SLICER_EINVAL;
    return SLICER_OK;
}

// Two-dimensional instances: the flat encode (any kernel family) writes its stream into the workspace, the
// repack kernels turn it into the CSR form.  Workspace: the flat plan's, then the flat stream, then its offsets.
struct CsrPlan {
    Plan flat;
    int wc, wp;
    u64 cap_words;          // per instance, CSR form
    size_t off_tmp, off_flat_off, total;
};

static CsrPlan make_csr_plan(int dt, int64_t instances, int64_t n_rows, int64_t n_cols, double keep_ratio, int n_blocks,
                             uint32_t bit_set)
{
    CsrPlan c;
    c.flat = make_plan(dt, instances, n_rows * n_cols, keep_ratio, n_blocks, n_blocks, bit_set);
    c.wc = index_bits(n_cols); c.wp = count_bits(c.flat.k);
    c.cap_words = ((u64)(2 * n_blocks) * (u64)(n_rows + 1) * (u64)c.wp + (u64)c.flat.k * (u64)(c.wc + c.flat.qmax) + 31) / 32;
    size_t o = align256(c.flat.total);
    c.off_tmp = o;      o = align256(o + 4 * (size_t)instances * (size_t)c.flat.cap_words + 8);   // (+ one readable word)
    c.off_flat_off = o; o = align256(o + 8 * (size_t)instances);
    c.total = o;
    return c;
}

int slicer_sizes_csr(slicer_dtype dt, int64_t instances, int64_t n_rows, int64_t n_cols, double keep_ratio, int n_blocks,
                     uint32_t bit_set, size_t* stream_capacity_bytes, size_t* meta_bytes_out, size_t* workspace_bytes)
{
    int rc = check_csr_shape(n_rows, n_cols);
    if (rc) return rc;
    rc = check_args((int)dt, instances, n_rows * n_cols, keep_ratio, n_blocks, bit_set);
    if (rc) return rc;
    const CsrPlan c = make_csr_plan((int)dt, instances, n_rows, n_cols, keep_ratio, n_blocks, bit_set);
    if (stream_capacity_bytes) *stream_capacity_bytes = (size_t)(c.cap_words * 4ull * (u64)instances);
    if (meta_bytes_out) *meta_bytes_out = meta_bytes(instances, 2 * n_blocks);
    if (workspace_bytes) *workspace_bytes = c.total;
    return SLICER_OK;
}

int slicer_encode_csr(const void* x, slicer_dtype dt, int64_t instances, int64_t n_rows, int64_t n_cols, double keep_ratio,
                      int n_blocks, uint32_t bit_set, double distortion_budget, void* stream, void* meta, void* workspace,
                      void* hip_stream)
{
    int rc = check_csr_shape(n_rows, n_cols);
    if (rc) return rc;
    rc = check_args((int)dt, instances, n_rows * n_cols, keep_ratio, n_blocks, bit_set);
    if (rc) return rc;
    if (!x || !stream || !meta || !workspace) return SLICER_EINVAL;
    const CsrPlan c = make_csr_plan((int)dt, instances, n_rows, n_cols, keep_ratio, n_blocks, bit_set);
    const u64 nwin = std::max<u64>(1, (c.cap_words + kCsrWin - 1) / kCsrWin);
    if ((u64)instances * nwin >= (1ull << 31)) return SLICER_EINVAL;
    char* ws = (char*)workspace;
    hipStream_t st = (hipStream_t)hip_stream;
    Ladder none;
    none.on = 0;
    for (int j = 0; j < kMaxBlocks / 8; ++j) none.nib[j] = 0;
    // flat encode: kept set, blocks, ranges, bitwidths, codes, flat indices (its stream goes to the workspace)
    rc = encode_impl(x, dt, instances, n_rows * n_cols, keep_ratio, n_blocks, n_blocks, bit_set, distortion_budget, none, 0,
                     ws + c.off_tmp, meta, workspace, hip_stream);
    if (rc) return rc;
    CsrArgs ca;
    ca.R = instances; ca.n_rows = n_rows; ca.n_cols = n_cols; ca.k = c.flat.k;
    ca.M = n_blocks; ca.Mn = n_blocks; ca.w = c.flat.w; ca.wc = c.wc; ca.wp = c.wp; ca.dt = (int)dt;
    ca.bit_set = bit_set;
    ca.nwin = (int)nwin;
    ca.flat = (const u32*)(ws + c.off_tmp);
    ca.flat_off = (u64*)(ws + c.off_flat_off);
    ca.row_words = (u64*)(ws + c.flat.off_row_words);
    ca.row_off_local = (const u64*)(ws + c.flat.off_row_local);
    ca.chunk_tot = (const u64*)(ws + c.flat.off_chunk_tot);
    ca.stream = (u32*)stream; ca.meta = meta;
    ca.mv = meta_view(meta, instances, 2 * n_blocks);
    hipLaunchKernelGGL(csr_sizes_kernel, dim3((unsigned)((instances + 255) / 256)), dim3(256), 0, st, ca);
    FinishArgs fa;                                           // the row-offset scan, now over the CSR segment lengths
    fa.R = instances; fa.N = n_rows * n_cols; fa.k = c.flat.k;
    fa.M = n_blocks; fa.Mn = n_blocks; fa.w = c.flat.w; fa.dt = (int)dt; fa.bit_set = bit_set;
    fa.row_words = ca.row_words;
    fa.row_off_local = (u64*)(ws + c.flat.off_row_local);
    fa.chunk_tot = (u64*)(ws + c.flat.off_chunk_tot);
    fa.slots = nullptr; fa.cap_words = c.cap_words; fa.chunks_per_row = 1;
    fa.stream = (u32*)stream; fa.meta = meta; fa.mv = ca.mv;
    hipLaunchKernelGGL(enc_rowscan_kernel, dim3((unsigned)((instances + kScanRows - 1) / kScanRows)), dim3(kScanRows), 0, st, fa);
    hipLaunchKernelGGL(csr_repack_kernel, dim3((unsigned)((u64)instances * nwin)), dim3(256), 0, st, ca);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? SLICER_OK : hip_fail(e);
}

static int launch_decode_csr(const void* stream, const void* meta, void* y, int dt, int64_t instances, int64_t n_rows,
                             int64_t n_cols, int n_blocks, int n_blocks_neg, hipStream_t st)
{
    DecCsrArgs da;
    da.stream = (const u32*)stream; da.y = y;
    da.R = instances; da.n_rows = n_rows; da.n_cols = n_cols;
    da.M = n_blocks; da.Mn = n_blocks_neg; da.wc = index_bits(n_cols);
    da.mv = meta_view(const_cast<void*>(meta), instances, n_blocks + n_blocks_neg);
    da.k_keep = (const u64*)meta + 4;
    // several short tensor rows per workgroup, as long as about a thousand workgroups remain
    da.rows_per_wg = (int)std::max<int64_t>(1, std::min<int64_t>(std::min<int64_t>(kCsrRows, instances * n_rows / 1024), kCsrImage / n_cols));
    da.groups = (n_rows + da.rows_per_wg - 1) / da.rows_per_wg;
    const u64 grid = (u64)instances * (u64)da.groups;
    if (grid >= (1ull << 31)) return SLICER_EINVAL;
    const bool timed = g_ev_start && g_ev_stop;
    if (timed) SLICER_HIP(hipEventRecord(g_ev_start, st));
    if (dt == SLICER_F32) hipLaunchKernelGGL((dec_csr_kernel<0>), dim3((unsigned)grid), dim3(256), 0, st, da);
    else hipLaunchKernelGGL((dec_csr_kernel<1>), dim3((unsigned)grid), dim3(256), 0, st, da);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e);
    if (timed) SLICER_HIP(hipEventRecord(g_ev_stop, st));
    return SLICER_OK;
}

int slicer_decode_as_csr(const void* stream, const void* meta, void* y, slicer_dtype dt, int64_t instances, int64_t n_rows,
                         int64_t n_cols, int n_blocks, void* hip_stream)
{
    int rc = check_csr_shape(n_rows, n_cols);
    if (rc) return rc;
    rc = check_shape((int)dt, instances, n_rows * n_cols, n_blocks);
    if (rc) return rc;
    if (!stream || !meta || !y) return SLICER_EINVAL;
    return launch_decode_csr(stream, meta, y, (int)dt, instances, n_rows, n_cols, n_blocks, n_blocks, (hipStream_t)hip_stream);
}

int slicer_encode_atkf(const void* x, slicer_dtype dt, int64_t rows, int64_t row_len, double keep_ratio, double lambda,
                       int n_blocks, int n_blocks_neg, uint32_t bit_set, double distortion_budget, void* stream,
                       void* meta, void* workspace, void* hip_stream)
{
    Ladder none;
    none.on = 0;
    for (int j = 0; j < kMaxBlocks / 8; ++j) none.nib[j] = 0;
    return encode_impl(x, dt, rows, row_len, keep_ratio, n_blocks, n_blocks_neg, bit_set, distortion_budget, none, 0,
                       stream, meta, workspace, hip_stream, lambda);
}

int slicer_encode_ds(const void* x, slicer_dtype dt, int64_t rows, int64_t row_len, double keep_ratio,
                     int n_blocks, uint32_t bit_set, double delta, void* stream, void* meta, void* workspace,
                     void* hip_stream)
{
    Ladder none;
    none.on = 0;
    for (int j = 0; j < kMaxBlocks / 8; ++j) none.nib[j] = 0;
    return encode_impl(x, dt, rows, row_len, keep_ratio, n_blocks, n_blocks, bit_set, delta, none, 1,
                       stream, meta, workspace, hip_stream);
}

uint32_t slicer_ladder_bit_set(const uint8_t* ladder, int n_blocks)
{
    if (!ladder || n_blocks < 1 || n_blocks > kMaxBlocks) return 0;
    uint32_t bs = 0;
    for (int m = 0; m < n_blocks; ++m) {
        if (ladder[m] < 1 || ladder[m] > 16) return 0;
        bs |= 1u << ladder[m];
    }
    return bs;
}

int slicer_encode_ladder(const void* x, slicer_dtype dt, int64_t rows, int64_t row_len, double keep_ratio,
                         int n_blocks, const uint8_t* ladder, void* stream, void* meta, void* workspace,
                         void* hip_stream)
{
    const uint32_t bit_set = slicer_ladder_bit_set(ladder, n_blocks);
    if (!bit_set) return SLICER_EINVAL;
    Ladder lad;
    lad.on = 1;
    for (int j = 0; j < kMaxBlocks / 8; ++j) lad.nib[j] = 0;
    for (int m = 0; m < n_blocks; ++m) {
        uint32_t t = 0;                                  // position of ladder[m] among the set's bitwidths, ascending
        for (int q = 1; q < ladder[m]; ++q) t += (bit_set >> q) & 1u;
        lad.nib[m >> 3] |= t << ((m & 7) * 4);
    }
    return encode_impl(x, dt, rows, row_len, keep_ratio, n_blocks, n_blocks, bit_set, 0.0, lad, 0, stream, meta, workspace,
                       hip_stream);
}

int slicer_bound(slicer_dtype dt, int64_t rows, int64_t row_len, double keep_ratio, int n_blocks,
                 uint32_t bit_set, uint64_t* value_bits, uint64_t* index_bits_out, uint64_t* header_bits)
{
    int rc = check_args((int)dt, rows, row_len, keep_ratio, n_blocks, bit_set);
    if (rc) return rc;
    const Plan p = make_plan((int)dt, rows, row_len, keep_ratio, n_blocks, n_blocks, bit_set);
    const u64 R = (u64)rows, k = (u64)p.k;
    if (value_bits) *value_bits = R * k * (u64)p.qmax;
    if (index_bits_out) *index_bits_out = R * k * (u64)p.w;
    if (header_bits) *header_bits = 8ull * (u64)meta_bytes(rows, 2 * n_blocks) + R * (32ull * p.cap_words - k * (u64)(p.w + p.qmax));
    return SLICER_OK;
}

int slicer_decode_as_pn(const void* stream, const void* meta, void* y, slicer_dtype dt, int64_t rows,
                        int64_t row_len, int n_blocks, int n_blocks_neg, void* hip_stream)
{
    int rc = check_shape((int)dt, rows, row_len, n_blocks);
    if (rc) return rc;
    if (n_blocks_neg < 1 || n_blocks_neg > SLICER_MAX_BLOCKS) return SLICER_EINVAL;
    if (!stream || !meta || !y) return SLICER_EINVAL;
    return launch_decode(stream, meta, y, (int)dt, rows, row_len, n_blocks, n_blocks_neg, (hipStream_t)hip_stream);
}

int slicer_decode_as(const void* stream, const void* meta, void* y, slicer_dtype dt, int64_t rows,
                     int64_t row_len, int n_blocks, void* hip_stream)
{
    return slicer_decode_as_pn(stream, meta, y, dt, rows, row_len, n_blocks, n_blocks, hip_stream);
}

static int read_header(const void* meta, hipStream_t st, uint32_t* h32)
{
    SLICER_HIP(hipMemcpyAsync(h32, meta, kHeaderBytes, hipMemcpyDeviceToHost, st));
    SLICER_HIP(hipStreamSynchronize(st));
    if (h32[0] != kMagic || h32[1] != kVersion) return SLICER_EFORMAT;
    return SLICER_OK;
}

int slicer_decode(const void* stream, const void* meta, void* y, void* hip_stream)
{
    if (!stream || !meta || !y) return SLICER_EINVAL;
    hipStream_t st = (hipStream_t)hip_stream;
    alignas(8) uint32_t h32[kHeaderBytes / 4];
    int rc = read_header(meta, st, h32);
    if (rc) return rc;
    const uint64_t* h64 = (const uint64_t*)h32;
    const int dt = (int)h32[2], M = (int)h32[3];
    const int64_t rows = (int64_t)h64[2], row_len = (int64_t)h64[3];
    const int Mn = h32[14] ? (int)h32[14] : M;           // 0: the negative class has M blocks too
    rc = check_shape(dt, rows, row_len, M);
    if (rc || Mn < 1 || Mn > SLICER_MAX_BLOCKS) return SLICER_EFORMAT;
    if (h32[15]) {                                        // two-dimensional instances: blocks stored as CSR triples
        const int64_t n_cols = (int64_t)h32[15];
        if (row_len % n_cols || (int)h32[11] != index_bits(n_cols)) return SLICER_EFORMAT;
        return launch_decode_csr(stream, meta, y, dt, rows, row_len / n_cols, n_cols, M, Mn, st);
    }
    if ((int)h32[11] != index_bits(row_len)) return SLICER_EFORMAT;
    return launch_decode(stream, meta, y, dt, rows, row_len, M, Mn, st);
}

int slicer_stream_words(const void* meta, uint64_t* words, void* hip_stream)
{
    if (!meta || !words) return SLICER_EINVAL;
    alignas(8) uint32_t h32[kHeaderBytes / 4];
    int rc = read_header(meta, (hipStream_t)hip_stream, h32);
    if (rc) return rc;
    *words = ((const uint64_t*)h32)[6];
    return SLICER_OK;
}

int slicer_check(const void* meta, uint64_t stream_words, slicer_dtype dt, int64_t rows, int64_t row_len,
                 int n_blocks, void* scratch, void* hip_stream)
{
    return slicer_check_pn(meta, stream_words, dt, rows, row_len, n_blocks, n_blocks, scratch, hip_stream);
}

static int check_impl(const void* meta, uint64_t stream_words, slicer_dtype dt, int64_t rows, int64_t row_len,
                      int n_blocks, int n_blocks_neg, int64_t csr_cols, void* scratch, void* hip_stream);

int slicer_check_pn(const void* meta, uint64_t stream_words, slicer_dtype dt, int64_t rows, int64_t row_len,
                    int n_blocks, int n_blocks_neg, void* scratch, void* hip_stream)
{
    return check_impl(meta, stream_words, dt, rows, row_len, n_blocks, n_blocks_neg, 0, scratch, hip_stream);
}

int slicer_check_csr(const void* meta, uint64_t stream_words, slicer_dtype dt, int64_t instances, int64_t n_rows,
                     int64_t n_cols, int n_blocks, void* scratch, void* hip_stream)
{
    int rc = check_csr_shape(n_rows, n_cols);
    if (rc) return rc;
    return check_impl(meta, stream_words, dt, instances, n_rows * n_cols, n_blocks, n_blocks, n_cols, scratch, hip_stream);
}

static int check_impl(const void* meta, uint64_t stream_words, slicer_dtype dt, int64_t rows, int64_t row_len,
                      int n_blocks, int n_blocks_neg, int64_t csr_cols, void* scratch, void* hip_stream)
{
    int rc = check_shape((int)dt, rows, row_len, n_blocks);
    if (rc) return rc;
    if (n_blocks_neg < 1 || n_blocks_neg > SLICER_MAX_BLOCKS) return SLICER_EINVAL;
    if (!meta || !scratch) return SLICER_EINVAL;
    hipStream_t st = (hipStream_t)hip_stream;
    CheckArgs ca;
    ca.meta = meta; ca.R = rows; ca.N = row_len; ca.M = n_blocks; ca.Mn = n_blocks_neg; ca.dt = (int)dt;
    ca.csr_cols = csr_cols;
    ca.w = csr_cols > 0 ? index_bits(csr_cols) : index_bits(row_len);
    ca.avail_words = stream_words;
    ca.flag = (u32*)scratch;
    hipLaunchKernelGGL(meta_flag_clear_kernel, dim3(1), dim3(64), 0, st, ca.flag);
    hipLaunchKernelGGL(meta_check_kernel, dim3((unsigned)((rows + 255) / 256)), dim3(256), 0, st, ca);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e);
    u32 flag = 0;
    SLICER_HIP(hipMemcpyAsync(&flag, scratch, 4, hipMemcpyDeviceToHost, st));
    SLICER_HIP(hipStreamSynchronize(st));
    return flag ? SLICER_EFORMAT : SLICER_OK;
}

int slicer_profile_events(void* start_event, void* stop_event)
{
    if ((start_event == nullptr) != (stop_event == nullptr)) return SLICER_EINVAL;
    g_ev_start = (hipEvent_t)start_event;
    g_ev_stop = (hipEvent_t)stop_event;
    return SLICER_OK;
}

int slicer_last_hip_error(void) { return g_last_hip_error; }

const char* slicer_strerror(int code)
{
    switch (code) {
        case SLICER_OK: return "ok";
        case SLICER_EINVAL: return "invalid argument";
        case SLICER_EUNSUPPORTED: return "unsupported dtype";
        case SLICER_EHIP: return "HIP call failed (see slicer_last_hip_error)";
        case SLICER_EFORMAT: return "meta header is not a version-1 SLICER header";
        case SLICER_ETOOBIG: return "shape needs more scratch than the library's static buffer holds";
        default: return "unknown error";
    }
}

}  // extern "C"
