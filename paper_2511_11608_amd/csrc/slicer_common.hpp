// Device-side helpers shared by the encode and decode kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace slicer {

typedef unsigned long long u64;
typedef uint32_t u32;

constexpr int kWave = 64;
constexpr u32 kMagic = 0x52434C53u;
constexpr u32 kVersion = 1u;
constexpr int kHeaderBytes = 64;
constexpr int kMaxBlocks = 64;          // per sign class
constexpr int kMaxB2 = 2 * kMaxBlocks;  // blocks per row
constexpr int kMaxQ = 16;

// ---- meta layout ---------------------------------------------------------

struct MetaView {
    u64* row_off;
    u32* n_pos;
    u32* n_neg;
    float* vmin;
    float* vmax;
    uint8_t* q;
};

// B2 = blocks per row = M(+) + M(-)
__host__ __device__ inline size_t meta_bytes(int64_t R, int B2)
{
    size_t s = kHeaderBytes + 16 * (size_t)R + 9 * (size_t)R * (size_t)B2;
    return (s + 7) & ~(size_t)7;
}

__host__ __device__ inline MetaView meta_view(void* meta, int64_t R, int B2)
{
    uint8_t* p = (uint8_t*)meta + kHeaderBytes;
    MetaView v;
    v.row_off = (u64*)p;              p += 8 * (size_t)R;
    v.n_pos = (u32*)p;                p += 4 * (size_t)R;
    v.n_neg = (u32*)p;                p += 4 * (size_t)R;
    v.vmin = (float*)p;               p += 4 * (size_t)R * B2;
    v.vmax = (float*)p;               p += 4 * (size_t)R * B2;
    v.q = p;
    return v;
}

// ---- fixed multi-level mode (Sec. 4.1: Q = [q_1 > ... > q_M]) --------------------------------
// Block m of either sign class takes the bitwidth qlist[index(m)]; four bits per block.
struct Ladder {
    int on;
    u32 nib[kMaxBlocks / 8];
};

__host__ __device__ inline u32 ladder_index(const Ladder& l, int m)
{
    u32 wsel = l.nib[0];
#pragma unroll
    for (int j = 1; j < kMaxBlocks / 8; ++j) wsel = (m >> 3) == j ? l.nib[j] : wsel;   // no indexed access to kernel arguments
    return (wsel >> ((m & 7) * 4)) & 15u;
}

// ---- element types ---------------------------------------------------------
// Magnitude key: the bit pattern with the sign cleared orders finite values by
// |x| (ATKF, Sec. 3.1).  bf16 keys are kept as 15-bit integers.

template <int DT> struct Elem;

template <> struct Elem<0> {  // fp32
    typedef u32 raw_t;
    static constexpr int kKeyBits = 31;
    __device__ static inline u32 key(raw_t r) { return r & 0x7FFFFFFFu; }
    __device__ static inline u32 neg(raw_t r) { return r >> 31; }
    __device__ static inline u32 value_bits(u32 key) { return key; }  // |x| as fp32 bits
};

template <> struct Elem<1> {  // bf16
    typedef uint16_t raw_t;
    static constexpr int kKeyBits = 15;
    __device__ static inline u32 key(raw_t r) { return (u32)r & 0x7FFFu; }
    __device__ static inline u32 neg(raw_t r) { return (u32)r >> 15; }
    __device__ static inline u32 value_bits(u32 key) { return key << 16; }  // exact widening
};

__device__ inline u32 f32_to_bf16_rne(float f)
{
    u32 u = __float_as_uint(f);
    u32 lsb = (u >> 16) & 1u;
    return (u + 0x7FFFu + lsb) >> 16;
}

// ---- wave / block primitives -------------------------------------------------

__device__ inline u32 lane_id() { return __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u)); }

// number of set bits of `mask` strictly below the calling lane
__device__ inline u32 mask_rank(u64 mask)
{
    return __builtin_amdgcn_mbcnt_hi((u32)(mask >> 32), __builtin_amdgcn_mbcnt_lo((u32)mask, 0u));
}

__device__ inline u32 wave_incl_scan(u32 v)
{
    const u32 lane = lane_id();
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        u32 t = __shfl_up(v, d);
        if (lane >= (u32)d) v += t;
    }
    return v;
}


// Exclusive prefix sum over the threads of a block (thread order); `total`
// receives the block sum.  `scratch` holds BLOCK/64 + 1 words.  Two barriers.
template <int BLOCK>
__device__ inline u32 block_excl_scan(u32 v, u32* scratch, u32* total)
{
    constexpr int NW = BLOCK / kWave;
    const u32 lane = lane_id(), wid = threadIdx.x / kWave;
    u32 inc = wave_incl_scan(v);
    if (lane == kWave - 1) scratch[wid] = inc;
    __syncthreads();
    u32 base = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < NW; ++i) {
        u32 s = scratch[i];
        if ((u32)i < wid) base += s;
        tot += s;
    }
    __syncthreads();
    *total = tot;
    return base + inc - v;
}

// ilogb of a positive finite fp32 given by its bit pattern (subnormals included)
__device__ inline int ilogb_bits(u32 bits)
{
    int ex = (int)(bits >> 23);
    if (ex) return ex - 127;
    return (31 - __clz((int)bits)) - 149;
}

// rint(a * 2^(20-e)) for a positive finite fp32 `bits` with ilogb(a) < e: the
// 20-bit energy grid of ABQ, computed on the significand with round-half-even.
__device__ inline u32 energy_grid(u32 bits, int e)
{
    int ex = (int)(bits >> 23);
    u32 m = bits & 0x7FFFFFu;
    int ea;
    if (ex) { m |= 0x800000u; ea = ex - 127; } else { ea = -126; }
    int s = 3 + e - ea;                 // a * 2^(20-e) = m / 2^s; s >= 4 for normal numbers
    if (s > 25) return 0u;
    if (s <= 0) return m << (-s);       // blocks of deep subnormals (largest value below 2^-129): exact, below 2^21
    u32 q = m >> s;
    u32 rem = m & ((1u << s) - 1u);
    u32 half = 1u << (s - 1);
    if (rem > half || (rem == half && (q & 1u))) ++q;
    return q;
}

// The quantiser of Sec. 3.2.1 works on the block's own scale: with er = ilogb(range), the range
// and every offset a - vmin are multiplied by 2^-er (exact), so the scale L / range stays an
// ordinary fp32 number however small or large the tensor's values are.
__device__ inline int range_exp(float rng) { return ilogb_bits(__float_as_uint(rng)); }   // rng > 0
__device__ inline float unit_range(float rng, int er) { return ldexpf(rng, -er); }        // in [1, 2)
__device__ inline float to_unit(float d, int er) { return ldexpf(d, -er); }

// ---- wave-level primitives without LDS traffic -------------------------------------

__device__ inline void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

__device__ inline u32 bcast(u32 v, int src) { return (u32)__builtin_amdgcn_readlane((int)v, src); }

template <int CTRL, int ROW_MASK, int BANK_MASK>
__device__ inline u32 dpp_get(u32 v)
{
    return (u32)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, BANK_MASK, false);
}

// Inclusive prefix sum over the 64 lanes with data-parallel-primitive moves:
// shifts inside each row of 16 lanes, then the row totals carried across rows.
__device__ inline u32 wave_scan_dpp(u32 v)
{
    u32 r = v + dpp_get<0x111, 0xf, 0xf>(v);     // row_shr:1
    r += dpp_get<0x112, 0xf, 0xf>(v);            // row_shr:2
    r += dpp_get<0x113, 0xf, 0xf>(v);            // row_shr:3
    r += dpp_get<0x114, 0xf, 0xe>(r);            // row_shr:4, lanes 4..15 of a row
    r += dpp_get<0x118, 0xf, 0xc>(r);            // row_shr:8, lanes 8..15 of a row
    r += dpp_get<0x142, 0xa, 0xf>(r);            // lane 15 of rows 0,2 -> rows 1,3
    r += dpp_get<0x143, 0xc, 0xf>(r);            // lane 31 -> rows 2,3
    return r;
}

// Inclusive prefix sum inside each row of 16 lanes: lane 15 of a row ends up with the row's total.
__device__ inline u32 row_scan_dpp(u32 v)
{
    u32 r = v + dpp_get<0x111, 0xf, 0xf>(v);     // row_shr:1
    r += dpp_get<0x112, 0xf, 0xf>(v);            // row_shr:2
    r += dpp_get<0x113, 0xf, 0xf>(v);            // row_shr:3
    r += dpp_get<0x114, 0xf, 0xe>(r);            // row_shr:4, lanes 4..15 of a row
    r += dpp_get<0x118, 0xf, 0xc>(r);            // row_shr:8, lanes 8..15 of a row
    return r;
}

// Sum over the 64 lanes, in every lane (data-parallel-primitive moves: no LDS crossbar traffic).
__device__ inline u32 wave_sum(u32 v) { return bcast(wave_scan_dpp(v), kWave - 1); }

// Maximum over the 64 lanes (unsigned), same data movement as the scan.
__device__ inline u32 wave_max_dpp(u32 v)
{
    u32 r = max(v, dpp_get<0x111, 0xf, 0xf>(v));
    r = max(r, dpp_get<0x112, 0xf, 0xf>(v));
    r = max(r, dpp_get<0x113, 0xf, 0xf>(v));
    r = max(r, dpp_get<0x114, 0xf, 0xe>(r));
    r = max(r, dpp_get<0x118, 0xf, 0xc>(r));
    r = max(r, dpp_get<0x142, 0xa, 0xf>(r));
    r = max(r, dpp_get<0x143, 0xc, 0xf>(r));
    return bcast(r, kWave - 1);
}

// Two unsigned 16-bit lanes in one 32-bit register (packed 16-bit integer instructions): bf16
// magnitude keys are handled two at a time.
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
__device__ inline u16x2 as_u16x2(u32 v) { return __builtin_bit_cast(u16x2, v); }
__device__ inline u32 from_u16x2(u16x2 v) { return __builtin_bit_cast(u32, v); }
__device__ inline u32 pk_max_u16(u32 a, u32 b) { return from_u16x2(__builtin_elementwise_max(as_u16x2(a), as_u16x2(b))); }
__device__ inline u32 pk_min_u16(u32 a, u32 b) { return from_u16x2(__builtin_elementwise_min(as_u16x2(a), as_u16x2(b))); }
__device__ inline u32 pk_sub_sat_u16(u32 a, u32 b) { return from_u16x2(__builtin_elementwise_sub_sat(as_u16x2(a), as_u16x2(b))); }
__device__ inline u32 pk_add_u16(u32 a, u32 b) { return from_u16x2(as_u16x2(a) + as_u16x2(b)); }
__device__ inline u32 pk_mul_lo_u16(u32 a, u32 b) { return from_u16x2(as_u16x2(a) * as_u16x2(b)); }
__device__ inline u32 pk_shl_u16(u32 a, int n) { return from_u16x2(as_u16x2(a) << (unsigned short)n); }
__device__ inline u32 pk_shr_u16(u32 a, int n) { return from_u16x2(as_u16x2(a) >> (unsigned short)n); }

// x / d for x < 2^16 and 1 <= d < 2^16.  (x + 0.5) / d lies at least 0.5 / d away from every
// integer, far more than the error of the reciprocal and the product (a few 2^-24 of the
// quotient, and quotient * d < 2^16), so the truncation needs no repair.
__device__ inline u32 udiv16(u32 x, u32 d)
{
    const float rd = __builtin_amdgcn_rcpf((float)d);
    return (u32)(((float)x + 0.5f) * rd);
}

// ---- workgroup -> row mapping that keeps neighbouring rows on one XCD ---------------------------
// Workgroups are handed to the 8 XCDs round-robin, and every XCD has its own L2.  Rows that
// are neighbours in memory share cache lines (meta arrays, the ends of stream segments), so
// workgroup i takes row (i % 8) * ceil(R / 8) + i / 8: each XCD walks one contiguous eighth of
// the rows.  Launch 8 * ceil(R / 8) workgroups; the result is >= R for the few surplus ones.
constexpr int kXcds = 8;

__host__ __device__ inline int64_t xcd_grid(int64_t R) { return kXcds * ((R + kXcds - 1) / kXcds); }

__device__ inline int64_t xcd_row(int64_t i, int64_t R)
{
    const int64_t chunk = (R + kXcds - 1) / kXcds;
    return (i % kXcds) * chunk + i / kXcds;
}

// ---- bit fields in a word stream (LSB first) -------------------------------------

__device__ inline u32 read_bits(const u32* __restrict__ words, u64 bitpos, int nbits)
{
    u64 wi = bitpos >> 5;
    u32 sh = (u32)bitpos & 31u;
    u64 lo = words[wi];
    if (sh + (u32)nbits > 32u) lo |= (u64)words[wi + 1] << 32;
    return (u32)(lo >> sh) & ((nbits >= 32) ? 0xFFFFFFFFu : ((1u << nbits) - 1u));
}

}  // namespace slicer
