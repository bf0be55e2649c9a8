"""Arithmetic parity of the elementary operations (GPU, through the C ABI): every fp32 / fp64 / bf16 step
the codec's arithmetic rests on - divisions, products, sums, round-half-even, power-of-two scaling,
the unfused multiply-then-add of the residual, the bf16 narrowing, the energy grid - computed by the
HIP build exactly as the kernels write it and compared bit for bit with IEEE arithmetic on the host
(numpy: one correctly rounded operation per step, denormals kept), on 10^7 operand pairs per operation."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

N = 10_000_000


def operands(seed):
    """fp32 bit patterns: finite values of every exponent (denormals included), plus values at and next to
    half-integers and powers of two, where a wrong rounding rule shows."""
    rng = np.random.default_rng(seed)
    u = rng.integers(0, 1 << 32, N, dtype=np.uint64).astype(np.uint32)
    ex = (u >> np.uint32(23)) & np.uint32(0xFF)
    u = np.where(ex == 255, u & np.uint32(0xBFFFFFFF), u)                      # no infinities, no NaNs
    # a third of them in a moderate range (|x| in [2^-20, 2^20]): sums and products that stay finite
    mod = rng.random(N) < 0.34
    e_mod = rng.integers(107, 148, N, dtype=np.uint32)
    u = np.where(mod, (u & np.uint32(0x807FFFFF)) | (e_mod << np.uint32(23)), u)
    f = u.view(np.float32).copy()
    k = N // 10
    half = (rng.integers(0, 1 << 22, k).astype(np.float32) + np.float32(0.5)) * rng.choice(np.array([-1, 1], np.float32), k)
    f[:k] = half
    f[k:2 * k] = np.nextafter(half, np.float32(np.inf))
    f[2 * k:3 * k] = np.nextafter(half, np.float32(-np.inf))
    f[3 * k:3 * k + 277] = np.ldexp(np.float32(1), np.arange(-149, 128)).astype(np.float32)      # every power of two
    return f.view(np.uint32)


def bf16_rne(v32):
    bits = v32.view(np.uint32)
    lo = bits & np.uint32(0xFFFF0000)
    hi = lo + np.uint32(0x10000)
    v64 = v32.astype(np.float64)
    fhi = hi.view(np.float32).astype(np.float64)
    fhi = np.where(np.isinf(fhi), np.sign(fhi) * 2.0 ** 128, fhi)          # the neighbour above the largest bf16 number
    dlo, dhi = np.abs(v64 - lo.view(np.float32).astype(np.float64)), np.abs(fhi - v64)
    lo_even = ((lo >> np.uint32(16)) & np.uint32(1)) == 0
    return (np.where((dlo < dhi) | ((dlo == dhi) & lo_even), lo, hi) >> np.uint32(16)).astype(np.uint32)


def expected(op, au, bu):
    a, b = au.view(np.float32), bu.view(np.float32)
    with np.errstate(all="ignore"):
        if op in (0, 1):
            return (a / b).view(np.uint32)
        if op == 2:
            return (a * b).view(np.uint32)
        if op == 3:
            return (a + b).view(np.uint32)
        if op == 4:
            return (a - b).view(np.uint32)
        if op == 5:
            return np.rint(a).view(np.uint32)
        if op == 6:
            return np.ldexp(a, (bu % np.uint32(301)).astype(np.int32) - 150).astype(np.float32).view(np.uint32)
        if op == 7:
            return ((a * b) + np.float32(8388608.0)).view(np.uint32)
        if op == 8:
            return bf16_rne(a)
        if op == 9:
            return (a + (b * b)).view(np.uint32)
        if op == 10:
            mag = np.abs(a).astype(np.float64)
            m, ex = np.frexp(mag)                                    # mag = m * 2^ex, m in [0.5, 1): ilogb = ex - 1
            e = ex + (bu % np.uint32(3)).astype(np.int64)
            return np.where(mag > 0, np.rint(np.ldexp(mag, (20 - e).astype(np.int32))), 0).astype(np.uint32)
        if op == 11:
            d = (a.astype(np.float64) * a.astype(np.float64)) * bu.astype(np.float64) * 2.0 ** -30
            w = d.view(np.uint64)
            return ((w >> np.uint64(32)) ^ (w & np.uint64(0xFFFFFFFF))).astype(np.uint32)
    raise ValueError(op)


@pytest.mark.parametrize("op", range(12))
def test_elementary_operation_matches_ieee(op):
    import torch
    from paper_2511_11608_amd import binding
    au, bu = operands(2 * op), operands(2 * op + 1)
    if op in (0, 1):
        bu = np.where((bu & np.uint32(0x7FFFFFFF)) == 0, np.uint32(0x3F800000), bu)      # no division by zero
    if op == 10:
        au = au & np.uint32(0x7FFFFFFF)
    ad = torch.from_numpy(au.view(np.int32)).cuda()
    bd = torch.from_numpy(bu.view(np.int32)).cuda()
    out = torch.empty_like(ad)
    binding.slicer_arith_probe(op, ad, bd, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy().view(np.uint32)
    want = expected(op, au, bu)
    if op in (0, 1, 2, 3, 4, 6, 7, 9):                   # NaNs (0 * inf cannot occur, inf - inf can): compare as "both NaN"
        nan = np.isnan(want.view(np.float32))
        assert np.array_equal(np.isnan(got.view(np.float32)), nan)
        got, want = got[~nan], want[~nan]
    bad = np.nonzero(got != want)[0]
    assert bad.size == 0, (op, bad[:5], [hex(int(v)) for v in au[bad[:5]]], [hex(int(v)) for v in bu[bad[:5]]],
                           [hex(int(v)) for v in got[:5]], [hex(int(v)) for v in want[:5]])
