"""Host logic of the encode-time model and configuration search (Sec. 3.3): the outage factor of
Eq. "comm_latency" in closed form, the additive time model read from a lookup table, and the order in
which the hierarchical policy visits the knobs.  The GPU test calibrates a small table through the C ABI."""
import math

import pytest

from paper_2511_11608_amd import zeta


def toy_table():
    t = {"t_atkf": {}, "t_ms": {}, "t_abq": {}, "total": {}}
    for keep in (0.05, 0.1, 0.2):
        for lam in (0.0, 0.1):
            t["t_atkf"][f"{keep},{lam}"] = 1.0 + 2 * keep + lam
        for M in (1, 4, 16):
            t["t_ms"][f"{keep},{M}"] = 0.01 * M
            t["t_abq"][f"{keep},{M}"] = 0.5 * keep
    return t


def test_outage_factor_closed_form():
    # R = W: 2^(R/W) - 1 = 1, P_o = 1 - exp(-1/gamma); gamma = 10, eps = 1e-3: ln(1e-3) / ln(0.09516) = 2.94 -> 3
    assert zeta.outage_retransmissions(10e6, 10e6, 10.0, 1e-3) == 3
    p_o = 1 - math.exp(-(2 ** 2.0 - 1) / 10.0)
    assert zeta.outage_retransmissions(20e6, 10e6, 10.0, 1e-3) == math.ceil(math.log(1e-3) / math.log(p_o))
    # latency = bits / R * retransmissions + encode time
    assert zeta.predicted_latency_ms(10_000_000, 0.25, 10e6, 10e6, 10.0, 1e-3) == pytest.approx(1e3 * 1.0 * 3 + 0.25)


def test_time_model_is_the_sum_of_its_three_terms():
    t = toy_table()
    assert zeta.zeta_hat(t, 0.1, 4) == pytest.approx(1.2 + 0.04 + 0.05)
    assert zeta.zeta_hat(t, 0.1, 4, lam=0.1) == pytest.approx(1.3 + 0.04 + 0.05)
    assert zeta.zeta_hat(t, 0.12, 5) == zeta.zeta_hat(t, 0.1, 4)          # nearest entries


def test_search_tunes_blocks_first_then_raises_sparsity():
    t = toy_table()
    bits = lambda keep, M: int(1e6 * keep * 20 + 1e4 * M)               # payload grows with keep ratio and block count
    args = dict(dt=1, rows=1, row_len=1, bit_set=0x1FC, R=10e6, bound=bits)
    lat = lambda keep, M: zeta.predicted_latency_ms(bits(keep, M), zeta.zeta_hat(t, keep, M), 10e6, 10e6, 10.0, 1e-3)
    # generous budget: the lowest sparsity and the finest blocks
    assert zeta.search(t, budget_ms=1e9, **args)[:2] == (0.2, 16)
    # a budget between M = 16 and M = 4 at keep 0.2: the block count gives way first
    b = 0.5 * (lat(0.2, 16) + lat(0.2, 4))
    assert zeta.search(t, budget_ms=b, **args)[:2] == (0.2, 4)
    # below every M at keep 0.2: the sparsity is raised, and M starts from the top again
    b = 0.5 * (lat(0.2, 1) + lat(0.1, 16))
    assert lat(0.1, 16) < b < lat(0.2, 1)
    keep, M, ms, nbits = zeta.search(t, budget_ms=b, **args)
    assert (keep, M) == (0.1, 16) and ms == pytest.approx(lat(0.1, 16)) and nbits == bits(0.1, 16)
    # nothing fits: the caller has to retreat the split point
    assert zeta.search(t, budget_ms=0.1, **args) is None
    # a starting sparsity below the table's lowest is respected
    assert zeta.search(t, budget_ms=1e9, keep_start=0.1, **args)[:2] == (0.1, 16)


@pytest.mark.gpu
def test_calibrated_table_and_search_on_the_gpu():
    import torch
    from paper_2511_11608_amd import binding, synth
    from paper_2511_11608_amd.devmem import to_device
    wl = synth.llm_prefill(seed=1, rows=512)
    x = to_device(wl.x, wl.dtype)
    t = zeta.calibrate(x, wl.bit_set, reps=3, keeps=(0.05, 0.1), blocks=(1, 8), lambdas=(0.0, 0.1))
    for keep in (0.05, 0.1):
        for M in (1, 8):
            parts = t["t_atkf"][f"{keep},0.0"] + t["t_ms"][f"{keep},{M}"] + t["t_abq"][f"{keep},{M}"]
            assert parts > 0 and zeta.zeta_hat(t, keep, M) == pytest.approx(parts)
            assert parts >= t["total"][f"{keep},{M}"] * 0.999          # equal unless a difference was clamped at 0
    got = zeta.search(t, binding.SLICER_BF16, 512, 4096, wl.bit_set, budget_ms=1e9, R=10e6)
    v, i, h = binding.slicer_bound(binding.SLICER_BF16, 512, 4096, got[0], got[1], wl.bit_set)
    assert got[:2] == (0.1, 8) and got[3] == v + i + h
