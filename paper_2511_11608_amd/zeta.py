"""Encode-time model and configuration search of Sec. 3.3 ("Constraint-Aware Predictive Configuration").

Two parts, both outside the kernels' hot path:

* ``calibrate`` measures, on the GPU and through the C ABI only, the device-specific lookup table the
  section calls for: encode time of one tensor shape as a function of the knobs theta = (s, M, lambda)
  and of the bitwidth set, split into the three terms of

      zeta_hat(theta, delta) = t_ATKF(s, lambda) + t_MS(M+, M-) + sum t_ABQ(q)

  by differences of whole-call times: t_ATKF = one block per sign class, one fixed bitwidth (no block
  boundaries to find, no search); t_MS(M) = what M blocks add to that; t_ABQ = what the bitwidth search
  over the set adds to the fixed-bitwidth call with the same M.  Times are HIP-event averages.
* ``search`` is the section's hierarchical policy as a small host routine: for a latency budget D and a
  link (rate R, bandwidth W, SNR gamma, outage epsilon; Eq. "comm_latency") it first tunes the block
  count M, then raises the sparsity s, and reports the first knob setting whose predicted latency
  B_UB / R * ceil(ln eps / ln P_o(R)) + zeta_hat fits, with B_UB from ``slicer_bound`` (the library's
  payload bound).  Retreating the split point is the caller's step: it owns the models.

Run ``python -m paper_2511_11608_amd.zeta --workload 4 -o profiles/zeta_llm_prefill.json`` on the GPU machine.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

KEEPS = (0.05, 0.10, 0.20, 0.35)
BLOCKS = (1, 2, 4, 8, 16)
LAMBDAS = (0.0, 0.1)


def _time_calls(fn, reps: int) -> float:
    """Average milliseconds of fn() over reps calls on the current stream (HIP events)."""
    import torch
    for _ in range(3):
        fn()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / reps


def calibrate(x, bit_set: int, reps: int = 20, keeps=KEEPS, blocks=BLOCKS, lambdas=LAMBDAS) -> dict:
    """Lookup table for tensors shaped like x ([rows, row_len] on the GPU)."""
    from . import binding
    rows, row_len = x.shape
    q_bit = bit_set.bit_length() - 1
    table = {"shape": [rows, row_len], "dtype": str(x.dtype).replace("torch.", ""), "bit_set": bit_set,
             "unit": "ms per encode call", "t_atkf": {}, "t_ms": {}, "t_abq": {}, "total": {}}
    for keep in keeps:
        for lam in lambdas:
            sb, meta, ws = binding.alloc_buffers(x, keep, 1, 1 << q_bit)
            if lam == 0.0:
                t = _time_calls(lambda: binding.slicer_encode_ladder(x, keep, [q_bit], sb, meta, ws), reps)
            else:
                t = _time_calls(lambda: binding.slicer_encode_atkf(x, keep, lam, 1, 1, 1 << q_bit, 1e30, sb, meta, ws), reps)
            table["t_atkf"][f"{keep},{lam}"] = t
        base = table["t_atkf"][f"{keep},0.0"]
        for M in blocks:
            sb, meta, ws = binding.alloc_buffers(x, keep, M, bit_set)
            t_fixed = _time_calls(lambda: binding.slicer_encode_ladder(x, keep, [q_bit] * M, sb, meta, ws), reps)
            t_search = _time_calls(lambda: binding.slicer_encode(x, keep, M, bit_set, 1e-3, sb, meta, ws), reps)
            table["t_ms"][f"{keep},{M}"] = max(0.0, t_fixed - base)
            table["t_abq"][f"{keep},{M}"] = max(0.0, t_search - t_fixed)
            table["total"][f"{keep},{M}"] = t_search
    return table


def _nearest(keys, want: float) -> float:
    return min(keys, key=lambda v: abs(v - want))


def zeta_hat(table: dict, keep: float, M: int, lam: float = 0.0) -> float:
    """Predicted encode time in ms: t_ATKF(s, lambda) + t_MS(M) + sum t_ABQ, from the nearest table entries."""
    keeps = sorted({float(k.split(",")[0]) for k in table["t_ms"]})
    blocks = sorted({int(k.split(",")[1]) for k in table["t_ms"]})
    lams = sorted({float(k.split(",")[1]) for k in table["t_atkf"]})
    kq, mq, lq = _nearest(keeps, keep), int(_nearest(blocks, M)), _nearest(lams, lam)
    return table["t_atkf"][f"{kq},{lq}"] + table["t_ms"][f"{kq},{mq}"] + table["t_abq"][f"{kq},{mq}"]


def outage_retransmissions(R: float, W: float, gamma: float, eps: float) -> int:
    """ceil(ln eps / ln P_o(R)), P_o(R) = 1 - exp(-(2^(R/W) - 1) / gamma)  (Eq. "comm_latency")."""
    p_o = 1.0 - math.exp(-(2.0 ** (R / W) - 1.0) / gamma)
    if p_o <= 0.0:
        return 1
    if p_o >= 1.0:
        return 1 << 30
    return max(1, math.ceil(math.log(eps) / math.log(p_o)))


def predicted_latency_ms(bound_bits: int, zeta_ms: float, R: float, W: float, gamma: float, eps: float) -> float:
    """L_c_hat = B_UB / R * ceil(ln eps / ln P_o(R)) + zeta_hat, in ms (R in bit/s)."""
    return 1e3 * bound_bits / R * outage_retransmissions(R, W, gamma, eps) + zeta_ms


def search(table: dict, dt: int, rows: int, row_len: int, bit_set: int, budget_ms: float, R: float,
           W: float = 10e6, gamma: float = 10.0, eps: float = 1e-3, keep_start: float = 0.35,
           keeps=None, blocks=None, bound=None):
    """Hierarchical policy of Sec. 3.3: (1) tune the block count M at the current sparsity, (2) raise the
    sparsity (lower keep ratio) only if no M fits.  Returns (keep, M, predicted ms, bound bits) of the first
    fit, preferring the largest M that fits (finer blocks cost header bits but track the values better),
    or None when nothing fits and the caller has to retreat the split point.  `bound` defaults to the
    library's slicer_bound."""
    if bound is None:
        from . import binding

        def bound(keep, M):
            v, i, h = binding.slicer_bound(dt, rows, row_len, keep, M, bit_set)
            return v + i + h
    keeps = sorted(keeps if keeps is not None else {float(k.split(",")[0]) for k in table["t_ms"]}, reverse=True)
    blocks = sorted(blocks if blocks is not None else {int(k.split(",")[1]) for k in table["t_ms"]}, reverse=True)
    for keep in keeps:
        if keep > keep_start:
            continue
        for M in blocks:
            bits = bound(keep, M)
            ms = predicted_latency_ms(bits, zeta_hat(table, keep, M), R, W, gamma, eps)
            if ms <= budget_ms:
                return keep, M, ms, bits
    return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", type=int, default=4)
    ap.add_argument("--rows", type=int, default=0, help="rows of the workload to calibrate on (0: its full size)")
    ap.add_argument("--reps", type=int, default=20)
    ap.add_argument("-o", "--out", type=str, default="")
    args = ap.parse_args()
    sys.path.insert(0, ROOT)
    from . import binding, synth
    from .devmem import to_device
    binding.load()
    wl = synth.make_config(args.workload, **({"rows": args.rows} if args.rows else {}))
    x = to_device(wl.x, wl.dtype)
    table = calibrate(x, wl.bit_set, reps=args.reps)
    table["workload"] = wl.name
    text = json.dumps(table, indent=1)
    if args.out:
        open(args.out, "w").write(text + "\n")
    print(text)
    return 0


if __name__ == "__main__":
    sys.exit(main())
