#!/usr/bin/env python3
"""Benchmark of the SLICER IF codec hot path on one MI355X.

A step = one encode (ATKF -> MS -> ABQ -> packing) followed by one decode of one
batch of synthetic intermediate features, inputs already resident in HBM.  The
default workload is the LLM-prefill configuration (bf16 [16384, 4096], the largest
of the five); input buffers rotate over > 256 MB of distinct device memory so that
the Infinity Cache does not stand in for HBM.

Consecutive steps work on independent batches (the paper's many clients, or the successive
token batches of one client), so the K timed steps alternate over three HIP streams by default:
step i+1 fills the ramp, the drain and the launch gaps of step i.  `value` is the throughput of
those K steps; `single_stream` in the same line is the figure with every step on one stream,
`step_latency_us` the time of one step submitted alone.

Prints ONE JSON line: whole-step throughput in GB/s of input IF, the roofline
record of the dominant kernel (the encode kernel that does the selection, quantisation
and packing of a row; its duration is read with HIP events recorded around it on its stream), and the CPU oracle timed on
a bounded sample of the same workload.  The same line carries `workloads`: all five
configurations at full size, each measured in a short single-stream loop (encode and decode call,
dominant kernel, step latency, bits per element, oracle on a small sample; the AR-decode
workload over its 512 steps with fresh seeds), and `device_copy`: a plain device copy timed in
the same run, the practical HBM rate next to the published 8 TB/s.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published


class HipEvents:
    """Raw hipEvent_t handles through libamdhip64 (torch's Event does not expose a
    handle that can be passed across the C ABI before it has been recorded)."""

    def __init__(self):
        self.hip = C.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [C.c_void_p]
        self.hip.hipEventDestroy.argtypes = [C.c_void_p]

    def create(self) -> int:
        e = C.c_void_p()
        rc = self.hip.hipEventCreate(C.byref(e))
        if rc:
            raise RuntimeError(f"hipEventCreate: {rc}")
        return e.value

    def elapsed_ms(self, a: int, b: int) -> float:
        self.hip.hipEventSynchronize(b)
        ms = C.c_float(0)
        rc = self.hip.hipEventElapsedTime(C.byref(ms), a, b)
        if rc:
            raise RuntimeError(f"hipEventElapsedTime: {rc}")
        return ms.value


AR_STEPS = 512          # the AR-decode workload: 512 steps, a fresh seed per step


def make_workload(which: int, ar_steps: int = AR_STEPS):
    from paper_2511_11608_amd import synth
    if which == 5:
        from concurrent.futures import ThreadPoolExecutor
        workers = max(1, min(16, os.cpu_count() or 1))
        with ThreadPoolExecutor(max_workers=workers) as ex:     # numpy's generators release the GIL
            steps = list(ex.map(lambda s: synth.ar_decode_step(seed=0, step=s), range(ar_steps)))
        return steps[0], [s.x for s in steps]
    wl = synth.make_config(which)
    return wl, [wl.x]


def cpu_baseline(wl, threads: int, ladder=None, ds=None, lam=None, seconds: float = 15.0) -> dict:
    """The oracle as it stands (encode + decode) on a bounded sample of the rows."""
    from oracle import ref
    ref.lib()

    def ref_encode(x, n_threads):
        if ladder:
            return ref.encode_ladder(x, wl.dtype, wl.keep_ratio, ladder, n_threads=n_threads)
        if ds is not None:
            return ref.encode_ds(x, wl.dtype, wl.keep_ratio, wl.n_blocks, wl.bit_set, ds, n_threads=n_threads)
        if lam is not None:
            return ref.encode_atkf(x, wl.dtype, wl.keep_ratio, lam, wl.n_blocks, wl.n_blocks, wl.bit_set, wl.budget,
                                   n_threads=n_threads)
        return ref.encode(x, wl.dtype, wl.keep_ratio, wl.n_blocks, wl.bit_set, wl.budget, n_threads=n_threads)

    rows = wl.rows
    probe = max(1, min(rows, 64 if wl.row_len < 100_000 else 2))
    t0 = time.perf_counter()
    s, m = ref_encode(wl.x[:probe], threads)
    ref.decode(s, m, n_threads=threads)
    per_row = (time.perf_counter() - t0) / probe * min(threads, probe)      # core-seconds per row
    take = int(max(probe, min(rows, seconds / max(per_row, 1e-9))))
    x = wl.x[:take]
    t0 = time.perf_counter()
    s, m = ref_encode(x, threads)
    t1 = time.perf_counter()
    ref.decode(s, m, n_threads=threads)
    t2 = time.perf_counter()
    nbytes = x.nbytes
    # one thread, on a slice of the sample sized for a few seconds
    take1 = int(max(1, min(take, 0.27 * seconds / max(per_row, 1e-9))))
    x1 = wl.x[:take1]
    t3 = time.perf_counter()
    s1, m1 = ref_encode(x1, 1)
    ref.decode(s1, m1, n_threads=1)
    t4 = time.perf_counter()
    return {"value": nbytes / (t2 - t0) / 1e9, "unit": "GB/s of input IF (encode+decode)",
            "cores": int(min(threads, take)), "kind": "oracle",
            "sample": f"first {take} of {rows} rows of the same workload, OpenMP over rows",
            "encode_GBps": nbytes / (t1 - t0) / 1e9, "decode_GBps": nbytes / (t2 - t1) / 1e9,
            "single_thread_GBps": x1.nbytes / (t4 - t3) / 1e9, "single_thread_rows": take1}


VALU_PEAK_TLOPS = 256 * 4 * 16 * 2.4e9 / 1e12    # lane-operations/s: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz, one plain op per lane and cycle


def alu_view(workload: str, kernel: str, kernel_ms: float):
    """How close the kernel runs to the vector-ALU issue rate: VALU wave-instructions per launch (a committed
    rocprofv3 --pmc SQ_INSTS_VALU count, 64 lane-operations each) over the duration measured in this run."""
    try:
        n = json.load(open(os.path.join(ROOT, "profiles", "valu_counts.json")))[workload][kernel]
    except Exception:
        return None
    achieved = n * 64 / (kernel_ms * 1e-3) / 1e12
    return {"bound": "alu", "achieved": achieved, "peak": VALU_PEAK_TLOPS, "unit": "T lane-op/s",
            "frac": achieved / VALU_PEAK_TLOPS, "valu_wave_instructions_per_launch": n}


def load_traffic(workload: str, kernel: str):
    """HBM bytes per launch from committed rocprofv3 --pmc summaries, if present."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        table = json.load(open(path))
        return table[workload][kernel]
    except Exception:
        return None


def measure_workload(which: int, ev: "HipEvents", threads: int, cpu_seconds: float, pregenerated=None,
                     steps: int = 40) -> dict:
    """One entry of the line's `workloads` array: a short single-stream measurement of workload `which`
    at its full size (encode call, decode call, dominant encode kernel, step latency, compressed size)
    and the oracle on a bounded sample.  The AR-decode workload runs its 512 steps, each with its own seed."""
    import torch
    from paper_2511_11608_amd import binding
    from paper_2511_11608_amd.devmem import to_device

    wl, xs = pregenerated if pregenerated is not None else make_workload(which)
    M, bits, keep, beta = wl.n_blocks, wl.bit_set, wl.keep_ratio, wl.budget
    dt = binding.SLICER_F32 if wl.dtype == "f32" else binding.SLICER_BF16
    in_bytes = wl.nbytes
    x0 = [to_device(x, wl.dtype) for x in xs]
    n_buf = min(max(len(x0), int(np.ceil(320e6 / in_bytes)) + 1), 512)      # > 256 MB of distinct inputs in flight
    xd, shift = list(x0), 1
    while len(xd) < n_buf:
        xd.append(torch.roll(x0[len(xd) % len(x0)], shifts=shift, dims=0).contiguous())
        shift += 1
    n_out = min(n_buf, 4)
    bufs = [binding.alloc_buffers(xd[0], keep, M, bits) for _ in range(n_out)]
    ys = [torch.empty_like(xd[0]) for _ in range(n_out)]
    K = len(xs) if which == 5 else steps

    def enc(i):
        binding.slicer_encode(xd[i % n_buf], keep, M, bits, beta, *bufs[i % n_out])

    def dec(i):
        binding.slicer_decode_as(bufs[i % n_out][0], bufs[i % n_out][1], ys[i % n_out], M)

    for i in range(max(3, min(n_buf, 8))):
        enc(i); dec(i)
    torch.cuda.synchronize()
    st = torch.cuda.current_stream().cuda_stream
    ev.hip.hipEventRecord.argtypes = [C.c_void_p, C.c_void_p]

    def timed_loop(fn):
        a, b = ev.create(), ev.create()
        ev.hip.hipEventRecord(a, st)
        for i in range(K):
            fn(i)
        ev.hip.hipEventRecord(b, st)
        return ev.elapsed_ms(a, b) / K

    enc_ms = timed_loop(enc)
    dec_ms = timed_loop(dec)
    # dominant encode kernel (or the chain of long-row stages): HIP events recorded inside the call
    pairs = [(ev.create(), ev.create()) for _ in range(min(K, 40))]
    for i, pr in enumerate(pairs):
        binding.slicer_profile_events(*pr)
        enc(i)
    binding.slicer_profile_events(None, None)
    torch.cuda.synchronize()
    kern_ms = float(np.mean([ev.elapsed_ms(a, b) for a, b in pairs]))
    lats = []
    for i in range(min(K, 512)):
        t_a = time.perf_counter()
        enc(i); dec(i)
        torch.cuda.synchronize()
        lats.append((time.perf_counter() - t_a) * 1e6)
    enc(0)
    words = binding.slicer_stream_words(bufs[0][1])
    _, meta_bytes, _ = binding.slicer_sizes(dt, wl.rows, wl.row_len, keep, M, bits)
    out_bytes = 4 * words + meta_bytes
    path = binding.slicer_encode_path(dt, wl.rows, wl.row_len, keep, M, bits)
    kernel = {0: "enc_generic_kernel", 1: "enc_small_kernel", 2: "lr_* stages (hist..pack)", 3: "enc_wg_kernel"}[path]
    alg = in_bytes + out_bytes
    rec = {
        "workload": f"{wl.name} [{wl.rows}x{wl.row_len}] keep={keep} M={M} bits=2..8 budget={beta}",
        "config": which, "dtype": wl.dtype, "input_bytes": in_bytes, "steps": K,
        "encode_ms": enc_ms, "decode_ms": dec_ms,
        "encode_GBps": in_bytes / (enc_ms * 1e-3) / 1e9, "decode_GBps": in_bytes / (dec_ms * 1e-3) / 1e9,
        "frac_hbm_peak": in_bytes / (enc_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "decode_frac_hbm_peak": in_bytes / (dec_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "bits_per_element": 8.0 * out_bytes / (wl.rows * wl.row_len),
        "roofline": {"bound": "hbm", "kernel": kernel, "kernel_ms": kern_ms, "algorithmic_bytes_per_launch": alg,
                     "achieved": alg / (kern_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": alg / (kern_ms * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "step_latency_us": {"p50": float(np.percentile(lats, 50)), "p99": float(np.percentile(lats, 99)), "n": len(lats)},
        "inputs": f"{len(xs)} seeded batch(es), {n_buf} distinct device buffers",
    }
    if cpu_seconds > 0:
        c = cpu_baseline(wl, threads, seconds=cpu_seconds)
        rec["cpu_baseline"] = {k: c[k] for k in ("value", "unit", "cores", "kind", "sample", "single_thread_GBps")}
    del xd, x0, bufs, ys
    torch.cuda.empty_cache()
    return rec


def copy_rate(ev: "HipEvents", nbytes: int = 256 << 20, reps: int = 20) -> dict:
    """A plain device copy measured in this run, next to the published 8 TB/s: bytes read + written per second."""
    import torch
    src = [torch.empty(nbytes, dtype=torch.uint8, device="cuda").fill_(i) for i in range(3)]
    dst = [torch.empty(nbytes, dtype=torch.uint8, device="cuda") for _ in range(3)]
    for i in range(3):
        dst[i].copy_(src[i])
    torch.cuda.synchronize()
    st = torch.cuda.current_stream().cuda_stream
    ev.hip.hipEventRecord.argtypes = [C.c_void_p, C.c_void_p]
    a, b = ev.create(), ev.create()
    ev.hip.hipEventRecord(a, st)
    for i in range(reps):
        dst[i % 3].copy_(src[i % 3])
    ev.hip.hipEventRecord(b, st)
    ms = ev.elapsed_ms(a, b) / reps
    return {"GBps_read_plus_write": 2 * nbytes / (ms * 1e-3) / 1e9, "bytes_per_copy": nbytes, "kernel": "device-to-device copy (torch copy_)",
            "frac_of_published_peak": 2 * nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}


def profile_source() -> dict:
    """Which commit the committed counter tables (HBM traffic, VALU counts) were taken at."""
    out = {}
    for name in ("hbm_traffic.json", "valu_counts.json"):
        try:
            out[name] = json.load(open(os.path.join(ROOT, "profiles", name))).get("_source", "unrecorded")
        except Exception:
            out[name] = "missing"
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", type=int, default=4, help="1..5 (default 4: LLM prefill, the headline config)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--no-workloads", action="store_true",
                    help="skip the per-workload array (all five configurations measured in short loops)")
    ap.add_argument("--ladder", type=str, default="",
                    help="time the fixed multi-level mode instead of the bitwidth search: comma-separated "
                         "bitwidths, one per block of a sign class, e.g. 8,7,6,5,4,3,2,2")
    ap.add_argument("--ds", type=float, default=None,
                    help="time the paper's DS guard with greedy descent at this delta instead of the budget search")
    ap.add_argument("--lam", type=float, default=None,
                    help="time the asymmetric thresholds of Sec. 3.1 at this asymmetry factor (0 < lambda < 1; rows of up to "
                         "8192 bf16 / 4096 fp32 elements on the one-wavefront-per-row kernel, everything else on the generic kernel)")
    ap.add_argument("--csr-cols", type=int, default=None,
                    help="time the two-dimensional instance of Sec. 3.2 step 3: every row of the workload is one tensor of "
                         "(row_len / K) x K whose blocks are stored as CSR triples; K must divide the row length")
    ap.add_argument("--keep-ratio", type=float, default=None, help="override the workload's keep ratio (1 - s)")
    ap.add_argument("--n-blocks", type=int, default=None, help="override the workload's block count M per sign class")
    ap.add_argument("--streams", type=int, default=3,
                    help="HIP streams the steps alternate over (default 3): consecutive steps work on independent "
                         "batches, so step i+1 fills the ramp, the drain and the launch gaps of step i; 1 = one stream")
    ap.add_argument("--eager", action="store_true",
                    help="time plain launches instead of replaying a captured HIP graph of the steps")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run plain device copies of the input tensor (known size), the yardstick that "
                         "scales the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this codec build runs on ONE GPU (rows are independent codec instances, so more GPUs "
              "would each take a share of the rows with nothing exchanged); run with --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2511_11608_amd import binding
    from paper_2511_11608_amd.devmem import to_device     # numpy -> device tensor (plumbing only)

    binding.load()
    wl, xs = make_workload(args.workload)
    if args.keep_ratio is not None:
        wl.keep_ratio = args.keep_ratio
    if args.n_blocks is not None:
        wl.n_blocks = args.n_blocks
    M, bits, keep, beta = wl.n_blocks, wl.bit_set, wl.keep_ratio, wl.budget
    ladder = [int(q) for q in args.ladder.split(",")] if args.ladder else None
    if ladder:
        M, bits = len(ladder), binding.slicer_ladder_bit_set(ladder)
        if not bits:
            print("bench.py: --ladder entries must be 1..16", file=sys.stderr)
            return 2

    csr = args.csr_cols
    if csr is not None and (csr < 1 or wl.row_len % csr):
        print("bench.py: --csr-cols must divide the row length", file=sys.stderr)
        return 2

    def decode(sb, meta, y, st=None):
        if csr is not None:
            binding.slicer_decode_as_csr(sb, meta, y, wl.row_len // csr, csr, M, stream=st)
        else:
            binding.slicer_decode_as(sb, meta, y, M, stream=st)

    def encode(x, sb, meta, ws, st=None):
        if csr is not None:
            binding.slicer_encode_csr(x, wl.row_len // csr, csr, keep, M, bits, beta, sb, meta, ws, stream=st)
        elif ladder:
            binding.slicer_encode_ladder(x, keep, ladder, sb, meta, ws, stream=st)
        elif args.ds is not None:
            binding.slicer_encode_ds(x, keep, M, bits, args.ds, sb, meta, ws, stream=st)
        elif args.lam is not None:
            binding.slicer_encode_atkf(x, keep, args.lam, M, M, bits, beta, sb, meta, ws, stream=st)
        else:
            binding.slicer_encode(x, keep, M, bits, beta, sb, meta, ws, stream=st)
    in_bytes = wl.nbytes

    # distinct input buffers: > 256 MB in flight so that reads come from HBM
    x0 = [to_device(x, wl.dtype) for x in xs]
    n_buf = max(len(x0), int(np.ceil(320e6 / in_bytes)) + 1)
    n_buf = min(n_buf, 512)
    xd = list(x0)
    shift = 1
    while len(xd) < n_buf:
        xd.append(torch.roll(x0[len(xd) % len(x0)], shifts=shift, dims=0).contiguous())
        shift += 1
    # Steps alternate over S streams (default priority).  Output buffer set j is only ever used by
    # stream j % S (n_out is a multiple of S), so the steps that share buffers stay in order.
    S = max(1, min(int(args.streams), 8))
    side = [torch.cuda.Stream() for _ in range(S)] if S > 1 else []
    n_out = S * max(1, -(-min(n_buf, 4) // S))
    if csr is not None:
        bufs = [binding.alloc_buffers_csr(xd[0], wl.row_len // csr, csr, keep, M, bits) for _ in range(n_out)]
    else:
        bufs = [binding.alloc_buffers(xd[0], keep, M, bits) for _ in range(n_out)]
    ys = [torch.empty_like(xd[0]) for _ in range(n_out)]

    ev = HipEvents()
    K, W = args.steps, args.warmup
    e_enc = [(ev.create(), ev.create()) for _ in range(K)]
    e_dec = [(ev.create(), ev.create()) for _ in range(K)]

    def step(i: int, timed_idx: int | None, multi: bool = False):
        x = xd[i % n_buf]
        sb, meta, ws = bufs[i % n_out]
        st = side[i % S] if (multi and S > 1) else None      # None: the current stream
        if timed_idx is not None:
            binding.slicer_profile_events(*e_enc[timed_idx])
        encode(x, sb, meta, ws, st)
        if timed_idx is not None:
            binding.slicer_profile_events(*e_dec[timed_idx])
        decode(sb, meta, ys[i % n_out], st)

    def fork():                                   # the side streams start after everything queued on the current one
        cur = torch.cuda.current_stream()
        for sd in side:
            sd.wait_stream(cur)

    def join():
        cur = torch.cuda.current_stream()
        for sd in side:
            cur.wait_stream(sd)

    for i in range(max(W, n_buf)):               # every kernel is loaded and every buffer touched before a capture
        step(i, None)
    torch.cuda.synchronize()

    # single stream, plain launches: the figure without any overlap between steps (reported beside `value`)
    t0 = time.perf_counter()
    for i in range(K):
        step(W + i, None)
    torch.cuda.synchronize()
    single_ms = (time.perf_counter() - t0) * 1e3 / K

    # The launch-bound part of a step (four short kernels back to back) is captured once into a
    # HIP graph of n_cap consecutive steps (over the S streams: fork, steps, join) and replayed;
    # every replay is checked against the plain launches.  Anything wrong with capture or replay
    # falls back to plain launches.
    n_cap = max(n_buf, n_out)
    graph, launch = None, "plain launches"
    # (with several streams the launch gaps of one step are filled by its neighbours, and plain launches
    #  overlap better than a replayed graph, whose fork and join drain the device every n_cap steps)
    if not args.eager and S == 1:
        try:
            def snapshot():
                torch.cuda.synchronize()
                return [(b[0].clone(), b[1].clone(), y.clone()) for b, y in zip(bufs, ys)]
            for i in range(n_cap):
                step(i, None)
            want = snapshot()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                fork()
                for i in range(n_cap):
                    step(i, None, multi=True)
                join()
            ok = True
            for _ in range(3):
                for b, y in zip(bufs, ys):
                    b[0].fill_(-1); b[1].fill_(0); y.fill_(1)
                g.replay()
                got = snapshot()
                meta_b = binding.slicer_sizes(binding.SLICER_F32 if wl.dtype == "f32" else binding.SLICER_BF16,
                                              wl.rows, wl.row_len, keep, M, bits)[1]
                for (s0, m0, y0), (s1, m1, y1) in zip(want, got):
                    nw = int(m0[:64].view(torch.int64)[6].item())
                    ok = ok and torch.equal(m0[:meta_b], m1[:meta_b]) and torch.equal(y0, y1) \
                        and torch.equal(s0.view(torch.int32)[:nw], s1.view(torch.int32)[:nw])
            if ok:
                graph, launch = g, f"hipGraph of {n_cap} steps"
            else:
                print("bench.py: graph replay differs from plain launches; timing plain launches", file=sys.stderr)
        except Exception as e:                   # capture unsupported: plain launches
            print(f"bench.py: graph capture failed ({e}); timing plain launches", file=sys.stderr)
            graph = None
    torch.cuda.synchronize()

    if S > 1:                                      # the side streams' first launches create their queues: not timed
        fork()
        for i in range(max(W, 2 * S)):
            step(i, None, multi=True)
        join()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    if graph is not None:
        for _ in range(K // n_cap):
            graph.replay()
        if K % n_cap:
            fork()
            for i in range(K - K % n_cap, K):
                step(i, None, multi=True)
            join()
    else:
        fork()
        for i in range(K):
            step(W + i, None, multi=True)
        join()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / K
    launch += f", steps alternate over {S} streams" if S > 1 else ", one stream"

    # kernel durations: the same K steps with HIP events around the dominant kernels
    for i in range(K):
        step(W + i, i)
    torch.cuda.synchronize()
    binding.slicer_profile_events(None, None)

    # latency of single steps (submit, wait): the figure that matters for step-by-step decoding
    lats = []
    for i in range(min(K, 200)):
        t_a = time.perf_counter()
        step(W + i, None)
        torch.cuda.synchronize()
        lats.append((time.perf_counter() - t_a) * 1e6)
    lat = {"p50": float(np.percentile(lats, 50)), "p99": float(np.percentile(lats, 99)), "n": len(lats),
           "note": "one step submitted and waited for from the host, plain launches"}

    enc_ms = float(np.mean([ev.elapsed_ms(a, b) for a, b in e_enc]))
    dec_ms = float(np.mean([ev.elapsed_ms(a, b) for a, b in e_dec]))

    # encode-only and decode-only loops (whole call, all kernels), HIP events on the stream
    def timed_loop(fn):
        a, b = ev.create(), ev.create()
        st = torch.cuda.current_stream().cuda_stream
        ev.hip.hipEventRecord.argtypes = [C.c_void_p, C.c_void_p]
        ev.hip.hipEventRecord(a, st)
        for i in range(K):
            fn(i)
        ev.hip.hipEventRecord(b, st)
        return ev.elapsed_ms(a, b) / K

    enc_call_ms = timed_loop(lambda i: encode(xd[i % n_buf], *bufs[i % n_out]))
    dec_call_ms = timed_loop(lambda i: decode(bufs[i % n_out][0], bufs[i % n_out][1], ys[i % n_out]))

    # compressed size of the last batch encoded into bufs[0]
    encode(xd[0], *bufs[0])
    words = binding.slicer_stream_words(bufs[0][1])
    _, meta_bytes, _ = binding.slicer_sizes(binding.SLICER_F32 if wl.dtype == "f32" else binding.SLICER_BF16,
                                            wl.rows, wl.row_len, keep, M, bits)
    n_el = wl.rows * wl.row_len
    out_bytes = 4 * words + meta_bytes
    bpe = 8.0 * out_bytes / n_el
    # where the bits go (Sec. 3.3: value bits, index bits, header): counts from the meta arrays
    torch.cuda.synchronize()
    mh = bufs[0][1][:meta_bytes].cpu().numpy()
    R_, M_ = wl.rows, M
    n_kept = int(mh[64 + 8 * R_: 64 + 16 * R_].view(np.uint32).sum())
    w_bits = max(1, int(np.ceil(np.log2(csr if csr is not None else wl.row_len)))) if (csr or wl.row_len) > 1 else 1   # (CSR: column bits; the row pointers count with the values below)
    idx_bits_total = n_kept * w_bits
    value_bits_total = 32 * words - idx_bits_total          # codes + the word padding of each row
    bit_split = {"index_bits_per_element": idx_bits_total / n_el, "value_bits_per_element": value_bits_total / n_el,
                 "header_bits_per_element": 8.0 * meta_bytes / n_el, "kept_elements": n_kept}

    path = binding.slicer_encode_path(binding.SLICER_F32 if wl.dtype == "f32" else binding.SLICER_BF16,
                                      wl.rows, wl.row_len, keep, M, bits)
    asym = args.lam is not None and args.lam > 0
    if (asym or args.ds is not None) and path == 3:      # the workgroup-per-row kernel takes the budget guard at lambda = 0 only:
        path = binding.slicer_encode_path(binding.SLICER_F32 if wl.dtype == "f32" else binding.SLICER_BF16,
                                          2048, wl.row_len, keep, M, bits)      # what a large batch of these rows runs on
        path = 0 if path == 3 else path
    if asym and path != 1:
        path = 0                                         # the second selection: one-wavefront-per-row kernel, else the generic kernel
    enc_kernel = {0: "enc_generic_kernel", 1: "enc_small_kernel", 2: "lr_* stages (hist..pack)", 3: "enc_wg_kernel"}[path]
    # (two-dimensional instances: the flat encoder of the shape is the dominant kernel; csr_repack_kernel follows it)
    dec_kernel = "dec_small_kernel" if wl.row_len * (4 if wl.dtype == "f32" else 2) <= 16384 else "dec_kernel"
    if csr is not None:
        dec_kernel = "dec_csr_kernel"
    enc_alg_bytes = in_bytes + out_bytes                 # read x once, write stream + meta
    dec_alg_bytes = out_bytes + in_bytes                 # read stream + meta, write y once
    achieved = enc_alg_bytes / (enc_ms * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": enc_kernel, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBS, "traffic": load_traffic(wl.name, enc_kernel),
                "algorithmic_bytes_per_launch": enc_alg_bytes, "kernel_ms": enc_ms,
                "alu": None if (ladder or args.ds is not None or args.lam is not None) else alu_view(wl.name, enc_kernel, enc_ms),
                "decode_kernel": {"kernel": dec_kernel, "kernel_ms": dec_ms,
                                  "achieved": dec_alg_bytes / (dec_ms * 1e-3) / 1e9,
                                  "frac": dec_alg_bytes / (dec_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                  "traffic": load_traffic(wl.name, dec_kernel)}}

    if args.copy_probe:
        for i in range(4):
            ys[i % n_out].copy_(xd[i % n_buf])          # reads in_bytes, writes in_bytes
        torch.cuda.synchronize()

    threads = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)))
    cpu = None if args.no_cpu else cpu_baseline(wl, threads, ladder, args.ds, args.lam)
    roofline["traffic_source"] = profile_source()
    copy = copy_rate(ev)

    # all five configurations, each at its full size, in short single-stream loops
    workloads = None
    plain = csr is None and not (ladder or args.ds is not None or args.lam is not None or args.keep_ratio is not None or args.n_blocks is not None)
    if plain and not args.no_workloads:
        del xd, x0, bufs, ys
        torch.cuda.empty_cache()
        workloads = []
        for which in (1, 2, 3, 4, 5):
            pre = (wl, xs) if which == args.workload and which != 5 else None
            workloads.append(measure_workload(which, ev, threads, 0.0 if args.no_cpu else 3.0, pre))

    out = {
        "metric": "codec encode+decode throughput, GB/s of input IF",
        "value": in_bytes / (ms_per_step * 1e-3) / 1e9,
        "unit": "GB/s",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic", "launch": launch,
        "config": {"workload": f"{wl.name} [{wl.rows}x{wl.row_len}] keep={keep} M={M} "
                               + (f"ladder={ladder}" if ladder else f"bits=2..8 DS delta={args.ds}" if args.ds is not None
                                  else f"bits=2..8 budget={beta}") + (f" lambda={args.lam}" if args.lam is not None else "")
                               + (f" CSR blocks, instances of {wl.row_len // csr}x{csr}" if csr is not None else ""),
                   "input_bytes": in_bytes, "distinct_input_buffers": n_buf},
        "encode": {"GBps": in_bytes / (enc_call_ms * 1e-3) / 1e9, "ms": enc_call_ms,
                   "elements_per_s": n_el / (enc_call_ms * 1e-3),
                   "frac_hbm_peak": in_bytes / (enc_call_ms * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "decode": {"GBps": in_bytes / (dec_call_ms * 1e-3) / 1e9, "ms": dec_call_ms,
                   "elements_per_s": n_el / (dec_call_ms * 1e-3),
                   "frac_hbm_peak": in_bytes / (dec_call_ms * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "bits_per_element": bpe, "bit_split": bit_split, "stream_words": words, "meta_bytes": meta_bytes,
        "step_latency_us": lat,
        "single_stream": {"ms_per_step": single_ms, "value": in_bytes / (single_ms * 1e-3) / 1e9,
                          "note": "the same steps on one stream, plain launches: no overlap between steps"},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "device_copy": copy,
        "workloads": workloads,
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
