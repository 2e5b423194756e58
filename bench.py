#!/usr/bin/env python3
"""Benchmark of the bit-level compression hot path on one MI355X.

A step is one pass of the whole path over one batch at a partition boundary, at the
ResNet-50-style stage-boundary shape 64x256x56x56 (51.4 M elements, fp32):

    forward features : scheme M (multi-bit, k=4) compress  -> decompress
    backward gradient: scheme U (uniform,   k=8) compress  -> decompress

Inputs are synthetic (seeded) and already resident in HBM; two buffer sets alternate so
that nothing a call reads was produced or read by the previous ~1 GB of traffic (the
256 MB memory-side cache cannot serve a call's first read).  One JSON line is printed:
value = GB/s of uncompressed fp32 bytes through the step's four calls; the breakdown holds
each call's own rate and its algorithmic fraction of the 8 TB/s HBM peak; "roofline"
describes the dominant kernel from HIP-event stage timings taken inside this run;
"cells" holds every cell of the benchmark configuration as its description words it (per
tensor and per channel, 4/6/8 bits, fp32 and bf16, the gradient tensor, the forward widths
2/3/4) as single calls: cold median and minimum, warm (back-to-back) median, and the
algorithmic fraction of the HBM peak; "cpu_baseline" is the CPU oracle timed on the same
workload (one thread, as it stands), "cpu_baseline_all_cores" the same oracle functions run on
row chunks by a pool of processes; with --sweep, "cpu_cells" times the oracle (one thread, best
of three) on the small configurations as well.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--sweep]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E peak
METRIC = "compress / decompress GB/s of fp32 input and % of MI355X HBM peak"
SHAPE = (64, 256, 56, 56)
K_FWD, K_BWD = 4, 8
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_cfg4.txt")


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def alg_bytes(kernel, N, n, m, k, b_in=4, b_out=4):
    """Algorithmic HBM bytes one launch of a kernel must move."""
    if kernel == "range":
        return N * b_in
    if kernel == "quantize_pack":
        return N * b_in + (N * k + 7) // 8 + 4
    if kernel == "unpack_dequant":
        return (N * k + 7) // 8 + 4 + N * b_out
    if kernel == "mbq_encode":
        return N * b_in + ((n + 7) // 8) * m * k
    if kernel == "mbq_decode":
        return ((n + 7) // 8) * m * k + 4 * (k + 1) + N * b_out
    return 0


def read_traffic():
    """Measured HBM bytes per launch from committed rocprofv3 --pmc summaries, if present."""
    out = {}
    if os.path.exists(TRAFFIC_FILE):
        for line in open(TRAFFIC_FILE):
            line = line.split("#", 1)[0].strip()
            if "=" in line:
                k, v = line.split("=", 1)
                try:
                    out[k.strip()] = float(v)
                except ValueError:
                    pass
    return out


class Slot:
    """One set of device buffers for the four calls of a step."""

    def __init__(self, A, torch, act, grad, alpha, dm, du):
        self.act = act.clone()
        self.grad = grad.clone()
        self.alpha = alpha.clone()
        self.mh, self.mp, self.mw = A.alloc_outputs(dm, act.device)
        self.uh, self.up, self.uw = A.alloc_outputs(du, act.device)
        self.xhat_m = torch.empty(dm.n * dm.m, dtype=torch.float32, device=act.device)
        self.xhat_u = torch.empty(du.n * du.m, dtype=torch.float32, device=act.device)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--sweep", action="store_true",
                    help="time the cells of all five configurations (default: those of the benchmark configuration)")
    ap.add_argument("--sweep-json", default=None, help="also write the cells to this JSON file")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-cells", action="store_true",
                    help="skip the single-call cells (for profiler runs that want the timed steps' kernels only)")
    ap.add_argument("--graph", action="store_true",
                    help="replay a captured HIP graph of two steps instead of launching every call eagerly "
                         "(measured: no gain at this size, the kernels are long enough to hide the launches)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run plain device copies of the benchmark tensor's size (205,520,896 B read + "
                         "as many written per copy): the reference for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE")
    ap.add_argument("--calls", default=None, metavar="CFG:S:K:C:DTYPE[,...]",
                    help="only run compress + decompress of the named cells three times each, cold, e.g. "
                         "cfg3_act:M:3:0:f32,cfg4_grad:U:8:256:f32 (for rocprofv3 counter runs per configuration)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on one GPU only (the codec has no multi-GPU path); use --gpus 1")
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2311_05827_amd as A
    import synthetic_inputs as si

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    n, m = SHAPE[0], SHAPE[1] * SHAPE[2] * SHAPE[3]
    N = n * m

    if args.copy_calibration:
        src = torch.zeros(N, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        evict = torch.zeros(1 << 28, dtype=torch.float32, device=dev)
        for _ in range(10):
            evict.sum()          # read-only traffic between copies: the copy's source comes from HBM
            dst.copy_(src)
        torch.cuda.synchronize()
        log("copy calibration: 10 copies of %d bytes" % (N * 4))
        return

    if args.calls:
        evict = torch.zeros(1 << 28, dtype=torch.float32, device=dev)
        for cell in args.calls.split(","):
            name, scheme, k, C, dt = cell.split(":")
            k, C, bf = int(k), int(C), dt == "bf16"
            x_np = si.make(name)
            cn, cm = si.as_nm(x_np)
            x = torch.from_numpy(x_np.reshape(-1)).to(dev)
            x = x.to(torch.bfloat16) if bf else x
            tcode = A.BF16 if bf else A.F32
            if scheme == "U":
                d = A.make_desc(A.UNIFORM, k, cn, cm, channels=C, in_dtype=tcode, out_dtype=tcode)
                alpha = None
            else:
                d = A.make_desc(A.MBQ, k, cn, cm, t=1, in_dtype=tcode, out_dtype=tcode)
                alpha = A.accept_mbq_init(d, x)
            h, p, w = A.alloc_outputs(d, dev)
            out = torch.empty(cn * cm, dtype=x.dtype, device=dev)
            for _ in range(3):
                evict.sum()
                A.accept_compress(d, x, alpha_prev=alpha, header=h, payload=p, workspace=w)
                evict.sum()
                A.accept_decompress(d, h, p, out=out)
            torch.cuda.synchronize()
            log("calls: %s done" % cell)
        return

    t0 = time.time()
    act_np = si.make("cfg4_act")
    grad_np = si.make("cfg4_grad")
    log("inputs generated in %.1fs" % (time.time() - t0))
    act = torch.from_numpy(act_np.reshape(-1)).to(dev)
    grad = torch.from_numpy(grad_np.reshape(-1)).to(dev)

    dm = A.make_desc(A.MBQ, K_FWD, n, m, t=1)
    du = A.make_desc(A.UNIFORM, K_BWD, n, m)
    alpha0 = A.accept_mbq_init(dm, act)  # residue initialisation on the GPU
    torch.cuda.synchronize()

    slots = [Slot(A, torch, act, grad, alpha0, dm, du) for _ in range(2)]

    def compress_m(s):
        A.accept_compress(dm, s.act, alpha_prev=s.alpha, header=s.mh, payload=s.mp, workspace=s.mw)

    def decompress_m(s):
        A.accept_decompress(dm, s.mh, s.mp, out=s.xhat_m)

    def compress_u(s):
        A.accept_compress(du, s.grad, header=s.uh, payload=s.up, workspace=s.uw)

    def decompress_u(s):
        A.accept_decompress(du, s.uh, s.up, out=s.xhat_u)

    def step(j):
        a, b = slots[j % 2], slots[(j + 1) % 2]
        compress_m(a)      # forward features of this batch
        decompress_m(b)    # receiver side: a payload produced a whole step ago
        compress_u(a)      # backward gradients
        decompress_u(b)

    # fill both slots so that every decompress has a valid payload
    for s in slots:
        compress_m(s)
        compress_u(s)
    torch.cuda.synchronize()

    for j in range(args.warmup):
        step(j)
    torch.cuda.synchronize()
    use_graph = args.graph
    graph = None
    if use_graph:
        # two consecutive steps (slot parity 0 and 1) captured once; K steps = K/2 replays (+ one
        # eager step when K is odd).  The graph holds the library's kernels only.
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step(0); step(1)
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                step(0); step(1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    if use_graph:
        for j in range(args.steps // 2):
            graph.replay()
        if args.steps % 2:
            step(0)
    else:
        for j in range(args.steps):
            step(j)
    ev1.record()
    torch.cuda.synchronize()
    ms_per_step = ev0.elapsed_time(ev1) / args.steps
    step_bytes = 4 * N * 4
    value = step_bytes / (ms_per_step * 1e-3) / 1e9

    # per-call rates on cold inputs, two ways.  "ms": the two calls before the timed one are
    # other calls of the step (they write up to 411 MB, and those dirty lines drain to HBM while
    # the timed call runs).  "ms_clean": a read-only sweep of 1 GiB precedes the timed call, so
    # the call's own traffic is all there is.
    sweep_buf = torch.zeros(1 << 28, dtype=torch.float32, device=dev)

    def time_call(fn, other, clean):
        for j in range(3):
            fn(slots[j % 2]); other(slots[(j + 1) % 2])
        torch.cuda.synchronize()
        tot = 0.0
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = max(10, args.steps // 8)
        for j in range(reps):
            if clean:
                sweep_buf.sum()
            else:
                other(slots[(j + 1) % 2])
                other(slots[j % 2])
            e0.record()
            fn(slots[j % 2])
            e1.record()
            e1.synchronize()
            tot += e0.elapsed_time(e1)
        return tot / reps

    calls = {
        "mbq_compress_k4": (compress_m, decompress_u, alg_bytes("mbq_encode", N, n, m, K_FWD)),
        "mbq_decompress_k4": (decompress_m, compress_u, alg_bytes("mbq_decode", N, n, m, K_FWD)),
        "uniform_compress_k8": (compress_u, decompress_m,
                                alg_bytes("range", N, n, m, K_BWD) + alg_bytes("quantize_pack", N, n, m, K_BWD)),
        "uniform_decompress_k8": (decompress_u, compress_m, alg_bytes("unpack_dequant", N, n, m, K_BWD)),
    }
    breakdown = {}
    for name, (fn, other, ab) in calls.items():
        ms = time_call(fn, other, False)
        ms_clean = time_call(fn, other, True)
        breakdown[name] = {
            "ms": round(ms, 5),
            "input_GBps": round(N * 4 / (ms * 1e-3) / 1e9, 1),
            "alg_bytes": ab,
            "alg_hbm_frac": round(ab / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
            "ms_clean": round(ms_clean, 5),
            "input_GBps_clean": round(N * 4 / (ms_clean * 1e-3) / 1e9, 1),
            "alg_hbm_frac_clean": round(ab / (ms_clean * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
        }

    # per-kernel durations from HIP events recorded by the library around each launch
    stage_ms = {}
    reps = max(10, args.steps // 4)
    for j in range(reps):
        a, b = slots[j % 2], slots[(j + 1) % 2]
        for nm_, ms in A.accept_compress_timed(dm, a.act, a.alpha, a.mh, a.mp, a.mw):
            stage_ms.setdefault(nm_, []).append(ms)
        for nm_, ms in A.accept_decompress_timed(dm, b.mh, b.mp, b.xhat_m):
            stage_ms.setdefault(nm_, []).append(ms)
        for nm_, ms in A.accept_compress_timed(du, a.grad, None, a.uh, a.up, a.uw):
            stage_ms.setdefault(nm_, []).append(ms)
        for nm_, ms in A.accept_decompress_timed(du, b.uh, b.up, b.xhat_u):
            stage_ms.setdefault(nm_, []).append(ms)
    kernels = {}
    kbits = {"range": K_BWD, "quantize_pack": K_BWD, "unpack_dequant": K_BWD, "mbq_encode": K_FWD,
             "mbq_decode": K_FWD}
    for nm_, v in stage_ms.items():
        avg = sum(v) / len(v)
        ab = alg_bytes(nm_, N, n, m, kbits.get(nm_, 0))
        kernels[nm_] = {"avg_ms": round(avg, 5), "alg_bytes": ab,
                        "GBps": round(ab / (avg * 1e-3) / 1e9, 1) if ab else None}
    # the longest kernel of the path in the rocprofv3 trace of this command (profiles/): the MBQ encoder
    dominant = "mbq_encode"
    traffic = read_traffic().get(dominant)
    roofline = {
        "bound": "hbm",
        "kernel": dominant,
        "achieved": kernels[dominant]["GBps"],
        "peak": HBM_PEAK_GBPS,
        "unit": "GB/s",
        "frac": round(kernels[dominant]["GBps"] / HBM_PEAK_GBPS, 4),
        "traffic": traffic,
        "alg_bytes_per_launch": kernels[dominant]["alg_bytes"],
        "avg_launch_ms": kernels[dominant]["avg_ms"],
        "kernels": kernels,
    }

    # the same for whole calls (every kernel the call launches: range + quantize_pack, encode +
    # finalize), from the in-mix timings above
    call_roofline = {name: {"bound": "hbm", "achieved": round(v["alg_bytes"] / (v["ms"] * 1e-3) / 1e9, 1),
                            "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": v["alg_hbm_frac"]}
                     for name, v in breakdown.items()}

    cpu = cpu_all = None
    if not args.no_cpu:
        cpu = cpu_baseline(np, act_np, grad_np, n, m)
        cpu_all = cpu_baseline_all_cores(np, act_np, grad_np, n, m)

    cells = [] if args.no_cells else run_cells(A, torch, si, ALL_CELLS if args.sweep else CFG4_CELLS)
    cpu_small = cpu_cells(np, si) if args.sweep and not args.no_cpu else None
    if args.sweep_json:
        with open(args.sweep_json, "w") as f:
            json.dump(cells, f, indent=1)

    out = {
        "metric": METRIC,
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": "cfg4 stage-boundary tensor 64x256x56x56 fp32 (51.4M elems): per step MBQ k=4 compress+"
                        "decompress of post-ReLU features and uniform k=8 compress+decompress of gradients",
            "elements": N,
            "uncompressed_bytes_per_step": step_bytes,
            "cold_inputs": "two buffer sets alternate; decompress reads a payload written one step earlier",
            "launch": "HIP graph of two steps, replayed" if use_graph else "eager launches",
        },
        "hbm_frac_of_value": round(value / HBM_PEAK_GBPS, 4),
        "breakdown": breakdown,
        "roofline": roofline,
        "roofline_calls": call_roofline,
        "cells": cells,
        "cpu_baseline": cpu,
        "cpu_baseline_all_cores": cpu_all,
        "cpu_cells": cpu_small,
    }
    print(json.dumps(out), flush=True)


def _pool_uniform_max(args):
    from oracle import accept_oracle as orc
    lo, hi = args
    return float(orc.uniform_range(_G["grad"][lo:hi], hi - lo, _G["m"])[0])


def _pool_uniform_pack(args):
    from oracle import accept_oracle as orc
    lo, hi, r = args
    import numpy as np
    rows = hi - lo
    q = orc.uniform_quantize(_G["grad"][lo:hi], np.array([r], np.float32), K_BWD, rows, _G["m"])
    pl = orc.pack_stream(orc.uniform_codes(q, K_BWD), K_BWD)
    _G["upay"][lo * _G["m"] * K_BWD // 8: hi * _G["m"] * K_BWD // 8] = pl
    return pl.size


def _pool_uniform_unpack(args):
    from oracle import accept_oracle as orc
    lo, hi, s = args
    import numpy as np
    rows = hi - lo
    pl = _G["upay"][lo * _G["m"] * K_BWD // 8: hi * _G["m"] * K_BWD // 8]
    xh = orc.uniform_decompress(np.array([s], "<f4").tobytes(), pl, K_BWD, rows, _G["m"])
    return float(xh[0])


def _pool_mbq_encode(args):
    from oracle import accept_oracle as orc
    lo, hi = args
    rows = hi - lo
    x = _G["act"][lo:hi]
    code = orc.mbq_assign(x, _G["alpha"])
    pl = orc.mbq_pack(code, K_FWD, rows, _G["m"])
    _G["mpay"][(lo // 8) * _G["m"] * K_FWD: (hi // 8) * _G["m"] * K_FWD] = pl
    return orc.mbq_stats(x, code, K_FWD)


def _pool_mbq_decode(args):
    from oracle import accept_oracle as orc
    lo, hi, header = args
    rows = hi - lo
    pl = _G["mpay"][(lo // 8) * _G["m"] * K_FWD: (hi // 8) * _G["m"] * K_FWD]
    return float(orc.mbq_decompress(header, pl, K_FWD, rows, _G["m"])[0])


_G = {}


def cpu_baseline_all_cores(np, act_np, grad_np, n, m):
    """The oracle's own functions on chunks of eight batch rows, run by a pool of processes (the
    chunks' bit streams and bit planes concatenate; the range and the least-squares sums are
    combined between the passes).  Forked workers see the tensors without copying them."""
    import multiprocessing as mp
    from oracle import accept_oracle as orc
    cores = min(16, os.cpu_count() or 1)
    shm = mp.get_context("fork")
    _G.update(act=act_np.reshape(n, m), grad=grad_np.reshape(n, m), m=m)
    _G["upay"] = np.frombuffer(mp.RawArray("B", n * m * K_BWD // 8), dtype=np.uint8)
    _G["mpay"] = np.frombuffer(mp.RawArray("B", ((n + 7) // 8) * m * K_FWD), dtype=np.uint8)
    _G["alpha"], _ = orc.mbq_residue_init(_G["act"][:8], K_FWD)  # any plausible previous alpha (not timed)
    chunks = [(lo, min(lo + 8, n)) for lo in range(0, n, 8)]
    N = n * m
    with shm.Pool(cores) as pool:
        pool.map(_pool_uniform_max, chunks[:cores])  # start the workers before the clock
        t0 = time.perf_counter()
        # forward features: assign + pack + sums per chunk, then the update; decode per chunk
        stats = pool.map(_pool_mbq_encode, chunks)
        G = sum(s[0] for s in stats); h = sum(s[1] for s in stats)
        Sb = sum(s[2] for s in stats); Sx = sum(s[3] for s in stats)
        alpha_t, _ = orc.mbq_alpha_update(_G["alpha"], G, h, 1, N)
        mq = orc.mbq_mean_error(alpha_t, Sb, Sx, N)
        header = np.concatenate([alpha_t, np.array([mq], np.float32)]).astype("<f4").tobytes()
        pool.map(_pool_mbq_decode, [(lo, hi, header) for lo, hi in chunks])
        # backward gradients: range per chunk, then quantize + pack per chunk; decode per chunk
        c = np.float32(max(pool.map(_pool_uniform_max, chunks)))
        s_, r_ = orc.uniform_scale(np.array([c], np.float32), K_BWD)
        pool.map(_pool_uniform_pack, [(lo, hi, float(r_[0])) for lo, hi in chunks])
        pool.map(_pool_uniform_unpack, [(lo, hi, float(s_[0])) for lo, hi in chunks])
        dt = time.perf_counter() - t0
    nbytes = 4 * N * 4
    log("cpu oracle, %d processes: %.2fs for the same four calls" % (cores, dt))
    return {
        "value": round(nbytes / dt / 1e9, 4),
        "unit": "GB/s",
        "cores": cores,
        "kind": "oracle functions on 8-row chunks, process pool",
        "sample": "the whole workload: all %d batch rows of the same two tensors, the same four calls" % n,
        "seconds": round(dt, 3),
    }


def cpu_baseline(np, act_np, grad_np, n, m):
    """The oracle as it stands, single thread, on the same two tensors (all 64 batch rows: about
    10 s of CPU work on the GPU machine's host)."""
    from oracle import accept_oracle as orc
    rows = n
    a = np.ascontiguousarray(act_np.reshape(n, m)[:rows])
    g = np.ascontiguousarray(grad_np.reshape(n, m)[:rows])
    t0 = time.perf_counter()
    alpha0, _ = orc.mbq_residue_init(a, K_FWD)
    t_init = time.perf_counter() - t0
    t0 = time.perf_counter()
    mh, mp = orc.mbq_compress(a, K_FWD, rows, m, alpha0, 1)
    orc.mbq_decompress(mh, mp, K_FWD, rows, m)
    uh, up = orc.uniform_compress(g, K_BWD, rows, m)
    orc.uniform_decompress(uh, up, K_BWD, rows, m)
    dt = time.perf_counter() - t0
    nbytes = 4 * rows * m * 4
    log("cpu oracle: %.2fs for %d elements x 4 calls (init %.2fs not counted)" % (dt, rows * m, t_init))
    return {
        "value": round(nbytes / dt / 1e9, 4),
        "unit": "GB/s",
        "cores": 1,
        "kind": "oracle",
        "sample": "the whole workload: all %d batch rows (%d elements) of the same two tensors, the same four "
                  "calls, NumPy oracle, single thread" % (rows, rows * m),
        "seconds": round(dt, 3),
    }


def cpu_cells(np, si):
    """The oracle, single thread, best of three, on the small configurations (1, 2, 5) and one
    width of configuration 3: seconds per compress and per decompress call, and GB/s of input."""
    from oracle import accept_oracle as orc
    plans = [("cfg1_act", "U", 8), ("cfg1_act", "M", 2), ("cfg1_act", "M", 4), ("cfg2_grad", "U", 4),
             ("cfg2_grad", "U", 2), ("cfg5_hidden", "U", 3), ("cfg5_hidden", "U", 7), ("cfg5_hidden", "M", 3),
             ("cfg5_grad", "U", 5), ("cfg3_act", "U", 4), ("cfg3_act", "M", 3)]
    out = []
    log("%-12s %-2s %1s | %10s %10s | %9s %9s" % ("config", "S", "k", "comp_ms", "dec_ms", "comp_GB/s", "dec_GB/s"))
    for name, scheme, k in plans:
        x = si.make(name)
        n, m = si.as_nm(x)
        if scheme == "U":
            comp = lambda: orc.uniform_compress(x, k, n, m)
            deco = lambda hp: orc.uniform_decompress(hp[0], hp[1], k, n, m)
        else:
            alpha, _ = orc.mbq_residue_init(x, k)
            comp = lambda: orc.mbq_compress(x, k, n, m, alpha, 1)
            deco = lambda hp: orc.mbq_decompress(hp[0], hp[1], k, n, m)
        tc = td = 1e30
        for _ in range(3):
            t0 = time.perf_counter(); hp = comp(); tc = min(tc, time.perf_counter() - t0)
            t0 = time.perf_counter(); deco(hp); td = min(td, time.perf_counter() - t0)
        nb = n * m * 4
        c = dict(config=name, scheme=scheme, k=k, cores=1, compress_s=round(tc, 5), decompress_s=round(td, 5),
                 compress_in_GBps=round(nb / tc / 1e9, 4), decompress_out_GBps=round(nb / td / 1e9, 4))
        out.append(c)
        log("%-12s %-2s %1d | %10.2f %10.2f | %9.3f %9.3f" % (name, scheme, k, tc * 1e3, td * 1e3,
                                                           c["compress_in_GBps"], c["decompress_out_GBps"]))
    return out


class CellTimer:
    """Single-call timings of one (tensor, scheme, k, channels, dtype) cell."""

    def __init__(self, A, torch, dev):
        self.A, self.torch, self.dev = A, torch, dev
        self.scratch = torch.zeros(1 << 28, dtype=torch.float32, device=dev)  # 1 GiB, read between cold calls

    def _cold(self, fn, reps):
        torch = self.torch
        fn(); torch.cuda.synchronize()
        t = []
        for _ in range(reps):
            self.scratch.sum()          # read-only 1 GiB: nothing of the call's data is left in a cache
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(); fn(); e1.record(); e1.synchronize()
            t.append(e0.elapsed_time(e1))
        t.sort()
        return t[len(t) // 2], t[0]

    def _warm(self, fn, reps):
        torch = self.torch
        fn(); torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record(); e1.synchronize()
        return e0.elapsed_time(e1) / reps

    def cell(self, name, x32, x16, n, m, scheme, k, C, bf, reps=50):
        A, torch, dev = self.A, self.torch, self.dev
        N = n * m
        x = x16 if bf else x32
        b = 2 if bf else 4
        tcode = A.BF16 if bf else A.F32
        layout = {"b": A.LAYOUT_BATCH, "u": A.LAYOUT_UNENCODED}.get(scheme[1:], A.LAYOUT_PACKED)
        if scheme[0] == "U":
            d = A.make_desc(A.UNIFORM, k, n, m, channels=C, in_dtype=tcode, out_dtype=tcode, layout=layout,
                            rounding=A.ROUND_STOCHASTIC if scheme == "Us" else A.ROUND_NEAREST_EVEN, seed=7)
            alpha = None
        else:
            d = A.make_desc(A.MBQ, k, n, m, t=1, in_dtype=tcode, out_dtype=tcode, layout=layout)
            alpha = A.accept_mbq_init(d, x)
        # algorithmic bytes of the call: the input (twice for scheme U: range pass, quantize pass),
        # the header and the payload of this layout one way; the same plus the output back
        hb, pb = A.accept_packed_size(d)
        cb = (2 if scheme[0] == "U" else 1) * N * b + hb + pb
        db = hb + pb + N * b
        h, p, w = A.alloc_outputs(d, dev)
        out = torch.empty(N, dtype=torch.bfloat16 if bf else torch.float32, device=dev)
        comp = lambda: A.accept_compress(d, x, alpha_prev=alpha, header=h, payload=p, workspace=w)
        deco = lambda: A.accept_decompress(d, h, p, out=out)
        tc, tc_min = self._cold(comp, reps)
        td, td_min = self._cold(deco, reps)
        tcw, tdw = self._warm(comp, reps), self._warm(deco, reps)
        frac = lambda nbytes, ms: round(nbytes / ms / 1e6 / HBM_PEAK_GBPS, 4)
        # scheme U reads its input twice; the tensors here fit the memory-side cache, so the second
        # read need not reach HBM: the same fraction priced with one read is the lower bound
        extra = {}
        if scheme[0] == "U":
            extra = dict(compress_alg_bytes_one_read=cb - N * b, compress_alg_frac_one_read=frac(cb - N * b, tc))
        return dict(config=name, scheme=scheme, k=k, channels=C, dtype="bf16" if bf else "f32",
                    compress_us=round(tc * 1e3, 2), compress_us_min=round(tc_min * 1e3, 2),
                    compress_us_warm=round(tcw * 1e3, 2),
                    decompress_us=round(td * 1e3, 2), decompress_us_min=round(td_min * 1e3, 2),
                    decompress_us_warm=round(tdw * 1e3, 2),
                    compress_in_GBps=round(N * b / tc / 1e6, 1), decompress_out_GBps=round(N * b / td / 1e6, 1),
                    compress_alg_bytes=cb, decompress_alg_bytes=db,
                    compress_alg_frac=frac(cb, tc), decompress_alg_frac=frac(db, td),
                    compress_alg_frac_best=frac(cb, tc_min), decompress_alg_frac_best=frac(db, td_min), **extra)


CFG4_CELLS = [
    ("cfg4_act", [("U", k, c, b) for k in (4, 6, 8) for c in (0, 256) for b in (False, True)]
     + [("M", k, 0, False) for k in (2, 3, 4)] + [("M", 4, 0, True)]),
    ("cfg4_grad", [("U", k, c, False) for k in (4, 6, 8) for c in (0, 256)]),
]
ALL_CELLS = [
    ("cfg1_act", [("U", 8, 0, False), ("M", 2, 0, False), ("M", 3, 0, False), ("M", 4, 0, False)]),
    ("cfg2_grad", [("U", 4, 0, False), ("U", 2, 0, False)]),
    ("cfg3_act", [("U", k, 0, False) for k in range(2, 9)] + [("M", k, 0, False) for k in (2, 3, 4)]),
    ("cfg4_act", CFG4_CELLS[0][1] + [("M", 2, 0, True), ("Mu", 4, 0, False)]),  # Mu: one byte per binary base
    ("cfg4_grad", CFG4_CELLS[1][1]
     + [("Us", k, 0, False) for k in (4, 8)]          # Us: stochastic rounding
     + [("Ub", 4, 0, False), ("Uu", 4, 0, False)]),   # Ub: batch-pair layout, Uu: one byte per code
    ("cfg5_hidden", [("U", k, 0, False) for k in (3, 5, 6, 7)] + [("M", 3, 0, False)]),
    ("cfg5_grad", [("U", k, 0, False) for k in (3, 5, 6, 7)]),
]


def run_cells(A, torch, si, plans, extra_views=True):
    """Time the cells of `plans`; table on stderr, list of dicts returned."""
    dev = torch.device("cuda:0")
    ct = CellTimer(A, torch, dev)
    cells = []
    log("%-12s %-2s %1s %4s %5s | %8s %8s %8s %6s | %8s %8s %8s %6s" % (
        "config", "S", "k", "C", "dtype", "comp_us", "min", "warm", "alg%", "dec_us", "min", "warm", "alg%"))

    def show(c):
        log("%-12s %-2s %1d %4d %5s | %8.1f %8.1f %8.1f %5.1f%% | %8.1f %8.1f %8.1f %5.1f%%" % (
            c["config"], c["scheme"], c["k"], c["channels"], c["dtype"], c["compress_us"], c["compress_us_min"],
            c["compress_us_warm"], 100 * c["compress_alg_frac"], c["decompress_us"], c["decompress_us_min"],
            c["decompress_us_warm"], 100 * c["decompress_alg_frac"]))

    for name, cases in plans:
        x_np = si.make(name)
        n, m = si.as_nm(x_np)
        x32 = torch.from_numpy(x_np.reshape(-1)).to(dev)
        x16 = x32.to(torch.bfloat16)
        for scheme, k, C, bf in cases:
            c = ct.cell(name, x32, x16, n, m, scheme, k, C, bf)
            cells.append(c); show(c)
        if extra_views and name == "cfg4_grad":
            # the same bytes read as a channels-last tensor (64*3136 rows of 256 channels): one range
            # per element of a row, the geometry the column range pass is for
            c = ct.cell("cfg4_grad_nhwc", x32, x16, n * (m // 256), 256, "U", 8, 256, False)
            cells.append(c); show(c)
        del x32, x16
    return cells


if __name__ == "__main__":
    main()
