#!/usr/bin/env python3
"""Benchmark of the RTN weight-only quantised linear path on one MI355X.

Workload: the four linear modules of a Llama-3.1-8B-shaped
Transformer layer (Section 4: QKV 4096->6144, attention output 4096->4096, gate_up
4096->28672, down 14336->4096), symmetric RTN int4 with group 128 and fp16 scales
(Section 2.2), fp16 activations at the token-generation batch sizes M = 1, 2, 4, 8, 16
(Sections 1, 5).  Weights ~ N(0, 0.02), activations ~ N(0, 1), seeded, synthetic.

One step = one pass of the hot path over one batch of input: for every M, the layer's four
modules through rtn_layer_forward (20 fused dequantise-GEMMs).  Every pass streams a different
copy of the packed layer (enough copies to exceed twice the 256 MB Infinity Cache), as token
generation does when it walks a model's layers, so the weights come from HBM, not from cache.
The load-time quantise/pack pass (Section 5) runs once during set-up, is checked to reproduce,
and its throughput is reported in the "quantize" object; it is not inside the timed steps,
which measure the metric itself: weight-stream GB/s of the linear layers.

Prints one JSON line: metric, value (GB/s of packed weights and scales streamed, whole job), unit, n_gpus, steps, warmup,
ms_per_step, dtype, data, config, plus `roofline` (the dominant kernel against the 8 TB/s HBM peak: algorithmic bytes per
launch over the measured average launch duration, and the HBM traffic per launch from hardware counters), `cpu_baseline`
(the CPU oracle timed on a bounded sample of the same workload) and `quantize` (load-time pass throughput).
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

HBM_PEAK_GBS = 8000.0
BATCHES = (1, 2, 4, 8, 16)
BITS, GROUP = 4, 128
CACHE_BYTES = 256e6
# HBM bytes per launch of the dominant kernel come from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this very
# command, scaled by a copy kernel of known size; the committed summary of those runs carries the figure on a line
# "traffic_bytes_per_launch: <n>", which is read at run time (null if the summary is not there).
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "skinny_mfma_llama8b_w4a16_hbm_traffic.txt")
W8_BATCHES = (1, 4, 16, 64)
WARM_MS = float(os.environ.get("RTN_BENCH_WARM_MS", "200"))      # untimed work before each event-bracketed measurement
SETTLE_MS = float(os.environ.get("RTN_BENCH_SETTLE_MS", "300"))  # the step graphs run this long, untimed, before the warm-up steps (clocks)


def _measured_traffic():
    try:
        for line in open(TRAFFIC_PROFILE):
            if line.startswith("traffic_bytes_per_launch:"):
                return int(float(line.split(":", 1)[1].split()[0]))
    except OSError:
        pass
    return None


def _bracket_us(torch, np, run, samples):
    """Microseconds one run() takes on the GPU: a pair of events brackets enough back-to-back runs for about 4 ms of work,
    so that the fixed cost of the first submission (some 10 us, which the bracket cannot avoid) stays under half a percent;
    median of `samples` brackets."""
    run()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    run()
    e1.record()
    torch.cuda.synchronize()
    once_ms = max(e0.elapsed_time(e1), 1e-3)
    rounds = int(min(64, max(1, np.ceil(4.0 / once_ms))))
    for _ in range(int(min(256, np.ceil(WARM_MS / once_ms)))):      # clocks settle before anything is timed
        run()
    ts = []
    for _ in range(samples):
        e0.record()
        for _ in range(rounds):
            run()
        e1.record()
        torch.cuda.synchronize()
        ts.append(e0.elapsed_time(e1) * 1e3 / rounds)
    return float(np.median(ts))


def _time_linear(rtn, torch, np, A, qws, sc, bits, g, cfg, ws, reps=3, graph=True):
    """Microseconds per rtn_linear launch: launches rotate over distinct weight copies, replayed as a HIP graph
    (or issued directly, graph=False: for counter collection)."""
    M, K = A.shape
    N = sc.shape[0]
    out = torch.empty((M, N), dtype=torch.float16, device=A.device)
    for q in qws[:2]:
        rtn.rtn_linear(A, q, sc, bits, g, out=out, workspace=ws, cfg=cfg)
    torch.cuda.synchronize()

    def issue():
        for _ in range(reps):
            for q in qws:
                rtn.rtn_linear(A, q, sc, bits, g, out=out, workspace=ws, cfg=cfg)

    if graph:
        cg = torch.cuda.CUDAGraph()
        st = torch.cuda.Stream()
        with torch.cuda.stream(st):
            with torch.cuda.graph(cg, stream=st):
                issue()
        run = cg.replay
    else:
        run = issue
    n = reps * len(qws)
    return _bracket_us(torch, np, run, 5 if graph else 1) / n


def _read_ceiling_us(rtn, torch, np, nbytes, pool, sink, kib_options=(2, 4, 8)):
    """Microseconds a plain read kernel (rtn_bench_read_stream) takes per launch on nbytes, under the protocol of the
    linear launches: HIP-graph replay of back-to-back launches that rotate over distinct regions of `pool` (>= 600 MB in
    total, or the pool), median of 5 replays; the best of the KiB-per-wavefront settings tried."""
    nbytes = (int(nbytes) + 1023) // 1024 * 1024
    if nbytes > pool.numel():
        raise ValueError(f"read ceiling: {nbytes} bytes asked of a pool of {pool.numel()}")
    copies = max(1, min(int(pool.numel() // nbytes), max(2, int(np.ceil(600e6 / nbytes)))))
    views = [pool[c * nbytes:(c + 1) * nbytes] for c in range(copies)]
    reps = 3
    best = None
    for kib in kib_options:
        def issue():
            for _ in range(reps):
                for v in views:
                    rtn.rtn_bench_read_stream(v, nbytes, kib, sink)
        issue()
        torch.cuda.synchronize()
        cg = torch.cuda.CUDAGraph()
        st = torch.cuda.Stream()
        with torch.cuda.stream(st):
            with torch.cuda.graph(cg, stream=st):
                issue()
        t = _bracket_us(torch, np, cg.replay, 5) / (reps * copies)
        best = t if best is None else min(best, t)
    return best


def _ceiling_pool(torch, dev, nbytes=1 << 30):
    pool = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    pool.fill_(1)
    return pool, torch.zeros(16, dtype=torch.uint8, device=dev)


def report_ceiling(args, rtn, synth, torch, np, dev) -> int:
    """The read-stream ceiling: a plain 16-byte-per-lane read kernel timed on buffers of exactly the packed size (codes +
    scales) of every matrix of every workload, and on 512 MB, under the same graph-replay protocol as the linear launches."""
    pool, sink = _ceiling_pool(torch, dev, 2 << 30)        # the largest matrix here (405B gate_up at 8 bit) is 1.75 GB
    print("# plain read kernel (rtn_bench_read_stream): us per launch, HIP-graph replay, launches rotate over >= 600 MB of a 1 GiB "
          "buffer; best of 2 / 4 / 8 KiB per wavefront; sizes = packed codes + scales of each matrix")
    t512 = _read_ceiling_us(rtn, torch, np, 512e6, pool, sink)
    print(f"512 MB: {t512:8.2f} us  {512e6 / t512 / 1e3:7.0f} GB/s  {512e6 / t512 / 80e3:5.1f} % of 8 TB/s")
    for fam, shapes in (("8b", synth.LLAMA_8B), ("70b", synth.LLAMA_70B), ("405b", synth.LLAMA_405B)):
        for label, bits_of in (("int4 group 128", lambda n: 4), ("int8 per-channel", lambda n: 8),
                               ("selective (o, down int8 per-channel; qkv, gate_up int4 group 128)", lambda n: 8 if n in ("o", "down") else 4)):
            if label.startswith("selective") and fam != "405b":
                continue
            tot_b, tot_t = 0.0, 0.0
            for name, (K, N) in shapes.items():
                bits = bits_of(name)
                nbytes = N * K * bits // 8 + (N * (K // 128) * 2 if bits == 4 else N * 2)
                t = _read_ceiling_us(rtn, torch, np, nbytes, pool, sink)
                tot_b += nbytes
                tot_t += t
                print(f"{fam:5s} {label:18.18s} {name:8s} {K:6d}->{N:6d}  {nbytes / 1e6:8.2f} MB  {t:8.2f} us  {nbytes / t / 1e3:7.0f} GB/s  "
                      f"{nbytes / t / 80e3:5.1f} % of 8 TB/s", flush=True)
            print(f"{fam:5s} {label}: layer set {tot_b / 1e6:.1f} MB in {tot_t:.2f} us = {tot_b / tot_t / 1e3:.0f} GB/s = "
                  f"{tot_b / tot_t / 80e3:.1f} % of 8 TB/s: the ceiling of four dependent weight-streaming launches on these sizes", flush=True)
    return 0


def report(args, rtn, synth, torch, np, dev) -> int:
    """Per (matrix, M): launch time, weight-stream GB/s, % of the 8 TB/s HBM peak, useful TFLOP/s; and per layer set."""
    shapes = {"8b": synth.LLAMA_8B, "70b": synth.LLAMA_70B, "405b": synth.LLAMA_405B}[args.report]
    std = {"8b": 0.02, "70b": 0.02, "405b": 0.01}[args.report]
    Ms = [int(x) for x in args.batches.split(",")]
    ws = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
    tot = {M: 0.0 for M in Ms}
    totb = 0
    ceil_t = 0.0
    largest = max(N * K for K, N in shapes.values()) + (2 << 20)          # an int8 matrix plus its scales
    pool, sink = _ceiling_pool(torch, dev, max(1 << 30, (largest + 1023) // 1024 * 1024))
    what = ("selective precision: qkv and gate_up int4 group 128, o and down int8 per-channel" if args.selective
            else f"int{args.bits} {'group 128' if args.bits == 4 else 'per-channel'}")
    print(f"# {args.report} shapes, {what}; launches rotate over >= 600 MB of "
          f"distinct packed copies; HIP-graph replay; times include the ~1.5 us dispatch gap")
    for idx, (name, (K, N)) in enumerate(shapes.items()):
        bits = 8 if args.selective and name in ("o", "down") else (4 if args.selective else args.bits)
        g = 128 if bits == 4 else 0
        W = synth.normal_weight(N, K, std, idx, dev)
        qw, sc = rtn.rtn_quantize(W, bits, g)
        del W
        nbytes = qw.numel() + sc.numel() * 2
        totb += nbytes
        ceil_t += _read_ceiling_us(rtn, torch, np, nbytes, pool, sink)
        L = max(2, int(np.ceil(600e6 / nbytes)))
        qws = [qw] + [qw.clone() for _ in range(L - 1)]
        for M in Ms:
            A = synth.activation(M, K, 100 + M, dev)
            t = _time_linear(rtn, torch, np, A, qws, sc, bits, g, None, ws, graph=not args.no_graph)
            tot[M] += t
            t_hot = _time_linear(rtn, torch, np, A, qws[:1], sc, bits, g, None, ws, reps=12) if args.hot else None
            plan = rtn.rtn_linear_query(M, N, K, bits, g)
            line = (f"{name:8s} {'int' + str(bits) if args.selective else '':4s} {K:6d}->{N:6d} M={M:3d}  {t:8.2f} us  {nbytes / t / 1e3:7.0f} GB/s  "
                    f"{nbytes / t / 80e3:5.1f} %  {2.0 * M * N * K / t / 1e6:7.2f} TFLOP/s  ")
            if plan["path"] == 3:
                line += (f"wide {plan['waves_n']} waves x {16 * plan['m_rows16']}x{16 * plan['n_tiles16']} split {plan['split_k']}")
            elif plan["path"] == 4:
                line += f"tile kernel (128 or 256 rows x 256 columns per workgroup) split {plan['split_k']}"
            else:
                line += f"skinny {plan['waves_n']}x{plan['waves_k']} split {plan['split_k']} rows16 {plan['m_rows16']}"
            if t_hot is not None:
                line += f"  | one buffer (cache-hot) {t_hot:7.2f} us"
            if args.compare_paths and M <= 4:
                c2 = dict(path=2, waves_n=plan["waves_n"], waves_k=plan["waves_k"], split_k=plan["split_k"])
                try:
                    line += f"  | v_dot2 variant {_time_linear(rtn, torch, np, A, qws, sc, bits, g, c2, ws):8.2f} us"
                except rtn.RtnError:
                    line += "  | v_dot2 variant n/a"
            print(line, flush=True)
        del qws, qw
    for M in Ms:
        print(f"layer set M={M:3d}: {tot[M]:8.2f} us  {totb / tot[M] / 1e3:7.0f} GB/s  {totb / tot[M] / 80e3:5.1f} % of 8 TB/s"
              f"  ({100.0 * ceil_t / tot[M]:5.1f} % of what a plain read kernel reaches on buffers of these four sizes: {ceil_t:.2f} us)")
    return 0


def report_quantize(args, rtn, synth, torch, np, dev) -> int:
    """rtn_quantize throughput per matrix: bytes = fp16 read + packed codes and scales written."""
    shapes = {"8b": synth.LLAMA_8B, "70b": synth.LLAMA_70B, "405b": synth.LLAMA_405B}[args.report_quantize]
    print(f"# rtn_quantize on {args.report_quantize} shapes; bytes = 2 B read + packed codes + scales written per weight; "
          f"HIP events around 10 back-to-back calls")
    for bits, g in ((4, 128), (4, 0), (8, 128), (8, 0)):
        for idx, (name, (K, N)) in enumerate(shapes.items()):
            W = synth.normal_weight(N, K, 0.02, idx, dev)
            q, s = rtn.rtn_quantize(W, bits, g)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            ts = []
            for _ in range(3):
                e0.record()
                for _ in range(10):
                    rtn.rtn_quantize(W, bits, g, out=(q, s))
                e1.record()
                torch.cuda.synchronize()
                ts.append(e0.elapsed_time(e1) * 1e2)
            t = float(np.median(ts))
            nbytes = W.numel() * 2 + q.numel() + s.numel() * 2
            print(f"int{bits} {'g=128' if g else 'per-channel':11s} {name:8s} {K:6d}->{N:6d}  {t:8.1f} us  {nbytes / t / 1e3:6.0f} GB/s  "
                  f"{nbytes / t / 80e3:5.1f} % of 8 TB/s", flush=True)
            del W, q, s
    return 0


def report_load(args, rtn, synth, torch, np, dev) -> int:
    """Load-time pipeline: fp16 weights in pinned host memory -> packed weights on the GPU, shard by shard."""
    shapes = {"8b": synth.LLAMA_8B, "70b": synth.LLAMA_70B, "405b": synth.LLAMA_405B}[args.report_load]
    bits = args.bits
    g = 128 if bits == 4 else 0
    cs = torch.cuda.Stream()
    print(f"# load-time quantise from pinned host memory, {args.report_load} shapes, int{bits}; ms per matrix (host timer around a "
          f"synchronised call, best of 3): copy = host-to-device copy of the fp16 tensor alone; serial = that copy, then rtn_quantize; "
          f"pipeline = rtn_quantize_from_host with 4096-row shards (copies overlap the kernels; 2 shards of device staging instead of the whole tensor)")
    tot = [0.0, 0.0, 0.0]
    totb = 0
    for idx, (name, (K, N)) in enumerate(shapes.items()):
        W_host = synth.normal_weight(N, K, 0.02, idx, "cpu").pin_memory()
        W_dev = torch.empty((N, K), dtype=torch.float16, device=dev)
        q, s = rtn.rtn_quantize(W_dev, bits, g)
        rows = 4096
        staging = torch.empty(rtn._lib.rtn_quantize_host_staging_nbytes(K, rows), dtype=torch.uint8, device=dev)

        def best(fn):
            ts = []
            for _ in range(3):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                fn()
                torch.cuda.synchronize()
                ts.append((time.perf_counter() - t0) * 1e3)
            return min(ts)

        t_copy = best(lambda: W_dev.copy_(W_host, non_blocking=True))
        t_serial = best(lambda: (W_dev.copy_(W_host, non_blocking=True), rtn.rtn_quantize(W_dev, bits, g, out=(q, s))))
        t_pipe = best(lambda: rtn.rtn_quantize_from_host(W_host, bits, g, rows, cs, staging=staging, out=(q, s), device=dev))
        q2, s2 = rtn.rtn_quantize(W_host.to(dev), bits, g)
        assert torch.equal(q, q2) and torch.equal(s, s2)
        nb = N * K * 2
        totb += nb
        for i, t in enumerate((t_copy, t_serial, t_pipe)):
            tot[i] += t
        print(f"{name:8s} {K:6d}->{N:6d}  {nb / 1e6:8.1f} MB fp16  copy {t_copy:7.2f} ms ({nb / t_copy / 1e6:5.1f} GB/s)  serial {t_serial:7.2f} ms  "
              f"pipeline {t_pipe:7.2f} ms ({nb / t_pipe / 1e6:5.1f} GB/s of fp16 source, {t_pipe / t_copy:4.2f} x copy)", flush=True)
        del W_host, W_dev, q, s, staging
    print(f"layer: {totb / 1e6:.1f} MB fp16  copy {tot[0]:.2f} ms  serial {tot[1]:.2f} ms  pipeline {tot[2]:.2f} ms "
          f"({totb / tot[2] / 1e6:.1f} GB/s; the on-GPU quantise alone runs at 4.5-6 TB/s, so the link is the bound)")
    return 0


def report_crossover(args, rtn, synth, torch, np, dev) -> int:
    """Fused kernels against dequantise + dense GEMM (the dual path of Section 5) over M, on one model's shapes."""
    shapes = {"8b": synth.LLAMA_8B, "70b": synth.LLAMA_70B, "405b": synth.LLAMA_405B}[args.report_crossover]
    bits = args.bits
    g = 128 if bits == 4 else 0
    Ms = [int(x) for x in args.batches.split(",")]
    ws = torch.empty(256 << 20, dtype=torch.uint8, device=dev)      # room for the split-K partials of either path
    print(f"# {args.report_crossover} shapes, int{bits}; us per call (HIP events, 6 back-to-back calls, best of 3; one weight copy, "
          f"so matrices under 256 MB are cache-resident): fused = rtn_linear; dual = rtn_linear_dense (dequantise to fp16 + "
          f"own dense GEMM); gemm = the dense GEMM alone on already dequantised weights; last column (reference): the same dequantise followed by torch.matmul (hipBLASLt)")

    def timeit(fn, n=6):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ts = []
        for _ in range(3):
            e0.record()
            for _ in range(n):
                fn()
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1) * 1e3 / n)
        return min(ts)

    for idx, (name, (K, N)) in enumerate(shapes.items()):
        W = synth.normal_weight(N, K, 0.02, idx, dev)
        qw, sc = rtn.rtn_quantize(W, bits, g)
        del W
        tmp = torch.empty(rtn.rtn_dense_weight_nbytes(N, K), dtype=torch.uint8, device=dev)
        Wd = tmp.view(torch.float16).view(N, K)
        for M in Ms:
            A = synth.activation(M, K, 100 + M, dev)
            out = torch.empty((M, N), dtype=torch.float16, device=dev)
            fl = 2.0 * M * N * K
            tf = timeit(lambda: rtn.rtn_linear(A, qw, sc, bits, g, out=out, workspace=ws))
            td = timeit(lambda: rtn.rtn_linear_dense(A, qw, sc, bits, g, tmp, out=out, workspace=ws))
            tg = timeit(lambda: rtn.rtn_gemm_fp16(A, Wd, out=out, workspace=ws))

            def dual_vendor():                      # reference only: the same dequantise, then the vendor library's GEMM
                rtn.rtn_dequantize(qw, sc, K, bits, g, out=Wd)
                torch.matmul(A, Wd.t(), out=out)
            tv = timeit(dual_vendor)
            path = rtn.rtn_linear_query(M, N, K, bits, g)["path"]
            print(f"{name:8s} {K:6d}->{N:6d} M={M:5d}  fused(path {path}) {tf:9.1f} us {fl / tf / 1e6:6.0f} TFLOP/s | dual {td:9.1f} us "
                  f"{fl / td / 1e6:6.0f} TFLOP/s | gemm {tg:9.1f} us {fl / tg / 1e6:6.0f} TFLOP/s | fused/dual {tf / td:5.2f} | "
                  f"dequantise + vendor GEMM {tv:9.1f} us, fused/that {tf / tv:5.2f}", flush=True)
        del qw, tmp, Wd
    return 0


def report_grouped(args, rtn, synth, torch, np, dev) -> int:
    """Expert-like independent modules: rtn_layer_forward (one launch per module) against rtn_grouped_forward."""
    bits = args.bits
    g = 128 if bits == 4 else 0
    Ms = [int(x) for x in args.batches.split(",") if int(x) <= 16]
    configs = [("experts 7168/2048 (8 active)", 7168, 2048, 8), ("experts 6144/16384 (8 active)", 6144, 16384, 8),
               ("experts 2048/1024 (8 active)", 2048, 1024, 8)]
    print(f"# int{bits}; us per call over all active experts (HIP-graph replay, calls rotate over >= 600 MB of distinct expert "
          f"weights); serial = rtn_layer_forward, grouped = rtn_grouped_forward; every expert gets M rows of its own")
    for label, hidden, inter, active in configs:
        for mod, (K, N) in (("gate_up", (hidden, 2 * inter)), ("down", (inter, hidden))):
            W = synth.normal_weight(N, K, 0.02, 1, dev)
            qw, sc = rtn.rtn_quantize(W, bits, g)
            del W
            nbytes = qw.numel() + sc.numel() * 2
            calls = max(1, int(np.ceil(600e6 / (nbytes * active))))
            pool = [qw] + [qw.clone() for _ in range(calls * active - 1)]
            for M in Ms:
                plans = []
                for c in range(calls):
                    mods = [dict(A=synth.activation(M, K, 100 + e, dev), qweight=pool[c * active + e], scales=sc, bits=bits,
                                 group_size=g, C=torch.empty((M, N), dtype=torch.float16, device=dev)) for e in range(active)]
                    plans.append(rtn.LayerPlan(mods))
                res = []
                for grouped in (False, True):
                    def issue():
                        for _ in range(3):
                            for pl in plans:
                                pl.run_grouped() if grouped else pl.run()
                    issue()
                    torch.cuda.synchronize()
                    cg = torch.cuda.CUDAGraph()
                    st = torch.cuda.Stream()
                    with torch.cuda.stream(st):
                        with torch.cuda.graph(cg, stream=st):
                            issue()
                    cg.replay()
                    torch.cuda.synchronize()
                    ts = []
                    for _ in range(5):
                        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                        e0.record()
                        cg.replay()
                        e1.record()
                        torch.cuda.synchronize()
                        ts.append(e0.elapsed_time(e1) * 1e3 / (3 * calls))
                    res.append(float(np.median(ts)))
                tot = nbytes * active
                print(f"{label:30s} {mod:8s} {K:6d}->{N:6d} M={M:2d}  serial {res[0]:8.2f} us {tot / res[0] / 1e3:6.0f} GB/s | grouped "
                      f"{res[1]:8.2f} us {tot / res[1] / 1e3:6.0f} GB/s ({tot / res[1] / 80e3:4.1f} % of 8 TB/s) | grouped/serial {res[1] / res[0]:5.2f}",
                      flush=True)
                del plans
            del pool, qw
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3000)
    ap.add_argument("--warmup", type=int, default=2000)
    ap.add_argument("--no-graph", action="store_true", help="launch every step directly instead of replaying HIP graphs")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--headline-only", action="store_true",
                    help="time the int4 layer set alone: no read-stream ceiling, no W8A16 layer set, no CPU baseline (for profiler runs)")
    ap.add_argument("--report", choices=["8b", "70b", "405b"], default=None,
                    help="instead of the JSON line, print a per-matrix, per-M table for that model's shapes")
    ap.add_argument("--report-quantize", choices=["8b", "70b", "405b"], default=None,
                    help="instead of the JSON line, print rtn_quantize throughput per matrix and (bits, group) setting")
    ap.add_argument("--report-load", choices=["8b", "70b", "405b"], default=None,
                    help="instead of the JSON line, time the load-time pipeline from pinned host memory per matrix")
    ap.add_argument("--report-crossover", choices=["8b", "70b", "405b"], default=None,
                    help="instead of the JSON line, print fused kernels vs dequantise + dense GEMM over --batches")
    ap.add_argument("--report-ceiling", action="store_true",
                    help="instead of the JSON line, time a plain read kernel on buffers of every workload matrix's packed size and on 512 MB")
    ap.add_argument("--report-grouped", action="store_true",
                    help="instead of the JSON line, time expert-like independent modules serially and through the grouped call")
    ap.add_argument("--bits", type=int, default=4, help="--report only: 4 (group 128) or 8 (per-channel)")
    ap.add_argument("--selective", action="store_true",
                    help="--report only: the selective-precision layer (modules 2 and 4 at 8 bit per-channel, the others at 4 bit g128)")
    ap.add_argument("--batches", type=str, default="1,2,4,8,16", help="--report only")
    ap.add_argument("--hot", action="store_true",
                    help="--report only: also time launches on a single weight copy (cache-resident when it fits the 256 MB Infinity Cache)")
    ap.add_argument("--compare-paths", action="store_true",
                    help="--report only: also time the vector-ALU v_dot2 variant (M <= 4) in the same workgroup shape")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (--gpus 1); nothing here uses a second GPU.", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import paper_2505_15909_amd as rtn
    from paper_2505_15909_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.report:
        return report(args, rtn, synth, torch, np, dev)
    if args.report_quantize:
        return report_quantize(args, rtn, synth, torch, np, dev)
    if args.report_crossover:
        return report_crossover(args, rtn, synth, torch, np, dev)
    if args.report_load:
        return report_load(args, rtn, synth, torch, np, dev)
    if args.report_grouped:
        return report_grouped(args, rtn, synth, torch, np, dev)
    if args.report_ceiling:
        return report_ceiling(args, rtn, synth, torch, np, dev)
    modules = list(synth.LLAMA_8B.items())

    # ---- set-up: synthetic fp16 weights, load-time quantise (timed separately) ---------------
    W = [synth.normal_weight(N, K, 0.02, seed=i, device=dev) for i, (_, (K, N)) in enumerate(modules)]
    packed = [rtn.rtn_quantize(w, BITS, GROUP) for w in W]           # warm-up + the copy used below
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    q_reps = 5
    e0.record()
    for _ in range(q_reps):
        for w, (q, s) in zip(W, packed):
            rtn.rtn_quantize(w, BITS, GROUP, out=(q, s))
    e1.record()
    torch.cuda.synchronize()
    q_ms = e0.elapsed_time(e1) / q_reps
    q_bytes = sum(w.numel() * 2 + q.numel() + s.numel() * 2 for w, (q, s) in zip(W, packed))
    del W

    layer_bytes = sum(q.numel() + s.numel() * 2 for q, s in packed)   # packed codes + scales of one layer
    n_copies = max(2, int(np.ceil(2.4 * CACHE_BYTES / layer_bytes)))
    copies = [packed] + [[(q.clone(), s.clone()) for q, s in packed] for _ in range(n_copies - 1)]
    acts = {M: [synth.activation(M, K, seed=100 + M, device=dev) for _, (K, N) in modules] for M in BATCHES}
    outs = {M: [torch.empty((M, N), dtype=torch.float16, device=dev) for _, (K, N) in modules] for M in BATCHES}
    ws = torch.empty(16 << 20, dtype=torch.uint8, device=dev)

    # one prepared rtn_layer_forward call per (weight copy, M)
    plans = [[rtn.LayerPlan([dict(A=acts[M][i], qweight=cp[i][0], scales=cp[i][1], bits=BITS, group_size=GROUP,
                                  C=outs[M][i]) for i in range(len(modules))], workspace=ws)
              for M in BATCHES] for cp in copies]
    pass_no = [0]

    def step_direct():
        for j in range(len(BATCHES)):
            plans[pass_no[0] % n_copies][j].run()
            pass_no[0] += 1

    stream = torch.cuda.Stream()
    graphs = []
    if not args.no_graph:
        # a step replays one HIP graph; n_copies graphs cover every phase of the weight rotation
        with torch.cuda.stream(stream):
            for _ in range(2):
                step_direct()
            stream.synchronize()
            for v in range(n_copies):
                pass_no[0] = v * len(BATCHES)
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=stream):
                    step_direct()
                graphs.append(g)
            # and one graph that holds a whole rotation (n_copies consecutive steps): replaying it issues n_copies
            # steps with one submission, which takes the per-submission gap out of long runs
            pass_no[0] = 0
            rotation = torch.cuda.CUDAGraph()
            with torch.cuda.graph(rotation, stream=stream):
                for _ in range(n_copies):
                    step_direct()
            # a short timed region (up to 120 steps) is one graph of exactly that many steps, starting at the rotation phase
            # the warm-up steps leave off at: one submission, no gaps between graphs inside the timed region
            timed_graph = None
            if args.steps <= 120:
                pass_no[0] = args.warmup * len(BATCHES)
                timed_graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(timed_graph, stream=stream):
                    for _ in range(args.steps):
                        step_direct()
    step_no = [0]

    def run_steps(n):
        """Exactly n steps, in rotation order: whole rotations through the rotation graph, the rest step by step."""
        done = 0
        while done < n:
            phase = step_no[0] % n_copies
            if graphs and phase == 0 and n - done >= n_copies:
                rotation.replay()
                k = n_copies
            elif graphs:
                graphs[phase].replay()
                k = 1
            else:
                step_direct()
                k = 1
            step_no[0] += k
            done += k

    with torch.cuda.stream(stream):
        # Clocks: the set-up above is short bursts with idle gaps, and the first 100-200 ms of work after idling run
        # 3-8 % slower on this chip.  Part of set-up, before the warm-up steps and outside the timed region: the same
        # step graphs for SETTLE_MS (whole rotations, so the rotation phase is unchanged); reported in the JSON line.
        if graphs and SETTLE_MS > 0:
            t_settle = time.perf_counter()
            while (time.perf_counter() - t_settle) * 1e3 < SETTLE_MS:
                for _ in range(16):
                    rotation.replay()
                stream.synchronize()
        run_steps(args.warmup)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        if graphs and timed_graph is not None:
            timed_graph.replay()                    # exactly args.steps steps
        else:
            run_steps(args.steps)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    step_weight_bytes = layer_bytes * len(BATCHES)
    value = step_weight_bytes / (ms_per_step * 1e-3) / 1e9
    flops = sum(2.0 * M * N * K for M in BATCHES for _, (K, N) in modules)

    # ---- roofline of the dominant kernel (the int4 skinny MFMA dequantise-GEMM: all 20 launches of a
    # step).  A pair of HIP events on the launch stream brackets the launches of the same passes issued
    # back to back (one rtn_linear per launch, direct launches, no graph); the stream is first held busy
    # so that the host has enqueued everything before the GPU gets there, and the bracket times the GPU.
    # (Events around every single launch cost several microseconds each on this runtime and were not
    # usable.)  Average launch duration = bracket / launches; dispatch gaps are inside it.
    algo_bytes = 0.0
    calls = []
    for s_i in range(min(args.steps, 20)):
        for j, M in enumerate(BATCHES):
            cp = copies[pass_no[0] % n_copies]
            pass_no[0] += 1
            for i, (_, (K, N)) in enumerate(modules):
                calls.append((acts[M][i], cp[i][0], cp[i][1], outs[M][i]))
                algo_bytes += cp[i][0].numel() + cp[i][1].numel() * 2 + 2 * M * K + 2 * M * N
    n_launch = len(calls)
    hold = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    with torch.cuda.stream(stream):
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for _ in range(12):
            hold.fill_(1)                                   # a few milliseconds of head start for the host
        ev0.record(stream)
        for A_, q_, s_, o_ in calls:
            rtn.rtn_linear(A_, q_, s_, BITS, GROUP, out=o_, workspace=ws)
        ev1.record(stream)
        torch.cuda.synchronize()
        launch_us = ev0.elapsed_time(ev1) * 1e3 / n_launch
    del hold
    achieved = algo_bytes / n_launch / (launch_us * 1e-6) / 1e9
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": _measured_traffic(),
                "kernel": "rtn::skinny_mfma_kernel<4,4,1,*,1> (fused int4 g128 dequantise-GEMM; a launch = one rtn_linear)",
                "launches": n_launch, "avg_launch_us": round(launch_us, 3),
                "algorithmic_bytes_per_launch": round(algo_bytes / n_launch, 1)}

    # ---- read-stream ceiling: a plain read kernel on buffers of the four matrices' packed sizes, same protocol ----
    read_ceiling_gbs = None
    if not args.headline_only:
        pool, sink = _ceiling_pool(torch, dev)
        ceil_us = [_read_ceiling_us(rtn, torch, np, q.numel() + s.numel() * 2, pool, sink) for q, s in packed]
        t512 = _read_ceiling_us(rtn, torch, np, 512e6, pool, sink)
        del pool
        read_ceiling_gbs = layer_bytes / sum(ceil_us) / 1e3
        roofline["read_ceiling"] = {"layer_set_GB/s": round(read_ceiling_gbs, 1), "layer_set_us": round(sum(ceil_us), 2),
                                "per_matrix_us": [round(t, 2) for t in ceil_us], "stream_512MB_GB/s": round(512e6 / t512 / 1e3, 1),
                                "kernel": "rtn::read_stream_kernel (16 bytes per lane, nothing else), graph replay, rotating buffers"}

    # ---- the other precision the metric names: the same layer at W8A16 (int8, per-channel scales), M = 1, 4, 16, 64 ----
    w8 = {}
    w8_layer_bytes = 0
    w8_times = {M: 0.0 for M in W8_BATCHES}
    ws_big = torch.empty(64 << 20, dtype=torch.uint8, device=dev)
    for i, (name, (K, N)) in enumerate(() if args.headline_only else modules):
        w = synth.normal_weight(N, K, 0.02, seed=i, device=dev)
        q8, s8 = rtn.rtn_quantize(w, 8, 0)
        del w
        nb8 = q8.numel() + s8.numel() * 2
        w8_layer_bytes += nb8
        q8s = [q8] + [q8.clone() for _ in range(max(2, int(np.ceil(600e6 / nb8))) - 1)]
        for M in W8_BATCHES:
            A8 = synth.activation(M, K, seed=100 + M, device=dev)
            w8_times[M] += _time_linear(rtn, torch, np, A8, q8s, s8, 8, 0, None, ws_big)
        del q8s, q8
    for M in () if args.headline_only else W8_BATCHES:
        w8[f"M{M}"] = {"layer_set_us": round(w8_times[M], 2), "GB/s": round(w8_layer_bytes / w8_times[M] / 1e3, 1),
                       "pct_hbm_peak": round(w8_layer_bytes / w8_times[M] / 80e3, 2)}

    # ---- CPU oracle timed beside it (bounded sample of the same workload) ------------------------
    cpu = None
    if not (args.no_cpu_baseline or args.headline_only):
        from oracle import rtn_oracle as O
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count() or 1
        sample = []
        for i, (name, (K, N)) in enumerate(modules):
            w = synth.normal_weight(N, K, 0.02, seed=i, device="cpu").numpy()
            codes, scales = O.rtn_quantize(w, BITS, GROUP)
            sample.append((codes, scales, K, N))
        cpu_bytes = 0
        cpu_steps = 0
        host_acts = {M: [a.cpu().numpy() for a in acts[M]] for M in BATCHES}
        tc = time.perf_counter()
        while time.perf_counter() - tc < 10.0:
            for M in BATCHES:
                for i, (codes, scales, K, N) in enumerate(sample):
                    O.rtn_linear(host_acts[M][i], codes, scales, GROUP)
                    cpu_bytes += codes.size * BITS // 8 + scales.size * 2
            cpu_steps += 1
        tc = time.perf_counter() - tc
        cpu = {"value": round(cpu_bytes / tc / 1e9, 4), "unit": "GB/s", "cores": int(cores), "kind": "oracle",
               "sample": f"{cpu_steps} full steps (each 20 float64 linears of the same layer set, M=1,2,4,8,16), "
                         f"{tc:.1f} s wall; quantisation of the sample not timed"}

    line = {
        "metric": "weight-stream GB/s (% HBM peak) of RTN W4A16/W8A16 linear at M=1..16",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": "llama8b_w4a16_g128_layer_set_M1-16", "bits": BITS, "group_size": GROUP,
                   "batches": list(BATCHES), "modules": {k: list(v) for k, v in synth.LLAMA_8B.items()},
                   "weight_copies_rotated": n_copies, "launch": "hip_graph_replay" if graphs else "direct",
                   "clock_settle_ms_before_warmup": SETTLE_MS if graphs else 0.0},
        "pct_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
        "tflops": round(flops / (ms_per_step * 1e-3) / 1e12, 3),
        "weight_bytes_per_step": int(step_weight_bytes),
        "read_ceiling_gbs": round(read_ceiling_gbs, 1) if read_ceiling_gbs else None,
        "value_over_read_ceiling": round(value / read_ceiling_gbs, 4) if read_ceiling_gbs else None,
        "extra": {"w8a16_llama8b_int8_per_channel_layer_set": w8 or None,
                  "w8a16_note": "same four modules, symmetric RTN int8 with per-output-channel scales; per-matrix HIP-graph replay over "
                                ">= 600 MB of rotating packed copies, layer set = sum of the four"},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "quantize": {"GB/s": round(q_bytes / (q_ms * 1e-3) / 1e9, 1), "ms_per_layer": round(q_ms, 4),
                     "bytes": "fp16 read + packed codes and scales written, four modules"},
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
