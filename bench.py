#!/usr/bin/env python3
"""Benchmark of the PTQTP decode hot path on one MI355X.

A step is one decode step through the linear layers of an 8B-shaped decoder
stack at batch 1: `--layers` (default 32) layers x the seven linears q, k, v,
o, gate, up, down, every linear with its own packed blob and its own x, run
back to back on one stream.  The shapes are those of an 8B LLaMA-3 decoder; walking 32
distinct layer copies (3.7 GB of packed planes + scales) keeps every launch
cold in HBM instead of warm in the 256 MB Infinity Cache.

Prints ONE JSON line: metric, value (GB/s of algorithmic bytes), ms_per_step, the roofline of the
dominant kernel (measured with HIP events on the launch stream) and the fp64 CPU oracle timed beside it;
`--per-shape` adds small-batch, dependent-chain, 70B, prefill and quantizer figures under "per_shape".
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth
CHAIN_O_SCALE, CHAIN_DOWN_SCALE = 0.125, 0.03125   # applied to the scales of o and down in the dependent chain


def algorithmic_bytes(N: int, K: int, M: int = 1, group: int = 128) -> int:
    """Bytes one call has to move: 2-bit planes + fp16 scales (appendix memory model,
    0.53125 B per weight at G = 128) + fp16 x + fp32 y."""
    return N * K // 2 + 4 * N * (K // group) + 2 * M * K + 4 * M * N


def build_stack(ptq, torch, workloads, layers: int, dev, log=True):
    """Generate (seeded recipe, host) and pack (device) `layers` x 7 linears.  Returns the
    per-linear blobs, activations, outputs, (layer, name) jobs, shapes, and layer 0's host copy."""
    t0 = time.time()
    names = workloads.LINEAR_ORDER
    pool = ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1))
    jobs = [(layer, name) for layer in range(layers) for name in names]

    def gen(job):
        return workloads.linear_8b(job[1], job[0])

    blobs, xs, ys = [], [], []
    layer0 = {}
    window = 14
    pending = [pool.submit(gen, j) for j in jobs[:window]]
    nxt = window
    for idx, job in enumerate(jobs):
        lin = pending.pop(0).result()
        if nxt < len(jobs):
            pending.append(pool.submit(gen, jobs[nxt]))
            nxt += 1
        N, K = lin["N"], lin["K"]
        blob = ptq.ptqtp_pack(*(torch.from_numpy(lin[k]).to(dev) for k in ("T1", "T2", "a1", "a2")), check=False)
        blobs.append(blob)
        xs.append(torch.from_numpy(workloads.x_for(job[1], 1, K, 1, job[0])).to(dev).reshape(-1))
        ys.append(torch.empty((1, N), dtype=torch.float32, device=dev))
        if job[0] == 0:
            layer0[job[1]] = lin
        if log and idx % 56 == 55:
            print(f"[bench] packed {idx + 1}/{len(jobs)} linears ({time.time() - t0:.0f} s)", file=sys.stderr, flush=True)
    pool.shutdown()
    torch.cuda.synchronize()
    dims = [workloads.SHAPES_8B[name] for _, name in jobs]
    return blobs, xs, ys, jobs, dims, layer0


def make_step(ptq, torch, mode, blobs, xs, ys, dims, stream):
    """A callable that enqueues one decode step on `stream` (must be the current stream)."""
    def run_calls():
        for blob, x, y, (n, k) in zip(blobs, xs, ys, dims):
            ptq.ptqtp_gemv(blob, x, n, k, out=y)

    if mode == "eager":
        return run_calls, len(blobs)
    if mode == "graph":
        run_calls()
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            run_calls()
        return graph.replay, len(blobs)
    if mode == "fused4":
        # what a real decode step can fuse without breaking dependencies: {q,k,v}, {o}, {gate,up}, {down} per layer
        ents = [(b, x, y, n, k) for b, x, y, (n, k) in zip(blobs, xs, ys, dims)]
        plans = []
        for layer in range(len(blobs) // 7):
            e = ents[7 * layer:7 * layer + 7]
            plans += [ptq.ptqtp_gemv_batch_plan(e[0:3]), ptq.ptqtp_gemv_batch_plan(e[3:4]),
                      ptq.ptqtp_gemv_batch_plan(e[4:6]), ptq.ptqtp_gemv_batch_plan(e[6:7])]

        def run_plans():
            for p in plans:
                ptq.ptqtp_gemv_batch(p)
        run_plans()
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            run_plans()
        graph._keep = plans
        return graph.replay, len(plans)
    plan = ptq.ptqtp_gemv_batch_plan([(b, x, y, n, k) for b, x, y, (n, k) in zip(blobs, xs, ys, dims)])
    stream.synchronize()
    return (lambda: ptq.ptqtp_gemv_batch(plan)), 1


def time_steps(torch, step, steps, warmup, stream, stats=None):
    """ms per step over EXACTLY `steps` steps, bracketed by synchronisation on both sides (HIP events recorded on
    `stream`, the stream the kernels are launched on).  With `stats` (a dict) a second pass of the same length
    records an event after every step and leaves their median and minimum there."""
    for _ in range(warmup):
        step()
    stream.synchronize()
    torch.cuda.synchronize()
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    wall0 = time.perf_counter()
    ev0.record(stream)
    for _ in range(steps):
        step()
    ev1.record(stream)
    stream.synchronize()
    torch.cuda.synchronize()
    wall = time.perf_counter() - wall0
    if stats is not None:
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        evs[0].record(stream)
        for i in range(steps):
            step()
            evs[i + 1].record(stream)
        stream.synchronize()
        per = sorted(evs[i].elapsed_time(evs[i + 1]) * 1e3 for i in range(steps))
        stats["median_us"] = round(per[len(per) // 2], 2)
        stats["min_us"] = round(per[0], 2)
        stats["mean_us"] = round(ev0.elapsed_time(ev1) * 1e3 / steps, 2)
    return max(ev0.elapsed_time(ev1), wall * 1e3) / steps


def preheat(step, stream, ms=150.0):
    """Run `step` untimed for `ms` milliseconds: every figure is taken at the clocks of a GPU that is serving, not of
    one that has just waited for the host to set up the next case (the first steps after an idle spell run 5-10 %
    slower and would sit in the mean)."""
    t0 = time.perf_counter()
    while (time.perf_counter() - t0) * 1e3 < ms:
        for _ in range(10):
            step()
        stream.synchronize()


MFMA_F16_PEAK_TFLOPS = 2500.0   # MI355X published dense fp16 matrix rate
RIDGE_TOKENS = 41               # 7.5 * M operations per byte of the packed stream: the two roofs cross near 41 tokens


def roof_entry(us, N_K_list, M):
    """One per-config entry: time, GB/s of algorithmic bytes, and the fraction of the binding roof (HBM below the
    ridge, the fp16 matrix rate above; both planes counted: 2 * 2 * M * N * K operations)."""
    nbytes = sum(algorithmic_bytes(n, k, M) for n, k in N_K_list)
    flops = sum(4.0 * M * n * k for n, k in N_K_list)
    ent = {"us": round(us, 2), "GBps": round(nbytes / us / 1e3, 1)}
    if M < RIDGE_TOKENS:
        ent["bound"], ent["frac"] = "hbm", round(nbytes / us / 1e3 / HBM_PEAK_GBS, 4)
    else:
        ent["TFLOPs"] = round(flops / us / 1e6, 1)
        ent["bound"], ent["frac"] = "mfma", round(flops / us / 1e6 / MFMA_F16_PEAK_TFLOPS, 4)
    return ent


def random_blob(ptq, torch, n, k, dev, seed):
    """A packed layer with the recipe's distributions drawn on the device (seeded): for timing only -- the kernels
    are data-oblivious -- where generating on the host would cost more than the measurement."""
    g = torch.Generator(device=dev)
    g.manual_seed(16989 * 1000 + seed)
    lut = torch.tensor([-1, -1, -1, 1, 1, 1, 0, 0, 0, 0], dtype=torch.int8, device=dev)
    T1 = lut[torch.randint(0, 10, (n, k), device=dev, generator=g)]
    T2 = lut[torch.randint(0, 10, (n, k), device=dev, generator=g)]
    a1 = (0.02 * torch.randn(n, k // 128, device=dev, generator=g)).abs().half()
    a2 = (a1.float() * (0.1 + 0.4 * torch.rand(n, k // 128, device=dev, generator=g))).half()
    return ptq.ptqtp_pack(T1, T2, a1, a2, check=False)


def per_config_timing(ptq, torch, workloads, blobs, jobs, dims, stream, note):
    """The configurations beside the headline, compact: the dependent decode step (config 3 with real dependencies),
    the whole 8B stack in one launch at 4 / 16 / 64 tokens (config 2), 70B gate and down at 1 / 32 / 2048 tokens
    (config 4), each with its fraction of the roof that binds it."""
    dev = blobs[0].device
    res = {}
    with torch.cuda.stream(stream):
        for M in (4, 16, 64):
            xm = [torch.randn(M, k, device=dev).half() for (n, k) in dims]
            ym = [torch.empty(M, n, device=dev) for (n, k) in dims]
            plan = ptq.ptqtp_gemv_batch_plan([(b, x, y, n, k) for b, x, y, (n, k) in zip(blobs, xm, ym, dims)])
            stream.synchronize()
            st = {}
            preheat(lambda: ptq.ptqtp_gemm_batch(plan, M), stream)
            ms = time_steps(torch, lambda: ptq.ptqtp_gemm_batch(plan, M), 50, 10, stream, stats=st)
            ent = roof_entry(ms * 1e3, dims, M)
            ent.update(median_us=st["median_us"], min_us=st["min_us"])
            res[f"8b_stack_one_launch_M{M}"] = ent
            if M == 64:
                # the same launch with the planes summed in fp16 before the matrix pipe (ptqtp_gemm_batch_fused)
                st = {}
                preheat(lambda: ptq.ptqtp_gemm_batch_fused(plan, M), stream)
                ms = time_steps(torch, lambda: ptq.ptqtp_gemm_batch_fused(plan, M), 50, 10, stream, stats=st)
                us = ms * 1e3
                nbytes = sum(algorithmic_bytes(n, k, M) for n, k in dims)
                flops = sum(4.0 * M * n * k for n, k in dims)
                # half the matrix operations are executed: the HBM stream is the roof that binds (465 us against 357)
                res[f"8b_stack_one_launch_M{M}_fused_planes"] = {
                    "us": round(us, 2), "GBps": round(nbytes / us / 1e3, 1),
                    "TFLOPs_counted_as_two_planes": round(flops / us / 1e6, 1), "bound": "hbm",
                    "frac": round(nbytes / us / 1e3 / HBM_PEAK_GBS, 4),
                    "median_us": st["median_us"], "min_us": st["min_us"], "arithmetic": "PTQTP_FUSED_PLANES"}
            del xm, ym, plan
            note(f"stack at M={M} done")
        for name in ("gate", "down"):
            n, k = workloads.SHAPES_70B[name]
            copies = [random_blob(ptq, torch, n, k, dev, 70 + i) for i in range(3)]    # 375 MB walked: cold in the 256 MB cache
            for M in (1, 32, 2048):
                x = torch.randn(M, k, device=dev).half()
                y = torch.empty(M, n, device=dev)
                us = _graph_time(torch, stream, lambda: [ptq.ptqtp_gemm(b, x, n, k, out=y) for b in copies], len(copies), reps=5)
                res[f"70b_{name}_{n}x{k}_M{M}"] = roof_entry(us, [(n, k)], M)
            del copies
            note(f"70B {name} done")
    return res


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--mode", choices=["batch", "chain", "fused4", "graph", "eager"], default="batch",
                    help="what one timed step is.  batch: one ptqtp_gemv_batch launch over all 7*layers linears (every "
                         "linear's input known in advance: the packed-weight stream at its best); chain: the dependent "
                         "decode step, 4 fused stages per layer (ptqtp_chain_run) replayed as one hipGraph; fused4: 4 "
                         "batched launches per layer ({q,k,v},{o},{gate,up},{down}) replayed as one hipGraph; graph: "
                         "7*layers ptqtp_gemv launches replayed as one hipGraph; eager: the same launches call by call")
    ap.add_argument("--preheat-ms", type=float, default=300.0,
                    help="run the step untimed for this long before the warmup steps (0 = not at all)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-config", action="store_true",
                    help="time only the step of --mode (for runs under a profiler)")
    ap.add_argument("--no-chain", action="store_true",
                    help="leave the dependent decode chain (and its hipGraph) out: for counter runs, where rocprofv3's "
                         "counter collection has crashed on the replay of that graph")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run 5 plain 1 GiB device copies (known HBM traffic) and exit: the reference that "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE readings are scaled by")
    ap.add_argument("--per-shape", action="store_true",
                    help="also time the other configs one linear per launch: 8B shapes at M = 1/4/16/64, 70B shapes at "
                         "M = 1/32 and prefill M = 2048, the quantizer, pack / unpack")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path needs no second device); use --gpus 1",
              file=sys.stderr)
        return 2

    import torch

    import paper_2509_16989_amd as ptq
    import workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    names = workloads.LINEAR_ORDER
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy": {"bytes_read_per_copy": 1 << 30, "bytes_written_per_copy": 1 << 30,
                                             "copies": 5}}), flush=True)
        return 0

    def note(what):
        print(f"[bench] {what}", file=sys.stderr, flush=True)

    blobs, xs, ys, jobs, dims, layer0 = build_stack(ptq, torch, workloads, args.layers, dev)
    bytes_step = sum(algorithmic_bytes(n, k) for n, k in dims)

    stream = torch.cuda.Stream()          # default priority
    extra = {}
    chain = None
    with torch.cuda.stream(stream):
        if args.mode == "chain" or not (args.no_per_config or args.no_chain):
            chain = DecodeChain(ptq, torch, blobs, jobs, dims, stream)
        if args.mode == "chain":
            step, launches_step, bytes_step = chain.replay, chain.launches, chain.nbytes
        else:
            step, launches_step = make_step(ptq, torch, args.mode, blobs, xs, ys, dims, stream)
        # The stack was just generated on the host with the GPU idle: run the step untimed for a moment so that the
        # warmup and the timed steps see the clocks of a GPU that is serving, not of one that has just woken up
        # (the first 130 ms after idling measure 1.5 % slower than any later 130 ms).
        t_pre = time.perf_counter()
        while (time.perf_counter() - t_pre) * 1e3 < args.preheat_ms:
            for _ in range(20):
                step()
            stream.synchronize()
        stats = {}
        ms_per_step = time_steps(torch, step, args.steps, args.warmup, stream, stats=stats)
        note(f"timed step ({args.mode}) done")
        if not args.no_per_config:
            others = {}
            for mode in ("batch", "fused4", "graph"):
                if mode != args.mode:
                    st, _ = make_step(ptq, torch, mode, blobs, xs, ys, dims, stream)
                    others[mode] = round(time_steps(torch, st, max(3, args.steps // 5), 2, stream) * 1e3, 2)
            extra["us_per_stack_pass_other_launch_modes"] = others
            if args.mode != "chain" and chain is not None:
                cst = {}
                preheat(chain.replay, stream)
                chain_us = time_steps(torch, chain.replay, 100, 20, stream, stats=cst) * 1e3
            else:
                cst, chain_us = stats, ms_per_step * 1e3
            note("dependent chain done")
            if chain is not None:
                extra["us_per_decode_step"] = round(chain_us, 2)
                extra["decode_step"] = {
                    "what": "dependent decode step: per layer qkv -> o (+residual) -> gate|up (silu(gate)*up) -> down "
                            "(+residual), fp16 activations, ptqtp_chain_run replayed from one hipGraph",
                    "us": round(chain_us, 2), "median_us": cst["median_us"], "min_us": cst["min_us"],
                    "launches": chain.launches, "bytes_per_step": chain.nbytes,
                    "GBps": round(chain.nbytes / chain_us / 1e3, 1), "bound": "hbm",
                    "frac": round(chain.nbytes / chain_us / 1e3 / HBM_PEAK_GBS, 4),
                    "agrees_with_unfused_calls": chain.self_check()}
            extra["per_config"] = per_config_timing(ptq, torch, workloads, blobs, jobs, dims, stream, note)
        if args.per_shape:
            extra["per_shape"] = per_shape_timing(ptq, torch, blobs, xs, ys, jobs, dims, stream, args.no_cpu_baseline,
                                                  quick=args.steps < 50, chain=chain, no_chain=args.no_chain)

    gbs = bytes_step / (ms_per_step * 1e-3) / 1e9
    launch_us = ms_per_step * 1e3 / launches_step
    bytes_launch = bytes_step / launches_step
    kernel = {"batch": "gemv_items_kernel<true, 2>", "chain": "chain_level_kernel (one launch per level; launch gaps included)",
              "fused4": "gemv_items_kernel<true, 1>"}.get(args.mode, "gemv_items_kernel<false, 1>")
    step_what = {"batch": "one pass over the stack's 7 x layers linears, every input known in advance (one launch)",
                 "chain": "one dependent decode step (4 fused stages per layer)"}.get(args.mode, "one pass over the stack, " + args.mode)
    out = {
        "metric": "ternary GEMV effective HBM GB/s (% of 8 TB/s peak), 8B shapes b=1; us per dependent decode step beside it",
        "value": round(gbs, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"configs[1] 8B-shaped decoder linears (q,k,v,o,gate,up,down) at batch 1, group 128, "
                               f"walked over {args.layers} distinct layer copies (= configs[3] stack)",
                   "step": step_what,
                   "layers": args.layers, "launches_per_step": launches_step, "launch_mode": args.mode,
                   "bytes_per_step": bytes_step, "untimed_preheat_ms": args.preheat_ms},
        "pct_hbm_peak": round(100.0 * gbs / HBM_PEAK_GBS, 2),
        "step_us": {"mean": round(ms_per_step * 1e3, 2), "median": stats["median_us"], "min": stats["min_us"]},
        "roofline": {"bound": "hbm", "achieved": round(bytes_launch / (launch_us * 1e-6) / 1e9, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(bytes_launch / (launch_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                     "kernel": kernel, "avg_launch_us": round(launch_us, 3),
                     "bytes_per_launch": round(bytes_launch)},
    }
    out["roofline"].update(recorded_traffic(args.mode, args.layers))
    if args.mode == "batch":
        out["us_per_stack_pass_independent"] = round(ms_per_step * 1e3, 2)
    out.update(extra)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(layer0, names)
    print(json.dumps(out), flush=True)
    return 0


def kernel_source_hash() -> str:
    """sha256 (first 16 hex digits) over the library's sources, in a fixed order: ties a committed rocprofv3
    summary to the code it was taken from."""
    import hashlib
    h = hashlib.sha256()
    base = os.path.join(ROOT, "paper_2509_16989_amd", "csrc")
    for name in sorted(os.listdir(base)):
        if name.endswith((".hip", ".hpp")):
            h.update(open(os.path.join(base, name), "rb").read())
    return h.hexdigest()[:16]


def recorded_traffic(mode: str, layers: int) -> dict:
    """HBM bytes per launch of the dominant kernel as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled
    by the plain-copy calibration).  The counters cannot be read from inside the benchmark: the figure comes from
    the committed profile summary and is handed out only for the launch shape that was profiled and only while the
    library's sources still hash to what the summary names; otherwise "traffic" is None."""
    path = os.path.join(ROOT, "profiles", "gemv_items_batch_8b_stack.txt")
    none = {"traffic": None, "traffic_source": None}
    if mode != "batch" or layers != 32 or not os.path.exists(path):
        return none
    traffic = src_hash = None
    for line in open(path):
        if line.startswith("traffic_bytes_per_launch:"):
            traffic = int(float(line.split(":")[1].split()[0]))
        if line.startswith("kernel_source_hash:"):
            src_hash = line.split(":")[1].split()[0]
    if traffic is None or src_hash != kernel_source_hash():
        return none
    return {"traffic": traffic,
            "traffic_source": "profiles/gemv_items_batch_8b_stack.txt: rocprofv3 --pmc runs of this command at library "
                              f"source hash {src_hash}; not measured by this run"}


def _graph_time(torch, stream, run, launches, reps=10, heat_ms=30.0):
    """us per launch of `run` (which enqueues `launches` library calls), replayed from a hipGraph."""
    run()
    stream.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=stream):
        run()
    g.replay()
    stream.synchronize()
    preheat(g.replay, stream, ms=heat_ms)
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(reps):
        g.replay()
    e1.record(stream)
    stream.synchronize()
    return e0.elapsed_time(e1) * 1e3 / (reps * launches)


def per_shape_timing(ptq, torch, blobs, xs, ys, jobs, dims, stream, no_cpu=False, quick=False, chain=None, no_chain=False):
    """The workloads beside the headline, one linear per launch:
    each 8B shape at M = 1, 4, 16, 64, cold (walking the 32 layer copies) -- and M = 1 hot, and short prompts
    (M = 128, 512) on the small MFMA tiles;
    70B shapes at M = 1 and 32 (hot: one copy) and prefill M = 2048 on the MFMA tiles;
    the whole stack in one launch at M = 4, 16, 64; the dependent decode chain;
    plus the quantizer (ptqtp_quantize) on two 8B shapes, with the oracle quantizer timed on a 256 x 4096 sample,
    and ptqtp_pack / ptqtp_unpack on an 8B and a 70B shape."""
    import workloads
    res = {"8b": {}, "70b": {}}
    dev = xs[0].device
    reps = 2 if quick else 10              # quick: few replays, for runs under a profiler (chosen by --steps < 50)

    def note(what):
        print(f"[bench] per-shape: {what}", file=sys.stderr, flush=True)
    with torch.cuda.stream(stream):
        for name in ("q", "k", "gate", "down"):
            idxs = [i for i, j in enumerate(jobs) if j[1] == name]
            n, k = dims[idxs[0]]
            for M in (1, 4, 16, 64):
                x = torch.randn(M, k, device=dev).half()
                y = torch.empty(M, n, device=dev)
                us = _graph_time(torch, stream, lambda: [ptq.ptqtp_gemm(blobs[i], x, n, k, out=y) for i in idxs], len(idxs), reps=reps)
                res["8b"][f"{name}_{n}x{k}_M{M}_cold"] = {"us": round(us, 2), "GBps": round(algorithmic_bytes(n, k, M) / us / 1e3, 1)}
            x = xs[idxs[0]].reshape(1, -1)
            y = ys[idxs[0]]
            us = _graph_time(torch, stream, lambda: [ptq.ptqtp_gemm(blobs[idxs[0]], x, n, k, out=y) for _ in range(32)], 32, reps=reps)
            note(f"8B {name} done")
            res["8b"][f"{name}_{n}x{k}_M1_hot"] = {"us": round(us, 2), "GBps": round(algorithmic_bytes(n, k, 1) / us / 1e3, 1)}
            # a short prompt (the paper's prefill length, Sec. "Inference Efficiency"): few tiles, the small MFMA tiles
            for M in (128, 512):
                x = torch.randn(M, k, device=dev).half()
                y = torch.empty(M, n, device=dev)
                us = _graph_time(torch, stream, lambda: [ptq.ptqtp_gemm(blobs[idxs[0]], x, n, k, out=y) for _ in range(8)], 8, reps=reps)
                res["8b"][f"{name}_{n}x{k}_M{M}_prefill"] = {"us": round(us, 2), "TFLOPs": round(4.0 * M * n * k / us / 1e6, 1)}
        for name in ("q", "k", "gate", "down"):
            lin = workloads.linear_70b(name)
            n, k = lin["N"], lin["K"]
            blob = ptq.ptqtp_pack(*(torch.from_numpy(lin[key]).to(dev) for key in ("T1", "T2", "a1", "a2")), check=False)
            del lin
            for M in (1, 32, 2048):
                x = torch.randn(M, k, device=dev).half()
                y = torch.empty(M, n, device=dev)
                us = _graph_time(torch, stream, lambda: [ptq.ptqtp_gemm(blob, x, n, k, out=y) for _ in range(4)], 4, reps=min(reps, 5))
                ent = {"us": round(us, 2), "GBps": round(algorithmic_bytes(n, k, M) / us / 1e3, 1)}
                if M == 2048:
                    ent["TFLOPs"] = round(4.0 * M * n * k / us / 1e6, 1)      # two planes: 2*2*M*N*K
                res["70b"][f"{name}_{n}x{k}_M{M}"] = ent
                if M == 2048:
                    # planes summed in fp16 before the matrix pipe (one more rounding per weight, half the MFMAs)
                    flag = ptq.PTQTP_F32 | ptq.PTQTP_FUSED_PLANES
                    us = _graph_time(torch, stream, lambda: [ptq.ptqtp_gemm(blob, x, n, k, out=y, y_dtype=flag) for _ in range(4)], 4, reps=min(reps, 5))
                    res["70b"][f"{name}_{n}x{k}_M{M}_fused_planes"] = {"us": round(us, 2), "TFLOPs_counted_as_two_planes": round(4.0 * M * n * k / us / 1e6, 1)}
            if name == "down" and not quick:
                # longer prompts on the largest shape
                for M in (4096, 8192):
                    x = torch.randn(M, k, device=dev).half()
                    y = torch.empty(M, n, device=dev)
                    for flag, tag in ((ptq.PTQTP_F32, ""), (ptq.PTQTP_F32 | ptq.PTQTP_FUSED_PLANES, "_fused_planes")):
                        us = _graph_time(torch, stream, lambda: [ptq.ptqtp_gemm(blob, x, n, k, out=y, y_dtype=flag) for _ in range(2)], 2, reps=3)
                        res["70b"][f"{name}_{n}x{k}_M{M}{tag}"] = {"us": round(us, 1), "TFLOPs_counted_as_two_planes": round(4.0 * M * n * k / us / 1e6, 1)}
                    del x, y
            del blob
            note(f"70B {name} done")
        # config 2 on the whole stack: one batched launch per step, M tokens per linear
        res["stack_batched"] = {}
        for M in (4, 16, 64):
            xm = [torch.randn(M, k, device=dev).half() for (n, k) in dims]
            ym = [torch.empty(M, n, device=dev) for (n, k) in dims]
            plan = ptq.ptqtp_gemv_batch_plan([(b, x, y, n, k) for b, x, y, (n, k) in zip(blobs, xm, ym, dims)])
            stream.synchronize()
            ms = time_steps(torch, lambda: ptq.ptqtp_gemm_batch(plan, M), 5 if quick else 30, 2 if quick else 10, stream)
            note(f"stack at M={M} done")
            nbytes = sum(algorithmic_bytes(n, k, M) for n, k in dims)
            res["stack_batched"][f"M{M}"] = {"us_per_step": round(ms * 1e3, 1), "GBps": round(nbytes / ms / 1e6, 1)}
            del xm, ym, plan
        # config 3 with the activations really depending on each other: per layer qkv -> o (+residual) ->
        # gate|up (silu(gate)*up) -> down (+residual), fp16 activations, one launch per stage (128 launches)
        # replayed from a hipGraph.  Attention itself is not part of the path: o reads the q part of qkv's output.
        if not no_chain:
            if chain is None:
                chain = DecodeChain(ptq, torch, blobs, jobs, dims, stream)
            res["dependent_chain"] = chain.extras(quick)
            note("dependent chain done")
        # the step before the path: PTQTP decomposition of Gaussian fp16 weights (paper settings: T_max 50, eps 1e-4)
        res["quantize"] = {}
        for name in ("q", "gate"):
            n, k = workloads.SHAPES_8B[name]
            W = (torch.randn(n, k, device=dev) * 0.02).half()
            ptq.ptqtp_quantize(W)
            stream.synchronize()
            t0 = time.perf_counter()
            out = ptq.ptqtp_quantize(W)
            stream.synchronize()
            dt = time.perf_counter() - t0
            it = int(out[4].item())
            res["quantize"][f"{name}_{n}x{k}"] = {"ms": round(dt * 1e3, 2), "iters": it, "us_per_iter": round(dt * 1e6 / it, 1),
                                                  "state_GBps": round(6.0 * n * k * it / dt / 1e9, 1)}
        # the step between quantizer and path: ptqtp_pack / ptqtp_unpack on random planes (2 B of int8 + 0.53 B of
        # records per weight, one side read, the other written)
        res["pack"] = {}
        from paper_2509_16989_amd import binding
        lib = binding.raw()
        for n, k in ((4096, 4096), (28672, 8192)):
            T1 = torch.randint(-1, 2, (n, k), device=dev, dtype=torch.int8)
            T2 = torch.randint(-1, 2, (n, k), device=dev, dtype=torch.int8)
            a1 = torch.rand(n, k // 128, device=dev).half()
            a2 = torch.rand(n, k // 128, device=dev).half()
            blob = ptq.ptqtp_pack(T1, T2, a1, a2, check=False)
            o1, o2 = torch.empty_like(T1), torch.empty_like(T2)
            nb = blob.numel()
            calls = {"pack": lambda: lib.ptqtp_pack(T1.data_ptr(), T2.data_ptr(), a1.data_ptr(), a2.data_ptr(), 1, n, k, 128,
                                                    blob.data_ptr(), nb, None, stream.cuda_stream),
                     "unpack": lambda: lib.ptqtp_unpack(blob.data_ptr(), 1, n, k, 128, o1.data_ptr(), o2.data_ptr(), None, None,
                                                        stream.cuda_stream)}
            entry = {}
            for what, call in calls.items():
                us = _graph_time(torch, stream, lambda: [call() for _ in range(4)], 4, reps=3 if quick else 10)
                entry[what + "_us"] = round(us, 1)
                entry[what + "_GBps"] = round((2 * n * k + nb) / us / 1e3, 1)
            assert torch.equal(o1, T1) and torch.equal(o2, T2)
            res["pack"][f"{n}x{k}"] = entry
            del T1, T2, o1, o2, blob
        note("pack done")
    if not no_cpu:
        import numpy as np
        import oracle
        Wh = (np.random.default_rng(1).standard_normal((256, 4096)) * 0.02).astype(np.float16)
        t0 = time.perf_counter()
        q = oracle.quantize(Wh)
        dt = time.perf_counter() - t0
        res["quantize"]["cpu_oracle_256x4096"] = {"ms": round(dt * 1e3, 1), "iters": q["iters"], "cores": 1,
                                                  "ns_per_weight_iter": round(dt * 1e9 / (256 * 4096 * q["iters"]), 2)}
    return res


def build_decode_chain(ptq, torch, blobs, jobs, dims):
    """The stack's linears as a dependent decode chain: per layer qkv -> o (+residual) -> gate|up
    (silu(gate)*up) -> down (+residual), fp16 activations, one level per stage.  The q|k|v and gate|up blobs
    are fused on the device (unpack, stack the rows, pack).  The scales of o and down are multiplied by 1/8
    and 1/32 so that the residual stream of 32 random layers stays finite.  Attention itself is not part of
    the path: o reads the q part of qkv's output.  Returns (stages, x0, algorithmic bytes per step)."""
    dev = blobs[0].device
    by = {(layer, name): i for i, (layer, name) in enumerate(jobs)}
    layers = 1 + max(layer for layer, _ in jobs)

    def parts(layer, names, scale=None):
        T1, T2, a1, a2 = [], [], [], []
        for nm in names:
            i = by[(layer, nm)]
            t1, t2, s1, s2 = ptq.ptqtp_unpack(blobs[i], dims[i][0], dims[i][1])
            T1.append(t1); T2.append(t2); a1.append(s1); a2.append(s2)
        cat = [torch.cat(v) for v in (T1, T2, a1, a2)]
        if scale is not None:
            cat[2] = cat[2] * scale
            cat[3] = cat[3] * scale
        return ptq.ptqtp_pack(*cat, check=False), cat[0].shape[0], cat[0].shape[1]

    H = dims[by[(0, "q")]][1]
    x0 = torch.randn(H, device=dev).half()
    stages, cur, level, nbytes = [], x0, 0, 0
    for layer in range(layers):
        fused = {"qkv": parts(layer, ("q", "k", "v")), "o": parts(layer, ("o",), CHAIN_O_SCALE),
                 "gu": parts(layer, ("gate", "up")), "dn": parts(layer, ("down",), CHAIN_DOWN_SCALE)}
        I = fused["gu"][1] // 2
        t_qkv = torch.zeros(fused["qkv"][1], dtype=torch.float16, device=dev)
        t_attn = torch.zeros(H, dtype=torch.float16, device=dev)
        t_h = torch.zeros(I, dtype=torch.float16, device=dev)
        t_out = torch.zeros(H, dtype=torch.float16, device=dev)
        for key, xin, yout, resid, epi in (("qkv", cur, t_qkv, None, ptq.PTQTP_EPI_NONE), ("o", t_qkv, t_attn, cur, ptq.PTQTP_EPI_NONE),
                                          ("gu", t_attn, t_h, None, ptq.PTQTP_EPI_SWIGLU), ("dn", t_h, t_out, t_attn, ptq.PTQTP_EPI_NONE)):
            b, n, k = fused[key]
            stages.append(dict(packed=b, x=xin, y=yout, N=n, K=k, level=level, residual=resid, epilogue=epi))
            nbytes += algorithmic_bytes(n, k, 1)
            level += 1
        cur = t_out
    return stages, x0, nbytes


class DecodeChain:
    """The dependent decode step over the whole stack (build_decode_chain), captured once in a hipGraph."""

    def __init__(self, ptq, torch, blobs, jobs, dims, stream):
        self.ptq, self.torch, self.stream = ptq, torch, stream
        self.stages, self.x0, self.nbytes = build_decode_chain(ptq, torch, blobs, jobs, dims)
        self.launches = len(self.stages)
        self.layers = self.launches // 4
        self.plan = ptq.ptqtp_chain_plan(self.stages)
        ptq.ptqtp_chain_run(self.plan)
        stream.synchronize()
        self.graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self.graph, stream=stream):
            ptq.ptqtp_chain_run(self.plan)
        self.replay = self.graph.replay

    def self_check(self) -> bool:
        """Product-side consistency (no oracle here; the parity test of this chain lives in tests/): every stage of
        the first and the last layer, recomputed from the fp16 input the chain gave it with a plain ptqtp_gemv call
        and the epilogue in torch, must agree with what the chain stored to within fp16 rounding of the output."""
        ptq, torch = self.ptq, self.torch
        self.replay()
        self.stream.synchronize()
        ok = bool(all(torch.isfinite(st["y"].float()).all() for st in self.stages))
        for li in sorted({0, self.layers - 1}):
            for st in self.stages[4 * li: 4 * li + 4]:
                n, k = st["N"], st["K"]
                y = ptq.ptqtp_gemv(st["packed"], st["x"][:k].contiguous(), n, k)[0]
                if st["epilogue"] == ptq.PTQTP_EPI_SWIGLU:
                    y = torch.nn.functional.silu(y[: n // 2]) * y[n // 2:]
                if st["residual"] is not None:
                    y = y + st["residual"].float()
                got = st["y"].float()
                ok = ok and bool(((got - y).abs() <= 2.0 ** -10 * y.abs() + 1e-3 * y.abs().mean()).all())
        return ok

    def extras(self, quick=False):
        """The same chain at 16 tokens per stage and for a 512-token prompt (ptqtp_chain_run_batch); o reads a buffer
        of its own there (with several tokens the q part of qkv's output is not a contiguous [M, K] matrix), the
        launches stay in stream order."""
        ptq, torch, stream = self.ptq, self.torch, self.stream
        dev = self.x0.device

        def chain_at(M, steps, warmup, fused=False):
            stages_m, prev = [], None
            for i, st in enumerate(self.stages):
                n_out = st["N"] // 2 if st["epilogue"] == ptq.PTQTP_EPI_SWIGLU else st["N"]
                ym = torch.zeros((M, n_out), dtype=torch.float16, device=dev)
                xm = (torch.randn(M, st["K"], device=dev) * 0.5).half() if i % 4 == 1 or prev is None else prev
                resid = None if st["residual"] is None else torch.zeros((M, n_out), dtype=torch.float16, device=dev)
                stages_m.append(dict(packed=st["packed"], x=xm, y=ym, N=st["N"], K=st["K"], level=st["level"], residual=resid,
                                     epilogue=st["epilogue"], fused_planes=fused))
                prev = ym
            plan_m = ptq.ptqtp_chain_plan(stages_m)
            ptq.ptqtp_chain_run_batch(plan_m, M)
            stream.synchronize()
            gm = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gm, stream=stream):
                ptq.ptqtp_chain_run_batch(plan_m, M)
            return time_steps(torch, lambda: gm.replay(), steps, warmup, stream)

        ms = time_steps(torch, self.replay, 5 if quick else 100, 2 if quick else 20, stream)
        out = {"us_per_step": round(ms * 1e3, 1), "GBps": round(self.nbytes / ms / 1e6, 1), "launches": self.launches,
               "layers": self.layers}
        out["M16_us_per_step"] = round(chain_at(16, 5 if quick else 50, 2 if quick else 10) * 1e3, 1)
        out["M512_us_per_step"] = round(chain_at(512, 3 if quick else 10, 1 if quick else 3) * 1e3, 1)
        out["M512_fused_planes_us_per_step"] = round(chain_at(512, 3 if quick else 10, 1 if quick else 3, fused=True) * 1e3, 1)
        return out


def cpu_baseline(layer0, names):
    """The fp64 oracle, as it stands, on the host cores: layer 0's seven linears at batch 1, once on all the
    threads the box gives a one-GPU job (at most 16) and once on a single thread."""
    import oracle
    import workloads

    nproc = os.cpu_count() or 1
    threads = min(16, nproc)
    xs = {name: workloads.x_for(name, 1, layer0[name]["K"], 1, 0) for name in names}
    layer_bytes = sum(algorithmic_bytes(layer0[n]["N"], layer0[n]["K"]) for n in names)

    def one_pass(nthreads):
        t = time.perf_counter()
        for name in names:
            lin = layer0[name]
            oracle.forward(lin["T1"], lin["T2"], lin["a1"], lin["a2"], xs[name], threads=nthreads, want_bound=False)
        return time.perf_counter() - t

    # at least 3 passes and about 16 CPU-seconds of oracle work (wall time x threads), at most 12 s of wall clock
    t_start, times = time.perf_counter(), []
    while time.perf_counter() - t_start < 12.0 and (len(times) < 3 or sum(times) * threads < 16.0):
        times.append(one_pass(threads))
    t_start, single = time.perf_counter(), []
    while time.perf_counter() - t_start < 8.0 and len(single) < 3:
        single.append(one_pass(1))
    per_layer = sum(times) / len(times)
    return {"value": round(layer_bytes / per_layer / 1e9, 3), "unit": "GB/s", "cores": threads, "kind": "oracle",
            "sample": f"layer 0 of the stack (seven 8B-shaped linears, batch 1), {len(times)} pass(es), "
                      f"{per_layer * 1e3:.0f} ms per layer (median {sorted(times)[len(times) // 2] * 1e3:.0f}, "
                      f"min {min(times) * 1e3:.0f}), {sum(times) * threads:.0f} CPU-seconds in all; "
                      "same algorithmic bytes as the GPU figure",
            "nproc": nproc,
            "single_thread": {"value": round(layer_bytes / (sum(single) / len(single)) / 1e9, 4), "unit": "GB/s",
                              "cores": 1, "passes": len(single), "ms_per_layer": round(sum(single) / len(single) * 1e3)},
            "us_per_decode_step_extrapolated_x32": round(per_layer * 32 * 1e6)}


if __name__ == "__main__":
    sys.exit(main())
