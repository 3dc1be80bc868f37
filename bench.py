#!/usr/bin/env python3
"""Benchmark of the fused Quantized-Adam-with-error-feedback step on one MI355X.

A "step" is one pass of the whole hot path (error-feedback add, per-layer scales, Q_g + residual
for all N workers, mean, Adam moments, parameter step, Q_x with weight error feedback) through
qadam_step_fused over one batch of synthetic gradients that is already resident in HBM.

Prints ONE JSON line: parameters updated per second (value), ms per step, the HBM roofline of the
dominant kernel (the fused main pass, timed with HIP events inside the library on the stream it is
launched on) and the CPU oracle timed on a bounded sample of the same workload.

The step is timed with the library's filtered scale pass (qadam_trust_error_buffers: the error
buffers belong to the optimizer between steps, so the scales, bit for bit the same, need e only
where |g| can still reach the layer's maximum); the same number of steps is then timed with the
option off and reported beside it (config.same_steps_with_full_scale_pass).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X published HBM3E bandwidth

# HBM bytes per launch of the fused main pass on the default workload (config 5), from two
# rocprofv3 --pmc runs (FETCH_SIZE x 2.0, WRITE_SIZE x 1.0 after scaling by a 4 GiB copy of known
# traffic); summary in profiles/fused_step_gpt1p3b_pmc_traffic.txt.  Other workloads: not measured.
MEASURED_TRAFFIC_BYTES = {5: 174.33e9}


def algorithmic_bytes_per_param(N, code_bits, wcode_bytes, weight_ef):
    """Bytes the method itself must move per parameter in the fused main pass, one trip per buffer:
    per worker read g and e, write e and the packed code; server read and write m, v, x, read and
    write (or only write) e^x, write the weight code.  code_bits == 0: Q_g is the identity (the
    workers' gradients are read, nothing else); wcode_bytes == 0: Q_x is the identity."""
    worker = 12.0 + code_bits / 8.0 if code_bits else 4.0
    server = 24.0 + ((8.0 if weight_ef else 4.0) + wcode_bytes if wcode_bytes else 0.0)
    return N * worker + server


def cpu_baseline(wl, sample_layers, seconds_hint=20.0):
    """The oracle as it stands, one thread, on a bounded sample of the workload's layers; then the same
    calls once more spread over the host's cores (layers are independent), as a second figure."""
    import torch
    from concurrent.futures import ThreadPoolExecutor
    from oracle import qadam_oracle as oracle
    offs = wl.seg_offsets
    N = wl.num_workers
    std = wl.layer_std()
    ocfg = oracle.OracleConfig(k_g=wl.k_g, k_x=wl.k_x, weight_ef=wl.weight_ef, beta1=wl.beta1, eps=wl.eps)
    g = torch.Generator().manual_seed(1234)

    def inputs(l):
        n = offs[l + 1] - offs[l]
        s = float(std[l])
        shared = torch.randn(n, generator=g) * s
        grads = [(shared + torch.randn(n, generator=g) * (0.5 * s)).numpy() for _ in range(N)]
        errs = [(torch.randn(n, generator=g) * (0.2 * s)).numpy() for _ in range(N)]
        x = (torch.randn(n, generator=g) * 0.02).numpy()
        m = (torch.randn(n, generator=g) * (0.3 * s)).numpy()
        v = (torch.randn(n, generator=g) * s).square().numpy()
        w = ((torch.rand(n, generator=g) - 0.5) * 2.0 ** -(wl.k_x + 1)).numpy()
        return n, grads, errs, x, m, v, w

    def step(l, data):
        n, grads, errs, x, m, v, w = data
        oracle.step_s(ocfg, [0, n], 3, wl.lr, wl.beta2, grads, errs, x, m, v, w, index_base=offs[l], want_tie=False)

    total, elapsed = 0, 0.0
    used, kept = [], []
    for l in sample_layers:
        data = inputs(l)
        t0 = time.perf_counter()
        step(l, data)
        elapsed += time.perf_counter() - t0
        total += data[0]
        used.append(l)
        kept.append((l, data))
        if elapsed > seconds_hint:
            break
    out = {"value": total / elapsed, "unit": "params/s", "cores": 1, "kind": "oracle",
           "sample": "one oracle step (variant S, %d workers) over layers %s of the workload = %d parameters, %.1f s"
                     % (N, used, total, elapsed)}
    # the same layers again (one more step from the state the first left), one layer per thread
    threads = min(16, os.cpu_count() or 1, len(kept))
    if threads > 1:
        t0 = time.perf_counter()
        with ThreadPoolExecutor(threads) as ex:
            list(ex.map(lambda ld: step(*ld), kept))
        dt = time.perf_counter() - t0
        out["all_cores"] = {"value": total / dt, "unit": "params/s", "cores": threads,
                            "note": "the same oracle calls, independent layers on %d threads, %.1f s" % (threads, dt)}
    return out


def condition_allocator(nbytes_list, cycles, device):
    """Allocate and free the working set `cycles` times without touching it.

    On a freshly provisioned box the driver hands out device memory in physical address order, and
    the main pass (20 read + 13 write streams at a fixed distance from each other) runs ~12 % slower
    on that placement than on the placement any later process gets once allocations have been freed
    and reused (the scale pass, read only, is ~5 % faster on it).  Cycling the allocations puts the
    driver's free lists into that used state, so the timed run measures the steady state of a
    machine that has run jobs before rather than the first minute after provisioning."""
    import gc
    import torch
    for _ in range(cycles):
        bufs = [torch.empty(n, dtype=torch.uint8, device=device) for n in nbytes_list]
        del bufs
        gc.collect()
        torch.cuda.empty_cache()
    torch.cuda.synchronize()


def measure_ceilings(dev):
    """Plain torch streams over 6 GiB, best of 5, HIP events on torch's current stream."""
    import torch
    n = (6 << 30) // 4
    t = torch.zeros(n, dtype=torch.float32, device=dev)
    half = n // 2

    def best(fn):
        ms = []
        for _ in range(5):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(); fn(); b.record()
            torch.cuda.synchronize()
            ms.append(a.elapsed_time(b))
        return min(ms)

    inplace = best(lambda: t.mul_(1.0))
    copy = best(lambda: t[half:].copy_(t[:half]))
    fill = best(lambda: t.fill_(1.0))
    del t
    torch.cuda.empty_cache()
    return {"inplace_update_GBs": round(2 * 4 * n / inplace / 1e6, 1),
            "device_copy_GBs": round(2 * 4 * half / copy / 1e6, 1),
            "fill_GBs": round(4 * n / fill / 1e6, 1),
            "note": "torch x.mul_(1.0) over 6 GiB (reads + writes counted), a 3 GiB -> 3 GiB copy, x.fill_(1.0) over 6 GiB"}


def bench_calls(args, wl, q, grads, errs, codes, scales, x, m, v, werr, wcodes, code_bits, wcode_bytes):
    """The step as the three separate entry points; each group of launches is timed with HIP events
    on the stream the library launches on (torch's current stream)."""
    import torch
    P, N = wl.num_params, wl.num_workers
    ev = lambda: torch.cuda.Event(enable_timing=True)
    step_ms, part_ms = [], []
    for t in range(1, args.warmup + args.steps + 1):
        wl.fill_gradients(t, grads)
        torch.cuda.synchronize()
        e0, e1, e2, e3 = ev(), ev(), ev(), ev()
        t0 = time.perf_counter()
        e0.record()
        for i in range(N):
            q.worker_quantize(i, t, grads[i], errs[i], codes[i], scales[i])
        e1.record()
        q.server_step(t, wl.lr, wl.beta2, codes, scales, x, m, v)
        e2.record()
        q.weight_quantize(t, x, werr, wcodes)
        e3.record()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) * 1e3
        if t > args.warmup:
            step_ms.append(dt)
            part_ms.append((e0.elapsed_time(e1), e1.elapsed_time(e2), e2.elapsed_time(e3)))
    ms_per_step = sum(step_ms) / len(step_ms)
    w_ms, s_ms, x_ms = (sum(p[k] for p in part_ms) / len(part_ms) for k in range(3))
    filt = args.scale_pass == "filtered"               # the scale read is g only (plus the few e that matter)
    a_worker = N * ((4.0 if filt else 8.0) + 12.0 + code_bits / 8.0)   # scale read; then g, e in, e and code out
    a_server = N * code_bits / 8.0 + 24.0             # codes in; m, v, x in and out
    a_weight = 4.0 + 8.0 + wcode_bytes                # x in; e^x in and out; weight code out
    gbs = lambda a, ms: round(a * P / (ms * 1e-3) / 1e9, 1)
    out = {
        "metric": "parameters updated/sec (full QAdam-EF step)",
        "value": P / (ms_per_step * 1e-3), "unit": "params/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "config %d: %s, %d logical workers, %d parameters, the step as %d x "
                               "qadam_worker_quantize + qadam_server_step + qadam_weight_quantize"
                               % (wl.config, wl.name, N, P, N),
                   "status_word": q.get_status()},
        "roofline": {"bound": "hbm", "kernel": "qadam_worker_quantize x %d (k_amax + k_worker_quantize per worker)" % N,
                     "achieved": gbs(a_worker, w_ms), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(gbs(a_worker, w_ms) / HBM_PEAK_GBS, 4), "traffic": None,
                     "algorithmic_bytes_per_param": a_worker, "avg_launch_ms": round(w_ms, 4),
                     "server_step": {"algorithmic_bytes_per_param": a_server, "avg_launch_ms": round(s_ms, 4),
                                     "achieved": gbs(a_server, s_ms)},
                     "weight_quantize": {"algorithmic_bytes_per_param": a_weight, "avg_launch_ms": round(x_ms, 4),
                                         "achieved": gbs(a_weight, x_ms)}},
    }
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=5, help="workload 1..5 (default: the 1.3B headline)")
    ap.add_argument("--shrink", type=int, default=1, help="divide model dims (debugging only)")
    ap.add_argument("--variant", choices=["s", "w"], default="s",
                    help="s: workers quantize g+e, server owns the moments (the headline path); "
                         "w: Algorithms 2-3 as printed, workers own the moments (qadam_step_fused_w)")
    ap.add_argument("--path", choices=["fused", "calls"], default="fused",
                    help="fused: qadam_step_fused (the headline); calls: the same step as N x "
                         "qadam_worker_quantize + qadam_server_step + qadam_weight_quantize (variant S only)")
    ap.add_argument("--rounding", type=int, choices=[0, 1], default=0,
                    help="0: nearest (the paper's quantizers, the headline); 1: unbiased stochastic rounding "
                         "driven by Philox4x32-10")
    ap.add_argument("--scale-pass", choices=["full", "filtered"], default="filtered",
                    help="full: the scale pass reads g and e of every element; filtered: "
                         "qadam_trust_error_buffers(1), it reads e only where |g| can still reach the layer's "
                         "maximum (same results; the error buffers are the library's between steps)")
    ap.add_argument("--graph", action="store_true",
                    help="capture the step in a HIP graph after the warm-up and time replays of it (pays on "
                         "launch-bound workloads such as config 1; kernels are then not timed one by one)")
    ap.add_argument("--no-full-comparison", action="store_true",
                    help="with the filtered scale pass: do not time the same steps again with the full one "
                         "(for profiles of one mode)")
    ap.add_argument("--k-g", type=int, default=None,
                    help="override the workload's gradient grid (0: 2-bit codes, 1-2: 3-bit, 3-6: 4-bit, "
                         "-1: no gradient quantization)")
    ap.add_argument("--k-x", type=int, default=None,
                    help="override the workload's weight grid (0-6: int8, 7-14: int16, -1: no weight quantization)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--alloc-cycles", type=int, default=5,
                    help="allocate and free the working set this many times before the real allocation "
                         "(0: measure on whatever placement a fresh process gets; see condition_allocator)")
    ap.add_argument("--ceilings", action="store_true",
                    help="also time plain torch streams over 6 GiB (an in-place update: half reads, half "
                         "writes; a device copy) and add them to the JSON line as memory_system: what "
                         "this box delivers to the simplest kernels, next to the 8 TB/s peak")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 4 GiB device copy (a kernel of known traffic, to scale "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (logical workers are in-memory shards of one "
                 "device); --gpus %d is not supported" % args.gpus)

    import torch
    from paper_2004_14180_amd import QAdam, QAdamConfig
    from paper_2004_14180_amd.workloads import make_workload

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    wl = make_workload(args.config, shrink=args.shrink)
    if args.k_g is not None:
        wl.k_g = args.k_g
    if args.k_x is not None:
        wl.k_x = args.k_x
    P, N = wl.num_params, wl.num_workers
    weight_ef = 1
    cfg = QAdamConfig(k_g=wl.k_g, k_x=wl.k_x, rounding=args.rounding, weight_ef=weight_ef, beta1=wl.beta1,
                      eps=wl.eps)
    q = QAdam(cfg, wl.seg_offsets, N)
    q.profile_enable(not args.graph)
    if args.scale_pass == "filtered":
        q.trust_error_buffers(True)
    code_bits = q.grad_code_bytes() * 8.0 / P
    wcode_bytes = q.weight_code_bytes() / P

    n_f32 = 4 + 2 * N + (2 * N if args.variant == "w" else 0)
    working_set = [4 * P] * n_f32 + [q.grad_code_bytes()] * N + [q.weight_code_bytes()]
    if args.alloc_cycles > 0:
        condition_allocator(working_set, args.alloc_cycles, dev)

    z = lambda: torch.zeros(P, dtype=torch.float32, device=dev)
    x = wl.init_weights(dev)
    m, v, werr = z(), z(), z()
    errs = [z() for _ in range(N)]
    grads = [torch.empty(P, dtype=torch.float32, device=dev) for _ in range(N)]
    if args.variant == "w":
        mw = [z() for _ in range(N)]
        vw = [z() for _ in range(N)]
    codes = [torch.empty(max(q.grad_code_bytes() // 4, 4), dtype=torch.int32, device=dev) for _ in range(N)]
    scales = [torch.empty(q.num_segments, dtype=torch.float32, device=dev) for _ in range(N)]
    wcodes = torch.empty(P, dtype=torch.int8 if wl.k_x <= 6 else torch.int16, device=dev)

    if args.copy_calibration:
        src = torch.ones(1 << 30, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)                      # reads 4 GiB, writes 4 GiB
        torch.cuda.synchronize()
        del src, dst

    memory_system = measure_ceilings(dev) if args.ceilings else None

    if args.path == "calls":
        if args.variant != "s":
            sys.exit("bench.py: --path calls is for variant S")
        return bench_calls(args, wl, q, grads, errs, codes, scales, x, m, v, werr, wcodes, code_bits, wcode_bytes)

    def step_call(t):
        if args.variant == "s":
            q.step_fused(t, wl.lr, wl.beta2, grads, errs, codes, scales, x, m, v, werr, wcodes)
        else:
            q.step_fused_w(t, wl.lr, wl.beta2, grads, mw, vw, errs, codes, scales, x, werr, wcodes)

    def timed_steps(first, warmup, steps):
        """`warmup` untimed then `steps` timed steps; each timed between two device synchronisations,
        with the step's gradients already resident.  Returns per-step (wall, scale pass, main pass) ms."""
        out = []
        graph = None
        for t in range(first, first + warmup + steps):
            wl.fill_gradients(t, grads)        # untimed: inputs are resident before the clock starts
            torch.cuda.synchronize()
            if args.graph and graph is None and t >= first + warmup:
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph):  # capture only records: nothing runs, no state changes
                    step_call(t)
                torch.cuda.synchronize()
            t0 = time.perf_counter()
            if graph is not None:
                graph.replay()
            else:
                step_call(t)
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t0) * 1e3
            # per-pass HIP events are not recorded into a graph: split the wall time evenly as a placeholder
            a, b = (dt / 2, dt / 2) if args.graph else q.profile_read()
            if t >= first + warmup:
                out.append((dt, a, b))
        return out

    # the library applies the filter from about four million worker-elements on (4096 tiles of 4096)
    tiles = sum((n + 4095) // 4096 for n in wl.sizes)
    filtered = args.scale_pass == "filtered" and args.variant == "s" and wl.k_g >= 0 and tiles * N >= 4096
    res = timed_steps(1, args.warmup, args.steps)
    step_ms, scale_ms, main_ms = ([r[k] for r in res] for k in range(3))
    full_pass = None
    if filtered and not args.no_full_comparison:
        # the same steps once more with the option off (every element's g and e read for the scales)
        q.trust_error_buffers(False)
        res_full = timed_steps(1 + args.warmup + args.steps, 1, args.steps)
        full_ms = sum(r[0] for r in res_full) / len(res_full)
        full_pass = {"ms_per_step": round(full_ms, 4), "value": P / (full_ms * 1e-3),
                     "scale_pass_ms": round(sum(r[1] for r in res_full) / len(res_full), 4),
                     "main_pass_ms": round(sum(r[2] for r in res_full) / len(res_full), 4)}
    if os.environ.get("QADAM_BENCH_VERBOSE"):
        print("per-step main ms:", [round(v_, 2) for v_ in main_ms], file=sys.stderr)
        print("per-step scale ms:", [round(v_, 2) for v_ in scale_ms], file=sys.stderr)
    status = q.get_status()
    total_ms = sum(step_ms)
    ms_per_step = total_ms / len(step_ms)
    main_avg = sum(main_ms) / len(main_ms)
    scale_avg = sum(scale_ms) / len(scale_ms)

    gbs = lambda bytes_per_param, ms: round(bytes_per_param * P / (max(ms, 1e-6) * 1e-3) / 1e9, 1)
    if args.variant == "w":
        # first pass (dominant): per worker read g, m_i, v_i, e_i and write m_i, v_i, p = 28 B;
        # second pass: per worker read p, write e and the code; server read/write x and e^x, weight code
        a_first = 28.0 * N
        a_second = N * (8.0 + code_bits / 8.0) + 8.0 + (8.0 if weight_ef else 4.0) + wcode_bytes
        roofline = {"bound": "hbm", "kernel": "k_moments_w (first pass of qadam_step_fused_w)",
                    "achieved": gbs(a_first, scale_avg), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(gbs(a_first, scale_avg) / HBM_PEAK_GBS, 4), "traffic": None,
                    "algorithmic_bytes_per_param": a_first, "avg_launch_ms": round(scale_avg, 4),
                    "second_pass": {"algorithmic_bytes_per_param": a_second, "avg_launch_ms": round(main_avg, 4),
                                    "achieved": gbs(a_second, main_avg)},
                    "whole_step_GBs": gbs(a_first + a_second, ms_per_step)}
    else:
        a_main = algorithmic_bytes_per_param(N, code_bits, wcode_bytes, weight_ef)
        # scale pass: g and e of every worker; filtered: g, plus e of the few elements that can be the maximum
        a_scale = (4.0 if filtered else 8.0) * N if code_bits else 0.0
        headline = args.shrink == 1 and args.k_g is None and args.k_x is None and args.rounding == 0
        roofline = {"bound": "hbm", "kernel": "k_fused (main pass of qadam_step_fused)",
                    "achieved": gbs(a_main, main_avg), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(gbs(a_main, main_avg) / HBM_PEAK_GBS, 4),
                    "traffic": MEASURED_TRAFFIC_BYTES.get(args.config) if headline else None,
                    "algorithmic_bytes_per_param": a_main, "avg_launch_ms": round(main_avg, 4),
                    "scale_pass": {"mode": "filtered" if filtered else "full",
                                   "algorithmic_bytes_per_param": a_scale, "avg_launch_ms": round(scale_avg, 4),
                                   "achieved": gbs(a_scale, scale_avg)},
                    "whole_step_GBs": gbs(a_main + a_scale, ms_per_step),
                    # the method's own minimum (every buffer once, no read for the scales) over the step time
                    "a_min_over_step_GBs": gbs(a_main, ms_per_step)}

    if args.graph:
        # the passes are not timed one by one inside a graph: report the whole step against the roofline
        whole = roofline["whole_step_GBs"]
        roofline = {"bound": "hbm", "kernel": "whole step (HIP graph replay)", "achieved": whole,
                    "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(whole / HBM_PEAK_GBS, 4), "traffic": None,
                    "avg_launch_ms": round(ms_per_step, 4)}
    out = {
        "metric": "parameters updated/sec (full QAdam-EF step)",
        "value": P / (ms_per_step * 1e-3),
        "unit": "params/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "config %d: %s, %d logical workers, %d parameters in %d layers, "
                               "k_g=%d (%d-bit codes), k_x=%d (%d-bit weights; 0 bits = quantizer off), weight_ef=1, %s rounding, %s"
                               % (wl.config, wl.name, N, P, len(wl.sizes), wl.k_g, round(code_bits), wl.k_x,
                                  8 * round(wcode_bytes), "stochastic (Philox)" if args.rounding else "nearest",
                                  "variant S (server moments)" if args.variant == "s" else
                                  "variant W (worker moments, Algorithms 2-3)"),
                   "worker_elements_per_s": N * P / (ms_per_step * 1e-3),
                   "resident_bytes": sum(working_set),
                   "allocator_conditioning_cycles": args.alloc_cycles,
                   "hip_graph_replay": bool(args.graph),
                   "scale_pass": "filtered: exact scales, e read only where |g| can reach the layer maximum "
                                 "(qadam_trust_error_buffers)" if filtered else "full: g and e of every element",
                   "same_steps_with_full_scale_pass": full_pass,
                   "status_word": status},
        "roofline": roofline,
    }
    if not args.no_cpu_baseline and args.variant == "s" and args.rounding == 0 and wl.k_g >= 0 and wl.k_x >= 0:
        # a bounded sample: the first layers after the token embedding, up to ~75 M parameters
        # (about 10 s of single-threaded oracle work); stops early after ~25 s
        sizes = wl.sizes
        pick, tot = [], 0
        for l in range(len(sizes)):
            if 0 < sizes[l] <= 20_000_000 and tot < 75_000_000:
                pick.append(l); tot += sizes[l]
        out["cpu_baseline"] = cpu_baseline(wl, pick or [0], seconds_hint=25.0)
    if memory_system:
        out["memory_system"] = memory_system
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
