#!/usr/bin/env python3
"""Benchmark of the fused Quantized-Adam-with-error-feedback step on one MI355X.

A "step" is one pass of the whole hot path (error-feedback add, per-layer scales, Q_g + residual
for all N workers, mean, Adam moments, parameter step, Q_x with weight error feedback) through
qadam_step_fused over one batch of synthetic gradients that is already resident in HBM.

Prints ONE JSON line: parameters updated per second (value), ms per step, the HBM roofline of the
dominant kernel (the fused main pass, timed with HIP events inside the library on the stream it is
launched on) and of the whole step, the same steps in the library's default mode, the other
workloads side by side, and the CPU oracle timed (and compared) on a bounded sample of the workload.

Two set-up choices are part of the headline and are reported next to it:
  * scale pass: the step is timed with the library's filtered scale pass (qadam_trust_error_buffers:
    an opt-in whose contract is that the error buffers belong to the optimizer between steps; the
    scales, bit for bit the same, then need e only where |g| can still reach the layer's maximum).
    The same number of steps is timed again with the option off: value_full_scale_pass.
  * placement: the buffers are carved out of ONE allocation at the offsets qadam_arena_layout gives
    (every second buffer in the far half of the block), which keeps the step's 33 concurrent streams
    from falling into one third of the device's memory.  --placement separate allocates every buffer
    on its own instead, as a caller without the layout would.
"""
import argparse
import hashlib
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X published HBM3E bandwidth
KERNEL_SOURCE = os.path.join(ROOT, "paper_2004_14180_amd", "csrc", "qadam_kernels.hip")
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "fused_step_gpt1p3b_pmc_traffic.txt")


def measured_traffic_bytes(key="k_fused_traffic_bytes_per_launch"):
    """HBM bytes of the headline workload's kernels as the rocprofv3 counter summary under profiles/ records
    them (per launch of the fused main pass; per step for the scale pass) -- only if that summary was taken
    from the kernel source that is being timed now (it stores the source's SHA-256); otherwise None."""
    try:
        text = open(TRAFFIC_PROFILE).read()
        m_sha = re.search(r"^kernel_source_sha256:\s*([0-9a-f]{64})", text, re.M)
        m_val = re.search(r"^%s:\s*([0-9.eE+]+)" % re.escape(key), text, re.M)
        if not m_sha or not m_val:
            return None
        if hashlib.sha256(open(KERNEL_SOURCE, "rb").read()).hexdigest() != m_sha.group(1):
            return None
        return float(m_val.group(1))
    except OSError:
        return None


def algorithmic_bytes_per_param(N, code_bits, wcode_bytes, weight_ef):
    """Bytes the method itself must move per parameter in the fused main pass, one trip per buffer:
    per worker read g and e, write e and the packed code; server read and write m, v, x, read and
    write (or only write) e^x, write the weight code.  code_bits == 0: Q_g is the identity (the
    workers' gradients are read, nothing else); wcode_bytes == 0: Q_x is the identity."""
    worker = 12.0 + code_bits / 8.0 if code_bits else 4.0
    server = 24.0 + ((8.0 if weight_ef else 4.0) + wcode_bytes if wcode_bytes else 0.0)
    return N * worker + server


# ------------------------------------------------------------------------------------------ buffers
class Buffers:
    """Device buffers of one handle: carved out of one block at qadam_arena_layout's offsets, or
    allocated one by one."""

    def __init__(self, q, wl, dev, placement, variant_w=False, reserve_bytes=24 << 30):
        import torch
        P, N, L = wl.num_params, wl.num_workers, q.num_segments
        self.placement = placement
        self.arena = None
        wdt = torch.int8 if wl.k_x <= 6 else torch.int16
        ncode = max(q.grad_code_bytes() // 4, 4)
        if placement == "arena":
            need = q.arena_layout(1 << 60, variant_w)["bytes_needed"]
            free_b, _ = torch.cuda.mem_get_info()
            # as large as the device allows (the two groups of buffers then lie far apart), leaving room
            # for the generator's temporaries
            arena_bytes = max(need, free_b - reserve_bytes)
            try:
                self.arena = torch.empty(arena_bytes, dtype=torch.uint8, device=dev)
            except RuntimeError:                      # the device cannot give one block of that size
                torch.cuda.empty_cache()
                placement = self.placement = "separate (one block of %d bytes was refused)" % arena_bytes
        if self.arena is not None:
            lay = q.arena_layout(arena_bytes, variant_w)
            self.arena_bytes = arena_bytes
            f32 = lambda off, n: self.arena[off:off + 4 * n].view(torch.float32)
            self.x, self.m, self.v, self.werr = (f32(lay[k], P) for k in ("x", "m", "v", "werr"))
            self.errs = [f32(o, P) for o in lay["errs"]]
            self.grads = [f32(o, P) for o in lay["grads"]]
            self.codes = [self.arena[o:o + 4 * ncode].view(torch.int32) for o in lay["codes"]] \
                if q.grad_code_bytes() else [torch.empty(4, dtype=torch.int32, device=dev) for _ in range(N)]
            self.scales = [f32(o, max(L, 1)) for o in lay["scales"]]
            nb = max(q.weight_code_bytes(), 4)
            self.wcodes = self.arena[lay["wcodes"]:lay["wcodes"] + nb].view(wdt)
            if variant_w:
                self.mw = [f32(o, P) for o in lay["mw"]]
                self.vw = [f32(o, P) for o in lay["vw"]]
            for t in [self.m, self.v, self.werr] + self.errs + (self.mw + self.vw if variant_w else []):
                t.zero_()
            self.x.copy_(wl.init_weights(dev))
        else:
            self.arena_bytes = 0
            z = lambda: torch.zeros(P, dtype=torch.float32, device=dev)
            self.x = wl.init_weights(dev)
            self.m, self.v, self.werr = z(), z(), z()
            self.errs = [z() for _ in range(N)]
            self.grads = [torch.empty(P, dtype=torch.float32, device=dev) for _ in range(N)]
            if variant_w:
                self.mw = [z() for _ in range(N)]
                self.vw = [z() for _ in range(N)]
            self.codes = [torch.empty(ncode, dtype=torch.int32, device=dev) for _ in range(N)]
            self.scales = [torch.empty(max(L, 1), dtype=torch.float32, device=dev) for _ in range(N)]
            self.wcodes = torch.empty(max(P, 4), dtype=wdt, device=dev)


def condition_allocator(nbytes_list, cycles, device):
    """Allocate and free the working set `cycles` times without touching it (--placement separate only;
    off by default).  On a freshly provisioned box the driver hands out device memory in physical address
    order; cycling the allocations puts its free lists into the scattered state every later process sees."""
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
            "note": "torch x.mul_(1.0) over 6 GiB (reads + writes counted), a 3 GiB -> 3 GiB copy, x.fill_(1.0) over "
                    "6 GiB; the hand-written probes of the step's own access patterns are "
                    "paper_2004_14180_amd/qadam_probe.bin (summary under profiles/)"}


# ---------------------------------------------------------------------------------------- utilities
def bench_utilities(wl, dev, reps=5):
    """The kernels around the step (what a worker does with the broadcast weight codes; the norm diagnostic),
    each timed alone with HIP events on the stream the library launches on, against its algorithmic bytes.
    Twice: with one allocation per buffer, and with the buffers spread over one block that spans the device
    (input at 1/4, codes at 1/2, output at 3/4 of it) -- where the buffers lie matters for these kernels as it
    does for the step."""
    import torch
    from paper_2004_14180_amd import QAdam, QAdamConfig
    P, N = wl.num_params, 1

    def timed(fn):
        ms = []
        for _ in range(reps + 1):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(); fn(); b.record()
            torch.cuda.synchronize()
            ms.append(a.elapsed_time(b))
        ms = ms[1:]
        return sum(ms) / len(ms)

    def measure(alloc):
        """alloc(which, dtype) -> a P-element tensor; which in 'in', 'codes', 'out'."""
        out = {}

        def entry(name, bytes_per_param, ms):
            gbs = bytes_per_param * P / (ms * 1e-3) / 1e9
            out[name] = {"avg_launch_ms": round(ms, 4), "algorithmic_bytes_per_param": bytes_per_param,
                         "achieved_GBs": round(gbs, 1), "frac": round(gbs / HBM_PEAK_GBS, 4)}

        x = alloc("in", torch.float32)
        x.copy_(wl.init_weights(dev))
        for k_x, dt in ((6, torch.int8), (14, torch.int16)):
            q = QAdam(QAdamConfig(k_g=wl.k_g, k_x=k_x, weight_ef=0, beta1=wl.beta1, eps=wl.eps), wl.seg_offsets, N)
            wcodes = alloc("codes", dt)
            werr = alloc("out", torch.float32)
            nb = wcodes.element_size()
            entry("qadam_weight_quantize, int%d codes, weight_ef=0 (k_weight_quantize)" % (8 * nb), 8.0 + nb,
                  timed(lambda: q.weight_quantize(1, x, werr, wcodes)))
            xhat = werr                                     # reuse the buffer
            entry("qadam_weight_dequantize, int%d -> fp32 (k_weight_dequantize)" % (8 * nb), 4.0 + nb,
                  timed(lambda: q.weight_dequantize(wcodes, xhat)))
            xh16 = alloc("out", torch.float16)
            entry("qadam_weight_dequantize_f16, int%d -> binary16 (k_weight_dequantize)" % (8 * nb), 2.0 + nb,
                  timed(lambda: q.weight_dequantize_f16(wcodes, xh16)))
            if k_x == 6:
                sums = torch.empty(q.num_segments, dtype=torch.float64, device=dev)
                werr.normal_(0.0, 1e-3)
                entry("qadam_layer_sumsq(a, b) (k_sumsq_tiles + k_sumsq_layers)", 8.0, timed(lambda: q.layer_sumsq(x, werr, sums)))
                entry("qadam_layer_sumsq(a) (k_sumsq_tiles + k_sumsq_layers)", 4.0, timed(lambda: q.layer_sumsq(x, None, sums)))
                del sums
            del wcodes, werr, xh16, xhat
            q.close()
        return out

    result = {"one allocation per buffer": measure(lambda which, dt: torch.empty(P, dtype=dt, device=dev))}
    torch.cuda.empty_cache()
    free_b, _ = torch.cuda.mem_get_info()
    block_bytes = (free_b - (8 << 30)) >> 30 << 30
    try:
        block = torch.empty(block_bytes, dtype=torch.uint8, device=dev)
    except RuntimeError:
        block = None
    if block is not None and block_bytes >= 16 * P:
        where = {"in": block_bytes // 4, "codes": block_bytes // 2, "out": block_bytes // 4 * 3}

        def carve(which, dt):
            nbytes = P * torch.empty(0, dtype=dt).element_size()
            return block[where[which]:where[which] + nbytes].view(dt)
        result["one block of %d bytes: input at 1/4, codes at 1/2, output at 3/4" % block_bytes] = measure(carve)
    del block
    torch.cuda.empty_cache()
    return result


# ------------------------------------------------------------------------------------- CPU baseline
def cpu_baseline(wl, dev, max_params=75_000_000, seconds_hint=25.0):
    """The oracle as it stands, timed on the host next to the GPU library on a bounded sample of the
    workload: the workload's layer list cut down to its first layers after the token embedding (up to
    max_params parameters), the workload's own seeded generators for the gradients and for a synthetic
    mid-training state, one step.  The library makes the same step on the same inputs and the outputs are
    compared, so the line also carries the tie and mismatch counts of this sample."""
    import numpy as np
    import torch
    from concurrent.futures import ThreadPoolExecutor
    from oracle import qadam_oracle as oracle
    from paper_2004_14180_amd import QAdam, QAdamConfig
    from paper_2004_14180_amd.workloads import Workload

    pick, tot = [], 0
    for l, n in enumerate(wl.sizes):
        if 0 < n <= 20_000_000 and tot + n <= max_params:
            pick.append(l); tot += n
    pick = pick or [0]
    sub = Workload(wl.config, wl.name, [wl.sizes[l] for l in pick], wl.num_workers, 1, k_g=wl.k_g, k_x=wl.k_x,
                   weight_ef=1, lr=wl.lr, beta1=wl.beta1, beta2=wl.beta2, eps=wl.eps, seed=wl.seed)
    if wl.config in (3, 4):
        sub.embedding_rows, sub.embedding_dim = 0, 0
    N, P, offs = sub.num_workers, sub.num_params, sub.seg_offsets
    q = QAdam(QAdamConfig(k_g=sub.k_g, k_x=sub.k_x, weight_ef=1, beta1=sub.beta1, eps=sub.eps), offs, N)
    st = sub.synthetic_state(dev)
    x = sub.init_weights(dev)
    grads = [torch.empty(P, dtype=torch.float32, device=dev) for _ in range(N)]
    sub.fill_gradients(1, grads)
    host = lambda t: t.cpu().numpy()
    h = dict(grads=[host(g) for g in grads], errs=[host(e) for e in st["errs"]], x=host(x), m=host(st["m"]),
             v=host(st["v"]), werr=host(st["werr"]))
    h2 = dict(errs=[e.copy() for e in h["errs"]], x=h["x"].copy(), m=h["m"].copy(), v=h["v"].copy(),
              werr=h["werr"].copy())
    codes = [torch.empty(max(q.grad_code_bytes() // 4, 4), dtype=torch.int32, device=dev) for _ in range(N)]
    scales = [torch.empty(len(pick), dtype=torch.float32, device=dev) for _ in range(N)]
    wcodes = torch.empty(P, dtype=torch.int8 if sub.k_x <= 6 else torch.int16, device=dev)
    q.step_fused(3, sub.lr, sub.beta2, grads, st["errs"], codes, scales, x, st["m"], st["v"], st["werr"], wcodes)
    torch.cuda.synchronize()
    status = q.get_status()
    ocfg = oracle.OracleConfig(k_g=sub.k_g, k_x=sub.k_x, weight_ef=1, beta1=sub.beta1, eps=sub.eps)

    def step(l, state):
        a, b = offs[l], offs[l + 1]
        return oracle.step_s(ocfg, [0, b - a], 3, sub.lr, sub.beta2, [g[a:b] for g in h["grads"]],
                             [e[a:b] for e in state["errs"]], state["x"][a:b], state["m"][a:b], state["v"][a:b],
                             state["werr"][a:b], index_base=a)

    outs, elapsed, done = [], 0.0, 0
    for l in range(len(pick)):
        t0 = time.perf_counter()
        outs.append(step(l, h))
        elapsed += time.perf_counter() - t0
        done += offs[l + 1] - offs[l]
        if elapsed > seconds_hint:
            break
    # parity of the sample: gradient and weight codes bit for bit, floats bit for bit
    bits = oracle.grad_code_bits(sub.k_g)
    cmp_ = dict(params_compared=done, ties_g=0, ties_x=0, code_mismatch=0, wcode_mismatch=0, float_bit_diffs=0,
                scale_mismatch=0, status_word=status)
    woff = 0
    dwords = [c.cpu().numpy().view(np.uint32) for c in codes]
    dsc = [s.cpu().numpy() for s in scales]
    dw = wcodes.cpu().numpy()
    dstate = dict(errs=[host(e) for e in st["errs"]], x=host(x), m=host(st["m"]), v=host(st["v"]), werr=host(st["werr"]))
    for l, out in enumerate(outs):
        a, b = offs[l], offs[l + 1]
        nw = len(out["words"][0])
        for i in range(N):
            gc = oracle.unpack_codes(bits, dwords[i][woff:woff + nw], b - a)
            oc = oracle.unpack_codes(bits, out["words"][i], b - a)
            cmp_["code_mismatch"] += int((gc != oc).sum())
            cmp_["ties_g"] += int(np.count_nonzero(out["tie_g"][i]))
            cmp_["scale_mismatch"] += int(dsc[i][l].view(np.uint32) != out["scales"][i][0].view(np.uint32))
            cmp_["float_bit_diffs"] += int((dstate["errs"][i][a:b].view(np.uint32) != h["errs"][i][a:b].view(np.uint32)).sum())
        woff += nw
        cmp_["wcode_mismatch"] += int((dw[a:b] != out["wcodes"]).sum())
        cmp_["ties_x"] += int(np.count_nonzero(out["tie_x"]))
        for k in ("x", "m", "v", "werr"):
            cmp_["float_bit_diffs"] += int((dstate[k][a:b].view(np.uint32) != h[k][a:b].view(np.uint32)).sum())
    res = {"value": done / elapsed, "unit": "params/s", "cores": 1, "kind": "oracle",
           "sample": "one oracle step (variant S, %d workers) over the first %d of the workload's layers after the "
                     "token embedding (layers %d..%d, %d parameters), gradients and a synthetic mid-training state "
                     "from the workload's seeded generators, %.1f s" % (N, len(outs), pick[0], pick[len(outs) - 1],
                                                                          done, elapsed),
           "gpu_vs_oracle_on_this_sample": cmp_}
    # the same layers again from the same start state, one layer per thread
    threads = min(16, os.cpu_count() or 1, len(outs))
    if threads > 1:
        t0 = time.perf_counter()
        with ThreadPoolExecutor(threads) as ex:
            list(ex.map(lambda l: step(l, h2), range(len(outs))))
        dt = time.perf_counter() - t0
        res["all_cores"] = {"value": done / dt, "unit": "params/s", "cores": threads,
                            "note": "the same oracle calls, independent layers on %d threads, %.1f s" % (threads, dt)}
    q.close()
    return res


# ------------------------------------------------------------------------------ the three-call path
def bench_calls(args, wl, q, B, code_bits, wcode_bytes):
    """The step as the three separate entry points; each group of launches is timed with HIP events
    on the stream the library launches on (torch's current stream)."""
    import torch
    P, N = wl.num_params, wl.num_workers
    ev = lambda: torch.cuda.Event(enable_timing=True)
    step_ms, part_ms = [], []
    for t in range(1, args.warmup + args.steps + 1):
        wl.fill_gradients(t, B.grads)
        torch.cuda.synchronize()
        e0, e1, e2, e3 = ev(), ev(), ev(), ev()
        t0 = time.perf_counter()
        e0.record()
        for i in range(N):
            q.worker_quantize(i, t, B.grads[i], B.errs[i], B.codes[i], B.scales[i])
        e1.record()
        q.server_step(t, wl.lr, wl.beta2, B.codes, B.scales, B.x, B.m, B.v)
        e2.record()
        q.weight_quantize(t, B.x, B.werr, B.wcodes)
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
                   "placement": B.placement, "status_word": q.get_status()},
        "roofline": {"bound": "hbm", "kernel": "qadam_worker_quantize x %d (scale kernels + k_worker_quantize per worker)" % N,
                     "achieved": gbs(a_worker, w_ms), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(gbs(a_worker, w_ms) / HBM_PEAK_GBS, 4), "traffic": None,
                     "algorithmic_bytes_per_param": a_worker, "avg_launch_ms": round(w_ms, 4),
                     "server_step": {"algorithmic_bytes_per_param": a_server, "avg_launch_ms": round(s_ms, 4),
                                     "achieved": gbs(a_server, s_ms)},
                     "weight_quantize": {"algorithmic_bytes_per_param": a_weight, "avg_launch_ms": round(x_ms, 4),
                                         "achieved": gbs(a_weight, x_ms)}},
    }
    print(json.dumps(out), flush=True)


# ------------------------------------------------------------------------------------- one workload
def run_fused(args, config, dev, steps, warmup, placement, headline):
    """Time qadam_step_fused (or _w) on one workload.  Returns the metrics of the line."""
    import torch
    from paper_2004_14180_amd import QAdam, QAdamConfig
    from paper_2004_14180_amd.workloads import make_workload

    wl = make_workload(config, shrink=args.shrink if headline else 1, misalign=bool(headline and args.misalign))
    if headline and args.k_g is not None:
        wl.k_g = args.k_g
    if headline and args.k_x is not None:
        wl.k_x = args.k_x
    P, N = wl.num_params, wl.num_workers
    weight_ef = 1
    variant_w = headline and args.variant == "w"
    rounding = args.rounding if headline else 0
    q = QAdam(QAdamConfig(k_g=wl.k_g, k_x=wl.k_x, rounding=rounding, weight_ef=weight_ef, beta1=wl.beta1,
                          eps=wl.eps), wl.seg_offsets, N)
    use_graph = headline and args.graph
    q.profile_enable(not use_graph)
    if args.scale_pass == "filtered":
        q.trust_error_buffers(True)
    code_bits = q.grad_code_bytes() * 8.0 / P
    wcode_bytes = q.weight_code_bytes() / P

    n_f32 = 4 + 2 * N + (2 * N if variant_w else 0)
    working_set = [4 * P] * n_f32 + [q.grad_code_bytes()] * N + [q.weight_code_bytes()]
    if placement == "separate" and headline and args.alloc_cycles > 0:
        condition_allocator(working_set, args.alloc_cycles, dev)
    B = Buffers(q, wl, dev, placement, variant_w)

    if headline and args.copy_calibration:
        src = torch.ones(1 << 30, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)                      # reads 4 GiB, writes 4 GiB
        torch.cuda.synchronize()
        del src, dst

    if headline and args.path == "calls":
        if args.variant != "s":
            sys.exit("bench.py: --path calls is for variant S")
        bench_calls(args, wl, q, B, code_bits, wcode_bytes)
        return None

    def step_call(t):
        if not variant_w:
            q.step_fused(t, wl.lr, wl.beta2, B.grads, B.errs, B.codes, B.scales, B.x, B.m, B.v, B.werr, B.wcodes)
        else:
            q.step_fused_w(t, wl.lr, wl.beta2, B.grads, B.mw, B.vw, B.errs, B.codes, B.scales, B.x, B.werr, B.wcodes)

    def timed_steps(first, warm, count):
        """`warm` untimed then `count` timed steps; each timed between two device synchronisations,
        with the step's gradients already resident.  Returns per-step (wall, scale pass, main pass) ms."""
        out = []
        graph = None
        for t in range(first, first + warm + count):
            wl.fill_gradients(t, B.grads)      # untimed: inputs are resident before the clock starts
            torch.cuda.synchronize()
            if use_graph and graph is None and t >= first + warm:
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
            a, b = (dt / 2, dt / 2) if use_graph else q.profile_read()
            if t >= first + warm:
                out.append((dt, a, b))
        return out

    # the library applies the filter from 32768 (tile, worker) pairs on (about 1.3e8 worker-elements);
    # a recorded graph always takes the full pass
    tiles = sum((n + 4095) // 4096 for n in wl.sizes)
    filtered = (args.scale_pass == "filtered" and not variant_w and wl.k_g >= 0 and tiles * N >= 32768
                and not use_graph)
    res = timed_steps(1, warmup, steps)
    step_ms, scale_ms, main_ms = ([r[k] for r in res] for k in range(3))
    full_pass = None
    if filtered and not args.no_full_comparison:
        # the same steps once more with the option off (every element's g and e read for the scales)
        q.trust_error_buffers(False)
        res_full = timed_steps(1 + warmup + steps, 1, steps)
        full_ms = sum(r[0] for r in res_full) / len(res_full)
        full_pass = {"ms_per_step": round(full_ms, 4), "value": P / (full_ms * 1e-3),
                     "scale_pass_ms": round(sum(r[1] for r in res_full) / len(res_full), 4),
                     "main_pass_ms": round(sum(r[2] for r in res_full) / len(res_full), 4)}
    if os.environ.get("QADAM_BENCH_VERBOSE"):
        print("config %d per-step main ms:" % config, [round(v_, 3) for v_ in main_ms], file=sys.stderr)
        print("config %d per-step scale ms:" % config, [round(v_, 3) for v_ in scale_ms], file=sys.stderr)
    status = q.get_status()
    ms_per_step = sum(step_ms) / len(step_ms)
    main_avg = sum(main_ms) / len(main_ms)
    scale_avg = sum(scale_ms) / len(scale_ms)
    gbs = lambda bytes_per_param, ms: round(bytes_per_param * P / (max(ms, 1e-6) * 1e-3) / 1e9, 1)

    if variant_w:
        # first pass (dominant): per worker read g, m_i, v_i, e_i and write m_i, v_i, p = 28 B;
        # second pass: per worker read p, write e and the code; server read/write x and e^x, weight code
        a_first = 28.0 * N
        a_second = N * (8.0 + code_bits / 8.0) + 8.0 + (8.0 if weight_ef else 4.0) + wcode_bytes
        roofline = {"bound": "hbm", "kernel": "k_moments_w (first pass of qadam_step_fused_w)",
                    "scope": "this kernel's launches only",
                    "achieved": gbs(a_first, scale_avg), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(gbs(a_first, scale_avg) / HBM_PEAK_GBS, 4), "traffic": None,
                    "algorithmic_bytes_per_param": a_first, "avg_launch_ms": round(scale_avg, 4),
                    "second_pass": {"algorithmic_bytes_per_param": a_second, "avg_launch_ms": round(main_avg, 4),
                                    "achieved": gbs(a_second, main_avg)},
                    "whole_step": {"bytes_per_param": a_first + a_second, "GBs": gbs(a_first + a_second, ms_per_step),
                                   "frac": round(gbs(a_first + a_second, ms_per_step) / HBM_PEAK_GBS, 4)}}
    else:
        a_main = algorithmic_bytes_per_param(N, code_bits, wcode_bytes, weight_ef)
        # scale pass: g and e of every worker; filtered: g, plus e of the few elements that can be the maximum
        a_scale = (4.0 if filtered else 8.0) * N if code_bits else 0.0
        is_headline_cfg = (headline and args.shrink == 1 and args.k_g is None and args.k_x is None
                           and args.rounding == 0 and config == 5)
        traffic = measured_traffic_bytes() if is_headline_cfg else None
        scale_traffic = measured_traffic_bytes("filtered_scale_pass_traffic_bytes_per_step" if filtered else
                                               "full_scale_pass_traffic_bytes_per_step") if is_headline_cfg else None
        roofline = {"bound": "hbm", "kernel": "k_fused (main pass of qadam_step_fused)",
                    "scope": "this kernel's launches only; whole_step below covers the scale pass as well",
                    "achieved": gbs(a_main, main_avg), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(gbs(a_main, main_avg) / HBM_PEAK_GBS, 4),
                    "traffic": traffic,
                    "traffic_source": ("profiles/fused_step_gpt1p3b_pmc_traffic.txt (rocprofv3 FETCH_SIZE / WRITE_SIZE "
                                       "of this kernel source, copy-calibrated)" if traffic else None),
                    "algorithmic_bytes_per_param": a_main, "avg_launch_ms": round(main_avg, 4),
                    "scale_pass": {"mode": "filtered" if filtered else "full",
                                   "algorithmic_bytes_per_param": a_scale, "avg_launch_ms": round(scale_avg, 4),
                                   "achieved": gbs(a_scale, scale_avg),
                                   # HBM bytes of the pass per step by the same counters (filtered: g of every
                                   # element, the sampled tiles and the few e that can matter)
                                   "traffic": scale_traffic},
                    # bytes the step moves by design (main pass + scale pass) over the step's wall time
                    "whole_step": {"bytes_per_param": a_main + a_scale, "GBs": gbs(a_main + a_scale, ms_per_step),
                                   "frac": round(gbs(a_main + a_scale, ms_per_step) / HBM_PEAK_GBS, 4)},
                    # the method's own minimum (every buffer once, no read for the scales) over the step time
                    "a_min_over_step": {"bytes_per_param": a_main, "GBs": gbs(a_main, ms_per_step),
                                        "frac": round(gbs(a_main, ms_per_step) / HBM_PEAK_GBS, 4)}}
    if use_graph:
        whole = roofline["whole_step"]["GBs"]
        roofline = {"bound": "hbm", "kernel": "whole step (HIP graph replay)", "scope": "whole step",
                    "achieved": whole, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(whole / HBM_PEAK_GBS, 4),
                    "traffic": None, "avg_launch_ms": round(ms_per_step, 4)}
    workload = ("config %d: %s, %d logical workers, %d parameters in %d layers, k_g=%d (%d-bit codes), k_x=%d "
                "(%d-bit weights; 0 bits = quantizer off), weight_ef=1, %s rounding, %s"
                % (wl.config, wl.name, N, P, len(wl.sizes), wl.k_g, round(code_bits), wl.k_x, 8 * round(wcode_bytes),
                   "stochastic (Philox)" if rounding else "nearest",
                   "variant W (worker moments, Algorithms 2-3)" if variant_w else "variant S (server moments)"))
    # the step as the GPU sees it: HIP events on the stream, from before its first kernel to after its last
    gpu_ms = None if use_graph else scale_avg + main_avg
    out = dict(wl=wl, workload=workload, ms_per_step=ms_per_step, value=P / (ms_per_step * 1e-3), roofline=roofline,
               gpu_ms=gpu_ms, step_bytes_per_param=(roofline.get("whole_step") or {}).get("bytes_per_param"),
               full_pass=full_pass, status=status, filtered=filtered, resident=sum(working_set),
               arena_bytes=B.arena_bytes, worker_elements=N * P / (ms_per_step * 1e-3))
    q.close()
    del B
    torch.cuda.empty_cache()
    return out


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
                    help="full: the scale pass reads g and e of every element (the library's default mode); "
                         "filtered: qadam_trust_error_buffers(1), it reads e only where |g| can still reach the "
                         "layer's maximum (same results; the error buffers are the library's between steps)")
    ap.add_argument("--placement", choices=["arena", "separate"], default="arena",
                    help="arena: one allocation, buffers at the offsets of qadam_arena_layout; separate: one "
                         "allocation per buffer")
    ap.add_argument("--misalign", action="store_true",
                    help="put one 1001-element layer in front of the workload's layer list, so that every other "
                         "layer starts off a 16-byte boundary (the kernels then move their data with 4-byte-aligned "
                         "128-bit accesses)")
    ap.add_argument("--graph", action="store_true",
                    help="capture the step in a HIP graph after the warm-up and time replays of it (pays on "
                         "launch-bound workloads such as config 1; kernels are then not timed one by one)")
    ap.add_argument("--no-full-comparison", action="store_true",
                    help="with the filtered scale pass: do not time the same steps again with the full one "
                         "(for profiles of one mode)")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="do not add the short runs of the other workloads (config.other_workloads)")
    ap.add_argument("--k-g", type=int, default=None,
                    help="override the workload's gradient grid (0: 2-bit codes, 1-2: 3-bit, 3-6: 4-bit, "
                         "-1: no gradient quantization)")
    ap.add_argument("--k-x", type=int, default=None,
                    help="override the workload's weight grid (0-6: int8, 7-14: int16, -1: no weight quantization)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--alloc-cycles", type=int, default=0,
                    help="--placement separate only: allocate and free the working set this many times before "
                         "the real allocation (see condition_allocator)")
    ap.add_argument("--ceilings", action="store_true",
                    help="also time plain torch streams over 6 GiB (an in-place update: half reads, half "
                         "writes; a device copy) and add them to the JSON line as memory_system")
    ap.add_argument("--utilities", action="store_true",
                    help="also time the kernels around the step alone (weight quantize / dequantize, the norm "
                         "diagnostic) on the workload's vector and add them to the JSON line as utilities")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 4 GiB device copy (a kernel of known traffic, to scale "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (logical workers are in-memory shards of one "
                 "device); --gpus %d is not supported" % args.gpus)

    import torch
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    memory_system = measure_ceilings(dev) if args.ceilings else None

    import gc
    r = run_fused(args, args.config, dev, args.steps, args.warmup, args.placement, headline=True)
    if r is None:
        return
    gc.collect()
    torch.cuda.empty_cache()        # the block goes back to the driver before anything else is allocated
    wl = r["wl"]
    out = {
        "metric": "parameters updated/sec (full QAdam-EF step)",
        "value": r["value"],
        "unit": "params/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(r["ms_per_step"], 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        # the same steps with the library's default scale pass (no caller contract)
        "value_full_scale_pass": r["full_pass"]["value"] if r["full_pass"] else None,
        "ms_per_step_full_scale_pass": r["full_pass"]["ms_per_step"] if r["full_pass"] else None,
        "config": {"workload": r["workload"],
                   "worker_elements_per_s": r["worker_elements"],
                   "resident_bytes": r["resident"],
                   "placement": ("one allocation of %d bytes, offsets from qadam_arena_layout" % r["arena_bytes"])
                   if r["arena_bytes"] else
                   ("one allocation per buffer, %d allocator conditioning cycles" % args.alloc_cycles),
                   "hip_graph_replay": bool(args.graph),
                   "scale_pass": "filtered: exact scales, e read only where |g| can reach the layer maximum "
                                 "(qadam_trust_error_buffers, opt-in with a caller contract)" if r["filtered"]
                   else "full: g and e of every element (library default)",
                   "same_steps_with_full_scale_pass": r["full_pass"],
                   "status_word": r["status"]},
        "roofline": r["roofline"],
    }
    plain = args.variant == "s" and args.rounding == 0 and args.path == "fused" and not args.graph
    if plain and not args.no_other_configs and args.shrink == 1 and args.k_g is None and args.k_x is None \
            and not args.misalign:
        # the other workloads, briefly, in the same launch configuration and placement
        others = {}
        for c in (1, 2, 3, 4):
            if c == args.config:
                continue
            o = run_fused(args, c, dev, 20, 5, args.placement, headline=False)
            gc.collect()
            torch.cuda.empty_cache()
            rf = o["roofline"]
            others["config %d" % c] = {
                "workload": o["workload"], "ms_per_step": round(o["ms_per_step"], 4), "value": o["value"],
                "main_pass_ms": rf["avg_launch_ms"], "main_pass_GBs": rf["achieved"],
                "scale_pass": rf["scale_pass"]["mode"], "scale_pass_ms": rf["scale_pass"]["avg_launch_ms"],
                "whole_step_GBs": rf["whole_step"]["GBs"], "whole_step_frac": rf["whole_step"]["frac"],
                # the same bytes over the step's time on the GPU (HIP events around its launches; the wall time
                # above also holds the host's launch and synchronisation cost, which dominates tiny steps)
                "gpu_ms_per_step": round(o["gpu_ms"], 4),
                "whole_step_frac_gpu_time": round(o["step_bytes_per_param"] * o["wl"].num_params / (o["gpu_ms"] * 1e-3) / 1e9
                                                  / HBM_PEAK_GBS, 4),
                "ms_per_step_full_scale_pass": o["full_pass"]["ms_per_step"] if o["full_pass"] else None,
                "status_word": o["status"]}
        out["config"]["other_workloads"] = others
    if not args.no_cpu_baseline and plain and wl.k_g >= 0 and wl.k_x >= 0:
        out["cpu_baseline"] = cpu_baseline(wl, dev)
    if args.utilities:
        out["utilities"] = bench_utilities(wl, dev)
    if memory_system:
        out["memory_system"] = memory_system
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
