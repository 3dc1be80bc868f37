"""GPU parity with the CPU oracle at the FULL sizes of configurations 3, 4 and 5: every layer, every
element, every step of each configuration's schedule, in the launch configuration the benchmark
times (qadam_step_fused, default tile size, filtered scale pass switched on as the benchmark does,
so it is active from the second step on).

How 1.3 G parameters x 8 workers go through an oracle that runs on the host: the oracle keeps the
COMPLETE optimizer state (e_1..e_N, x, m, v, e^x) in host memory, initialised from the same seeded
start state as the device and from then on advanced only by the oracle itself.  A step is
element-wise apart from the per-layer scale, so after the device has made its step the test streams
the vector piece by piece: a piece is a whole layer (up to 2^22 elements: the oracle computes its
own scale) or a chunk of a larger layer (the layer's scale is then its definition, max |g + e| in
fp32, evaluated by plain CPU tensor operations on the seeded gradient and the oracle's own e).  For
each piece the step's seeded gradients are copied to the host, the oracle makes its step in place on
its state, and every output of the device is compared with it: codes and scales bit for bit (a
difference is tolerated only on elements the oracle flags as lying within one ulp of a rounding
boundary, and counted), floats within 1e-6 relative / 1e-7 absolute.  Nothing that the oracle reads
comes from the library.
"""
import threading
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

from oracle import qadam_oracle as oracle
from paper_2004_14180_amd import QAdam
from paper_2004_14180_amd.workloads import make_workload

from parity_util import THREADS, Report, close, configs, seg_word_offsets

pytestmark = pytest.mark.gpu

WHOLE_LAYER_MAX = 1 << 22     # layers up to this many elements go through the oracle whole
CHUNK = 1 << 21               # larger layers: chunks of this many elements (a multiple of 32)


@pytest.fixture(autouse=True)
def _release_cached_memory():
    """Each test here stages tens of GB through pinned host memory in pieces of its own sizes and fills most
    of the device: hand what the previous test's allocators still cache (pinned host blocks, device blocks)
    back before and after, so that no test depends on what ran before it."""
    import gc

    def release():
        gc.collect()
        torch.cuda.synchronize()
        torch.cuda.empty_cache()
        empty_host = getattr(torch._C, "_host_emptyCache", None)
        if empty_host is not None:
            empty_host()
    release()
    yield
    release()


def _say(msg):
    print(msg, flush=True)


def _host(t):
    """Device tensor (slice) -> numpy array through a pinned staging tensor (torch caches these)."""
    h = torch.empty(t.shape, dtype=t.dtype, pin_memory=True)
    h.copy_(t, non_blocking=True)
    return h


def _pull(t):
    """A whole device tensor as a numpy array, copied piece by piece through pinned staging."""
    out = np.empty(t.numel(), np.float32)
    for c in range(0, t.numel(), 1 << 26):
        d = min(t.numel(), c + (1 << 26))
        h = _host(t[c:d])
        torch.cuda.current_stream().synchronize()
        out[c:d] = h.numpy()
    return out


class FullRun:
    """Device buffers of a workload, the oracle's complete state on the host, and the streaming
    comparison of a step."""

    def __init__(self, wl, start_state="synthetic", rounding=0, path="fused"):
        self.wl = wl
        dev = torch.device("cuda:0")
        self.dev = dev
        self.path = path
        self.gcfg, self.ocfg = configs(k_g=wl.k_g, k_x=wl.k_x, weight_ef=1, beta1=wl.beta1, eps=wl.eps,
                                       rounding=rounding, seed=wl.seed + 17)
        self.seg = wl.seg_offsets
        self.q = QAdam(self.gcfg, self.seg, wl.num_workers)
        # as the benchmark runs it: from the second step of a handle on, the scale pass is the filtered one
        self.q.trust_error_buffers(True)
        P, N = wl.num_params, wl.num_workers
        if start_state == "synthetic":          # a plausible mid-training state: every buffer non-trivial
            st = wl.synthetic_state(dev)
            self.errs, self.m, self.v, self.werr = st["errs"], st["m"], st["v"], st["werr"]
        else:
            z = lambda: torch.zeros(P, dtype=torch.float32, device=dev)
            self.errs, self.m, self.v, self.werr = [z() for _ in range(N)], z(), z(), z()
        self.x = wl.init_weights(dev)
        self.grads = [torch.empty(P, dtype=torch.float32, device=dev) for _ in range(N)]
        self.codes = [torch.zeros(self.q.grad_code_bytes() // 4, dtype=torch.int32, device=dev) for _ in range(N)]
        self.scales = [torch.zeros(len(self.seg) - 1, dtype=torch.float32, device=dev) for _ in range(N)]
        self.wcodes = torch.zeros(P, dtype=torch.int8 if wl.k_x <= 6 else torch.int16, device=dev)
        self.woffs = seg_word_offsets(wl.k_g, self.seg)
        self.bits = oracle.grad_code_bits(wl.k_g)
        self.host = None
        self.excused = np.zeros(P, bool)

    def init_host_state(self):
        """The oracle's state: host copies of the seeded start state (taken before the first step)."""
        self.host = dict(errs=[_pull(e) for e in self.errs], x=_pull(self.x), m=_pull(self.m), v=_pull(self.v),
                         werr=_pull(self.werr))

    def step(self, t):
        wl = self.wl
        if self.path == "fused":
            self.q.step_fused(t, wl.lr, wl.beta2, self.grads, self.errs, self.codes, self.scales,
                              self.x, self.m, self.v, self.werr, self.wcodes)
        else:       # the same step as the separate calls of the boundary
            for i in range(wl.num_workers):
                self.q.worker_quantize(i, t, self.grads[i], self.errs[i], self.codes[i], self.scales[i])
            self.q.server_step(t, wl.lr, wl.beta2, self.codes, self.scales, self.x, self.m, self.v)
            self.q.weight_quantize(t, self.x, self.werr, self.wcodes)
        torch.cuda.synchronize()
        assert self.q.get_status() == 0

    # ---- pieces ---------------------------------------------------------------------------------
    def state_views(self, a, b):
        """The oracle's state on [a, b): views, advanced in place by the oracle."""
        h = self.host
        return dict(errs=[e[a:b] for e in h["errs"]], x=h["x"][a:b], m=h["m"][a:b], v=h["v"][a:b], werr=h["werr"][a:b])

    def fetch_outputs(self, layer, a, b):
        """Pinned host copies of what the device wrote for [a, b) of `layer` (a 32-aligned inside it)."""
        N = self.wl.num_workers
        off = a - self.seg[layer]
        assert off % 32 == 0
        w0 = self.woffs[layer] + off // 32 * self.bits
        nw = (b - a + 31) // 32 * self.bits
        return dict(errs=[_host(e[a:b]) for e in self.errs], x=_host(self.x[a:b]), m=_host(self.m[a:b]),
                    v=_host(self.v[a:b]), werr=_host(self.werr[a:b]), wcodes=_host(self.wcodes[a:b]),
                    words=[_host(c[w0:w0 + nw]) for c in self.codes])

    def compare(self, rep, lock, name, a, b, want, got, codes_want, wcodes_want, tie_g, tie_x):
        """`want`: the oracle's state on [a, b) after its step.  An element whose code differed on a
        flagged boundary (tolerated, counted) has a different trajectory from then on: it stays excused."""
        N = self.wl.num_workers
        n = b - a
        excused = self.excused[a:b]
        skip = excused.copy()
        local = Report()
        for i in range(N):
            gc = oracle.unpack_codes(self.bits, got["words"][i].numpy().view(np.uint32), n)
            diff = (gc != codes_want[i]) & ~excused
            if diff.any():
                local.code_mismatch += int(diff.sum())
                bad = diff & (tie_g[i] == 0)
                local.code_mismatch_unflagged += int(bad.sum())
                assert not bad.any(), "%s: worker %d code mismatch on unflagged elements" % (name, i)
                skip |= diff
            local.ties_g += int(np.count_nonzero(tie_g[i]))
            sk = (diff | excused) if (diff.any() or excused.any()) else None
            close(local, name + " err", got["errs"][i].numpy(), want["errs"][i], sk)
        sk = skip if skip.any() else None
        close(local, name + " m", got["m"].numpy(), want["m"], sk)
        close(local, name + " v", got["v"].numpy(), want["v"], sk)
        close(local, name + " x", got["x"].numpy(), want["x"], sk)
        wdiff = (got["wcodes"].numpy() != wcodes_want) & ~skip
        local.wcode_mismatch += int(wdiff.sum())
        local.ties_x += int(np.count_nonzero(tie_x))
        assert not (wdiff & (tie_x == 0)).any(), name + ": weight code mismatch on unflagged elements"
        skip |= wdiff
        close(local, name + " werr", got["werr"].numpy(), want["werr"], skip if skip.any() else None)
        if skip.any():
            self.excused[a:b] = skip
        local.checked = n * (N + 1)
        with lock:
            for f in ("code_mismatch", "code_mismatch_unflagged", "wcode_mismatch", "wcode_mismatch_unflagged",
                      "ties_g", "ties_x", "float_not_bit_exact", "checked"):
                setattr(rep, f, getattr(rep, f) + getattr(local, f))
            rep.max_rel = max(rep.max_rel, local.max_rel)

    def host_layer_scales(self, layer):
        """||g_i + e_i||_inf of a large layer by its definition: fp32 add, abs, max, on host copies of
        the seeded gradient and on the oracle's own e (plain CPU tensor operations)."""
        a, b = self.seg[layer], self.seg[layer + 1]
        out = []
        for i in range(self.wl.num_workers):
            s = np.float32(0)
            for c in range(a, b, 1 << 25):
                d = min(b, c + (1 << 25))
                p = _host(self.grads[i][c:d])
                torch.cuda.current_stream().synchronize()
                s = max(s, np.float32(p.add_(torch.from_numpy(self.host["errs"][i][c:d])).abs_().max().item()))
            out.append(np.float32(s))
        return out

    def check_step(self, rep, t, progress=""):
        """Every element of every layer: the oracle's step t, in place on its own state, against what the
        device wrote in its step t (call after self.step(t); the gradients are still in place)."""
        wl = self.wl
        N = wl.num_workers
        lock = threading.Lock()
        dscales = [s.cpu().numpy() for s in self.scales]
        inflight = threading.Semaphore(2 * THREADS)

        def whole(l, a, b, grads, got):
            try:
                st = self.state_views(a, b)
                out = oracle.step_s(self.ocfg, [0, b - a], t, wl.lr, wl.beta2, [g.numpy() for g in grads],
                                    st["errs"], st["x"], st["m"], st["v"], st["werr"], index_base=a)
                assert out["status"] == 0
                for i in range(N):
                    assert dscales[i][l].view(np.uint32) == out["scales"][i][0].view(np.uint32), \
                        "step %d: scale of worker %d, layer %d" % (t, i, l)
                codes = [oracle.unpack_codes(self.bits, out["words"][i], b - a) for i in range(N)]
                self.compare(rep, lock, "step %d layer %d" % (t, l), a, b, st, got, codes, out["wcodes"],
                             out["tie_g"], out["tie_x"])
            finally:
                inflight.release()

        def chunk(l, k, a, b, scales, grads, got):
            try:
                st = self.state_views(a, b)
                out = oracle.step_s_window(self.ocfg, a, t, wl.lr, wl.beta2, scales, [g.numpy() for g in grads],
                                           st["errs"], st["x"], st["m"], st["v"], st["werr"])
                assert out["status"] == 0
                self.compare(rep, lock, "step %d layer %d chunk %d" % (t, l, k), a, b, st, got, out["codes"],
                             out["wcodes"], out["tie_g"], out["tie_x"])
            finally:
                inflight.release()

        futures = []
        with ThreadPoolExecutor(THREADS) as ex:
            for l in sorted(range(len(wl.sizes)), key=lambda l: -wl.sizes[l]):
                a, b = self.seg[l], self.seg[l + 1]
                if b == a:
                    continue
                if b - a <= WHOLE_LAYER_MAX:
                    inflight.acquire()
                    grads, got = [_host(g[a:b]) for g in self.grads], self.fetch_outputs(l, a, b)
                    torch.cuda.current_stream().synchronize()
                    futures.append(ex.submit(whole, l, a, b, grads, got))
                else:
                    # the scale first (it needs the oracle's e of the whole layer BEFORE any chunk advances it)
                    scales = self.host_layer_scales(l)
                    for i in range(N):
                        assert dscales[i][l].view(np.uint32) == scales[i].view(np.uint32), \
                            "step %d: scale of worker %d, layer %d against its definition" % (t, i, l)
                    for k, c in enumerate(range(a, b, CHUNK)):
                        d = min(b, c + CHUNK)
                        inflight.acquire()
                        grads, got = [_host(g[c:d]) for g in self.grads], self.fetch_outputs(l, c, d)
                        torch.cuda.current_stream().synchronize()
                        futures.append(ex.submit(chunk, l, k, c, d, scales, grads, got))
                        if progress and (k + 1) % 32 == 0:
                            _say("%s: layer %d, %d of %d elements streamed" % (progress, l, d - a, b - a))
                # surface a failure early instead of streaming the rest
                for f in [f for f in futures if f.done()]:
                    f.result()
                    futures.remove(f)
            for f in futures:
                f.result()


def run_full_schedule(config, start_state, misalign=False, steps=None):
    """The configuration's whole schedule at full size, every element compared after every step."""
    wl = make_workload(config, misalign=misalign)
    if steps is not None:
        wl.steps = steps
    return run_workload(wl, start_state, "config%d full%s" % (config, " misaligned" if misalign else ""))


def run_workload(wl, start_state, tag, **kw):
    run = FullRun(wl, start_state=start_state, **kw)
    run.init_host_state()
    rep = Report()
    for t in range(1, wl.steps + 1):
        wl.fill_gradients(t, run.grads)
        run.step(t)
        run.check_step(rep, t, progress="%s step %d" % (tag, t))
        _say("%s step %d/%d (every layer, every element): %s" % (tag, t, wl.steps, rep.line()))
        assert rep.ok()
    assert rep.checked == wl.steps * wl.num_params * (wl.num_workers + 1)
    run.q.close()
    return rep


# ------------------------------------------------------------------------------------------------
def test_config3_gpt2_full_size_all_20_steps():
    """Config 3 at full size (124 439 808 parameters, 148 layers, 8 workers; Student-t gradients, zeroed
    embedding rows): its whole schedule of 20 steps from the workload's initial state."""
    run_full_schedule(3, "initial")


def test_config4_adversarial_full_size_all_10_steps():
    """Config 4 at full size (2^28 parameters in one segment, 16 workers; 8 decades of block scales plus
    +-1e3 outliers): its whole schedule of 10 steps, the whole vector on every step; the 16 scales are
    also compared with their definition on every step."""
    run_full_schedule(4, "initial")


def test_config5_gpt13b_full_size_all_5_steps():
    """Config 5 at full size (1 315 723 264 parameters, 292 layers, 8 workers; the benchmark's workload
    and launch configuration), from a synthetic mid-training state so that the first step already
    exercises every buffer: its 5 steps, every layer on every step."""
    run_full_schedule(5, "synthetic")


def test_config5_gpt13b_full_size_off_alignment():
    """Config 5 at full size behind one 1001-element layer, so that every one of its 292 layers starts at
    a flat index = 1 mod 4 (the kernels then use their dword-aligned wide accesses everywhere): two steps,
    the second with the filtered scale pass, every layer and every element."""
    run_full_schedule(5, "synthetic", misalign=True, steps=2)


@pytest.mark.parametrize("rounding", [0, 1])
def test_vector_beyond_2_to_31_elements(rounding):
    """The largest shape the index arithmetic has to carry: a flat vector of more than 2^31 elements
    (8.6 GB per buffer), with one layer that crosses element 2^31 and, behind it, an odd-sized layer and
    layers that lie wholly beyond 2^31 off the 16-byte grid.  Two workers, gradients by config 2's
    recipe, two steps (the second with the filtered scale pass), every element against the oracle;
    with stochastic rounding as well, whose random stream is indexed by the flat element number."""
    from paper_2004_14180_amd.workloads import Workload
    sizes = [5000, (1 << 31) + 3 * 4096 + 77, 1001, 300000, 64, 2 * 4096]
    wl = Workload(2, "beyond-2^31", sizes, 2, 2)
    assert wl.seg_offsets[2] > (1 << 31) and wl.seg_offsets[3] % 4 != 0
    run_workload(wl, "synthetic", "2^31+ elements, rounding %d" % rounding, rounding=rounding)


def test_config5_gpt13b_full_size_separate_calls():
    """Config 5 at full size through the separate calls of the boundary (8 x qadam_worker_quantize,
    qadam_server_step, qadam_weight_quantize: the codes go through memory and are decoded again), as
    `bench.py --path calls` launches it: one step from a synthetic mid-training state, every layer and
    every element against the oracle (the filtered scale pass of the worker call, which a second step
    would use, is covered at smaller sizes)."""
    wl = make_workload(5)
    wl.steps = 1
    run_workload(wl, "synthetic", "config5 separate calls", path="calls")


# ------------------------------------------------------------------------------------------------
class FullRunW(FullRun):
    """Variant W (Algorithms 2-3: the workers own the moments and quantize the update) at full size.
    The server has no m, v here; every worker has its own, on the device and in the oracle's host state.
    The scale of a layer is the maximum of a quantity the oracle itself computes (alpha m' / sqrt(v' +
    eps) + e), so every layer goes through the oracle whole, largest first, one layer per thread."""

    def __init__(self, wl):
        super().__init__(wl, start_state="synthetic")
        self.q.trust_error_buffers(False)       # the scale pass of variant W has no filtered form
        # per-worker moments: the synthetic server moments, scaled differently per worker
        self.mw = [self.m * (1.0 + 0.125 * i) for i in range(wl.num_workers)]
        self.vw = [self.v * (1.0 + 0.25 * i) for i in range(wl.num_workers)]
        del self.m, self.v

    def init_host_state(self):
        self.host = dict(errs=[_pull(e) for e in self.errs], mw=[_pull(u) for u in self.mw],
                         vw=[_pull(u) for u in self.vw], x=_pull(self.x), werr=_pull(self.werr))

    def step(self, t):
        wl = self.wl
        self.q.step_fused_w(t, wl.lr, wl.beta2, self.grads, self.mw, self.vw, self.errs, self.codes, self.scales,
                            self.x, self.werr, self.wcodes)
        torch.cuda.synchronize()
        assert self.q.get_status() == 0

    def check_step(self, rep, t, progress=""):
        wl = self.wl
        N = wl.num_workers
        lock = threading.Lock()
        dscales = [s.cpu().numpy() for s in self.scales]
        inflight = threading.Semaphore(THREADS)
        h = self.host

        def layer(l, a, b, grads, got):
            try:
                n = b - a
                he, hm, hv = ([u[a:b] for u in h[k]] for k in ("errs", "mw", "vw"))
                hx, hw = h["x"][a:b], h["werr"][a:b]
                out = oracle.step_w(self.ocfg, [0, n], t, wl.lr, wl.beta2, [g.numpy() for g in grads],
                                    he, hm, hv, hx, hw, index_base=a)
                assert out["status"] == 0
                local = Report()
                skip = np.zeros(n, bool)
                for i in range(N):
                    assert dscales[i][l].view(np.uint32) == out["scales"][i][0].view(np.uint32), \
                        "step %d: scale of worker %d, layer %d" % (t, i, l)
                    gc = oracle.unpack_codes(self.bits, got["words"][i].numpy().view(np.uint32), n)
                    diff = gc != oracle.unpack_codes(self.bits, out["words"][i], n)
                    if diff.any():
                        local.code_mismatch += int(diff.sum())
                        assert not (diff & (out["tie_g"][i] == 0)).any(), \
                            "step %d layer %d: worker %d code mismatch on unflagged elements" % (t, l, i)
                        skip |= diff
                    local.ties_g += int(np.count_nonzero(out["tie_g"][i]))
                    close(local, "err", got["errs"][i].numpy(), he[i], diff if diff.any() else None)
                    close(local, "mw", got["mw"][i].numpy(), hm[i])
                    close(local, "vw", got["vw"][i].numpy(), hv[i])
                assert not skip.any(), "a flagged code difference would need the excused-element bookkeeping"
                close(local, "x", got["x"].numpy(), hx)
                wdiff = got["wcodes"].numpy() != out["wcodes"]
                local.wcode_mismatch += int(wdiff.sum())
                local.ties_x += int(np.count_nonzero(out["tie_x"]))
                assert not wdiff.any(), "step %d layer %d: weight codes" % (t, l)
                close(local, "werr", got["werr"].numpy(), hw)
                with lock:
                    for f in ("code_mismatch", "wcode_mismatch", "ties_g", "ties_x", "float_not_bit_exact"):
                        setattr(rep, f, getattr(rep, f) + getattr(local, f))
                    rep.checked += n * (N + 1)
                    rep.max_rel = max(rep.max_rel, local.max_rel)
                    if progress and n >= (1 << 22):
                        _say("%s: layer %d (%d elements) done" % (progress, l, n))
            finally:
                inflight.release()

        futures = []
        with ThreadPoolExecutor(THREADS) as ex:
            for l in sorted(range(len(wl.sizes)), key=lambda l: -wl.sizes[l]):
                a, b = self.seg[l], self.seg[l + 1]
                if b == a:
                    continue
                inflight.acquire()
                w0 = self.woffs[l]
                nw = (b - a + 31) // 32 * self.bits
                grads = [_host(g[a:b]) for g in self.grads]
                got = dict(errs=[_host(e[a:b]) for e in self.errs], mw=[_host(u[a:b]) for u in self.mw],
                           vw=[_host(u[a:b]) for u in self.vw], x=_host(self.x[a:b]), werr=_host(self.werr[a:b]),
                           wcodes=_host(self.wcodes[a:b]), words=[_host(c[w0:w0 + nw]) for c in self.codes])
                torch.cuda.current_stream().synchronize()
                futures.append(ex.submit(layer, l, a, b, grads, got))
                for f in [f for f in futures if f.done()]:
                    f.result()
                    futures.remove(f)
            for f in futures:
                f.result()


def test_config5_gpt13b_full_size_variant_w():
    """Config 5 at full size through qadam_step_fused_w (Algorithms 2-3 as printed: 16 more P-sized
    buffers for the workers' moments, 190 GB on the device), as `bench.py --variant w` launches it:
    two steps from a synthetic mid-training state, every layer and every element against the oracle
    (the second step starts from the residuals the first one left in the error buffers, which this
    variant also uses to park the update between its two passes)."""
    wl = make_workload(5)
    wl.steps = 2
    run = FullRunW(wl)
    run.init_host_state()
    rep = Report()
    for t in range(1, wl.steps + 1):
        wl.fill_gradients(t, run.grads)
        run.step(t)
        run.check_step(rep, t, progress="config5 variant W step %d" % t)
        _say("config5 variant W step %d/%d (every layer, every element): %s" % (t, wl.steps, rep.line()))
        assert rep.ok()
    assert rep.checked == wl.steps * wl.num_params * (wl.num_workers + 1)
    run.q.close()
