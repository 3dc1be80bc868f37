"""Helpers of the GPU parity tests: run the HIP library and the CPU oracle on the same seeded
inputs and compare element by element.

Bar (from the build's target statement): packed gradient codes, scales and weight codes bit-exact,
except elements the ORACLE flags as lying within one fp32 ulp of a rounding boundary (counted);
m, v, x, e, e^x within 1e-6 relative / 1e-7 absolute.  Both sides do the same fp32 operations in
the same order, so in practice everything is expected to be bit-identical; `Report` records that.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import List

import numpy as np
import torch

from oracle import qadam_oracle as oracle
from oracle.qadam_oracle import OracleConfig
from paper_2004_14180_amd import QAdam, QAdamConfig

RTOL, ATOL = 1e-6, 1e-7
THREADS = min(16, os.cpu_count() or 1)


def configs(k_g=2, k_x=6, rounding=0, weight_ef=1, adam_flavor=0, beta1=0.9, eps=1e-8, seed=0):
    kw = dict(k_g=k_g, k_x=k_x, rounding=rounding, weight_ef=weight_ef, adam_flavor=adam_flavor,
              beta1=beta1, eps=eps, seed=seed)
    return QAdamConfig(**kw), OracleConfig(**kw)


@dataclass
class Report:
    code_mismatch: int = 0          # gradient codes differing (must all be oracle-flagged)
    code_mismatch_unflagged: int = 0
    wcode_mismatch: int = 0
    wcode_mismatch_unflagged: int = 0
    ties_g: int = 0                 # elements the oracle flagged
    ties_x: int = 0
    float_not_bit_exact: int = 0    # fp32 outputs that differ in any bit (still inside tolerance)
    max_rel: float = 0.0
    checked: int = 0
    notes: List[str] = field(default_factory=list)

    def ok(self):
        return self.code_mismatch_unflagged == 0 and self.wcode_mismatch_unflagged == 0

    def line(self):
        return ("checked=%d ties_g=%d ties_x=%d code_mismatch=%d wcode_mismatch=%d float_bit_diffs=%d max_rel=%.2e"
                % (self.checked, self.ties_g, self.ties_x, self.code_mismatch, self.wcode_mismatch,
                   self.float_not_bit_exact, self.max_rel))


def close(rep: Report, name, got: np.ndarray, want: np.ndarray, skip: np.ndarray = None):
    """fp32 arrays within tolerance (skip = elements excused by a flagged code mismatch)."""
    assert got.shape == want.shape, name
    g, w = got, want
    if skip is not None and skip.any():
        g, w = got[~skip], want[~skip]
    same = g.view(np.uint32) == w.view(np.uint32)
    if same.all():
        return
    both_zero = (g == 0) & (w == 0)          # +0 / -0
    diff = ~(same | both_zero)
    rep.float_not_bit_exact += int(diff.sum())
    if not diff.any():
        return
    gd, wd = g[diff].astype(np.float64), w[diff].astype(np.float64)
    err = np.abs(gd - wd)
    tol = ATOL + RTOL * np.abs(wd)
    bad = ~(err <= tol)                      # also catches NaN
    rel = float(np.max(err / np.maximum(np.abs(wd), 1e-30))) if err.size else 0.0
    rep.max_rel = max(rep.max_rel, rel)
    assert not bad.any(), "%s: %d elements outside 1e-6 rel / 1e-7 abs (max rel %.3e)" % (name, int(bad.sum()), rel)


# --------------------------------------------------------------------------------- device state
class DeviceState:
    """Buffers of one handle on the GPU."""

    def __init__(self, q: QAdam, x0: torch.Tensor, device="cuda"):
        P, N, L = q.num_params, q.num_workers, q.num_segments
        self.q = q
        z = lambda: torch.zeros(P, dtype=torch.float32, device=device)
        self.x = x0.to(device).clone()
        self.m, self.v, self.werr = z(), z(), z()
        self.errs = [z() for _ in range(N)]
        self.grads = [z() for _ in range(N)]
        nbytes = q.grad_code_bytes()
        self.codes = [torch.full((max(nbytes // 4, 1),), -1, dtype=torch.int32, device=device) for _ in range(N)]
        self.scales = [torch.full((max(L, 1),), -1.0, dtype=torch.float32, device=device) for _ in range(N)]
        wdt = torch.int8 if q.cfg.k_x <= 6 else torch.int16
        self.wcodes = torch.full((max(P, 1),), -1, dtype=wdt, device=device)
        self.code_words = nbytes // 4

    def step_fused(self, t, lr, beta2):
        self.q.step_fused(t, lr, beta2, self.grads, self.errs, self.codes, self.scales,
                          self.x, self.m, self.v, self.werr, self.wcodes)

    def step_unfused(self, t, lr, beta2, weight_quant=True):
        for i in range(self.q.num_workers):
            self.q.worker_quantize(i, t, self.grads[i], self.errs[i], self.codes[i], self.scales[i])
        self.q.server_step(t, lr, beta2, self.codes, self.scales, self.x, self.m, self.v)
        if weight_quant:
            self.q.weight_quantize(t, self.x, self.werr, self.wcodes)

    def host_codes(self, i):
        return self.codes[i][: self.code_words].cpu().numpy().view(np.uint32)


class HostState:
    def __init__(self, P, N, x0: np.ndarray):
        self.x = x0.astype(np.float32).copy()
        self.m = np.zeros(P, np.float32)
        self.v = np.zeros(P, np.float32)
        self.werr = np.zeros(P, np.float32)
        self.errs = [np.zeros(P, np.float32) for _ in range(N)]


def seg_word_offsets(k_g, seg_off):
    offs = [0]
    for l in range(len(seg_off) - 1):
        offs.append(offs[-1] + int(oracle.lib().oq_grad_code_words_segment(k_g, int(seg_off[l + 1] - seg_off[l]))))
    return offs


def oracle_step_layers(ocfg, seg_off, t, lr, beta2, grads, hs: HostState, weight_quant=True, threads=THREADS):
    """One oracle step, layer by layer on a thread pool (layers are independent: the scale is per
    layer and the rest is element-wise; tests/test_oracle_steps.py checks that property).
    Returns dict(words[N], scales[N], wcodes, tie_g[N], tie_x)."""
    seg_off = [int(s) for s in seg_off]
    L, N, P = len(seg_off) - 1, len(grads), seg_off[-1]
    woffs = seg_word_offsets(ocfg.k_g, seg_off)
    words = [np.zeros(woffs[-1], np.uint32) for _ in range(N)]
    scales = [np.zeros(L, np.float32) for _ in range(N)]
    wcodes = np.zeros(P, oracle.weight_code_dtype(ocfg.k_x))
    tie_g = [np.zeros(P, np.uint8) for _ in range(N)]
    tie_x = np.zeros(P, np.uint8)
    status = [0]

    def one(l):
        a, b = seg_off[l], seg_off[l + 1]
        if not weight_quant:
            # gradient quantization + error feedback + server only
            outs = [oracle.worker_quantize(ocfg, [0, b - a], i, t, grads[i][a:b], hs.errs[i][a:b], index_base=a)
                    for i in range(N)]
            oracle.server_step(ocfg, [0, b - a], t, lr, beta2, [o["words"] for o in outs],
                               [o["scales"] for o in outs], hs.x[a:b], hs.m[a:b], hs.v[a:b])
            for i in range(N):
                words[i][woffs[l]:woffs[l + 1]] = outs[i]["words"]
                scales[i][l] = outs[i]["scales"][0]
                tie_g[i][a:b] = outs[i]["tie"]
                status[0] |= outs[i]["status"]
            return
        out = oracle.step_s(ocfg, [0, b - a], t, lr, beta2, [g[a:b] for g in grads],
                            [e[a:b] for e in hs.errs], hs.x[a:b], hs.m[a:b], hs.v[a:b], hs.werr[a:b],
                            index_base=a)
        status[0] |= out["status"]
        for i in range(N):
            words[i][woffs[l]:woffs[l + 1]] = out["words"][i]
            scales[i][l] = out["scales"][i][0]
            tie_g[i][a:b] = out["tie_g"][i]
        wcodes[a:b] = out["wcodes"]
        tie_x[a:b] = out["tie_x"]

    order = sorted(range(L), key=lambda l: -(seg_off[l + 1] - seg_off[l]))
    if threads > 1 and L > 1:
        with ThreadPoolExecutor(threads) as ex:
            list(ex.map(one, order))
    else:
        for l in order:
            one(l)
    return dict(words=words, scales=scales, wcodes=wcodes, tie_g=tie_g, tie_x=tie_x, status=status[0])


def compare_step(rep: Report, ocfg, seg_off, ds: DeviceState, hs: HostState, out, weight_quant=True):
    """Device buffers after a step against the oracle's."""
    torch.cuda.synchronize()
    N = len(hs.errs)
    P = hs.x.size
    skip_any = np.zeros(P, bool)
    for i in range(N):
        gw = ds.host_codes(i)
        ow = out["words"][i]
        rep.ties_g += int(out["tie_g"][i].sum())
        # scales: bit-exact
        gs = ds.scales[i][: len(seg_off) - 1].cpu().numpy()
        assert np.array_equal(gs.view(np.uint32), out["scales"][i].view(np.uint32)) or \
            np.array_equal(np.isnan(gs), np.isnan(out["scales"][i])) and \
            np.array_equal(gs[~np.isnan(gs)], out["scales"][i][~np.isnan(gs)]), "scales of worker %d" % i
        skip = np.zeros(P, bool)
        if not np.array_equal(gw, ow):
            gc = oracle.unpack_all(ocfg.k_g, seg_off, gw)
            oc = oracle.unpack_all(ocfg.k_g, seg_off, ow)
            diff = gc != oc
            rep.code_mismatch += int(diff.sum())
            unflagged = diff & (out["tie_g"][i] == 0)
            rep.code_mismatch_unflagged += int(unflagged.sum())
            assert not unflagged.any(), "worker %d: %d code mismatches on unflagged elements, first at %d" % (
                i, int(unflagged.sum()), int(np.argmax(unflagged)))
            # padding bits / words must still agree
            assert np.array_equal(oracle.unpack_all(ocfg.k_g, seg_off, gw)[~diff], oc[~diff])
            skip = diff
        close(rep, "err[%d]" % i, ds.errs[i].cpu().numpy(), hs.errs[i], skip)
        skip_any |= skip
    close(rep, "m", ds.m.cpu().numpy(), hs.m, skip_any)
    close(rep, "v", ds.v.cpu().numpy(), hs.v, skip_any)
    close(rep, "x", ds.x.cpu().numpy(), hs.x, skip_any)
    if weight_quant:
        rep.ties_x += int(out["tie_x"].sum())
        gwc = ds.wcodes[:P].cpu().numpy()
        wdiff = gwc != out["wcodes"]
        wdiff &= ~skip_any
        rep.wcode_mismatch += int(wdiff.sum())
        unfl = wdiff & (out["tie_x"] == 0)
        rep.wcode_mismatch_unflagged += int(unfl.sum())
        assert not unfl.any(), "%d weight-code mismatches on unflagged elements" % int(unfl.sum())
        close(rep, "werr", ds.werr.cpu().numpy(), hs.werr, skip_any | wdiff)
    rep.checked += P * (N + 1)


def run_workload_parity(wl, steps, fused=True, k_g=None, k_x=None, rounding=0, weight_ef=None,
                        adam_flavor=0, seed=0, gen_device="cpu", threads=THREADS, check_every=1,
                        progress=None, trust_errs=False):
    """Run `steps` steps of a workload on the GPU and in the oracle, comparing after each step."""
    k_g = wl.k_g if k_g is None else k_g
    k_x = wl.k_x if k_x is None else k_x
    weight_ef = wl.weight_ef if weight_ef is None else weight_ef
    gcfg, ocfg = configs(k_g=k_g, k_x=k_x, rounding=rounding, weight_ef=weight_ef, adam_flavor=adam_flavor,
                         beta1=wl.beta1, eps=wl.eps, seed=seed)
    seg_off = wl.seg_offsets
    q = QAdam(gcfg, seg_off, wl.num_workers)
    if trust_errs:
        q.trust_error_buffers(2)        # filtered scale pass from the second step on
    x0 = wl.init_weights(gen_device)
    ds = DeviceState(q, x0)
    hs = HostState(wl.num_params, wl.num_workers, x0.cpu().numpy())
    rep = Report()
    gbuf = [torch.empty(wl.num_params, dtype=torch.float32, device=gen_device) for _ in range(wl.num_workers)]
    for t in range(1, steps + 1):
        wl.fill_gradients(t, gbuf)
        grads_np = []
        for i in range(wl.num_workers):
            ds.grads[i].copy_(gbuf[i])
            grads_np.append(gbuf[i].cpu().numpy())
        if fused and wl.weight_quant:
            ds.step_fused(t, wl.lr, wl.beta2)
        else:
            ds.step_unfused(t, wl.lr, wl.beta2, weight_quant=wl.weight_quant)
        out = oracle_step_layers(ocfg, seg_off, t, wl.lr, wl.beta2, grads_np, hs, weight_quant=wl.weight_quant,
                                 threads=threads)
        if t % check_every == 0 or t == steps:
            compare_step(rep, ocfg, seg_off, ds, hs, out, weight_quant=wl.weight_quant)
        assert q.get_status() == 0 and out["status"] == 0
        if progress:
            print("%s step %d/%d %s" % (progress, t, steps, rep.line()), flush=True)
    q.close()
    return rep
