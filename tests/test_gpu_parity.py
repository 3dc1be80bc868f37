"""GPU parity: the HIP library (through its C boundary) against the CPU oracle, element by element,
on the seeded synthetic workloads and on edge cases.  Sizes are chosen so the oracle finishes in
seconds while every tile shape occurs: full 4096-element tiles, ragged tails, segments that start
off a 16-byte boundary (dword-aligned wide accesses), tiny and empty segments, small layers (one
workgroup, no scale pass) and layers whose tile maxima the quantizing kernel folds itself."""
import numpy as np
import pytest
import torch

from oracle import qadam_oracle as oracle
from paper_2004_14180_amd import QAdam, QAdamConfig, QAdamError
from paper_2004_14180_amd.workloads import make_workload

from parity_util import (DeviceState, HostState, Report, compare_step, configs, oracle_step_layers,
                         run_workload_parity)

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


# ------------------------------------------------------------------------------- the five configs
@pytest.mark.parametrize("k_g", [2, 0])
@pytest.mark.parametrize("fused", [False, True])
def test_config1_flat_1m(k_g, fused):
    """Config 1: one worker, 2^20 parameters in one layer, 10 steps, gradient quantization + EF."""
    wl = make_workload(1)
    if fused:
        wl.weight_quant, wl.weight_ef = True, 1
    rep = run_workload_parity(wl, wl.steps, fused=fused, k_g=k_g, progress="cfg1 k_g=%d fused=%s" % (k_g, fused))
    _say("config1 k_g=%d fused=%s: %s" % (k_g, fused, rep.line()))
    assert rep.ok()


def test_config2_resnet18_full_size_all_50_steps():
    """Config 2 at full size (11 689 512 parameters, 62 layers, 4 workers), its whole schedule of 50
    steps, every element of every output compared after every step; the filtered scale pass (what the
    benchmark runs) is on from step 2."""
    wl = make_workload(2)
    rep = run_workload_parity(wl, wl.steps, fused=True, gen_device="cuda", trust_errs=True)
    _say("config2 full, 50 steps: " + rep.line())
    assert rep.ok() and rep.checked == wl.steps * wl.num_params * (wl.num_workers + 1)


def test_config3_gpt2_shrunk():
    """Config 3 (8 workers, Student-t gradients, zeroed embedding rows), model dims / 4, first 6 steps
    through the separate calls (the fused call runs the whole schedule at full size elsewhere)."""
    wl = make_workload(3, shrink=4)
    rep = run_workload_parity(wl, 6, fused=False, check_every=2, progress="cfg3/4")
    _say("config3/4: " + rep.line())
    assert rep.ok()


def test_config4_adversarial_shrunk():
    """Config 4 (16 workers, one segment, 8 decades of block scales plus +-1e3 outliers), 2^20."""
    wl = make_workload(4, shrink=256)
    rep = run_workload_parity(wl, wl.steps, fused=True, threads=1, progress="cfg4/256")
    _say("config4/256: %s" % rep.line())
    assert rep.ok()


def test_config5_gpt13b_shrunk():
    """Config 5's layer list with model dims / 8 (292 layers, 8 workers), its 5 steps."""
    wl = make_workload(5, shrink=8)
    rep = run_workload_parity(wl, wl.steps, fused=True, progress="cfg5/8")
    _say("config5/8: " + rep.line())
    assert rep.ok()


@pytest.mark.parametrize("fused", [True, False])
def test_config5_shrunk_with_every_layer_off_alignment(fused):
    """Config 5's layer list (dims / 8) behind one 1001-element layer: every layer then starts at a flat
    index = 1 mod 4, so every kernel takes its shifted (lane-to-lane) access path on full-size tiles."""
    wl = make_workload(5, shrink=8, misalign=True)
    assert all(o % 4 == 1 for o in wl.seg_offsets[1:-1])
    rep = run_workload_parity(wl, wl.steps, fused=fused, gen_device="cuda", trust_errs=fused)
    _say("config5/8 misaligned fused=%s: %s" % (fused, rep.line()))
    assert rep.ok()


@pytest.mark.parametrize("shift", [1, 2, 3])
@pytest.mark.parametrize("cfgkw", [dict(k_g=2, k_x=6), dict(k_g=0, k_x=14), dict(k_g=5, k_x=6, rounding=1, seed=3)])
def test_every_misalignment_and_code_width(shift, cfgkw):
    """Segments that start 1, 2 and 3 elements off a 16-byte boundary, with ragged ends, for 2-, 3- and 4-bit
    gradient codes, int8 and int16 weight codes, nearest and stochastic rounding (whose random stream is
    indexed by the flat element number, so it must shift with the data)."""
    sizes = [shift, 4096 * 2 + 5, 33, 20000 - shift, 4096, 7, 70001]
    for fused in (True, False):
        rep, st = _custom(sizes, 3, 3, seed=70 + shift, cfgkw=cfgkw, fused=fused, trust=2 if fused else 0)
        assert rep.ok() and st == 0, (shift, cfgkw, fused)


@pytest.mark.parametrize("seed", range(24))
def test_random_layer_lists_and_settings(seed):
    """Seeded random layer lists (empty, tiny, odd and tile-multiple sizes, so every alignment and every
    kind of layer -- small, folded-by-the-quantizer, large -- occurs in changing order) under random
    settings of N, k_g, k_x, rounding, weight feedback, fused or separate calls, filtered scale pass."""
    rng = np.random.default_rng(1000 + seed)
    pool = [0, 1, 2, 3, 5, 31, 32, 33, 64, 255, 1000, 1001, 4095, 4096, 4097, 8192, 12289, 16384, 16385, 20000,
            4096 * 7 + 2, 65536, 100003]
    sizes = [int(rng.choice(pool)) for _ in range(int(rng.integers(1, 9)))]
    if rng.random() < 0.3:
        sizes.append(4096 * 641 + int(rng.integers(0, 5)))      # a layer of more than 640 tiles
    if sum(sizes) == 0:
        sizes.append(7)
    N = int(rng.choice([1, 2, 3, 4, 5, 8]))
    cfgkw = dict(k_g=int(rng.integers(0, 7)), k_x=int(rng.choice([0, 3, 6, 7, 10, 14])),
                 rounding=int(rng.integers(0, 2)), weight_ef=int(rng.integers(0, 2)), seed=int(rng.integers(0, 1 << 30)))
    fused = bool(rng.integers(0, 2))
    trust = int(rng.choice([0, 2]))
    rep, st = _custom(sizes, N, 3, seed=2000 + seed, cfgkw=cfgkw, fused=fused, trust=trust,
                      scale=float(10.0 ** rng.uniform(-4, 0)))
    assert rep.ok() and st == 0 and rep.float_not_bit_exact == 0, (sizes, N, cfgkw, fused, trust, rep.line())


# ------------------------------------------------------------------------------------- edge cases
RAGGED = [1, 3, 31, 33, 0, 255, 257, 4095, 4097, 5000, 0, 64, 8192, 2, 12289, 7]


def _custom(sizes, N, steps, seed=1, cfgkw=None, fused=True, scale=1e-2, weight_quant=True, gsel=None, trust=0):
    cfgkw = cfgkw or {}
    gcfg, ocfg = configs(**cfgkw)
    seg_off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    P = int(seg_off[-1])
    rng = np.random.default_rng(seed)
    q = QAdam(gcfg, seg_off, N)
    q.trust_error_buffers(trust)
    x0 = (rng.standard_normal(P) * 0.02).astype(np.float32)
    ds = DeviceState(q, torch.from_numpy(x0))
    hs = HostState(P, N, x0)
    rep = Report()
    for t in range(1, steps + 1):
        grads = [(rng.standard_normal(P) * scale).astype(np.float32) for _ in range(N)]
        if gsel:
            grads = gsel(t, grads)
        for i in range(N):
            ds.grads[i].copy_(torch.from_numpy(grads[i]))
        if fused:
            ds.step_fused(t, 1e-3, 0.999)
        else:
            ds.step_unfused(t, 1e-3, 0.999, weight_quant=weight_quant)
        out = oracle_step_layers(ocfg, seg_off, t, 1e-3, 0.999, grads, hs, weight_quant=weight_quant)
        compare_step(rep, ocfg, seg_off, ds, hs, out, weight_quant=weight_quant)
    st = q.get_status()
    q.close()
    return rep, st


@pytest.mark.parametrize("fused", [True, False])
def test_ragged_and_unaligned_segments(fused):
    """Segments of every awkward length: tails, starts off a 16-byte boundary, empty ones."""
    rep, st = _custom(RAGGED, 3, 4, fused=fused)
    _say("ragged fused=%s: %s" % (fused, rep.line()))
    assert rep.ok() and st == 0


@pytest.mark.parametrize("k_g", [0, 1, 2, 3, 4, 5, 6])
def test_all_gradient_grids(k_g):
    rep, st = _custom([5000, 37, 4096], 2, 3, cfgkw=dict(k_g=k_g), seed=10 + k_g)
    assert rep.ok() and st == 0


@pytest.mark.parametrize("k_x,weight_ef", [(0, 1), (6, 0), (7, 1), (14, 1), (14, 0), (3, 1)])
def test_weight_grids_and_feedback_modes(k_x, weight_ef):
    rep, st = _custom([9000, 130], 2, 5, cfgkw=dict(k_x=k_x, weight_ef=weight_ef), seed=20 + k_x)
    assert rep.ok() and st == 0


@pytest.mark.parametrize("N", [1, 3, 5, 8, 32])
def test_worker_counts(N):
    """Powers of two take the multiply-by-1/N path, others the division; 32 is the maximum."""
    rep, st = _custom([4100, 60], N, 2, seed=30 + N)
    assert rep.ok() and st == 0


@pytest.mark.parametrize("fused", [True, False])
def test_stochastic_rounding(fused):
    """Unbiased rounding: the GPU draws exactly the oracle's Philox numbers."""
    rep, st = _custom(RAGGED, 3, 3, cfgkw=dict(rounding=1, seed=0xDEADBEEFCAFE), fused=fused, seed=40)
    _say("stochastic fused=%s: %s" % (fused, rep.line()))
    assert rep.ok() and st == 0


def test_bias_corrected_flavour():
    rep, st = _custom([6000, 100], 2, 6, cfgkw=dict(adam_flavor=1, eps=1e-6), seed=50)
    assert rep.ok() and st == 0


def test_extreme_magnitudes_and_subnormals():
    """Gradients from subnormal to 1e30 in one vector; zero layers; exact zeros."""
    def sel(t, grads):
        out = []
        for g in grads:
            g = g.copy()
            n = g.size
            g[: n // 4] *= np.float32(1e-38)          # subnormal range after scaling
            g[n // 4: n // 2] *= np.float32(1e30)
            g[n // 2: n // 2 + 100] = 0.0
            out.append(g)
        return out
    sizes = [2048, 2048, 2048, 2048, 100]
    rep, st = _custom(sizes, 2, 3, gsel=sel, seed=60)
    assert rep.ok() and st == 0

    def zero_layer(t, grads):
        for g in grads:
            g[4096:4096 + 2048] = 0.0
        return grads
    rep, st = _custom([4096, 2048, 512], 2, 2, gsel=zero_layer, seed=61)
    assert rep.ok() and st == 0


@pytest.mark.parametrize("k_g", [0, 2, 6])
def test_values_around_decision_thresholds(k_g):
    """Gradients placed within +-12 ulp of every rounding threshold of Q_g for many scales: the
    kernel takes the level from p * (1/s) and falls back to the IEEE quotient near a threshold;
    every decision must still equal the oracle's, which always divides."""
    rng = np.random.default_rng(70 + k_g)
    taus = [2.0 ** (-k_g - 1)] + [0.75 * 2.0 ** -j for j in range(0, k_g)] + [2.0 ** -j for j in range(0, k_g + 1)]
    sizes, chunks = [], []
    for trial in range(24):
        s_val = np.float32(10.0 ** rng.uniform(-30, 30)) if trial % 3 else np.float32(2.0 ** rng.integers(-90, 90))
        vals = [s_val]
        for tau in taus:
            centre = np.float32(np.float64(s_val) * tau)
            v = centre
            ups, downs = [], []
            for _ in range(12):
                v = np.nextafter(v, np.float32(np.inf)); ups.append(v)
            v = centre
            for _ in range(12):
                v = np.nextafter(v, np.float32(0)); downs.append(v)
            vals += [centre] + ups + downs
        arr = np.array(vals, np.float32)
        arr = np.concatenate([arr, -arr[1:]])
        arr = np.minimum(np.abs(arr), s_val) * np.sign(arr)       # the scale stays s_val
        rng.shuffle(arr[1:])
        chunks.append(arr.astype(np.float32))
        sizes.append(arr.size)
    gvec = np.concatenate(chunks)

    def sel(t, grads):
        return [gvec.copy() for _ in grads]
    rep, st = _custom(sizes, 2, 2, gsel=sel, cfgkw=dict(k_g=k_g), seed=80)
    _say("thresholds k_g=%d: %s" % (k_g, rep.line()))
    assert rep.ok() and st == 0 and rep.ties_g > 0


def test_nonfinite_gradient_sets_status():
    gcfg, ocfg = configs()
    seg_off = [0, 1000, 3000]
    q = QAdam(gcfg, seg_off, 1)
    x0 = torch.zeros(3000)
    ds = DeviceState(q, x0)
    g = torch.randn(3000) * 0.01
    g[1500] = float("nan")
    ds.grads[0].copy_(g)
    ds.step_fused(1, 1e-3, 0.999)
    assert q.get_status(clear=True) == 1
    assert q.get_status() == 0
    sc = ds.scales[0].cpu().numpy()
    assert np.isfinite(sc[0]) and np.isnan(sc[1])
    # codes stay in range, the finite layer is unaffected
    hs = HostState(3000, 1, x0.numpy())
    out = oracle_step_layers(ocfg, seg_off, 1, 1e-3, 0.999, [g.numpy()], hs)
    assert out["status"] == 1
    gw = ds.host_codes(0)
    nw0 = 32 * 3
    assert np.array_equal(gw[:nw0], out["words"][0][:nw0])
    assert np.array_equal(ds.errs[0][:1000].cpu().numpy(), hs.errs[0][:1000])
    g[1500] = float("inf")
    ds.grads[0].copy_(g)
    ds.step_unfused(2, 1e-3, 0.999)
    assert q.get_status(clear=True) == 1
    q.close()


def test_empty_vector_and_argument_errors():
    gcfg, _ = configs()
    q = QAdam(gcfg, [0], 2)
    assert q.num_params == 0 and q.grad_code_bytes() == 0
    e = torch.zeros(0, device="cuda")
    sc = [torch.zeros(1, device="cuda") for _ in range(2)]
    cd = [torch.zeros(4, dtype=torch.int32, device="cuda") for _ in range(2)]
    q.step_fused(1, 1e-3, 0.999, [e, e], [e, e], cd, sc, e, e, e, e, torch.zeros(1, dtype=torch.int8, device="cuda"))
    torch.cuda.synchronize()
    q.close()
    q = QAdam(gcfg, [0, 64], 2)
    buf = torch.zeros(128, device="cuda")
    codes = torch.zeros(64, dtype=torch.int32, device="cuda")
    with pytest.raises(QAdamError) as ei:
        q.worker_quantize(2, 1, buf[:64], buf[64:], codes, buf[:1])
    assert ei.value.code == -1
    with pytest.raises(QAdamError) as ei:
        q.worker_quantize(0, 1, buf[1:65], buf[64:], codes, buf[:1])       # 4-byte aligned only
    assert ei.value.code == -2
    with pytest.raises(QAdamError) as ei:
        q.worker_quantize(0, 0, buf[:64], buf[64:], codes, buf[:1])        # step is 1-based
    assert ei.value.code == -1
    # the binding refuses buffers a kernel would overrun or misread, before the library is called
    for bad in (lambda: q.worker_quantize(0, 1, buf[:32], buf[64:], codes, buf[:1]),              # too few elements
                lambda: q.worker_quantize(0, 1, buf[:64].double(), buf[64:], codes, buf[:1]),     # wrong type
                lambda: q.worker_quantize(0, 1, buf[:64], buf[64:], codes[:2], buf[:1]),          # codes too short
                lambda: q.worker_quantize(0, 1, buf[:64].cpu(), buf[64:], codes, buf[:1]),        # host memory
                lambda: q.worker_quantize(0, 1, buf[:64], buf[64:], codes, buf[:0]),              # no room for the scale
                lambda: q.server_step(1, 1e-3, 0.999, [codes], [buf[:1]], buf[:64], buf[:64], buf[:64])):  # N = 2 expected
        with pytest.raises(ValueError):
            bad()
    q.close()


def test_arena_layout_places_every_buffer_and_changes_no_result():
    """qadam_arena_layout: offsets are aligned, inside the block and disjoint; the two groups of buffers
    lie in the two halves of a large block; a step on buffers carved out of one block gives the bits of a
    step on separately allocated buffers."""
    gcfg, _ = configs(k_g=2, k_x=6)
    sizes = RAGGED + [70000]
    seg_off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    P, N, L = int(seg_off[-1]), 4, len(sizes)
    q = QAdam(gcfg, seg_off, N)
    need = q.arena_layout(1 << 40)["bytes_needed"]
    with pytest.raises(QAdamError) as ei:
        q.arena_layout(need - 1)
    assert ei.value.code == -3
    for arena_bytes, wm in [(need, False), (need, True), (4 * need + 12345, False), (64 << 20, True)]:
        if wm:
            need_w = q.arena_layout(1 << 40, True)["bytes_needed"]
            arena_bytes = max(arena_bytes, need_w)
        lay = q.arena_layout(arena_bytes, wm)
        spans = []
        for name, nbytes in [("x", 4 * P), ("m", 4 * P), ("v", 4 * P), ("werr", 4 * P), ("wcodes", q.weight_code_bytes())]:
            spans.append((lay[name], lay[name] + nbytes, name))
        per_worker = [("grads", 4 * P), ("errs", 4 * P), ("codes", q.grad_code_bytes()), ("scales", 4 * L)]
        if wm:
            per_worker += [("mw", 4 * P), ("vw", 4 * P)]
        for name, nbytes in per_worker:
            assert len(lay[name]) == N
            spans += [(o, o + nbytes, "%s[%d]" % (name, i)) for i, o in enumerate(lay[name])]
        spans.sort()
        for (a0, a1, an), (b0, b1, bn) in zip(spans, spans[1:]):
            assert a1 <= b0, (an, bn)
        assert all(a % 256 == 0 for a, _, _ in spans) and spans[-1][1] <= arena_bytes
        if arena_bytes >= 4 * need:     # roomy block: half of the fp32 buffers start in its second half
            big = [a for a, b, n in spans if b - a == 4 * P]
            assert sum(a >= arena_bytes // 2 - (2 << 20) for a in big) == len(big) // 2
    # same bits in the block as in separate allocations
    arena_bytes = 3 * need
    lay = q.arena_layout(arena_bytes)
    block = torch.zeros(arena_bytes, dtype=torch.uint8, device="cuda")
    f32 = lambda off, n: block[off:off + 4 * n].view(torch.float32)
    gen = torch.Generator().manual_seed(21)
    x0 = torch.randn(P, generator=gen) * 0.02
    ref = DeviceState(q, x0)
    x, m, v, werr = (f32(lay[k], P) for k in ("x", "m", "v", "werr"))
    x.copy_(x0)
    grads = [f32(o, P) for o in lay["grads"]]
    errs = [f32(o, P) for o in lay["errs"]]
    codes = [block[o:o + q.grad_code_bytes()].view(torch.int32) for o in lay["codes"]]
    scales = [f32(o, L) for o in lay["scales"]]
    wcodes = block[lay["wcodes"]:lay["wcodes"] + P].view(torch.int8)
    for t in range(1, 4):
        for i in range(N):
            g = torch.randn(P, generator=gen) * 0.01
            grads[i].copy_(g); ref.grads[i].copy_(g)
        q.step_fused(t, 1e-3, 0.999, grads, errs, codes, scales, x, m, v, werr, wcodes)
        ref.step_fused(t, 1e-3, 0.999)
        torch.cuda.synchronize()
        assert torch.equal(x, ref.x) and torch.equal(m, ref.m) and torch.equal(v, ref.v) and torch.equal(werr, ref.werr)
        assert torch.equal(wcodes, ref.wcodes[:P])
        for i in range(N):
            assert torch.equal(errs[i], ref.errs[i]) and torch.equal(scales[i], ref.scales[i][:L])
            assert torch.equal(codes[i], ref.codes[i][: q.grad_code_bytes() // 4])
    assert q.get_status() == 0
    q.close()


def test_fused_equals_three_calls_on_device():
    """qadam_step_fused and the three separate calls give the same bits on the GPU itself."""
    gcfg, _ = configs(k_g=2, k_x=6)
    sizes = RAGGED + [20000]
    seg_off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    P, N = int(seg_off[-1]), 4
    q = QAdam(gcfg, seg_off, N)
    g = torch.Generator().manual_seed(5)
    x0 = torch.randn(P, generator=g) * 0.02
    a, b = DeviceState(q, x0), DeviceState(q, x0)
    for t in range(1, 6):
        for i in range(N):
            gr = torch.randn(P, generator=g) * 0.01
            a.grads[i].copy_(gr); b.grads[i].copy_(gr)
        a.step_fused(t, 1e-3, 0.999)
        b.step_unfused(t, 1e-3, 0.999)
        torch.cuda.synchronize()
        for name in ("x", "m", "v", "werr", "wcodes"):
            assert torch.equal(getattr(a, name), getattr(b, name)), name
        for i in range(N):
            assert torch.equal(a.errs[i], b.errs[i]) and torch.equal(a.codes[i], b.codes[i])
            assert torch.equal(a.scales[i], b.scales[i])
    q.close()


def test_weight_dequantize_roundtrip():
    gcfg, ocfg = configs(k_x=6)
    P = 10000
    q = QAdam(gcfg, [0, P], 1)
    x = (torch.rand(P) - 0.5).cuda()
    werr = torch.zeros(P, device="cuda")
    wc = torch.zeros(P, dtype=torch.int8, device="cuda")
    xh = torch.zeros(P, device="cuda")
    q.weight_quantize(1, x, werr, wc)
    q.weight_dequantize(wc, xh)
    torch.cuda.synchronize()
    want = oracle.qx(ocfg, x.cpu().numpy())[1]
    assert np.array_equal(xh.cpu().numpy(), want)
    assert torch.equal(xh + werr, x)
    q.close()


@pytest.mark.parametrize("k_x", [6, 10, 14])
def test_weight_dequantize_half_precision(k_x):
    """binary16 output: exact up to k_x = 10 (|j| <= 1024 fits 11 significand bits), round to nearest
    even of the fp32 value beyond; checked against numpy's float32 -> float16 conversion."""
    gcfg, ocfg = configs(k_x=k_x)
    P = 70001
    q = QAdam(gcfg, [0, P], 1)
    x = ((torch.rand(P, generator=torch.Generator().manual_seed(k_x)) - 0.5) * 1.1).cuda()
    werr = torch.zeros(P, device="cuda")
    wc = torch.zeros(P, dtype=torch.int8 if k_x <= 6 else torch.int16, device="cuda")
    xh = torch.zeros(P, dtype=torch.float16, device="cuda")
    q.weight_quantize(1, x, werr, wc)
    q.weight_dequantize_f16(wc, xh)
    torch.cuda.synchronize()
    want32 = oracle.qx(ocfg, x.cpu().numpy())[1]
    want16 = want32.astype(np.float16)
    got = xh.cpu().numpy()
    assert np.array_equal(got, want16)          # as values: the sign of a zero is not part of x^
    if k_x <= 10:
        assert np.array_equal(got.astype(np.float32), want32)
    q.close()


# ------------------------------------------------------------- variant W (Algorithms 2-3 as printed)
@pytest.mark.parametrize("rounding", [0, 1])
def test_variant_w_worker_moments(rounding):
    """Workers own m_i, v_i and quantize alpha m / sqrt(v + eps) + e (Algorithm 3); the server
    subtracts the mean message (Algorithm 2) and emits Q_x."""
    gcfg, ocfg = configs(k_g=2, k_x=6, rounding=rounding, seed=77, eps=1e-5)
    sizes = RAGGED + [20000]
    seg_off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    P, N = int(seg_off[-1]), 3
    rng = np.random.default_rng(90 + rounding)
    q = QAdam(gcfg, seg_off, N)
    x0 = (rng.standard_normal(P) * 0.02).astype(np.float32)
    ds = DeviceState(q, torch.from_numpy(x0))
    mw = [torch.zeros(P, device="cuda") for _ in range(N)]
    vw = [torch.zeros(P, device="cuda") for _ in range(N)]
    hx = x0.copy()
    he = [np.zeros(P, np.float32) for _ in range(N)]
    hm = [np.zeros(P, np.float32) for _ in range(N)]
    hv = [np.zeros(P, np.float32) for _ in range(N)]
    hw = np.zeros(P, np.float32)
    rep = Report()
    for t in range(1, 6):
        grads = [(rng.standard_normal(P) * 1e-2).astype(np.float32) for _ in range(N)]
        for i in range(N):
            ds.grads[i].copy_(torch.from_numpy(grads[i]))
            q.worker_step_w(i, t, 1e-3, 0.999, ds.grads[i], mw[i], vw[i], ds.errs[i], ds.codes[i], ds.scales[i])
        q.server_apply_w(t, ds.codes, ds.scales, ds.x)
        q.weight_quantize(t, ds.x, ds.werr, ds.wcodes)
        out = oracle.step_w(ocfg, seg_off, t, 1e-3, 0.999, grads, he, hm, hv, hx, hw)
        torch.cuda.synchronize()
        for i in range(N):
            assert np.array_equal(ds.host_codes(i), out["words"][i]), "codes of worker %d step %d" % (i, t)
            assert np.array_equal(ds.scales[i][: len(sizes)].cpu().numpy(), out["scales"][i])
            from parity_util import close
            close(rep, "err", ds.errs[i].cpu().numpy(), he[i])
            close(rep, "mw", mw[i].cpu().numpy(), hm[i])
            close(rep, "vw", vw[i].cpu().numpy(), hv[i])
        close(rep, "x", ds.x.cpu().numpy(), hx)
        close(rep, "werr", ds.werr.cpu().numpy(), hw)
        assert np.array_equal(ds.wcodes[:P].cpu().numpy(), out["wcodes"])
    assert q.get_status() == 0 and rep.float_not_bit_exact == 0
    q.close()


@pytest.mark.parametrize("N,rounding", [(4, 0), (3, 0), (2, 1), (1, 0), (8, 0)])
def test_variant_w_fused_step(N, rounding):
    """qadam_step_fused_w against the oracle's Algorithms 2-3 and against the separate calls
    (N = 1 is the single-machine Algorithm 1)."""
    gcfg, ocfg = configs(k_g=2, k_x=6, rounding=rounding, seed=5, eps=1e-6)
    sizes = RAGGED + [30000]
    seg_off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    P = int(seg_off[-1])
    rng = np.random.default_rng(120 + N)
    q = QAdam(gcfg, seg_off, N)
    x0 = (rng.standard_normal(P) * 0.02).astype(np.float32)
    a, b = DeviceState(q, torch.from_numpy(x0)), DeviceState(q, torch.from_numpy(x0))
    zeros = lambda: [torch.zeros(P, device="cuda") for _ in range(N)]
    amw, avw, bmw, bvw = zeros(), zeros(), zeros(), zeros()
    hx = x0.copy()
    he, hm, hv = ([np.zeros(P, np.float32) for _ in range(N)] for _ in range(3))
    hw = np.zeros(P, np.float32)
    rep = Report()
    from parity_util import close
    for t in range(1, 5):
        grads = [(rng.standard_normal(P) * 1e-2).astype(np.float32) for _ in range(N)]
        for i in range(N):
            a.grads[i].copy_(torch.from_numpy(grads[i])); b.grads[i].copy_(a.grads[i])
        q.step_fused_w(t, 1e-3, 0.999, a.grads, amw, avw, a.errs, a.codes, a.scales, a.x, a.werr, a.wcodes)
        for i in range(N):
            q.worker_step_w(i, t, 1e-3, 0.999, b.grads[i], bmw[i], bvw[i], b.errs[i], b.codes[i], b.scales[i])
        q.server_apply_w(t, b.codes, b.scales, b.x)
        q.weight_quantize(t, b.x, b.werr, b.wcodes)
        out = oracle.step_w(ocfg, seg_off, t, 1e-3, 0.999, grads, he, hm, hv, hx, hw)
        torch.cuda.synchronize()
        for name in ("x", "werr", "wcodes"):
            assert torch.equal(getattr(a, name), getattr(b, name)), name
        for i in range(N):
            assert torch.equal(a.errs[i], b.errs[i]) and torch.equal(a.codes[i], b.codes[i])
            assert torch.equal(amw[i], bmw[i]) and torch.equal(avw[i], bvw[i]) and torch.equal(a.scales[i], b.scales[i])
            assert np.array_equal(a.host_codes(i), out["words"][i])
            close(rep, "err", a.errs[i].cpu().numpy(), he[i])
            close(rep, "mw", amw[i].cpu().numpy(), hm[i])
            close(rep, "vw", avw[i].cpu().numpy(), hv[i])
        close(rep, "x", a.x.cpu().numpy(), hx)
        close(rep, "werr", a.werr.cpu().numpy(), hw)
        assert np.array_equal(a.wcodes[:P].cpu().numpy(), out["wcodes"])
    assert q.get_status() == 0 and rep.float_not_bit_exact == 0
    q.close()


@pytest.mark.filterwarnings("ignore:The CUDA Graph is empty")     # the two refused captures record nothing
def test_step_is_capturable_in_a_hip_graph():
    """The compute calls only enqueue kernels (no allocation, no memset, no synchronisation), so a
    step can be captured once and replayed; every replay must equal the eager call on a twin state."""
    gcfg, _ = configs(k_g=2, k_x=6)
    sizes = RAGGED + [50000]
    seg_off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    P, N = int(seg_off[-1]), 4
    q = QAdam(gcfg, seg_off, N)
    q.trust_error_buffers(2)       # a recorded call must take the full scale pass all the same
    qb = QAdam(gcfg, seg_off, N)   # the eager twin has its own handle (replays update q's residual bounds)
    qb.trust_error_buffers(2)
    gen = torch.Generator().manual_seed(11)
    x0 = torch.randn(P, generator=gen) * 0.02
    a, b = DeviceState(q, x0), DeviceState(qb, x0)
    for i in range(N):
        a.grads[i].copy_(torch.randn(P, generator=gen) * 0.01)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        a.step_fused(1, 1e-3, 0.999)
    # capture does not execute: a's state is untouched so far
    assert torch.equal(a.x.cpu(), x0)
    for rep in range(4):
        for i in range(N):
            gr = torch.randn(P, generator=gen) * 0.01
            a.grads[i].copy_(gr); b.grads[i].copy_(gr)
        if rep == 2:
            # the caller changes the error buffers between replays: allowed, the recorded scale pass reads everything
            for i in range(N):
                e = torch.randn(P, generator=gen) * 0.05
                a.errs[i].copy_(e); b.errs[i].copy_(e)
            qb.trust_error_buffers(2)  # the eager twin must say so (contract of the filtered pass); the graph need not
        graph.replay()
        # with nearest rounding and the paper's Adam the step number enters no kernel: a replay stands for any t
        b.step_fused(rep + 1, 1e-3, 0.999)
        torch.cuda.synchronize()
        for name in ("x", "m", "v", "werr", "wcodes"):
            assert torch.equal(getattr(a, name), getattr(b, name)), (rep, name)
        for i in range(N):
            assert torch.equal(a.errs[i], b.errs[i]) and torch.equal(a.codes[i], b.codes[i]), rep
            assert torch.equal(a.scales[i], b.scales[i])
        # eager work between replays
        _ = (a.x * 2).sum().item()
    assert q.get_status() == 0 and qb.get_status() == 0
    q.close()
    qb.close()
    # what a replay cannot follow is refused while a graph is being recorded: the per-step random stream
    # of stochastic rounding and the per-step bias corrections
    for kw in (dict(rounding=1), dict(adam_flavor=1)):
        gcfg2, _ = configs(k_g=2, k_x=6, **kw)
        q2 = QAdam(gcfg2, seg_off, N)
        c = DeviceState(q2, x0)
        torch.cuda.synchronize()
        g2 = torch.cuda.CUDAGraph()
        refused = False
        with torch.cuda.graph(g2):
            try:
                c.step_fused(1, 1e-3, 0.999)
            except QAdamError as ex:
                refused = ex.code == -1
        assert refused, kw
        c.step_fused(1, 1e-3, 0.999)          # the same call outside a capture is fine
        torch.cuda.synchronize()
        q2.close()


@pytest.mark.parametrize("rounding", [0, 1])
def test_checkpoint_and_resume_is_bit_identical(rounding):
    """The complete state of the method is (x, m, v, e^x, e_1..e_N, t): all caller-owned buffers.
    Ten steps in one go equal five steps, a copy of those buffers to the host, a NEW handle with new
    device buffers restored from the copy, and five more steps -- bit for bit, also with stochastic
    rounding (its random stream is a function of seed, step, worker and index only)."""
    gcfg, _ = configs(k_g=2, k_x=6, rounding=rounding, seed=99)
    sizes = RAGGED + [30000]
    seg_off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    P, N = int(seg_off[-1]), 3
    gen = torch.Generator().manual_seed(5)
    x0 = torch.randn(P, generator=gen) * 0.02
    grads = [[torch.randn(P, generator=gen) * 0.01 for _ in range(N)] for _ in range(10)]

    def run(ds, t0, t1):
        for t in range(t0, t1 + 1):
            for i in range(N):
                ds.grads[i].copy_(grads[t - 1][i])
            ds.step_fused(t, 1e-3 / np.sqrt(t), 1.0 - 0.5 / t)     # Assumption 4 style schedules

    q1 = QAdam(gcfg, seg_off, N)
    full = DeviceState(q1, x0)
    run(full, 1, 10)
    q2 = QAdam(gcfg, seg_off, N)
    first = DeviceState(q2, x0)
    run(first, 1, 5)
    torch.cuda.synchronize()
    saved = dict(x=first.x.cpu(), m=first.m.cpu(), v=first.v.cpu(), werr=first.werr.cpu(),
                 errs=[e.cpu() for e in first.errs])
    del first
    q2.close()
    q3 = QAdam(gcfg, seg_off, N)
    second = DeviceState(q3, saved["x"])
    second.m.copy_(saved["m"]); second.v.copy_(saved["v"]); second.werr.copy_(saved["werr"])
    for i in range(N):
        second.errs[i].copy_(saved["errs"][i])
    run(second, 6, 10)
    torch.cuda.synchronize()
    for name in ("x", "m", "v", "werr", "wcodes"):
        assert torch.equal(getattr(full, name), getattr(second, name)), name
    for i in range(N):
        assert torch.equal(full.errs[i], second.errs[i]) and torch.equal(full.codes[i], second.codes[i])
        assert torch.equal(full.scales[i], second.scales[i])
    assert q1.get_status() == 0 and q3.get_status() == 0
    q1.close(); q3.close()


def test_layer_sumsq_and_assumption2_on_device():
    """qadam_layer_sumsq: fp64 per-layer sums in a fixed order (same bits on every run), equal to a
    plain fp64 sum within accumulation error; used before and after a step it gives the empirical
    ||p - Q_g(p)||^2 / ||p||^2 of Assumption 2, which must stay below 1 in every layer."""
    gcfg, _ = configs(k_g=2, k_x=6)
    sizes = RAGGED + [1 << 20, 300000]
    seg_off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    L, P, N = len(sizes), int(seg_off[-1]), 2
    q = QAdam(gcfg, seg_off, N)
    gen = torch.Generator().manual_seed(21)
    x0 = torch.randn(P, generator=gen) * 0.02
    ds = DeviceState(q, x0)
    for i in range(N):
        ds.grads[i].copy_(torch.randn(P, generator=gen) * 0.01)
        ds.errs[i].copy_(torch.randn(P, generator=gen) * 0.002)
    before = [torch.zeros(L, dtype=torch.float64, device="cuda") for _ in range(N)]
    again = torch.zeros(L, dtype=torch.float64, device="cuda")
    after = [torch.zeros(L, dtype=torch.float64, device="cuda") for _ in range(N)]
    for i in range(N):
        q.layer_sumsq(ds.grads[i], ds.errs[i], before[i])
    q.layer_sumsq(ds.grads[0], ds.errs[0], again)
    torch.cuda.synchronize()
    assert torch.equal(before[0], again)                       # fixed order: bit-identical reruns
    p_host = [(ds.grads[i] + ds.errs[i]).cpu().numpy().astype(np.float64) for i in range(N)]
    ds.step_fused(1, 1e-3, 0.999)
    for i in range(N):
        q.layer_sumsq(ds.errs[i], None, after[i])
    torch.cuda.synchronize()
    for i in range(N):
        e_host = ds.errs[i].cpu().numpy().astype(np.float64)
        b, a = before[i].cpu().numpy(), after[i].cpu().numpy()
        for l in range(L):
            lo, hi = int(seg_off[l]), int(seg_off[l + 1])
            want_b = float(np.sum(p_host[i][lo:hi] ** 2))
            want_a = float(np.sum(e_host[lo:hi] ** 2))
            assert abs(b[l] - want_b) <= 1e-12 * want_b and abs(a[l] - want_a) <= 1e-12 * max(want_a, 1e-300), (i, l)
            if hi > lo:
                assert a[l] < b[l], "Assumption 2 violated in layer %d of worker %d" % (l, i)
    assert q.get_status() == 0
    q.close()


@pytest.mark.parametrize("variant", ["s", "w"])
def test_closed_loop_on_device_follows_the_oracle(variant):
    """The loop of Algorithms 2-3 run end to end on the device: workers take gradients of
    f(x) = 1/2 ||x - x*||^2 at the dequantized broadcast Q_x(x_t) (qadam_weight_dequantize), the step
    runs in the library, 300 iterations with alpha_t = alpha / sqrt(t).  The oracle runs the same loop
    from its own state; the two trajectories stay bit-identical, and the iterate ends within a few
    weight-grid steps of x* (Theorems 2-3, qualitatively)."""
    n, N, T = 5000, 4, 300
    gcfg, ocfg = configs(k_g=0, k_x=6, weight_ef=0)
    rng = np.random.default_rng(17)
    xstar = rng.uniform(-0.4, 0.4, n).astype(np.float32)
    noise = (rng.standard_normal((T, N, n)) * 0.01).astype(np.float32)
    seg = [0, 3000, n]
    q = QAdam(gcfg, seg, N)
    dev = "cuda"
    z = lambda: torch.zeros(n, device=dev)
    x, m, v, werr, xhat = z(), z(), z(), z(), z()
    errs, grads = [z() for _ in range(N)], [z() for _ in range(N)]
    mw, vw = [z() for _ in range(N)], [z() for _ in range(N)]
    codes = [torch.zeros(q.grad_code_bytes() // 4, dtype=torch.int32, device=dev) for _ in range(N)]
    scales = [torch.zeros(2, device=dev) for _ in range(N)]
    wcodes = torch.zeros(n, dtype=torch.int8, device=dev)
    xs_d, noise_d = torch.from_numpy(xstar).to(dev), torch.from_numpy(noise).to(dev)
    # oracle state
    hx, hw = np.zeros(n, np.float32), np.zeros(n, np.float32)
    hm, hv = np.zeros(n, np.float32), np.zeros(n, np.float32)
    he = [np.zeros(n, np.float32) for _ in range(N)]
    hmw, hvw = [np.zeros(n, np.float32) for _ in range(N)], [np.zeros(n, np.float32) for _ in range(N)]
    hxhat = np.zeros(n, np.float32)
    for t in range(1, T + 1):
        lr = float(np.float32(2e-2 / np.sqrt(t)))
        for i in range(N):
            grads[i].copy_((xhat - xs_d) + noise_d[t - 1, i])
        hg = [((hxhat - xstar) + noise[t - 1, i]).astype(np.float32) for i in range(N)]
        if variant == "s":
            q.step_fused(t, lr, 0.999, grads, errs, codes, scales, x, m, v, werr, wcodes)
            out = oracle.step_s(ocfg, seg, t, lr, 0.999, hg, he, hx, hm, hv, hw)
        else:
            q.step_fused_w(t, lr, 0.999, grads, mw, vw, errs, codes, scales, x, werr, wcodes)
            out = oracle.step_w(ocfg, seg, t, lr, 0.999, hg, he, hmw, hvw, hx, hw)
        q.weight_dequantize(wcodes, xhat)
        hxhat = out["wcodes"].astype(np.float32) * np.float32(2.0 ** -7)
        if t % 50 == 0 or t == T:
            assert np.array_equal(xhat.cpu().numpy(), hxhat), t
            assert np.array_equal(x.cpu().numpy().view(np.uint32), hx.view(np.uint32)), t
    dist = np.abs(hxhat - xstar)
    assert dist.max() < 6 * 2.0 ** -7
    assert q.get_status() == 0
    q.close()


def test_workers_on_concurrent_streams():
    """Worker calls of different workers enqueued on different streams (the handle keeps separate
    scratch per worker), joined by events before the server call: same bits as the fused call."""
    gcfg, _ = configs(k_g=2, k_x=6)
    sizes = RAGGED + [1 << 20, 200000]
    seg_off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    P, N = int(seg_off[-1]), 4
    q = QAdam(gcfg, seg_off, N)
    gen = torch.Generator().manual_seed(31)
    x0 = torch.randn(P, generator=gen) * 0.02
    a, b = DeviceState(q, x0), DeviceState(q, x0)
    streams = [torch.cuda.Stream() for _ in range(N)]
    main = torch.cuda.current_stream()
    for t in range(1, 4):
        for i in range(N):
            g = torch.randn(P, generator=gen) * 0.01
            a.grads[i].copy_(g); b.grads[i].copy_(g)
        torch.cuda.synchronize()
        for i in range(N):
            q.worker_quantize(i, t, a.grads[i], a.errs[i], a.codes[i], a.scales[i], stream=streams[i])
        for i in range(N):
            main.wait_stream(streams[i])
        q.server_step(t, 1e-3, 0.999, a.codes, a.scales, a.x, a.m, a.v)
        q.weight_quantize(t, a.x, a.werr, a.wcodes)
        torch.cuda.synchronize()
        b.step_fused(t, 1e-3, 0.999)
        torch.cuda.synchronize()
        for name in ("x", "m", "v", "werr", "wcodes"):
            assert torch.equal(getattr(a, name), getattr(b, name)), (t, name)
        for i in range(N):
            assert torch.equal(a.errs[i], b.errs[i]) and torch.equal(a.codes[i], b.codes[i]), (t, i)
            assert torch.equal(a.scales[i], b.scales[i])
    assert q.get_status() == 0
    q.close()


# --------------------------------------------- identity quantizers (settings of Theorems 1 and 2)
@pytest.mark.parametrize("variant", ["s", "w"])
@pytest.mark.parametrize("idg,idx", [(True, False), (False, True), (True, True)])
def test_identity_quantizers_on_device(variant, idg, idx):
    """k_g = QADAM_IDENTITY (full-precision messages, Theorem 2's setting), k_x = QADAM_IDENTITY
    (full-precision weights, Theorem 1's setting), and both (plain distributed generic Adam), in the
    whole-step calls of both variants, against the oracle's identity-quantizer steps."""
    from paper_2004_14180_amd import QADAM_IDENTITY
    from parity_util import close
    k_g, k_x = (QADAM_IDENTITY if idg else 2), (QADAM_IDENTITY if idx else 6)
    gcfg = QAdamConfig(k_g=k_g, k_x=k_x, weight_ef=1, beta1=0.9, eps=1e-6)
    ocfg = oracle.OracleConfig(k_g=2, k_x=6, weight_ef=1, beta1=0.9, eps=1e-6,
                               identity_g=int(idg), identity_x=int(idx))
    sizes = RAGGED + [40000]
    seg_off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    P, N, L = int(seg_off[-1]), 4, len(sizes)
    rng = np.random.default_rng(300 + 2 * idg + idx)
    q = QAdam(gcfg, seg_off, N)
    assert (q.grad_code_bytes() == 0) == idg and (q.weight_code_bytes() == 0) == idx
    dev = "cuda"
    z = lambda: torch.zeros(P, device=dev)
    x0 = (rng.standard_normal(P) * 0.02).astype(np.float32)
    x, m, v, werr = torch.from_numpy(x0).to(dev), z(), z(), z()
    errs, grads, mw, vw = ([z() for _ in range(N)] for _ in range(4))
    codes = None if idg else [torch.zeros(max(q.grad_code_bytes() // 4, 1), dtype=torch.int32, device=dev) for _ in range(N)]
    scales = None if idg else [torch.zeros(L, device=dev) for _ in range(N)]
    wcodes = None if idx else torch.zeros(P, dtype=torch.int8, device=dev)
    hx, hm, hv, hw = x0.copy(), np.zeros(P, np.float32), np.zeros(P, np.float32), np.zeros(P, np.float32)
    he, hmw, hvw = ([np.zeros(P, np.float32) for _ in range(N)] for _ in range(3))
    rep = Report()
    for t in range(1, 5):
        g = [(rng.standard_normal(P) * 1e-2).astype(np.float32) for _ in range(N)]
        for i in range(N):
            grads[i].copy_(torch.from_numpy(g[i]))
        if variant == "s":
            q.step_fused(t, 1e-3, 0.999, grads, None if idg else errs, codes, scales, x, m, v,
                         None if idx else werr, wcodes)
            out = oracle.step_s(ocfg, seg_off, t, 1e-3, 0.999, g, he, hx, hm, hv, hw)
        else:
            q.step_fused_w(t, 1e-3, 0.999, grads, mw, vw, errs, codes, scales, x, None if idx else werr, wcodes)
            out = oracle.step_w(ocfg, seg_off, t, 1e-3, 0.999, g, he, hmw, hvw, hx, hw)
        torch.cuda.synchronize()
        close(rep, "x", x.cpu().numpy(), hx)
        if variant == "s":
            close(rep, "m", m.cpu().numpy(), hm); close(rep, "v", v.cpu().numpy(), hv)
        else:
            for i in range(N):
                close(rep, "mw", mw[i].cpu().numpy(), hmw[i]); close(rep, "vw", vw[i].cpu().numpy(), hvw[i])
        for i in range(N):
            close(rep, "err", errs[i].cpu().numpy(), he[i])
            if not idg:
                assert np.array_equal(codes[i][: q.grad_code_bytes() // 4].cpu().numpy().view(np.uint32), out["words"][i])
        if not idx:
            assert np.array_equal(wcodes.cpu().numpy(), out["wcodes"])
            close(rep, "werr", werr.cpu().numpy(), hw)
    assert rep.float_not_bit_exact == 0 and q.get_status() == 0
    # the calls of a quantizer that is switched off are refused
    if idg:
        with pytest.raises(QAdamError):
            q.worker_quantize(0, 1, grads[0], errs[0], torch.zeros(P, dtype=torch.int32, device=dev), errs[2])
    if idx:
        with pytest.raises(QAdamError):
            q.weight_quantize(1, x, werr, torch.zeros(P, dtype=torch.int8, device=dev))
    q.close()


# ------------------------------------------------ filtered scale pass (qadam_trust_error_buffers)
@pytest.mark.parametrize("config,shrink,steps", [(2, 8, 12), (3, 4, 8), (4, 64, 6), (5, 16, 6)])
def test_filtered_scale_pass_matches_the_oracle(config, shrink, steps):
    """With qadam_trust_error_buffers the scale pass reads e only where |g| can still reach the
    layer's maximum; every output must stay what the oracle computes (Gaussian, heavy-tailed and
    adversarial gradients; the first step reads everything, the later ones are filtered)."""
    wl = make_workload(config, shrink=shrink)
    rep = run_workload_parity(wl, steps, fused=True, trust_errs=True, progress="filtered cfg%d" % config)
    _say("filtered scale pass, config %d/%d: %s" % (config, shrink, rep.line()))
    assert rep.ok() and rep.float_not_bit_exact == 0


@pytest.mark.parametrize("k_g,rounding", [(2, 0), (0, 0), (1, 1), (6, 0)])
def test_filtered_scale_pass_equals_the_full_one(k_g, rounding):
    """Same inputs through a handle with the option and one without, on ragged and unaligned
    layers with gradients whose size changes from step to step (so the lower bound from the sample
    and the bound on e are of different orders): bit-identical state after every step."""
    gcfg, _ = configs(k_g=k_g, k_x=6, rounding=rounding, seed=3)
    sizes = RAGGED + [1 << 19, 300001, 70000]
    seg_off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    P, N = int(seg_off[-1]), 3
    qa, qb = QAdam(gcfg, seg_off, N), QAdam(gcfg, seg_off, N)
    qa.trust_error_buffers(2)
    gen = torch.Generator().manual_seed(41 + k_g)
    x0 = torch.randn(P, generator=gen) * 0.02
    a, b = DeviceState(qa, x0), DeviceState(qb, x0)
    # shrinking, growing and all-zero gradients, then layers that live entirely among the subnormals
    amp = [1e-2, 1e-2, 1e-4, 1e-4, 1.0, 1e-3, 0.0, 1e-2, 1e-2, 1e-30, 1e-39, 1e-39, 1e-43, 1e-43, 1e-44, 1e-2]
    for t, scale in enumerate(amp, start=1):
        for i in range(N):
            g = torch.randn(P, generator=gen) * scale
            if t == 5:
                g[torch.rand(P, generator=gen) < 1e-4] = 50.0            # sparse outliers
            a.grads[i].copy_(g); b.grads[i].copy_(g)
        a.step_fused(t, 1e-3, 0.999)
        b.step_fused(t, 1e-3, 0.999)
        torch.cuda.synchronize()
        for name in ("x", "m", "v", "werr", "wcodes"):
            assert torch.equal(getattr(a, name), getattr(b, name)), (t, name)
        for i in range(N):
            assert torch.equal(a.scales[i], b.scales[i]), (t, i)
            assert torch.equal(a.errs[i], b.errs[i]) and torch.equal(a.codes[i], b.codes[i]), (t, i)
    assert qa.get_status() == 0 and qb.get_status() == 0
    qa.close(); qb.close()


def test_filtered_scale_pass_in_the_separate_calls():
    """qadam_worker_quantize with the option on (per-worker record of the bounds), mixed with whole-step
    calls on the same handle: same bits as a handle without the option."""
    gcfg, _ = configs(k_g=2, k_x=6)
    sizes = RAGGED + [1 << 19, 123457]
    seg_off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    P, N = int(seg_off[-1]), 3
    qa, qb = QAdam(gcfg, seg_off, N), QAdam(gcfg, seg_off, N)
    qa.trust_error_buffers(2)
    gen = torch.Generator().manual_seed(77)
    x0 = torch.randn(P, generator=gen) * 0.02
    a, b = DeviceState(qa, x0), DeviceState(qb, x0)
    for t in range(1, 7):
        for i in range(N):
            g = torch.randn(P, generator=gen) * (1e-2 if t != 4 else 1e-5)
            a.grads[i].copy_(g); b.grads[i].copy_(g)
        if t % 3 == 0:
            a.step_fused(t, 1e-3, 0.999)
        else:
            a.step_unfused(t, 1e-3, 0.999)
        b.step_fused(t, 1e-3, 0.999)
        torch.cuda.synchronize()
        for name in ("x", "m", "v", "werr", "wcodes"):
            assert torch.equal(getattr(a, name), getattr(b, name)), (t, name)
        for i in range(N):
            assert torch.equal(a.scales[i], b.scales[i]) and torch.equal(a.errs[i], b.errs[i]), (t, i)
            assert torch.equal(a.codes[i], b.codes[i]), (t, i)
    qa.close(); qb.close()


def test_filtered_scale_pass_keeps_nonfinite_detection():
    """A NaN or Inf gradient must still surface in the scale (and the status word) when the filter is on."""
    gcfg, _ = configs(k_g=2, k_x=6)
    seg_off = [0, 5000, 5000 + (1 << 19)]
    P, N = seg_off[-1], 2
    q = QAdam(gcfg, seg_off, N)
    q.trust_error_buffers(2)
    gen = torch.Generator().manual_seed(8)
    ds = DeviceState(q, torch.randn(P, generator=gen) * 0.02)
    for t in range(1, 4):
        for i in range(N):
            ds.grads[i].copy_(torch.randn(P, generator=gen) * 1e-2)
        if t == 3:
            ds.grads[1][5000 + 4096 * 70 + 17] = float("inf")        # in a tile that is not sampled
        ds.step_fused(t, 1e-3, 0.999)
        st = q.get_status()
        assert (st != 0) == (t == 3), (t, st)
    assert not torch.isfinite(ds.scales[1][1]) and torch.isfinite(ds.scales[0][1])
    q.close()


@pytest.mark.parametrize("k_g,trust", [(2, 0), (2, 2), (0, 2), (5, 2)])
def test_gradients_of_random_bit_patterns(k_g, trust):
    """Gradients whose sign, exponent and significand are drawn independently (magnitudes from
    2^-140, far inside the subnormals, to 2^15, over 150 binades in one layer), in many short ragged
    layers: the scale, the fast quotient with its fallback and the residual must follow the oracle
    bit for bit, with the full and with the filtered scale pass."""
    def bits(t, grads):
        rng = np.random.default_rng(1000 * k_g + t)
        out = []
        for g in grads:
            n = g.size
            expo = rng.integers(-140, 16, n)
            frac = 1.0 + rng.integers(0, 1 << 23, n) * 2.0 ** -23
            val = np.ldexp(frac, expo) * rng.choice([-1.0, 1.0], n)
            val[rng.random(n) < 0.02] = 0.0
            out.append(val.astype(np.float32))
        return out
    sizes = [int(v) for v in np.random.default_rng(5).integers(1, 3000, 40)] + [0, 50000]
    rep, st = _custom(sizes, 3, 4, cfgkw=dict(k_g=k_g), gsel=bits, seed=90 + k_g, trust=trust)
    _say("random bit patterns k_g=%d trust=%d: %s" % (k_g, trust, rep.line()))
    assert rep.ok() and st == 0 and rep.float_not_bit_exact == 0


def test_contract_of_the_filtered_pass_can_be_verified():
    """qadam_trust_error_buffers(h, 3): a loop that leaves the error buffers alone runs clean; one that
    changes them between steps gets QADAM_STATUS_ERR_BOUND_VIOLATED (and still correct scales: this
    mode reads everything)."""
    from paper_2004_14180_amd.binding import QADAM_STATUS_ERR_BOUND_VIOLATED
    gcfg, _ = configs(k_g=2, k_x=6)
    seg_off = [0, 3000, 3000 + 70000]
    P, N = seg_off[-1], 2
    qa, qb = QAdam(gcfg, seg_off, N), QAdam(gcfg, seg_off, N)
    qa.trust_error_buffers(3)
    gen = torch.Generator().manual_seed(13)
    x0 = torch.randn(P, generator=gen) * 0.02
    a, b = DeviceState(qa, x0), DeviceState(qb, x0)
    for t in range(1, 6):
        for i in range(N):
            g = torch.randn(P, generator=gen) * 1e-2
            a.grads[i].copy_(g); b.grads[i].copy_(g)
        if t == 4:                       # the caller meddles with one error buffer
            a.errs[1].mul_(8.0); b.errs[1].mul_(8.0)
        a.step_fused(t, 1e-3, 0.999)
        b.step_fused(t, 1e-3, 0.999)
        st = qa.get_status(clear=True)
        assert st == (QADAM_STATUS_ERR_BOUND_VIOLATED if t == 4 else 0), (t, st)
        for i in range(N):
            assert torch.equal(a.scales[i], b.scales[i]) and torch.equal(a.errs[i], b.errs[i])
        assert torch.equal(a.x, b.x)
    qa.close(); qb.close()
