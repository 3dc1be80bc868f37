"""Pins of the oracle's optimizer steps (moments, error feedback across steps, the
two placements of the moments) against closed forms, identities of the paper's
analysis, a library Adam and fp64 re-derivations that do not share its code."""
import numpy as np
import pytest

from oracle.qadam_oracle import OracleConfig


def _zeros(n, k=1):
    return [np.zeros(n, np.float32) for _ in range(k)]


# ------------------------------------------------------------------ closed form
def test_constant_gradient_closed_form(oracle):
    """Moment and update steps of Algorithm 1 with Q_g = Q_x = id and a constant gradient g:
    m_t = (1 - beta^t) g, v_t = (1 - theta^t) g^2 (unrolling the recursions from m_0 = v_0 = 0),
    x_{t+1} = x_t - alpha (1-beta^t) g / sqrt((1-theta^t) g^2 + eps): eps inside the root, no bias
    correction.  beta != theta and a large eps make swapped or misplaced constants visible."""
    n, T = 257, 25
    beta, theta, eps, lr = 0.8, 0.95, 1e-4, 3e-3
    rng = np.random.default_rng(0)
    g = (rng.standard_normal(n) * 1e-2).astype(np.float32)
    x0 = rng.standard_normal(n).astype(np.float32)
    cfg = OracleConfig(identity_g=1, identity_x=1, beta1=beta, eps=eps, weight_ef=0)
    x = x0.copy()
    m, v, e, w = _zeros(n, 4)
    b32, t32, e32, l32 = (np.float64(np.float32(c)) for c in (beta, theta, eps, lr))
    g64 = g.astype(np.float64)
    x_ref = x0.astype(np.float64)
    for t in range(1, T + 1):
        oracle.step_s(cfg, [0, n], t, lr, theta, [g], [e], x, m, v, w)
        m_ref = (1 - b32 ** t) * g64
        v_ref = (1 - t32 ** t) * g64 ** 2
        x_ref = x_ref - l32 * m_ref / np.sqrt(v_ref + e32)
        assert np.allclose(m, m_ref, rtol=2e-6, atol=1e-12)
        assert np.allclose(v, v_ref, rtol=2e-6, atol=1e-14)
        assert np.allclose(x, x_ref, rtol=2e-6, atol=1e-7)
    assert not e.any()


def test_identity_quantizers_reduce_to_generic_adam(oracle):
    """Sec. 3.1.1 / 3.1.2 / after Theorem 3: with Q_g and Q_x the identity the method is
    (distributed) generic Adam.  Variant S must equal an fp64 generic Adam on the mean gradient;
    with one worker variants S and W and Algorithm 1 coincide bit for bit."""
    n, T, N = 1000, 30, 4
    beta, theta, eps, lr = 0.9, 0.999, 1e-5, 1e-3
    rng = np.random.default_rng(1)
    segs = [0, 100, 100, 613, n]
    cfg = OracleConfig(identity_g=1, identity_x=1, beta1=beta, eps=eps)
    x0 = (rng.standard_normal(n) * 0.02).astype(np.float32)
    x = x0.copy()
    m, v, w = _zeros(n, 3)
    errs = _zeros(n, N)
    xr = x0.astype(np.float64)
    mr = np.zeros(n)
    vr = np.zeros(n)
    b, th, ep, l = (np.float64(np.float32(c)) for c in (beta, theta, eps, lr))
    x1 = x0.copy(); m1, v1, w1 = _zeros(n, 3); e1 = _zeros(n, 1)
    x2 = x0.copy(); w2 = _zeros(n, 1)[0]; e2 = _zeros(n, 1); mw = _zeros(n, 1); vw = _zeros(n, 1)
    for t in range(1, T + 1):
        grads = [(rng.standard_normal(n) * 1e-2).astype(np.float32) for _ in range(N)]
        oracle.step_s(cfg, segs, t, lr, theta, grads, errs, x, m, v, w)
        gbar = np.mean(np.stack(grads).astype(np.float64), axis=0)
        vr = th * vr + (1 - th) * gbar ** 2
        mr = b * mr + (1 - b) * gbar
        xr = xr - l * mr / np.sqrt(vr + ep)
        assert np.allclose(x, xr, rtol=1e-6, atol=1e-7)
        assert np.allclose(m, mr, rtol=1e-5, atol=1e-9)
        assert np.allclose(v, vr, rtol=1e-5, atol=1e-12)
        # N = 1: S == W == Algorithm 1
        oracle.step_s(cfg, segs, t, lr, theta, grads[:1], e1, x1, m1, v1, w1)
        oracle.step_w(cfg, segs, t, lr, theta, grads[:1], e2, mw, vw, x2, w2)
        assert np.array_equal(x1, x2) and np.array_equal(m1, mw[0]) and np.array_equal(v1, vw[0])


def test_bias_corrected_flavour_matches_library_adam(oracle):
    """The textbook special case (bias correction, eps outside the root) against torch.optim.Adam
    on CPU in fp32; independent of the paper's flavour, it pins the moment recursions and the
    worker averaging."""
    torch = pytest.importorskip("torch")
    n, T, N = 512, 20, 2
    beta, theta, eps, lr = 0.9, 0.99, 1e-3, 1e-2
    rng = np.random.default_rng(2)
    x0 = rng.standard_normal(n).astype(np.float32)
    cfg = OracleConfig(identity_g=1, identity_x=1, beta1=beta, eps=eps, adam_flavor=1)
    x = x0.copy()
    m, v, w = _zeros(n, 3)
    errs = _zeros(n, N)
    xt = torch.tensor(x0.copy(), requires_grad=True)
    opt = torch.optim.Adam([xt], lr=lr, betas=(beta, theta), eps=eps)
    for t in range(1, T + 1):
        grads = [(rng.standard_normal(n) * 1e-2).astype(np.float32) for _ in range(N)]
        oracle.step_s(cfg, [0, n], t, lr, theta, grads, errs, x, m, v, w)
        xt.grad = torch.tensor((grads[0] + grads[1]) / np.float32(2))
        opt.step()
        assert np.allclose(x, xt.detach().numpy(), rtol=1e-5, atol=1e-6)


def test_theta_schedule_argument(oracle):
    """Assumption 4: theta_t = 1 - theta/t and alpha_t = alpha/sqrt(t) are per-step arguments."""
    n, T = 64, 12
    rng = np.random.default_rng(3)
    cfg = OracleConfig(identity_g=1, identity_x=1, beta1=0.9, eps=1e-6)
    x = np.zeros(n, np.float32)
    m, v, w = _zeros(n, 3)
    e = _zeros(n, 1)
    xr = np.zeros(n); mr = np.zeros(n); vr = np.zeros(n)
    for t in range(1, T + 1):
        g = rng.standard_normal(n).astype(np.float32)
        th = np.float32(1 - 0.5 / t)
        lr = np.float32(1e-2 / np.sqrt(t))
        oracle.step_s(cfg, [0, n], t, float(lr), float(th), [g], e, x, m, v, w)
        vr = np.float64(th) * vr + (1 - np.float64(th)) * g.astype(np.float64) ** 2
        mr = np.float64(np.float32(0.9)) * mr + (1 - np.float64(np.float32(0.9))) * g
        xr = xr - np.float64(lr) * mr / np.sqrt(vr + np.float64(np.float32(1e-6)))
        assert np.allclose(x, xr, rtol=2e-6, atol=1e-7)


# ------------------------------------------------------------ error feedback
@pytest.mark.parametrize("k_g", [0, 2])
def test_error_feedback_telescoping_variant_s(oracle, k_g):
    """Notation 1 (x~_t = x_t - e_t telescopes): what a worker has sent plus what it still holds
    equals what it was given, sum_t q_t = sum_t g_t - e_{T+1}; and the residual stays bounded
    (lemma on ||e_t||)."""
    n, T, N = 3000, 40, 3
    rng = np.random.default_rng(10 + k_g)
    segs = [0, 1000, 1024, n]
    cfg = OracleConfig(k_g=k_g, k_x=6)
    errs = _zeros(n, N)
    sum_q = [np.zeros(n) for _ in range(N)]
    sum_g = [np.zeros(n) for _ in range(N)]
    for t in range(1, T + 1):
        for i in range(N):
            g = (rng.standard_normal(n) * 1e-2).astype(np.float32)
            out = oracle.worker_quantize(cfg, segs, i, t, g, errs[i], want_q=True)
            sum_q[i] += out["q"]
            sum_g[i] += g
            # decoded packed codes are the same numbers
            codes = oracle.unpack_all(k_g, segs, out["words"])
            assert np.array_equal(codes, out["codes"])
    for i in range(N):
        assert np.allclose(sum_q[i], sum_g[i] - errs[i], rtol=0, atol=1e-6)
        assert np.max(np.abs(errs[i])) < 0.2      # a few gradient magnitudes, not growing with T


@pytest.mark.parametrize("k_g", [0, 2])
def test_error_buffer_obeys_the_geometric_bound(oracle, k_g):
    """Lemma on the error term (proof of Theorem 1): with contraction factor c = 1 - delta_g of the
    quantizer (Assumption 2), ||e_{t+1}|| <= sum_{i<=t} c^(t-i+1) ||Delta_i||.  Here Delta_i is what
    the worker feeds in at step i (its gradient in variant S) and c is the largest per-step ratio
    ||p - Q_g(p)|| / ||p|| actually observed (< 1); norms per layer in fp64.  An error buffer that
    accumulated instead of being replaced, or a residual of the wrong sign, breaks the bound."""
    n, T = 4096, 60
    rng = np.random.default_rng(40 + k_g)
    cfg = OracleConfig(k_g=k_g, k_x=6)
    err = np.zeros(n, np.float32)
    d_norm, e_norm, ratios = [], [], []
    for t in range(1, T + 1):
        g = (rng.standard_normal(n) * (1e-2 * (1 + (t % 7)))).astype(np.float32)   # uneven step sizes
        p = (g + err).astype(np.float64)
        oracle.worker_quantize(cfg, [0, n], 0, t, g, err)
        d_norm.append(np.linalg.norm(g.astype(np.float64)))
        e_norm.append(np.linalg.norm(err.astype(np.float64)))
        ratios.append(e_norm[-1] / np.linalg.norm(p))
    c = max(ratios)
    assert c < 1.0                                   # Assumption 2 held at every step
    for t in range(T):
        bound = sum(c ** (t - i + 1) * d_norm[i] for i in range(t + 1))
        assert e_norm[t] <= bound * (1 + 1e-9), t
    # the bound's limit: the buffer never exceeds c/(1-c) times the largest input
    assert max(e_norm) <= c / (1 - c) * max(d_norm)


def test_variant_w_telescoping(oracle):
    """Notation 3: x~_t = x_t - mean_i e_t^(i) follows the un-quantized recursion
    x~_{t+1} = x~_t + mean_i Delta_t^(i), Delta = -alpha m / sqrt(v + eps) with the workers' own
    moments (moment steps of Algorithm 3).  The gradients are given, so the right-hand side is an fp64
    per-worker generic Adam that never sees a quantizer."""
    n, T, N = 2048, 30, 4
    beta, theta, eps, lr = 0.9, 0.999, 1e-5, 1e-3
    rng = np.random.default_rng(20)
    cfg = OracleConfig(k_g=2, k_x=6, beta1=beta, eps=eps, weight_ef=1)
    x0 = (rng.standard_normal(n) * 0.02).astype(np.float32)
    x = x0.copy()
    errs, mw, vw = _zeros(n, N), _zeros(n, N), _zeros(n, N)
    werr = np.zeros(n, np.float32)
    b, th, ep, l = (np.float64(np.float32(c)) for c in (beta, theta, eps, lr))
    mr = [np.zeros(n) for _ in range(N)]
    vr = [np.zeros(n) for _ in range(N)]
    xt = x0.astype(np.float64)
    for t in range(1, T + 1):
        grads = [(rng.standard_normal(n) * 1e-2).astype(np.float32) for _ in range(N)]
        out = oracle.step_w(cfg, [0, 2000, n], t, lr, theta, grads, errs, mw, vw, x, werr)
        assert out["status"] == 0
        upd = np.zeros(n)
        for i in range(N):
            g = grads[i].astype(np.float64)
            vr[i] = th * vr[i] + (1 - th) * g * g
            mr[i] = b * mr[i] + (1 - b) * g
            upd += l * mr[i] / np.sqrt(vr[i] + ep)
            assert np.allclose(mw[i], mr[i], rtol=1e-5, atol=1e-9)
        xt = xt - upd / N
        x_tilde = x.astype(np.float64) - np.mean(np.stack(errs).astype(np.float64), axis=0)
        assert np.allclose(x_tilde, xt, rtol=0, atol=2e-6)
    # the quantizer really was active: iterate differs from the un-quantized one
    assert np.max(np.abs(x.astype(np.float64) - xt)) > 1e-5


def test_variant_s_server_mean_and_order(oracle):
    """Gather step of Algorithm 2 (mean of the N worker messages) applied to dequantized gradients: the
    server's m after one step from zero is (1-beta) * mean_i q_i, with the q_i decoded
    independently here from the packed words and scales."""
    n, N = 1500, 8
    rng = np.random.default_rng(30)
    segs = [0, 700, n]
    cfg = OracleConfig(k_g=2, k_x=6, beta1=0.75, eps=1e-8)
    grads = [(rng.standard_normal(n) * 10.0 ** rng.uniform(-3, 0)).astype(np.float32) for _ in range(N)]
    errs = _zeros(n, N)
    x = np.zeros(n, np.float32)
    m, v, w = _zeros(n, 3)
    out = oracle.step_s(cfg, segs, 1, 1e-3, 0.5, grads, errs, x, m, v, w)
    w_mu = oracle.grad_code_bits(2) - 1
    tot = np.zeros(n)
    for i in range(N):
        codes = oracle.unpack_all(2, segs, out["words"][i]).astype(np.int64)
        mu = codes & ((1 << w_mu) - 1)
        sign = np.where(codes >> w_mu == 1, -1.0, 1.0)
        scale = np.concatenate([np.full(700, out["scales"][i][0], np.float64),
                                np.full(n - 700, out["scales"][i][1], np.float64)])
        q = np.where(mu == 0, 0.0, sign * scale * 2.0 ** (mu - 1.0 - 2))
        assert np.array_equal((grads[i].astype(np.float64) - q).astype(np.float32), errs[i])
        tot += q
    gbar = tot / N
    # fp32 accumulation over 8 terms of mixed magnitude: absolute slack tied to the largest term
    big = max(float(np.max(sc)) for sc in out["scales"])
    assert np.allclose(m, 0.25 * gbar, rtol=1e-6, atol=1e-7 * big)
    assert np.allclose(v, 0.5 * gbar ** 2, rtol=1e-5, atol=1e-7 * big ** 2)
    assert np.allclose(x, -1e-3 * 0.25 * gbar / np.sqrt(0.5 * gbar ** 2 + 1e-8), rtol=1e-4, atol=1e-8)


def test_fused_step_equals_three_calls(oracle):
    """The whole step is exactly worker_quantize (per worker) + server_step + weight_quantize."""
    n, N, T = 5000, 4, 6
    rng = np.random.default_rng(40)
    segs = [0, 64, 3000, 3001, n]
    for k_g, k_x, wef, rnd in [(2, 6, 1, 0), (0, 14, 0, 0), (2, 6, 1, 1)]:
        cfg = OracleConfig(k_g=k_g, k_x=k_x, weight_ef=wef, rounding=rnd, seed=99)
        x0 = (rng.standard_normal(n) * 0.02).astype(np.float32)
        xa, xb = x0.copy(), x0.copy()
        ma, va, wa = _zeros(n, 3)
        mb, vb, wb = _zeros(n, 3)
        ea, eb = _zeros(n, N), _zeros(n, N)
        for t in range(1, T + 1):
            grads = [(rng.standard_normal(n) * 1e-2).astype(np.float32) for _ in range(N)]
            oa = oracle.step_s(cfg, segs, t, 1e-3, 0.999, grads, ea, xa, ma, va, wa)
            outs = [oracle.worker_quantize(cfg, segs, i, t, grads[i], eb[i]) for i in range(N)]
            oracle.server_step(cfg, segs, t, 1e-3, 0.999, [o["words"] for o in outs],
                               [o["scales"] for o in outs], xb, mb, vb)
            ob = oracle.weight_quantize(cfg, t, xb, wb)
            for i in range(N):
                assert np.array_equal(oa["words"][i], outs[i]["words"])
                assert np.array_equal(oa["scales"][i], outs[i]["scales"])
                assert np.array_equal(ea[i], eb[i])
            for a, b in [(xa, xb), (ma, mb), (va, vb), (wa, wb), (oa["wcodes"], ob["wcodes"])]:
                assert np.array_equal(a, b)


def test_layers_are_independent(oracle):
    """The scale is per layer segment and everything else is element-wise, so running a layer
    alone (with its global index base) gives the same bits as running it inside the vector --
    the property that lets large configurations be checked layer by layer."""
    n, N = 4000, 2
    rng = np.random.default_rng(50)
    segs = [0, 1000, 2500, n]
    for rnd in (0, 1):
        cfg = OracleConfig(k_g=2, k_x=6, rounding=rnd, seed=5)
        grads = [(rng.standard_normal(n) * 1e-2).astype(np.float32) for _ in range(N)]
        x0 = (rng.standard_normal(n) * 0.02).astype(np.float32)
        x = x0.copy(); m, v, w = _zeros(n, 3); errs = _zeros(n, N)
        full = oracle.step_s(cfg, segs, 3, 1e-3, 0.999, grads, errs, x, m, v, w)
        a, b = segs[1], segs[2]
        xs = x0[a:b].copy(); ms, vs, ws = _zeros(b - a, 3); es = _zeros(b - a, N)
        part = oracle.step_s(cfg, [0, b - a], 3, 1e-3, 0.999, [g[a:b].copy() for g in grads], es,
                             xs, ms, vs, ws, index_base=a)
        assert np.array_equal(xs, x[a:b]) and np.array_equal(ws, w[a:b])
        assert np.array_equal(part["wcodes"], full["wcodes"][a:b])
        for i in range(N):
            assert np.array_equal(es[i], errs[i][a:b])
            assert part["scales"][i][0] == full["scales"][i][1]


def test_zero_padding_of_layers_changes_nothing(oracle):
    """A layer padded with zeros in every buffer gives the same results on its real elements, and the
    padding stays zero: p = 0 quantizes to 0 for any scale and leaves no residual, a zero mean gradient
    keeps m = v = 0 and moves x by alpha * 0 / sqrt(eps) = 0, and Q_x(0) = 0 (Sec. 5.1, Alg. 1).  This is
    what lets a caller round layer lengths up to the access width of a device."""
    sizes, N, steps = [1001, 7, 2500], 3, 4
    pad = [(-n) % 4 for n in sizes]
    segs = np.concatenate([[0], np.cumsum(sizes)])
    psegs = np.concatenate([[0], np.cumsum([n + q for n, q in zip(sizes, pad)])])
    P, PP = int(segs[-1]), int(psegs[-1])
    real = np.concatenate([np.arange(psegs[l], psegs[l] + sizes[l]) for l in range(len(sizes))])
    fill = np.setdiff1d(np.arange(PP), real)
    rng = np.random.default_rng(77)
    for flavor in (0, 1):
        cfg = OracleConfig(k_g=2, k_x=6, weight_ef=1, adam_flavor=flavor)
        x = (rng.standard_normal(P) * 0.02).astype(np.float32)
        m, v, w = _zeros(P, 3); errs = _zeros(P, N)
        xp = np.zeros(PP, np.float32); xp[real] = x
        mp, vp, wp = _zeros(PP, 3); errp = _zeros(PP, N)
        for t in range(1, steps + 1):
            grads = [(rng.standard_normal(P) * 1e-2).astype(np.float32) for _ in range(N)]
            gp = []
            for g in grads:
                z = np.zeros(PP, np.float32); z[real] = g; gp.append(z)
            a = oracle.step_s(cfg, segs, t, 1e-3, 0.999, grads, errs, x, m, v, w)
            b = oracle.step_s(cfg, psegs, t, 1e-3, 0.999, gp, errp, xp, mp, vp, wp)
            for u, up in [(x, xp), (m, mp), (v, vp), (w, wp), (a["wcodes"], b["wcodes"])]:
                assert np.array_equal(u, up[real]) and not up[fill].any()
            for i in range(N):
                assert np.array_equal(errs[i], errp[i][real]) and not errp[i][fill].any()
                assert np.array_equal(a["scales"][i], b["scales"][i])
                ca = oracle.unpack_all(cfg.k_g, segs, a["words"][i])
                cb = oracle.unpack_all(cfg.k_g, psegs, b["words"][i])
                assert np.array_equal(ca, cb[real]) and not cb[fill].any()


def test_window_equals_layer(oracle):
    """Given the layer's scale, a window of the layer quantizes to the same codes."""
    n = 10000
    rng = np.random.default_rng(60)
    g = (rng.standard_normal(n) * 1e-2).astype(np.float32)
    e = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    for rnd in (0, 1):
        cfg = OracleConfig(k_g=2, rounding=rnd, seed=11)
        err = e.copy()
        full = oracle.worker_quantize(cfg, [0, n], 1, 4, g, err, index_base=128)
        s = full["scales"][0]
        assert s == np.max(np.abs(g + e))
        a, b = 3000, 4111
        ew = e[a:b].copy()
        code, tie, q = oracle.worker_quantize_window(cfg, g[a:b].copy(), ew, s, j0=128 + a, step=4, worker=1)
        assert np.array_equal(code, full["codes"][a:b]) and np.array_equal(ew, err[a:b])


def test_step_window_equals_step(oracle):
    """With the layer scales given (here: numpy's max of |g+e| in fp32, the definition of the
    infinity norm), any window of a layer steps to the same bits as inside the whole vector."""
    n, N = 6000, 3
    rng = np.random.default_rng(70)
    segs = [0, 1500, n]
    for rnd in (0, 1):
        cfg = OracleConfig(k_g=2, k_x=6, rounding=rnd, seed=3)
        grads = [(rng.standard_normal(n) * 1e-2).astype(np.float32) for _ in range(N)]
        e0 = [(rng.standard_normal(n) * 1e-3).astype(np.float32) for _ in range(N)]
        x0 = (rng.standard_normal(n) * 0.02).astype(np.float32)
        m0 = (rng.standard_normal(n) * 1e-3).astype(np.float32)
        v0 = (rng.standard_normal(n) ** 2 * 1e-5).astype(np.float32)
        w0 = (rng.uniform(-1, 1, n) * 2.0 ** -9).astype(np.float32)
        x, m, v, w = x0.copy(), m0.copy(), v0.copy(), w0.copy()
        errs = [e.copy() for e in e0]
        full = oracle.step_s(cfg, segs, 2, 1e-3, 0.999, grads, errs, x, m, v, w)
        a, b = 2000, 5003                       # a window inside layer 1
        scales = [np.max(np.abs(grads[i][1500:] + e0[i][1500:])) for i in range(N)]
        assert [float(full["scales"][i][1]) for i in range(N)] == [float(s) for s in scales]
        xw, mw, vw, ww = x0[a:b].copy(), m0[a:b].copy(), v0[a:b].copy(), w0[a:b].copy()
        ew = [e[a:b].copy() for e in e0]
        win = oracle.step_s_window(cfg, a, 2, 1e-3, 0.999, scales, [g[a:b].copy() for g in grads], ew,
                                   xw, mw, vw, ww)
        for got, want in [(xw, x[a:b]), (mw, m[a:b]), (vw, v[a:b]), (ww, w[a:b]),
                          (win["wcodes"], full["wcodes"][a:b]), (win["tie_x"], full["tie_x"][a:b])]:
            assert np.array_equal(got, want)
        for i in range(N):
            assert np.array_equal(ew[i], errs[i][a:b])
            codes = oracle.unpack_all(2, segs, full["words"][i])
            assert np.array_equal(win["codes"][i], codes[a:b])


@pytest.mark.parametrize("variant", ["s", "w"])
def test_closed_loop_quadratic_reaches_a_neighbourhood(oracle, variant):
    """Theorems 2-3 (qualitatively): with gradients sampled at the quantized weights Q_x(x_t), the
    iterates reach a neighbourhood of the stationary point whose size is set by the weight grid, and
    error feedback keeps coarse (ternary) gradient quantization from stalling the descent.
    f(x) = 1/2 ||x - x*||^2, worker gradients = (Q_x(x) - x*) + noise."""
    n, N, T = 256, 4, 1500
    rng = np.random.default_rng(7)
    xstar = rng.uniform(-0.4, 0.4, n).astype(np.float32)
    cfg = OracleConfig(k_g=0, k_x=6, weight_ef=0, beta1=0.9, eps=1e-8)
    x = np.zeros(n, np.float32)
    werr = np.zeros(n, np.float32)
    errs = _zeros(n, N)
    m, v = _zeros(n, 2)
    mw, vw = _zeros(n, N), _zeros(n, N)
    xhat = np.zeros(n, np.float32)
    d0 = np.linalg.norm(xhat - xstar)
    for t in range(1, T + 1):
        lr = 2e-2 / np.sqrt(t)
        grads = [((xhat - xstar) + rng.standard_normal(n) * 0.01).astype(np.float32) for _ in range(N)]
        if variant == "s":
            out = oracle.step_s(cfg, [0, n], t, float(lr), 0.999, grads, errs, x, m, v, werr)
        else:
            out = oracle.step_w(cfg, [0, n], t, float(lr), 0.999, grads, errs, mw, vw, x, werr)
        xhat = out["wcodes"].astype(np.float32) * np.float32(2.0 ** -7)
        assert np.array_equal(xhat, (x - werr).astype(np.float32))        # emitted weights = Q_x(x)
    dist = np.abs(xhat - xstar)
    assert np.linalg.norm(xhat - xstar) < 0.05 * d0
    assert dist.max() < 4 * 2.0 ** -7                                    # a few weight-grid steps


def _real_qg(p, k_g):
    """Q_g of Sec. 5.1 from its definition, in fp64: ||p||_inf times the nearest point of
    G = {0, +-2^-k_g, ..., +-1} to p / ||p||_inf.  Returns (q, distance of |p|/s to the nearest midpoint)."""
    s = np.max(np.abs(p))
    if s == 0:
        return np.zeros_like(p), np.ones_like(p)
    grid = np.array([0.0] + [2.0 ** (c - 1 - k_g) for c in range(1, k_g + 2)])
    a = np.abs(p) / s
    idx = np.argmin(np.abs(a[:, None] - grid[None, :]), axis=1)
    mids = 0.5 * (grid[:-1] + grid[1:])
    margin = np.min(np.abs(a[:, None] - mids[None, :]), axis=1)
    return np.sign(p) * s * grid[idx], margin


@pytest.mark.parametrize("variant", ["s", "w"])
def test_whole_step_against_the_definitions_in_fp64(oracle, variant):
    """One step of each variant re-evaluated from the paper's formulas over the reals (numpy fp64,
    arg-min by enumeration of the grids, no shared code): the oracle's binary32 result agrees to
    rounding, and its integer codes agree wherever the value is not within 1e-5 of a midpoint."""
    n, N, k_g, k_x = 6000, 3, 2, 6
    segs = [0, 2500, 2600, n]
    rng = np.random.default_rng(77)
    cfg = OracleConfig(k_g=k_g, k_x=k_x, weight_ef=1, beta1=0.9, eps=1e-8)
    beta, theta, eps, lr = (np.float64(np.float32(c)) for c in (0.9, 0.999, 1e-8, 1e-3))
    grads = [(rng.standard_normal(n) * 1e-2).astype(np.float32) for _ in range(N)]
    errs = [(rng.standard_normal(n) * 2e-3).astype(np.float32) for _ in range(N)]
    x = (rng.standard_normal(n) * 0.02).astype(np.float32)
    werr = ((rng.random(n) - 0.5) * 2.0 ** -(k_x + 1)).astype(np.float32)
    m = (rng.standard_normal(n) * 3e-3).astype(np.float32)
    v = ((rng.standard_normal(n) * 1e-2) ** 2).astype(np.float32)
    mw = [(rng.standard_normal(n) * 3e-3).astype(np.float32) for _ in range(N)]
    vw = [((rng.standard_normal(n) * 1e-2) ** 2).astype(np.float32) for _ in range(N)]
    # ---- the definitions, fp64
    acc = np.zeros(n)
    pmax = 0.0
    e_want, safe = [], np.ones(n, bool)
    m_want = v_want = None
    mw_want, vw_want = [], []
    for i in range(N):
        if variant == "s":
            value = grads[i].astype(np.float64)
        else:                                   # Algorithm 3: local moments, then the Adam update
            g = grads[i].astype(np.float64)
            vv = theta * vw[i] + (1 - theta) * g * g
            mm = beta * mw[i] + (1 - beta) * g
            mw_want.append(mm); vw_want.append(vv)
            value = lr * mm / np.sqrt(vv + eps)
        p = value + errs[i]
        q = np.zeros(n)
        for l in range(len(segs) - 1):
            a, b = segs[l], segs[l + 1]
            q[a:b], margin = _real_qg(p[a:b], k_g)
            safe[a:b] &= margin > 1e-5
        e_want.append(p - q)
        pmax = max(pmax, float(np.max(np.abs(p))))
        acc += q
    mean = acc / N
    if variant == "s":
        v_want = theta * v + (1 - theta) * mean * mean
        m_want = beta * m + (1 - beta) * mean
        x_want = x - lr * m_want / np.sqrt(v_want + eps)
    else:
        x_want = x - mean
    y = x_want + werr
    u = y * 2.0 ** (k_x + 1)
    safe_x = np.abs(np.abs(u - np.floor(u)) - 0.5) > 1e-3
    j_want = np.clip(np.sign(u) * np.floor(np.abs(u) + 0.5), -2.0 ** k_x, 2.0 ** k_x)
    werr_want = y - j_want * 2.0 ** -(k_x + 1)
    # ---- the oracle, binary32
    if variant == "s":
        out = oracle.step_s(cfg, segs, 5, float(lr), float(theta), grads, errs, x, m, v, werr)
    else:
        out = oracle.step_w(cfg, segs, 5, float(lr), float(theta), grads, errs, mw, vw, x, werr)
    assert safe.mean() > 0.99 and safe_x.mean() > 0.99
    # binary32 rounds the scale s = ||p||_inf, and with it every q = s * level, by up to half an ulp of s
    tol = dict(rtol=3e-6, atol=2.0 ** -22 * pmax)
    for i in range(N):
        assert np.allclose(errs[i][safe], e_want[i][safe], **tol), i
        if variant == "w":
            assert np.allclose(mw[i], mw_want[i], **tol) and np.allclose(vw[i], vw_want[i], rtol=3e-6, atol=1e-12)
    if variant == "s":
        assert np.allclose(m[safe], m_want[safe], **tol) and np.allclose(v[safe], v_want[safe], rtol=3e-6, atol=1e-12)
    assert np.allclose(x[safe], x_want[safe], rtol=3e-6, atol=max(1e-8, 2.0 ** -22 * pmax))
    ok = safe & safe_x
    assert np.array_equal(out["wcodes"][ok].astype(np.float64), j_want[ok])
    assert np.allclose(werr[ok], werr_want[ok], rtol=0, atol=1e-7)
