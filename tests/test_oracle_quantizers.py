"""Pins of the oracle's quantizers against what the paper and the mathematics fix.

Each test names the passage of arXiv 2004.14180 it takes its expectation from.
None of them recomputes the oracle's own formula: expectations come from
hand-worked values (tests/golden), brute-force arg-min over the grid in fp64,
the inequalities of Assumptions 2-3, exactness of the residual, and the sizes
printed in Tables 1-2.
"""
import os

import numpy as np
import pytest

from oracle.qadam_oracle import OracleConfig

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    out = []
    for line in open(os.path.join(GOLD, name)):
        line = line.strip()
        if line and not line.startswith("#"):
            out.append(line.split())
    return out


# ---------------------------------------------------------------- hand-worked
def test_qg_handworked(oracle):
    """Sec. 5.1 grid G, values worked by hand for layers with infinity norm 1."""
    for k_g, val, want in _rows("qg_handworked.txt"):
        k_g, val, want = int(k_g), float(val), float(want)
        p = np.array([val, 1.0], np.float32)          # the 1.0 fixes the scale to 1
        st, s, code, q, tie = oracle.qg_layer(OracleConfig(k_g=k_g), p)
        assert st == 0 and s == 1.0
        assert q[0] == np.float32(want), (k_g, val, q[0], want)
        assert q[1] == 1.0


def test_qg_scale_invariance(oracle):
    """Q_g(c*p) = c*Q_g(p) for a power-of-two c (the scale is the infinity norm, Sec. 5.1)."""
    rng = np.random.default_rng(1)
    p = rng.standard_normal(1000).astype(np.float32)
    for k_g in (0, 1, 2, 4):
        _, s1, c1, q1, _ = oracle.qg_layer(OracleConfig(k_g=k_g), p)
        _, s2, c2, q2, _ = oracle.qg_layer(OracleConfig(k_g=k_g), p * np.float32(2.0 ** -7))
        assert s2 == s1 * np.float32(2.0 ** -7)
        assert np.array_equal(c1, c2)
        assert np.array_equal(q2, q1 * np.float32(2.0 ** -7))


def test_qx_handworked(oracle):
    """Sec. 5.1 grid X, values worked by hand."""
    for k_x, x, want, j in _rows("qx_handworked.txt"):
        k_x, x, want, j = int(k_x), float(x), float(want), int(j)
        jj, xh, _ = oracle.qx(OracleConfig(k_x=k_x), np.array([x], np.float32))
        assert xh[0] == np.float32(want), (k_x, x, xh[0], want)
        assert jj[0] == j


# ---------------------------------------------------------------- brute force
def _grid_G(k_g):
    pos = [2.0 ** (-k) for k in range(k_g, -1, -1)]
    return np.array(sorted([-v for v in pos] + [0.0] + pos), dtype=np.float64)


@pytest.mark.parametrize("k_g", [0, 1, 2, 3, 6])
def test_qg_bruteforce_argmin(oracle, k_g):
    """Sec. 5.1: Q_g(p) = ||p||_inf * argmin over G^d of ||p/||p||_inf - g^||, which is
    element-wise; enumerate G in fp64 on tiny layers (<= 64 elements)."""
    rng = np.random.default_rng(100 + k_g)
    G = _grid_G(k_g)
    for trial in range(200):
        n = int(rng.integers(1, 65))
        scale = 10.0 ** rng.uniform(-6, 3)
        kind = trial % 3
        if kind == 0:
            p = rng.standard_normal(n)
        elif kind == 1:
            p = rng.standard_t(3, n)
        else:   # spread over many octaves so that all levels occur
            p = rng.choice([-1, 1], n) * 2.0 ** rng.uniform(-k_g - 3, 0, n)
        p = (p * scale).astype(np.float32)
        st, s, code, q, tie = oracle.qg_layer(OracleConfig(k_g=k_g), p)
        assert st == 0
        s_want = np.max(np.abs(p))
        assert s == s_want
        if s_want == 0:
            continue
        r = (p / np.float32(s_want)).astype(np.float32).astype(np.float64)   # fp32 ratio, as fixed
        d = np.abs(r[:, None] - G[None, :])
        best = G[np.argmin(d, axis=1)]
        want = (np.float64(s_want) * best).astype(np.float32)
        free = tie == 0
        assert np.array_equal(q[free], want[free])
        # on flagged elements the oracle must still pick one of the two nearest points
        dsort = np.sort(d, axis=1)
        got_d = np.abs(r - q.astype(np.float64) / np.float64(s_want))
        assert np.all(got_d <= dsort[:, 1] + 1e-12)


@pytest.mark.parametrize("k_x", [0, 1, 3, 6, 10, 14])
def test_qx_bruteforce_argmin(oracle, k_x):
    """Sec. 5.1: Q_x(x) = 0.5 * argmin over X of |2x - xh|; enumerate X in fp64."""
    rng = np.random.default_rng(200 + k_x)
    X = np.arange(-2 ** k_x, 2 ** k_x + 1, dtype=np.float64) / 2.0 ** k_x
    x = np.concatenate([rng.uniform(-0.7, 0.7, 600), rng.normal(0, 0.02, 600),
                        [0.0, 0.5, -0.5, 1.5, -3.0]]).astype(np.float32)
    j, xh, tie = oracle.qx(OracleConfig(k_x=k_x), x)
    d = np.abs(2.0 * x.astype(np.float64)[:, None] - X[None, :])
    want = 0.5 * X[np.argmin(d, axis=1)]
    free = tie == 0
    assert np.array_equal(xh[free].astype(np.float64), want[free])
    assert np.array_equal(j.astype(np.float64) * 2.0 ** -(k_x + 1), xh.astype(np.float64))
    assert np.all(np.abs(j) <= 2 ** k_x)


# ------------------------------------------------- exact residual, ranges, signs
@pytest.mark.parametrize("k_g", [0, 1, 2, 5])
def test_qg_exact_residual_and_ranges(oracle, k_g):
    """Error feedback (residual step of Algorithm 1): e' = p - Q_g(p).  With nearest rounding on a
    power-of-two grid p/q lies in [1/2, 2] for every non-zero code, so the fp32 subtraction is
    exact and q + e' == p bit for bit.  Codes stay in range; the arg-max element is reproduced."""
    rng = np.random.default_rng(300 + k_g)
    n = 50_000
    g = (rng.standard_normal(n) * 10.0 ** rng.uniform(-8, 2, n)).astype(np.float32)
    e = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    p = (g + e).astype(np.float32)
    cfg = OracleConfig(k_g=k_g)
    err = e.copy()
    out = oracle.worker_quantize(cfg, [0, n], 0, 1, g, err, want_q=True)
    q = out["q"]
    assert np.array_equal((q + err).astype(np.float32), p)            # fp32 add, exact
    assert np.array_equal(q.astype(np.float64) + err.astype(np.float64), p.astype(np.float64))
    w = oracle.grad_code_bits(k_g) - 1
    mu = out["codes"] & ((1 << w) - 1)
    sign = out["codes"] >> w
    assert mu.max() <= k_g + 1 and sign.max() <= 1
    assert not np.any((sign == 1) & (mu == 0))                        # no negative zero
    s = out["scales"][0]
    top = np.argmax(np.abs(p))
    assert s == np.abs(p[top]) and mu[top] == k_g + 1 and err[top] == 0.0 and q[top] == p[top]
    # sign(q) in {0, sign(p)}
    assert np.all((q == 0) | (np.sign(q) == np.sign(p)))


@pytest.mark.parametrize("k_g", [0, 1, 2, 4])
def test_assumption2_contraction(oracle, k_g):
    """Assumption 2: ||p - Q_g(p)|| <= (1 - delta_g) ||p|| with delta_g > 0; element-wise the
    residual never exceeds |p_j| (0 is in G) nor half the widest gap below level 1."""
    rng = np.random.default_rng(400 + k_g)
    for trial in range(20):
        n = int(rng.integers(1, 5000))
        p = (rng.standard_t(3, n) * 10.0 ** rng.uniform(-5, 2)).astype(np.float32)
        st, s, code, q, tie = oracle.qg_layer(OracleConfig(k_g=k_g), p)
        r = p.astype(np.float64) - q.astype(np.float64)
        assert np.linalg.norm(r) < np.linalg.norm(p.astype(np.float64))
        assert np.all(np.abs(r) <= np.abs(p.astype(np.float64)))
        bound = (0.5 if k_g == 0 else 0.25) * float(s)
        assert np.all(np.abs(r) <= bound * (1 + 1e-6))


@pytest.mark.parametrize("k_x", [0, 3, 6, 14])
def test_assumption3_bounded_weight_error(oracle, k_x):
    """Assumption 3: ||x - Q_x(x)|| <= delta_x; inside [-1/2, 1/2] each element is within half a
    grid step 2^-(k_x+2), and x^ + residual == y exactly."""
    rng = np.random.default_rng(500 + k_x)
    x = rng.uniform(-0.5, 0.5, 20000).astype(np.float32)
    cfg = OracleConfig(k_x=k_x, weight_ef=0)
    werr = np.zeros_like(x)
    out = oracle.weight_quantize(cfg, 1, x, werr)
    assert np.all(np.abs(werr) <= 2.0 ** -(k_x + 2))
    assert np.array_equal((out["xhat"] + werr).astype(np.float32), x)
    assert np.array_equal(out["wcodes"].astype(np.float64) * 2.0 ** -(k_x + 1),
                          out["xhat"].astype(np.float64))
    assert out["wcodes"].dtype == (np.int8 if k_x <= 6 else np.int16)


def test_weight_error_feedback_modes(oracle):
    """Algorithm 2 keeps the full-precision iterate and only emits Q_x(x_t): with weight_ef = 0 the
    residual is reported and not fed back; with weight_ef = 1 the quantizer sees x + e^x and the
    running sum of emitted values tracks the running sum of x (sigma-delta telescoping)."""
    rng = np.random.default_rng(7)
    n, T, k_x = 4096, 40, 3
    xs = [rng.uniform(-0.4, 0.4, n).astype(np.float32) for _ in range(T)]
    cfg0 = OracleConfig(k_x=k_x, weight_ef=0)
    cfg1 = OracleConfig(k_x=k_x, weight_ef=1)
    w0 = np.full(n, 123.0, np.float32)
    w1 = np.zeros(n, np.float32)
    sum_hat = np.zeros(n)
    sum_x = np.zeros(n)
    for t, x in enumerate(xs, 1):
        o0 = oracle.weight_quantize(cfg0, t, x, w0)
        direct = oracle.qx(cfg0, x)[1]
        assert np.array_equal(o0["xhat"], direct)          # previous residual ignored
        assert np.array_equal(w0, (x - direct).astype(np.float32))
        o1 = oracle.weight_quantize(cfg1, t, x, w1)
        sum_hat += o1["xhat"]
        sum_x += x
        assert np.allclose(sum_hat + w1, sum_x, atol=1e-5)
    assert np.all(np.abs(w1) <= 2.0 ** -(k_x + 2) + 1e-6)


def test_qx_saturation(oracle):
    """The grid X ends at +-1, so Q_x saturates at +-1/2."""
    x = np.array([0.6, -0.7, 5.0, -1e9, 0.5, -0.5], np.float32)
    j, xh, _ = oracle.qx(OracleConfig(k_x=6), x)
    assert list(xh) == [0.5, -0.5, 0.5, -0.5, 0.5, -0.5]
    assert list(j) == [64, -64, 64, -64, 64, -64]


# ------------------------------------------------------------ degenerate layers
def test_zero_and_nonfinite_layers(oracle):
    cfg = OracleConfig(k_g=2)
    st, s, code, q, tie = oracle.qg_layer(cfg, np.zeros(100, np.float32))
    assert st == 0 and s == 0 and not code.any() and not q.any()
    e = np.zeros(64, np.float32)
    g = np.zeros(64, np.float32)
    g[3] = -0.0
    out = oracle.worker_quantize(cfg, [0, 64], 0, 1, g, e)
    assert not out["words"].any() and not e.any()
    for bad in (np.nan, np.inf, -np.inf):
        p = np.ones(10, np.float32)
        p[4] = bad
        st, s, code, q, tie = oracle.qg_layer(cfg, p)
        assert st == 1 and not np.isfinite(s)
    # empty layer and empty vector
    out = oracle.worker_quantize(cfg, [0, 0, 5, 5], 0, 1, np.ones(5, np.float32), np.zeros(5, np.float32))
    assert out["status"] == 0 and list(out["scales"]) == [0.0, 1.0, 0.0]


def test_tie_flags(oracle):
    """Elements whose ratio sits within one ulp of a midpoint are flagged; others are not."""
    cfg = OracleConfig(k_g=2)
    mids = [0.125, 0.375, 0.75]
    vals = []
    for m in mids:
        m32 = np.float32(m)
        vals += [m32, np.nextafter(m32, np.float32(0)), np.nextafter(m32, np.float32(1)),
                 np.float32(m * 1.01), np.float32(m * 0.99)]
    p = np.array(vals + [1.0], np.float32)
    _, s, code, q, tie = oracle.qg_layer(cfg, p)
    want = [1, 1, 1, 0, 0] * 3 + [0]
    assert list(tie) == want
    j, xh, tie = oracle.qx(OracleConfig(k_x=2), np.array([0.0625, 0.07, 0.1875, 0.2], np.float32))
    assert list(tie) == [1, 0, 1, 0]


# ------------------------------------------------------------------ bit budget
def test_bit_budget_matches_tables(oracle):
    """Tables 1-2: Comm and Size columns.  The packed layouts must cost exactly 2 or 3 bits per
    gradient element and 8 or 16 per weight, which reproduces the printed megabytes."""
    assert oracle.grad_code_bits(0) == 2
    assert oracle.grad_code_bits(1) == 3 and oracle.grad_code_bits(2) == 3
    assert oracle.grad_code_bits(3) == 4 and oracle.grad_code_bits(6) == 4
    P = 1 << 20
    for table, kind, full, quant, bits in _rows("tables_bits.txt"):
        full, quant, bits = float(full), float(quant), int(bits)
        if kind == "comm":
            k_g = 0 if bits == 2 else 2
            stored_bits = oracle.grad_code_words(k_g, [0, P]) * 32 / P
        else:
            k_x = 6 if bits == 8 else 14
            stored_bits = np.dtype(oracle.weight_code_dtype(k_x)).itemsize * 8
        assert stored_bits == bits
        # both numbers are printed to 4 significant digits
        half_full = 0.5 * 10 ** (np.floor(np.log10(full)) - 3)
        half_quant = 0.5 * 10 ** (np.floor(np.log10(quant)) - 3)
        assert abs(full * stored_bits / 32 - quant) <= half_full * stored_bits / 32 + half_quant + 1e-9


def test_pack_unpack_layout(oracle):
    """Bit-plane layout: group of 32 elements -> b words, word k = bit k of each code, bit n of the
    word = element 32*group + n; tail zero-padded; segments padded to 16 bytes."""
    rng = np.random.default_rng(3)
    for bits in (2, 3, 4):
        for n in (1, 31, 32, 33, 255, 256, 1000):
            code = rng.integers(0, 1 << bits, n).astype(np.uint8)
            words = oracle.pack_codes(bits, code)
            assert words.size % 4 == 0 and words.size >= (n + 31) // 32 * bits
            # independent reconstruction with python integers
            for j in (0, n // 2, n - 1):
                g, b = divmod(j, 32)
                c = sum(((int(words[g * bits + k]) >> b) & 1) << k for k in range(bits))
                assert c == code[j]
            assert np.array_equal(oracle.unpack_codes(bits, words, n), code)
            # padding bits are zero
            total_set = sum(bin(int(w)).count("1") for w in words)
            assert total_set == sum(bin(int(c)).count("1") for c in code)
    # one explicit example: element 5 with code 0b101 sets bit 5 of words 0 and 2
    code = np.zeros(32, np.uint8)
    code[5] = 0b101
    words = oracle.pack_codes(3, code)
    assert list(words[:3]) == [1 << 5, 0, 1 << 5]


# ------------------------------------------------- scaling by powers of two (Sec. 5.1 grids)
def test_grid_points_are_exact_power_of_two_multiples_down_to_subnormals(oracle):
    """Sec. 5.1: the points of G are s * 2^(mu-1-k_g) and those of X are j * 2^-(k_x+1).  The oracle forms
    them as a product with an exactly representable power of two; a correctly rounded product with a
    power of two is the same number as ldexp of it (one rounding, also when the result is subnormal or
    underflows to zero).  Checked bit for bit against numpy's ldexp for scales from the smallest
    subnormal to the largest finite value, every level of every grid."""
    rng = np.random.default_rng(7)
    mant = np.concatenate([[0, 1, 0x400000, 0x7fffff], rng.integers(0, 1 << 23, 12)]).astype(np.uint32)
    scales = []
    for e in range(0, 255):                       # exponent field 0 = subnormals, 254 = largest binade
        for mnt in mant:
            bits = np.uint32((e << 23) | int(mnt))
            if bits:
                scales.append(bits)
    scales = np.array(scales, np.uint32).view(np.float32)
    lib = oracle.lib()
    for k_g in range(0, 7):
        w = oracle.grad_code_bits(k_g) - 1
        for mu in range(1, k_g + 2):
            want = np.ldexp(scales, mu - 1 - k_g).astype(np.float32)
            for neg in (0, 1):
                code = (neg << w) | mu
                got = np.array([lib.oq_qg_decode(k_g, float(s), code) for s in scales], np.float32)
                ref = -want if neg else want
                assert np.array_equal(got.view(np.uint32), ref.view(np.uint32)), (k_g, mu, neg)
    # Q_x: u = y * 2^(k_x+1) and x^ = j * 2^-(k_x+1)
    ys = np.concatenate([scales, -scales])
    ys = ys[np.abs(ys) < 4.0]                     # beyond the grid everything saturates (checked elsewhere)
    for k_x in (0, 3, 6, 7, 14):
        j, xh, _ = oracle.qx(OracleConfig(k_x=k_x), ys)
        u = np.ldexp(ys.astype(np.float64), k_x + 1)                 # exact in fp64
        jw = np.clip(np.sign(u) * np.floor(np.abs(u) + 0.5), -(1 << k_x), 1 << k_x)
        # u is also exact in fp32 here (a power-of-two scaling without overflow or underflow of a normal
        # value; a subnormal y scaled up stays exactly representable), so the fp32 decision equals this one
        assert np.array_equal(j.astype(np.float64), jw), k_x
        # (values, not bit patterns: a negative y that rounds to j = 0 gives x^ = -0.0)
        assert np.array_equal(xh, np.ldexp(j.astype(np.float32), -(k_x + 1))), k_x
