"""Property tests of the oracle's quantizers on generated inputs (hypothesis): arbitrary finite
binary32 values -- subnormals, huge magnitudes, signed zeros, repeated values, any layer length --
must satisfy what Sec. 5.1 and Assumptions 2-3 of arXiv 2004.14180 fix for EVERY input, not only
for the Gaussian-like vectors of the other tests."""
import numpy as np
from hypothesis import given, settings, HealthCheck
from hypothesis import strategies as st
from hypothesis.extra import numpy as hnp

from oracle.qadam_oracle import OracleConfig

finite32 = st.floats(width=32, allow_nan=False, allow_infinity=False)
layers = hnp.arrays(np.float32, st.integers(1, 200), elements=finite32)
common = dict(max_examples=150, deadline=None, suppress_health_check=[HealthCheck.function_scoped_fixture])


@settings(**common)
@given(p=layers, k_g=st.integers(0, 6))
def test_qg_properties(oracle, p, k_g):
    status, s, code, q, tie = oracle.qg_layer(OracleConfig(k_g=k_g), p)
    assert status == 0 and s == np.max(np.abs(p))                      # the scale is the infinity norm
    w = oracle.grad_code_bits(k_g) - 1
    mu, neg = code & ((1 << w) - 1), code >> w
    assert mu.max() <= k_g + 1 and not np.any((mu == 0) & (neg == 1))   # codes in range, no "-0"
    if s == 0:
        assert not code.any() and not q.any()
        return
    p64, q64, s64 = p.astype(np.float64), q.astype(np.float64), np.float64(s)
    top = np.argmax(np.abs(p))
    assert q[top] == p[top]                                             # the arg-max is reproduced exactly
    assert np.all(np.sign(q64) * np.sign(p64) >= 0)
    # every value of the message is s times a grid point (up to the rounding of s * level near underflow)
    level = np.where(mu > 0, np.ldexp(1.0, mu.astype(np.int64) - 1 - k_g), 0.0)
    assert np.allclose(np.abs(q64), s64 * level, rtol=0, atol=2.0 ** -149)
    # nearest grid point: no other point of G is closer to |p| / s (slack: rounding of the quotient)
    grid = np.array([0.0] + [2.0 ** (c - 1 - k_g) for c in range(1, k_g + 2)])
    a = np.abs(p64) / s64
    best = np.min(np.abs(a[:, None] - grid[None, :]), axis=1)
    assert np.all(np.abs(a - level) <= best + 2.0 ** -22)
    # Assumption 2: the quantizer contracts; element-wise never beyond half the widest gap
    e = p64 - q64
    assert np.linalg.norm(e) < np.linalg.norm(p64) or not p64.any()
    assert np.all(np.abs(e) <= s64 * (0.25 if k_g >= 1 else 0.5) * (1 + 2.0 ** -20) + 2.0 ** -140)
    # the residual is a binary32 number: q + e' == p exactly
    assert np.array_equal((q + (p - q)).view(np.uint32)[np.abs(p) > 0], p.view(np.uint32)[np.abs(p) > 0])
    # packed layout round trip
    words = oracle.pack_codes(w + 1, code)
    assert np.array_equal(oracle.unpack_codes(w + 1, words, p.size), code)


@settings(**common)
@given(y=hnp.arrays(np.float32, st.integers(1, 200), elements=st.floats(-4, 4, width=32)), k_x=st.integers(0, 14))
def test_qx_properties(oracle, y, k_x):
    j, xhat, tie = oracle.qx(OracleConfig(k_x=k_x), y)
    assert np.all(np.abs(j) <= 2 ** k_x)
    assert np.array_equal(xhat.astype(np.float64), j * 2.0 ** -(k_x + 1))
    y64 = y.astype(np.float64)
    inside = np.abs(y64) <= 0.5
    assert np.all(np.abs(y64 - xhat)[inside] <= 2.0 ** -(k_x + 2))      # Assumption 3
    assert np.all(xhat[y64 > 0.5] == 0.5) and np.all(xhat[y64 < -0.5] == -0.5)   # saturation
    # nearest grid index, halves away from zero
    u = y64 * 2.0 ** (k_x + 1)
    want = np.clip(np.sign(u) * np.floor(np.abs(u) + 0.5), -2 ** k_x, 2 ** k_x)
    assert np.array_equal(j.astype(np.float64), want)
