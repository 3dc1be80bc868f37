"""Pins of the oracle's counter-based random stream and of the optional unbiased rounding."""
import os

import numpy as np

from oracle.qadam_oracle import OracleConfig

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_philox_known_answers(oracle):
    """Philox4x32-10 against the known-answer vectors published with the generator
    (Salmon et al., SC'11)."""
    n = 0
    for line in open(os.path.join(GOLD, "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        v = [int(t, 16) for t in line.split()]
        assert oracle.philox4x32_10(v[:4], v[4:6]) == v[6:]
        n += 1
    assert n == 3


def test_uniform_stream_keying(oracle):
    """U depends on (seed, floor(j/4), j mod 4, step, worker, stream) exactly as documented: the
    four elements of one counter block take the four output words, top 24 bits each."""
    seed, step, worker, stream = 0x1234567890ABCDEF, 7, 3, 1
    for j in (0, 5, 1 << 33, (1 << 33) + 2):
        blk = j >> 2
        out = oracle.philox4x32_10([blk & 0xFFFFFFFF, blk >> 32, step, worker + (stream << 16)],
                                   [seed & 0xFFFFFFFF, seed >> 32])
        want = (out[j & 3] >> 8) / 2.0 ** 24
        assert oracle.uniform24(seed, j, step, worker, stream) == want
    u = np.array([oracle.uniform24(1, j, 1, 0, 0) for j in range(20000)])
    assert 0 <= u.min() and u.max() < 1
    assert abs(u.mean() - 0.5) < 0.01 and abs(u.var() - 1 / 12) < 0.005
    assert abs(np.corrcoef(u[:-1], u[1:])[0, 1]) < 0.03
    # different step / worker / stream give different streams
    base = [oracle.uniform24(1, j, 1, 0, 0) for j in range(64)]
    for args in [(2, 0, 0), (1, 1, 0), (1, 0, 1)]:
        other = [oracle.uniform24(1, j, *args) for j in range(64)]
        assert sum(a == b for a, b in zip(base, other)) < 4


def test_stochastic_rounding_is_unbiased_and_adjacent(oracle):
    """Unbiased rounding (the alternative the comparison systems use, Sec. 5.2): the value goes to
    one of its two neighbouring grid points with probabilities that make the mean exact."""
    n = 200_000
    for k_g, val in [(2, 0.3), (2, 0.05), (0, 0.3), (2, 0.6)]:
        p = np.full(n, val, np.float32)
        p[0] = 1.0
        cfg = OracleConfig(k_g=k_g, rounding=1, seed=42)
        st, s, code, q, tie = oracle.qg_layer(cfg, p, j0=0, step=3, worker=2)
        vals = np.unique(q[1:])
        assert len(vals) == 2
        grid = np.array([0.0] + [2.0 ** -k for k in range(k_g, -1, -1)])
        lo = grid[grid <= val].max()
        hi = grid[grid > val].min()
        assert set(vals.tolist()) == {np.float32(lo), np.float32(hi)}
        assert abs(q[1:].mean() - val) < 4 * (hi - lo) / np.sqrt(n)
    x = np.full(n, 0.1234, np.float32)
    j, xh, _ = oracle.qx(OracleConfig(k_x=2, rounding=1, seed=9), x, step=5)
    assert set(np.unique(xh).tolist()) == {0.0, 0.125}
    assert abs(xh.mean() - 0.1234) < 4 * 0.125 / np.sqrt(n)
    # same counters, same draws
    j2, xh2, _ = oracle.qx(OracleConfig(k_x=2, rounding=1, seed=9), x, step=5)
    assert np.array_equal(xh, xh2)
