"""Pins for the oracle's quantiser Q (Section 4.1) on single groups.

The level decision is checked against exact rational arithmetic, the
hand-worked example, and the properties Theorem 3.1 asks of Q (bounded error,
unbiasedness under stochastic rounding).
"""
from fractions import Fraction
from pathlib import Path

import numpy as np
import pytest

GOLDEN = Path(__file__).parent / "golden"
BITS = [2, 3, 4, 6, 8]


def exact_position(d, bits):
    """Exact position of each element on the level axis 0..L (Fractions)."""
    L = 2**bits - 1
    fd = [Fraction(float(v)) for v in d]
    s = max(abs(v) for v in fd)
    return [v / s * Fraction(L, 2) + Fraction(L, 2) for v in fd], s, L


@pytest.mark.parametrize("bits", BITS)
def test_nearest_level_vs_exact_rationals(oracle, bits):
    rng = np.random.default_rng(100 + bits)
    checked = 0
    for trial in range(60):
        G = int(rng.choice([8, 16, 24, 64]))
        scale = 10.0 ** rng.uniform(-6, 4)
        d = (rng.standard_normal(G) * scale).astype(np.float32)
        q, s, dhat = oracle.quantize_group(d, bits)
        pos, s_exact, L = exact_position(d, bits)
        assert Fraction(float(s)) == s_exact                     # max-abs, exact
        for e in range(G):
            k_exact = int((pos[e] + Fraction(1, 2)).__floor__())  # nearest, ties up
            k_exact = min(max(k_exact, 0), L)
            frac = (pos[e] + Fraction(1, 2)) % 1
            if min(frac, 1 - frac) > Fraction(1, 10_000):        # away from a tie
                assert q[e] == k_exact
                checked += 1
            else:
                assert abs(int(q[e]) - k_exact) <= 1
            # reconstruction sits on the level: (k - L/2) * 2s/L
            want = (Fraction(int(q[e])) - Fraction(L, 2)) * s_exact * 2 / L
            err = abs(Fraction(float(dhat[e])) - want)
            assert err <= abs(want) * Fraction(1, 2**22)
            # Theorem 3.1's requirement in its elementwise form: |d - Q(d)| <= s/L
            assert abs(Fraction(float(d[e])) - Fraction(float(dhat[e]))) \
                <= s_exact / L * (1 + Fraction(1, 2**18))
    assert checked > 1000


@pytest.mark.parametrize("bits", BITS)
def test_extremes_and_sign(oracle, bits):
    """+s maps to the top level, -s to level 0, and both reconstruct exactly."""
    L = 2**bits - 1
    d = np.array([5.0, -5.0, 0.0, 2.5, -2.5, 1.0, -1.0, 4.999], dtype=np.float32)
    q, s, dhat = oracle.quantize_group(d, bits)
    assert s == np.float32(5.0)
    assert q[0] == L and q[1] == 0
    assert dhat[0] == np.float32(5.0) and dhat[1] == np.float32(-5.0)
    # antisymmetric inputs land on mirrored levels (no tie among these values)
    assert q[3] + q[4] == L and q[5] + q[6] == L
    assert np.all(np.sign(dhat[[3, 5]]) > 0) and np.all(np.sign(dhat[[4, 6]]) < 0)
    # monotone: larger input never gets a lower level
    order = np.argsort(d, kind="stable")
    assert np.all(np.diff(q[order]) >= 0)


def test_ties_go_up(oracle):
    # b=2: levels at -3,-1,1,3 for s=3; 0 and +-2 are exact ties
    d = np.array([3, -3, 0, 2, -2, 1, -1, 0], dtype=np.float32)
    q, s, dhat = oracle.quantize_group(d, 2)
    assert list(q) == [3, 0, 2, 3, 1, 2, 1, 2]
    assert list(dhat) == [3, -3, 1, 3, -1, 1, -1, 1]


def _golden_example():
    out = {}
    for line in (GOLDEN / "two_visit_example.txt").read_text().splitlines():
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        out[k] = v
    return out


def test_hand_worked_two_visits(oracle):
    g = _golden_example()
    bits, G = int(g["bits"][0]), int(g["group"][0])
    m = np.zeros((1, G), dtype=np.float32)
    ids = np.array([0], dtype=np.int64)
    a1 = np.array([float(v) for v in g["visit1_act"]], dtype=np.float32).reshape(1, G)
    codes, scales = oracle.encode(a1, ids, m, dtype="f32", bits=bits, group=G)
    assert scales[0] == np.float32(float(g["visit1_scale"][0]))
    assert list(oracle.unpack(codes, G, bits)) == [int(v) for v in g["visit1_levels"]]
    assert codes.tobytes().hex() == g["visit1_byte"][0]
    assert list(m[0]) == [float(v) for v in g["visit1_m"]]
    a2 = np.array([float(v) for v in g["visit2_act"]], dtype=np.float32).reshape(1, G)
    codes, scales = oracle.encode(a2, ids, m, dtype="f32", bits=bits, group=G)
    assert scales[0] == np.float32(float(g["visit2_scale"][0]))
    assert list(oracle.unpack(codes, G, bits)) == [int(v) for v in g["visit2_levels"]]
    assert codes.tobytes().hex() == g["visit2_byte"][0]
    assert [f"{b:08x}" for b in m[0].view(np.uint32)] == g["visit2_m_bits"]
    # the fixture's own last line, re-derived exactly: m = RN(m1 + RN((k-1.5) * RN(s/1.5)))
    m1 = [3, -3, 1, 1]
    step = Fraction(float(np.float32(1.0) / np.float32(1.5)))
    for e, k in enumerate([2, 3, 2, 1]):
        dh = np.float32(float((Fraction(k) - Fraction(3, 2)) * step))   # RN to binary32
        want = np.float32(float(Fraction(m1[e]) + Fraction(float(dh))))
        assert m[0, e] == want


@pytest.mark.parametrize("bits", BITS)
def test_stochastic_level_vs_exact_rationals(oracle, bits):
    """With the offset r given, the level is floor(position + r)."""
    rng = np.random.default_rng(200 + bits)
    checked = 0
    for trial in range(40):
        G = 32
        d = (rng.standard_normal(G) * 10.0 ** rng.uniform(-3, 3)).astype(np.float32)
        r = (rng.integers(0, 2**24, size=G) / 2.0**24).astype(np.float32)
        q, s, dhat = oracle.quantize_group(d, bits, r)
        pos, s_exact, L = exact_position(d, bits)
        for e in range(G):
            y = pos[e] + Fraction(float(r[e]))
            k = min(max(int(y.__floor__()), 0), L)
            frac = y % 1
            if min(frac, 1 - frac) > Fraction(1, 10_000):
                assert q[e] == k
                checked += 1
            # stochastic rounding moves to one of the two neighbouring levels
            assert abs(Fraction(float(d[e])) - Fraction(float(dhat[e]))) \
                <= 2 * s_exact / L * (1 + Fraction(1, 2**18))
    assert checked > 1000


@pytest.mark.parametrize("bits", BITS)
def test_levels_stay_in_range_at_offset_extremes(oracle, bits):
    """position + r can round up to L + 1 in binary32; the level must not."""
    L = 2**bits - 1
    top = np.float32(1.0) - np.float32(2.0**-24)
    d = np.array([7.0, -7.0, 7.0, -7.0, 6.9999995, -6.9999995, 0.0, 0.0], dtype=np.float32)
    r = np.array([top, 0.0, 0.0, top, top, 0.0, top, 0.0], dtype=np.float32)
    q, s, dhat = oracle.quantize_group(d, bits, r)
    assert q.min() >= 0 and q.max() <= L
    assert q[0] == L and q[2] == L and q[1] == 0
    assert q[3] in (0, 1)      # -s * RN(hL/s) may land a hair above level 0
    assert np.all(np.abs(dhat) <= s)


@pytest.mark.parametrize("bits", BITS)
def test_unbiased_under_philox_rounding(oracle, bits):
    """E[Q(d)] = d when the offsets are the generator's uniforms (Theorem 3.1)."""
    G, M = 64, 3000
    rng = np.random.default_rng(300 + bits)
    d = rng.standard_normal(G).astype(np.float32)
    L = 2**bits - 1
    acc = np.zeros(G, dtype=np.float64)
    for seed in range(M):
        r = np.array([oracle.uniform(seed * 7919 + 13, j) for j in range(G)], dtype=np.float32)
        q, s, dhat = oracle.quantize_group(d, bits, r)
        acc += dhat
    mean = acc / M
    step = 2 * float(s) / L
    tol = 5 * (step / 2) / np.sqrt(M) + 1e-6        # 5 sigma of a two-point law
    inner = np.abs(d) < float(s)                    # the extremes are exact anyway
    assert np.all(np.abs(mean - d)[inner] < tol), np.abs(mean - d).max() / tol
    # and nearest rounding is NOT unbiased for generic inputs: the test can fail
    q, s, dn = oracle.quantize_group(d, bits)
    if bits <= 4:
        assert np.abs(dn - d).max() > tol


def test_tiny_or_zero_group_sends_nothing(oracle):
    for val in [0.0, 1e-37, 2.0**-121]:
        d = np.full(8, val, dtype=np.float32)
        d[3] = -val
        q, s, dhat = oracle.quantize_group(d, 4)
        assert s == 0.0 and not q.any() and not dhat.any()
        assert not np.signbit(dhat).any()
    # just above the floor the group is sent normally and stays finite
    d = np.full(8, 2.0**-120, dtype=np.float32)
    q, s, dhat = oracle.quantize_group(d, 8)
    assert s == np.float32(2.0**-120) and np.all(q == 255)
    assert np.all(np.isfinite(dhat)) and np.all(np.abs(dhat / d - 1) < 2.0**-22)
    # receiver with scale 0 reconstructs +0 whatever the codes say
    assert not oracle.dequantize_group(np.arange(8), 0.0, 4).any()


@pytest.mark.parametrize("bits", BITS)
def test_dequantize_matches_quantize(oracle, bits):
    """The receiver's Q^-1(codes, scale) equals the sender's own Q(d), bit for bit."""
    rng = np.random.default_rng(400 + bits)
    for _ in range(50):
        d = (rng.standard_normal(64) * 10.0 ** rng.uniform(-5, 5)).astype(np.float32)
        q, s, dhat = oracle.quantize_group(d, bits)
        back = oracle.dequantize_group(q, s, bits)
        assert np.array_equal(back.view(np.uint32), dhat.view(np.uint32))
