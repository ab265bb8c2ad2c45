"""Pins for the oracle's building blocks: storage formats, Philox, bit stream.

Each check compares the oracle with something it does not contain: numpy's and
torch's own conversions, the published Philox known-answer vectors, Python
big-integer arithmetic.
"""
from pathlib import Path

import numpy as np
import pytest
import torch

GOLDEN = Path(__file__).parent / "golden"


# ---------------------------------------------------------------- float16
def test_half_to_float_exhaustive_vs_numpy(oracle):
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float32)
    got = np.array([oracle.half_to_float(int(b)) for b in bits], dtype=np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))


def _interesting_floats(rng, count):
    raw = rng.integers(0, 2**32, size=count, dtype=np.uint64).astype(np.uint32)
    x = raw.view(np.float32)
    # dense around half's normal / subnormal / overflow boundaries and ties
    h = np.arange(0, 0x7C00, 7, dtype=np.uint16).view(np.float16).astype(np.float32)
    up = np.nextafter(h, np.float32(np.inf))
    ties = ((h.astype(np.float64) + up.astype(np.float64)) / 2)
    near = np.concatenate([h, up, ties.astype(np.float32),
                           np.nextafter(ties.astype(np.float32), np.float32(0)),
                           np.nextafter(ties.astype(np.float32), np.float32(np.inf))])
    edge = np.array([0.0, -0.0, 65504.0, 65519.99, 65520.0, 65536.0, 1e10, -1e10,
                     2.0**-24, 2.0**-25, 2.0**-25 * 1.0000001, 2.0**-26, 2.0**-14,
                     2.0**-14 * (1 - 2.0**-12), 2.0**-126, 1e-45, np.inf, -np.inf],
                    dtype=np.float32)
    allx = np.concatenate([x, near, -near, edge])
    return allx[~np.isnan(allx)]


def test_float_to_half_vs_numpy(oracle):
    x = _interesting_floats(np.random.default_rng(1), 150_000)
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    got = np.array([oracle.float_to_half(v) for v in x], dtype=np.uint16)
    bad = np.nonzero(got != want)[0]
    assert bad.size == 0, (x[bad[:5]], got[bad[:5]], want[bad[:5]])


# --------------------------------------------------------------- bfloat16
def test_bf16_roundtrip_vs_torch(oracle):
    rng = np.random.default_rng(2)
    raw = rng.integers(0, 2**32, size=150_000, dtype=np.uint64).astype(np.uint32)
    # exact ties and their neighbours in the low 16 bits
    ties = (raw & np.uint32(0xFFFF0000)) | np.uint32(0x8000)
    x = np.concatenate([raw, ties, ties + 1, ties - 1]).view(np.float32)
    x = x[np.isfinite(x)]
    want = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([oracle.float_to_bf16(v) for v in x], dtype=np.uint16)
    assert np.array_equal(got, want)
    back = np.array([oracle.bf16_to_float(int(b)) for b in want[:5000]], dtype=np.float32)
    want_back = torch.from_numpy(want[:5000].view(np.int16).copy()).view(torch.bfloat16).float().numpy()
    assert np.array_equal(back.view(np.uint32), want_back.view(np.uint32))


# ----------------------------------------------------------------- Philox
def _kat():
    rows = []
    for line in (GOLDEN / "philox4x32_10_kat.txt").read_text().splitlines():
        if line.startswith("#") or not line.strip():
            continue
        w = [int(t, 16) for t in line.split()]
        rows.append((w[0:4], w[4:6], w[6:10]))
    return rows


def test_philox_known_answers(oracle):
    rows = _kat()
    assert len(rows) == 3
    for ctr, key, want in rows:
        assert list(oracle.philox4x32_10(ctr, key)) == want


def test_uniform_mapping(oracle):
    """Element j uses word j%4 of block j//4, key = seed; u = top 24 bits / 2^24."""
    seed = 0xA4093822_299F31D0
    for j in [0, 1, 2, 3, 4, 7, 1023, 2**32 * 4 + 5, 2**40 + 2]:
        blk = j // 4
        w = oracle.philox4x32_10([blk & 0xFFFFFFFF, blk >> 32, 0, 0],
                                 [seed & 0xFFFFFFFF, seed >> 32])
        want = np.float32((int(w[j % 4]) >> 8) / 2.0**24)
        got = oracle.uniform(seed, j)
        assert got == want and 0.0 <= got < 1.0
    # the third published vector: counter words (hi, lo) = digits of pi cannot be
    # reached (words 2, 3 are zero here), but the first one can: seed 0, j in 0..3
    want0 = [0x6627e8d5, 0xe169c58d, 0xbc57ac4c, 0x9b00dbd8]
    for j in range(4):
        assert oracle.uniform(0, j) == np.float32((want0[j] >> 8) / 2.0**24)


def test_uniform_is_uniform(oracle):
    u = np.array([oracle.uniform(12345, j) for j in range(40_000)], dtype=np.float64)
    assert abs(u.mean() - 0.5) < 4 * (1 / 12) ** 0.5 / 200       # 4 sigma
    hist, _ = np.histogram(u, bins=16, range=(0, 1))
    assert hist.min() > 2500 * 0.9 and hist.max() < 2500 * 1.1
    # different seeds decorrelate the same index
    v = np.array([oracle.uniform(s, 17) for s in range(20_000)], dtype=np.float64)
    assert abs(v.mean() - 0.5) < 0.01


# ------------------------------------------------------------- bit stream
@pytest.mark.parametrize("bits", [2, 3, 4, 6, 8])
def test_pack_is_little_endian_bitstream(oracle, bits):
    """Element j sits at stream bits [j*b, j*b+b): the stream read as one
    little-endian integer is sum_j q_j << (j*b)."""
    rng = np.random.default_rng(bits)
    for count in [8, 16, 24, 64, 200]:
        q = rng.integers(0, 2**bits, size=count).astype(np.int32)
        big = 0
        for j, v in enumerate(q):
            big |= int(v) << (j * bits)
        want = big.to_bytes(count * bits // 8, "little")
        got = oracle.pack(q, bits)
        assert bytes(got) == want
        assert np.array_equal(oracle.unpack(got, count, bits), q)


@pytest.mark.parametrize("bits", [2, 3, 4, 6, 8])
def test_pack_unpack_exhaustive_small(oracle, bits):
    """Every level in every position of one 8-element block round-trips."""
    for pos in range(8):
        for v in range(2**bits):
            q = np.zeros(8, dtype=np.int32)
            q[pos] = v
            b = oracle.pack(q, bits)
            assert b.size == bits
            assert np.array_equal(oracle.unpack(b, 8, bits), q)
            # only the owner's bits are set
            assert int.from_bytes(bytes(b), "little") == v << (pos * bits)


def test_three_bit_block_layout(oracle):
    """Eight 3-bit codes fill exactly three bytes."""
    q = np.array([1, 2, 3, 4, 5, 6, 7, 0], dtype=np.int32)
    b = oracle.pack(q, 3)
    # 1 | 2<<3 | 3<<6 ... written out by hand:
    # bits: 001 010 011 100 101 110 111 000 (LSB first per code)
    assert list(b) == [0b11010001, 0b01011000, 0b00011111]
