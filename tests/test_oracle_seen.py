"""Pins for the oracle's Algorithm 1 with its first-visit branch: a sample that has
no previous message travels uncompressed and seeds m; every later visit sends the
quantised change.

Fixed independently of the code under test:
  * a first visit reproduces the activation bit for bit on both machines (the
    algorithm sends it in full precision and both set m(xi) to it);
  * a second visit with an unchanged activation sends nothing (scale 0, codes 0);
  * a seen sample's slices are what the plain, separately pinned encoder gives for
    the same call (same flat indices, same random offsets);
  * the two machines' buffers and flags stay identical over a stream in which new
    samples keep appearing;
  * the reconstruction error of a first visit is exactly zero, whereas starting
    from m = 0 leaves the quantiser's error.
"""
import numpy as np
import pytest

from paper_2206_01299_amd import workloads as W


def _acts(rng, shape, dtype):
    return W.to_storage(rng.standard_normal(shape).astype(np.float32), dtype)


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_first_visit_is_uncompressed_on_both_machines(oracle, dtype):
    rng = np.random.default_rng(1)
    n_rows, B, n_per, G = 8, 3, 256, 64
    a = _acts(rng, (B, n_per), dtype)
    ids = np.array([5, 0, 7])
    m_s = np.zeros((n_rows, n_per), dtype=a.dtype); m_r = m_s.copy()
    seen_s = np.zeros(n_rows, dtype=np.uint8); seen_r = seen_s.copy()
    first, codes, scales = oracle.encode_seen(a, ids, m_s, seen_s, dtype=dtype, bits=4, group=G, fill=0xAB)
    assert list(first) == [1, 1, 1]
    assert (codes == 0xAB).all() and (scales == float(0xAB)).all()       # nothing written for first visits
    assert np.array_equal(m_s[ids].view(np.uint8), a.view(np.uint8))
    assert sorted(np.flatnonzero(seen_s)) == [0, 5, 7]
    out = oracle.decode_seen(codes, scales, a, ids, m_r, seen_r, dtype=dtype, bits=4, group=G)
    assert np.array_equal(out.view(np.uint8), a.reshape(-1).view(np.uint8))
    assert np.array_equal(m_r.view(np.uint8), m_s.view(np.uint8)) and np.array_equal(seen_r, seen_s)


def test_second_visit_with_unchanged_activation_sends_nothing(oracle):
    rng = np.random.default_rng(2)
    a = _acts(rng, (2, 128), "f16")
    ids = np.array([1, 3])
    m = np.zeros((4, 128), dtype=np.float16); seen = np.zeros(4, dtype=np.uint8)
    oracle.encode_seen(a, ids, m, seen, dtype="f16", bits=2, group=32)
    first, codes, scales = oracle.encode_seen(a, ids, m, seen, dtype="f16", bits=2, group=32, fill=0xFF)
    assert list(first) == [0, 0]
    assert (scales == 0).all() and (codes == 0).all()
    assert np.array_equal(m[ids].view(np.uint8), a.view(np.uint8))


@pytest.mark.parametrize("rounding", [0, 1])
def test_seen_samples_get_what_the_plain_encoder_gives(oracle, rounding):
    rng = np.random.default_rng(3)
    n_rows, B, n_per, G, bits = 10, 4, 384, 128, 3
    ids = np.array([2, 9, 4, 6])
    m0 = _acts(rng, (n_rows, n_per), "f32")
    a = _acts(rng, (B, n_per), "f32")
    seen = np.zeros(n_rows, dtype=np.uint8)
    seen[[9, 6]] = 1                                                     # samples 1 and 3 of the call are known
    m_a = m0.copy()
    first, codes, scales = oracle.encode_seen(a, ids, m_a, seen, dtype="f32", bits=bits, group=G,
                                              rounding=rounding, seed=11, fill=0x55)
    m_b = m0.copy()
    pc, ps = oracle.encode(a, ids, m_b, dtype="f32", bits=bits, group=G, rounding=rounding, seed=11)
    assert list(first) == [1, 0, 1, 0]
    cps, gps = n_per * bits // 8, n_per // G
    for i in (1, 3):
        assert np.array_equal(codes[i * cps:(i + 1) * cps], pc[i * cps:(i + 1) * cps])
        assert np.array_equal(scales[i * gps:(i + 1) * gps], ps[i * gps:(i + 1) * gps])
        assert np.array_equal(m_a[ids[i]], m_b[ids[i]])
    for i in (0, 2):
        assert (codes[i * cps:(i + 1) * cps] == 0x55).all()
        assert np.array_equal(m_a[ids[i]], a[i])
    untouched = np.setdiff1d(np.arange(n_rows), ids)
    assert np.array_equal(m_a[untouched], m0[untouched])
    assert seen[ids].all() and seen.sum() == 4


def test_replicas_stay_identical_while_new_samples_keep_appearing(oracle):
    rng = np.random.default_rng(4)
    n_rows, B, n_per, G = 12, 4, 256, 64
    base = rng.standard_normal((n_rows, n_per)).astype(np.float32)
    m_s = np.zeros((n_rows, n_per), dtype=np.float16); m_r = m_s.copy()
    seen_s = np.zeros(n_rows, dtype=np.uint8); seen_r = seen_s.copy()
    for step in range(9):
        pool = min(n_rows, 4 + step)                                     # the id range grows: new samples arrive late
        ids = rng.choice(pool, size=B, replace=False)
        a = W.to_storage(base[ids] + 0.05 * step * rng.standard_normal((B, n_per)).astype(np.float32), "f16")
        was_seen = seen_s[ids].copy()
        first, codes, scales = oracle.encode_seen(a, ids, m_s, seen_s, dtype="f16", bits=4, group=G,
                                                  rounding=1, seed=100 + step)
        assert np.array_equal(first, 1 - was_seen.astype(np.int32))
        full = np.where(first[:, None] == 1, a, np.float16(0))          # only first-visit rows travel in full
        out = oracle.decode_seen(codes, scales, full, ids, m_r, seen_r, dtype="f16", bits=4, group=G)
        assert np.array_equal(m_s.view(np.uint8), m_r.view(np.uint8))
        assert np.array_equal(seen_s, seen_r)
        assert np.array_equal(out.reshape(B, n_per).view(np.uint8), m_r[ids].view(np.uint8))
        for i in range(B):
            if first[i]:
                assert np.array_equal(out.reshape(B, n_per)[i], a[i])


def test_first_visit_error_is_zero_unlike_a_zero_start(oracle):
    rng = np.random.default_rng(5)
    a = _acts(rng, (1, 512), "f32")
    ids = np.array([0])
    m_alg1 = np.zeros((1, 512), dtype=np.float32); seen = np.zeros(1, dtype=np.uint8)
    oracle.encode_seen(a, ids, m_alg1, seen, dtype="f32", bits=2, group=512)
    m_zero = np.zeros((1, 512), dtype=np.float32)
    oracle.encode(a, ids, m_zero, dtype="f32", bits=2, group=512)
    assert np.abs(m_alg1 - a).max() == 0
    assert np.abs(m_zero - a).max() > 0.1


def test_once_everything_is_seen_it_is_the_plain_codec(oracle):
    rng = np.random.default_rng(6)
    n_rows, B, n_per = 6, 3, 192
    ids = np.array([4, 1, 2])
    m0 = _acts(rng, (n_rows, n_per), "bf16")
    a = _acts(rng, (B, n_per), "bf16")
    seen = np.ones(n_rows, dtype=np.uint8)
    m_a, m_b = m0.copy(), m0.copy()
    first, codes, scales = oracle.encode_seen(a, ids, m_a, seen, dtype="bf16", bits=8, group=64)
    pc, ps = oracle.encode(a, ids, m_b, dtype="bf16", bits=8, group=64)
    assert not first.any()
    assert np.array_equal(codes, pc) and np.array_equal(scales, ps) and np.array_equal(m_a, m_b)
    r_a, r_b = m0.copy(), m0.copy()
    out_a = oracle.decode_seen(codes, scales, np.zeros_like(a), ids, r_a, seen, dtype="bf16", bits=8, group=64)
    out_b = oracle.decode(pc, ps, ids, r_b, dtype="bf16", bits=8, group=64)
    assert np.array_equal(out_a, out_b.reshape(-1)) and np.array_equal(r_a, r_b)
