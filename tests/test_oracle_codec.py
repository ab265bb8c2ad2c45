"""Pins for the oracle's four boundary calls, from what the paper fixes.

  * m starts at 0 (Algorithm 1, initialisation), so a first visit is direct
    quantisation of the activation.
  * Sender and receiver apply the same update to their own copy of m, so the
    two copies stay identical (Section 3.1).
  * The activation handed to the next stage is m(xi) (Algorithm 2, network b).
  * |a - m_new| is bounded by the group's level half-spacing (Theorem 3.1's
    requirement on Q, elementwise), plus the storage rounding.
  * The message error feeds back: with a constant activation the scale of the
    next message shrinks by the number of levels (Section 3.1's recursion).
  * Message size is b bits per element (Table 3's communication times).
"""
import numpy as np
import pytest

from paper_2206_01299_amd import workloads as W

DTYPES = ["f32", "f16", "bf16"]
BITS = [2, 3, 4, 6, 8]


def _ulp_of(x32, dtype):
    """Half a unit in the last place of the storage dtype at |x| (as float64)."""
    keep = {"f32": 24, "f16": 11, "bf16": 8}[dtype]
    ax = np.maximum(np.abs(x32.astype(np.float64)), 2.0**-14 if dtype == "f16" else 2.0**-126)
    return 2.0 ** (np.floor(np.log2(ax)) - (keep - 1))


def _rand_act(rng, shape, dtype, scale=1.0):
    x = rng.standard_normal(shape).astype(np.float32) * np.float32(scale)
    return W.to_storage(x, dtype)


def _levels_f64(d, s, bits):
    """Nearest level in float64, with the distance to the nearest tie."""
    L = 2**bits - 1
    pos = d.astype(np.float64) / np.float64(s) * (L / 2) + L / 2 + 0.5
    k = np.clip(np.floor(pos), 0, L).astype(np.int64)
    frac = pos - np.floor(pos)
    return k, np.minimum(frac, 1 - frac)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("bits", BITS)
def test_first_visit_is_direct_quantisation(oracle, dtype, bits):
    rng = np.random.default_rng(bits)
    B, n_per, G = 3, 256, 64
    act = _rand_act(rng, (B, n_per), dtype)
    m = np.zeros((5, n_per), dtype=act.dtype)
    ids = np.array([4, 0, 2], dtype=np.int64)
    codes, scales = oracle.encode(act, ids, m, dtype=dtype, bits=bits, group=G)
    gcodes, gscales = oracle.grad_quant(act.reshape(-1), dtype=dtype, bits=bits, group=G)
    assert np.array_equal(codes, gcodes) and np.array_equal(scales, gscales)
    direct = oracle.grad_dequant(gcodes, gscales, dtype=dtype, bits=bits, group=G)
    assert np.array_equal(m[ids].reshape(-1).view(np.uint8), direct.view(np.uint8))
    # rows that were not visited stay zero
    assert not m[[1, 3]].any()


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("bits,G", [(2, 128), (3, 64), (4, 200), (8, 8)])
def test_codes_and_scales_follow_the_definition(oracle, dtype, bits, G):
    """Whole-call check in float64 of scale = max|a - m| per group and of the
    level of every element, with rows gathered by sample id."""
    rng = np.random.default_rng(10 * bits + len(dtype))
    B, n_per, N = 4, 3200, 9
    m = _rand_act(rng, (N, n_per), dtype)
    # groups of very different magnitude, so a wrong group index cannot pass
    mag = 10.0 ** rng.uniform(-2, 2, size=(B, n_per // G, 1))
    a32 = (rng.standard_normal((B, n_per // G, G)) * mag).astype(np.float32).reshape(B, n_per)
    ids = np.array([7, 0, 8, 3], dtype=np.int64)
    a32 += W.storage_to_f32(m, dtype)[ids]
    act = W.to_storage(a32, dtype)
    m_before = m.copy()
    codes, scales = oracle.encode(act, ids, m, dtype=dtype, bits=bits, group=G)

    d = W.storage_to_f32(act, dtype) - W.storage_to_f32(m_before, dtype)[ids]     # binary32 subtraction
    d64 = W.storage_to_f32(act, dtype).astype(np.float64) - W.storage_to_f32(m_before, dtype)[ids].astype(np.float64)
    dg = d64.reshape(-1, G)
    # binary32 subtraction of two storage values, then max-abs (exact)
    want_s = np.abs((W.storage_to_f32(act, dtype) - W.storage_to_f32(m_before, dtype)[ids])
                    .reshape(-1, G)).max(axis=1)
    assert np.array_equal(scales, want_s)
    assert codes.size == B * n_per * bits // 8
    q = oracle.unpack(codes, B * n_per, bits).reshape(-1, G)
    k, margin = _levels_f64(d.reshape(-1, G), scales[:, None], bits)
    safe = margin > 1e-4
    assert safe.mean() > 0.9      # coarse dtypes hit exact ties often
    assert np.array_equal(q[safe], k[safe])
    assert np.abs(q - k).max() <= 1
    # m_new = storage(m_old + Q): within half an ulp of the exact sum
    L = 2**bits - 1
    dhat = (q - L / 2) * (scales[:, None].astype(np.float64) * 2 / L)
    exact = W.storage_to_f32(m_before, dtype)[ids].astype(np.float64).reshape(-1, G) + dhat
    got = W.storage_to_f32(m, dtype)[ids].astype(np.float64).reshape(-1, G)
    tol = 0.5 * _ulp_of(got.astype(np.float32), dtype) * (1 + 2.0**-10) + np.abs(dhat) * 2.0**-22
    assert np.all(np.abs(got - exact) <= tol)
    # untouched rows untouched
    rest = np.setdiff1d(np.arange(N), ids)
    assert np.array_equal(m[rest].view(np.uint8), m_before[rest].view(np.uint8))
    # element error bound against the true activation (dg is the true delta)
    err = np.abs(dg - dhat)
    assert np.all(err <= scales[:, None] / L * (1 + 2.0**-18))


@pytest.mark.parametrize("dtype", DTYPES)
def test_sample_order_only_permutes_the_message(oracle, dtype):
    rng = np.random.default_rng(5)
    B, n_per, G, bits = 4, 512, 64, 4
    act = _rand_act(rng, (B, n_per), dtype)
    m0 = _rand_act(rng, (6, n_per), dtype)
    ids = np.array([5, 1, 0, 3], dtype=np.int64)
    ma = m0.copy()
    ca, sa = oracle.encode(act, ids, ma, dtype=dtype, bits=bits, group=G)
    perm = np.array([2, 0, 3, 1])
    mb = m0.copy()
    cb, sb = oracle.encode(np.ascontiguousarray(act[perm]), ids[perm], mb, dtype=dtype, bits=bits, group=G)
    assert np.array_equal(ma.view(np.uint8), mb.view(np.uint8))
    assert np.array_equal(ca.reshape(B, -1)[perm], cb.reshape(B, -1))
    assert np.array_equal(sa.reshape(B, -1)[perm], sb.reshape(B, -1))


def _run_stream(oracle, cfg, stream, check_every_call=None):
    """Replay a stream through sender and receiver; return both buffers and stats."""
    np_dt = W.storage_numpy_dtype(cfg.dtype)
    rows = {int(s): i for i, s in enumerate(sorted(set(stream.epoch_ids(0).reshape(-1).tolist())))}
    m_send = np.zeros((len(rows), cfg.n_per), dtype=np_dt)
    m_recv = np.zeros((len(rows), cfg.n_per), dtype=np_dt)
    stats = []
    for t, k, ids, act in stream:
        local = np.array([rows[int(s)] for s in ids], dtype=np.int64)
        seed = W.call_seed(cfg, t, k)
        act2 = act.reshape(cfg.batch, cfg.n_per)
        codes, scales = oracle.encode(act2, local, m_send, dtype=cfg.dtype, bits=cfg.fwd_bits,
                                      group=cfg.fwd_group, rounding=cfg.fwd_rounding, seed=seed)
        out = oracle.decode(codes, scales, local, m_recv, dtype=cfg.dtype, bits=cfg.fwd_bits,
                            group=cfg.fwd_group)
        if check_every_call:
            check_every_call(t, k, local, act2, codes, scales, out, m_send, m_recv)
        stats.append((t, float(scales.mean())))
    return m_send, m_recv, stats


@pytest.mark.parametrize("dtype,rounding", [("f32", W.NEAREST), ("f16", W.NEAREST),
                                            ("bf16", W.NEAREST), ("f16", W.STOCHASTIC)])
def test_replicas_stay_identical_and_output_is_m(oracle, dtype, rounding):
    cfg = W.tiny().scaled(dtype=dtype, n_samples=16, seq=16, hidden=64, fwd_group=64,
                          fwd_rounding=rounding, epochs=3, shuffle_ids=True)
    stream = W.ActivationStream(cfg)
    L = 2**cfg.fwd_bits - 1

    def check(t, k, local, act, codes, scales, out, m_send, m_recv):
        assert np.array_equal(m_send.view(np.uint8), m_recv.view(np.uint8))
        assert np.array_equal(out.view(np.uint8), m_recv[local].reshape(-1).view(np.uint8))
        # reconstruction error against the true activation
        a = W.storage_to_f32(act, dtype).astype(np.float64).reshape(-1, cfg.fwd_group)
        r = W.storage_to_f32(out, dtype).astype(np.float64).reshape(-1, cfg.fwd_group)
        width = (1 if rounding == W.NEAREST else 2) * scales[:, None].astype(np.float64) / L
        bound = width * (1 + 2.0**-18) + 0.5 * _ulp_of(r.astype(np.float32), dtype) * 1.001
        assert np.all(np.abs(a - r) <= bound)

    m_send, m_recv, stats = _run_stream(oracle, cfg, stream, check)
    # later epochs send much smaller messages than the first (drift 0.01 vs N(0,1))
    first = np.mean([s for t, s in stats if t == 0])
    last = np.mean([s for t, s in stats if t == cfg.epochs - 1])
    assert last < first / 4


@pytest.mark.parametrize("bits", BITS)
def test_constant_activation_contracts_by_number_of_levels(oracle, bits):
    """delta_k = delta_{k-1} - Q(delta_{k-1}): each visit the group's max-abs
    falls to at most (previous scale)/L."""
    rng = np.random.default_rng(bits)
    L = 2**bits - 1
    G = 64
    act = rng.standard_normal((1, G)).astype(np.float32)
    m = np.zeros((1, G), dtype=np.float32)
    ids = np.zeros(1, dtype=np.int64)
    prev = None
    for visit in range(5 if bits <= 4 else 3):
        codes, scales = oracle.encode(act, ids, m, dtype="f32", bits=bits, group=G)
        s = float(scales[0])
        if prev is not None:
            assert s <= prev / L * (1 + 1e-5) + 2.0**-23     # + binary32 floor near |a|~1
        prev = s
    assert np.abs(act - m).max() <= prev / L * (1 + 1e-5) + 2.0**-23


def test_equal_activation_sends_zeros_and_keeps_m(oracle):
    rng = np.random.default_rng(9)
    for dtype in DTYPES:
        m = _rand_act(rng, (3, 128), dtype)
        before = m.copy()
        ids = np.array([2, 0], dtype=np.int64)
        act = np.ascontiguousarray(m[ids])
        codes, scales = oracle.encode(act, ids, m, dtype=dtype, bits=3, group=64)
        assert not codes.any() and not scales.any()
        assert np.array_equal(W.storage_to_f32(m, dtype), W.storage_to_f32(before, dtype))


@pytest.mark.parametrize("bits", BITS)
def test_message_size_is_b_bits_per_element(oracle, bits):
    """Table 3: one GPT2 micro-batch (1024 x 1600) at 4 bits takes 13 ms at
    500 Mbps and 8 bits 25 ms, i.e. the wire carries b bits per element."""
    n = 1024 * 1600
    assert oracle.codes_bytes(n, bits) * 8 == n * bits
    ms_500 = oracle.codes_bytes(n, bits) * 8 / 500e6 * 1e3
    if bits == 4:
        assert round(ms_500) == 13
    if bits == 8:
        assert 25 <= ms_500 < 27
    # per-row scales are negligible beside the codes
    assert 4 * 1024 < 0.02 * oracle.codes_bytes(n, bits)


def test_backward_roundtrip_error_bound(oracle):
    rng = np.random.default_rng(11)
    for dtype in DTYPES:
        for bits, G, rounding in [(8, 1600, W.NEAREST), (4, 128, W.STOCHASTIC), (8, 64, W.NEAREST)]:
            g = _rand_act(rng, (2, 3200), dtype, scale=1e-3)
            codes, scales = oracle.grad_quant(g.reshape(-1), dtype=dtype, bits=bits, group=G,
                                              rounding=rounding, seed=77)
            out = oracle.grad_dequant(codes, scales, dtype=dtype, bits=bits, group=G)
            L = 2**bits - 1
            a = W.storage_to_f32(g, dtype).astype(np.float64).reshape(-1, G)
            r = W.storage_to_f32(out, dtype).astype(np.float64).reshape(-1, G)
            width = (1 if rounding == W.NEAREST else 2) * scales[:, None].astype(np.float64) / L
            bound = width * (1 + 2.0**-18) + 0.5 * _ulp_of(r.astype(np.float32), dtype) * 1.001
            assert np.all(np.abs(a - r) <= bound)
            assert np.array_equal(scales, np.abs(W.storage_to_f32(g, dtype)).reshape(-1, G).max(1))


def test_stochastic_rounding_depends_on_seed_and_index_only(oracle):
    """Same seed -> same message; another seed -> another; and the draw of an
    element depends on its flat index in the call, not on the group size."""
    rng = np.random.default_rng(12)
    g = rng.standard_normal(2048).astype(np.float32)
    c1, s1 = oracle.grad_quant(g, dtype="f32", bits=2, group=128, rounding=W.STOCHASTIC, seed=5)
    c2, s2 = oracle.grad_quant(g, dtype="f32", bits=2, group=128, rounding=W.STOCHASTIC, seed=5)
    c3, s3 = oracle.grad_quant(g, dtype="f32", bits=2, group=128, rounding=W.STOCHASTIC, seed=6)
    assert np.array_equal(c1, c2) and not np.array_equal(c1, c3)
    # element j's level from the building blocks: position + uniform(seed, j)
    q = oracle.unpack(c1, 2048, 2)
    for j in [0, 1, 5, 127, 128, 777, 2047]:
        grp = j // 128
        r = np.full(128, 0.5, dtype=np.float32)
        r[j % 128] = oracle.uniform(5, j)
        qq, _, _ = oracle.quantize_group(g[grp * 128:(grp + 1) * 128], 2, r)
        assert qq[j % 128] == q[j]


def test_rejects_bad_shapes(oracle):
    a = np.zeros((1, 64), dtype=np.float32)
    m = np.zeros((1, 64), dtype=np.float32)
    ids = np.zeros(1, dtype=np.int64)
    for bits, group in [(5, 64), (4, 48), (3, 4), (4, 0)]:
        with pytest.raises((ValueError, ZeroDivisionError)):
            oracle.encode(a, ids, m, dtype="f32", bits=bits, group=group)


def test_empty_call(oracle):
    m = np.ones((2, 64), dtype=np.float32)
    codes, scales = oracle.encode(np.zeros((0, 64), np.float32), np.zeros(0, np.int64), m,
                                  dtype="f32", bits=4, group=64)
    assert codes.size == 0 and scales.size == 0 and np.all(m == 1)


# ---------------------------------------------------------------------------
# uncompressed first visit (Algorithm 1, lines "if xi not seen before")
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", DTYPES)
def test_seed_sets_m_to_the_activation(oracle, dtype):
    rng = np.random.default_rng(21)
    m = _rand_act(rng, (6, 200), dtype)
    before = m.copy()
    act = _rand_act(rng, (3, 200), dtype)
    ids = np.array([4, 0, 5], dtype=np.int64)
    oracle.seed(act, ids, m, dtype=dtype)
    assert np.array_equal(m[ids].view(np.uint8), act.view(np.uint8))
    rest = [1, 2, 3]
    assert np.array_equal(m[rest].view(np.uint8), before[rest].view(np.uint8))
    # the message error of a seeded sample is zero (used at the start of the proof of
    # Theorem 3.1): encoding the same activation again sends nothing
    codes, scales = oracle.encode(act.reshape(3, 200), ids, m, dtype=dtype, bits=4, group=8)
    assert not scales.any() and not codes.any()
    assert np.array_equal(W.storage_to_f32(m[ids], dtype), W.storage_to_f32(act, dtype))


def test_seeded_start_beats_zero_start_on_the_second_visit(oracle):
    """Algorithm 1 (full-precision first visit) against an all-zero m: after the
    seed, the second visit quantises only the drift, so its error is far smaller
    than what direct quantisation of the first visit leaves behind."""
    cfg = W.tiny().scaled(n_samples=8, seq=16, hidden=64, fwd_group=64, fwd_bits=2)
    stream = W.ActivationStream(cfg)
    ids = stream.epoch_ids(0)[0]
    a0 = stream.activations(ids, 0).reshape(cfg.batch, -1)
    a1 = stream.activations(ids, 1).reshape(cfg.batch, -1)
    m_seed = np.zeros((cfg.n_samples, cfg.n_per), dtype=np.float32)
    m_zero = np.zeros_like(m_seed)
    oracle.seed(a0, ids, m_seed, dtype="f32")
    oracle.encode(a0, ids, m_zero, dtype="f32", bits=2, group=64)
    oracle.encode(a1, ids, m_seed, dtype="f32", bits=2, group=64)
    oracle.encode(a1, ids, m_zero, dtype="f32", bits=2, group=64)
    err_seed = np.abs(m_seed[ids] - a1).mean()
    err_zero = np.abs(m_zero[ids] - a1).mean()
    assert err_seed < err_zero / 5
