"""Pins for the oracle's low-precision storage of previous messages ("m z",
Appendix H.5).  The appendix fixes little (z bits for m; 8 bits lose nothing
noticeable, 2 bits are a little worse than full precision and still clearly
better than direct quantisation); the rest follows from Algorithm 2 applied to
the stored value: replicas identical, the handed-on activation within the wire
quantiser's error of the true one, the stored value within the storage
quantiser's error of the handed-on one, zero storage = first visit.
"""
import numpy as np
import pytest

from paper_2206_01299_amd import workloads as W

DTYPES = ["f32", "f16", "bf16"]


def _ulp_half(x32, dtype):
    keep = {"f32": 24, "f16": 11, "bf16": 8}[dtype]
    ax = np.maximum(np.abs(x32.astype(np.float64)), 2.0**-14 if dtype == "f16" else 2.0**-126)
    return 0.5 * 2.0 ** (np.floor(np.log2(ax)) - (keep - 1))


def _stored_value(oracle, m_codes_row, m_scales_row, m_bits, group):
    """m^ of one sample from the oracle's building blocks."""
    n_per = m_codes_row.size * 8 // m_bits
    q = oracle.unpack(m_codes_row, n_per, m_bits).reshape(-1, group)
    return np.stack([oracle.dequantize_group(q[g], m_scales_row[g], m_bits) for g in range(q.shape[0])])


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("m_bits", [2, 8])
def test_zero_storage_first_visit_is_direct_quantisation(oracle, dtype, m_bits):
    rng = np.random.default_rng(m_bits)
    n_per, G, bits = 512, 64, 4
    act = W.to_storage(rng.standard_normal((3, n_per)).astype(np.float32), dtype)
    mc, ms = oracle.lowbit_state(6, n_per, m_bits, G)
    ids = np.array([5, 0, 2], dtype=np.int64)
    codes, scales = oracle.encode_lowbit(act, ids, mc, ms, dtype=dtype, bits=bits, m_bits=m_bits, group=G)
    gc, gs = oracle.grad_quant(act.reshape(-1), dtype=dtype, bits=bits, group=G)
    assert np.array_equal(codes, gc) and np.array_equal(scales, gs)
    assert not mc[[1, 3, 4]].any() and not ms[[1, 3, 4]].any()        # other rows untouched
    # what was stored is Q_z of the reconstructed first message
    direct = W.storage_to_f32(oracle.grad_dequant(gc, gs, dtype="f32", bits=bits, group=G), "f32")
    for k, row in enumerate(ids):
        want_q, want_s, _ = zip(*[oracle.quantize_group(direct.reshape(3, -1, G)[k, g], m_bits)
                                  for g in range(n_per // G)])
        assert np.array_equal(ms[row], np.array(want_s, dtype=np.float32))
        assert np.array_equal(oracle.unpack(mc[row], n_per, m_bits), np.concatenate(want_q))


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("bits,m_bits,rounding", [(2, 8, W.NEAREST), (4, 2, W.NEAREST), (3, 8, W.STOCHASTIC),
                                                  (8, 2, W.NEAREST), (6, 8, W.NEAREST)])
def test_replicas_identical_and_errors_bounded(oracle, dtype, bits, m_bits, rounding):
    cfg = W.tiny().scaled(dtype=dtype, n_samples=8, seq=8, hidden=64, fwd_group=64, fwd_bits=bits,
                          fwd_rounding=rounding, epochs=3, shuffle_ids=True)
    stream = W.ActivationStream(cfg)
    G, L, Lz = cfg.fwd_group, 2**bits - 1, 2**m_bits - 1
    mc_s, ms_s = oracle.lowbit_state(cfg.n_samples, cfg.n_per, m_bits, G)
    mc_r, ms_r = oracle.lowbit_state(cfg.n_samples, cfg.n_per, m_bits, G)
    for t, k, ids, act in stream:
        act2 = act.reshape(cfg.batch, cfg.n_per)
        before = np.stack([_stored_value(oracle, mc_s[i], ms_s[i], m_bits, G) for i in ids])
        codes, scales = oracle.encode_lowbit(act2, ids, mc_s, ms_s, dtype=dtype, bits=bits, m_bits=m_bits,
                                             group=G, rounding=rounding, seed=W.call_seed(cfg, t, k))
        out = oracle.decode_lowbit(codes, scales, ids, mc_r, ms_r, dtype=dtype, bits=bits, m_bits=m_bits,
                                   group=G)
        assert np.array_equal(mc_s, mc_r) and np.array_equal(ms_s, ms_r)
        a = W.storage_to_f32(act2, dtype).astype(np.float64).reshape(-1, G)
        o = W.storage_to_f32(out, dtype).astype(np.float64).reshape(-1, G)
        # the scale on the wire is max |a - m^| of the group
        d32 = (W.storage_to_f32(act2, dtype).reshape(-1, G) - before.reshape(-1, G)).astype(np.float32)
        assert np.array_equal(scales, np.abs(d32).max(axis=1))
        # handed-on activation: within the wire quantiser's error of the true one
        width = (1 if rounding == W.NEAREST else 2) * scales[:, None].astype(np.float64) / L
        assert np.all(np.abs(a - o) <= width * (1 + 2.0**-18) + _ulp_half(o.astype(np.float32), dtype) * 1.001)
        # stored value: within the storage quantiser's error of what was handed on
        after = np.stack([_stored_value(oracle, mc_s[i], ms_s[i], m_bits, G) for i in ids]).reshape(-1, G)
        s_store = ms_s[ids].reshape(-1)[:, None].astype(np.float64)
        assert np.all(np.abs(after - o) <= s_store / Lz * (1 + 2.0**-18)
                      + _ulp_half(o.astype(np.float32), dtype) * 1.001)


def test_paper_ordering_m8_close_to_full_m2_between_full_and_direct(oracle):
    """Appendix H.5 on a synthetic drifting stream: 8-bit storage loses next to
    nothing against full-precision m; 2-bit storage is worse but still clearly
    better than quantising the activation directly."""
    cfg = W.tiny().scaled(n_samples=16, seq=16, hidden=64, fwd_group=64, fwd_bits=4, epochs=4, drift=0.02)
    G, bits = cfg.fwd_group, cfg.fwd_bits

    def run(mode, m_bits=None):
        stream = W.ActivationStream(cfg)
        m = np.zeros((cfg.n_samples, cfg.n_per), dtype=np.float32)
        mc_s = ms_s = mc_r = ms_r = None
        if mode == "lowbit":
            mc_s, ms_s = oracle.lowbit_state(cfg.n_samples, cfg.n_per, m_bits, G)
            mc_r, ms_r = oracle.lowbit_state(cfg.n_samples, cfg.n_per, m_bits, G)
        errs = []
        for t, k, ids, act in stream:
            a = act.reshape(cfg.batch, cfg.n_per)
            if mode == "direct":
                c, s = oracle.grad_quant(a.reshape(-1), dtype="f32", bits=bits, group=G)
                out = oracle.grad_dequant(c, s, dtype="f32", bits=bits, group=G)
            elif mode == "full":
                oracle.encode(a, ids, m, dtype="f32", bits=bits, group=G)
                out = m[ids].reshape(-1)
            else:
                c, s = oracle.encode_lowbit(a, ids, mc_s, ms_s, dtype="f32", bits=bits, m_bits=m_bits, group=G)
                out = oracle.decode_lowbit(c, s, ids, mc_r, ms_r, dtype="f32", bits=bits, m_bits=m_bits, group=G)
            if t == cfg.epochs - 1:
                errs.append(np.abs(out - a.reshape(-1)).mean())
        return float(np.mean(errs))

    direct, full, m8, m2 = run("direct"), run("full"), run("lowbit", 8), run("lowbit", 2)
    assert full < direct / 5
    assert m8 < 1.5 * full                 # "no significant drop with 8 bits"
    assert full < m2 < direct / 2          # "slightly worse ... still significantly better than DirectQ"


def test_lowbit_rejects_bad_storage_width(oracle):
    mc, ms = oracle.lowbit_state(2, 64, 4, 64)      # 4-bit storage is not one of the appendix's widths
    with pytest.raises(ValueError):
        oracle.encode_lowbit(np.zeros((1, 64), np.float32), np.zeros(1, np.int64), mc, ms,
                             dtype="f32", bits=4, m_bits=4, group=64)
