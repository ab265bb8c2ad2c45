"""GPU parity for previous messages kept at low precision (Appendix H.5, "m z"):
aqsgd_encode_lowbit / aqsgd_decode_lowbit against the oracle, bit for bit, on
the message (codes, scales), both machines' storage (levels, scales) and the
handed-on activation.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_2206_01299_amd import binding as B
from paper_2206_01299_amd import workloads as W


@pytest.fixture(scope="module")
def H():
    if not torch.cuda.is_available():
        pytest.fail("these tests need the MI355X; run them with -m gpu on the GPU box")
    B.lib()
    import oracle
    oracle.build()
    import gpu_harness
    return gpu_harness


@pytest.fixture(autouse=True)
def _release_device_memory():
    yield
    if torch.cuda.is_available():
        torch.cuda.synchronize()
        torch.cuda.empty_cache()


def _replay(H, cfg, m_bits, calls_per_epoch, epochs, log=lambda *a, **k: None):
    """Stream through sender and receiver on the device and on the host."""
    import oracle
    d = H.dev()
    visited = W.parity_ids(cfg, calls_per_epoch)
    order = np.sort(visited)
    local = {int(s): i for i, s in enumerate(order)}
    stream = W.ActivationStream(cfg, visited=visited)
    G, bits = cfg.fwd_group, cfg.fwd_bits
    desc0 = B.make_desc(batch=cfg.batch, n_per=cfg.n_per, n_samples=cfg.n_samples, bits=bits, group=G,
                        dtype=cfg.dtype, rounding=cfg.fwd_rounding)
    row = B.lowbit_row_bytes(desc0, m_bits)
    assert row == cfg.n_per * m_bits // 8
    dev_state = [(torch.zeros((cfg.n_samples, row), dtype=torch.uint8, device=d),
                  torch.zeros((cfg.n_samples, cfg.n_per // G), dtype=torch.float32, device=d)) for _ in range(2)]
    host_state = [oracle.lowbit_state(len(order), cfg.n_per, m_bits, G) for _ in range(2)]
    torch.cuda.synchronize()
    idx = torch.from_numpy(order).to(d)
    for t in range(epochs):
        for k, ids in enumerate(stream.epoch_ids(t)):
            log(f"[{cfg.name} m{m_bits}] epoch {t} call {k}", flush=True)
            act = stream.activations(ids, t).reshape(cfg.batch, cfg.n_per)
            seed = W.call_seed(cfg, t, k)
            desc = B.make_desc(batch=cfg.batch, n_per=cfg.n_per, n_samples=cfg.n_samples, bits=bits,
                               group=G, dtype=cfg.dtype, rounding=cfg.fwd_rounding, rng_seed=seed)
            codes = torch.empty(B.codes_bytes(desc), dtype=torch.uint8, device=d)
            scales = torch.empty(B.scales_count(desc), dtype=torch.float32, device=d)
            out = torch.empty((cfg.batch, cfg.n_per), dtype=B.DTYPE_NAME[cfg.dtype], device=d)
            ids_d = torch.from_numpy(ids).to(d)
            B.encode_lowbit(desc, m_bits, W.to_torch(act, cfg.dtype, d), ids_d, dev_state[0][0],
                            dev_state[0][1], codes, scales)
            B.decode_lowbit(desc, m_bits, codes, scales, ids_d, dev_state[1][0], dev_state[1][1], out)
            loc = np.array([local[int(s)] for s in ids], dtype=np.int64)
            wc, ws = oracle.encode_lowbit(act, loc, host_state[0][0], host_state[0][1], dtype=cfg.dtype,
                                          bits=bits, m_bits=m_bits, group=G, rounding=cfg.fwd_rounding,
                                          seed=seed)
            wo = oracle.decode_lowbit(wc, ws, loc, host_state[1][0], host_state[1][1], dtype=cfg.dtype,
                                      bits=bits, m_bits=m_bits, group=G)
            torch.cuda.synchronize()
            tag = f"{cfg.name} m{m_bits} e{t} c{k}"
            assert H.same_bytes(scales.cpu().numpy(), ws), f"{tag} scales: {H.first_diff(scales.cpu().numpy(), ws)}"
            assert H.same_bytes(codes.cpu().numpy(), wc), f"{tag} codes: {H.first_diff(codes.cpu().numpy(), wc)}"
            g_out = W.from_torch(out, cfg.dtype).reshape(-1)
            assert H.same_bytes(g_out, wo), f"{tag} out: {H.first_diff(g_out, wo)}"
        for side in range(2):
            got_c = dev_state[side][0].index_select(0, idx).cpu().numpy()
            got_s = dev_state[side][1].index_select(0, idx).cpu().numpy()
            assert H.same_bytes(got_s, host_state[side][1]), f"{cfg.name} m{m_bits} side {side} storage scales"
            assert H.same_bytes(got_c, host_state[side][0]), f"{cfg.name} m{m_bits} side {side} storage levels"
    assert np.array_equal(host_state[0][0], host_state[1][0])


def _cfg(dtype, bits, group, rounding, gps, batch=3, n_samples=7):
    return W.BoundaryConfig(
        name=f"lowbit_{dtype}_b{bits}_g{group}_r{rounding}", n_samples=n_samples, batch=batch, seq=gps,
        hidden=group, dtype=dtype, fwd_bits=bits, fwd_group=group, fwd_rounding=rounding, bwd_bits=8,
        bwd_group=group, bwd_rounding=W.NEAREST, law="normal", drift=0.05, epochs=2, shuffle_ids=True,
        seed=2000 + bits * 11 + group)


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("m_bits", [2, 8])
def test_lowbit_sweep(H, dtype, m_bits):
    """Every team shape of the low-precision-storage kernels, ragged tails included (520, 576,
    1560 and 1600: groups whose last round of chunks is taken as single elements per lane)."""
    for group in [8, 24, 64, 128, 200, 520, 576, 1000, 1088, 1536, 1560, 1600, 2048, 4096, 8200, 16384]:
        gps = 37 if group <= 2048 else 5
        for bits, rounding in [(4, W.NEAREST), (2, W.STOCHASTIC), (3, W.NEAREST), (6, W.STOCHASTIC), (8, W.NEAREST),
                               (2, W.NEAREST)]:
            if group > 2048 and bits not in (4, 2):
                continue
            print(f"lowbit {dtype} m{m_bits} b{bits} G{group} r{rounding}", flush=True)
            _replay(H, _cfg(dtype, bits, group, rounding, gps), m_bits, calls_per_epoch=2, epochs=2)


@pytest.mark.parametrize("dtype,scale", [("f16", 3e-7), ("f16", 2e-5), ("bf16", 1e-37), ("f32", 1e-36)])
@pytest.mark.parametrize("m_bits", [2, 8])
def test_lowbit_subnormal_activations(H, dtype, scale, m_bits):
    """Activations in and just above the storage type's subnormal range (float16), and around
    the 2^-120 floor below which a group is sent as zero (bfloat16, binary32): widening,
    differences and sums must not flush anything to zero."""
    for group, bits in ((1600, 4), (64, 8), (128, 2)):
        cfg = _cfg(dtype, bits, group, W.NEAREST, gps=9).scaled(outlier_channel_frac=1.0, outlier_scale=scale,
                                                                  name=f"lowbit_small_{dtype}_{scale}_g{group}")
        _replay(H, cfg, m_bits, calls_per_epoch=2, epochs=2)


def test_lowbit_rejects_what_it_does_not_support(H):
    import ctypes
    L = B.lib()
    p = ctypes.c_void_p(4096)
    ok = B.make_desc(batch=2, n_per=1600, n_samples=4, bits=4, group=1600, dtype="f16")
    assert L.aqsgd_encode_lowbit(ctypes.byref(ok), 4, p, p, p, p, p, p, None) == -2       # m_bits
    odd = B.make_desc(batch=2, n_per=1600, n_samples=4, bits=4, group=100, dtype="f16")   # not chunks of 8
    assert L.aqsgd_encode_lowbit(ctypes.byref(odd), 8, p, p, p, p, p, p, None) == -3
    big = B.make_desc(batch=2, n_per=32768, n_samples=4, bits=4, group=32768, dtype="f16")
    assert L.aqsgd_decode_lowbit(ctypes.byref(big), 8, p, p, p, p, p, p, None) == -3
    assert B.lowbit_row_bytes(ok, 8) == 1600 and B.lowbit_row_bytes(ok, 2) == 400
    assert B.lowbit_row_bytes(ok, 3) == 0


@pytest.mark.parametrize("m_bits", [8, 2])
def test_lowbit_gpt2_shape_full_size(H, m_bits):
    """Config 2's per-call shape with the storage allocated for all 8192 samples
    (13.4 GB of levels at 8 bits), first and last row visited."""
    cfg = W.gpt2_4bit()
    _replay(H, cfg, m_bits, calls_per_epoch=2, epochs=2, log=print)
