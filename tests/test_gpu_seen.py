"""GPU parity of Algorithm 1 with its first-visit branch (aqsgd_encode_seen /
aqsgd_decode_seen) against the CPU oracle: a stream in which new samples keep
appearing, so calls mix first visits (uncompressed, seed m) with later visits
(quantised change).  Every byte the calls define is compared; the library's 32-bit
first-visit stamps are compared with the oracle's flags as zero / non-zero."""
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


def _replay(H, dtype, bits, group, n_per, n_rows, batch, steps, rounding, seed, as_jobs=False):
    import oracle
    d = H.dev()
    td = B.DTYPE_NAME[dtype]
    rng = np.random.default_rng(seed)
    base = rng.standard_normal((n_rows, n_per)).astype(np.float32)
    m_s = torch.zeros((n_rows, n_per), dtype=td, device=d); m_r = torch.zeros_like(m_s)
    seen_s = torch.zeros(n_rows, dtype=torch.int32, device=d); seen_r = torch.zeros_like(seen_s)
    npdt = W.to_storage(np.zeros(1, dtype=np.float32), dtype).dtype
    om_s = np.zeros((n_rows, n_per), dtype=npdt); om_r = om_s.copy()
    oseen_s = np.zeros(n_rows, dtype=np.uint8); oseen_r = oseen_s.copy()
    firsts = 0
    for step in range(steps):
        pool = min(n_rows, batch + step * max(1, batch // 2))            # the id range grows with time
        ids_np = rng.choice(pool, size=batch, replace=False).astype(np.int64)
        a_np = W.to_storage(base[ids_np] + 0.05 * step * rng.standard_normal((batch, n_per)).astype(np.float32),
                            dtype)
        desc = B.make_desc(batch=batch, n_per=n_per, n_samples=n_rows, bits=bits, group=group, dtype=dtype,
                           rounding=rounding, rng_seed=1000 + step)
        act = W.to_torch(a_np, dtype, d)
        ids = torch.from_numpy(ids_np).to(d)
        codes = torch.full((B.codes_bytes(desc),), 0x5A, dtype=torch.uint8, device=d)
        scales = torch.full((B.scales_count(desc),), float(0x5A), dtype=torch.float32, device=d)
        first = torch.full((batch,), -7, dtype=torch.int32, device=d)
        out = W.to_torch(W.to_storage(np.full((batch, n_per), 9.0, dtype=np.float32), dtype), dtype, d)
        if as_jobs:
            # the calls as jobs of a stage's launch, next to a backward message of that stage
            gdesc = B.make_desc(batch=batch, n_per=n_per, bits=8, group=group, dtype=dtype)
            g_np = W.to_storage(1e-3 * rng.standard_normal((batch, n_per)).astype(np.float32), dtype)
            grad = W.to_torch(g_np, dtype, d)
            gcodes = torch.empty(B.codes_bytes(gdesc), dtype=torch.uint8, device=d)
            gscales = torch.empty(B.scales_count(gdesc), dtype=torch.float32, device=d)
            gout = torch.empty((batch, n_per), dtype=td, device=d)
            B.run_jobs([B.grad_quant_job(gdesc, grad, gcodes, gscales),
                        B.encode_seen_job(desc, act, ids, m_s, seen_s, 1 + step, first, codes, scales)])
        else:
            B.encode_seen(desc, act, ids, m_s, seen_s, 1 + step, first, codes, scales)
        # the receiver is handed the uncompressed rows of the first visits only
        full = torch.where(first.view(-1, 1) == 1, act.view(batch, n_per), torch.zeros_like(act.view(batch, n_per)))
        full = full.contiguous()
        if as_jobs:
            B.run_jobs([B.decode_seen_job(desc, codes, scales, full, ids, m_r, seen_r, 77 + step, out),
                        B.grad_dequant_job(gdesc, gcodes, gscales, gout)])
        else:
            B.decode_seen(desc, codes, scales, full, ids, m_r, seen_r, 77 + step, out)
        torch.cuda.synchronize()
        if as_jobs:
            wgc, wgs = oracle.grad_quant(g_np.reshape(-1), dtype=dtype, bits=8, group=group, rounding=0, seed=0)
            wgo = oracle.grad_dequant(wgc, wgs, dtype=dtype, bits=8, group=group)
            assert H.same_bytes(gcodes.cpu().numpy(), wgc) and H.same_bytes(gscales.cpu().numpy(), wgs)
            assert H.same_bytes(W.from_torch(gout, dtype).reshape(-1), wgo.reshape(-1))

        wf, wc, ws = oracle.encode_seen(a_np, ids_np, om_s, oseen_s, dtype=dtype, bits=bits, group=group,
                                        rounding=rounding, seed=1000 + step, fill=0x5A)
        ofull = np.where(wf[:, None] == 1, a_np, np.zeros_like(a_np))
        wo = oracle.decode_seen(wc, ws, ofull, ids_np, om_r, oseen_r, dtype=dtype, bits=bits, group=group)
        tag = f"{dtype} b={bits} G={group} step {step}"
        assert np.array_equal(first.cpu().numpy(), wf), f"{tag}: first flags"
        assert H.same_bytes(codes.cpu().numpy(), wc), f"{tag}: codes: {H.first_diff(codes.cpu().numpy(), wc)}"
        assert H.same_bytes(scales.cpu().numpy(), ws), f"{tag}: scales"
        got = W.from_torch(out, dtype).reshape(-1)
        assert H.same_bytes(got, wo), f"{tag}: out: {H.first_diff(got, wo)}"
        assert H.same_bytes(W.from_torch(m_s, dtype), om_s), f"{tag}: sender m"
        assert H.same_bytes(W.from_torch(m_r, dtype), om_r), f"{tag}: receiver m"
        assert np.array_equal(seen_s.cpu().numpy() != 0, oseen_s != 0), f"{tag}: sender's seen words"
        assert np.array_equal(seen_r.cpu().numpy() != 0, oseen_r != 0), f"{tag}: receiver's seen words"
        firsts += int(wf.sum())
    assert 0 < firsts < steps * batch            # the stream really mixed first and later visits


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
def test_first_visits_mixed_with_later_visits(H, dtype):
    _replay(H, dtype, bits=4, group=256, n_per=2048, n_rows=40, batch=6, steps=10, rounding=0, seed=3)
    _replay(H, dtype, bits=2, group=64, n_per=1600, n_rows=24, batch=4, steps=8, rounding=1, seed=4)


def test_rows_that_are_not_whole_16_byte_units_and_odd_groups(H):
    _replay(H, "f16", bits=8, group=5, n_per=35, n_rows=16, batch=3, steps=8, rounding=0, seed=5)   # any-shape kernels
    _replay(H, "f32", bits=4, group=6, n_per=18, n_rows=16, batch=3, steps=8, rounding=1, seed=6)


def test_gpt2_shape_first_epoch_then_second(H):
    """The GPT2-1.5B per-call shape: an epoch of first visits, then the same samples again."""
    _replay(H, "f16", bits=4, group=1600, n_per=1024 * 1600, n_rows=8, batch=4, steps=4, rounding=0, seed=7)


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
def test_first_visit_calls_as_jobs_of_a_stage_launch(H, dtype):
    """aqsgd_run_jobs with the two first-visit kinds: each shares a launch with a backward
    message of its stage, on streams that mix first and later visits."""
    _replay(H, dtype, bits=4, group=256, n_per=2048, n_rows=40, batch=6, steps=10, rounding=0, seed=13,
            as_jobs=True)
    _replay(H, dtype, bits=3, group=64, n_per=1600, n_rows=24, batch=4, steps=8, rounding=1, seed=14,
            as_jobs=True)


def test_seen_jobs_reject_bad_arguments(H):
    import ctypes
    ok = B.make_desc(batch=2, n_per=1600, n_samples=4, bits=4, group=1600, dtype="f16")
    p = 4096
    enc = B.Job(B.JOB_ENCODE_SEEN, ok, p, p, p, p, p, None, p, p, None, 1, 0)
    dec = B.Job(B.JOB_DECODE_SEEN, ok, None, p, p, p, p, p, p, None, p, 1, 0)
    L = B.lib()
    def run(job):
        return L.aqsgd_run_jobs((B.Job * 1)(job), 1, None)
    for field, job, want in (("seen", enc, -1), ("first", enc, -1), ("seen", dec, -1), ("full", dec, -1)):
        keep = getattr(job, field)
        setattr(job, field, None)
        assert run(job) == want, field
        setattr(job, field, keep)
    enc.stamp = 0
    dec.stamp = 0
    assert run(enc) == -5 and run(dec) == -5
    enc.stamp = 1
    enc.first = 4098
    assert run(enc) == -6


def test_seen_entry_points_reject_bad_arguments(H):
    import ctypes
    L = B.lib()
    p = ctypes.c_void_p(4096)
    ok = B.make_desc(batch=2, n_per=1600, n_samples=4, bits=4, group=1600, dtype="f16")
    assert L.aqsgd_encode_seen(ctypes.byref(ok), p, p, p, None, 1, p, p, p, None) == -1
    assert L.aqsgd_decode_seen(ctypes.byref(ok), p, p, None, p, p, p, 1, p, None) == -1
    assert L.aqsgd_encode_seen(ctypes.byref(ok), p, p, p, p, 1, ctypes.c_void_p(4098), p, p, None) == -6
    assert L.aqsgd_encode_seen(ctypes.byref(ok), p, p, p, p, 0, p, p, p, None) == -5        # stamp 0
    assert L.aqsgd_decode_seen(ctypes.byref(ok), p, p, p, p, p, p, 0, p, None) == -5
    bad = B.make_desc(batch=2, n_per=1600, n_samples=4, bits=5, group=1600, dtype="f16")
    assert L.aqsgd_encode_seen(ctypes.byref(bad), p, p, p, p, 1, p, p, p, None) == -2
